// The bf16 backward kernels once more, for head_dim 64 (launch_bf16_d64_backward): same code, 128-byte token rows,
// four column tiles per stage.
#define CLEAR_HEAD_DIM 64
#define CLEAR_TILES_PER_STAGE 4
#include "kernels_bf16_bwd.hip"
