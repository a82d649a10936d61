// The bf16 forward kernels once more, for head_dim 64 (launch_bf16_d64): same code, 128-byte token rows,
// 16 matrix instructions per staged tile instead of 32, and four tiles per stage so that a stage still
// fills the same LDS and carries the same matrix work per barrier.
#define CLEAR_HEAD_DIM 64
#define CLEAR_TILES_PER_STAGE 4
#include "kernels_bf16.hip"
