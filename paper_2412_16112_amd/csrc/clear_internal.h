// Internal declarations shared by the host API and the kernel launchers (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>
#include <vector>

namespace clear {

// Geometry of the bf16 MFMA kernels: a wave owns a 4 x 8 patch of queries (32 = one MFMA N
// dimension); a workgroup owns NWY x NWX such patches; a key tile is 8 x 8 image tokens staged as
// two 4 x 8 blocks of 32 keys (one MFMA M dimension each).
constexpr int kWaveQH = 4, kWaveQW = 8;
constexpr int kKeyBlockH = 4, kKeyBlockW = 8;
constexpr int kKeyTileH = 8, kKeyTileW = 8;
constexpr int kKeyTileKeys = kKeyTileH * kKeyTileW;  // 64 keys per staged tile
#ifndef CLEAR_NWY
#define CLEAR_NWY 4
#endif
constexpr int kBf16NWY = CLEAR_NWY, kBf16NWX = 2;    // workgroup = (4 NWY) x 16 queries, 2 NWY waves
constexpr int kBf16QTileH = kBf16NWY * kWaveQH, kBf16QTileW = kBf16NWX * kWaveQW;
constexpr int kTextQueriesPerWave = 32;

// fp32 accuracy path: one thread per query, 16 x 16 queries per workgroup, same key tiles.
constexpr int kF32QTileH = 16, kF32QTileW = 16;

struct Schedule {
    int gridH = 0, gridW = 0, r = 0;
    int mask_kind = 0, mask_shift = 0;  // MaskKind of block_class.h; shift: Swin windows only
    int qth = 0, qtw = 0, kth = 0, ktw = 0;
    int n_qty = 0, n_qtx = 0, n_kty = 0, n_ktx = 0;
    std::vector<int> row_ptr;        // n_q_tiles + 1
    std::vector<int> col_idx;        // key tile ids, ascending per query tile
    std::vector<unsigned char> flags;  // CLEAR_TILE_FULL / CLEAR_TILE_PARTIAL
};

// Host-side integer geometry (schedule.cpp)
void build_schedule(int gridH, int gridW, int r, int qth, int qtw, int kth, int ktw, Schedule* s, int mask_kind = 0, int mask_shift = 0);
// Upper bound, in 64 bits, on the (query tile, key tile) pairs build_schedule would list (it stores them with int indices).
long long schedule_pair_bound(int gridH, int gridW, int r, int qth, int qtw, int kth, int ktw);
constexpr long long kMaxSchedulePairs = 1LL << 28;  // 2.4 GB of host and device tables; create refuses more
unsigned long long mask_count(int n_text, int gridH, int gridW, int r, int mask_kind = 0, int mask_shift = 0);
// Pairs fed to the matrix pipeline per (batch, head) by the bf16 kernels (image pass + text-query pass).
unsigned long long executed_pairs_bf16(const Schedule& s, int n_text, int text_split_keys);
// The same for a strided context (s: the schedule of the class sub-grid; gridH, gridW: the real grid).
unsigned long long executed_pairs_bf16_strided(const Schedule& s, int n_text, int gridH, int gridW, int stride, int layer);
// Pairs visited by the fp32 path (it tests every slot of every staged tile).
unsigned long long executed_pairs_f32(const Schedule& s, int n_text);

// Where element (b, h, n, c) of a [B, H, N, head_dim] tensor lives: base + b * sb + h * sh + n * sn + c (in
// elements; channels are contiguous).  The plain layout is sn = head_dim, sh = N * head_dim, sb = H * N * head_dim.
struct TensorStrides {
    long long sb, sh, sn;
};

struct FwdParams {
    const void* Q;
    const void* K;
    const void* V;
    void* O;
    TensorStrides qs, ks, vs, os;  // bf16 kernels only; the fp32 kernel takes the plain layout
    int B, H, n_text, gridH, gridW, r2;
    long long N;       // tokens per (batch, head)
    int n_q_tiles;     // image query tiles per head
    int n_qtx;         // query tiles per tile row
    int n_ktx;         // key tiles per tile row
    const int* row_ptr;  // device CSR
    const int* col_idx;  // per query tile: key tile origins (row << 16 | col), tiles inside the grid first (ascending), then the ones cut by the border
    const int* n_plain;  // per query tile: how many of its key tiles lie inside the grid
    const int* qt_order;  // bf16 image-query kernel, whole-grid launches: the query tile that the i-th workgroup of a head takes (null: i)
    const unsigned long long* mask_tbl;  // bf16 kernels: lane masks per relative block offset (may be null)
    int mask_ry, mask_rx;
    const int* wave_desc;  // bf16 kernels, with mask_tbl: per listed key tile (kernel order) and wave of the workgroup, the mask-table
                           // entries of the tile's two blocks (low / high 16 bits), or kWaveSkipsTile (see build_wave_descriptors)
    float scale_log2e;  // log2(e) / sqrt(head_dim)
    // text-query pass: dense rows split along the keys, partial results merged afterwards
    int n_tq_tiles;   // text query tiles per head
    int n_splits;     // key splits
    int split_keys;   // keys per split, multiple of 64
    float* ws_o;      // [B*H][n_splits][n_text][head_dim] un-normalised partial outputs
    float* ws_ml;     // [B*H][n_splits][n_text][2]        running max (raw logit) and denominator
    // Row-band mode (one band of image rows with its halo; Sec. 3.4).  Whole grid: own_y0 = 0, own_y1 = gridH,
    // qt_begin = 0, n_q_tiles_launch = n_q_tiles, NV = N, vkeys_text = INT_MAX, vshift = 0, y_shift = 0, band_o = null.
    int own_y0, own_y1;    // image rows whose queries are computed; the other rows are halo: keys only
    int qt_begin;          // first query tile launched (tile rows covering the owned rows)
    int n_q_tiles_launch;  // query tiles launched per (batch, head)
    // key list of the text-query pass by "virtual" index v in [0, NV): token v for v < vkeys_text, else v + vshift
    long long NV;
    int vkeys_text;
    int vshift;
    int y_shift;      // tile coordinates (own_y0, own_y1, the tile lists) = image row + y_shift; the grid then spans rows [y_shift, y_shift + gridH)
    float* band_o;    // when set, the text merge writes fp32 softmax outputs [B*H][n_text][head_dim] here ...
    float* band_lse;  // ... and the natural log of the softmax denominators [B*H][n_text] here, not O's text rows
    int mask_kind, mask_r, mask_shift;  // MaskKind, radius / window size, Swin shift
    float* lse;       // optional [B*H][N]: natural log of every row's softmax denominator sum_j exp(q.k_j / sqrt(d))
    // Strided mask: n_classes = stride^2 dense problems per (batch, head), one per residue class (y % stride,
    // x % stride) of the queries; class (a, b) takes its keys from class ((a + stride_rx) % stride, (b + stride_ry)
    // % stride).  The tile lists then describe the class sub-grid.  Otherwise n_classes = 1, stride = 1.
    int n_classes, stride, stride_rx, stride_ry;
    // Query prologue applied while the query rows are loaded (bf16 kernels; all null: Q is used as it is).
    const float* q_gain;  // [head_dim] RMS-norm gain, or null: no normalisation
    const float* rope_y;  // [gridH][head_dim/2][2] (cos, sin) per row, or null: no rotation
    const float* rope_x;  // [gridW][head_dim/2][2] (cos, sin) per column
    float norm_eps;
};

// Launchers (kernels_bf16.hip, kernels_f32.hip).  Each returns the first HIP error met.
// phase: kPhaseAll, or one of the three kernels of a forward pass (used to time them one by one).
// kPhaseImageAndTextQuery (bf16 only): the first two in one launch.
enum Phase : int { kPhaseAll = -1, kPhaseImage = 0, kPhaseTextQuery = 1, kPhaseTextMerge = 2, kPhaseImageAndTextQuery = 3 };
hipError_t launch_bf16_d128(const FwdParams& p, hipStream_t stream, int phase);
hipError_t launch_bf16_d64(const FwdParams& p, hipStream_t stream, int phase);
hipError_t launch_f32_d64(const FwdParams& p, hipStream_t stream, int phase);
int bf16_text_queries_per_block();
// What each wave of a bf16 workgroup does with each listed key tile that lies inside the grid (those are masked from the
// table): desc[e * waves + w] for entry e of the kernel-order tile list `k_col` (origins row << 16 | col) and wave w
// (patch row w / 2, patch column w % 2 of the query tile) = table entry of block 0 | table entry of block 1 << 16,
// where a block that is wholly admitted takes the all-ones entry and one out of reach the all-zeros entry; or
// kWaveSkipsTile when neither block can be reached.  Entries of tiles cut by the border hold kWaveSkipsTile (not used).
constexpr int kWaveSkipsTile = -1;
void build_wave_descriptors(const Schedule& s, const std::vector<int>& k_col, const std::vector<int>& n_plain, int mask_ry, int mask_rx,
                            std::vector<int>* desc);
void build_bf16_mask_table(int r, int ry, int rx, int mask_kind, std::vector<unsigned long long>* tbl);
int f32_text_queries_per_block();
// Backward pass (kernels_bf16_bwd.hip).
struct BwdParams {
    const void* Q;
    const void* K;
    const void* V;
    const void* dO;
    const float* lse;    // [B*H][N] natural log of the softmax denominators (from the forward pass)
    const float* delta;  // [B*H][N] dO_i . O_i (in the context's workspace: from the delta kernel, or from the dQ kernels, see delta_out)
    const void* O;       // the forward output, read where delta is formed inside the dQ kernels
    float* delta_out;    // not null: the dQ kernels form delta of their own rows from O and dO, use it and store it here for
                         // the dK / dV kernels launched after them (null: every kernel reads `delta`)
    void* dQ;
    void* dK;
    void* dV;
    TensorStrides qs, ks, vs, os, dos, dqs, dks, dvs;  // lse and delta are plain [B*H][N]
    int B, H, n_text, gridH, gridW, r2;
    long long N;
    int n_q_tiles, n_qtx;
    const int* row_ptr;
    const int* col_idx;
    const int* n_plain;
    const int* qt_order;  // as in FwdParams
    const unsigned long long* mask_tbl;
    int mask_ry, mask_rx;
    const int* wave_desc;  // as in FwdParams (rows and columns swap roles for dK and dV; the masks with a table are symmetric)
    int mask_kind, mask_r, mask_shift;  // MaskKind, radius / window size, Swin shift
    int n_classes, stride, stride_rx, stride_ry;  // strided mask, as in FwdParams (otherwise 1, 1, 0, 0)
    float scale_log2e;  // log2(e) / sqrt(head_dim)
    float scale;        // 1 / sqrt(head_dim)
    // text rows: sums over every token, split along the columns, partial sums added up afterwards
    int n_tq_tiles, n_splits, split_keys;
    float* ws;  // [3 (dQ, dK, dV)][B*H][n_splits][n_text][head_dim]
};
// phase: kBwdPhaseAll (the dQ kernels, which form delta on their way, then the dK / dV kernels, then the reduction),
// or one kernel of the pass: delta first; the image-row and text-row kernels are independent
// of each other; the reduction of the text-row partial sums comes after the two text-row kernels.
// kBwdPhaseFour: the four kernels between delta and the reduction in one launch.
enum BwdPhase : int { kBwdPhaseAll = -1, kBwdPhaseDelta = 0, kBwdPhaseImageQ = 1, kBwdPhaseImageKV = 2, kBwdPhaseTextQ = 3, kBwdPhaseTextKV = 4, kBwdPhaseReduce = 5, kBwdPhaseFour = 6 };
hipError_t launch_bf16_d128_backward(const BwdParams& p, const void* O, float* delta, hipStream_t stream, int phase);
hipError_t launch_bf16_d64_backward(const BwdParams& p, const void* O, float* delta, hipStream_t stream, int phase);

// band_merge.hip: combination of the text-query outputs of several row bands.
constexpr int kMaxMergeParts = 64;
struct MergeParts {
    int n;
    const float* o[kMaxMergeParts];    // [B*H][n_text][head_dim] softmax outputs
    const float* lse[kMaxMergeParts];  // [B*H][n_text] natural log of the softmax denominators
};
hipError_t launch_merge_text(const MergeParts& parts, int BH, int n_text, long long N, int head_dim, int mode, void* O, int dtype,
                             hipStream_t stream);
// prologue.hip: RMS norm + rotary embedding of whole [BH][N][head_dim] bf16 tensors (the keys of a fused
// forward pass; also the stand-alone pass).  X == Y is allowed.
hipError_t launch_qk_prologue(const void* X, const TensorStrides& xs, void* Y, const TensorStrides& ys, int B, int H, int n_text, int gridH,
                              int gridW, int head_dim, const float* gain, float eps, const float* rope_y, const float* rope_x,
                              hipStream_t stream);
// mfma_peak.hip: sustained rate of back-to-back bf16 MFMAs on every SIMD, and the shader clock it ran at.
hipError_t measure_mfma_peak(int num_cus, double seconds, double* tflops, double* shader_mhz);

}  // namespace clear
