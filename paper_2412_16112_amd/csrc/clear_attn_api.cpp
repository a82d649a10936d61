// C ABI of the CLEAR local-attention library: argument checks, context, schedule upload, launch.
#include "../../include/clear_attn.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <algorithm>
#include <cstring>
#include <cstdlib>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "block_class.h"
#include "clear_internal.h"

using namespace clear;

// Tile lists of one raster and their copies on the device.
struct TileTables {
    Schedule sched;
    int* d_row_ptr = nullptr;
    int* d_col_idx = nullptr;   // kernel order: tiles inside the grid first, border tiles last
    int* d_n_plain = nullptr;
    int* d_qt_order = nullptr;   // bf16: the order in which a head's query tiles are dealt to the workgroups (see build_tile_tables)
    unsigned long long* d_mask_tbl = nullptr;
    int* d_wave_desc = nullptr;  // per listed key tile and wave: mask-table entries of its blocks (bf16, with d_mask_tbl)
    int mask_ry = 0, mask_rx = 0;
    void release()
    {
        if (d_row_ptr) (void)hipFree(d_row_ptr);
        if (d_col_idx) (void)hipFree(d_col_idx);
        if (d_n_plain) (void)hipFree(d_n_plain);
        if (d_qt_order) (void)hipFree(d_qt_order);
        if (d_mask_tbl) (void)hipFree(d_mask_tbl);
        if (d_wave_desc) (void)hipFree(d_wave_desc);
        d_row_ptr = d_col_idx = d_n_plain = d_qt_order = d_wave_desc = nullptr;
        d_mask_tbl = nullptr;
    }
};

struct clear_attn_ctx {
    int n_text = 0, gridH = 0, gridW = 0, head_dim = 0, r = 0, dtype = 0;
    int mask_kind = 0, mask_shift = 0;
    int device = 0;
    TileTables t;  // tile lists of the context's grid
    // Row bands whose first owned row is not a multiple of the query tile height: tile lists of the grid moved down
    // by 1 .. tile height - 1 rows, so that a tile row starts at the first owned row (built on first use).
    TileTables* band_t[kBf16QTileH > kF32QTileH ? kBf16QTileH : kF32QTileH] = {};
    int num_cus = 256;
    // text-query workspace, grown on demand
    int ws_BH = 0;         // capacity in (batch*head) units
    int ws_max_splits = 0;  // splits the workspace is sized for
    float* d_ws_o = nullptr;
    float* d_ws_ml = nullptr;
    // backward workspace, grown on demand
    int bwd_BH = 0;
    float* d_bwd_delta = nullptr;  // [B*H][N]
    float* d_bwd_ws = nullptr;     // [3][B*H][max splits][n_text][head_dim]
    // keys after the prologue (clear_attn_forward_prologue), grown on demand
    int kpro_BH = 0;
    void* d_kpro = nullptr;        // [B*H][N][head_dim] bf16
    void* scratch = nullptr;       // this device's copy of the static scratch array (clear_attn_forward_noalloc)
    std::string err;
};

static thread_local std::string g_create_error;

// Scratch of the entry point that allocates nothing (clear_attn_forward_noalloc): the key-split partial results of
// the text-query rows.  One copy per GPU, held from the first use of the library on that GPU until the process
// ends.  On the host `scratch` only names the symbol: its address on the current device comes from
// hipGetSymbolAddress (scratch_address below), and that pointer is what kernels and copies are given.
constexpr size_t kScratchBytes = (size_t)112 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];  // per device, filled on first use with that device current

// Device address of `scratch` on `device`, which must be the current device.
static hipError_t scratch_address(int device, void** out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

static int fail(clear_attn_ctx* ctx, int code, const std::string& msg)
{
    if (ctx) ctx->err = msg; else g_create_error = msg;
    return code;
}

// Whether work enqueued on `stream` is being recorded into a HIP graph (then nothing may allocate or synchronise).
static bool stream_is_capturing(hipStream_t stream)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}

static int check_shape(int n_text, int gridH, int gridW, int r, std::string* why)
{
    if (n_text < 0) { *why = "n_text must be >= 0"; return CLEAR_ERR_INVALID_ARG; }
    if (gridH < 1 || gridW < 1) { *why = "gridH and gridW must be >= 1"; return CLEAR_ERR_INVALID_ARG; }
    if (r < 1) { *why = "r must be >= 1"; return CLEAR_ERR_INVALID_ARG; }
    if (r > 32768) { *why = "r must be <= 32768"; return CLEAR_ERR_INVALID_ARG; }
    if (gridH > 32767 || gridW > 32767) { *why = "gridH and gridW must be <= 32767"; return CLEAR_ERR_INVALID_ARG; }
    if ((long long)gridH * gridW + n_text > 0x7fffffffLL) { *why = "n_text + gridH*gridW must fit in 31 bits"; return CLEAR_ERR_INVALID_ARG; }
    return CLEAR_OK;
}

static int check_kernel(int head_dim, int dtype, std::string* why)
{
    if (dtype != CLEAR_BF16 && dtype != CLEAR_F32) { *why = "dtype must be CLEAR_BF16 or CLEAR_F32"; return CLEAR_ERR_INVALID_ARG; }
    if (head_dim < 1) { *why = "head_dim must be >= 1"; return CLEAR_ERR_INVALID_ARG; }
    if (dtype == CLEAR_BF16 && (head_dim == 128 || head_dim == 64)) return CLEAR_OK;
    if (dtype == CLEAR_F32 && head_dim == 64) return CLEAR_OK;
    *why = "supported kernels: bf16 with head_dim 128 or 64, f32 with head_dim 64";
    return CLEAR_ERR_UNSUPPORTED;
}

// The maximum number of key splits of the text-query pass; the workspace is sized for it.
static int max_text_splits(long long N)
{
    // at least 512 keys per split, at most 64 splits
    long long s = (N + 511) / 512;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return (int)s;
}

// Splits for a given batch*heads: at least two workgroups per CU when the keys allow it, and a workgroup
// count that fills whole rounds of the CUs (a partial last round idles most of the chip).
// `together`: the text-query workgroups go out in one launch with the image-query ones (launch_all) and fill the CUs
// that those leave idle, so whole rounds do not matter; what then costs is the number of splits (partial results
// written, read back and merged) and the length of a text-query workgroup when it is the last to finish: one round
// of workgroups at most, of at least 2 048 keys each.  (Measured over 1 - 32 splits, 24 heads: 2 splits at a 64 x 64
// grid and 5 at 128 x 128 and 256 x 256 beat the whole-rounds choice of 5, 16 and 16 by 6 %, 8 % and 2 %.)
static void choose_text_splits(long long N, int BH, int n_tq_tiles, int num_cus, bool together, int* n_splits, int* split_keys)
{
    const int max_s = max_text_splits(N);
    const long long units = (long long)BH * n_tq_tiles;
    int best = 1;
    double best_score = -1.0;
    if (together && units < num_cus) {
        best = (int)std::min<long long>(max_s, num_cus / units);
        while (best > 1 && N / best < 2048) --best;
    } else {
        for (int s = 1; s <= max_s; ++s) {
            long long keys = (N + s - 1) / s;
            keys = ((keys + kKeyTileKeys - 1) / kKeyTileKeys) * kKeyTileKeys;
            const long long real = (N + keys - 1) / keys;  // splits that actually hold keys
            const long long wgs = units * real;
            const long long rounds = (wgs + num_cus - 1) / num_cus;
            double score = (double)wgs / (double)(rounds * num_cus);  // fraction of the rounds that is busy
            if (wgs < 2LL * num_cus) score *= 0.5;                    // too few workgroups to hide a workgroup's start-up
            if (score > best_score + 1e-9) {
                best_score = score;
                best = s;
            }
        }
    }
    long long keys = (N + best - 1) / best;
    keys = ((keys + kKeyTileKeys - 1) / kKeyTileKeys) * kKeyTileKeys;  // whole 64-key stages
    *split_keys = (int)keys;
    *n_splits = (int)((N + keys - 1) / keys);
}

// Builds the tile lists of a gridH x gridW raster for the kernels of (head_dim, dtype, mask) and copies them to the
// current device.  Returns CLEAR_OK, or an error code with *why set (the caller releases `t`).
static int build_tile_tables(int gridH, int gridW, int head_dim, int r, int dtype, int mask_kind, int shift, TileTables* t, std::string* why)
{
    const bool strided = mask_kind == CLEAR_MASK_STRIDED;
    int qth, qtw, kth, ktw;
    clear_attn_tile_shape(head_dim, dtype, &qth, &qtw, &kth, &ktw);
    // Strided: the tile lists describe one residue class, a (gridH / r) x (gridW / r) grid (rounded up) on which
    // every query tile meets every key tile; tiles count as inside the grid only if they are so for the
    // smallest class (extents rounded down).
    const int schedH = strided ? (gridH + r - 1) / r : gridH, schedW = strided ? (gridW + r - 1) / r : gridW;
    const int cutH = strided ? gridH / r : gridH, cutW = strided ? gridW / r : gridW;
    if (schedule_pair_bound(schedH, schedW, strided ? schedH + schedW : r, qth, qtw, kth, ktw) > kMaxSchedulePairs) {
        *why = "the tile schedule would exceed 2^28 (query tile, key tile) pairs: r is too close to the size of a grid this large";
        return CLEAR_ERR_UNSUPPORTED;
    }
    try {
        if (strided)
            build_schedule(schedH, schedW, schedH + schedW, qth, qtw, kth, ktw, &t->sched, CLEAR_MASK_DISC, 0);
        else
            build_schedule(gridH, gridW, r, qth, qtw, kth, ktw, &t->sched, mask_kind, shift);
    } catch (const std::bad_alloc&) {
        *why = "out of host memory building the schedule";
        return CLEAR_ERR_ALLOC;
    }
    // kernel-side tile lists: per query tile, the origins (row << 16 | col) of its key tiles, those inside the
    // grid first (mirror pairs adjacent), border tiles last
    std::vector<int> k_col(t->sched.col_idx.size()), n_plain(t->sched.row_ptr.size() - 1, 0);
    {
        const Schedule& sc = t->sched;
        auto cut = [&](int id) {
            const int ty = id / sc.n_ktx, tx = id % sc.n_ktx;
            return (ty + 1) * sc.kth > cutH || (tx + 1) * sc.ktw > cutW;
        };
        auto origin = [&](int id) { return ((id / sc.n_ktx) * sc.kth) << 16 | ((id % sc.n_ktx) * sc.ktw); };
        std::vector<int> plain, used;
        for (size_t qt = 0; qt + 1 < sc.row_ptr.size(); ++qt) {
            // Tiles inside the grid, reordered so that each stage (two consecutive tiles) holds a tile and its
            // point mirror through the centre of the query tile: what one wave's disc misses of the pair,
            // the wave sharing its SIMD tends to reach, which evens out the work between barriers.
            plain.clear();
            for (int e = sc.row_ptr[qt]; e < sc.row_ptr[qt + 1]; ++e)
                if (!cut(sc.col_idx[e])) plain.push_back(sc.col_idx[e]);
            used.assign(plain.size(), 0);
            const int qy0 = (int)(qt / sc.n_qtx) * sc.qth, qx0 = (int)(qt % sc.n_qtx) * sc.qtw;
            int w = sc.row_ptr[qt];
            std::vector<int> single;
            for (size_t i = 0; i < plain.size(); ++i) {
                if (used[i]) continue;
                used[i] = 1;
                const int ky = (plain[i] / sc.n_ktx) * sc.kth, kx = (plain[i] % sc.n_ktx) * sc.ktw;
                const int my = 2 * qy0 + sc.qth - sc.kth - ky, mx = 2 * qx0 + sc.qtw - sc.ktw - kx;
                int partner = -1;
                if (my >= 0 && mx >= 0 && my % sc.kth == 0 && mx % sc.ktw == 0) {
                    const int mid = (my / sc.kth) * sc.n_ktx + mx / sc.ktw;
                    for (size_t j = i + 1; j < plain.size(); ++j)
                        if (!used[j] && plain[j] == mid) { partner = (int)j; break; }
                }
                if (partner >= 0) {
                    used[partner] = 1;
                    k_col[w++] = origin(plain[i]);
                    k_col[w++] = origin(plain[partner]);
                } else {
                    single.push_back(plain[i]);
                }
            }
            for (int id : single) k_col[w++] = origin(id);
            n_plain[qt] = w - sc.row_ptr[qt];
            for (int e = sc.row_ptr[qt]; e < sc.row_ptr[qt + 1]; ++e)
                if (cut(sc.col_idx[e])) k_col[w++] = origin(sc.col_idx[e]);
        }
    }
    std::vector<unsigned long long> mask_tbl;
    if (dtype == CLEAR_BF16 && (mask_kind == CLEAR_MASK_DISC || mask_kind == CLEAR_MASK_SQUARE)) {
        // (masks that depend on the offset between the tokens alone; Swin windows take the arithmetic element mask)
        // relative block offsets that a non-empty (patch, block) pair can have
        t->mask_ry = std::min((r + 2) / 4, (gridH + 3) / 4);
        t->mask_rx = std::min((r + 6) / 8, (gridW + 7) / 8);
        const size_t entries = (size_t)(2 * t->mask_ry + 1) * (2 * t->mask_rx + 1) + 2;
        if (entries * 128 <= (64u << 20)) {  // beyond 64 MB the kernels fall back to arithmetic masks
            try {
                build_bf16_mask_table(r, t->mask_ry, t->mask_rx, mask_kind, &mask_tbl);
            } catch (const std::bad_alloc&) {
                *why = "out of host memory building the mask table";
                return CLEAR_ERR_ALLOC;
            }
        }
    }
    if (dtype == CLEAR_BF16 && mask_kind == CLEAR_MASK_SWIN && r % 8 == 0 && shift % 8 == 0) {
        // Windows whose edges fall on multiples of 8: a 4 x 8 query patch and a 4 x 8 key block each lie in one
        // window, so inside the grid a block is either wholly admitted or out of reach.  The table then only
        // needs its all-ones and all-zeros entries (the entry for offset (0, 0) in front of them is never used).
        t->mask_ry = t->mask_rx = 0;
        try {
            build_bf16_mask_table(r, 0, 0, mask_kind, &mask_tbl);
        } catch (const std::bad_alloc&) {
            *why = "out of host memory building the mask table";
            return CLEAR_ERR_ALLOC;
        }
    }
    std::vector<int> wave_desc;
    if (!mask_tbl.empty()) {
        // mask-table entries reach 16-bit indices only up to 65535; beyond that (r in the thousands) the kernels use arithmetic masks
        const size_t entries = mask_tbl.size() / 16;
        if (entries <= 0xffff && k_col.size() * (size_t)(kBf16NWY * kBf16NWX) * sizeof(int) <= ((size_t)256 << 20)) {
            try {
                build_wave_descriptors(t->sched, k_col, n_plain, t->mask_ry, t->mask_rx, &wave_desc);
            } catch (const std::bad_alloc&) {
                *why = "out of host memory building the per-wave tile descriptors";
                return CLEAR_ERR_ALLOC;
            }
        } else {
            mask_tbl.clear();
        }
    }
    // Order of a head's query tiles over its workgroups.  An XCD (32 CUs, one workgroup each, one 4 MB L2) works through
    // a contiguous range of that order, so the tiles in flight on it are 32 consecutive entries.  Row by row on a wide
    // grid they are a 1 x 32 strip of tiles, whose keys - 16 + 2 (r - 1) rows across 512 columns - the next strip
    // needs again but finds evicted.  Dealt out in blocks of 2 x 16 tiles, strips of 16 tile columns taken top to
    // bottom, the tiles in flight form a more compact patch: a quarter fewer L2 misses at a 512 x 512 grid (18.9 ->
    // 14.1 GB per launch of 24 heads), same time.  Grids up to 16 tiles wide keep the plain order (no table).
    constexpr int kOrderRows = 2, kOrderCols = 16;
    std::vector<int> qt_order;
    if (dtype == CLEAR_BF16 && !strided && t->sched.n_qtx > kOrderCols) {
        const Schedule& sc = t->sched;
        try {
            qt_order.reserve((size_t)sc.n_qty * sc.n_qtx);
            for (int bx = 0; bx < sc.n_qtx; bx += kOrderCols)
                for (int by = 0; by < sc.n_qty; by += kOrderRows)
                    for (int ty = by; ty < std::min(by + kOrderRows, sc.n_qty); ++ty)
                        for (int tx = bx; tx < std::min(bx + kOrderCols, sc.n_qtx); ++tx) qt_order.push_back(ty * sc.n_qtx + tx);
        } catch (const std::bad_alloc&) {
            *why = "out of host memory building the query-tile order";
            return CLEAR_ERR_ALLOC;
        }
    }
    hipError_t e = hipSuccess;
    if (e == hipSuccess && !qt_order.empty()) {
        e = hipMalloc((void**)&t->d_qt_order, qt_order.size() * sizeof(int));
        if (e == hipSuccess) e = hipMemcpy(t->d_qt_order, qt_order.data(), qt_order.size() * sizeof(int), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipMalloc((void**)&t->d_row_ptr, t->sched.row_ptr.size() * sizeof(int));
    if (e == hipSuccess) e = hipMalloc((void**)&t->d_col_idx, (k_col.size() + 1) * sizeof(int));
    if (e == hipSuccess) e = hipMalloc((void**)&t->d_n_plain, (n_plain.size() + 1) * sizeof(int));
    if (e == hipSuccess) e = hipMemcpy(t->d_row_ptr, t->sched.row_ptr.data(), t->sched.row_ptr.size() * sizeof(int), hipMemcpyHostToDevice);
    if (e == hipSuccess && !k_col.empty()) e = hipMemcpy(t->d_col_idx, k_col.data(), k_col.size() * sizeof(int), hipMemcpyHostToDevice);
    if (e == hipSuccess && !n_plain.empty()) e = hipMemcpy(t->d_n_plain, n_plain.data(), n_plain.size() * sizeof(int), hipMemcpyHostToDevice);
    if (e == hipSuccess && !mask_tbl.empty()) {
        e = hipMalloc((void**)&t->d_mask_tbl, mask_tbl.size() * sizeof(unsigned long long));
        if (e == hipSuccess) e = hipMemcpy(t->d_mask_tbl, mask_tbl.data(), mask_tbl.size() * sizeof(unsigned long long), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && !wave_desc.empty()) {
        e = hipMalloc((void**)&t->d_wave_desc, wave_desc.size() * sizeof(int));
        if (e == hipSuccess) e = hipMemcpy(t->d_wave_desc, wave_desc.data(), wave_desc.size() * sizeof(int), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        *why = std::string("HIP error building the tile lists: ") + hipGetErrorString(e);
        (void)hipGetLastError();
        return e == hipErrorOutOfMemory ? CLEAR_ERR_ALLOC : CLEAR_ERR_HIP;
    }
    return CLEAR_OK;
}

extern "C" {

int clear_attn_mask_count(int n_text, int gridH, int gridW, int r, unsigned long long* sumM)
{
    std::string why;
    if (!sumM) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "sumM is NULL");
    int rc = check_shape(n_text, gridH, gridW, r, &why);
    if (rc != CLEAR_OK) return fail(nullptr, rc, why);
    *sumM = mask_count(n_text, gridH, gridW, r);
    return CLEAR_OK;
}

int clear_attn_tile_shape(int head_dim, int dtype, int* q_tile_h, int* q_tile_w, int* k_tile_h, int* k_tile_w)
{
    std::string why;
    int rc = check_kernel(head_dim, dtype, &why);
    if (rc != CLEAR_OK) return fail(nullptr, rc, why);
    if (!q_tile_h || !q_tile_w || !k_tile_h || !k_tile_w) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "NULL output pointer");
    if (dtype == CLEAR_BF16) { *q_tile_h = kBf16QTileH; *q_tile_w = kBf16QTileW; }
    else { *q_tile_h = kF32QTileH; *q_tile_w = kF32QTileW; }
    *k_tile_h = kKeyTileH;
    *k_tile_w = kKeyTileW;
    return CLEAR_OK;
}

static int check_mask(int mask_kind, int r, int shift, std::string* why);

int clear_attn_schedule_host(int gridH, int gridW, int r, int q_tile_h, int q_tile_w, int k_tile_h, int k_tile_w,
                             int* n_q_tiles, long long* n_pairs, int* row_ptr, int* col_idx, unsigned char* flags)
{
    return clear_attn_schedule_host_masked(gridH, gridW, r, CLEAR_MASK_DISC, 0, q_tile_h, q_tile_w, k_tile_h, k_tile_w, n_q_tiles, n_pairs,
                                           row_ptr, col_idx, flags);
}

int clear_attn_schedule_host_masked(int gridH, int gridW, int r, int mask_kind, int shift, int q_tile_h, int q_tile_w, int k_tile_h,
                                    int k_tile_w, int* n_q_tiles, long long* n_pairs, int* row_ptr, int* col_idx, unsigned char* flags)
{
    std::string why;
    int rc = check_shape(0, gridH, gridW, r, &why);
    if (rc == CLEAR_OK) rc = check_mask(mask_kind, r, shift, &why);
    if (rc != CLEAR_OK) return fail(nullptr, rc, why);
    if (q_tile_h < 1 || q_tile_w < 1 || k_tile_h < 1 || k_tile_w < 1) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "tile sizes must be >= 1");
    if (mask_kind == CLEAR_MASK_STRIDED)
        return fail(nullptr, CLEAR_ERR_UNSUPPORTED, "the strided mask has no tile schedule on the raster grid: it runs as one dense problem per residue class");
    if (!n_q_tiles || !n_pairs) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "n_q_tiles / n_pairs is NULL");
    if (schedule_pair_bound(gridH, gridW, r, q_tile_h, q_tile_w, k_tile_h, k_tile_w) > kMaxSchedulePairs)
        return fail(nullptr, CLEAR_ERR_UNSUPPORTED, "the tile schedule would exceed 2^28 (query tile, key tile) pairs");
    const bool sizes_only = !row_ptr && !col_idx && !flags;
    if (!sizes_only && (!row_ptr || !col_idx || !flags)) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "row_ptr, col_idx and flags must be all NULL or all set");
    Schedule s;
    try {
        build_schedule(gridH, gridW, r, q_tile_h, q_tile_w, k_tile_h, k_tile_w, &s, mask_kind, shift);
    } catch (const std::bad_alloc&) {
        return fail(nullptr, CLEAR_ERR_ALLOC, "out of host memory building the schedule");
    }
    *n_q_tiles = (int)s.row_ptr.size() - 1;
    *n_pairs = (long long)s.col_idx.size();
    if (!sizes_only) {
        memcpy(row_ptr, s.row_ptr.data(), s.row_ptr.size() * sizeof(int));
        memcpy(col_idx, s.col_idx.data(), s.col_idx.size() * sizeof(int));
        memcpy(flags, s.flags.data(), s.flags.size());
    }
    return CLEAR_OK;
}

static int check_mask(int mask_kind, int r, int shift, std::string* why)
{
    if (mask_kind != CLEAR_MASK_DISC && mask_kind != CLEAR_MASK_SQUARE && mask_kind != CLEAR_MASK_SWIN && mask_kind != CLEAR_MASK_STRIDED) {
        *why = "mask_kind must be CLEAR_MASK_DISC, CLEAR_MASK_SQUARE, CLEAR_MASK_SWIN or CLEAR_MASK_STRIDED";
        return CLEAR_ERR_INVALID_ARG;
    }
    if (mask_kind == CLEAR_MASK_STRIDED) {
        if (shift < 0) { *why = "the layer index given as shift must be >= 0 for CLEAR_MASK_STRIDED"; return CLEAR_ERR_INVALID_ARG; }
        return CLEAR_OK;
    }
    if (mask_kind == CLEAR_MASK_SWIN ? (shift < 0 || shift >= r) : shift != 0) { *why = "shift must be 0, or in [0, r) for CLEAR_MASK_SWIN"; return CLEAR_ERR_INVALID_ARG; }
    return CLEAR_OK;
}

int clear_attn_create(clear_attn_ctx** out, int n_text, int gridH, int gridW, int head_dim, int r, int dtype)
{
    return clear_attn_create_masked(out, n_text, gridH, gridW, head_dim, r, dtype, CLEAR_MASK_DISC, 0);
}

int clear_attn_mask_count_masked(int n_text, int gridH, int gridW, int r, int mask_kind, int shift, unsigned long long* sumM)
{
    std::string why;
    if (!sumM) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "sumM is NULL");
    int rc = check_shape(n_text, gridH, gridW, r, &why);
    if (rc == CLEAR_OK) rc = check_mask(mask_kind, r, shift, &why);
    if (rc != CLEAR_OK) return fail(nullptr, rc, why);
    *sumM = mask_count(n_text, gridH, gridW, r, mask_kind, shift);
    return CLEAR_OK;
}

int clear_attn_create_masked(clear_attn_ctx** out, int n_text, int gridH, int gridW, int head_dim, int r, int dtype,
                             int mask_kind, int shift)
{
    std::string why;
    if (!out) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "out is NULL");
    int rc = check_shape(n_text, gridH, gridW, r, &why);
    if (rc != CLEAR_OK) return fail(nullptr, rc, why);
    rc = check_kernel(head_dim, dtype, &why);
    if (rc != CLEAR_OK) return fail(nullptr, rc, why);
    rc = check_mask(mask_kind, r, shift, &why);
    if (rc != CLEAR_OK) return fail(nullptr, rc, why);

    if (dtype == CLEAR_BF16 && (long long)n_text + (long long)gridH * gridW > (1LL << 24) - 1)
        return fail(nullptr, CLEAR_ERR_UNSUPPORTED, "bf16 kernels address one head with 32-bit byte offsets: n_text + gridH*gridW must be < 2^24");

    const bool strided = mask_kind == CLEAR_MASK_STRIDED;
    if (strided && dtype != CLEAR_BF16) return fail(nullptr, CLEAR_ERR_UNSUPPORTED, "the strided mask is built for the bf16 kernels only");
    if (strided && (gridH < r || gridW < r))
        return fail(nullptr, CLEAR_ERR_UNSUPPORTED, "the strided mask needs gridH >= r and gridW >= r (every residue class non-empty)");

    clear_attn_ctx* ctx = new (std::nothrow) clear_attn_ctx;
    if (!ctx) return fail(nullptr, CLEAR_ERR_ALLOC, "out of host memory");
    ctx->n_text = n_text; ctx->gridH = gridH; ctx->gridW = gridW;
    ctx->head_dim = head_dim; ctx->r = r; ctx->dtype = dtype;
    ctx->mask_kind = mask_kind; ctx->mask_shift = shift;
    rc = build_tile_tables(gridH, gridW, head_dim, r, dtype, mask_kind, shift, &ctx->t, &why);
    if (rc != CLEAR_OK) {
        clear_attn_destroy(ctx);
        return fail(nullptr, rc, why);
    }
    hipError_t e = hipGetDevice(&ctx->device);
    if (e == hipSuccess) {
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, ctx->device);
        if (e == hipSuccess && prop.multiProcessorCount > 0) ctx->num_cus = prop.multiProcessorCount;
    }
    if (e == hipSuccess) e = scratch_address(ctx->device, &ctx->scratch);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        std::string msg = std::string("HIP error in create: ") + hipGetErrorString(e);
        const int code = (e == hipErrorOutOfMemory) ? CLEAR_ERR_ALLOC : CLEAR_ERR_HIP;
        clear_attn_destroy(ctx);
        return fail(nullptr, code, msg);
    }
    *out = ctx;
    return CLEAR_OK;
}

int clear_attn_reserve(clear_attn_ctx* ctx, int BH)
{
    if (!ctx) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "ctx is NULL");
    if (BH < 1) return fail(ctx, CLEAR_ERR_INVALID_ARG, "BH must be >= 1");
    if (ctx->n_text == 0 || BH <= ctx->ws_BH) return CLEAR_OK;
    const long long N = (long long)ctx->n_text + (long long)ctx->gridH * ctx->gridW;
    const int splits = max_text_splits(N);
    hipError_t e = hipDeviceSynchronize();  // a running forward may still use the old workspace
    if (e == hipSuccess && ctx->d_ws_o) e = hipFree(ctx->d_ws_o);
    if (e == hipSuccess && ctx->d_ws_ml) e = hipFree(ctx->d_ws_ml);
    ctx->d_ws_o = ctx->d_ws_ml = nullptr;
    ctx->ws_BH = 0;
    const size_t rows = (size_t)BH * splits * ctx->n_text;
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->d_ws_o, rows * ctx->head_dim * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->d_ws_ml, rows * 2 * sizeof(float));
    if (e != hipSuccess) {
        if (ctx->d_ws_o) (void)hipFree(ctx->d_ws_o);
        ctx->d_ws_o = nullptr;
        (void)hipGetLastError();
        return fail(ctx, e == hipErrorOutOfMemory ? CLEAR_ERR_ALLOC : CLEAR_ERR_HIP,
                    std::string("workspace allocation failed: ") + hipGetErrorString(e));
    }
    ctx->ws_BH = BH;
    ctx->ws_max_splits = splits;
    return CLEAR_OK;
}

// Whether a forward call sends its image-query and text-query workgroups out in one launch (see launch_all).
static bool launches_together(const clear_attn_ctx* ctx, const FwdParams& p)
{
    const long long image_wgs = (long long)p.B * p.H * p.n_classes * p.n_q_tiles_launch;
    return ctx->dtype == CLEAR_BF16 && p.n_text > 0 && image_wgs <= 64LL * ctx->num_cus;
}

// Tile lists of the context's grid moved down by y_shift rows (row bands; see prepare_forward), built on first use.
static int band_tile_tables(clear_attn_ctx* ctx, int y_shift, hipStream_t stream, const TileTables** out)
{
    TileTables*& slot = ctx->band_t[y_shift];
    if (!slot) {
        if (stream_is_capturing(stream))
            return fail(ctx, CLEAR_ERR_INVALID_ARG, "the tile lists of this band's first owned row would have to be built while the stream is being captured: make one call with the same own_y0 beforehand");
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
            return fail(ctx, CLEAR_ERR_INVALID_ARG, "the context's device must be current");
        TileTables* t = new (std::nothrow) TileTables;
        if (!t) return fail(ctx, CLEAR_ERR_ALLOC, "out of host memory");
        std::string why;
        const int rc = build_tile_tables(ctx->gridH + y_shift, ctx->gridW, ctx->head_dim, ctx->r, ctx->dtype, ctx->mask_kind, ctx->mask_shift, t, &why);
        if (rc != CLEAR_OK) {
            t->release();
            delete t;
            return fail(ctx, rc, why);
        }
        slot = t;
    }
    *out = slot;
    return CLEAR_OK;
}

// Validates the arguments of a forward call and fills the kernel parameters.
// band == nullptr: the whole grid.
struct BandArgs {
    int own_y0, own_y1;  // image rows [own_y0, own_y1) of the context's grid carry queries; the rest is halo
    int text_keys;       // whether the text queries see the text keys in this band
    float* text_o;
    float* text_lse;
};

static int prepare_forward(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, int B, int H,
                           int n_text, int gridH, int gridW, int head_dim, int r, const BandArgs* band, FwdParams* out,
                           void* stream, const long long* strides = nullptr, bool noalloc = false)
{
    if (!ctx) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "ctx is NULL");
    if (!Q || !K || !V || !O) return fail(ctx, CLEAR_ERR_INVALID_ARG, "Q, K, V, O must be non-NULL");
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15) return fail(ctx, CLEAR_ERR_INVALID_ARG, "Q, K, V, O must be 16-byte aligned");
    if (B < 1 || H < 1) return fail(ctx, CLEAR_ERR_INVALID_ARG, "B and H must be >= 1");
    if ((long long)B * H > 65535) return fail(ctx, CLEAR_ERR_INVALID_ARG, "B*H must be <= 65535");
    if (n_text != ctx->n_text || gridH != ctx->gridH || gridW != ctx->gridW || head_dim != ctx->head_dim || r != ctx->r)
        return fail(ctx, CLEAR_ERR_MISMATCH, "shape arguments differ from those given to clear_attn_create");
    const long long N = (long long)n_text + (long long)gridH * gridW;
    TensorStrides ts[4];  // Q, K, V, O
    for (int t = 0; t < 4; ++t) {
        ts[t].sn = strides ? strides[3 * t + 2] : head_dim;
        ts[t].sh = strides ? strides[3 * t + 1] : N * head_dim;
        ts[t].sb = strides ? strides[3 * t] : (long long)H * N * head_dim;
    }
    if (strides) {
        if (ctx->dtype != CLEAR_BF16) return fail(ctx, CLEAR_ERR_UNSUPPORTED, "strided tensors are built for the bf16 kernels only");
        if (band) return fail(ctx, CLEAR_ERR_UNSUPPORTED, "row bands take the plain layout");
        for (int t = 0; t < 4; ++t) {
            if (ts[t].sn < head_dim || ts[t].sh < 0 || ts[t].sb < 0 || (t == 3 && (ts[t].sh <= 0 || (B > 1 && ts[t].sb <= 0))))
                return fail(ctx, CLEAR_ERR_INVALID_ARG, "strides: the token stride must be >= head_dim, the others >= 0 (> 0 for O)");
            if ((ts[t].sn | ts[t].sh | ts[t].sb) & 7) return fail(ctx, CLEAR_ERR_INVALID_ARG, "strides must be multiples of 8 elements (16-byte rows)");
        }
        for (int t = 1; t <= 2; ++t)
            if ((N - 1) * ts[t].sn * 2 + 2 * head_dim > 0xffffffffLL)
                return fail(ctx, CLEAR_ERR_UNSUPPORTED, "K and V are addressed with 32-bit byte offsets inside one head: N * token stride * 2 must be < 2^32");
    }
    {
        // O must not overlap an input (compared by the address ranges the tensors span)
        const size_t esz = ctx->dtype == CLEAR_BF16 ? 2 : 4;
        auto span = [&](const TensorStrides& st) { return (size_t)((B - 1) * st.sb + (H - 1) * st.sh + (N - 1) * st.sn + head_dim) * esz; };
        const uintptr_t o0 = (uintptr_t)O, o1 = o0 + span(ts[3]);
        const void* ins[3] = {Q, K, V};
        for (int t = 0; t < 3; ++t) {
            const uintptr_t i0 = (uintptr_t)ins[t], i1 = i0 + span(ts[t]);
            if (o0 < i1 && i0 < o1) return fail(ctx, CLEAR_ERR_INVALID_ARG, "O overlaps an input tensor");
        }
    }
    if (band) {
        if (band->own_y0 < 0 || band->own_y0 >= band->own_y1 || band->own_y1 > gridH)
            return fail(ctx, CLEAR_ERR_INVALID_ARG, "band rows must satisfy 0 <= own_y0 < own_y1 <= gridH");
        if (n_text > 0 && (!band->text_o || !band->text_lse)) return fail(ctx, CLEAR_ERR_INVALID_ARG, "text_o and text_lse must be non-NULL when n_text > 0");
        if (n_text > 0 && (((uintptr_t)band->text_o | (uintptr_t)band->text_lse) & 3)) return fail(ctx, CLEAR_ERR_INVALID_ARG, "text_o and text_lse must be 4-byte aligned");
    }
    const int BH = B * H;
    // A band whose first owned row is not on the query-tile lattice takes tile lists of the grid moved down by y_shift
    // rows, so that a tile row starts at that row and no workgroup straddles the cut (an owned range starting at row
    // 15 would otherwise launch five tile rows for four).  The rows above the grid are not masked, so every owned
    // query's reach (r - 1 rows) must stay inside the grid: own_y0 >= r - 1, which the halo of an inner band gives.
    const TileTables* tt = &ctx->t;
    int y_shift = 0;
    if (band && ctx->dtype == CLEAR_BF16 && ctx->mask_kind == CLEAR_MASK_DISC) {
        const int qth = ctx->t.sched.qth, rem = band->own_y0 % qth;
        if (rem != 0 && band->own_y0 >= r - 1 && gridH + qth - rem <= 32767) {
            y_shift = qth - rem;
            int rc = band_tile_tables(ctx, y_shift, (hipStream_t)stream, &tt);
            if (rc != CLEAR_OK) return rc;
        }
    }
    const Schedule& s = tt->sched;
    const long long n_q_tiles = (long long)s.n_qty * s.n_qtx;
    if (n_q_tiles * BH > 0x7fffffffLL) return fail(ctx, CLEAR_ERR_INVALID_ARG, "too many workgroups: B*H*query tiles must fit in 31 bits");

    FwdParams p;
    memset(&p, 0, sizeof(p));
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.qs = ts[0]; p.ks = ts[1]; p.vs = ts[2]; p.os = ts[3];
    p.B = B; p.H = H; p.n_text = n_text; p.gridH = gridH; p.gridW = gridW; p.r2 = r * r;
    p.N = N;
    p.n_q_tiles = (int)n_q_tiles;
    p.n_qtx = s.n_qtx;
    p.n_ktx = s.n_ktx;
    p.row_ptr = tt->d_row_ptr;
    p.col_idx = tt->d_col_idx;
    p.n_plain = tt->d_n_plain;
    p.qt_order = band ? nullptr : tt->d_qt_order;  // (a band launches a range of tile rows)
    p.mask_tbl = tt->d_mask_tbl;
    p.wave_desc = tt->d_wave_desc;
    p.mask_ry = tt->mask_ry;
    p.mask_rx = tt->mask_rx;
    p.y_shift = y_shift;
    p.mask_kind = ctx->mask_kind; p.mask_r = r; p.mask_shift = ctx->mask_shift;
    p.n_classes = 1; p.stride = 1; p.stride_rx = p.stride_ry = 0;
    if (ctx->mask_kind == CLEAR_MASK_STRIDED) {
        if (band) return fail(ctx, CLEAR_ERR_UNSUPPORTED, "row bands are not built for the strided mask");
        p.mask_kind = kMaskFull;  // inside a residue class every pair is admitted
        p.n_classes = r * r; p.stride = r;
        p.stride_rx = ctx->mask_shift % r; p.stride_ry = (ctx->mask_shift / r) % r;
        if (n_q_tiles * BH * p.n_classes > 0x7fffffffLL) return fail(ctx, CLEAR_ERR_INVALID_ARG, "too many workgroups: B*H*r*r*query tiles must fit in 31 bits");
    }
    p.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)head_dim));
    p.own_y0 = 0;
    p.own_y1 = gridH;
    p.qt_begin = 0;
    p.n_q_tiles_launch = (int)n_q_tiles;
    p.NV = N;
    p.vkeys_text = 0x7fffffff;
    p.vshift = 0;
    if (band) {
        p.own_y0 = band->own_y0 + y_shift;  // in tile coordinates
        p.own_y1 = band->own_y1 + y_shift;
        const int ty0 = p.own_y0 / s.qth, ty1 = (p.own_y1 + s.qth - 1) / s.qth;  // tile rows that hold owned rows
        p.qt_begin = ty0 * s.n_qtx;
        p.n_q_tiles_launch = (ty1 - ty0) * s.n_qtx;
        // keys of the text queries: [the text keys,] then the owned image rows
        p.vkeys_text = band->text_keys ? n_text : 0;
        p.NV = (long long)p.vkeys_text + (long long)(band->own_y1 - band->own_y0) * gridW;
        p.vshift = (int)((long long)n_text + (long long)band->own_y0 * gridW - p.vkeys_text);
        p.band_o = band->text_o;
        p.band_lse = band->text_lse;
    }
    if (n_text > 0) {
        const int per_block = ctx->dtype == CLEAR_BF16 ? bf16_text_queries_per_block() : f32_text_queries_per_block();
        p.n_tq_tiles = (n_text + per_block - 1) / per_block;
        choose_text_splits(p.NV, BH, p.n_tq_tiles, ctx->num_cus, launches_together(ctx, p), &p.n_splits, &p.split_keys);
        if (noalloc) {
            // partial outputs, then (maximum, denominator) pairs, both inside the static scratch array
            const size_t rows = (size_t)BH * p.n_splits * n_text;
            const size_t o_bytes = (rows * head_dim * sizeof(float) + 255) & ~(size_t)255, ml_bytes = rows * 2 * sizeof(float);
            if (o_bytes + ml_bytes > kScratchBytes)
                return fail(ctx, CLEAR_ERR_UNSUPPORTED,
                            "clear_attn_forward_noalloc: the text-query partial results need " + std::to_string(o_bytes + ml_bytes) +
                                " bytes, the static scratch array holds " + std::to_string(kScratchBytes) +
                                " (B*H * key splits * n_text * (head_dim + 2) floats); use clear_attn_forward");
            p.ws_o = (float*)ctx->scratch;
            p.ws_ml = (float*)((unsigned char*)ctx->scratch + o_bytes);
        } else {
            if (BH > ctx->ws_BH && stream_is_capturing((hipStream_t)stream))
                return fail(ctx, CLEAR_ERR_INVALID_ARG, "the text-query workspace would have to grow while the stream is being captured: call clear_attn_reserve beforehand");
            int rc = clear_attn_reserve(ctx, BH);
            if (rc != CLEAR_OK) return rc;
            if (p.n_splits > ctx->ws_max_splits) return fail(ctx, CLEAR_ERR_HIP, "internal: split count exceeds workspace");
            p.ws_o = ctx->d_ws_o;
            p.ws_ml = ctx->d_ws_ml;
        }
    }
    *out = p;
    return CLEAR_OK;
}

static hipError_t launch(const clear_attn_ctx* ctx, const FwdParams& p, hipStream_t stream, int phase)
{
    if (ctx->dtype == CLEAR_BF16) return ctx->head_dim == 128 ? launch_bf16_d128(p, stream, phase) : launch_bf16_d64(p, stream, phase);
    return launch_f32_d64(p, stream, phase);
}

// A whole forward pass.  The image-query rows and the text-query rows are independent (they read Q, K, V and
// write disjoint rows of O).  Up to 64 image-query workgroups per CU the two go out as one launch, image-query
// workgroups first: the text-query workgroups then fill the CUs that the last round of image-query workgroups
// leaves idle, and a launch is saved.  Measured against one launch after the other (bit-identical output): 12 %
// faster at a 64 x 64 grid, 5 % at 128 x 128, 0.5 % at 256 x 256, 7 % at head_dim 64 on 256 x 256 with 38 heads;
// at 512 x 512 x 24 heads (96 workgroups per CU) 0.6 % slower, so the largest problems keep two launches.  (An
// earlier version ran the text-query kernels on a second stream beside the image-query kernel: slower than this
// at every size, and a stream and two events to create.)
static hipError_t launch_all(clear_attn_ctx* ctx, const FwdParams& p, hipStream_t stream)
{
    if (!launches_together(ctx, p)) return launch(ctx, p, stream, kPhaseAll);
    hipError_t e = launch(ctx, p, stream, kPhaseImageAndTextQuery);
    if (e == hipSuccess) e = launch(ctx, p, stream, kPhaseTextMerge);
    return e;
}

int clear_attn_forward(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, int B, int H,
                       int n_text, int gridH, int gridW, int head_dim, int r, void* stream)
{
    FwdParams p;
    int rc = prepare_forward(ctx, Q, K, V, O, B, H, n_text, gridH, gridW, head_dim, r, nullptr, &p, stream);
    if (rc != CLEAR_OK) return rc;
    hipError_t e = launch_all(ctx, p, (hipStream_t)stream);
    if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

int clear_attn_forward_noalloc(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, int B, int H,
                               int n_text, int gridH, int gridW, int head_dim, int r, void* stream)
{
    if (!ctx) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "ctx is NULL");
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
        return fail(ctx, CLEAR_ERR_INVALID_ARG, "clear_attn_forward_noalloc: the context's device must be current (the scratch array is per device)");
    if (!ctx->scratch) return fail(ctx, CLEAR_ERR_HIP, "internal: the scratch array has no address on this device");
    FwdParams p;
    int rc = prepare_forward(ctx, Q, K, V, O, B, H, n_text, gridH, gridW, head_dim, r, nullptr, &p, stream, nullptr, true);
    if (rc != CLEAR_OK) return rc;
    // Nothing in the scratch array has to start at zero: the text-query kernel writes every (split, row) entry
    // that the merge reads.
    hipError_t e = launch_all(ctx, p, (hipStream_t)stream);
    if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

int clear_attn_forward_strided(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, float* lse,
                               const long long* strides, int B, int H, int n_text, int gridH, int gridW, int head_dim, int r, void* stream)
{
    if (!strides) return fail(ctx, CLEAR_ERR_INVALID_ARG, "strides is NULL");
    FwdParams p;
    int rc = prepare_forward(ctx, Q, K, V, O, B, H, n_text, gridH, gridW, head_dim, r, nullptr, &p, stream, strides);
    if (rc != CLEAR_OK) return rc;
    if ((uintptr_t)lse & 3) return fail(ctx, CLEAR_ERR_INVALID_ARG, "lse must be 4-byte aligned");
    p.lse = lse;
    hipError_t e = launch_all(ctx, p, (hipStream_t)stream);
    if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

int clear_attn_forward_profile(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, int B, int H,
                               int n_text, int gridH, int gridW, int head_dim, int r, void* stream, int reps,
                               float* phase_ms)
{
    FwdParams p;
    int rc = prepare_forward(ctx, Q, K, V, O, B, H, n_text, gridH, gridW, head_dim, r, nullptr, &p, stream);
    if (rc != CLEAR_OK) return rc;
    if (!phase_ms || reps < 1 || reps > 256) return fail(ctx, CLEAR_ERR_INVALID_ARG, "phase_ms must be non-NULL and 1 <= reps <= 256");
    // The three kernels are timed inside the sequence they run in (image, text, merge, image, ...): timed
    // one kind at a time they would each run at the clock that kind settles at, not at the one the mix gets.
    hipStream_t st = (hipStream_t)stream;
    std::vector<hipEvent_t> ev((size_t)reps * 4, nullptr);
    hipError_t e = hipSuccess;
    for (size_t i = 0; i < ev.size() && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
    const bool text = n_text > 0;
    for (int i = 0; i < reps && e == hipSuccess; ++i) {
        hipEvent_t* v = &ev[(size_t)i * 4];
        e = hipEventRecord(v[0], st);
        if (e == hipSuccess) e = launch(ctx, p, st, kPhaseImage);
        if (e == hipSuccess) e = hipEventRecord(v[1], st);
        if (e == hipSuccess && text) e = launch(ctx, p, st, kPhaseTextQuery);
        if (e == hipSuccess) e = hipEventRecord(v[2], st);
        if (e == hipSuccess && text) e = launch(ctx, p, st, kPhaseTextMerge);
        if (e == hipSuccess) e = hipEventRecord(v[3], st);
    }
    if (e == hipSuccess) e = hipEventSynchronize(ev.back());
    phase_ms[0] = phase_ms[1] = phase_ms[2] = 0.f;
    for (int i = 0; i < reps && e == hipSuccess; ++i)
        for (int ph = 0; ph < 3 && e == hipSuccess; ++ph) {
            float ms = 0.f;
            e = hipEventElapsedTime(&ms, ev[(size_t)i * 4 + ph], ev[(size_t)i * 4 + ph + 1]);
            phase_ms[ph] += ms / (float)reps;
        }
    for (hipEvent_t x : ev)
        if (x) (void)hipEventDestroy(x);
    if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("profile run failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

int clear_attn_forward_lse(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, float* lse, int B, int H,
                           int n_text, int gridH, int gridW, int head_dim, int r, void* stream)
{
    FwdParams p;
    int rc = prepare_forward(ctx, Q, K, V, O, B, H, n_text, gridH, gridW, head_dim, r, nullptr, &p, stream);
    if (rc != CLEAR_OK) return rc;
    if (!lse || ((uintptr_t)lse & 3)) return fail(ctx, CLEAR_ERR_INVALID_ARG, "lse must be non-NULL and 4-byte aligned");
    p.lse = lse;
    hipError_t e = launch_all(ctx, p, (hipStream_t)stream);
    if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

// Arguments of the query/key prologue shared by the two entry points below.
static int check_prologue(clear_attn_ctx* ctx, int head_dim, const float* gain_a, const float* gain_b, float eps, const float* rope_y,
                          const float* rope_x)
{
    if (head_dim % 8 != 0) return fail(ctx, CLEAR_ERR_UNSUPPORTED, "the prologue needs head_dim to be a multiple of 8");
    if ((rope_y == nullptr) != (rope_x == nullptr)) return fail(ctx, CLEAR_ERR_INVALID_ARG, "rope_y and rope_x must be given together");
    if (((uintptr_t)gain_a | (uintptr_t)gain_b | (uintptr_t)rope_y | (uintptr_t)rope_x) & 15)
        return fail(ctx, CLEAR_ERR_INVALID_ARG, "gains and rotary tables must be 16-byte aligned");
    if ((gain_a || gain_b) && !(eps >= 0.f)) return fail(ctx, CLEAR_ERR_INVALID_ARG, "norm_eps must be >= 0");
    return CLEAR_OK;
}

int clear_attn_qk_prologue(const void* X, void* Y, int B, int H, int n_text, int gridH, int gridW, int head_dim, const float* gain,
                           float norm_eps, const float* rope_y, const float* rope_x, void* stream)
{
    if (!X || !Y) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "X and Y must be non-NULL");
    if (((uintptr_t)X | (uintptr_t)Y) & 15) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "X and Y must be 16-byte aligned");
    if (B < 1 || H < 1) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "B and H must be >= 1");
    if (n_text < 0 || gridH < 0 || gridW < 0) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "n_text, gridH, gridW must be >= 0");
    if (head_dim != 64 && head_dim != 128) return fail(nullptr, CLEAR_ERR_UNSUPPORTED, "the prologue is built for head_dim 64 and 128");
    int rc = check_prologue(nullptr, head_dim, gain, nullptr, norm_eps, rope_y, rope_x);
    if (rc != CLEAR_OK) return rc;
    const long long N = (long long)n_text + (long long)gridH * gridW;
    if (X != Y) {
        const size_t bytes = (size_t)B * H * N * head_dim * 2;
        const uintptr_t x0 = (uintptr_t)X, y0 = (uintptr_t)Y;
        if (x0 < y0 + bytes && y0 < x0 + bytes) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "X and Y must be the same tensor or must not overlap");
    }
    const TensorStrides plain = {(long long)H * N * head_dim, N * head_dim, head_dim};
    hipError_t e = launch_qk_prologue(X, plain, Y, plain, B, H, n_text, gridH, gridW, head_dim, gain, norm_eps, rope_y, rope_x, (hipStream_t)stream);
    if (e != hipSuccess) return fail(nullptr, CLEAR_ERR_HIP, std::string("prologue launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

int clear_attn_reserve_prologue(clear_attn_ctx* ctx, int BH)
{
    if (!ctx) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "ctx is NULL");
    if (BH < 1 || BH > 65535) return fail(ctx, CLEAR_ERR_INVALID_ARG, "BH must be in [1, 65535]");
    if (ctx->dtype != CLEAR_BF16) return fail(ctx, CLEAR_ERR_UNSUPPORTED, "the fused prologue is built for bf16 only");
    if (BH <= ctx->kpro_BH) return CLEAR_OK;
    hipError_t e = hipDeviceSynchronize();  // a running forward may still read the old buffer
    if (e == hipSuccess && ctx->d_kpro) e = hipFree(ctx->d_kpro);
    ctx->d_kpro = nullptr;
    ctx->kpro_BH = 0;
    const long long N = (long long)ctx->n_text + (long long)ctx->gridH * ctx->gridW;
    if (e == hipSuccess) e = hipMalloc(&ctx->d_kpro, (size_t)BH * N * ctx->head_dim * 2);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, e == hipErrorOutOfMemory ? CLEAR_ERR_ALLOC : CLEAR_ERR_HIP, std::string("prologue workspace allocation failed: ") + hipGetErrorString(e));
    }
    ctx->kpro_BH = BH;
    return CLEAR_OK;
}

static int forward_prologue_impl(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, const long long* strides, int B,
                                 int H, int n_text, int gridH, int gridW, int head_dim, int r, const float* q_gain, const float* k_gain,
                                 float norm_eps, const float* rope_y, const float* rope_x, float logit_scale, void* stream)
{
    FwdParams p;
    int rc = prepare_forward(ctx, Q, K, V, O, B, H, n_text, gridH, gridW, head_dim, r, nullptr, &p, stream, strides);
    if (rc != CLEAR_OK) return rc;
    if (ctx->dtype != CLEAR_BF16) return fail(ctx, CLEAR_ERR_UNSUPPORTED, "the fused prologue is built for bf16 only");
    rc = check_prologue(ctx, head_dim, q_gain, k_gain, norm_eps, rope_y, rope_x);
    if (rc != CLEAR_OK) return rc;
    if (!(logit_scale > 0.f) || !std::isfinite(logit_scale)) return fail(ctx, CLEAR_ERR_INVALID_ARG, "logit_scale must be positive and finite");
    p.scale_log2e *= logit_scale;
    p.q_gain = q_gain;
    p.rope_y = rope_y;
    p.rope_x = rope_x;
    p.norm_eps = norm_eps;
    if (k_gain || rope_y) {
        // Every key row is staged by up to 36 workgroups, so its prologue runs once, ahead of the attention
        // kernels, into the context's buffer; the query rows are handled as each workgroup loads its own.
        if (B * H > ctx->kpro_BH && stream_is_capturing((hipStream_t)stream))
            return fail(ctx, CLEAR_ERR_INVALID_ARG, "the key buffer of the prologue would have to grow while the stream is being captured: call clear_attn_reserve_prologue beforehand");
        rc = clear_attn_reserve_prologue(ctx, B * H);
        if (rc != CLEAR_OK) return rc;
        const TensorStrides plain = {(long long)H * p.N * head_dim, p.N * head_dim, head_dim};  // the context's buffer
        hipError_t e = launch_qk_prologue(K, p.ks, ctx->d_kpro, plain, B, H, n_text, gridH, gridW, head_dim, k_gain, norm_eps, rope_y, rope_x,
                                          (hipStream_t)stream);
        if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("prologue launch failed: ") + hipGetErrorString(e));
        p.K = ctx->d_kpro;
        p.ks = plain;
    }
    hipError_t e = launch_all(ctx, p, (hipStream_t)stream);
    if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

int clear_attn_forward_prologue(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, int B, int H, int n_text,
                                int gridH, int gridW, int head_dim, int r, const float* q_gain, const float* k_gain, float norm_eps,
                                const float* rope_y, const float* rope_x, float logit_scale, void* stream)
{
    return forward_prologue_impl(ctx, Q, K, V, O, nullptr, B, H, n_text, gridH, gridW, head_dim, r, q_gain, k_gain, norm_eps, rope_y, rope_x,
                                 logit_scale, stream);
}

int clear_attn_forward_prologue_strided(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, const long long* strides,
                                        int B, int H, int n_text, int gridH, int gridW, int head_dim, int r, const float* q_gain,
                                        const float* k_gain, float norm_eps, const float* rope_y, const float* rope_x, float logit_scale,
                                        void* stream)
{
    if (!strides) return fail(ctx, CLEAR_ERR_INVALID_ARG, "strides is NULL");
    return forward_prologue_impl(ctx, Q, K, V, O, strides, B, H, n_text, gridH, gridW, head_dim, r, q_gain, k_gain, norm_eps, rope_y, rope_x,
                                 logit_scale, stream);
}

int clear_attn_reserve_backward(clear_attn_ctx* ctx, int BH)
{
    if (!ctx) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "ctx is NULL");
    if (BH < 1 || BH > 65535) return fail(ctx, CLEAR_ERR_INVALID_ARG, "BH must be in [1, 65535]");
    if (ctx->dtype != CLEAR_BF16) return fail(ctx, CLEAR_ERR_UNSUPPORTED, "the backward pass is built for bf16 only");

    if (BH <= ctx->bwd_BH) return CLEAR_OK;
    if (ctx->d_bwd_delta) (void)hipFree(ctx->d_bwd_delta);
    if (ctx->d_bwd_ws) (void)hipFree(ctx->d_bwd_ws);
    ctx->d_bwd_delta = ctx->d_bwd_ws = nullptr;
    ctx->bwd_BH = 0;
    const long long N = (long long)ctx->n_text + (long long)ctx->gridH * ctx->gridW;
    hipError_t e = hipMalloc((void**)&ctx->d_bwd_delta, (size_t)BH * N * sizeof(float));
    if (e == hipSuccess && ctx->n_text > 0)
        e = hipMalloc((void**)&ctx->d_bwd_ws, (size_t)3 * BH * max_text_splits(N) * ctx->n_text * ctx->head_dim * sizeof(float));
    if (e != hipSuccess) {
        if (ctx->d_bwd_delta) (void)hipFree(ctx->d_bwd_delta);
        ctx->d_bwd_delta = nullptr;
        (void)hipGetLastError();
        return fail(ctx, e == hipErrorOutOfMemory ? CLEAR_ERR_ALLOC : CLEAR_ERR_HIP, std::string("backward workspace allocation failed: ") + hipGetErrorString(e));
    }
    ctx->bwd_BH = BH;
    return CLEAR_OK;
}

static int backward_impl(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* lse,
                         void* dQ, void* dK, void* dV, const long long* strides, int B, int H, int n_text, int gridH, int gridW,
                         int head_dim, int r, void* stream)
{
    if (!ctx) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "ctx is NULL");
    if (!Q || !K || !V || !O || !dO || !lse || !dQ || !dK || !dV) return fail(ctx, CLEAR_ERR_INVALID_ARG, "NULL tensor pointer");
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O | (uintptr_t)dO | (uintptr_t)dQ | (uintptr_t)dK | (uintptr_t)dV) & 15)
        return fail(ctx, CLEAR_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    if ((uintptr_t)lse & 3) return fail(ctx, CLEAR_ERR_INVALID_ARG, "lse must be 4-byte aligned");
    if (B < 1 || H < 1 || (long long)B * H > 65535) return fail(ctx, CLEAR_ERR_INVALID_ARG, "B, H must be >= 1 and B*H <= 65535");
    if (n_text != ctx->n_text || gridH != ctx->gridH || gridW != ctx->gridW || head_dim != ctx->head_dim || r != ctx->r)
        return fail(ctx, CLEAR_ERR_MISMATCH, "shape arguments differ from those given to clear_attn_create");
    if (ctx->dtype != CLEAR_BF16) return fail(ctx, CLEAR_ERR_UNSUPPORTED, "the backward pass is built for bf16 only");

    const long long N = (long long)n_text + (long long)gridH * gridW;
    TensorStrides ts[8];  // Q, K, V, O, dO, dQ, dK, dV
    for (int t = 0; t < 8; ++t) {
        ts[t].sn = strides ? strides[3 * t + 2] : head_dim;
        ts[t].sh = strides ? strides[3 * t + 1] : N * head_dim;
        ts[t].sb = strides ? strides[3 * t] : (long long)H * N * head_dim;
    }
    if (strides) {
        for (int t = 0; t < 8; ++t) {
            const bool output = t >= 5;
            if (ts[t].sn < head_dim || ts[t].sh < 0 || ts[t].sb < 0 || (output && (ts[t].sh <= 0 || (B > 1 && ts[t].sb <= 0))))
                return fail(ctx, CLEAR_ERR_INVALID_ARG, "strides: the token stride must be >= head_dim, the others >= 0 (> 0 for dQ, dK, dV)");
            if ((ts[t].sn | ts[t].sh | ts[t].sb) & 7) return fail(ctx, CLEAR_ERR_INVALID_ARG, "strides must be multiples of 8 elements (16-byte rows)");
        }
        for (int t : {0, 1, 2, 4})  // the tensors staged as column tiles
            if ((N - 1) * ts[t].sn * 2 + 2 * head_dim > 0xffffffffLL)
                return fail(ctx, CLEAR_ERR_UNSUPPORTED, "Q, K, V, dO are addressed with 32-bit byte offsets inside one head: N * token stride * 2 must be < 2^32");
    }
    {
        // outputs must not overlap inputs or each other (compared by the address ranges the tensors span)
        auto span = [&](const TensorStrides& st) { return (size_t)((B - 1) * st.sb + (H - 1) * st.sh + (N - 1) * st.sn + head_dim) * 2; };
        const void* all[8] = {dQ, dK, dV, Q, K, V, O, dO};
        const int idx[8] = {5, 6, 7, 0, 1, 2, 3, 4};
        for (int a = 0; a < 3; ++a)
            for (int b = a + 1; b < 8; ++b) {
                const uintptr_t a0 = (uintptr_t)all[a], b0 = (uintptr_t)all[b];
                if (a0 < b0 + span(ts[idx[b]]) && b0 < a0 + span(ts[idx[a]]))
                    return fail(ctx, CLEAR_ERR_INVALID_ARG, "dQ, dK, dV must not overlap each other or an input");
            }
    }
    const int BH = B * H;
    if (BH > ctx->bwd_BH && stream_is_capturing((hipStream_t)stream))
        return fail(ctx, CLEAR_ERR_INVALID_ARG, "the backward workspace would have to grow while the stream is being captured: call clear_attn_reserve_backward beforehand");
    int rc = clear_attn_reserve_backward(ctx, BH);
    if (rc != CLEAR_OK) return rc;
    const Schedule& s = ctx->t.sched;
    BwdParams p;
    memset(&p, 0, sizeof(p));
    p.Q = Q; p.K = K; p.V = V; p.dO = dO; p.lse = lse; p.delta = ctx->d_bwd_delta;
    p.dQ = dQ; p.dK = dK; p.dV = dV;
    p.qs = ts[0]; p.ks = ts[1]; p.vs = ts[2]; p.os = ts[3]; p.dos = ts[4]; p.dqs = ts[5]; p.dks = ts[6]; p.dvs = ts[7];
    p.B = B; p.H = H; p.n_text = n_text; p.gridH = gridH; p.gridW = gridW; p.r2 = r * r;
    p.N = N;
    p.n_q_tiles = s.n_qty * s.n_qtx;
    p.n_qtx = s.n_qtx;
    p.row_ptr = ctx->t.d_row_ptr; p.col_idx = ctx->t.d_col_idx; p.n_plain = ctx->t.d_n_plain; p.qt_order = ctx->t.d_qt_order; p.mask_tbl = ctx->t.d_mask_tbl;
    p.wave_desc = ctx->t.d_wave_desc;
    p.mask_ry = ctx->t.mask_ry; p.mask_rx = ctx->t.mask_rx;
    p.mask_kind = ctx->mask_kind; p.mask_r = r; p.mask_shift = ctx->mask_shift;
    p.n_classes = 1; p.stride = 1; p.stride_rx = p.stride_ry = 0;
    if (ctx->mask_kind == CLEAR_MASK_STRIDED) {
        p.mask_kind = kMaskFull;  // inside a residue class every pair is admitted
        p.n_classes = r * r; p.stride = r;
        p.stride_rx = ctx->mask_shift % r; p.stride_ry = (ctx->mask_shift / r) % r;
        if ((long long)p.n_q_tiles * B * H * p.n_classes > 0x7fffffffLL) return fail(ctx, CLEAR_ERR_INVALID_ARG, "too many workgroups: B*H*r*r*row tiles must fit in 31 bits");
    }
    p.scale = (float)(1.0 / std::sqrt((double)head_dim));
    p.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)head_dim));
    const bool together = (long long)BH * p.n_classes * p.n_q_tiles <= 64LL * ctx->num_cus;  // one launch for the four kernels, see below
    if (n_text > 0) {
        const int per_block = bf16_text_queries_per_block();
        p.n_tq_tiles = (n_text + per_block - 1) / per_block;
        choose_text_splits(N, BH, p.n_tq_tiles, ctx->num_cus, together, &p.n_splits, &p.split_keys);
        p.ws = ctx->d_bwd_ws;
    }
    auto run = [&](hipStream_t st, int phase) {
        return ctx->head_dim == 128 ? launch_bf16_d128_backward(p, O, ctx->d_bwd_delta, st, phase) : launch_bf16_d64_backward(p, O, ctx->d_bwd_delta, st, phase);
    };
    // After delta, the four kernels (dQ and dK/dV of the image rows and of the text rows) are independent.  Up to 64
    // image workgroups per CU they go out as one launch, longest workgroups first, so that each kind fills the CUs the
    // others leave idle (64 x 64 grid, the paper's training size: 0.59 -> 0.48 ms against one launch after the other,
    // 0.54 with the kinds on two streams as an earlier version ran them; 128 x 128: 2.18 -> 1.89 ms; 256 x 256: 1 %);
    // the largest problems, where it gains nothing, keep one launch per kernel.
    hipError_t e = hipSuccess;
    if (together) {
        e = run((hipStream_t)stream, kBwdPhaseDelta);
        if (e == hipSuccess) e = run((hipStream_t)stream, kBwdPhaseFour);
        if (e == hipSuccess && p.n_text > 0) e = run((hipStream_t)stream, kBwdPhaseReduce);
    } else {
        e = run((hipStream_t)stream, kBwdPhaseAll);
    }
    if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("backward launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

int clear_attn_backward(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                        const float* lse, void* dQ, void* dK, void* dV, int B, int H, int n_text, int gridH, int gridW,
                        int head_dim, int r, void* stream)
{
    return backward_impl(ctx, Q, K, V, O, dO, lse, dQ, dK, dV, nullptr, B, H, n_text, gridH, gridW, head_dim, r, stream);
}

int clear_attn_backward_strided(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                                const float* lse, void* dQ, void* dK, void* dV, const long long* strides, int B, int H, int n_text,
                                int gridH, int gridW, int head_dim, int r, void* stream)
{
    if (!strides) return fail(ctx, CLEAR_ERR_INVALID_ARG, "strides is NULL");
    return backward_impl(ctx, Q, K, V, O, dO, lse, dQ, dK, dV, strides, B, H, n_text, gridH, gridW, head_dim, r, stream);
}

int clear_attn_forward_band(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, int B, int H,
                            int n_text, int gridH, int gridW, int head_dim, int r, int own_y0, int own_y1,
                            int text_keys, float* text_o, float* text_lse, void* stream)
{
    const BandArgs band = {own_y0, own_y1, text_keys != 0, text_o, text_lse};
    FwdParams p;
    int rc = prepare_forward(ctx, Q, K, V, O, B, H, n_text, gridH, gridW, head_dim, r, &band, &p, stream);
    if (rc != CLEAR_OK) return rc;
    hipError_t e = launch_all(ctx, p, (hipStream_t)stream);
    if (e != hipSuccess) return fail(ctx, CLEAR_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

int clear_attn_band_layout(int gridH, int r, int n_bands, int band, int* y0, int* y1, int* halo_top, int* halo_bottom)
{
    if (gridH < 1 || r < 1 || n_bands < 1 || band < 0 || band >= n_bands) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "need gridH, r, n_bands >= 1 and 0 <= band < n_bands");
    if (!y0 || !y1 || !halo_top || !halo_bottom) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "NULL output pointer");
    if (n_bands > gridH) return fail(nullptr, CLEAR_ERR_UNSUPPORTED, "more bands than image rows");
    const int base = gridH / n_bands, extra = gridH % n_bands;  // the first `extra` bands hold one row more
    // a halo of r - 1 rows must come from the adjacent band alone (one exchange with each neighbour)
    if (n_bands > 1 && base < r - 1) return fail(nullptr, CLEAR_ERR_UNSUPPORTED, "bands narrower than the r - 1 halo rows are not supported");
    const int b0 = band * base + std::min(band, extra);
    const int b1 = b0 + base + (band < extra ? 1 : 0);
    *y0 = b0;
    *y1 = b1;
    *halo_top = std::min(r - 1, b0);
    *halo_bottom = std::min(r - 1, gridH - b1);
    return CLEAR_OK;
}

int clear_attn_merge_text(int n_parts, const float* const* text_o, const float* const* text_lse, int B, int H, int n_text,
                          long long N, int head_dim, int mode, void* O, int dtype, void* stream)
{
    if (n_parts < 1 || n_parts > kMaxMergeParts) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "n_parts must be in [1, 64]");
    if (!text_o || !text_lse || !O) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "NULL argument");
    if (B < 1 || H < 1 || n_text < 1 || N < n_text || head_dim < 1 || head_dim > 1024) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "need B, H, n_text >= 1, N >= n_text, 1 <= head_dim <= 1024");
    if (mode != CLEAR_MERGE_EXACT && mode != CLEAR_MERGE_AVERAGE) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "mode must be CLEAR_MERGE_EXACT or CLEAR_MERGE_AVERAGE");
    if (dtype != CLEAR_BF16 && dtype != CLEAR_F32) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "dtype must be CLEAR_BF16 or CLEAR_F32");
    if ((long long)B * H * n_text > 0x7fffffffLL) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "B*H*n_text must fit in 31 bits");
    MergeParts parts;
    parts.n = n_parts;
    for (int i = 0; i < n_parts; ++i) {
        if (!text_o[i] || !text_lse[i]) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "NULL part pointer");
        parts.o[i] = text_o[i];
        parts.lse[i] = text_lse[i];
    }
    hipError_t e = launch_merge_text(parts, B * H, n_text, N, head_dim, mode, O, dtype, (hipStream_t)stream);
    if (e != hipSuccess) return fail(nullptr, CLEAR_ERR_HIP, std::string("merge launch failed: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

void clear_attn_destroy(clear_attn_ctx* ctx)
{
    if (!ctx) return;
    ctx->t.release();
    for (TileTables*& bt : ctx->band_t)
        if (bt) {
            bt->release();
            delete bt;
            bt = nullptr;
        }
    if (ctx->d_ws_o) (void)hipFree(ctx->d_ws_o);
    if (ctx->d_ws_ml) (void)hipFree(ctx->d_ws_ml);
    if (ctx->d_bwd_delta) (void)hipFree(ctx->d_bwd_delta);
    if (ctx->d_bwd_ws) (void)hipFree(ctx->d_bwd_ws);
    if (ctx->d_kpro) (void)hipFree(ctx->d_kpro);
    delete ctx;
}

int clear_attn_schedule_size(const clear_attn_ctx* ctx, int* q_tile_h, int* q_tile_w, int* k_tile_h, int* k_tile_w,
                             int* n_q_tiles, long long* n_pairs)
{
    if (!ctx) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "ctx is NULL");
    const Schedule& s = ctx->t.sched;
    if (q_tile_h) *q_tile_h = s.qth;
    if (q_tile_w) *q_tile_w = s.qtw;
    if (k_tile_h) *k_tile_h = s.kth;
    if (k_tile_w) *k_tile_w = s.ktw;
    if (n_q_tiles) *n_q_tiles = (int)s.row_ptr.size() - 1;
    if (n_pairs) *n_pairs = (long long)s.col_idx.size();
    return CLEAR_OK;
}

int clear_attn_schedule_copy(const clear_attn_ctx* ctx, int* row_ptr, int* col_idx, unsigned char* flags)
{
    if (!ctx) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "ctx is NULL");
    const Schedule& s = ctx->t.sched;
    if (row_ptr) memcpy(row_ptr, s.row_ptr.data(), s.row_ptr.size() * sizeof(int));
    if (col_idx) memcpy(col_idx, s.col_idx.data(), s.col_idx.size() * sizeof(int));
    if (flags) memcpy(flags, s.flags.data(), s.flags.size());
    return CLEAR_OK;
}

int clear_attn_executed_pairs(const clear_attn_ctx* ctx, unsigned long long* pairs_per_head)
{
    if (!ctx || !pairs_per_head) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "NULL argument");
    if (ctx->mask_kind == CLEAR_MASK_STRIDED)
        *pairs_per_head = executed_pairs_bf16_strided(ctx->t.sched, ctx->n_text, ctx->gridH, ctx->gridW, ctx->r, ctx->mask_shift);
    else
        *pairs_per_head = (ctx->dtype == CLEAR_BF16) ? executed_pairs_bf16(ctx->t.sched, ctx->n_text, 0) : executed_pairs_f32(ctx->t.sched, ctx->n_text);
    return CLEAR_OK;
}

int clear_attn_measure_mfma_peak(double seconds, double* tflops, double* shader_mhz)
{
    if (!tflops || !shader_mhz) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "NULL argument");
    if (!(seconds > 0.0) || seconds > 5.0) return fail(nullptr, CLEAR_ERR_INVALID_ARG, "seconds must be in (0, 5]");
    int dev = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess) e = measure_mfma_peak(prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256, seconds, tflops, shader_mhz);
    if (e != hipSuccess) return fail(nullptr, CLEAR_ERR_HIP, std::string("HIP error in measure_mfma_peak: ") + hipGetErrorString(e));
    return CLEAR_OK;
}

const char* clear_attn_last_error(const clear_attn_ctx* ctx)
{
    return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

}  // extern "C"
