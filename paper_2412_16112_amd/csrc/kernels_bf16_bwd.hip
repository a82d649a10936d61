// Backward pass of the CLEAR local attention for gfx950 (bf16, head_dim 128; kernels_bf16_bwd_d64.hip compiles
// this file a second time for head_dim 64): dQ, dK, dV of Eq. 1 under the
// mask of Eq. 3, given dO and the per-row log-sum-exp the forward pass can return.  With
//   s_ij = q_i.k_j / sqrt(d),  p_ij = exp(s_ij - lse_i) for M_ij = 1 (else 0),  delta_i = dO_i . O_i,
//   dp_ij = dO_i . v_j,        ds_ij = p_ij (dp_ij - delta_i):
//   dQ_i = sum_j ds_ij k_j / sqrt(d),   dK_j = sum_i ds_ij q_i / sqrt(d),   dV_j = sum_i p_ij dO_i.
//
// One kernel template computes any of the three.  Its "rows" are the tokens whose gradient a workgroup
// produces (queries for dQ, keys for dK and dV), held one per lane as MFMA B operands like Q in the forward
// kernel; its "columns" are the tokens summed over, staged in LDS tiles exactly like K and V in the forward
// kernel, taken from the same tile schedule (the mask is symmetric, so the key tiles a query tile reaches
// are also the query tiles that reach a key tile at its place):
//   mode  rows      column tiles (C1 | C2)   S = C1 r1^T   dP = C2 r2^T   X    accumulator += T^T X
//   dQ    queries   K | V                    K q^T         V dO^T         dS   K^T dS
//   dK    keys      Q | dO                   Q k^T         dO v^T         dS   Q^T dS
//   dV    keys      Q | dO                   Q k^T         -              P    dO^T P
//   dK+dV keys      Q | dO                   Q k^T         dO v^T         both of the above from one S (image rows)
// lse and delta belong to the query: a per-lane scalar for dQ, a per-column vector (staged next to the tile)
// for dK and dV.  Text rows sum over every token: they are split along the columns into partial sums that a
// small kernel adds up, like the text-query rows of the forward pass.  dK and dV of a key tile are produced
// by one pass from one S and one dP (the separate modes remain for reference).  The blocks are hand-ordered
// pipelines like the forward kernel's tiles: do_block_q for dQ, do_block_kv for dK + dV at head_dim 64 and
// do_block_kv_early at head_dim 128 (do_block, the compiler's order, serves the separate dK and dV modes).
// delta is formed by the dQ kernels on their way when they run before the dK / dV kernels (BwdParams::delta_out),
// otherwise by clear_bwd_delta_kernel.
#include <hip/hip_runtime.h>

#include "bf16_common.h"
#include "block_class.h"
#include "clear_internal.h"

#ifndef CLEAR_BWD_FUSED_KV
#define CLEAR_BWD_FUSED_KV 1
#endif
#ifndef CLEAR_BWD_PIPELINED_KV
#define CLEAR_BWD_PIPELINED_KV (CLEAR_HEAD_DIM == 64 ? 1 : 2)  // dK + dV blocks: 1 = do_block_kv, 2 = do_block_kv_early, 0 = do_block (the compiler's order)
#endif
#ifndef CLEAR_BWD_ISSUE_SHARE
#define CLEAR_BWD_ISSUE_SHARE 2  // 2: the waves stage whole stages in turns, half of them each time; 1: every wave its share of every stage
#endif
#ifndef CLEAR_BWD_KV_FRESH_ADDR
#define CLEAR_BWD_KV_FRESH_ADDR 1  // do_block_kv_early: operand addresses formed at every read (0: sixteen registers hold them; spills)
#endif
#ifndef CLEAR_BWD_KV_RING_SLACK
#define CLEAR_BWD_KV_RING_SLACK 1  // do_block_kv_early: entries of the operand ring beyond the prefetch distance
#endif
#ifndef CLEAR_BWD_KV_OPERAND_PREFETCH
#define CLEAR_BWD_KV_OPERAND_PREFETCH 2  // slots between an LDS operand read and the matrix instruction that takes it (3, 4: spills, slower)
#endif
// do_block at 128 channels (only reached with CLEAR_BWD_PIPELINED_KV = 0): form the probabilities and round them to
// bf16 before the dP products, and take dS from those rounded values, which then carries the rounding of P that dV's
// operand has anyway.  do_block_kv_early does the same: with the fp32 scores dead that early the block fits the 256
// registers of two waves per SIMD.
#ifndef CLEAR_BWD_KV_EARLY_P
#define CLEAR_BWD_KV_EARLY_P (CLEAR_HEAD_DIM == 128)
#endif
#ifndef CLEAR_BWD_PIPELINED_Q
#define CLEAR_BWD_PIPELINED_Q 1  // dQ blocks as a hand-ordered pipeline (0: the compiler's order, as for dK and dV)
#endif

#if CLEAR_HEAD_DIM == 64
// second compilation of this file: its own kernel and launcher names
#define clear_bwd_bf16_kernel clear_bwd_bf16_d64_kernel
#define clear_bwd_delta_kernel clear_bwd_delta_d64_kernel
#define clear_bwd_reduce_kernel clear_bwd_reduce_d64_kernel
#define clear_bwd_bf16_all_kernel clear_bwd_bf16_d64_all_kernel
#define launch_bf16_backward launch_bf16_d64_backward
#else
#define launch_bf16_backward launch_bf16_d128_backward
#endif

namespace clear {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

enum BwdMode : int { kBwdQ = 0, kBwdK = 1, kBwdV = 2, kBwdKV = 3 };

constexpr int STATS_BYTES = TILE_KEYS * 2 * 4;                           // per staged tile: lse2 and delta of its 64 columns
constexpr int BWD_LDS_BYTES = NBUF * STAGE_BYTES + NBUF * TPS * STATS_BYTES;

// One workgroup of a backward launch: workgroup `bid` of `nblk`.
template <int MODE, bool LINROWS, int CODE>
__device__ __forceinline__ void clear_bwd_bf16_workgroup(const BwdParams& p, const int bid, const int nblk)
{
    constexpr int NWY = kBf16NWY, NWX = kBf16NWX, NW = NWY * NWX;
    constexpr int NI = TILE_KEYS / ROWS_PER_LOAD / NW;  // 1 KB load instructions per wave per tile, for each of the two tiles
    constexpr int ISSUE_SHARE = CLEAR_BWD_ISSUE_SHARE;  // 2: the waves take turns, half of them staging a whole stage
    constexpr bool COLSTAT = MODE != kBwdQ;  // lse / delta indexed by column
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];  // [NBUF][TPS][C1 tile | C2 tile], then the column statistics
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    float* const stats = (float*)(smem + NBUF * STAGE_BYTES);  // [NBUF][TPS][2][64]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qi = lane & 31;
    const int hh = lane >> 5;

    // ---- workgroup -> (batch*head, row tile[, column split]); XCD-aware like the forward kernel
    int vid;
    {
        const int xcd = bid & 7, idx = bid >> 3;
        const int q = nblk >> 3, rem = nblk & 7;
        vid = xcd * q + imin(xcd, rem) + idx;
    }
    int bh, rt, split = 0;
    if (LINROWS) {
        split = vid % p.n_splits;
        const int t = vid / p.n_splits;
        rt = t % p.n_tq_tiles;
        bh = t / p.n_tq_tiles;
    } else {
        rt = vid % p.n_q_tiles;
        if (p.qt_order) rt = ((const_int_ptr)p.qt_order)[rt];  // the order in which a head's row tiles are dealt out
        bh = vid / p.n_q_tiles;
    }
    // Image rows live on an rH x rW grid and image columns on a cH x cW grid; grid point (y, x) is image token
    // (y * stride + oy, x * stride + ox) of the raster.  Plain masks: both are the raster.  Strided mask: the
    // workgroup belongs to one residue class of its rows; queries of class c meet the keys of class c + (ry, rx),
    // so the columns of a key class are the queries of class c - (ry, rx).
    int stride = 1, r_oy = 0, r_ox = 0, c_oy = 0, c_ox = 0;
    int rH = p.gridH, rW = p.gridW, cH = p.gridH, cW = p.gridW;
    if (!LINROWS && CODE == kCodeFull) {
        const int cls = bh % p.n_classes;
        bh /= p.n_classes;
        stride = p.stride;
        r_oy = cls / stride;
        r_ox = cls % stride;
        const int dy = MODE == kBwdQ ? p.stride_ry : stride - p.stride_ry, dx = MODE == kBwdQ ? p.stride_rx : stride - p.stride_rx;
        c_oy = (r_oy + dy) % stride;
        c_ox = (r_ox + dx) % stride;
        rH = (p.gridH - r_oy + stride - 1) / stride;  // >= 1: the host requires gridH, gridW >= stride
        rW = (p.gridW - r_ox + stride - 1) / stride;
        cH = (p.gridH - c_oy + stride - 1) / stride;
        cW = (p.gridW - c_ox + stride - 1) / stride;
    }
    const int batch = bh / p.H, head = bh % p.H;
    auto head_of = [&](const void* ptr, const TensorStrides& st) { return (const __bf16*)ptr + batch * st.sb + head * st.sh; };
    const TensorStrides& r1s = MODE == kBwdQ ? p.qs : p.ks;
    const TensorStrides& r2s = MODE == kBwdQ ? p.dos : p.vs;
    const TensorStrides& c1s = MODE == kBwdQ ? p.ks : p.qs;
    const TensorStrides& c2s = MODE == kBwdQ ? p.vs : p.dos;
    const __bf16* const R1 = head_of(MODE == kBwdQ ? p.Q : p.K, r1s);
    const __bf16* const R2 = head_of(MODE == kBwdQ ? p.dO : p.V, r2s);
    const unsigned char* const C1 = (const unsigned char*)head_of(MODE == kBwdQ ? p.K : p.Q, c1s);
    const unsigned char* const C2 = (const unsigned char*)head_of(MODE == kBwdQ ? p.V : p.dO, c2s);
    const unsigned c1_pitch = (unsigned)c1s.sn * 2, c2_pitch = (unsigned)c2s.sn * 2;  // bytes from one token row to the next
    const float* const lse = p.lse + (long long)bh * p.N;
    const float* const delta = p.delta + (long long)bh * p.N;

    // ---- this wave's rows, and this lane's one among them.  What depends on the lane (row coordinates, token, validity,
    // the half of the wave) is worked out again from the hardware's lane count wherever it is needed (here, per masked
    // tile, in the epilogue) instead of being carried through the tile loop: the fused dK / dV kernel has no register
    // to spare there, and a value spilled to scratch memory costs, on its way back, a wait for every load in flight.
    int wy0 = 0, wx0 = 0, r0 = 0;
    bool wave_has_rows;
    if (LINROWS) {
        r0 = rt * (NW * 32) + wave * 32;
        wave_has_rows = r0 < p.n_text;
    } else {
        wy0 = (rt / p.n_qtx) * (NWY * kWaveQH) + (wave / NWX) * kWaveQH;
        wx0 = (rt % p.n_qtx) * (NWX * kWaveQW) + (wave % NWX) * kWaveQW;
        wave_has_rows = wy0 < rH && wx0 < rW;
    }
    struct LaneRow {
        int hh, ry, rx, token;
        bool valid;
    };
    auto lane_row = [&]() {
        LaneRow L;
        const int ln = fresh_lane_id();
        const int q = ln & 31;
        L.hh = ln >> 5;
        L.ry = L.rx = 0;
        if (LINROWS) {
            L.token = r0 + q;
            L.valid = L.token < p.n_text;
            if (!L.valid) L.token = p.n_text - 1;
        } else {
            L.ry = wy0 + (q >> 3);
            L.rx = wx0 + (q & 7);
            L.valid = L.ry < rH && L.rx < rW;
            L.token = p.n_text + (imin(L.ry, rH - 1) * stride + r_oy) * p.gridW + imin(L.rx, rW - 1) * stride + r_ox;
        }
        return L;
    };
    const int r_token = lane_row().token;
    // B operands: KS contraction steps of 16 channels, this lane supplying channels 16 s + 8 hh .. + 7
    bf16x8 r1f[KS], r2f[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        r1f[s] = *(const bf16x8*)(R1 + (long long)r_token * r1s.sn + 8 * hh + 16 * s);
        if (MODE != kBwdV) r2f[s] = *(const bf16x8*)(R2 + (long long)r_token * r2s.sn + 8 * hh + 16 * s);
    }
    // lse in units of log2 (the exponentials are 2^x); dQ: this lane's query
    constexpr float LOG2E = 1.4426950408889634f;
    float lse2_row = 0.f, delta_row = 0.f;
    if (!COLSTAT) {
        lse2_row = lse[r_token] * LOG2E;
        if (p.delta_out) {
            // delta of this lane's row from the dO fragments it holds and the matching pieces of its O row; the other half
            // of the row's channels sits 32 lanes away
            const __bf16* orow = head_of(p.O, p.os) + (long long)r_token * p.os.sn + 8 * (fresh_lane_id() >> 5);
            float part = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const bf16x8 o = *(const bf16x8*)(orow + 16 * s);
#pragma unroll
                for (int j = 0; j < 8; ++j) part += (float)o[j] * (float)r2f[s][j];
            }
            delta_row = part + __shfl_xor(part, 32, 64);
            const LaneRow own = lane_row();
            if (own.valid && own.hh == 0 && split == 0) p.delta_out[(long long)bh * p.N + own.token] = delta_row;
        } else {
            delta_row = delta[r_token];
        }
    }
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        asm volatile("" : "+v"(r1f[s]));
        if (MODE != kBwdV) asm volatile("" : "+v"(r2f[s]));
    }
    asm volatile("" : "+v"(lse2_row), "+v"(delta_row));

    const const_int_ptr row_ptr = (const_int_ptr)p.row_ptr, col_idx = (const_int_ptr)p.col_idx, n_plain = (const_int_ptr)p.n_plain;
    const const_u64_ptr mask_tbl = (const_u64_ptr)p.mask_tbl;

    // ---- column tile list: tokens [lin_begin, lin_limit) in 64-token tiles, then (image rows) the CSR row:
    //   [0, cb1) whole linear tiles   [cb1, cb2) the ragged linear tile   [cb2, cb3) image tiles inside the grid
    //   [cb3, cb4) image tiles cut by the border
    int n_tiles, n_lin_tiles, csr_begin = 0;
    int lin_begin = 0, lin_limit = 0;
    if (LINROWS) {
        lin_begin = split * p.split_keys;
        lin_limit = (long long)lin_begin + p.split_keys < p.N ? lin_begin + p.split_keys : (int)p.N;
        n_lin_tiles = (lin_limit - lin_begin + TILE_KEYS - 1) / TILE_KEYS;
        n_tiles = n_lin_tiles;
    } else {
        lin_limit = p.n_text;
        n_lin_tiles = (p.n_text + TILE_KEYS - 1) / TILE_KEYS;
        csr_begin = row_ptr[rt];
        n_tiles = n_lin_tiles + (row_ptr[rt + 1] - csr_begin);
    }
    const int cb1 = (lin_limit - lin_begin) / TILE_KEYS, cb2 = n_lin_tiles;
    constexpr bool dense_image = !LINROWS && CODE == kCodeFull;  // strided: tiles inside the class grid need no mask
    const int cb3 = LINROWS ? n_lin_tiles : ((p.mask_tbl || dense_image) ? n_lin_tiles + n_plain[rt] : n_lin_tiles);
    const int cb4 = n_tiles;
    auto stage_len = [&](int t) {
        const int e = t < cb1 ? cb1 : (t < cb2 ? cb2 : (t < cb3 ? cb3 : cb4));
        return imin(TPS, e - t);
    };
    auto tile_origin = [&](int i, int& a, int& b) {  // linear -> (first token, -1); image -> (row, col) of the 8 x 8 tile
        if (i < n_lin_tiles) {
            a = lin_begin + i * TILE_KEYS;
            b = -1;
        } else {
            const int packed = col_idx[csr_begin + i - n_lin_tiles];
            a = packed >> 16;
            b = packed & 0xffff;
        }
    };
    auto slot_token = [&](int a, int b, int slot) {  // token staged in slot `slot` (0..63) of the tile with origin (a, b)
        if (b < 0) return imin(a + slot, lin_limit - 1);
        const int ky = imin(a + (slot >> 3), cH - 1);
        const int kx = imin(b + (slot & 7), cW - 1);
        return p.n_text + (ky * stride + c_oy) * p.gridW + kx * stride + c_ox;
    };

    // ---- staging: LDS-direct loads of the two column tiles (same layout and swizzle as K and V in the
    // forward kernel), and for dK / dV the statistics of the tile's 64 queries (wave j of the first TPS waves
    // fetches them for tile j of the stage and writes them to LDS before the next barrier)
    auto issue_tile = [&](int i, unsigned lds_tile) {
        int a, b;
        tile_origin(i, a, b);
        // The lane's place in the tile is worked out again from the hardware's lane count: values kept in registers
        // since the kernel's start get spilled in the fused dK / dV kernel, and their reload from scratch memory would
        // wait for every load issued before it, the staged tile in front included.
        const int ln = fresh_lane_id();
#pragma unroll
        for (int n = 0; n < NI * ISSUE_SHARE; ++n) {
            const int ii = (wave % (NW / ISSUE_SHARE)) * (NI * ISSUE_SHARE) + n;
            const int row = ROWS_PER_LOAD * ii + ln / CHUNKS;
            const int token = slot_token(a, b, row);
            const unsigned chunk_off = (unsigned)(((ln % CHUNKS) ^ swz(row)) << 4);
            load_to_lds_16B(C1, (unsigned)token * c1_pitch + chunk_off, lds_tile + ii * 1024);
            load_to_lds_16B(C2, (unsigned)token * c2_pitch + chunk_off, lds_tile + TILE_BYTES + ii * 1024);
        }
    };
    float st_lse = 0.f, st_delta = 0.f;  // in flight: statistics of slot `lane` of tile `wave` of the next stage
    // Half of the waves stage a whole stage, the other half the next one (each SIMD holds one wave of either half): while
    // one wave of a SIMD stands at its load instructions the other one is already at its matrix products.
    int issue_turn = 0;
    auto issue_stage = [&](int t, int buf) {
        const int len = stage_len(t);
        const bool mine = ISSUE_SHARE == 1 || (wave / (NW / ISSUE_SHARE)) == (issue_turn & (ISSUE_SHARE - 1));
        ++issue_turn;
#pragma unroll
        for (int j = 0; j < TPS; ++j)
            if (j < len && mine) issue_tile(t + j, lds_base + (unsigned)buf * STAGE_BYTES + (unsigned)j * (2 * TILE_BYTES));
        if (COLSTAT && wave < len) {
            int a, b;
            tile_origin(t + wave, a, b);
            const int token = slot_token(a, b, fresh_lane_id());
            st_lse = lse[token];  // (scaled when it is published: no wait for it here)
            st_delta = delta[token];
        }
    };
    auto publish_stats = [&](int buf, int len) {  // called before the barrier that opens stage buffer buf
        if (COLSTAT && wave < len) {
            float* dst = stats + ((buf * TPS + wave) * 2) * TILE_KEYS;
            const int ln = fresh_lane_id();
            dst[ln] = st_lse * LOG2E;
            dst[TILE_KEYS + ln] = st_delta;
        }
    };

    LaneOffsets lo;
    lo.k0 = (unsigned)(qi * ROW_BYTES + ((hh ^ swz(qi)) << 4));
    {
        const int j = lane & 15, g2 = (lane >> 4) & 1;
        const int row = 4 * hh + (j >> 2);
        const int chunk = 2 * g2 + ((j & 3) >> 1);
        lo.v0 = (unsigned)(row * ROW_BYTES + ((chunk ^ swz(row)) << 4) + 8 * (j & 1));
    }

    f32x16 acc[NDB];  // gradient^T tiles: channel 32 db + 8 (reg / 4) + 4 hh + reg % 4 of this lane's row
    f32x16 acc_v[MODE == kBwdKV ? NDB : 1];  // fused mode: acc holds dK, acc_v holds dV
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc[db][r] = 0.f;
            if constexpr (MODE == kBwdKV) acc_v[db][r] = 0.f;
        }
    const float c = p.scale_log2e;

    // One 32-column block of a staged tile.
    auto do_block = [&](auto mask_tag, unsigned tile_lds, int blk, const MaskArgs& ma, const float* tile_stats) __attribute__((always_inline)) {
        constexpr int MASK = decltype(mask_tag)::value;
        // C1 is read row-wise for the scores and (dQ, dK) transposed for the accumulation; C2, TILE_BYTES further on
        // in the staged tile, through the same lane addresses and an immediate offset
        const TileAddr ta = tile_addr(tile_lds, lo, 0);
        constexpr unsigned kTransposedHalf = MODE == kBwdV ? TILE_BYTES : 0;  // the tile read transposed for the accumulation
        f32x16 s = qk_block(ta, blk, r1f);
        apply_mask<MASK, CODE>(s, blk, ma);
        bf16x8 xf[2];
        if (MODE == kBwdV) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float l2 = COLSTAT ? tile_stats[32 * blk + 8 * (r >> 2) + 4 * hh + (r & 3)] : lse2_row;
                xf[r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -l2));
            }
        } else if constexpr (MODE == kBwdKV && CLEAR_BWD_KV_EARLY_P) {
            // The probabilities first, rounded to bf16 (they are the operand of the dV product anyway), so that the
            // fp32 scores are dead before dP is formed: eight registers less at the block's peak.
            bf16x8 pf[2];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float l2 = COLSTAT ? tile_stats[32 * blk + 8 * (r >> 2) + 4 * hh + (r & 3)] : lse2_row;
                pf[r >> 3][r & 7] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -l2));
            }
            asm volatile("" : "+v"(pf[0]), "+v"(pf[1]));  // (keeps the conversion in front of the dP products)
            const f32x16 dp = qk_block(ta, blk, r2f, TILE_BYTES);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float dl = COLSTAT ? tile_stats[TILE_KEYS + 32 * blk + 8 * (r >> 2) + 4 * hh + (r & 3)] : delta_row;
                xf[r >> 3][r & 7] = (__bf16)((float)pf[r >> 3][r & 7] * (dp[r] - dl));
            }
            pv_block(acc_v, ta, blk, pf, TILE_BYTES);
        } else {
            const f32x16 dp = qk_block(ta, blk, r2f, TILE_BYTES);
            bf16x8 pf[2];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int slot = 32 * blk + 8 * (r >> 2) + 4 * hh + (r & 3);
                const float l2 = COLSTAT ? tile_stats[slot] : lse2_row;
                const float dl = COLSTAT ? tile_stats[TILE_KEYS + slot] : delta_row;
                const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -l2));
                if constexpr (MODE == kBwdKV) pf[r >> 3][r & 7] = (__bf16)pr;
                xf[r >> 3][r & 7] = (__bf16)(pr * (dp[r] - dl));
            }
            if constexpr (MODE == kBwdKV) {
                // dV += dO^T P from the same probabilities (the dO tile read transposed)
                pv_block(acc_v, ta, blk, pf, TILE_BYTES);
            }
        }
        pv_block(acc, ta, blk, xf, kTransposedHalf);
    };

    // The same block for dQ (lse and delta are the lane's own scalars, 64 accumulator registers: there is room)
    // as a hand-ordered pipeline in the manner of the forward kernel: 2 KS + 2 NDB matrix instructions in
    // program order, each LDS operand read two slots ahead of the instruction that consumes it,
    //   slots [0, KS)        S = K q^T
    //   slots [KS, 2 KS)     dP = V dO^T            | mask, P = 2^(S c - lse) of the finished S
    //   slots [2 KS, end)    dQ^T += K^T dS^T       | dS = P (dP - delta) first, in slot 2 KS
    auto do_block_q = [&](auto mask_tag, unsigned tile_lds, int blk, const MaskArgs& ma) __attribute__((always_inline)) {
        constexpr int MASK = decltype(mask_tag)::value;
        const TileAddr ta = tile_addr(tile_lds, lo, 0);
        constexpr int S_END = KS, DP_END = 2 * KS, NSLOT = 2 * KS + 2 * NDB;
        auto operand = [&](int slot) {
            if (slot < S_END) return read_k_operand(ta, blk, slot);
            if (slot < DP_END) return read_k_operand(ta, blk, slot - S_END, TILE_BYTES);
            const int i = slot - DP_END;  // s2-major, so that consecutive instructions write different accumulators
            return read_v_operand(ta, blk, i / NDB, i % NDB);
        };
        constexpr int PD = 2, RING = PD + 2;
        bf16x8 op[RING];
#pragma unroll
        for (int i = 0; i < PD; ++i) op[i] = operand(i);
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 sc = zero, dp = zero;
        bf16x8 xf[2];
        auto run_slot = [&](auto slot_tag) __attribute__((always_inline)) {
            constexpr int slot = decltype(slot_tag)::value;
            if (slot + PD < NSLOT) op[(slot + PD) % RING] = operand(slot + PD);
            if (slot == DP_END) {
#pragma unroll
                for (int r = 0; r < 16; ++r) xf[r >> 3][r & 7] = (__bf16)(sc[r] * (dp[r] - delta_row));
            }
            if (slot < S_END)
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], r1f[slot], sc, 0, 0, 0);
            else if (slot < DP_END)
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], r2f[slot - S_END], dp, 0, 0, 0);
            else {
                constexpr int i = slot >= DP_END ? slot - DP_END : 0;
                acc[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], xf[i / NDB], acc[i % NDB], 0, 0, 0);
            }
            if (slot == S_END) apply_mask<MASK, CODE>(sc, blk, ma);
            // the exponentials of the finished scores, 16 / KS per slot under the dP products
            constexpr int EPS = 16 / KS;
            if (slot >= S_END && slot < DP_END) {
#pragma unroll
                for (int e = 0; e < EPS; ++e) {
                    const int r = (slot - S_END) * EPS + e;
                    sc[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], c, -lse2_row));
                }
            }
            SCHED_FENCE();
        };
        static_for<NSLOT>(run_slot);
    };

    // The fused dK + dV block in the same manner, 2 KS + 4 NDB matrix instructions.  Used at head_dim 64; at 128
    // channels fp32 scores, dP and an operand ring do not fit the registers together (see do_block_kv_early).
    //   slots [0, KS)            S = Q k^T
    //   slots [KS, 2 KS)         dP = dO v^T          | mask, P = 2^(S c - lse) of the finished S
    //   next 2 NDB slots         dV^T += dO^T P^T     | dS = P (dP - delta)
    //   last 2 NDB slots         dK^T += Q^T dS^T
    auto do_block_kv = [&](auto mask_tag, unsigned tile_lds, int blk, const MaskArgs& ma, const float* tile_stats) __attribute__((always_inline)) {
        constexpr int MASK = decltype(mask_tag)::value;
        const TileAddr ta = tile_addr(tile_lds, lo, 0);
        constexpr int S_END = KS, DP_END = 2 * KS, DV_END = DP_END + 2 * NDB, NSLOT = DV_END + 2 * NDB;
        auto operand = [&](int slot) {
            if (slot < S_END) return read_k_operand(ta, blk, slot);
            if (slot < DP_END) return read_k_operand(ta, blk, slot - S_END, TILE_BYTES);
            if (slot < DV_END) return read_v_operand(ta, blk, (slot - DP_END) / NDB, (slot - DP_END) % NDB, TILE_BYTES);
            return read_v_operand(ta, blk, (slot - DV_END) / NDB, (slot - DV_END) % NDB);
        };
        constexpr int PD = CLEAR_BWD_KV_OPERAND_PREFETCH, RING = PD + 2;
        bf16x8 op[RING];
#pragma unroll
        for (int i = 0; i < PD; ++i) op[i] = operand(i);
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 sc = zero, dp = zero;
        bf16x8 pf[2], xf[2];
        const float* const st = tile_stats + 32 * blk + 4 * hh;  // statistics of this lane's 16 columns: 4 groups of 4
        constexpr int GS = KS / 4;  // slots per group of four columns under the dP products
        static_assert(KS % 4 == 0 && 2 * NDB >= 4, "four column groups are spread over the dP slots and the first dV slots");
        auto run_slot = [&](auto slot_tag) __attribute__((always_inline)) {
            constexpr int slot = decltype(slot_tag)::value;
            if (slot + PD < NSLOT) op[(slot + PD) % RING] = operand(slot + PD);
            if (slot < S_END)
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], r1f[slot], sc, 0, 0, 0);
            else if (slot < DP_END)
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], r2f[slot - S_END], dp, 0, 0, 0);
            else if (slot < DV_END) {
                constexpr int i = slot >= DP_END && slot < DV_END ? slot - DP_END : 0;
                acc_v[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], pf[i / NDB], acc_v[i % NDB], 0, 0, 0);
            } else {
                constexpr int i = slot >= DV_END ? slot - DV_END : 0;
                acc[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], xf[i / NDB], acc[i % NDB], 0, 0, 0);
            }
            if (slot == S_END) apply_mask<MASK, CODE>(sc, blk, ma);
            // P under the dP products: one group of four columns (one 16-byte read of their lse) every GS slots
            if (slot >= S_END && slot < DP_END && (slot - S_END) % GS == 0) {
                constexpr int g = slot >= S_END ? (slot - S_END) / GS : 0;
                const f32x4 l2 = *(const f32x4*)(st + 8 * g);
#pragma unroll
                for (int u = 0; u < 4; ++u) sc[4 * g + u] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[4 * g + u], c, -l2[u]));
                if (g == 1 || g == 3) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) pf[g >> 1][u] = (__bf16)sc[8 * (g >> 1) + u];
                }
            }
            // dS under the dV products, a group of four columns per slot from the second one on
            if (slot > DP_END && slot <= DP_END + 4) {
                constexpr int g = slot > DP_END ? slot - DP_END - 1 : 0;
                const f32x4 dl = *(const f32x4*)(st + TILE_KEYS + 8 * g);
#pragma unroll
                for (int u = 0; u < 4; ++u) xf[g >> 1][4 * (g & 1) + u] = (__bf16)(sc[4 * g + u] * (dp[4 * g + u] - dl[u]));
            }
            SCHED_FENCE();
        };
        static_for<NSLOT>(run_slot);
    };

    // The same products for 128 channels, where the registers do not hold fp32 scores and dP together with the
    // operand ring: the probabilities are rounded to bf16 as soon as the scores are complete (see
    // CLEAR_BWD_KV_EARLY_P), dV follows at once, and dS then takes the place of P in the same registers,
    //   slots [0, KS)            S = Q k^T
    //   next 2 NDB slots         dV^T += dO^T P^T     | first half of P before them, second half under the first NDB
    //   next KS slots            dP = dO v^T
    //   last 2 NDB slots         dK^T += Q^T dS^T     | dS = P (dP - delta) likewise, over P
    auto do_block_kv_early = [&](auto mask_tag, unsigned tile_lds, int blk, const MaskArgs& ma, const float* tile_stats) __attribute__((always_inline)) {
        constexpr int MASK = decltype(mask_tag)::value;
        TileAddr ta = tile_addr(tile_lds, lo, 0);
        constexpr int S_END = KS, DV_END = S_END + 2 * NDB, DP_END = DV_END + KS, NSLOT = DP_END + 2 * NDB;
        auto operand = [&](int slot) {
            // the lane addresses of the 8 + 8 operand positions are formed again at every read (one XOR each) instead
            // of living in sixteen registers through the loop
            if (CLEAR_BWD_KV_FRESH_ADDR) asm volatile("" : "+v"(ta.kb), "+v"(ta.vb0), "+v"(ta.vb1));
            if (slot < S_END) return read_k_operand(ta, blk, slot);
            if (slot < DV_END) return read_v_operand(ta, blk, (slot - S_END) / NDB, (slot - S_END) % NDB, TILE_BYTES);
            if (slot < DP_END) return read_k_operand(ta, blk, slot - DV_END, TILE_BYTES);
            return read_v_operand(ta, blk, (slot - DP_END) / NDB, (slot - DP_END) % NDB);
        };
        constexpr int PD = CLEAR_BWD_KV_OPERAND_PREFETCH, RING = PD + CLEAR_BWD_KV_RING_SLACK;
        bf16x8 op[RING];
#pragma unroll
        for (int i = 0; i < PD; ++i) op[i] = operand(i);
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 sc = zero, dp = zero;
        bf16x8 pf[2];  // P, then dS
        const float* const st = tile_stats + 32 * blk + 4 * (fresh_lane_id() >> 5);  // statistics of this lane's 16 columns: 4 groups of 4
        auto p_group = [&](int g) __attribute__((always_inline)) {
            const f32x4 l2 = *(const f32x4*)(st + 8 * g);
#pragma unroll
            for (int u = 0; u < 4; ++u) pf[g >> 1][4 * (g & 1) + u] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(sc[4 * g + u], c, -l2[u]));
        };
        auto ds_group = [&](int g) __attribute__((always_inline)) {
            const f32x4 dl = *(const f32x4*)(st + TILE_KEYS + 8 * g);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                // P back from the packed operand registers: an even element is the low half of its word
                const unsigned w = __builtin_bit_cast(u32x4, pf[g >> 1])[2 * (g & 1) + (u >> 1)];
                const float pr = __builtin_bit_cast(float, (u & 1) ? (w & 0xffff0000u) : (w << 16));
                pf[g >> 1][4 * (g & 1) + u] = (__bf16)(pr * (dp[4 * g + u] - dl[u]));
            }
        };
        auto run_slot = [&](auto slot_tag) __attribute__((always_inline)) {
            constexpr int slot = decltype(slot_tag)::value;
            if (slot + PD < NSLOT) op[(slot + PD) % RING] = operand(slot + PD);
            if (slot == S_END) {
                apply_mask<MASK, CODE>(sc, blk, ma);
                p_group(0);
                p_group(1);
            }
            constexpr int LATE = NDB > 2 ? 2 : 1;  // the second half is due at slot NDB of its product
            if (slot == S_END + 1) p_group(2);
            if (slot == S_END + LATE) p_group(3);
            if (slot == DP_END) {
                ds_group(0);
                ds_group(1);
            }
            if (slot == DP_END + 1) ds_group(2);
            if (slot == DP_END + LATE) ds_group(3);
            if (slot < S_END)
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], r1f[slot], sc, 0, 0, 0);
            else if (slot < DV_END) {
                constexpr int i = slot >= S_END && slot < DV_END ? slot - S_END : 0;
                acc_v[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], pf[i / NDB], acc_v[i % NDB], 0, 0, 0);
            } else if (slot < DP_END)
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], r2f[slot >= DV_END && slot < DP_END ? slot - DV_END : 0], dp, 0, 0, 0);
            else {
                constexpr int i = slot >= DP_END ? slot - DP_END : 0;
                acc[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], pf[i / NDB], acc[i % NDB], 0, 0, 0);
            }
            SCHED_FENCE();
        };
        static_assert(NDB >= 2, "the second half of P and of dS is formed under the first NDB slots of its product");
        static_for<NSLOT>(run_slot);
    };

    int pf_tile = 0;
    int pend_len = 0;  // tiles of the stage whose statistics are in flight
    auto begin_stage = [&](int buf) {
        publish_stats(buf, pend_len);
        wait_vmcnt<0>();
        __syncthreads();
        pend_len = 0;
        if (pf_tile < n_tiles) {
            pend_len = stage_len(pf_tile);
            issue_stage(pf_tile, buf ^ 1);
            pf_tile += pend_len;
        }
    };
    const const_int_ptr wave_desc = (const_int_ptr)p.wave_desc;
    // Runs the reachable blocks of one staged tile (one code shape per block product, whichever mode).
    auto run_blocks = [&](auto mask_tag, bool run0, bool run1, const MaskArgs& ma, int buf, int j) __attribute__((always_inline)) {
        const unsigned tile_lds = lds_base + (unsigned)buf * STAGE_BYTES + (unsigned)j * (2 * TILE_BYTES);
        const float* tile_stats = stats + ((buf * TPS + j) * 2) * TILE_KEYS;
        if constexpr (MODE == kBwdQ && CLEAR_BWD_PIPELINED_Q) {
            if (run0) do_block_q(mask_tag, tile_lds, 0, ma);
            if (run1) do_block_q(mask_tag, tile_lds, 1, ma);
        } else if constexpr (MODE == kBwdKV && CLEAR_BWD_PIPELINED_KV) {
            if constexpr (CLEAR_BWD_PIPELINED_KV == 2) {
                if (run0) do_block_kv_early(mask_tag, tile_lds, 0, ma, tile_stats);
                if (run1) do_block_kv_early(mask_tag, tile_lds, 1, ma, tile_stats);
            } else {
                if (run0) do_block_kv(mask_tag, tile_lds, 0, ma, tile_stats);
                if (run1) do_block_kv(mask_tag, tile_lds, 1, ma, tile_stats);
            }
        } else {
            if (run0) do_block(mask_tag, tile_lds, 0, ma, tile_stats);
            if (run1) do_block(mask_tag, tile_lds, 1, ma, tile_stats);
        }
    };
    auto run_tile = [&](auto mask_tag, int t, int buf, int j) __attribute__((always_inline)) {
        if constexpr (decltype(mask_tag)::value == kMaskTable) {
            // image tiles inside the grid: what this wave does with the tile was worked out on the host (the mask-table
            // entries of its two blocks, the all-zeros entry for a block out of reach, or kWaveSkipsTile)
            const int d = wave_desc[(long long)(csr_begin + t - n_lin_tiles) * NW + wave];
            if (d == kWaveSkipsTile || !wave_has_rows) return;
            const int zeros = (2 * p.mask_ry + 1) * (2 * p.mask_rx + 1) + 1;
            const int i0 = d & 0xffff, i1 = (int)((unsigned)d >> 16);
            MaskArgs ma;
            ma.row[0] = mask_tbl + 16 * i0;
            ma.row[1] = mask_tbl + 16 * i1;
            run_blocks(mask_tag, i0 != zeros, i1 != zeros, ma, buf, j);
            return;
        }
        int ta, tb;
        tile_origin(t, ta, tb);
        const bool linear = tb < 0;
        int cls0, cls1;
        if (!wave_has_rows) {
            cls0 = cls1 = kBlockSkip;
        } else if (linear) {
            cls0 = classify_linear_block(ta, 32, lin_limit);
            cls1 = classify_linear_block(ta + 32, 32, lin_limit);
        } else if (CODE == kCodeFull) {
            cls0 = classify_full_block(wy0, wx0, rH, rW, ta, tb, kKeyBlockH, kKeyBlockW, cH, cW);
            cls1 = classify_full_block(wy0, wx0, rH, rW, ta + kKeyBlockH, tb, kKeyBlockH, kKeyBlockW, cH, cW);
        } else if (CODE == kCodeDisc) {
            cls0 = classify_image_block(wy0, wx0, kWaveQH, kWaveQW, ta, tb, kKeyBlockH, kKeyBlockW, p.gridH, p.gridW, p.r2);
            cls1 = classify_image_block(wy0, wx0, kWaveQH, kWaveQW, ta + kKeyBlockH, tb, kKeyBlockH, kKeyBlockW, p.gridH, p.gridW, p.r2);
        } else {
            const MaskSpec spec = {p.mask_kind, p.mask_r, p.mask_shift};
            cls0 = classify_image_block_spec(spec, wy0, wx0, kWaveQH, kWaveQW, ta, tb, kKeyBlockH, kKeyBlockW, p.gridH, p.gridW);
            cls1 = classify_image_block_spec(spec, wy0, wx0, kWaveQH, kWaveQW, ta + kKeyBlockH, tb, kKeyBlockH, kKeyBlockW, p.gridH, p.gridW);
        }
        MaskArgs ma;
        const LaneRow tile_row = lane_row();
        ma.hh = tile_row.hh;
        ma.a = ta;
        ma.b = linear ? lin_limit : tb;
        ma.qy = tile_row.ry; ma.qx = tile_row.rx; ma.gridH = cH; ma.gridW = cW; ma.r2 = p.r2;
        ma.kind = p.mask_kind; ma.r = p.mask_r; ma.shift = p.mask_shift;
        ma.row[0] = ma.row[1] = mask_tbl;
        if (!LINROWS && !linear && p.mask_tbl) {
            const int ncol = 2 * p.mask_rx + 1;
            const int ones = (2 * p.mask_ry + 1) * ncol, zeros = ones + 1;
            const int dbx = (tb - wx0) >> 3, dby = (ta - wy0) >> 2;
            const int i0 = (cls0 == kBlockPartial) ? (dby + p.mask_ry) * ncol + dbx + p.mask_rx : (cls0 == kBlockFull ? ones : zeros);
            const int i1 = (cls1 == kBlockPartial) ? (dby + 1 + p.mask_ry) * ncol + dbx + p.mask_rx : (cls1 == kBlockFull ? ones : zeros);
            ma.row[0] = mask_tbl + 16 * i0;
            ma.row[1] = mask_tbl + 16 * i1;
        }
        run_blocks(mask_tag, cls0 != kBlockSkip, cls1 != kBlockSkip, ma, buf, j);
    };
    auto run_category = [&](auto mask_tag, int& t, int end, int& buf) __attribute__((always_inline)) {
        for (; t < end; t += TPS, buf ^= 1) {
            begin_stage(buf);
#pragma unroll 1
            for (int j = 0; j < imin(TPS, end - t); ++j) run_tile(mask_tag, t + j, buf, j);
        }
        t = end;
    };

    // prologue: the first stage is in flight
    if (n_tiles > 0) {
        pend_len = stage_len(0);
        issue_stage(0, 0);
        pf_tile = pend_len;
    }
    int buf = 0, t = 0;
    run_category(std::integral_constant<int, kMaskNone>{}, t, cb1, buf);
    run_category(std::integral_constant<int, kMaskLinear>{}, t, cb2, buf);
    if (!LINROWS) {
        if constexpr (dense_image)
            run_category(std::integral_constant<int, kMaskNone>{}, t, cb3, buf);
        else
            run_category(std::integral_constant<int, kMaskTable>{}, t, cb3, buf);
        run_category(std::integral_constant<int, kMaskImage>{}, t, cb4, buf);
    }
    // ---- epilogue
    const LaneRow out_row = lane_row();
    if (!out_row.valid) return;
    const int out_token = out_row.token, out_hh = out_row.hh;
    const float out_scale = MODE == kBwdV ? 1.0f : p.scale;  // dQ and dK carry the 1 / sqrt(d) of the logits
    if (LINROWS) {
        // partial sums of this column split: [mode][bh][split][row][d] fp32
        constexpr int slot0 = MODE == kBwdKV ? (int)kBwdK : MODE;
        float* wo = p.ws + ((((long long)slot0 * p.B * p.H + bh) * p.n_splits + split) * p.n_text + out_token) * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v = {acc[db][4 * g] * out_scale, acc[db][4 * g + 1] * out_scale, acc[db][4 * g + 2] * out_scale, acc[db][4 * g + 3] * out_scale};
                *(f32x4*)(wo + 32 * db + 8 * g + 4 * out_hh) = v;
            }
        if constexpr (MODE == kBwdKV) {
            float* wv = p.ws + ((((long long)kBwdV * p.B * p.H + bh) * p.n_splits + split) * p.n_text + out_token) * D;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 v = {acc_v[db][4 * g], acc_v[db][4 * g + 1], acc_v[db][4 * g + 2], acc_v[db][4 * g + 3]};
                    *(f32x4*)(wv + 32 * db + 8 * g + 4 * out_hh) = v;
                }
        }
    } else {
        const TensorStrides& outs = MODE == kBwdQ ? p.dqs : (MODE == kBwdV ? p.dvs : p.dks);
        __bf16* orow = (__bf16*)(MODE == kBwdQ ? p.dQ : (MODE == kBwdV ? p.dV : p.dK)) + batch * outs.sb + head * outs.sh + (long long)out_token * outs.sn;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 v;
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = (__bf16)(acc[db][4 * g + u] * out_scale);
                *(bf16x4*)(orow + 32 * db + 8 * g + 4 * out_hh) = v;
            }
        if constexpr (MODE == kBwdKV) {
            __bf16* vrow = (__bf16*)p.dV + batch * p.dvs.sb + head * p.dvs.sh + (long long)out_token * p.dvs.sn;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 v;
#pragma unroll
                    for (int u = 0; u < 4; ++u) v[u] = (__bf16)acc_v[db][4 * g + u];
                    *(bf16x4*)(vrow + 32 * db + 8 * g + 4 * out_hh) = v;
                }
        }
    }
}

template <int MODE, bool LINROWS, int CODE>
__global__ void __launch_bounds__(512, 1) clear_bwd_bf16_kernel(const BwdParams p)
{
    clear_bwd_bf16_workgroup<MODE, LINROWS, CODE>(p, (int)blockIdx.x, (int)gridDim.x);
}

// The four independent kernels of a backward pass in one launch, longest workgroups first: [0, n_image) dK and dV of
// the image keys, [n_image, 2 n_image) dQ of the image queries, then n_text_wgs workgroups for dK and dV of the text
// keys and as many for dQ of the text queries.  For problems of a few rounds of workgroups, where four launches, one
// after the other or on two streams, leave CUs idle between them.  (delta comes from clear_bwd_delta_kernel here.)
template <int CODE>
__global__ void __launch_bounds__(512, 1) clear_bwd_bf16_all_kernel(const BwdParams p, const int n_image, const int n_text_wgs)
{
    int bid = (int)blockIdx.x;
    if (bid < n_image) return clear_bwd_bf16_workgroup<kBwdKV, false, CODE>(p, bid, n_image);
    bid -= n_image;
    if (bid < n_image) return clear_bwd_bf16_workgroup<kBwdQ, false, CODE>(p, bid, n_image);
    bid -= n_image;
    if (bid < n_text_wgs) return clear_bwd_bf16_workgroup<kBwdKV, true, kCodeDisc>(p, bid, n_text_wgs);
    clear_bwd_bf16_workgroup<kBwdQ, true, kCodeDisc>(p, bid - n_text_wgs, n_text_wgs);
}

// delta_i = dO_i . O_i for every row: D / 8 lanes per row (8 channels = 16 bytes each).
__global__ void __launch_bounds__(256) clear_bwd_delta_kernel(const __bf16* O, TensorStrides os, const __bf16* dO, TensorStrides dos, int H,
                                                              long long N, float* delta, long long rows)
{
    auto offset = [&](long long row, const TensorStrides& st) {  // row = (b * H + h) * N + token
        const long long bh = row / N, t = row % N;
        return (bh / H) * st.sb + (bh % H) * st.sh + t * st.sn;
    };
    const long long row = (long long)blockIdx.x * (256 / CHUNKS) + threadIdx.x / CHUNKS;
    const int part = threadIdx.x % CHUNKS;
    float s = 0.f;
    if (row < rows) {
        const bf16x8 o = *(const bf16x8*)(O + offset(row, os) + 8 * part);
        const bf16x8 g = *(const bf16x8*)(dO + offset(row, dos) + 8 * part);
#pragma unroll
        for (int j = 0; j < 8; ++j) s += (float)o[j] * (float)g[j];
    }
#pragma unroll
    for (int off = CHUNKS / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (row < rows && part == 0) delta[row] = s;
}

// Adds up the column-split partial sums of the text rows and stores them as bf16: one workgroup per
// (mode, batch*head, text row), one thread per channel.
__global__ void __launch_bounds__(D) clear_bwd_reduce_kernel(const BwdParams p)
{
    const int ch = threadIdx.x;
    const long long BHn = (long long)p.B * p.H * p.n_text;
    const int mode = (int)(blockIdx.x / BHn);
    const long long row = blockIdx.x % BHn;
    const int bh = (int)(row / p.n_text), q = (int)(row % p.n_text);
    float s = 0.f;
    for (int k = 0; k < p.n_splits; ++k)
        s += p.ws[((((long long)mode * p.B * p.H + bh) * p.n_splits + k) * p.n_text + q) * D + ch];
    __bf16* out = (__bf16*)(mode == kBwdQ ? p.dQ : (mode == kBwdK ? p.dK : p.dV));
    const TensorStrides& st = mode == kBwdQ ? p.dqs : (mode == kBwdK ? p.dks : p.dvs);
    out[(bh / p.H) * st.sb + (bh % p.H) * st.sh + q * st.sn + ch] = (__bf16)s;
}

template <int MODE, bool LINROWS, int CODE>
hipError_t launch_bwd_code(const BwdParams& p, int nblk, hipStream_t stream)
{
    auto kern = clear_bwd_bf16_kernel<MODE, LINROWS, CODE>;
    static LdsLimitOnce lds_limit;  // one per kernel instantiation
    hipError_t e = lds_limit.ensure((const void*)kern, BWD_LDS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(nblk), dim3(512), BWD_LDS_BYTES, stream, p);
    return hipGetLastError();
}

template <int CODE>
hipError_t launch_bwd_all(const BwdParams& p, int n_image, int n_text_wgs, hipStream_t stream)
{
    auto kern = clear_bwd_bf16_all_kernel<CODE>;
    static LdsLimitOnce lds_limit;  // one per kernel instantiation
    hipError_t e = lds_limit.ensure((const void*)kern, BWD_LDS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(2 * n_image + 2 * n_text_wgs), dim3(512), BWD_LDS_BYTES, stream, p, n_image, n_text_wgs);
    return hipGetLastError();
}

// One kernel per family of image masks for the image rows; text rows meet every token and need none.
template <int MODE, bool LINROWS>
hipError_t launch_bwd(const BwdParams& p, int nblk, hipStream_t stream)
{
    if constexpr (LINROWS) {
        return launch_bwd_code<MODE, LINROWS, kCodeDisc>(p, nblk, stream);
    } else {
        const int code = mask_code_of(p.mask_kind);
        return code == kCodeDisc   ? launch_bwd_code<MODE, LINROWS, kCodeDisc>(p, nblk, stream)
               : code == kCodeFull ? launch_bwd_code<MODE, LINROWS, kCodeFull>(p, nblk, stream)
                                   : launch_bwd_code<MODE, LINROWS, kCodeGeneric>(p, nblk, stream);
    }
}

}  // namespace

hipError_t launch_bf16_backward(const BwdParams& p, const void* O, float* delta, hipStream_t stream, int phase)
{
    const int BH = p.B * p.H;
    const bool all = phase == kBwdPhaseAll;
    hipError_t e = hipSuccess;
    // (kBwdPhaseAll: no delta kernel; the dQ kernels form delta and run before the dK / dV kernels, which read it)
    if (phase == kBwdPhaseDelta) {
        const long long rows = (long long)BH * p.N;
        constexpr int rows_per_block = 256 / CHUNKS;
        hipLaunchKernelGGL(clear_bwd_delta_kernel, dim3((unsigned)((rows + rows_per_block - 1) / rows_per_block)), dim3(256), 0, stream, (const __bf16*)O, p.os, (const __bf16*)p.dO, p.dos, p.H, p.N, delta, rows);
        e = hipGetLastError();
    }
    const int nimg = BH * p.n_classes * p.n_q_tiles;
#if CLEAR_BWD_FUSED_KV
    if (phase == kBwdPhaseFour) {
        const int nlin4 = p.n_text > 0 ? BH * p.n_tq_tiles * p.n_splits : 0;
        const int code = mask_code_of(p.mask_kind);
        return code == kCodeDisc   ? launch_bwd_all<kCodeDisc>(p, nimg, nlin4, stream)
               : code == kCodeFull ? launch_bwd_all<kCodeFull>(p, nimg, nlin4, stream)
                                   : launch_bwd_all<kCodeGeneric>(p, nimg, nlin4, stream);
    }
#endif
    const int nlin = p.n_text > 0 ? BH * p.n_tq_tiles * p.n_splits : 0;
    BwdParams pq = p;  // for the dQ kernels
    if (all) {
        pq.O = O;
        pq.delta_out = delta;
    }
    if (e == hipSuccess && (all || phase == kBwdPhaseImageQ)) e = launch_bwd<kBwdQ, false>(pq, nimg, stream);
    if (e == hipSuccess && nlin > 0 && (all || phase == kBwdPhaseTextQ)) e = launch_bwd<kBwdQ, true>(pq, nlin, stream);
    if (e == hipSuccess && (all || phase == kBwdPhaseImageKV)) {
#if CLEAR_BWD_FUSED_KV
        e = launch_bwd<kBwdKV, false>(p, nimg, stream);
#else
        e = launch_bwd<kBwdK, false>(p, nimg, stream);
        if (e == hipSuccess) e = launch_bwd<kBwdV, false>(p, nimg, stream);
#endif
    }
    if (e != hipSuccess || p.n_text == 0) return e;
    if (e == hipSuccess && (all || phase == kBwdPhaseTextKV)) {
#if CLEAR_BWD_FUSED_KV
        e = launch_bwd<kBwdKV, true>(p, nlin, stream);
#else
        e = launch_bwd<kBwdK, true>(p, nlin, stream);
        if (e == hipSuccess) e = launch_bwd<kBwdV, true>(p, nlin, stream);
#endif
    }
    if (e == hipSuccess && (all || phase == kBwdPhaseReduce)) {
        hipLaunchKernelGGL(clear_bwd_reduce_kernel, dim3((unsigned)(3LL * BH * p.n_text)), dim3(D), 0, stream, p);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace clear
