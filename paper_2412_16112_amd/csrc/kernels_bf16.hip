// bf16 MFMA kernels for the CLEAR local-attention forward pass on gfx950 (head_dim 128; kernels_bf16_d64.hip
// compiles this file a second time for head_dim 64).
//
// Everything is computed "transposed" so that one lane owns one query for the whole pass:
//   S^T = K_blk * Q^T   (32 keys x 32 queries per MFMA tile, A = keys from LDS, B = queries in VGPRs)
//   O^T += V_blk^T * P^T (A = V read from LDS with the 16-bit transpose load, B = P^T straight from
//                         the S^T accumulators: the accumulator layout of one MFMA is the B-operand
//                         layout of the next, up to a fixed permutation of the contraction index
//                         that the V loads follow)
// With v_mfma_f32_32x32x16_bf16, lane l holds column n = l % 32 (its query) and rows
// 8*(reg/4) + 4*(l/32) + reg%4 of every 32 x 32 accumulator tile, so the row maximum and the
// softmax denominator of Eq. 1 need one exchange with lane l ^ 32 and no LDS round trip.
//
// A workgroup of NWY x NWX waves owns a (4*NWY) x (8*NWX) patch of image queries (or 32*NWY*NWX
// text queries) and walks a list of 64-key tiles: the text keys, then the 8 x 8 image key tiles its
// schedule row lists (Sec. 3.2: text keys for every query, image keys inside the radius-r disc).
// K and V tiles are staged in LDS once per workgroup, by four further waves that do nothing else
// (one per SIMD, one stage ahead of the computing waves, one workgroup barrier per stage); every
// computing wave classifies each 32-key block against its own 4 x 8 query patch and skips the blocks
// its disc cannot reach.
#include <hip/hip_runtime.h>

#include "bf16_common.h"
#include "block_class.h"
#include "clear_internal.h"

#if CLEAR_HEAD_DIM == 64
// second compilation of this file: its own kernel and launcher names
#define clear_fwd_bf16_kernel clear_fwd_bf16_d64_kernel
#define clear_fwd_bf16_both_kernel clear_fwd_bf16_d64_both_kernel
#define launch_bf16 launch_bf16_d64
#else
#define launch_bf16 launch_bf16_d128
#endif

namespace clear {
namespace {

// Careful pass, one staged tile: block by block, exact running maximum, O and the denominator rescaled
// at every block (Eq. 1 as a textbook online softmax).  Slow; only runs when the fast pass gave up.
template <int CODE>
__device__ __forceinline__ void careful_stage(WaveState& ws, const bf16x8 (&qf)[KS], const LaneOffsets& lo, unsigned tile_lds,
                                              int cls0, int cls1, bool linear, const MaskArgs& ma)
{
    const TileAddr ta = tile_addr(tile_lds, lo);
#pragma unroll 1
    for (int kb = 0; kb < 2; ++kb) {
        const int cls = kb ? cls1 : cls0;
        if (cls == kBlockSkip) continue;
        f32x16 s = qk_block(ta, kb, qf);
        if (cls == kBlockPartial) {
            if (linear)
                apply_mask<kMaskLinear, CODE>(s, kb, ma);
            else
                apply_mask<kMaskImage, CODE>(s, kb, ma);
        }
        const float m_new = fmaxf(ws.m_run, wave_pair_max(max_block(s)));
        const float alpha = __builtin_amdgcn_exp2f((ws.m_run - m_new) * ws.c);
        ws.l_run *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) ws.oacc[db][r] *= alpha;
        ws.m_run = m_new;
        bf16x8 pf[2];
        ws.l_run += exp_block(s, ws.c, m_new * ws.c, pf);
        pv_block(ws.oacc, ta, kb, pf);
    }
}

// Reference maximum of the fast pass: a query adopts the maximum of the first block in which it sees an
// admissible key (nothing has been accumulated for it before, so nothing needs rescaling) and keeps it:
// all later exponentials are taken relative to it, 2^{(s - m_ref) c}, whatever their size.  Whether that
// stayed within the range of fp32 is checked once, on the finished sums.
__device__ __forceinline__ void adopt_reference(WaveState& ws, float mx_pair)
{
    ws.m_run = (ws.m_run == M_INIT) ? fmaxf(mx_pair, M_INIT) : ws.m_run;
}

// Loading waves: CLEAR_LOADER_WAVES extra waves per workgroup do nothing but issue the staging loads, one stage
// ahead of the computing waves, which then never stall on the memory pipeline's issue queue.  0 = every
// wave stages its share of each tile itself, right after the stage barrier.
#ifndef CLEAR_LOADER_WAVES
#define CLEAR_LOADER_WAVES 4
#endif
constexpr int kLoaderWaves = CLEAR_LOADER_WAVES;

// Fast pass, one staged tile.  The reference maximum of a query never moves once set, so O is only
// ever touched by the matrix pipeline and there is no data-dependent branch.
// The tile's two 32-key blocks run as one hand-ordered pipeline of 32 matrix instructions (head_dim 128;
// 16 at head_dim 64, where every phase below is half as long and carries two score pairs per slot):
//   slots  0- 7  S of block 0
//   slots  8-15  S of block 1                      | mask, maximum, reference, P[0..7] of block 0
//   slots 16-19  P V of block 0, keys of P[0..7]   | P[8..15] of block 0
//   slots 20-23  P V of block 0, keys of P[8..15]  | mask, maximum, reference, P[0..7] of block 1
//   slots 24-27  P V of block 1, keys of P[0..7]   | P[8..15] of block 1
//   slots 28-31  P V of block 1, keys of P[8..15]
// LDS operands are read two slots ahead of the matrix instruction that consumes them.
// A wave runs the whole tile or none of it: a block its disc cannot reach is masked out entirely (its
// scores become -inf, its P zero), which keeps one code shape for every tile of a loop.
// ADOPT = true while some query of the wave still has no reference maximum (the first tiles): the block
// maxima are formed and adopted.  ADOPT = false afterwards: no maximum is needed at all.
template <int MASK, bool ADOPT, int CODE>
__device__ __forceinline__ void fast_stage(WaveState& ws, const bf16x8 (&qf)[KS], const LaneOffsets& lo,
                                           unsigned tile_lds, const MaskArgs& ma)
{
    constexpr int kb0 = 0;
    constexpr bool has1 = true;
    const TileAddr ta = tile_addr(tile_lds, lo);
    const float c = ws.c;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    bf16x8 pf0[2], pf1[2];
    float sum = 0.f;

    // slots: [0, S1) S of block 0, [S1, PV0) S of block 1, [PV0, PV1) P V of block 0, [PV1, NSLOT) P V of block 1
    constexpr int S1 = KS, PV0 = 2 * KS, PV1 = PV0 + 2 * NDB, NSLOT = PV1 + 2 * NDB;
    // operand ring: K operands for the S slots, V operands for the P V slots (V slot i: s2 = (i / NDB) % 2, db = i % NDB)
    auto k_operand = [&](int slot) { return read_k_operand(ta, slot / KS, slot % KS); };
    auto v_operand = [&](int slot) {
        const int i = slot - PV0;
        return read_v_operand(ta, i / (2 * NDB), (i / NDB) & 1, i % NDB);
    };
    auto block1_slot = [](int slot) { return (slot >= S1 && slot < PV0) || slot >= PV1; };
    // operands are read PD slots ahead into a ring of PD + 2 (the extra entry keeps a read from landing on
    // the registers the previous matrix instruction is still reading)
    constexpr int PD = CLEAR_OPERAND_PREFETCH, RING = PD + 2;
    bf16x8 op[RING];
#pragma unroll
    for (int i = 0; i < PD; ++i) op[i] = k_operand(i);
    f32x16 s0 = zero, s1 = zero;
    float mc = ws.m_run * c, mc1 = mc;
    // kMaskTable: the 16 lane masks of a block sit in scalar registers.  Block 0's are fetched before the
    // pipeline starts (their latency overlaps that of the first LDS operands), block 1's as soon as block
    // 0's have been used, a dozen slots before they are needed.
    unsigned long long mw[16];
    if (MASK == kMaskTable) {
#pragma unroll
        for (int r = 0; r < 16; ++r) mw[r] = ma.row[kb0 & 1][r];
    }
    auto run_slot = [&](auto slot_tag) __attribute__((always_inline)) {
        constexpr int slot = decltype(slot_tag)::value;
        // prefetch the operand of slot + PD
        if (slot + PD < NSLOT && (!block1_slot(slot + PD) || has1)) {
            if (slot + PD < PV0)
                op[(slot + PD) % RING] = k_operand(slot + PD);
            else
                op[(slot + PD) % RING] = v_operand(slot + PD);
        }
        // matrix instruction of this slot
        constexpr int pv_i = slot >= PV0 ? slot - PV0 : 0, pv_db = pv_i % NDB, pv_s2 = (pv_i / NDB) & 1;
        if (slot < S1)
            s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], qf[slot], s0, 0, 0, 0);
        else if (slot < PV0) {
            if (has1) s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], qf[slot - S1], s1, 0, 0, 0);
        } else if (slot < PV1)
            ws.oacc[pv_db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], pf0[pv_s2], ws.oacc[pv_db], 0, 0, 0);
        else if (has1)
            ws.oacc[pv_db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[slot % RING], pf1[pv_s2], ws.oacc[pv_db], 0, 0, 0);
        // vector work riding along
        if (slot == S1) {
            if (MASK == kMaskTable) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s0[r] = __builtin_amdgcn_inverse_ballot_w64(mw[r]) ? s0[r] : -INFINITY;
            } else {
                apply_mask<MASK, CODE>(s0, kb0, ma);
            }
            if (ADOPT) {
                adopt_reference(ws, wave_pair_max(max_block(s0)));
                mc = ws.m_run * c;
            }
        }
        if (slot == S1 + 1 && MASK == kMaskTable) {
#pragma unroll
            for (int r = 0; r < 16; ++r) mw[r] = ma.row[(kb0 + 1) & 1][r];
        }
        if (slot == PV0 && has1) {
            if (MASK == kMaskTable) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s1[r] = __builtin_amdgcn_inverse_ballot_w64(mw[r]) ? s1[r] : -INFINITY;
            } else {
                apply_mask<MASK, CODE>(s1, kb0 + 1, ma);
            }
            if (ADOPT) {
                adopt_reference(ws, wave_pair_max(max_block(s1)));
                mc1 = ws.m_run * c;
            }
        }
        // Exponentials as a three-deep vector pipeline over pairs of scores, so that the instructions of
        // one slot do not wait on each other: at head_dim 128 pair g of block 0 is scaled in slot 8 + g,
        // exponentiated in slot 9 + g, summed and packed in slot 10 + g; block 1 runs the same eight slots
        // later.  P[0..7] of a block is complete three slots before the matrix instruction that needs it.
        // (head_dim 64: two pairs per slot from slot 4 on, block 1 four slots later.)
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            constexpr int PPS = 8 / KS;  // score pairs per slot
            const int b0 = S1 + g / PPS, b1 = PV0 + g / PPS;
            if (slot == b0) {
                s0[2 * g] = __builtin_fmaf(s0[2 * g], c, -mc);
                s0[2 * g + 1] = __builtin_fmaf(s0[2 * g + 1], c, -mc);
            }
            if (slot == b0 + 1) {
                s0[2 * g] = __builtin_amdgcn_exp2f(s0[2 * g]);
                s0[2 * g + 1] = __builtin_amdgcn_exp2f(s0[2 * g + 1]);
            }
            if (slot == b0 + 2) {
                sum += s0[2 * g] + s0[2 * g + 1];
                pf0[g >> 2][2 * (g & 3)] = (__bf16)s0[2 * g];
                pf0[g >> 2][2 * (g & 3) + 1] = (__bf16)s0[2 * g + 1];
            }
            if (has1) {
                if (slot == b1) {
                    s1[2 * g] = __builtin_fmaf(s1[2 * g], c, -mc1);
                    s1[2 * g + 1] = __builtin_fmaf(s1[2 * g + 1], c, -mc1);
                }
                if (slot == b1 + 1) {
                    s1[2 * g] = __builtin_amdgcn_exp2f(s1[2 * g]);
                    s1[2 * g + 1] = __builtin_amdgcn_exp2f(s1[2 * g + 1]);
                }
                if (slot == b1 + 2) {
                    sum += s1[2 * g] + s1[2 * g + 1];
                    pf1[g >> 2][2 * (g & 3)] = (__bf16)s1[2 * g];
                    pf1[g >> 2][2 * (g & 3) + 1] = (__bf16)s1[2 * g + 1];
                }
            }
        }
        SCHED_FENCE();
    };
    static_for<NSLOT>(run_slot);  // (not a loop: one that contains inline asm is not unrolled)
    ws.l_run += sum;
}

// One workgroup of a forward launch: workgroup `bid` of `nblk` (image-query rows, or with TEXTQ the text-query rows).
template <int NWY, int NWX, bool TEXTQ, int CODE>
__device__ __forceinline__ void clear_fwd_bf16_workgroup(const FwdParams& p, const int bid, const int nblk)
{
    constexpr int NW = NWY * NWX;
    constexpr int NI = TILE_KEYS / ROWS_PER_LOAD / NW;  // 1 KB load instructions per wave per tile, for K and for V each, when every wave loads
    static_assert(NI * NW * ROWS_PER_LOAD == TILE_KEYS, "the waves' load instructions cover the tile's 64 rows exactly");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];  // [NBUF][TPS][K tile | V tile]
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qi = lane & 31;   // query slot inside the wave's patch
    const int hh = lane >> 5;   // which half of the contraction slice this lane feeds
    // waves NW .. NW + NLW - 1 only load; with NLW = 0 every wave loads its share (NI row groups per tile)
    constexpr int NLW = kLoaderWaves;
    static_assert(NLW > 0 || NBUF == 2, "without loading waves a stage is fetched while the one before it is computed");
    constexpr int NI_L = NLW > 0 ? TILE_KEYS / ROWS_PER_LOAD / NLW : NI;
    static_assert(NLW == 0 || NI_L * NLW * ROWS_PER_LOAD == TILE_KEYS, "the loading waves' instructions cover the tile's 64 rows exactly");
    const bool loader = NLW > 0 && wave >= NW;
    const int ldw = NLW > 0 ? wave - NW : wave;  // index among the waves that load

    // ---- workgroup -> (batch*head, query tile[, key split]); XCD-aware: workgroups are dealt
    // round-robin to the 8 XCDs, so give each XCD one contiguous range of the logical index.
    int vid;
    {
        const int xcd = bid & 7, idx = bid >> 3;
        const int q = nblk >> 3, rem = nblk & 7;
        vid = xcd * q + imin(xcd, rem) + idx;
    }
    int bh, qt, split = 0;
    // Image queries live on a qH x qW grid and their image keys on a kH x kW grid; grid point (y, x) is image
    // token (y * stride + oy, x * stride + ox) of the raster.  Plain masks: both are the raster itself.
    // Strided mask: the workgroup belongs to one residue class of the queries, (q_oy, q_ox) = (y % stride,
    // x % stride), and reads the keys of the class moved by (stride_ry, stride_rx).
    // Row bands may move the grid down by y_shift rows in these coordinates (so that a query tile starts at the first
    // owned row): grid rows then start at y_shift, and only where a token's address is formed is the shift taken off.
    int stride = 1, q_oy = 0, q_ox = 0, k_oy = 0, k_ox = 0;
    const int y_shift = TEXTQ ? 0 : p.y_shift;
    int qH = p.gridH + y_shift, qW = p.gridW, kH = p.gridH + y_shift, kW = p.gridW;
    if (TEXTQ) {
        split = vid % p.n_splits;
        const int t = vid / p.n_splits;
        qt = t % p.n_tq_tiles;
        bh = t / p.n_tq_tiles;
    } else {
        qt = p.qt_begin + vid % p.n_q_tiles_launch;
        if (p.qt_order) qt = ((const_int_ptr)p.qt_order)[qt];  // the order in which a head's query tiles are dealt out
        bh = vid / p.n_q_tiles_launch;
        if (CODE == kCodeFull) {
            const int cls = bh % p.n_classes;
            bh /= p.n_classes;
            stride = p.stride;
            q_oy = cls / stride;
            q_ox = cls % stride;
            k_oy = (q_oy + p.stride_ry) % stride;
            k_ox = (q_ox + p.stride_rx) % stride;
            qH = (p.gridH - q_oy + stride - 1) / stride;  // >= 1: the host requires gridH, gridW >= stride
            qW = (p.gridW - q_ox + stride - 1) / stride;
            kH = (p.gridH - k_oy + stride - 1) / stride;
            kW = (p.gridW - k_ox + stride - 1) / stride;
        }
    }
    const int batch = bh / p.H, head = bh % p.H;
    const __bf16* const Qh = (const __bf16*)p.Q + batch * p.qs.sb + head * p.qs.sh;
    const unsigned char* const Kh = (const unsigned char*)((const __bf16*)p.K + batch * p.ks.sb + head * p.ks.sh);
    const unsigned char* const Vh = (const unsigned char*)((const __bf16*)p.V + batch * p.vs.sb + head * p.vs.sh);
    const unsigned k_pitch = (unsigned)p.ks.sn * 2, v_pitch = (unsigned)p.vs.sn * 2;  // bytes from one token row to the next

    // ---- this lane's query
    int wy0 = 0, wx0 = 0;  // origin of the wave's 4 x 8 query patch (image mode)
    int qy = 0, qx = 0;
    int q_token;
    bool q_valid, wave_has_queries;
    if (TEXTQ) {
        const int q0 = qt * (NW * 32) + wave * 32;
        q_token = q0 + qi;
        q_valid = q_token < p.n_text;
        wave_has_queries = q0 < p.n_text;
        if (!q_valid) q_token = p.n_text - 1;
    } else {
        wy0 = (qt / p.n_qtx) * (NWY * kWaveQH) + (wave / NWX) * kWaveQH;
        wx0 = (qt % p.n_qtx) * (NWX * kWaveQW) + (wave % NWX) * kWaveQW;
        qy = wy0 + (qi >> 3);
        qx = wx0 + (qi & 7);
        // (row-band mode: only the rows [own_y0, own_y1) carry queries; the halo rows are keys only)
        q_valid = qy < qH && qx < qW && qy >= p.own_y0 && qy < p.own_y1;
        wave_has_queries = wy0 < qH && wx0 < qW && wy0 < p.own_y1 && wy0 + kWaveQH > p.own_y0;
        q_token = p.n_text + (imax(imin(qy, qH - 1) - y_shift, 0) * stride + q_oy) * p.gridW + imin(qx, qW - 1) * stride + q_ox;
    }

    // Q^T as MFMA B operand: KS contraction steps of 16 channels; this lane supplies channels 16*s + 8*hh .. +7
    bf16x8 qf[KS];
    {
        const __bf16* qrow = Qh + (long long)q_token * p.qs.sn + 8 * hh;
#pragma unroll
        for (int s = 0; s < KS; ++s)  // (read once: non-temporal, so that the rows do not push K and V tiles out of the L2)
            if (!loader) qf[s] = __builtin_nontemporal_load((const bf16x8*)(qrow + 16 * s));
    }
    const const_int_ptr row_ptr = (const_int_ptr)p.row_ptr, col_idx = (const_int_ptr)p.col_idx, n_plain = (const_int_ptr)p.n_plain;
    const const_u64_ptr mask_tbl = (const_u64_ptr)p.mask_tbl;

    // ---- tile list: tokens [lin_begin, lin_limit) in 64-key tiles, then (image mode) the CSR row.
    // Tiles fall into four consecutive categories, each with its own code shape:
    //   [cb0, cb1) whole linear tiles   [cb1, cb2) the ragged linear tile (at most one)
    //   [cb2, cb3) image tiles inside the grid (masks from the table)   [cb3, cb4) image tiles cut by the border
    // A stage is up to TPS consecutive tiles of one category.
    int n_tiles, n_lin_tiles, csr_begin = 0;
    int lin_begin = 0, lin_limit = 0;
    if (TEXTQ) {
        lin_begin = split * p.split_keys;
        lin_limit = (long long)lin_begin + p.split_keys < p.NV ? lin_begin + p.split_keys : (int)p.NV;
        n_lin_tiles = (lin_limit - lin_begin + TILE_KEYS - 1) / TILE_KEYS;
        n_tiles = n_lin_tiles;
    } else {
        lin_limit = p.n_text;
        n_lin_tiles = (p.n_text + TILE_KEYS - 1) / TILE_KEYS;
        csr_begin = row_ptr[qt];
        n_tiles = n_lin_tiles + (row_ptr[qt + 1] - csr_begin);
    }
    const int cb1 = (lin_limit - lin_begin) / TILE_KEYS, cb2 = n_lin_tiles;
    constexpr bool dense_image = !TEXTQ && CODE == kCodeFull;  // strided: tiles inside the class grid need no mask
    const int cb3 = TEXTQ ? n_lin_tiles : ((p.mask_tbl || dense_image) ? n_lin_tiles + n_plain[qt] : n_lin_tiles);
    const int cb4 = n_tiles;
    auto stage_len = [&](int t) {  // tiles in the stage that starts at tile t
        const int e = t < cb1 ? cb1 : (t < cb2 ? cb2 : (t < cb3 ? cb3 : cb4));
        return imin(TPS, e - t);
    };

    // Tile origin: linear -> (first token, -1); image -> (row, col) of the 8 x 8 tile.
    auto tile_origin = [&](int i, int& a, int& b) {
        if (i < n_lin_tiles) {
            a = lin_begin + i * TILE_KEYS;
            b = -1;
        } else {
            const int packed = col_idx[csr_begin + i - n_lin_tiles];  // tile origin, row << 16 | col
            a = packed >> 16;
            b = packed & 0xffff;
        }
    };

    // ---- LDS-direct staging.  Load instruction ii of a tile covers ROWS_PER_LOAD rows (4 at head_dim 128); lane i
    // writes slot i % CHUNKS of row ROWS_PER_LOAD ii + i / CHUNKS and therefore fetches logical chunk (i % CHUNKS) ^ swz(row).
    // Addresses are clamped to valid tokens; slots beyond the range or the grid are masked in the compute.
    auto issue_tile = [&](int i, unsigned lds_tile) {
        int a, b;
        tile_origin(i, a, b);
        auto load_row_group = [&](auto n_tag) __attribute__((always_inline)) {
            const int ii = ldw * NI_L + decltype(n_tag)::value;
            const int row = ROWS_PER_LOAD * ii + lane / CHUNKS;
            int token;
            if (b < 0) {
                token = imin(a + row, lin_limit - 1);
                if (TEXTQ && token >= p.vkeys_text) token += p.vshift;  // position in the key list -> token
            } else {
                const int ky = imax(imin(a + (row >> 3), kH - 1) - y_shift, 0);  // (rows above the grid: out of every owned query's reach)
                const int kx = imin(b + (row & 7), kW - 1);
                token = p.n_text + (ky * stride + k_oy) * p.gridW + kx * stride + k_ox;
            }
            const unsigned chunk_off = (unsigned)(((lane % CHUNKS) ^ swz(row)) << 4);
            load_to_lds_16B(Kh, (unsigned)token * k_pitch + chunk_off, lds_tile + ii * 1024);
            load_to_lds_16B(Vh, (unsigned)token * v_pitch + chunk_off, lds_tile + TILE_BYTES + ii * 1024);
        };
        static_for<NI_L>(load_row_group);  // (not a loop: one that contains inline asm is not unrolled)
    };
    auto issue_stage = [&](int t, int buf) {  // the stage that starts at tile t goes to stage buffer buf
        const int len = stage_len(t);
        auto load_tile = [&](auto j_tag) __attribute__((always_inline)) {
            constexpr int j = decltype(j_tag)::value;
            if (j < len) issue_tile(t + j, lds_base + (unsigned)buf * STAGE_BYTES + (unsigned)j * (2 * TILE_BYTES));
        };
        static_for<TPS>(load_tile);
    };

    __shared__ int s_redo;  // set when the fast pass has to be repeated by the careful one
    auto stage_sync = [&]() {
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    if (NLW > 0 && loader) {
        // A loading wave walks the stage list like the computing waves, one barrier per stage, and stays one
        // stage ahead: after the barrier that hands stage s over, everyone has left the other buffer, which it
        // refills with stage s + 1.  Same barrier count as run_pass below, pass for pass.
        auto loader_pass = [&]() {
            constexpr int PFD = NBUF - 1;        // stages in flight ahead of the one being computed
            constexpr int LPS = TPS * 2 * NI_L;  // this wave's load instructions per full stage
            static_assert(PFD == 1 || TPS == 1, "counting loads per stage needs stages of one size");
            static_assert(PFD <= 3 && (PFD - 1) * LPS < 64, "the waits below are written out for up to three stages ahead");
            int nx = 0, nbuf = 0, n_issued = 0;
            for (int i = 0; i < PFD && nx < n_tiles; ++i) {
                issue_stage(nx, nbuf);
                nx += stage_len(nx);
                nbuf = next_buf(nbuf);
                ++n_issued;
            }
            int k = 0;
            for (int t = 0; t < n_tiles; ++k) {
                // stage k has landed once at most the loads of the stages issued after it are outstanding
                const int ahead = n_issued - 1 - k;
                if (PFD > 2 && ahead >= 2)
                    wait_vmcnt<(PFD > 2 ? 2 * LPS : 0)>();
                else if (PFD > 1 && ahead == 1)
                    wait_vmcnt<(PFD > 1 ? LPS : 0)>();
                else
                    wait_vmcnt<0>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                t += stage_len(t);
                if (nx < n_tiles) {
                    issue_stage(nx, nbuf);
                    nx += stage_len(nx);
                    nbuf = next_buf(nbuf);
                    ++n_issued;
                }
            }
            wait_vmcnt<0>();
        };
        loader_pass();
        __syncthreads();
        if (s_redo != 0) {
            __syncthreads();
            loader_pass();
            __syncthreads();
        }
        return;
    }

    // ---- running softmax state: one query per lane (shared with lane ^ 32)
    WaveState ws;
    ws.c = p.scale_log2e;

    // ---- per-lane LDS read offsets inside a staged tile
    LaneOffsets lo;
    // K operand: key row qi of the block, logical chunk 2 ks + hh (16 bytes = 8 channels)
    lo.k0 = (unsigned)(qi * ROW_BYTES + ((hh ^ swz(qi)) << 4));
    // V operand (transpose read): within each group of 16 lanes, lane j addresses key row j / 4 and channels
    // 4 (j % 4) .. + 3 of the group's 16-channel slice; it receives channel lane % 16 for 4 rows.  Rows of
    // the first read: 4 hh + j / 4 (+ 16 s2 + 32 blk), of the second: + 8.
    {
        const int j = lane & 15, g2 = (lane >> 4) & 1;
        const int row = 4 * hh + (j >> 2);
        const int chunk = 2 * g2 + ((j & 3) >> 1);
        lo.v0 = (unsigned)(row * ROW_BYTES + ((chunk ^ swz(row)) << 4) + 8 * (j & 1));
    }

    // Stage hand-over: this wave's loads of the stage about to be computed have landed; after the barrier
    // so have everyone's, and every wave has left the other buffer, which is refilled with the next stage.
    int pf_tile = 0;  // first tile of the next stage to load
    auto begin_stage = [&](int buf) {
        stage_sync();
        if (NLW == 0 && pf_tile < n_tiles) {
            issue_stage(pf_tile, buf ^ 1);
            pf_tile += stage_len(pf_tile);
        }
    };
    // Classifies the two key blocks of tile t against this wave's query patch and gathers what the
    // element masks need.
    struct TileInfo {
        int cls0, cls1;
        bool linear;
        unsigned tile_lds;  // LDS address of the staged tile (K half, then V half)
        MaskArgs ma;
    };
    auto tile_info = [&](int t, int buf, int j) -> TileInfo {
        TileInfo si;
        int ta, tb;
        tile_origin(t, ta, tb);
        si.linear = tb < 0;
        if (!wave_has_queries) {
            si.cls0 = si.cls1 = kBlockSkip;
        } else if (si.linear) {
            si.cls0 = classify_linear_block(ta, 32, lin_limit);
            si.cls1 = classify_linear_block(ta + 32, 32, lin_limit);
        } else if (TEXTQ) {
            si.cls0 = si.cls1 = kBlockSkip;
        } else if (CODE == kCodeFull) {
            si.cls0 = classify_full_block(wy0, wx0, qH, qW, ta, tb, kKeyBlockH, kKeyBlockW, kH, kW);
            si.cls1 = classify_full_block(wy0, wx0, qH, qW, ta + kKeyBlockH, tb, kKeyBlockH, kKeyBlockW, kH, kW);
        } else if (CODE == kCodeDisc) {
            si.cls0 = classify_image_block(wy0, wx0, kWaveQH, kWaveQW, ta, tb, kKeyBlockH, kKeyBlockW, kH, kW, p.r2);
            si.cls1 = classify_image_block(wy0, wx0, kWaveQH, kWaveQW, ta + kKeyBlockH, tb, kKeyBlockH, kKeyBlockW, kH, kW, p.r2);
        } else {
            const MaskSpec spec = {p.mask_kind, p.mask_r, p.mask_shift};
            si.cls0 = classify_image_block_spec(spec, wy0, wx0, kWaveQH, kWaveQW, ta, tb, kKeyBlockH, kKeyBlockW, kH, kW);
            si.cls1 = classify_image_block_spec(spec, wy0, wx0, kWaveQH, kWaveQW, ta + kKeyBlockH, tb, kKeyBlockH, kKeyBlockW, kH, kW);
        }
        si.tile_lds = lds_base + (unsigned)buf * STAGE_BYTES + (unsigned)j * (2 * TILE_BYTES);
        si.ma.hh = hh;
        si.ma.a = ta;                          // linear: first token of the tile; image: tile origin row
        si.ma.b = si.linear ? lin_limit : tb;  // linear: token limit;             image: tile origin col
        si.ma.qy = qy; si.ma.qx = qx; si.ma.gridH = kH; si.ma.gridW = kW; si.ma.r2 = p.r2;
        si.ma.kind = p.mask_kind; si.ma.r = p.mask_r; si.ma.shift = p.mask_shift;
        si.ma.row[0] = si.ma.row[1] = mask_tbl;
        if (!TEXTQ && !si.linear && p.mask_tbl) {
            // lane masks of the two blocks: whole blocks use the all-ones entry, unreachable blocks the all-zeros
            // entry at the end of the table
            const int ncol = 2 * p.mask_rx + 1;
            const int ones = (2 * p.mask_ry + 1) * ncol, zeros = ones + 1;
            const int dbx = (tb - wx0) >> 3;
            const int dby = (ta - wy0) >> 2;
            const int i0 = (si.cls0 == kBlockPartial) ? (dby + p.mask_ry) * ncol + dbx + p.mask_rx : (si.cls0 == kBlockFull ? ones : zeros);
            const int i1 = (si.cls1 == kBlockPartial) ? (dby + 1 + p.mask_ry) * ncol + dbx + p.mask_rx : (si.cls1 == kBlockFull ? ones : zeros);
            si.ma.row[0] = mask_tbl + 16 * i0;
            si.ma.row[1] = mask_tbl + 16 * i1;
        }
        return si;
    };

    // Image tiles inside the grid, lane masks from the table: what this wave does with each of them was worked out
    // on the host when the context was made (one word per tile and wave: the table entries of the tile's two
    // blocks, or kWaveSkipsTile), so the tile loop neither classifies nor computes mask addresses.  The words of
    // a stage are fetched before its barrier, whose wait hides their latency.
    const const_int_ptr wave_desc = (const_int_ptr)p.wave_desc;
    struct TableStage {
        int d[TPS];
    };
    auto table_stage = [&](int t) {
        TableStage ts;
#pragma unroll
        for (int j = 0; j < TPS; ++j) {
            const int e = imin(t + j, cb3 - 1) - n_lin_tiles;  // (a stage may end early: its last word is read twice)
            const int d = wave_desc[(long long)(csr_begin + e) * NW + wave];
            ts.d[j] = (t + j < cb3 && wave_has_queries) ? d : kWaveSkipsTile;
        }
        return ts;
    };
    auto stage_tile_lds = [&](int buf, int j) { return lds_base + (unsigned)buf * STAGE_BYTES + (unsigned)j * (2 * TILE_BYTES); };
    auto table_mask_args = [&](int d) {
        MaskArgs ma;
        ma.row[0] = mask_tbl + 16 * (d & 0xffff);
        ma.row[1] = mask_tbl + 16 * ((unsigned)d >> 16);
        return ma;
    };

    // Prologue of the block on the query row (RMS norm over the head's channels - this lane holds half of them,
    // lane ^ 32 the others -, rotary embedding for image queries, back to bf16).  Runs once, after the first
    // stage's loads have been issued, so that the wait for the row and for the tables overlaps them.
    auto query_prologue = [&]() __attribute__((always_inline)) {
    if (p.q_gain || p.rope_y) {
        float ss = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int j = 0; j < 8; ++j) ss += (float)qf[s][j] * (float)qf[s][j];
        ss = wave_pair_sum(ss);
        const float inv_rms = 1.0f / sqrtf(ss * (1.0f / D) + p.norm_eps);
        const bool has_gain = p.q_gain != nullptr;
        const bool turn = !TEXTQ && p.rope_y;
        // Table entries are fetched without branches, half of the chunks at a time, so that the loads of a half
        // are in flight together (one memory round trip per half, not one per chunk).  A step that is switched
        // off reads the other step's table instead (any D readable floats) and ignores what it read.
        const float* const any_table = has_gain ? p.q_gain : p.rope_y;
        const float* const ysrc = turn ? p.rope_y + (size_t)(imax(imin(qy, qH - 1) - y_shift, 0) * stride + q_oy) * D : any_table;
        const float* const xsrc = turn ? p.rope_x + (size_t)(imin(qx, qW - 1) * stride + q_ox) * D : any_table;
        constexpr int HALF = KS / 2;
#pragma unroll
        for (int h0 = 0; h0 < KS; h0 += HALF) {
            f32x4 g[HALF][2], a[HALF][2], b[HALF][2];
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                const int c0 = 16 * (h0 + i) + 8 * hh;
                g[i][0] = *(const f32x4*)(any_table + c0);
                g[i][1] = *(const f32x4*)(any_table + c0 + 4);
                a[i][0] = *(const f32x4*)(ysrc + c0);
                a[i][1] = *(const f32x4*)(ysrc + c0 + 4);
                b[i][0] = *(const f32x4*)(xsrc + c0);
                b[i][1] = *(const f32x4*)(xsrc + c0 + 4);
            }
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                const int s = h0 + i;
                float x[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) x[j] = (float)qf[s][j];
                prologue_chunk_values(x, inv_rms, has_gain, g[i][0], g[i][1], turn, a[i][0], a[i][1], b[i][0], b[i][1]);
#pragma unroll
                for (int j = 0; j < 8; ++j) qf[s][j] = (__bf16)x[j];
            }
        }
    }

    };

    // One pass over the stage list.  CAREFUL = false: fast pass (fixed reference maximum); returns the
    // lanes that ran out of headroom.  CAREFUL = true: exact online softmax, slow.
    auto run_pass = [&](auto careful_tag) -> unsigned long long {
        constexpr bool CAREFUL = decltype(careful_tag)::value;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) ws.oacc[db][r] = 0.f;
        ws.m_run = M_INIT;
        ws.l_run = 0.f;
        unsigned long long bad = 0;
        // prologue: the first stage is in flight
        pf_tile = 0;
        if (NLW == 0 && n_tiles > 0) {
            issue_stage(0, 0);
            pf_tile = stage_len(0);
        }
        // The Q fragments are waited for here, once, with the first tiles already on their way: otherwise the
        // wait lands inside the key loop, where it would also drain the tile prefetches.
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(qf[s]));
        if (!CAREFUL) query_prologue();  // the fast pass always comes first
        int buf = 0;
        if (CAREFUL) {
            for (int t = 0; t < n_tiles;) {
                begin_stage(buf);
                const int len = stage_len(t);
                for (int j = 0; j < len; ++j) {
                    const TileInfo si = tile_info(t + j, buf, j);
                    careful_stage<CODE>(ws, qf, lo, si.tile_lds, si.cls0, si.cls1, si.linear, si.ma);
                }
                t += len;
                buf = next_buf(buf);
            }
        } else {
            // One loop per tile category (and per mode), so that every loop body has a single shape.  Each
            // category starts in "adopt" mode and switches to the leaner loop once every query of the wave
            // has its reference maximum.
            bool adopting = true;
            auto still_adopting = [&]() { return __builtin_amdgcn_ballot_w64(ws.m_run == M_INIT) != 0; };
            int t = 0;

            // whole linear tiles
            for (; t < cb1 && adopting; t += TPS, buf = next_buf(buf)) {
                begin_stage(buf);
#pragma unroll 1
                for (int j = 0; j < imin(TPS, cb1 - t); ++j) {
                    const TileInfo si = tile_info(t + j, buf, j);
                    if (wave_has_queries) fast_stage<kMaskNone, true, CODE>(ws, qf, lo, si.tile_lds, si.ma);
                }
                adopting = wave_has_queries && still_adopting();
            }
            for (; t < cb1; t += TPS, buf = next_buf(buf)) {
                begin_stage(buf);
#pragma unroll 1
                for (int j = 0; j < imin(TPS, cb1 - t); ++j) {
                    const TileInfo si = tile_info(t + j, buf, j);
                    if (wave_has_queries) fast_stage<kMaskNone, false, CODE>(ws, qf, lo, si.tile_lds, si.ma);
                }
            }
            t = cb1;
            // the ragged linear tile: at most one, keep it simple
            for (; t < cb2; t += TPS, buf = next_buf(buf)) {
                begin_stage(buf);
                const TileInfo si = tile_info(t, buf, 0);
                if (si.cls0 != kBlockSkip) {
                    fast_stage<kMaskLinear, true, CODE>(ws, qf, lo, si.tile_lds, si.ma);
                    adopting = still_adopting();
                }
            }
            t = cb2;
            if constexpr (dense_image) {
                // strided mask, tiles inside the class grid: every key of the tile is admitted for every query
                for (; t < cb3 && adopting; t += TPS, buf = next_buf(buf)) {
                    begin_stage(buf);
#pragma unroll 1
                    for (int j = 0; j < imin(TPS, cb3 - t); ++j) {
                        const TileInfo si = tile_info(t + j, buf, j);
                        if (wave_has_queries) fast_stage<kMaskNone, true, CODE>(ws, qf, lo, si.tile_lds, si.ma);
                    }
                    adopting = wave_has_queries && still_adopting();
                }
                for (; t < cb3; t += TPS, buf = next_buf(buf)) {
                    begin_stage(buf);
#pragma unroll 1
                    for (int j = 0; j < imin(TPS, cb3 - t); ++j) {
                        const TileInfo si = tile_info(t + j, buf, j);
                        if (wave_has_queries) fast_stage<kMaskNone, false, CODE>(ws, qf, lo, si.tile_lds, si.ma);
                    }
                }
            }
            if (!TEXTQ) {
                // image tiles inside the grid (lane masks from the table); the strided variant has run them above
                if constexpr (CODE != kCodeFull) {
                for (; t < cb3 && adopting; t += TPS, buf = next_buf(buf)) {
                    const TableStage ts = table_stage(t);
                    begin_stage(buf);
#pragma unroll
                    for (int j = 0; j < TPS; ++j)
                        if (ts.d[j] != kWaveSkipsTile) fast_stage<kMaskTable, true, CODE>(ws, qf, lo, stage_tile_lds(buf, j), table_mask_args(ts.d[j]));
                    adopting = wave_has_queries && still_adopting();
                }
                for (; t < cb3; t += TPS, buf = next_buf(buf)) {
                    const TableStage ts = table_stage(t);
                    begin_stage(buf);
#pragma unroll
                    for (int j = 0; j < TPS; ++j)
                        if (ts.d[j] != kWaveSkipsTile) fast_stage<kMaskTable, false, CODE>(ws, qf, lo, stage_tile_lds(buf, j), table_mask_args(ts.d[j]));
                }
                }
                t = cb3;
                // image tiles cut by the border: few, keep them simple
                for (; t < cb4; t += TPS, buf = next_buf(buf)) {
                    begin_stage(buf);
#pragma unroll 1
                    for (int j = 0; j < imin(TPS, cb4 - t); ++j) {
                        const TileInfo si = tile_info(t + j, buf, j);
                        if (si.cls0 != kBlockSkip || si.cls1 != kBlockSkip) fast_stage<kMaskImage, true, CODE>(ws, qf, lo, si.tile_lds, si.ma);
                    }
                }
            }
            // the fast pass stands only if every sum stayed finite and moderate
            float chk = ws.l_run;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) chk += __builtin_fabsf(ws.oacc[db][r]);
            bad = __builtin_amdgcn_ballot_w64(!(chk < FAST_SUM_LIMIT));
        }
        wait_vmcnt<0>();  // loads into slots that nothing reads must not outlive the pass (or the workgroup's LDS)
        return bad;
    };

    // Fast pass first.  If any query of the workgroup met a score more than 2^FAST_HEADROOM_LOG2 above
    // its reference (in the exponent), the whole workgroup repeats the tile walk with the careful pass.
    if (tid == 0) s_redo = 0;  // ordered before any write below by the barriers of the stage loop
    const unsigned long long bad = run_pass(std::false_type{});
    if (bad != 0 && lane == 0) s_redo = 1;
    __syncthreads();
    if (s_redo != 0) {
        __syncthreads();  // every wave has read the flag and left the ring buffers
        run_pass(std::true_type{});
        __syncthreads();  // the epilogue reuses the stage buffers
    }

    const float m_run = ws.m_run;
    const float l_run = ws.l_run;
    f32x16(&oacc)[NDB] = ws.oacc;
    // ---- epilogue
    const float l_tot = wave_pair_sum(l_run);
    if (TEXTQ) {
        if (q_valid) {
            const long long row = ((long long)bh * p.n_splits + split) * p.n_text + q_token;
            float* wo = p.ws_o + row * D;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 v = {oacc[db][4 * g], oacc[db][4 * g + 1], oacc[db][4 * g + 2], oacc[db][4 * g + 3]};
                    *(f32x4*)(wo + 32 * db + 8 * g + 4 * hh) = v;
                }
            if (hh == 0) {
                p.ws_ml[row * 2] = m_run;
                p.ws_ml[row * 2 + 1] = l_tot;
            }
        }
    } else {
        // The wave's 32 x D output tile is turned round in LDS (the stage buffers are idle by now: every wave
        // has passed the barrier above) so that it leaves as whole rows: a lane owns a query, and
        // storing from that layout would scatter 8-byte pieces over 32 rows per instruction.
        if (p.lse && q_valid && hh == 0) p.lse[(long long)bh * p.N + q_token] = __logf(l_tot) + m_run * p.scale_log2e * 0.6931471805599453f;
        constexpr int OROW = ROW_BYTES + 16;  // padded row pitch in LDS
        unsigned char* const wbase = smem + wave * (32 * OROW);
        const float inv = 1.0f / l_tot;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 v;
#pragma unroll
                for (int t = 0; t < 4; ++t) v[t] = (__bf16)(oacc[db][4 * g + t] * inv);
                *(bf16x4*)(wbase + qi * OROW + (32 * db + 8 * g + 4 * hh) * 2) = v;
            }
        // CHUNKS lanes per row, ROWS_PER_LOAD rows per store instruction
#pragma unroll
        for (int i = 0; i < 32 / ROWS_PER_LOAD; ++i) {
            const int row = ROWS_PER_LOAD * i + lane / CHUNKS;  // query slot of the patch
            const int oy = wy0 + (row >> 3), ox = wx0 + (row & 7);
            const f32x4 chunk = *(const f32x4*)(wbase + row * OROW + (lane % CHUNKS) * 16);
            if (oy < qH && ox < qW && oy >= p.own_y0 && oy < p.own_y1) {
                __bf16* orow = (__bf16*)p.O + batch * p.os.sb + head * p.os.sh + ((long long)p.n_text + (long long)((oy - y_shift) * stride + q_oy) * p.gridW + ox * stride + q_ox) * p.os.sn;
                __builtin_nontemporal_store(chunk, (f32x4*)(orow + (lane % CHUNKS) * 8));  // whole rows, never read again here
            }
        }
    }
}

template <int NWY, int NWX, bool TEXTQ, int CODE>
__global__ void __launch_bounds__((NWY * NWX + kLoaderWaves) * 64, (NWY * NWX <= 4 && kLoaderWaves == 0) ? 2 : 1) clear_fwd_bf16_kernel(const FwdParams p)
{
    clear_fwd_bf16_workgroup<NWY, NWX, TEXTQ, CODE>(p, (int)blockIdx.x, (int)gridDim.x);
}

// Image-query and text-query rows in one launch: workgroups [0, n_image) are the image-query ones, the rest the
// text-query ones.  For problems of a few rounds of workgroups, where the image-query launch alone leaves CUs idle
// at its end and a launch of its own for the text-query rows costs more than it computes.
template <int NWY, int NWX, int CODE>
__global__ void __launch_bounds__((NWY * NWX + kLoaderWaves) * 64, 1) clear_fwd_bf16_both_kernel(const FwdParams p, const int n_image)
{
    const int bid = (int)blockIdx.x;
    if (bid < n_image)
        clear_fwd_bf16_workgroup<NWY, NWX, false, CODE>(p, bid, n_image);
    else
        clear_fwd_bf16_workgroup<NWY, NWX, true, kCodeDisc>(p, bid - n_image, (int)gridDim.x - n_image);
}

// Combines the key-split partial results of the text-query rows: with m the largest running
// maximum, O = sum_i 2^{(m_i - m) c} O_i / sum_i 2^{(m_i - m) c} l_i.
template <typename OutT>
__global__ void __launch_bounds__(256) clear_text_merge_kernel(const FwdParams p, int d)
{
    // 256 / d text rows per workgroup, one thread per channel
    const int row = blockIdx.x * (256 / d) + threadIdx.x / d;  // bh * n_text + q
    if (row >= p.B * p.H * p.n_text) return;
    const int bh = row / p.n_text, q = row % p.n_text;
    const int ch = threadIdx.x % d;
    float m = -INFINITY;
    for (int s = 0; s < p.n_splits; ++s) {
        const long long r = ((long long)bh * p.n_splits + s) * p.n_text + q;
        m = fmaxf(m, p.ws_ml[r * 2]);
    }
    float num = 0.f, den = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {
        const long long r = ((long long)bh * p.n_splits + s) * p.n_text + q;
        const float w = __builtin_amdgcn_exp2f((p.ws_ml[r * 2] - m) * p.scale_log2e);
        den += w * p.ws_ml[r * 2 + 1];
        num += w * p.ws_o[r * d + ch];
    }
    if (p.band_o) {
        p.band_o[(long long)row * d + ch] = num / den;
        // sum_j exp(s_j / sqrt(d)) = den * 2^{m c}
        if (ch == 0) p.band_lse[row] = __logf(den) + m * p.scale_log2e * 0.6931471805599453f;
    } else {
        ((OutT*)p.O)[(bh / p.H) * p.os.sb + (bh % p.H) * p.os.sh + q * p.os.sn + ch] = (OutT)(num / den);
        if (p.lse && ch == 0) p.lse[(long long)bh * p.N + q] = __logf(den) + m * p.scale_log2e * 0.6931471805599453f;
    }
}

template <int NWY, int NWX, bool TEXTQ, int CODE>
hipError_t launch_fwd(const FwdParams& p, int nblk, hipStream_t stream)
{
    const size_t smem = (size_t)NBUF * STAGE_BYTES;
    auto kern = clear_fwd_bf16_kernel<NWY, NWX, TEXTQ, CODE>;
    static LdsLimitOnce lds_limit;  // one per kernel instantiation
    hipError_t e = lds_limit.ensure((const void*)kern, (int)smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(nblk), dim3((NWY * NWX + kLoaderWaves) * 64), smem, stream, p);
    return hipGetLastError();
}

template <int NWY, int NWX, int CODE>
hipError_t launch_fwd_both(const FwdParams& p, int n_image, int n_text_wgs, hipStream_t stream)
{
    const size_t smem = (size_t)NBUF * STAGE_BYTES;
    auto kern = clear_fwd_bf16_both_kernel<NWY, NWX, CODE>;
    static LdsLimitOnce lds_limit;  // one per kernel instantiation
    hipError_t e = lds_limit.ensure((const void*)kern, (int)smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(n_image + n_text_wgs), dim3((NWY * NWX + kLoaderWaves) * 64), smem, stream, p, n_image);
    return hipGetLastError();
}

}  // namespace

#if CLEAR_HEAD_DIM == 128
int bf16_text_queries_per_block() { return kBf16NWY * kBf16NWX * kTextQueriesPerWave; }

#endif  // CLEAR_HEAD_DIM == 128

hipError_t launch_bf16(const FwdParams& p, hipStream_t stream, int phase)
{
    const int BH = p.B * p.H;
    hipError_t e = hipSuccess;
    if (phase == kPhaseImageAndTextQuery) {
        const int n_image = BH * p.n_classes * p.n_q_tiles_launch, n_text_wgs = p.n_text > 0 ? BH * p.n_tq_tiles * p.n_splits : 0;
        const int code = mask_code_of(p.mask_kind);
        return code == kCodeDisc   ? launch_fwd_both<kBf16NWY, kBf16NWX, kCodeDisc>(p, n_image, n_text_wgs, stream)
               : code == kCodeFull ? launch_fwd_both<kBf16NWY, kBf16NWX, kCodeFull>(p, n_image, n_text_wgs, stream)
                                   : launch_fwd_both<kBf16NWY, kBf16NWX, kCodeGeneric>(p, n_image, n_text_wgs, stream);
    }
    if (phase == kPhaseAll || phase == kPhaseImage) {
        const int nblk = BH * p.n_classes * p.n_q_tiles_launch;
        const int code = mask_code_of(p.mask_kind);  // one kernel per family of image masks
        e = code == kCodeDisc   ? launch_fwd<kBf16NWY, kBf16NWX, false, kCodeDisc>(p, nblk, stream)
            : code == kCodeFull ? launch_fwd<kBf16NWY, kBf16NWX, false, kCodeFull>(p, nblk, stream)
                                : launch_fwd<kBf16NWY, kBf16NWX, false, kCodeGeneric>(p, nblk, stream);
        if (e != hipSuccess) return e;
    }
    if (p.n_text > 0 && (phase == kPhaseAll || phase == kPhaseTextQuery)) {
        e = launch_fwd<kBf16NWY, kBf16NWX, true, kCodeDisc>(p, BH * p.n_tq_tiles * p.n_splits, stream);
        if (e != hipSuccess) return e;
    }
    if (p.n_text > 0 && (phase == kPhaseAll || phase == kPhaseTextMerge)) {
        constexpr int rows_per_block = 256 / D;
        hipLaunchKernelGGL(clear_text_merge_kernel<__bf16>, dim3((BH * p.n_text + rows_per_block - 1) / rows_per_block), dim3(256), 0, stream, p, D);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace clear
