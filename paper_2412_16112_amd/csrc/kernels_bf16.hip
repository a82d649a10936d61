// bf16 MFMA kernels for the CLEAR local-attention forward pass on gfx950 (head_dim 128).
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
// K and V tiles are staged in LDS once per workgroup; every wave classifies each 32-key block
// against its own 4 x 8 query patch and skips the blocks its disc cannot reach.
#include <hip/hip_runtime.h>

#include "block_class.h"
#include "clear_internal.h"

namespace clear {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int D = 128;               // head_dim
constexpr int ROW_BYTES = D * 2;     // one token row of K or V
constexpr int TILE_KEYS = kKeyTileKeys;
constexpr int TILE_BYTES = TILE_KEYS * ROW_BYTES;  // 16 KB for K, same for V
constexpr int NSTAGE = 4;                          // ring of staged key tiles (K + V = 32 KB each)
constexpr float LAZY_RESCALE_LOG2 = 8.0f;  // re-base the running maximum only when it rises by more than 2^8
constexpr float M_INIT = -1.0e30f;         // finite "no key seen yet" (keeps exp2 arguments free of inf - inf)

// LDS layout of a staged tile: 64 rows of 256 B, unpadded (the LDS-direct load writes 1 KB = 4 rows per
// wave instruction), with the 16-byte chunks of each row permuted: logical chunk c of row k sits in
// slot c ^ swz(k).  swz is a bijection on 16 consecutive rows (the 32 key rows of a K read spread over
// all banks) and sends 4 consecutive rows to 4 different 64-byte quads (so does the transposed V read).
__host__ __device__ constexpr int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

__device__ __forceinline__ float wave_pair_max(float x)
{
    // lanes l and l ^ 32 hold the two halves of one query's scores
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float wave_pair_sum(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One 16-byte-per-lane load from global memory straight into LDS: the wave writes 1 KB starting at
// lds_addr (wave-uniform), lane i at lds_addr + 16 i; lane i reads gbase + voff.  Counted by vmcnt.
// Written as asm so that the compiler does not serialise later LDS reads behind it; the kernel waits
// with explicit s_waitcnt vmcnt before the barrier that publishes the tile.
__device__ __forceinline__ void load_to_lds_16B(const void* gbase, unsigned voff, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(gbase) : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));  // expcnt, lgkmcnt unconstrained
}

template <int NWY, int NWX, bool TEXTQ>
__global__ void __launch_bounds__(NWY* NWX * 64, 1) clear_fwd_bf16_kernel(const FwdParams p)
{
    constexpr int NW = NWY * NWX;
    constexpr int NI = 16 / NW;       // 1 KB load instructions per wave per tile, for K and for V each
    constexpr int LPT = 2 * NI;       // loads per thread per stage
    static_assert(NI * NW == 16, "64 rows = 16 instructions of 4 rows");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];  // [NSTAGE][K tile | V tile]
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qi = lane & 31;   // query slot inside the wave's patch
    const int hh = lane >> 5;   // which half of the contraction slice this lane feeds

    // ---- workgroup -> (batch*head, query tile[, key split]); XCD-aware: workgroups are dealt
    // round-robin to the 8 XCDs, so give each XCD one contiguous range of the logical index.
    int vid;
    {
        const int nblk = gridDim.x, bid = blockIdx.x;
        const int xcd = bid & 7, idx = bid >> 3;
        const int q = nblk >> 3, rem = nblk & 7;
        vid = xcd * q + imin(xcd, rem) + idx;
    }
    int bh, qt, split = 0;
    if (TEXTQ) {
        split = vid % p.n_splits;
        const int t = vid / p.n_splits;
        qt = t % p.n_tq_tiles;
        bh = t / p.n_tq_tiles;
    } else {
        qt = vid % p.n_q_tiles;
        bh = vid / p.n_q_tiles;
    }
    const long long head_off = (long long)bh * p.N * D;  // elements
    const __bf16* const Qh = (const __bf16*)p.Q + head_off;
    const unsigned char* const Kh = (const unsigned char*)((const __bf16*)p.K + head_off);
    const unsigned char* const Vh = (const unsigned char*)((const __bf16*)p.V + head_off);

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
        q_valid = qy < p.gridH && qx < p.gridW;
        wave_has_queries = wy0 < p.gridH && wx0 < p.gridW;
        q_token = p.n_text + imin(qy, p.gridH - 1) * p.gridW + imin(qx, p.gridW - 1);
    }

    // Q^T as MFMA B operand: 8 contraction steps of 16 channels; this lane supplies channels 16*s + 8*hh .. +7
    bf16x8 qf[8];
    {
        const __bf16* qrow = Qh + (long long)q_token * D + 8 * hh;
#pragma unroll
        for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8*)(qrow + 16 * s);
        // pin the fragments in registers now: otherwise the wait for these loads lands inside the key loop,
        // where it would also drain the tile prefetches
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(qf[s]));
    }

    // ---- stage list: tokens [lin_begin, lin_limit) in 64-key tiles, then (image mode) the CSR row
    int n_stages, n_lin_stages, csr_begin = 0;
    int lin_begin = 0, lin_limit = 0;
    if (TEXTQ) {
        lin_begin = split * p.split_keys;
        lin_limit = (long long)lin_begin + p.split_keys < p.N ? lin_begin + p.split_keys : (int)p.N;
        n_lin_stages = (lin_limit - lin_begin + TILE_KEYS - 1) / TILE_KEYS;
        n_stages = n_lin_stages;
    } else {
        lin_limit = p.n_text;
        n_lin_stages = (p.n_text + TILE_KEYS - 1) / TILE_KEYS;
        csr_begin = p.row_ptr[qt];
        n_stages = n_lin_stages + (p.row_ptr[qt + 1] - csr_begin);
    }

    // Tile origin of stage i: linear -> (first token, -1); image -> (row, col) of the 8 x 8 tile.
    auto stage_origin = [&](int i, int& a, int& b) {
        if (i < n_lin_stages) {
            a = lin_begin + i * TILE_KEYS;
            b = -1;
        } else {
            const int id = p.col_idx[csr_begin + i - n_lin_stages];
            a = (id / p.n_ktx) * kKeyTileH;
            b = (id % p.n_ktx) * kKeyTileW;
        }
    };

    // ---- LDS-direct staging.  Load instruction ii (0..15) of a tile covers rows 4 ii .. 4 ii + 3; lane i
    // writes slot i % 16 of row 4 ii + i / 16 and therefore fetches logical chunk (i % 16) ^ swz(row).
    // Addresses are clamped to valid tokens; slots beyond the range or the grid are masked in the compute.
    auto issue_stage = [&](int i) {
        int a, b;
        stage_origin(i, a, b);
        const unsigned buf = lds_base + (unsigned)(i % NSTAGE) * (2 * TILE_BYTES);
#pragma unroll
        for (int n = 0; n < NI; ++n) {
            const int ii = wave * NI + n;
            const int row = 4 * ii + (lane >> 4);
            int token;
            if (b < 0) {
                token = imin(a + row, lin_limit - 1);
            } else {
                const int ky = imin(a + (row >> 3), p.gridH - 1);
                const int kx = imin(b + (row & 7), p.gridW - 1);
                token = p.n_text + ky * p.gridW + kx;
            }
            const unsigned voff = (unsigned)token * ROW_BYTES + (unsigned)(((lane & 15) ^ swz(row)) << 4);
            load_to_lds_16B(Kh, voff, buf + ii * 1024);
            load_to_lds_16B(Vh, voff, buf + TILE_BYTES + ii * 1024);
        }
    };

    // ---- running softmax state: one query per lane (shared with lane ^ 32)
    f32x16 oacc[4];  // O^T tiles: channel 32*db + 8*(reg/4) + 4*hh + reg%4 of this lane's query
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_run = M_INIT;  // running maximum, raw logits (may lag the true maximum by < 2^8 in the exponent)
    float l_run = 0.f;     // this lane's share of the denominator
    const float c = p.scale_log2e;

    // ---- per-lane LDS read offsets inside a 32-key block (block and buffer offsets are added later)
    // K operand: row qi, logical chunk 2 ks + hh
    unsigned k_off[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) k_off[ks] = (unsigned)(qi * ROW_BYTES + (((2 * ks + hh) ^ swz(qi)) << 4));
    // V operand (transpose load): within each group of 16 lanes, lane j addresses key row j/4 and
    // channels 4*(j%4)..+3 of the group's 16-channel slice; it receives channel (lane % 16) for 4 rows.
    // Rows of the first load: 4 hh + j/4 (+ 16 s2); of the second: + 8.
    unsigned v_off[4][2];
    {
        const int j = lane & 15, g2 = (lane >> 4) & 1;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) {
                const int row = 4 * hh + (j >> 2) + 8 * hi;  // swz(row + 16 s2 + 32 kb) == swz(row)
                const int chunk = 4 * db + 2 * g2 + ((j & 3) >> 1);
                v_off[db][hi] = (unsigned)(row * ROW_BYTES + ((chunk ^ swz(row)) << 4) + 8 * (j & 1));
            }
    }

    // ---- prologue: NSTAGE - 1 tiles in flight
#pragma unroll
    for (int i = 0; i < NSTAGE - 1; ++i)
        if (i < n_stages) issue_stage(i);

    for (int st = 0; st < n_stages; ++st) {
        // tile st has landed once at most NSTAGE - 2 younger tiles are outstanding (all of them exist
        // only away from the tail)
        if (st + NSTAGE - 2 < n_stages)
            wait_vmcnt<(NSTAGE - 2) * LPT>();
        else
            wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();  // every wave's part of tile st is in LDS; every wave is done with tile st - 1
        asm volatile("" ::: "memory");
        if (st + NSTAGE - 1 < n_stages) issue_stage(st + NSTAGE - 1);  // overwrites the buffer of tile st - 1

        int ta, tb;
        stage_origin(st, ta, tb);
        const bool linear = tb < 0;
        int cls[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (!wave_has_queries)
                cls[kb] = kBlockSkip;
            else if (linear)
                cls[kb] = classify_linear_block(ta + 32 * kb, 32, lin_limit);
            else
                cls[kb] = TEXTQ ? kBlockSkip
                                : classify_image_block(wy0, wx0, kWaveQH, kWaveQW, ta + kKeyBlockH * kb, tb, kKeyBlockH,
                                                       kKeyBlockW, p.gridH, p.gridW, p.r2);
        }
        if (cls[0] == kBlockSkip && cls[1] == kBlockSkip) continue;

        const unsigned char* const tileK = smem + (st % NSTAGE) * (2 * TILE_BYTES);
        const unsigned char* const tileV = tileK + TILE_BYTES;

        // S^T = K_blk Q^T for the active blocks
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (cls[kb] == kBlockSkip) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = -INFINITY;
                continue;
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 a = *(const bf16x8*)(tileK + kb * 32 * ROW_BYTES + k_off[ks]);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
            }
            // element mask: register r of this lane is key slot 8*(r/4) + 4*hh + r%4 of the block
            if (cls[kb] == kBlockPartial) {
                if (linear) {
                    const int base = ta + 32 * kb + 4 * hh;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (base + 8 * (r >> 2) + (r & 3) >= lin_limit) s[kb][r] = -INFINITY;
                } else {
                    const int ky0 = ta + kKeyBlockH * kb, kx0 = tb + 4 * hh;
                    int dx2[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const int dx = kx0 + t - qx;
                        dx2[t] = (kx0 + t < p.gridW) ? dx * dx : 0x7fffffff;  // columns beyond the grid never pass
                    }
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int dy = ky0 + g - qy;
                        const int lim = (ky0 + g < p.gridH) ? p.r2 - dy * dy : 0;  // dx^2 must stay below lim
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (!(dx2[t] < lim)) s[kb][4 * g + t] = -INFINITY;
                    }
                }
            }
        }

        // online softmax (Eq. 1) over the 64 keys, lazily re-based
        float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s[0][r], s[1][r]));
        mx = wave_pair_max(mx);
        const float m_new = fmaxf(m_run, mx);
        if (__builtin_amdgcn_ballot_w64((m_new - m_run) * c > LAZY_RESCALE_LOG2) != 0) {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            m_run = m_new;
        }
        const float mc = m_run * c;

#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (cls[kb] == kBlockSkip) continue;
            bf16x8 pf[2];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r], c, -mc));
                l_run += pv;
                pf[r >> 3][r & 7] = (__bf16)pv;
            }
            // O^T += V_blk^T P^T: contraction step s2 pairs P registers 8*s2 .. 8*s2+7 with key slots
            // 16*s2 + 4*hh + {0..3} and 16*s2 + 8 + 4*hh + {0..3}
            const unsigned char* vb = tileV + kb * 32 * ROW_BYTES;
#pragma unroll
            for (int db = 0; db < 4; ++db) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (short4v __attribute__((address_space(3)))*)(vb + 16 * s2 * ROW_BYTES + v_off[db][0]));
                    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (short4v __attribute__((address_space(3)))*)(vb + 16 * s2 * ROW_BYTES + v_off[db][1]));
                    union { struct { short4v lo, hi; } h; bf16x8 v; } u;
                    u.h.lo = lo;
                    u.h.hi = hi;
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, pf[s2], oacc[db], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue
    const float l_tot = wave_pair_sum(l_run);
    if (TEXTQ) {
        if (q_valid) {
            const long long row = ((long long)bh * p.n_splits + split) * p.n_text + q_token;
            float* wo = p.ws_o + row * D;
#pragma unroll
            for (int db = 0; db < 4; ++db)
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
        if (q_valid) {
            const float inv = 1.0f / l_tot;
            __bf16* orow = (__bf16*)p.O + head_off + (long long)q_token * D;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 v;
#pragma unroll
                    for (int t = 0; t < 4; ++t) v[t] = (__bf16)(oacc[db][4 * g + t] * inv);
                    *(bf16x4*)(orow + 32 * db + 8 * g + 4 * hh) = v;
                }
        }
    }
}

// Combines the key-split partial results of the text-query rows: with m the largest running
// maximum, O = sum_i 2^{(m_i - m) c} O_i / sum_i 2^{(m_i - m) c} l_i.
template <typename OutT>
__global__ void __launch_bounds__(128) clear_text_merge_kernel(const FwdParams p, int d)
{
    const int row = blockIdx.x;  // bh * n_text + q
    const int bh = row / p.n_text, q = row % p.n_text;
    const int ch = threadIdx.x;
    if (ch >= d) return;
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
    ((OutT*)p.O)[((long long)bh * p.N + q) * d + ch] = (OutT)(num / den);
}

template <int NWY, int NWX, bool TEXTQ>
hipError_t launch_fwd(const FwdParams& p, int nblk, hipStream_t stream)
{
    const size_t smem = (size_t)NSTAGE * 2 * TILE_BYTES;
    auto kern = clear_fwd_bf16_kernel<NWY, NWX, TEXTQ>;
    static bool attr_set = false;  // the attribute is per function, set once per process
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(nblk), dim3(NWY * NWX * 64), smem, stream, p);
    return hipGetLastError();
}

}  // namespace

int bf16_text_queries_per_block() { return kBf16NWY * kBf16NWX * kTextQueriesPerWave; }

hipError_t launch_bf16_d128(const FwdParams& p, hipStream_t stream, int phase)
{
    const int BH = p.B * p.H;
    hipError_t e = hipSuccess;
    if (phase == kPhaseAll || phase == kPhaseImage) {
        e = launch_fwd<kBf16NWY, kBf16NWX, false>(p, BH * p.n_q_tiles, stream);
        if (e != hipSuccess) return e;
    }
    if (p.n_text > 0 && (phase == kPhaseAll || phase == kPhaseTextQuery)) {
        e = launch_fwd<kBf16NWY, kBf16NWX, true>(p, BH * p.n_tq_tiles * p.n_splits, stream);
        if (e != hipSuccess) return e;
    }
    if (p.n_text > 0 && (phase == kPhaseAll || phase == kPhaseTextMerge)) {
        hipLaunchKernelGGL(clear_text_merge_kernel<__bf16>, dim3(BH * p.n_text), dim3(128), 0, stream, p, D);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace clear
