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
constexpr int KS = ROW_BYTES + 16;   // LDS row stride of K tiles (bytes): 16-byte pad spreads the 32 key rows of a b128 read over all banks
constexpr int VS = ROW_BYTES + 64;   // LDS row stride of V tiles (bytes): 4 consecutive key rows x 64 B cover all 64 banks
constexpr int TILE_KEYS = kKeyTileKeys;
constexpr float LAZY_RESCALE_LOG2 = 8.0f;  // re-base the running maximum only when it rises by more than 2^8
constexpr float M_INIT = -1.0e30f;         // finite "no key seen yet" (keeps exp2 arguments free of inf - inf)

struct StageDesc {
    int linear;       // 1: keys are tokens [a, a + 64) clipped to limit b; 0: image tile with origin (a, b)
    long long a, b;
};

__device__ __forceinline__ float wave_pair_max(float x)
{
    // lanes l and l ^ 32 hold the two halves of one query's scores
#if __has_builtin(__builtin_amdgcn_permlane32_swap)
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
#else
    return fmaxf(x, __shfl_xor(x, 32));
#endif
}

__device__ __forceinline__ float wave_pair_sum(float x)
{
#if __has_builtin(__builtin_amdgcn_permlane32_swap)
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
#else
    return x + __shfl_xor(x, 32);
#endif
}

template <int NWY, int NWX, bool TEXTQ>
__global__ void __launch_bounds__(NWY* NWX * 64, 1) clear_fwd_bf16_kernel(const FwdParams p)
{
    constexpr int NW = NWY * NWX;
    constexpr int NT = NW * 64;
    constexpr int NCH = (TILE_KEYS * 16) / NT;  // 16-byte chunks of K (and of V) per thread per stage
    static_assert(NCH * NT == TILE_KEYS * 16, "tile must split evenly over the threads");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* const ldsK = smem;                          // [2][64][KS]
    unsigned char* const ldsV = smem + 2 * TILE_KEYS * KS;     // [2][64][VS]

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
    long long q_token;
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
        q_token = (long long)p.n_text + (long long)imin(qy, p.gridH - 1) * p.gridW + imin(qx, p.gridW - 1);
    }

    // Q^T as MFMA B operand: 8 contraction steps of 16 channels; this lane supplies channels 16*s + 8*hh .. +7
    bf16x8 qf[8];
    {
        const __bf16* qrow = Qh + q_token * D + 8 * hh;
#pragma unroll
        for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8*)(qrow + 16 * s);
    }

    // ---- stage list
    int n_stages, n_lin_stages, csr_begin = 0;
    long long lin_begin = 0, lin_limit = 0;
    if (TEXTQ) {
        lin_begin = (long long)split * p.split_keys;
        lin_limit = lin_begin + p.split_keys < p.N ? lin_begin + p.split_keys : p.N;
        n_lin_stages = (int)((lin_limit - lin_begin + TILE_KEYS - 1) / TILE_KEYS);
        n_stages = n_lin_stages;
    } else {
        lin_limit = p.n_text;
        n_lin_stages = (p.n_text + TILE_KEYS - 1) / TILE_KEYS;
        csr_begin = p.row_ptr[qt];
        n_stages = n_lin_stages + (p.row_ptr[qt + 1] - csr_begin);
    }

    auto stage_desc = [&](int i) -> StageDesc {
        StageDesc sd;
        if (i < n_lin_stages) {
            sd.linear = 1;
            sd.a = lin_begin + (long long)i * TILE_KEYS;
            sd.b = lin_limit;
        } else {
            const int id = p.col_idx[csr_begin + i - n_lin_stages];
            sd.linear = 0;
            sd.a = (id / p.n_ktx) * kKeyTileH;
            sd.b = (id % p.n_ktx) * kKeyTileW;
        }
        return sd;
    };

    // global -> register staging of one 64-key tile (addresses clamped to valid tokens; slots beyond
    // the range or the grid are masked in the compute)
    uint4 kreg[NCH], vreg[NCH];
    auto load_stage = [&](const StageDesc& sd) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = tid + i * NT;
            const int slot = c >> 4, cc = c & 15;
            long long token;
            if (sd.linear) {
                token = sd.a + slot;
                if (token > sd.b - 1) token = sd.b - 1;
            } else {
                const int ky = imin((int)sd.a + (slot >> 3), p.gridH - 1);
                const int kx = imin((int)sd.b + (slot & 7), p.gridW - 1);
                token = (long long)p.n_text + (long long)ky * p.gridW + kx;
            }
            const long long off = token * ROW_BYTES + cc * 16;
            kreg[i] = *(const uint4*)(Kh + off);
            vreg[i] = *(const uint4*)(Vh + off);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = tid + i * NT;
            const int slot = c >> 4, cc = c & 15;
            *(uint4*)(ldsK + buf * (TILE_KEYS * KS) + slot * KS + cc * 16) = kreg[i];
            *(uint4*)(ldsV + buf * (TILE_KEYS * VS) + slot * VS + cc * 16) = vreg[i];
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

    // LDS read offsets that do not depend on the stage
    const int k_read_off = qi * KS + 16 * hh;  // + 32*kb*KS + 32*s
    // transpose load: within each group of 16 lanes, lane j addresses key row j/4 and channels 4*(j%4)..+3;
    // it receives channel (lane % 16) of the group's 16-channel slice for the 4 key rows
    const int j16 = lane & 15;
    const int v_read_off = (4 * hh + (j16 >> 2)) * VS + 2 * (16 * ((lane >> 4) & 1) + 4 * (j16 & 3));

    StageDesc cur = stage_desc(0);
    if (n_stages > 0) {
        load_stage(cur);
        store_stage(0);
    }
    __syncthreads();

    for (int st = 0; st < n_stages; ++st) {
        const int buf = st & 1;
        StageDesc nxt = cur;
        if (st + 1 < n_stages) {
            nxt = stage_desc(st + 1);
            load_stage(nxt);
        }

        if (wave_has_queries) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                int cls;
                if (cur.linear)
                    cls = classify_linear_block(cur.a + 32 * kb, 32, cur.b);
                else
                    cls = TEXTQ ? kBlockSkip
                                : classify_image_block(wy0, wx0, kWaveQH, kWaveQW, (int)cur.a + kKeyBlockH * kb, (int)cur.b,
                                                       kKeyBlockH, kKeyBlockW, p.gridH, p.gridW, p.r2);
                if (cls == kBlockSkip) continue;

                // S^T = K_blk Q^T
                f32x16 s;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = 0.f;
                const unsigned char* kb_ptr = ldsK + buf * (TILE_KEYS * KS) + kb * 32 * KS + k_read_off;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 a = *(const bf16x8*)(kb_ptr + 32 * ks);
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s, 0, 0, 0);
                }

                // element mask: register r of this lane is key slot 8*(r/4) + 4*hh + r%4 of the block
                if (cls == kBlockPartial) {
                    if (cur.linear) {
                        const long long base = cur.a + 32 * kb + 4 * hh;
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (base + 8 * (r >> 2) + (r & 3) >= cur.b) s[r] = -INFINITY;
                    } else {
                        const int ky0 = (int)cur.a + kKeyBlockH * kb, kx0 = (int)cur.b + 4 * hh;
                        int dx2[4];
                        bool xin[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const int dx = kx0 + t - qx;
                            dx2[t] = dx * dx;
                            xin[t] = kx0 + t < p.gridW;
                        }
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int dy = ky0 + g - qy;
                            const int lim = (ky0 + g < p.gridH) ? p.r2 - dy * dy : 0;  // dx^2 must stay below lim
#pragma unroll
                            for (int t = 0; t < 4; ++t)
                                if (!(xin[t] && dx2[t] < lim)) s[4 * g + t] = -INFINITY;
                        }
                    }
                }

                // online softmax (Eq. 1), lazily re-based
                float mx = fmaxf(s[0], s[1]);
#pragma unroll
                for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s[r]);
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
                bf16x8 pf[2];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -mc));
                    l_run += pv;
                    pf[r >> 3][r & 7] = (__bf16)pv;
                }

                // O^T += V_blk^T P^T: contraction step s2 pairs P registers 8*s2 .. 8*s2+7 with key slots
                // 16*s2 + 4*hh + {0..3} and 16*s2 + 8 + 4*hh + {0..3}
                const unsigned char* vb_ptr = ldsV + buf * (TILE_KEYS * VS) + kb * 32 * VS + v_read_off;
#pragma unroll
                for (int db = 0; db < 4; ++db) {
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        const unsigned char* a0 = vb_ptr + (16 * s2) * VS + db * 64;
                        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(a0));
                        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(a0 + 8 * VS));
                        union { struct { short4v lo, hi; } h; bf16x8 v; } u;
                        u.h.lo = lo;
                        u.h.hi = hi;
                        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, pf[s2], oacc[db], 0, 0, 0);
                    }
                }
            }
        }

        if (st + 1 < n_stages) store_stage(buf ^ 1);
        __syncthreads();
        cur = nxt;
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
            __bf16* orow = (__bf16*)p.O + head_off + q_token * D;
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
    const size_t smem = 2 * TILE_KEYS * (KS + VS);
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
