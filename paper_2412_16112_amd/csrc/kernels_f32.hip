// fp32 accuracy path of the CLEAR local-attention forward pass (head_dim 64): plain vector-ALU
// arithmetic, one thread per query, exact online softmax (Eq. 1) over the keys the mask of Eq. 3
// admits.  It walks the same tile schedule as the MFMA path (text keys, then the listed 8 x 8 image
// key tiles), stages each 64-key tile in LDS, and tests every (query, key) pair against the mask.
// Text-query rows run the same loop over a contiguous key range, split along the keys and merged.
#include <hip/hip_runtime.h>

#include "block_class.h"
#include "clear_internal.h"

namespace clear {
namespace {

constexpr int D = 64;
constexpr int TILE_KEYS = kKeyTileKeys;
constexpr int NT = kF32QTileH * kF32QTileW;  // 256 threads, one query each

template <bool TEXTQ>
__global__ void __launch_bounds__(NT) clear_fwd_f32_kernel(const FwdParams p)
{
    __shared__ float4 ldsK[TILE_KEYS * D / 4];
    __shared__ float4 ldsV[TILE_KEYS * D / 4];

    const int tid = threadIdx.x;
    int bh, qt, split = 0;
    {
        const int vid = blockIdx.x;
        if (TEXTQ) {
            split = vid % p.n_splits;
            const int t = vid / p.n_splits;
            qt = t % p.n_tq_tiles;
            bh = t / p.n_tq_tiles;
        } else {
            qt = p.qt_begin + vid % p.n_q_tiles_launch;
            bh = vid / p.n_q_tiles_launch;
        }
    }
    const long long head_off = (long long)bh * p.N * D;
    const float* const Qh = (const float*)p.Q + head_off;
    const float4* const Kh = (const float4*)((const float*)p.K + head_off);
    const float4* const Vh = (const float4*)((const float*)p.V + head_off);

    int qy = 0, qx = 0;
    long long q_token;
    bool q_valid;
    if (TEXTQ) {
        q_token = (long long)qt * NT + tid;
        q_valid = q_token < p.n_text;
        if (!q_valid) q_token = p.n_text - 1;
    } else {
        qy = (qt / p.n_qtx) * kF32QTileH + tid / kF32QTileW;
        qx = (qt % p.n_qtx) * kF32QTileW + tid % kF32QTileW;
        q_valid = qy < p.gridH && qx < p.gridW && qy >= p.own_y0 && qy < p.own_y1;  // (row-band mode: owned rows only)
        q_token = (long long)p.n_text + (long long)imin(qy, p.gridH - 1) * p.gridW + imin(qx, p.gridW - 1);
    }

    float q[D], o[D];
#pragma unroll
    for (int c4 = 0; c4 < D / 4; ++c4) {
        const float4 v = *(const float4*)(Qh + q_token * D + 4 * c4);
        q[4 * c4] = v.x; q[4 * c4 + 1] = v.y; q[4 * c4 + 2] = v.z; q[4 * c4 + 3] = v.w;
    }
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float sc = p.scale_log2e;

    int n_stages, n_lin_stages, csr_begin = 0;
    long long lin_begin = 0, lin_limit = 0;
    if (TEXTQ) {
        lin_begin = (long long)split * p.split_keys;
        lin_limit = lin_begin + p.split_keys < p.NV ? lin_begin + p.split_keys : p.NV;
        n_lin_stages = (int)((lin_limit - lin_begin + TILE_KEYS - 1) / TILE_KEYS);
        n_stages = n_lin_stages;
    } else {
        lin_limit = p.n_text;
        n_lin_stages = (p.n_text + TILE_KEYS - 1) / TILE_KEYS;
        csr_begin = p.row_ptr[qt];
        n_stages = n_lin_stages + (p.row_ptr[qt + 1] - csr_begin);
    }

    for (int st = 0; st < n_stages; ++st) {
        const bool linear = st < n_lin_stages;
        long long a, b;  // linear: first token, limit; image: tile origin (row, col)
        if (linear) {
            a = lin_begin + (long long)st * TILE_KEYS;
            b = lin_limit;
        } else {
            const int packed = p.col_idx[csr_begin + st - n_lin_stages];  // tile origin, row << 16 | col
            a = packed >> 16;
            b = packed & 0xffff;
        }
        __syncthreads();  // previous tile fully consumed
        for (int ch = tid; ch < TILE_KEYS * D / 4; ch += NT) {
            const int slot = ch / (D / 4), cc = ch % (D / 4);
            long long token;
            if (linear) {
                token = a + slot;
                if (token > b - 1) token = b - 1;
                if (TEXTQ && token >= p.vkeys_text) token += p.vshift;  // position in the key list -> token
            } else {
                const int ky = imin((int)a + slot / kKeyTileW, p.gridH - 1);
                const int kx = imin((int)b + slot % kKeyTileW, p.gridW - 1);
                token = (long long)p.n_text + (long long)ky * p.gridW + kx;
            }
            ldsK[ch] = Kh[token * (D / 4) + cc];
            ldsV[ch] = Vh[token * (D / 4) + cc];
        }
        __syncthreads();

        for (int slot = 0; slot < TILE_KEYS; ++slot) {
            bool ok;
            if (linear) {
                ok = a + slot < b;
            } else {
                const int ky = (int)a + slot / kKeyTileW, kx = (int)b + slot % kKeyTileW;
                const int dy = ky - qy, dx = kx - qx;
                const MaskSpec spec = {p.mask_kind, p.mask_r, p.mask_shift};
                ok = !TEXTQ && ky < p.gridH && kx < p.gridW && (p.mask_kind == kMaskDisc ? dx * dx + dy * dy < p.r2 : mask_admits(spec, qy, qx, ky, kx));
            }
            if (!ok) continue;
            float s = 0.f;
#pragma unroll
            for (int c4 = 0; c4 < D / 4; ++c4) {
                const float4 kv = ldsK[slot * (D / 4) + c4];  // same address in every lane: LDS broadcast
                s = __builtin_fmaf(q[4 * c4], kv.x, s);
                s = __builtin_fmaf(q[4 * c4 + 1], kv.y, s);
                s = __builtin_fmaf(q[4 * c4 + 2], kv.z, s);
                s = __builtin_fmaf(q[4 * c4 + 3], kv.w, s);
            }
            if (s > m) {  // re-base on the new maximum
                const float alpha = exp2f((m - s) * sc);
                l *= alpha;
#pragma unroll
                for (int c = 0; c < D; ++c) o[c] *= alpha;
                m = s;
            }
            const float pr = exp2f((s - m) * sc);
            l += pr;
#pragma unroll
            for (int c4 = 0; c4 < D / 4; ++c4) {
                const float4 vv = ldsV[slot * (D / 4) + c4];
                o[4 * c4] = __builtin_fmaf(pr, vv.x, o[4 * c4]);
                o[4 * c4 + 1] = __builtin_fmaf(pr, vv.y, o[4 * c4 + 1]);
                o[4 * c4 + 2] = __builtin_fmaf(pr, vv.z, o[4 * c4 + 2]);
                o[4 * c4 + 3] = __builtin_fmaf(pr, vv.w, o[4 * c4 + 3]);
            }
        }
    }

    if (!q_valid) return;
    if (TEXTQ) {
        const long long row = ((long long)bh * p.n_splits + split) * p.n_text + q_token;
        float* wo = p.ws_o + row * D;
#pragma unroll
        for (int c4 = 0; c4 < D / 4; ++c4) *(float4*)(wo + 4 * c4) = make_float4(o[4 * c4], o[4 * c4 + 1], o[4 * c4 + 2], o[4 * c4 + 3]);
        p.ws_ml[row * 2] = m;
        p.ws_ml[row * 2 + 1] = l;
    } else {
        const float inv = 1.0f / l;
        if (p.lse) p.lse[(long long)bh * p.N + q_token] = logf(l) + m * p.scale_log2e * 0.6931471805599453f;
        float* orow = (float*)p.O + head_off + q_token * D;
#pragma unroll
        for (int c4 = 0; c4 < D / 4; ++c4)
            *(float4*)(orow + 4 * c4) = make_float4(o[4 * c4] * inv, o[4 * c4 + 1] * inv, o[4 * c4 + 2] * inv, o[4 * c4 + 3] * inv);
    }
}

// Log-sum-exp combination of the key-split partial results of the text-query rows.
__global__ void __launch_bounds__(D) clear_text_merge_f32_kernel(const FwdParams p)
{
    const int row = blockIdx.x;
    const int bh = row / p.n_text, q = row % p.n_text;
    const int ch = threadIdx.x;
    float m = -INFINITY;
    for (int s = 0; s < p.n_splits; ++s) m = fmaxf(m, p.ws_ml[(((long long)bh * p.n_splits + s) * p.n_text + q) * 2]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {
        const long long r = ((long long)bh * p.n_splits + s) * p.n_text + q;
        const float w = exp2f((p.ws_ml[r * 2] - m) * p.scale_log2e);
        den += w * p.ws_ml[r * 2 + 1];
        num += w * p.ws_o[r * D + ch];
    }
    if (p.band_o) {
        p.band_o[(long long)row * D + ch] = num / den;
        if (ch == 0) p.band_lse[row] = logf(den) + m * p.scale_log2e * 0.6931471805599453f;
    } else {
        ((float*)p.O)[((long long)bh * p.N + q) * D + ch] = num / den;
        if (p.lse && ch == 0) p.lse[(long long)bh * p.N + q] = logf(den) + m * p.scale_log2e * 0.6931471805599453f;
    }
}

}  // namespace

int f32_text_queries_per_block() { return NT; }

hipError_t launch_f32_d64(const FwdParams& p, hipStream_t stream, int phase)
{
    const int BH = p.B * p.H;
    hipError_t e = hipSuccess;
    if (phase == kPhaseAll || phase == kPhaseImage) {
        hipLaunchKernelGGL(clear_fwd_f32_kernel<false>, dim3(BH * p.n_q_tiles_launch), dim3(NT), 0, stream, p);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (p.n_text > 0 && (phase == kPhaseAll || phase == kPhaseTextQuery)) {
        hipLaunchKernelGGL(clear_fwd_f32_kernel<true>, dim3(BH * p.n_tq_tiles * p.n_splits), dim3(NT), 0, stream, p);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (p.n_text > 0 && (phase == kPhaseAll || phase == kPhaseTextMerge)) {
        hipLaunchKernelGGL(clear_text_merge_f32_kernel, dim3(BH * p.n_text), dim3(D), 0, stream, p);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace clear
