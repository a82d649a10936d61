// Query/key prologue of a FLUX-style attention block as a pass of its own (Sec. 3.1: rotary position
// embedding on the two image axes; Sec. 4.3: its frequencies are the caller's, through the tables): per-head
// RMS normalisation with a learned gain, rotation of adjacent channel pairs by the token's row angle plus
// column angle, result rounded to bf16.  Text tokens are normalised but not turned.
//
// HBM-bound: every row is read once and written once.  D / 8 lanes share a token row (16 bytes each, so a
// row is one contiguous 128- or 256-byte access); the sum of squares is combined with lane shuffles.
#include <hip/hip_runtime.h>

#include "bf16_common.h"

namespace clear {
namespace {

constexpr int kRowsPerThread = 4;  // independent 16-byte loads in flight per lane

template <int HD>
__global__ void __launch_bounds__(256) qk_prologue_kernel(const __bf16* __restrict__ X, TensorStrides xs, __bf16* __restrict__ Y, TensorStrides ys,
                                                          int H, long long rows_total, long long N, int n_text, int gridW,
                                                          const float* __restrict__ gain, float eps, const float* __restrict__ rope_y,
                                                          const float* __restrict__ rope_x)
{
    constexpr int LPR = HD / 8;        // lanes per row
    constexpr int RPB = 256 / LPR;     // rows per block and sweep
    const int c0 = 8 * (threadIdx.x % LPR);
    const long long row0 = (long long)blockIdx.x * (RPB * kRowsPerThread) + threadIdx.x / LPR;
    // row = (b * H + h) * N + token  ->  element offset in a strided [B, H, N, HD] tensor
    auto offset = [&](long long row, const TensorStrides& st) {
        const long long bh = row / N, t = row % N;
        return (bh / H) * st.sb + (bh % H) * st.sh + t * st.sn;
    };
    bf16x8 in[kRowsPerThread];
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
        const long long row = row0 + (long long)i * RPB;
        in[i] = *(const bf16x8*)(X + offset(row < rows_total ? row : rows_total - 1, xs) + c0);
    }
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
        const long long row = row0 + (long long)i * RPB;
        const bool live = row < rows_total;
        const long long rr = live ? row : rows_total - 1;
        float x[8], ss = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x[j] = (float)in[i][j];
            ss += x[j] * x[j];
        }
#pragma unroll
        for (int m = 1; m < LPR; m <<= 1) ss += __shfl_xor(ss, m, 64);
        const float inv_rms = 1.0f / sqrtf(ss * (1.0f / HD) + eps);
        const long long t = rr % N;
        const bool turn = rope_y && t >= n_text;
        const long long pix = turn ? t - n_text : 0;
        const float* const ry = rope_y + (size_t)(pix / gridW) * HD + c0;
        const float* const rx = rope_x + (size_t)(pix % gridW) * HD + c0;
        prologue_chunk(x, inv_rms, gain ? gain + c0 : nullptr, turn ? ry : nullptr, turn ? rx : nullptr);
        bf16x8 out;
#pragma unroll
        for (int j = 0; j < 8; ++j) out[j] = (__bf16)x[j];
        if (live) *(bf16x8*)(Y + offset(rr, ys) + c0) = out;
    }
}

}  // namespace

hipError_t launch_qk_prologue(const void* X, const TensorStrides& xs, void* Y, const TensorStrides& ys, int B, int H, int n_text, int gridH,
                              int gridW, int head_dim, const float* gain, float eps, const float* rope_y, const float* rope_x,
                              hipStream_t stream)
{
    const long long N = (long long)n_text + (long long)gridH * gridW;
    const long long rows = (long long)B * H * N;
    if (rows == 0) return hipSuccess;
    const int rows_per_block = 256 / (head_dim / 8) * kRowsPerThread;
    const long long blocks = (rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (head_dim == 128)
        hipLaunchKernelGGL(qk_prologue_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, stream, (const __bf16*)X, xs, (__bf16*)Y, ys, H, rows, N,
                           n_text, gridW, gain, eps, rope_y, rope_x);
    else if (head_dim == 64)
        hipLaunchKernelGGL(qk_prologue_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, stream, (const __bf16*)X, xs, (__bf16*)Y, ys, H, rows, N,
                           n_text, gridW, gain, eps, rope_y, rope_x);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace clear
