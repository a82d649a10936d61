// Row-band ("patch-parallel") inference, Sec. 3.4: combines the text-query outputs that each band computed
// over its own keys.  One workgroup per text row, one thread per channel.
//   exact:   O = sum_p w_p O_p,  w_p = exp(lse_p) / sum_p exp(lse_p)   (softmax over the union of disjoint key sets)
//   average: O = (1/n) sum_p O_p                                         (Eq. 7)
#include "../../include/clear_attn.h"

#include <hip/hip_runtime.h>

#include "clear_internal.h"

namespace clear {
namespace {

template <typename OutT>
__global__ void __launch_bounds__(1024) merge_text_kernel(const MergeParts parts, int n_text, long long N, int d, int mode, OutT* O)
{
    const int row = blockIdx.x;  // bh * n_text + q
    const int ch = threadIdx.x;
    if (ch >= d) return;
    float acc = 0.f;
    if (mode == CLEAR_MERGE_AVERAGE) {
        for (int i = 0; i < parts.n; ++i) acc += parts.o[i][(long long)row * d + ch];
        acc /= (float)parts.n;
    } else {
        float mx = -INFINITY;
        for (int i = 0; i < parts.n; ++i) mx = fmaxf(mx, parts.lse[i][row]);
        float den = 0.f;
        for (int i = 0; i < parts.n; ++i) {
            const float w = __expf(parts.lse[i][row] - mx);
            den += w;
            acc += w * parts.o[i][(long long)row * d + ch];
        }
        acc /= den;
    }
    const int bh = row / n_text, q = row % n_text;
    O[((long long)bh * N + q) * d + ch] = (OutT)acc;
}

}  // namespace

hipError_t launch_merge_text(const MergeParts& parts, int BH, int n_text, long long N, int head_dim, int mode, void* O, int dtype,
                             hipStream_t stream)
{
    const int threads = (head_dim + 63) / 64 * 64;
    if (dtype == CLEAR_BF16)
        hipLaunchKernelGGL(merge_text_kernel<__bf16>, dim3(BH * n_text), dim3(threads), 0, stream, parts, n_text, N, head_dim, mode, (__bf16*)O);
    else
        hipLaunchKernelGGL(merge_text_kernel<float>, dim3(BH * n_text), dim3(threads), 0, stream, parts, n_text, N, head_dim, mode, (float*)O);
    return hipGetLastError();
}

}  // namespace clear
