// Stand-ins for the kernel launchers, so that the host side of the library (argument checks, schedule builder,
// band layout) links without any kernel and can run under the host sanitizers on a machine
// without a GPU.  None of them is reached by the driver: every call it makes fails or finishes before a launch.
#include <algorithm>

#include "../../paper_2412_16112_amd/csrc/block_class.h"
#include "../../paper_2412_16112_amd/csrc/clear_internal.h"

namespace clear {
hipError_t launch_bf16_d128(const FwdParams&, hipStream_t, int) { return hipErrorNotSupported; }
hipError_t launch_bf16_d64(const FwdParams&, hipStream_t, int) { return hipErrorNotSupported; }
hipError_t launch_f32_d64(const FwdParams&, hipStream_t, int) { return hipErrorNotSupported; }
hipError_t launch_bf16_d128_backward(const BwdParams&, const void*, float*, hipStream_t, int) { return hipErrorNotSupported; }
hipError_t launch_bf16_d64_backward(const BwdParams&, const void*, float*, hipStream_t, int) { return hipErrorNotSupported; }
hipError_t launch_merge_text(const MergeParts&, int, int, long long, int, int, void*, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t measure_mfma_peak(int, double, double*, double*) { return hipErrorNotSupported; }
hipError_t launch_qk_prologue(const void*, const TensorStrides&, void*, const TensorStrides&, int, int, int, int, int, int, const float*, float,
                              const float*, const float*, hipStream_t)
{
    return hipErrorNotSupported;
}
int bf16_text_queries_per_block() { return kBf16NWY * kBf16NWX * kTextQueriesPerWave; }
int f32_text_queries_per_block() { return kF32QTileH * kF32QTileW; }
}  // namespace clear
