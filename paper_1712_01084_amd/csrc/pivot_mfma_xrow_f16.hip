// Matrix-core layer kernel whose B fragments are gathered from a copy of x in LDS (fp16 weights, batch 5..16):
// instantiations and dispatch.
#include "pivot_fc_kernels.h"

namespace pivot {

template <int KIND, int BH, int BW>
static int launch_t(const FcArgs& a, dim3 grid, size_t smem, hipStream_t st) {
    // more than 64 KB of dynamic LDS per workgroup has to be allowed per kernel and device
    static size_t allowed[16] = {};
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    size_t& have = allowed[dev & 15];
    if (smem > 64 * 1024 && smem > have) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&fc_mfma_xrow_kernel<KIND, BH, BW>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        have = smem;
    }
    hipLaunchKernelGGL((fc_mfma_xrow_kernel<KIND, BH, BW>), grid, dim3(8 * 64), smem, st, PIVOT_GEMV_ARGS(a), a);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

int launch_mfma_xrow_f16(const FcArgs& a, int kind, int bhs, int bw, dim3 grid, size_t smem, hipStream_t st) {
#define X(BH_, BW_)                                                                                        \
    if (bhs == BH_ && bw == BW_) {                                                                         \
        if constexpr (BW_ % 32 == 0 && BH_ % 16 == 0) { if (kind == 0) return launch_t<0, BH_, BW_>(a, grid, smem, st); } \
        if constexpr (BH_ % 32 == 0 && BW_ % 16 == 0) { if (kind == 1) return launch_t<1, BH_, BW_>(a, grid, smem, st); } \
        if constexpr (BH_ == 16 && BW_ == 16)          { if (kind == 2) return launch_t<2, BH_, BW_>(a, grid, smem, st); } \
    }
    PIVOT_SHAPES(X)
#undef X
    set_error("no matrix-core kernel (kind %d) for %dx%d row slices", kind, bhs, bw);
    return PIVOT_E_UNSUPPORTED;
}

}  // namespace pivot
