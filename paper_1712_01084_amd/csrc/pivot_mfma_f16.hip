// Matrix-core layer kernels (fp16 weights, batch >= 8): instantiations and dispatch.
#include "pivot_fc_kernels.h"

namespace pivot {

template <int KIND, int BH, int BW>
static int launch_t(const FcArgs& a, int nw, dim3 grid, size_t smem, hipStream_t st) {
    if (nw == 16)     hipLaunchKernelGGL((fc_mfma_kernel<KIND, BH, BW, 16>), grid, dim3(16 * 64), smem, st, PIVOT_LEAD_ARGS(a, a.col_idx), a);
    else if (nw == 8) hipLaunchKernelGGL((fc_mfma_kernel<KIND, BH, BW, 8>), grid, dim3(8 * 64), smem, st, PIVOT_LEAD_ARGS(a, a.col_idx), a);
    else              hipLaunchKernelGGL((fc_mfma_kernel<KIND, BH, BW, 4>), grid, dim3(4 * 64), smem, st, PIVOT_LEAD_ARGS(a, a.col_idx), a);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

int launch_mfma_f16(const FcArgs& a, int kind, int bhs, int bw, int nw, dim3 grid, size_t smem, hipStream_t st) {
#define X(BH_, BW_)                                                                                        \
    if (bhs == BH_ && bw == BW_) {                                                                         \
        if constexpr (BW_ % 32 == 0 && BH_ % 16 == 0) { if (kind == 0) return launch_t<0, BH_, BW_>(a, nw, grid, smem, st); } \
        if constexpr (BH_ % 32 == 0 && BW_ % 16 == 0) { if (kind == 1) return launch_t<1, BH_, BW_>(a, nw, grid, smem, st); } \
    }
    PIVOT_SHAPES(X)
#undef X
    set_error("no matrix-core kernel (kind %d) for %dx%d row slices", kind, bhs, bw);
    return PIVOT_E_UNSUPPORTED;
}

}  // namespace pivot
