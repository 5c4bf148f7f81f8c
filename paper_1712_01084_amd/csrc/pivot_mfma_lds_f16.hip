// Matrix-core layer kernels fed from LDS (fp16 weights, batch 3..16): instantiations and dispatch.
#include "pivot_fc_kernels.h"

namespace pivot {

template <int KIND, int BH, int BW, int NBS, int XR>
static int launch_w(const FcArgs& a, int nw, dim3 grid, size_t smem, hipStream_t st) {
    if (nw >= 8) hipLaunchKernelGGL((fc_mfma_lds_kernel<KIND, BH, BW, NBS, 8, XR>), grid, dim3(8 * 64), smem, st, PIVOT_GEMV_ARGS(a), a);
    else         hipLaunchKernelGGL((fc_mfma_lds_kernel<KIND, BH, BW, NBS, 4, XR>), grid, dim3(4 * 64), smem, st, PIVOT_GEMV_ARGS(a), a);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

template <int KIND, int BH, int BW>
static int launch_t(const FcArgs& a, int nbs, int nw, int xres, dim3 grid, size_t smem, hipStream_t st) {
    switch (nbs) {
        case 4:  return xres ? launch_w<KIND, BH, BW, 4, 2>(a, nw, grid, smem, st) : launch_w<KIND, BH, BW, 4, 0>(a, nw, grid, smem, st);
        case 8:  return xres ? launch_w<KIND, BH, BW, 8, 2>(a, nw, grid, smem, st) : launch_w<KIND, BH, BW, 8, 0>(a, nw, grid, smem, st);
        default: set_error("internal: %d staged batch rows", nbs); return PIVOT_E_UNSUPPORTED;
    }
}

// nw: 4 or 8 wavefronts per workgroup (plans that ask for 16 run with 8 here).
int launch_mfma_lds_f16(const FcArgs& a, int kind, int bhs, int bw, int nbs, int nw, int xres, dim3 grid, size_t smem, hipStream_t st) {
#define X(BH_, BW_)                                                                                        \
    if (bhs == BH_ && bw == BW_) {                                                                         \
        if constexpr (BW_ % 32 == 0 && BH_ % 16 == 0) { if (kind == 0) return launch_t<0, BH_, BW_>(a, nbs, nw, xres, grid, smem, st); } \
        if constexpr (BH_ % 32 == 0 && BW_ % 16 == 0) { if (kind == 1) return launch_t<1, BH_, BW_>(a, nbs, nw, xres, grid, smem, st); } \
        if constexpr (BH_ == 16 && BW_ == 16)          { if (kind == 2) return launch_t<2, BH_, BW_>(a, nbs, nw, xres, grid, smem, st); } \
    }
    PIVOT_SHAPES(X)
#undef X
    set_error("no matrix-core kernel (kind %d) for %dx%d row slices", kind, bhs, bw);
    return PIVOT_E_UNSUPPORTED;
}

}  // namespace pivot
