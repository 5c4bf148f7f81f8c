// Vector-ALU layer kernels, fp16 weights: instantiations and dispatch.
#include "pivot_fc_kernels.h"

namespace pivot {

template <int BH, int BW, int NB, int XR>
static int launch_t(const FcArgs& a, int nw, dim3 grid, size_t smem, hipStream_t st) {
    if constexpr (XR == 3) {
        // more than 64 KB of dynamic LDS per workgroup has to be allowed per kernel and device
        static size_t allowed[16] = {};
        int dev = 0;
        HIP_TRY(hipGetDevice(&dev));
        size_t& have = allowed[dev & 15];
        if (smem > 64 * 1024 && smem > have) {
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&fc_gemv_kernel<_Float16, BH, BW, NB, 8, XR>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
            have = smem;
        }
        hipLaunchKernelGGL((fc_gemv_kernel<_Float16, BH, BW, NB, 8, XR>), grid, dim3(8 * 64), smem, st, PIVOT_GEMV_ARGS(a), a);
    }
    else if (nw == 16) hipLaunchKernelGGL((fc_gemv_kernel<_Float16, BH, BW, NB, 16, XR>), grid, dim3(16 * 64), smem, st, PIVOT_GEMV_ARGS(a), a);
    else if (nw == 8)  hipLaunchKernelGGL((fc_gemv_kernel<_Float16, BH, BW, NB, 8, XR>), grid, dim3(8 * 64), smem, st, PIVOT_GEMV_ARGS(a), a);
    else if (nw == 1) {
        // one wavefront per work item: batch 1, gather from global memory only (the launcher asks for nothing else)
        if constexpr (NB == 1 && XR == 0) hipLaunchKernelGGL((fc_gemv_kernel<_Float16, BH, BW, 1, 1, 0>), grid, dim3(64), smem, st, PIVOT_GEMV_ARGS(a), a);
        else { set_error("internal: one-wavefront work items at batch %d, copy form %d", NB, XR); return PIVOT_E_UNSUPPORTED; }
    }
    else               hipLaunchKernelGGL((fc_gemv_kernel<_Float16, BH, BW, NB, 4, XR>), grid, dim3(4 * 64), smem, st, PIVOT_GEMV_ARGS(a), a);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

template <int BH, int BW>
static int launch_nb(const FcArgs& a, int nb, int nw, int xres, dim3 grid, size_t smem, hipStream_t st) {
    switch (nb) {
        case 1: return xres == 3 ? launch_t<BH, BW, 1, 3>(a, nw, grid, smem, st) : xres == 2 ? launch_t<BH, BW, 1, 2>(a, nw, grid, smem, st) : (xres ? launch_t<BH, BW, 1, 1>(a, nw, grid, smem, st) : launch_t<BH, BW, 1, 0>(a, nw, grid, smem, st));
        case 2: return xres == 2 ? launch_t<BH, BW, 2, 2>(a, nw, grid, smem, st) : (xres ? launch_t<BH, BW, 2, 1>(a, nw, grid, smem, st) : launch_t<BH, BW, 2, 0>(a, nw, grid, smem, st));
        default: return xres == 2 ? launch_t<BH, BW, 4, 2>(a, nw, grid, smem, st) : (xres ? launch_t<BH, BW, 4, 1>(a, nw, grid, smem, st) : launch_t<BH, BW, 4, 0>(a, nw, grid, smem, st));
    }
}

int launch_gemv_f16(const FcArgs& a, int bhs, int bw, int nb, int nw, int xres, dim3 grid, size_t smem, hipStream_t st) {
#define X(BH_, BW_) if (bhs == BH_ && bw == BW_) return launch_nb<BH_, BW_>(a, nb, nw, xres, grid, smem, st);
    PIVOT_SHAPES(X)
#undef X
    set_error("no vector kernel for %dx%d row slices", bhs, bw);
    return PIVOT_E_UNSUPPORTED;
}

}  // namespace pivot
