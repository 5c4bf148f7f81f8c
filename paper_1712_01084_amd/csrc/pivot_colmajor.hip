// Layer kernels for the two column-major tile layouts of the paper
// (Section 4.1.1): BCR (column-major inside a tile) and CBR (one column
// position of all tiles together).  They follow the paper's own mapping more
// closely than the row-major kernel: a lane owns output rows and walks along
// the columns, so no reduction across the lanes of a row is needed; only the
// lanes that work on different columns (BCR) or different tiles (CBR) of the
// same rows are summed at the end.  Batch rows are taken one per launch row.
//
// Each lane reads 16 bytes = VEC consecutive rows of one tile column;
// RQ = BH/VEC lanes cover the rows, so a wave covers G = 64/RQ columns (BCR:
// consecutive columns of the tile stream, contiguous 1 KB) or G tiles at one
// column position (CBR: contiguous 1 KB, then a stride of T*BH to the next
// column).
#include "pivot_fc_kernels.h"

namespace pivot {

template <typename WT, int LAYOUT, int BH, int BW, int NW>
__global__ void __launch_bounds__(NW * 64) fc_colmajor_kernel(PIVOT_LEAD_PARAMS, FcArgs a) {
    using V = typename Elem<WT>::vec;
    constexpr int VEC = Elem<WT>::VEC;
    constexpr int NT  = NW * 64;
    constexpr int RQ  = BH / VEC;                       // lanes that cover the rows of one tile column
    constexpr int G   = 64 / RQ;                        // tile columns (BCR) or tiles (CBR) per wave-load
    constexpr int U   = 8;                              // wave-loads in flight per wave
    constexpr int N   = BH;
    static_assert(BH % VEC == 0 && RQ <= 64, "tile height not supported");

    extern __shared__ __align__(16) char smem[];
    __shared__ int s_flag;
    WT* xs = reinterpret_cast<WT*>(smem);
    float* red = reinterpret_cast<float*>(smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b0 = blockIdx.y;
    const Chunk ck = load_chunk(a.uniform_ct, a.uniform_parts, p_chunks, p_part_base);
    const int br = ck.br, tile_begin = ck.tile_begin, ntiles = ck.ntiles, slot = ck.slot;
    const int first = ck.first, nparts = ck.nparts;
    const int row0 = br * BH;

    XStage<WT, BW, 1, NT> xst;
    xst.load_idx(p_idx, tile_begin, ntiles * BW, tid);
    RowPre<BH, N, NT> rp;
    rp.load(p_bias, p_scatter, row0, tid);

    const int rq = lane % RQ;                           // row group: rows rq*VEC .. rq*VEC+VEC-1
    const int cs = lane / RQ;                           // column slot (BCR) or tile slot (CBR)
    const WT* vals = reinterpret_cast<const WT*>(p_vals);

    // Wave-load i of the chunk -> (address of this lane's 16 bytes, index of its x value, valid).
    const int ncols = ntiles * BW;
    const int ntg = (ntiles + G - 1) / G;               // CBR: groups of G tiles
    const int nloads = (LAYOUT == PIVOT_BCR) ? (ncols + G - 1) / G : BW * ntg;
    auto locate = [&](int i, size_t& off, int& xi) -> bool {
        if constexpr (LAYOUT == PIVOT_BCR) {
            const int q = i * G + cs;                   // column of the chunk's tile stream: tile q/BW, column q%BW
            const int qc = q < ncols ? q : (ncols > 0 ? ncols - 1 : 0);
            off = ((size_t)tile_begin * BW + qc) * BH + rq * VEC;
            xi = qc;
            return q < ncols;
        } else {
            const int c = i / (ntg > 0 ? ntg : 1);
            const int tl = (i - c * ntg) * G + cs;
            const int tc = tl < ntiles ? tl : (ntiles > 0 ? ntiles - 1 : 0);
            const int cc = c < BW ? c : BW - 1;
            off = ((size_t)cc * a.T + tile_begin + tc) * BH + rq * VEC;
            xi = tc * BW + cc;
            return tl < ntiles && c < BW;
        }
    };

    // unconditional, clamped loads (the value array is followed by zero padding)
    const int imax = nloads > 0 ? nloads - 1 : 0;
    V w[U];
    auto fill = [&](int u, int i) {
        size_t off; int xi;
        locate(i < imax ? i : imax, off, xi);
        w[u] = load16<V>(vals + off);
    };
    #pragma unroll
    for (int u = 0; u < U; ++u) fill(u, wave + u * NW);

    xst.template gather<false>(a.batch, a.ldx, 0, a.xs_stride, p_idx, reinterpret_cast<const WT*>(p_x), xs, tile_begin, ncols, b0, tid);
    lds_barrier();

    float acc[VEC];
    #pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    auto consume = [&](int u, int i) {
        size_t off; int xi;
        if (locate(i, off, xi)) {
            const float xv = (float)xs[xi];
            #pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = fmaf((float)w[u][v], xv, acc[v]);
        }
    };
    int i0 = wave;
    for (; i0 + NW * U < nloads; i0 += NW * U) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            consume(u, i0 + u * NW);
            fill(u, i0 + u * NW + NW * U);
        }
    }
    #pragma unroll
    for (int u = 0; u < U; ++u)
        if (i0 + u * NW < nloads) consume(u, i0 + u * NW);

    // lanes that hold the same rows (different columns / tiles) -> one sum
    #pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = stride_sum<RQ>(acc[v]);

    __syncthreads();                                    // xs no longer needed; red aliases it
    if (cs == 0) {
        #pragma unroll
        for (int v = 0; v < VEC; ++v) red[wave * N + rq * VEC + v] = acc[v];
    }
    __syncthreads();
    finish_rows<BH, 1, NT>(a, red, NW, br, slot, first, nparts, rp, b0, tid, &s_flag);
}

template <typename WT, int LAYOUT, int BH, int BW>
static int launch_t(const FcArgs& a, int nw, dim3 grid, size_t smem, hipStream_t st) {
    if (nw >= 8) hipLaunchKernelGGL((fc_colmajor_kernel<WT, LAYOUT, BH, BW, 8>), grid, dim3(8 * 64), smem, st, PIVOT_LEAD_ARGS(a, a.xidx), a);
    else         hipLaunchKernelGGL((fc_colmajor_kernel<WT, LAYOUT, BH, BW, 4>), grid, dim3(4 * 64), smem, st, PIVOT_LEAD_ARGS(a, a.xidx), a);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

template <typename WT, int LAYOUT>
static int launch_shape(const FcArgs& a, int bh, int bw, int nw, dim3 grid, size_t smem, hipStream_t st) {
#define X(BH_, BW_) if (bh == BH_ && bw == BW_) return launch_t<WT, LAYOUT, BH_, BW_>(a, nw, grid, smem, st);
    PIVOT_SHAPES(X)
#undef X
    set_error("no column-major kernel for %dx%d tiles", bh, bw);
    return PIVOT_E_UNSUPPORTED;
}

int launch_colmajor(const FcArgs& a, int layout, int wdtype, int bh, int bw, int nw, dim3 grid, size_t smem, hipStream_t st) {
    if (layout == PIVOT_BCR) {
        if (wdtype == PIVOT_F32) return launch_shape<float, PIVOT_BCR>(a, bh, bw, nw, grid, smem, st);
        return launch_shape<_Float16, PIVOT_BCR>(a, bh, bw, nw, grid, smem, st);
    }
    if (wdtype == PIVOT_F32) return launch_shape<float, PIVOT_CBR>(a, bh, bw, nw, grid, smem, st);
    return launch_shape<_Float16, PIVOT_CBR>(a, bh, bw, nw, grid, smem, st);
}

}  // namespace pivot
