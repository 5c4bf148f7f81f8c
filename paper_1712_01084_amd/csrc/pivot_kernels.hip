// gfx950 kernels of the pruned fully-connected layer in PBP form
// (paper Eq. 2 and Listing 1, generalised per Section 4.1.5 to tiles that
// share block rows).
//
// One workgroup works on one "chunk": up to chunk_tiles consecutive kept
// tiles of one block row.  The steps of Listing 1 map as follows:
//   group fetch through P_col  -> gather the chunk's x-segments into LDS
//   block row dot products     -> 16-byte-per-lane coalesced stream of the
//                                 BRC tile values, FMA (or MFMA for batch >= 8)
//                                 against the staged x
//   (Section 4.1.5) reduction  -> lanes (DPP), waves (LDS), chunks of a split
//                                 block row (fixed-order sum by the last
//                                 workgroup to arrive)
//   group store through P_row  -> bias, activation, scatter
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "pivot_device.h"
#include "pivot_internal.h"

namespace pivot {

#define HIP_TRY(expr)                                                                  \
    do {                                                                               \
        hipError_t e_ = (expr);                                                        \
        if (e_ != hipSuccess) {                                                        \
            set_error("%s failed: %s", #expr, hipGetErrorString(e_));                  \
            return PIVOT_E_HIP;                                                        \
        }                                                                              \
    } while (0)

// Arguments of the layer kernels (passed by value).
struct FcArgs {
    const void*    vals;
    const int32_t* col_idx;
    const int4*    chunks;
    const int32_t* part_base;
    const float*   bias_p;
    const int32_t* xidx;        // [T*bw] index into x of every kept tile's columns (-1 = padding)
    const int32_t* scatter;
    const void*    x;
    void*          y;
    float*         partials;
    uint32_t*      tickets;
    long long ldx, ldy;
    int batch, act, out_f16, out_rows, nchunks, nbr, xs_stride;
};

template <typename WT> struct Elem;
template <> struct Elem<float>    { using vec = f32x4; static constexpr int VEC = 4; };
template <> struct Elem<_Float16> { using vec = f16x8; static constexpr int VEC = 8; };

__device__ __forceinline__ float dot_vec(const f32x4& w, const f32x4& x, float acc) {
    acc = fmaf(w.x, x.x, acc);
    acc = fmaf(w.y, x.y, acc);
    acc = fmaf(w.z, x.z, acc);
    acc = fmaf(w.w, x.w, acc);
    return acc;
}
__device__ __forceinline__ float dot_vec(const f16x8& w, const f16x8& x, float acc) {
    // fp16 products are exact in fp32; v_dot2_f32_f16 accumulates in fp32.
    acc = __builtin_amdgcn_fdot2(f16x2{w[0], w[1]}, f16x2{x[0], x[1]}, acc, false);
    acc = __builtin_amdgcn_fdot2(f16x2{w[2], w[3]}, f16x2{x[2], x[3]}, acc, false);
    acc = __builtin_amdgcn_fdot2(f16x2{w[4], w[5]}, f16x2{x[4], x[5]}, acc, false);
    acc = __builtin_amdgcn_fdot2(f16x2{w[6], w[7]}, f16x2{x[6], x[7]}, acc, false);
    return acc;
}

__device__ __forceinline__ void store_out(void* y, long long idx, float v, int out_f16) {
    if (out_f16) reinterpret_cast<_Float16*>(y)[idx] = (_Float16)v;
    else         reinterpret_cast<float*>(y)[idx] = v;
}

// Per-thread values that depend only on the block row, loaded at kernel start
// so that their latency overlaps the weight stream instead of following it:
// the bias and the destination index of every output this thread will finish
// (outputs idx = tid + k*NT, idx = j*BH + r).
template <int BH, int N, int NT>
struct RowPre {
    static constexpr int CNT = (N + NT - 1) / NT;
    float bias[CNT];
    int   dst[CNT];
    __device__ __forceinline__ void load(const FcArgs& a, int br, int tid) {
        #pragma unroll
        for (int k = 0; k < CNT; ++k) {
            const int idx = tid + k * NT;
            bias[k] = 0.f;
            dst[k] = -1;
            if (idx < N) {
                const int row = br * BH + idx % BH;
                bias[k] = a.bias_p[row];
                dst[k] = a.scatter ? a.scatter[row] : ((row < a.out_rows) ? row : -1);
            }
        }
    }
};

// Staging of the chunk's x-segments in LDS (Listing 1: the group fetch through
// P_col): xs[b][t*BW + c] = x[b][xidx[(tile_begin + t)*BW + c]].  xidx is the
// column index array already composed with the tile list, so one index load
// feeds the gather.  Index -1 (padding column) and batch rows past `batch`
// read as zero.  NBT consecutive threads share one column and take one batch
// row each.  The first XP indices per thread are fetched before the weight
// stream is issued (loads return in order: an index fetched after the weights
// would only arrive after them).
template <typename WT, int BW, int NBT, int NT>
struct XStage {
    static constexpr int XP = 2;
    static constexpr int STEP = NT / NBT;
    int src[XP];
    __device__ __forceinline__ void load_idx(const FcArgs& a, int tile_begin, int ne, int tid) {
        const int32_t* xi = a.xidx + (size_t)tile_begin * BW;
        #pragma unroll
        for (int k = 0; k < XP; ++k) {
            const int e = tid / NBT + k * STEP;
            src[k] = (e < ne) ? xi[e] : -1;
        }
    }
    __device__ __forceinline__ void gather(const FcArgs& a, WT* xs, int tile_begin, int ne, int b0, int tid) {
        const int b = tid % NBT;
        const bool row_ok = (b0 + b) < a.batch;
        const WT* xrow = reinterpret_cast<const WT*>(a.x) + (long long)(row_ok ? b0 + b : 0) * a.ldx;
        #pragma unroll
        for (int k = 0; k < XP; ++k) {
            const int e = tid / NBT + k * STEP;
            if (e < ne) {
                WT v = WT(0);
                if (src[k] >= 0 && row_ok) v = xrow[src[k]];
                xs[b * a.xs_stride + e] = v;
            }
        }
        const int32_t* xi = a.xidx + (size_t)tile_begin * BW;
        for (int e = tid / NBT + XP * STEP; e < ne; e += STEP) {
            const int sidx = xi[e];
            WT v = WT(0);
            if (sidx >= 0 && row_ok) v = xrow[sidx];
            xs[b * a.xs_stride + e] = v;
        }
    }
};

// Everything after the per-wave sums are in LDS `red[w*N + idx]`, idx = j*BH + r
// (j = batch column of this launch tile, r = row inside the block row):
// hand-over between the chunks of a split block row (Section 4.1.5: tiles that
// share rows need one more reduction), bias, activation, store through P_row.
template <int BH, int NBT, int NT>
__device__ __forceinline__ void finish_rows(const FcArgs& a, const float* red, int nred, int slot, int first,
                                            int nparts, const RowPre<BH, BH * NBT, NT>& rp,
                                            int b0, int gy, int tid, int* s_flag) {
    constexpr int N = BH * NBT;
    if (nparts > 1) {
        float* mine = a.partials + ((size_t)gy * a.nchunks + slot) * N;
        for (int idx = tid; idx < N; idx += NT) {
            float s = 0.f;
            for (int w = 0; w < nred; ++w) s += red[w * N + idx];
            agent_store(mine + idx, s);
        }
        // Hand-over without a device-wide fence.  The partials are written with
        // device-coherent (write-through) stores and read back with device-coherent
        // loads, so no cache write-back or invalidate is needed; all that has to
        // hold is that every store of this workgroup has completed before its
        // arrival is counted.  A release fence at device scope would write back the
        // whole L2 of the XCD for every workgroup and serialise the launch.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            uint32_t* tk = a.tickets + (size_t)gy * a.nbr + a.chunks[blockIdx.x].x;
            uint32_t prev = __hip_atomic_fetch_add(tk, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int last = (prev == (uint32_t)(nparts - 1));
            if (last) __hip_atomic_store(tk, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *s_flag = last;
        }
        __syncthreads();
        if (!*s_flag) return;
    }
    #pragma unroll
    for (int k = 0; k < RowPre<BH, N, NT>::CNT; ++k) {
        const int idx = tid + k * NT;
        if (idx >= N) break;
        const int j = idx / BH;
        if (b0 + j >= a.batch) continue;
        float s = 0.f;
        if (nparts > 1) {
            const float* p = a.partials + ((size_t)gy * a.nchunks + first) * N + idx;
            for (int q = 0; q < nparts; ++q) s += agent_load(p + (size_t)q * N);
        } else {
            for (int w = 0; w < nred; ++w) s += red[w * N + idx];
        }
        const float v = apply_act(s + rp.bias[k], a.act);
        if (rp.dst[k] >= 0) store_out(a.y, (long long)(b0 + j) * a.ldy + rp.dst[k], v, a.out_f16);
    }
}

// ---------------------------------------------------------------------------
// batch 1..4: vector-ALU kernel.  Lane l of a wave reads bytes [16 l, 16 l+16)
// of each 1 KB piece of the tile stream, i.e. VEC columns of one tile row;
// LPR lanes cover a row, a wave covers RPW rows per load.
// ---------------------------------------------------------------------------
template <typename WT, int BH, int BW, int NB, int NW>
__global__ void __launch_bounds__(NW * 64) fc_gemv_kernel(FcArgs a) {
    using V = typename Elem<WT>::vec;
    constexpr int VEC = Elem<WT>::VEC;
    constexpr int NT  = NW * 64;
    constexpr int LPR = BW / VEC;                       // lanes per tile row
    constexpr int RPW = 64 / LPR;                       // tile rows per wave-load
    constexpr int NL  = (BH >= RPW) ? BH / RPW : 1;     // wave-loads per tile
    constexpr int TPL = (BH >= RPW) ? 1 : RPW / BH;     // tiles per wave-load
    constexpr int U   = (NL >= 8) ? 1 : 8 / NL;         // groups in flight per wave
    constexpr int GROUP = TPL * BH * BW;                // elements per group of TPL tiles
    constexpr int N   = BH * NB;
    static_assert(BW >= VEC && LPR <= 64, "tile width not supported");

    extern __shared__ __align__(16) char smem[];
    __shared__ int s_flag;
    WT* xs = reinterpret_cast<WT*>(smem);
    float* red = reinterpret_cast<float*>(smem);        // reused after the stream phase

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int gy = blockIdx.y, b0 = gy * NB;
    const int4 cd = a.chunks[blockIdx.x];
    const int br = cd.x, tile_begin = cd.y, ntiles = cd.z - cd.y, slot = cd.w;
    const int ngroups = (ntiles + TPL - 1) / TPL;
    const int first = a.part_base[br];
    const int nparts = a.part_base[br + 1] - first;

    // order of issue = order of arrival: gather indices, epilogue operands, then the weights
    XStage<WT, BW, NB, NT> xst;
    xst.load_idx(a, tile_begin, ntiles * BW, tid);
    RowPre<BH, N, NT> rp;
    rp.load(a, br, tid);

    const int s  = lane / LPR;                          // row within the wave-load
    const int cg = lane % LPR;                          // column group
    const int ts = (TPL > 1) ? s / BH : 0;              // tile within the group
    const WT* vbase = reinterpret_cast<const WT*>(a.vals) + (size_t)tile_begin * BH * BW + lane * VEC;

    V w[U][NL];
    auto issue = [&](int g0) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + u * NW;
            const bool ok = (g < ngroups) && (g * TPL + ts < ntiles);
            #pragma unroll
            for (int j = 0; j < NL; ++j) {
                if (ok) w[u][j] = load16<V>(vbase + (size_t)g * GROUP + j * 64 * VEC);
                else    w[u][j] = V(0);
            }
        }
    };

    issue(wave);
    xst.gather(a, xs, tile_begin, ntiles * BW, b0, tid);
    lds_barrier();

    float acc[NL][NB];
    #pragma unroll
    for (int j = 0; j < NL; ++j)
        #pragma unroll
        for (int b = 0; b < NB; ++b) acc[j][b] = 0.f;

    for (int g0 = wave; g0 < ngroups; g0 += NW * U) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + u * NW;
            const int tl = g * TPL + ts;
            if (g < ngroups && tl < ntiles) {
                #pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const V xv = *reinterpret_cast<const V*>(xs + b * a.xs_stride + tl * BW + cg * VEC);
                    #pragma unroll
                    for (int j = 0; j < NL; ++j) acc[j][b] = dot_vec(w[u][j], xv, acc[j][b]);
                }
            }
        }
        if (g0 + NW * U < ngroups) issue(g0 + NW * U);
    }

    // lanes -> rows
    #pragma unroll
    for (int j = 0; j < NL; ++j)
        #pragma unroll
        for (int b = 0; b < NB; ++b) {
            float v = group_sum<LPR>(acc[j][b]);
            if constexpr (TPL > 1) v = stride_sum<BH * LPR>(v);
            acc[j][b] = v;
        }

    __syncthreads();                                    // xs no longer needed; red aliases it
    if (cg == 0 && (TPL == 1 || s < BH)) {
        #pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int r = (TPL > 1) ? s : j * RPW + s;
            #pragma unroll
            for (int b = 0; b < NB; ++b) red[wave * N + b * BH + r] = acc[j][b];
        }
    }
    __syncthreads();
    finish_rows<BH, NB, NT>(a, red, NW, slot, first, nparts, rp, b0, gy, tid, &s_flag);
}

// ---------------------------------------------------------------------------
// batch >= 8, fp16 weights: matrix-core kernels.  The tile is the A operand,
// the staged x-segment (k x batch) the B operand, accumulation in fp32.
// KIND 0: v_mfma_f32_16x16x32_f16, tiles with BH % 16 == 0, BW % 32 == 0, 16 batch columns.
//         lane l supplies A[row l%16][k 8(l/16)..+7] = 16 contiguous bytes of a BRC tile row.
// KIND 1: v_mfma_f32_32x32x16_f16, tiles with BH % 32 == 0, BW % 16 == 0, 32 batch columns.
//         lane l supplies A[row l%32][k 8(l/32)..+7].
// ---------------------------------------------------------------------------
template <int KIND> struct Mfma;
template <> struct Mfma<0> {
    static constexpr int MR = 16, MK = 32, NBT = 16, CV = 4;
    using acc_t = f32x4;
    __device__ static __forceinline__ acc_t run(f16x8 a, f16x8 b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
    // accumulator element v of lane l is C[row][col = l % 16]
    __device__ static __forceinline__ int row_of(int lane, int v) { return 4 * (lane / 16) + v; }
};
template <> struct Mfma<1> {
    static constexpr int MR = 32, MK = 16, NBT = 32, CV = 16;
    using acc_t = f32x16;
    __device__ static __forceinline__ acc_t run(f16x8 a, f16x8 b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ int row_of(int lane, int v) { return 8 * (v / 4) + 4 * (lane / 32) + (v % 4); }
};

template <int KIND, int BH, int BW, int NW>
__global__ void __launch_bounds__(NW * 64) fc_mfma_kernel(FcArgs a) {
    using MF = Mfma<KIND>;
    using acc_t = typename MF::acc_t;
    constexpr int MR = MF::MR, MK = MF::MK, NBT = MF::NBT, CV = MF::CV;
    constexpr int NT = NW * 64;
    constexpr int RB = BH / MR;                         // row blocks per tile
    constexpr int KS = BW / MK;                         // k steps per tile
    constexpr int LT = RB * KS;                         // 16-byte loads per lane per tile
    constexpr int U  = (LT >= 8) ? 1 : 8 / LT;          // tiles in flight per wave
    constexpr int N  = BH * NBT;
    static_assert(BH % MR == 0 && BW % MK == 0, "tile shape does not fit this MFMA");

    extern __shared__ __align__(16) char smem[];
    __shared__ int s_flag;
    _Float16* xs = reinterpret_cast<_Float16*>(smem);
    float* red = reinterpret_cast<float*>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int gy = blockIdx.y, b0 = gy * NBT;
    const int4 cd = a.chunks[blockIdx.x];
    const int br = cd.x, tile_begin = cd.y, ntiles = cd.z - cd.y, slot = cd.w;
    const int first = a.part_base[br];
    const int nparts = a.part_base[br + 1] - first;

    XStage<_Float16, BW, NBT, NT> xst;
    xst.load_idx(a, tile_begin, ntiles * BW, tid);
    RowPre<BH, N, NT> rp;
    rp.load(a, br, tid);

    const int li = lane % MR;                           // A row / B column of this lane
    const int lg = lane / MR;                           // k group of 8
    const _Float16* vbase = reinterpret_cast<const _Float16*>(a.vals) + (size_t)tile_begin * BH * BW
                            + li * BW + lg * 8;

    f16x8 w[U][LT];
    auto issue = [&](int t0) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * NW;
            #pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                #pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if (t < ntiles) w[u][rb * KS + ks] = load16<f16x8>(vbase + (size_t)t * BH * BW + rb * MR * BW + ks * MK);
                    else            w[u][rb * KS + ks] = f16x8(0);
                }
        }
    };

    issue(wave);
    xst.gather(a, xs, tile_begin, ntiles * BW, b0, tid);
    lds_barrier();

    acc_t acc[RB];
    #pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = acc_t(0);

    for (int t0 = wave; t0 < ntiles; t0 += NW * U) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * NW;
            if (t < ntiles) {
                #pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const f16x8 xv = *reinterpret_cast<const f16x8*>(xs + li * a.xs_stride + t * BW + ks * MK + lg * 8);
                    #pragma unroll
                    for (int rb = 0; rb < RB; ++rb) acc[rb] = MF::run(w[u][rb * KS + ks], xv, acc[rb]);
                }
            }
        }
        if (t0 + NW * U < ntiles) issue(t0 + NW * U);
    }

    __syncthreads();                                    // xs no longer needed; red aliases it
    #pragma unroll
    for (int rb = 0; rb < RB; ++rb)
        #pragma unroll
        for (int v = 0; v < CV; ++v)
            red[wave * N + li * BH + rb * MR + MF::row_of(lane, v)] = acc[rb][v];
    __syncthreads();
    finish_rows<BH, NBT, NT>(a, red, NW, slot, first, nparts, rp, b0, gy, tid, &s_flag);
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
static constexpr int kWaves = 4;

static int mfma_kind(int wdtype, int bh, int bw) {
    if (wdtype != PIVOT_F16) return -1;
    if (bw % 32 == 0 && bh % 16 == 0) return 0;
    if (bh % 32 == 0 && bw % 16 == 0) return 1;
    return -1;
}

int fc_batch_tile(int wdtype, int bh, int bw, int batch) {
    if (batch >= 8) {
        int k = mfma_kind(wdtype, bh, bw);
        if (k == 0) return 16;
        if (k == 1) return 32;
    }
    return batch >= 3 ? 4 : batch;
}

size_t fc_workspace_bytes(const HostPlan& hp, int batch) {
    if (batch < 1) return 0;
    int nbt = fc_batch_tile(hp.d.wdtype, hp.d.bh, hp.d.bw, batch);
    int ngy = (batch + nbt - 1) / nbt;
    size_t tickets = align_up((size_t)4 * hp.nbr * ngy, 256);
    size_t partials = (hp.max_parts > 1) ? (size_t)4 * hp.nchunks * hp.d.bh * nbt * ngy : 0;
    return tickets + align_up(partials, 256);
}

template <typename WT, int BH, int BW, int NB>
static int launch_gemv_t(const FcArgs& a, int nw, dim3 grid, size_t smem, hipStream_t st) {
    if (nw == 16)     hipLaunchKernelGGL((fc_gemv_kernel<WT, BH, BW, NB, 16>), grid, dim3(16 * 64), smem, st, a);
    else if (nw == 8) hipLaunchKernelGGL((fc_gemv_kernel<WT, BH, BW, NB, 8>), grid, dim3(8 * 64), smem, st, a);
    else              hipLaunchKernelGGL((fc_gemv_kernel<WT, BH, BW, NB, 4>), grid, dim3(4 * 64), smem, st, a);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

template <typename WT, int BH, int BW>
static int launch_gemv_nb(const FcArgs& a, int nb, int nw, dim3 grid, size_t smem, hipStream_t st) {
    switch (nb) {
        case 1: return launch_gemv_t<WT, BH, BW, 1>(a, nw, grid, smem, st);
        case 2: return launch_gemv_t<WT, BH, BW, 2>(a, nw, grid, smem, st);
        default: return launch_gemv_t<WT, BH, BW, 4>(a, nw, grid, smem, st);
    }
}

template <int KIND, int BH, int BW>
static int launch_mfma_t(const FcArgs& a, dim3 grid, size_t smem, hipStream_t st) {
    hipLaunchKernelGGL((fc_mfma_kernel<KIND, BH, BW, kWaves>), grid, dim3(kWaves * 64), smem, st, a);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

#define PIVOT_SHAPES(X) \
    X(8, 8) X(8, 16) X(8, 32) X(8, 64) \
    X(16, 8) X(16, 16) X(16, 32) X(16, 64) \
    X(32, 8) X(32, 16) X(32, 32) X(32, 64) \
    X(64, 8) X(64, 16) X(64, 32) X(64, 64)

int launch_fc(const FcLaunch& L) {
    const int nbt = fc_batch_tile(L.wdtype, L.bh, L.bw, L.batch);
    const int ngy = (L.batch + nbt - 1) / nbt;
    FcArgs a;
    a.vals = L.vals; a.col_idx = L.col_idx; a.chunks = reinterpret_cast<const int4*>(L.chunks);
    a.part_base = L.part_base; a.bias_p = L.bias_p; a.xidx = L.xidx; a.scatter = L.scatter;
    a.x = L.x; a.y = L.y; a.partials = L.partials; a.tickets = L.tickets;
    a.ldx = L.ldx; a.ldy = L.ldy; a.batch = L.batch; a.act = L.act; a.out_f16 = L.out_f16;
    a.out_rows = L.out_rows; a.nchunks = L.nchunks; a.nbr = L.nbr;
    const int es = elem_size(L.wdtype);
    // staged x: nbt rows of chunk_tiles*bw elements (+16 bytes to skew LDS banks)
    a.xs_stride = L.chunk_tiles * L.bw + 16 / es;
    size_t xs_bytes = (size_t)nbt * a.xs_stride * es;
    const int nw = (nbt >= 16) ? kWaves : ((L.wg_waves == 16 || L.wg_waves == 8) ? L.wg_waves : 4);
    size_t red_bytes = (size_t)nw * L.bh * nbt * 4;
    size_t smem = align_up(xs_bytes > red_bytes ? xs_bytes : red_bytes, 16);
    if (smem > 64 * 1024) { set_error("chunk does not fit in LDS (%zu bytes)", smem); return PIVOT_E_UNSUPPORTED; }
    dim3 grid(L.nchunks, ngy);
    hipStream_t st = reinterpret_cast<hipStream_t>(L.stream);

    if (nbt >= 16) {
        const int kind = mfma_kind(L.wdtype, L.bh, L.bw);
#define X(BH_, BW_)                                                                                   \
        if (L.bh == BH_ && L.bw == BW_) {                                                             \
            if constexpr (BW_ % 32 == 0 && BH_ % 16 == 0) { if (kind == 0) return launch_mfma_t<0, BH_, BW_>(a, grid, smem, st); } \
            else if constexpr (BH_ % 32 == 0 && BW_ % 16 == 0) { if (kind == 1) return launch_mfma_t<1, BH_, BW_>(a, grid, smem, st); } \
        }
        PIVOT_SHAPES(X)
#undef X
        set_error("no matrix-core kernel for %dx%d tiles", L.bh, L.bw);
        return PIVOT_E_UNSUPPORTED;
    }
    if (L.wdtype == PIVOT_F32) {
#define X(BH_, BW_) if (L.bh == BH_ && L.bw == BW_) return launch_gemv_nb<float, BH_, BW_>(a, nbt, nw, grid, smem, st);
        PIVOT_SHAPES(X)
#undef X
    } else {
#define X(BH_, BW_) if (L.bh == BH_ && L.bw == BW_) return launch_gemv_nb<_Float16, BH_, BW_>(a, nbt, nw, grid, smem, st);
        PIVOT_SHAPES(X)
#undef X
    }
    set_error("no kernel for %dx%d tiles", L.bh, L.bw);
    return PIVOT_E_UNSUPPORTED;
}

// ---------------------------------------------------------------------------
// small utility kernels
// ---------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint32_t* p, size_t nwords) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < nwords; i += stride) p[i] = 0u;
}

__global__ void null_kernel() {}

int launch_null(void* stream) {
    hipLaunchKernelGGL(null_kernel, dim3(1), dim3(64), 0, reinterpret_cast<hipStream_t>(stream));
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

int launch_fill_zero(void* dev, size_t bytes, void* stream) {
    if (bytes == 0) return PIVOT_OK;
    if (bytes % 4 != 0 || (reinterpret_cast<uintptr_t>(dev) % 4) != 0) { set_error("fill needs 4-byte alignment"); return PIVOT_E_SHAPE; }
    size_t nwords = bytes / 4;
    int blocks = (int)((nwords + 255) / 256 > 2048 ? 2048 : (nwords + 255) / 256);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<uint32_t*>(dev), nwords);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

// ---------------------------------------------------------------------------
// dense comparator: y = act(W x + b), W streamed once, one wave per R rows.
// ---------------------------------------------------------------------------
template <typename WT, int NB, int R>
__global__ void __launch_bounds__(256) dense_kernel(const WT* W, int M, int K, const WT* x, long long ldx,
                                                    const float* bias, float* y, long long ldy, int batch, int act) {
    using V = typename Elem<WT>::vec;
    constexpr int VEC = Elem<WT>::VEC;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = (blockIdx.x * 4 + wave) * R;
    if (row0 >= M) return;
    float acc[R][NB];
    #pragma unroll
    for (int r = 0; r < R; ++r)
        #pragma unroll
        for (int b = 0; b < NB; ++b) acc[r][b] = 0.f;
    const WT* wrow[R];
    #pragma unroll
    for (int r = 0; r < R; ++r) wrow[r] = W + (size_t)((row0 + r < M) ? row0 + r : M - 1) * K;
    #pragma unroll 2
    for (int k = lane * VEC; k < K; k += 64 * VEC) {
        V wv[R];
        #pragma unroll
        for (int r = 0; r < R; ++r) wv[r] = load16<V>(wrow[r] + k);
        #pragma unroll
        for (int b = 0; b < NB; ++b) {
            const V xv = (b < batch) ? load16<V>(x + (size_t)b * ldx + k) : V(0);
            #pragma unroll
            for (int r = 0; r < R; ++r) acc[r][b] = dot_vec(wv[r], xv, acc[r][b]);
        }
    }
    #pragma unroll
    for (int r = 0; r < R; ++r)
        #pragma unroll
        for (int b = 0; b < NB; ++b) {
            float v = group_sum<64>(acc[r][b]);
            if (lane == 0 && row0 + r < M && b < batch)
                y[(size_t)b * ldy + row0 + r] = apply_act(v + (bias ? bias[row0 + r] : 0.f), act);
        }
}

template <typename WT, int NB, int R>
static int launch_dense_t(const void* W, int M, int K, const void* x, int64_t ldx, const float* bias,
                          void* y, int64_t ldy, int batch, int act, hipStream_t st) {
    int rows_per_block = 4 * R;
    dim3 grid((M + rows_per_block - 1) / rows_per_block);
    hipLaunchKernelGGL((dense_kernel<WT, NB, R>), grid, dim3(256), 0, st, (const WT*)W, M, K, (const WT*)x,
                       (long long)ldx, bias, (float*)y, (long long)ldy, batch, act);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

int launch_dense(const void* W, int wdtype, int M, int K, const void* x, int64_t ldx, const float* bias,
                 void* y, int64_t ldy, int batch, int act, void* stream) {
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int vec = (wdtype == PIVOT_F32) ? 4 : 8;
    if (K % vec != 0 || ldx % vec != 0) { set_error("dense comparator needs K and ldx to be multiples of %d", vec); return PIVOT_E_UNSUPPORTED; }
    if (batch < 1 || batch > 16) { set_error("dense comparator supports batch 1..16"); return PIVOT_E_UNSUPPORTED; }
    if (wdtype == PIVOT_F32) {
        if (batch == 1) return launch_dense_t<float, 1, 4>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
        if (batch <= 4) return launch_dense_t<float, 4, 2>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
        return launch_dense_t<float, 16, 1>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
    }
    if (batch == 1) return launch_dense_t<_Float16, 1, 4>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
    if (batch <= 4) return launch_dense_t<_Float16, 4, 2>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
    return launch_dense_t<_Float16, 16, 1>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
}

// ---------------------------------------------------------------------------
// LSTM cell around the pruned gate matrix (gate order i,f,g,o).
// ---------------------------------------------------------------------------
__device__ __forceinline__ float sigmoidf_(float v) { return 1.0f / (1.0f + __expf(-v)); }

__global__ void lstm_cell_kernel(LstmCellLaunch L) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= L.batch * L.H) return;
    const int b = idx / L.H, j = idx - b * L.H;
    const float* z = L.z + (size_t)b * L.M_pad;
    const float zi = z[L.invprow[j]];
    const float zf = z[L.invprow[L.H + j]];
    const float zg = z[L.invprow[2 * L.H + j]];
    const float zo = z[L.invprow[3 * L.H + j]];
    const float c = sigmoidf_(zf) * L.c[idx] + sigmoidf_(zi) * tanhf(zg);
    const float h = sigmoidf_(zo) * tanhf(c);
    L.c[idx] = c;
    L.h[idx] = h;
    if (L.xg_next) {
        const size_t o = (size_t)b * L.K_pad + L.invpcol[j];
        if (L.wdtype == PIVOT_F16) reinterpret_cast<_Float16*>(L.xg_next)[o] = (_Float16)h;
        else                       reinterpret_cast<float*>(L.xg_next)[o] = h;
    }
    if (L.z_dbg) {
        float* zd = L.z_dbg + (size_t)b * 4 * L.H;
        zd[j] = zi; zd[L.H + j] = zf; zd[2 * L.H + j] = zg; zd[3 * L.H + j] = zo;
    }
}

int launch_lstm_cell(const LstmCellLaunch& L) {
    int n = L.batch * L.H;
    hipLaunchKernelGGL(lstm_cell_kernel, dim3((n + 255) / 256), dim3(256), 0, reinterpret_cast<hipStream_t>(L.stream), L);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

template <typename WT>
__global__ void lstm_place_inputs_kernel(const WT* xs, WT* xg_all, const int32_t* invpcol, int H, int I,
                                         int K_pad, size_t total) {
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; idx < total; idx += stride) {
        const size_t tb = idx / I;               // step*batch + b
        const int i = (int)(idx - tb * I);
        xg_all[tb * K_pad + invpcol[H + i]] = xs[idx];
    }
}

int launch_lstm_place_inputs(const void* xs, void* xg_all, const int32_t* invpcol, int H, int I, int K_pad,
                             int steps, int batch, int wdtype, void* stream) {
    size_t total = (size_t)steps * batch * I;
    if (total == 0) return PIVOT_OK;
    int blocks = (int)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (wdtype == PIVOT_F16)
        hipLaunchKernelGGL(lstm_place_inputs_kernel<_Float16>, dim3(blocks), dim3(256), 0, st,
                           (const _Float16*)xs, (_Float16*)xg_all, invpcol, H, I, K_pad, total);
    else
        hipLaunchKernelGGL(lstm_place_inputs_kernel<float>, dim3(blocks), dim3(256), 0, st,
                           (const float*)xs, (float*)xg_all, invpcol, H, I, K_pad, total);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

template <typename WT>
__global__ void lstm_place_state_kernel(const float* h, WT* xg, const int32_t* invpcol, int H, int K_pad, int n) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    const int b = idx / H, j = idx - b * H;
    xg[(size_t)b * K_pad + invpcol[j]] = (WT)h[idx];
}

int launch_lstm_place_state(const float* h, void* xg, const int32_t* invpcol, int H, int K_pad, int batch,
                            int wdtype, void* stream) {
    int n = batch * H;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (wdtype == PIVOT_F16)
        hipLaunchKernelGGL(lstm_place_state_kernel<_Float16>, dim3((n + 255) / 256), dim3(256), 0, st, h, (_Float16*)xg, invpcol, H, K_pad, n);
    else
        hipLaunchKernelGGL(lstm_place_state_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, st, h, (float*)xg, invpcol, H, K_pad, n);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

}  // namespace pivot
