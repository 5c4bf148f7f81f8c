// Device templates of the pruned-layer kernels for gfx950 (paper Eq. 2 and
// Listing 1, generalised per Section 4.1.5 to tiles that share block rows).
//
// One workgroup ("work item") handles one chunk of the schedule: up to
// chunk_tiles consecutive kept tiles of one block row, and within them one row
// slice (blockIdx.z) of every tile.  The steps of Listing 1 map as follows:
//   group fetch through P_col  -> the chunk's x-segments are gathered into LDS
//                                 (vector kernel) or read as MFMA B fragments
//                                 from an x already in block order (matrix kernel)
//   block row dot products     -> 16-byte-per-lane coalesced stream of the BRC
//                                 tile values, FMA / dot2 (batch <= 4) or MFMA
//   (Section 4.1.5) reduction  -> lanes (DPP), waves (LDS), chunks of a split
//                                 block row (fixed-order sum by the last
//                                 workgroup to arrive)
//   group store through P_row  -> bias, activation, scatter
#pragma once

#include <hip/hip_runtime.h>

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

static constexpr int kTicketStride = 64;   // uint32 words between arrival counters (one per 256-byte line)

// Arguments of the layer kernels (passed by value).
struct FcArgs {
    const void*    vals;
    const int32_t* col_idx;     // [T] block column of every kept tile (matrix kernel)
    const int32_t* xidx;        // [T*bw] index into x of every kept tile's columns, -1 = padding (vector kernel)
    const int4*    chunks;
    const int32_t* part_base;
    const float*   bias_p;
    const int32_t* scatter;     // [M_pad] destination of every block-space row, -1 = not stored
    const void*    x;
    void*          y;
    float*         partials;
    uint32_t*      tickets;
    long long ldx, ldy;
    int batch, act, out_f16, nchunks, nbr, xs_stride;
    int bh_full;                // rows of a whole tile (the kernels' BH is the height of one row slice)
    int tile_elems;             // bh_full * bw
    int uniform_ct;             // > 0: every chunk has exactly this many tiles and chunk i starts at tile i*uniform_ct,
    int uniform_parts;          //      uniform_parts chunks per block row: the descriptor is computed, not loaded
    int T;                      // kept tiles in the whole plan (the CBR layout strides by it)
    int chunk_tiles;            // the plan's chunk size (vector kernel: fixes the LDS row stride)
    int xn_vecs;                // x-resident vector kernel: 16-byte vectors per row of x (row length / VEC)
    int xn_stride;              //   elements between the LDS copies of consecutive batch rows (the row length)
    long long* trace;           // timeline builds only (PIVOT_TRACE): eight time stamps per wavefront, else unused
};

// Timeline builds (-DPIVOT_TRACE, see bench_timeline.py): the vector kernel records the constant 100 MHz
// clock at eight points per wavefront: 0 start, 1 every load issued, 2 copy of x stored to LDS, 3 past the
// barrier behind it, 4 x-segments staged, 5 last weight consumed, 6 sums of all wavefronts in LDS, 7 outputs
// stored.  In ordinary builds the stamps compile to nothing.
// Ablation builds (-DPIVOT_ABLATE=bits, see bench_timeline.py --ablations): the vector kernel with one part of
// its work left out, to measure what that part costs.  The results of such a build are wrong on purpose; every
// access stays in bounds.  1: no x at all (no copy, no gather index, no staging; the FMAs read whatever the LDS
// holds)  2: x copied into LDS but never staged (no barrier behind the copy, no gather)  4: no copy of x (barrier
// and LDS-to-LDS gather kept, from an LDS region nobody filled)  8: outputs computed but not stored
// 16: no reduction and no outputs (one value per workgroup is stored)  32: no permutations (batch 1, vector
// kernel; for plans whose permutations are the identity and whose M and K are whole tiles, see
// bench_paper_grid.py --gather-off): the launcher passes the tile list's block columns in place of the
// per-column gather index, an x-segment is the BW contiguous elements at block column * BW, and an output row
// is stored at its own index without a look-up.  The product build has PIVOT_ABLATE 0.
#ifndef PIVOT_ABLATE
#define PIVOT_ABLATE 0
#endif

#ifdef PIVOT_TRACE
#define PIVOT_STAMP_DECL long long tr_[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define PIVOT_STAMP(i) do { __builtin_amdgcn_sched_barrier(0); tr_[i] = wall_clock64(); __builtin_amdgcn_sched_barrier(0); } while (0)
#define PIVOT_STAMP_FLUSH(a, nw, wave, lane)                                                                     \
    do { if ((a).trace && (lane) == 0) {                                                                          \
        long long* t_ = (a).trace + ((((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * (nw) + (wave)) * 8; \
        for (int i_ = 0; i_ < 8; ++i_) t_[i_] = tr_[i_]; } } while (0)
#else
#define PIVOT_STAMP_DECL do {} while (0)
#define PIVOT_STAMP(i) do {} while (0)
#define PIVOT_STAMP_FLUSH(a, nw, wave, lane) do {} while (0)
#endif

// The seven pointers every wavefront needs first are separate leading kernel
// arguments: with kernel-argument preloading they arrive in SGPRs with the
// wave, so the first dependent load can be issued at once.
#define PIVOT_LEAD_PARAMS const int4* __restrict__ p_chunks, const int32_t* __restrict__ p_part_base, \
    const int32_t* __restrict__ p_idx, const void* __restrict__ p_vals, const float* __restrict__ p_bias, \
    const int32_t* __restrict__ p_scatter, const void* __restrict__ p_x
#define PIVOT_LEAD_ARGS(a, idx) (a).chunks, (a).part_base, (idx), (a).vals, (a).bias_p, (a).scatter, (a).x

// The vector kernel goes further: everything it needs before and while its
// loads are issued (six pointers and two packed scalars = the 14 dwords that
// are preloaded into SGPRs) comes first, so that nothing on the way to the
// first FMA waits for a fetch of the argument block; the rest of FcArgs is
// first touched in the epilogue (the row stride of x, needed only with more
// than one batch row, also comes from there).
// q_ct_parts = tiles per chunk | uniform_parts << 16 (uniform_parts 0: the schedule is not regular, the low half
//              is then the plan's chunk size); q_misc = bh_full | batch << 7 | xn_vecs << 14.
#define PIVOT_GEMV_PARAMS const int4* __restrict__ p_chunks, const int32_t* __restrict__ p_idx, \
    const void* __restrict__ p_vals, const void* __restrict__ p_x, const float* __restrict__ p_bias, \
    const int32_t* __restrict__ p_scatter, int q_ct_parts, int q_misc
#define PIVOT_GEMV_ARGS(a) (a).chunks, (a).xidx, (a).vals, (a).x, (a).bias_p, (a).scatter, \
    ((a).uniform_ct > 0 ? ((a).uniform_ct | ((a).uniform_parts << 16)) : (a).chunk_tiles), \
    ((a).bh_full | ((a).batch << 7) | (int)((unsigned)(a).xn_vecs << 14))

// Per-dtype / per-path launchers, each in its own translation unit.
int launch_gemv_f32(const FcArgs& a, int bhs, int bw, int nb, int nw, int xres, dim3 grid, size_t smem, hipStream_t st);
int launch_gemv_f16(const FcArgs& a, int bhs, int bw, int nb, int nw, int xres, dim3 grid, size_t smem, hipStream_t st);
int launch_mfma_f16(const FcArgs& a, int kind, int bhs, int bw, int nw, dim3 grid, size_t smem, hipStream_t st);
int launch_mfma_lds_f16(const FcArgs& a, int kind, int bhs, int bw, int nbs, int nw, int xres, dim3 grid, size_t smem, hipStream_t st);
int launch_mfma_xrow_f16(const FcArgs& a, int kind, int bhs, int bw, dim3 grid, size_t smem, hipStream_t st);
int launch_colmajor(const FcArgs& a, int layout, int wdtype, int bh, int bw, int nw, dim3 grid, size_t smem, hipStream_t st);

#define PIVOT_SHAPES(X) \
    X(8, 8) X(8, 16) X(8, 32) X(8, 64) \
    X(16, 8) X(16, 16) X(16, 32) X(16, 64) \
    X(32, 8) X(32, 16) X(32, 32) X(32, 64) \
    X(64, 8) X(64, 16) X(64, 32) X(64, 64)

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
// (outputs idx = tid + k*NT, idx = j*BH + r).  The loads are unconditional (the
// row is always inside the padded block row), so no branch hides them from the
// compiler's count of outstanding loads (loading only in the threads that finish
// an output was measured: 4096x9216 fp32 0.06 us slower cold, others +-0.05).
template <int BH, int N, int NT>
struct RowPre {
    static constexpr int CNT = (N + NT - 1) / NT;
    float bias[CNT];
    int   dst[CNT];
    __device__ __forceinline__ void load(const float* bias_p, const int32_t* scatter, int row0, int tid) {
        #pragma unroll
        for (int k = 0; k < CNT; ++k) {
            const int row = row0 + (tid + k * NT) % BH;
            bias[k] = bias_p[row];
            dst[k] = (PIVOT_ABLATE & 32) ? row : scatter[row];
        }
    }
};

// Staging of the chunk's x-segments in LDS (Listing 1: the group fetch through
// P_col): xs[b][t*BW + c] = x[b][xidx[(tile_begin + t)*BW + c]].  xidx is the
// column index array already composed with the tile list, so one index load
// feeds the gather.  Index -1 (padding column) and batch rows past `batch`
// read as zero.  A thread takes elements tid, tid + NT, ... and moves all NB
// batch rows of each: the index does not depend on the batch row, so the
// number of dependent index rounds is that of a single row.  The first XP
// indices per thread are fetched before the weight stream is issued (loads
// return in order: an index fetched after the weights would only arrive after
// them).  All of these loads and LDS writes are unconditional: out-of-range
// elements use a clamped index and land in a dump slot at the end of the LDS row.
// PK = true: xidx holds the chunk's packed source-ordered list instead (entry =
// source | staged position << kSortSrcBits, source field all ones = padding
// column): thread tid takes list entries tid, tid + NT, ..., so the lanes of a
// wavefront read neighbouring addresses of x (several elements per cache line)
// and each writes the staged position its entry names.
template <typename WT, int BW, int NB, int NT, int XP = 4, bool PK = false>
struct XStage {
    int src[XP];
    __device__ __forceinline__ void load_idx(const int32_t* xidx, int tile_begin, int ne, int tid) {
        const int32_t* xi = xidx + (size_t)tile_begin * BW;
        const int emax = ne > 0 ? ne - 1 : 0;       // index arrays carry 16 bytes of padding: xi[0] is readable
        #pragma unroll
        for (int k = 0; k < XP; ++k) {
            const int e = tid + k * NT;
            src[k] = xi[e < emax ? e : emax];
        }
    }
    // SRC_LDS = false: `x` is the global x (one dependent global load per element).
    // SRC_LDS = true:  `x` is the whole of x already copied into LDS (row b at
    // b * xn_stride), so the gather costs no second trip to memory.
    template <bool SRC_LDS>
    __device__ __forceinline__ void gather(int batch, long long ldx, int xn_stride, int xs_stride,
                                           const int32_t* xidx, const WT* x, WT* xs,
                                           int tile_begin, int ne, int b0, int tid) {
        const WT* xrow[NB];
        bool row_ok[NB];
        #pragma unroll
        for (int b = 0; b < NB; ++b) {
            row_ok[b] = (b0 + b) < batch;
            xrow[b] = SRC_LDS ? x + b * xn_stride : x + (long long)(row_ok[b] ? b0 + b : 0) * ldx;
        }
        const int dump = xs_stride - 1;
        // `eb` (the same in every thread) = first element of the round; a thread's k-th element is eb + tid + k*NT.
        // Gathering from global memory, a k whose NT elements all lie past the end is skipped by the whole
        // workgroup: with NB rows per element the clamped loads it would issue are NB times those of the one-row
        // form (4096x4096 at 5 % kept, batch 8: 5.05 -> 4.41 us).  From the LDS copy the spare reads cost less
        // than the branches (dense, batch 2: +0.6 us with them), so there every k runs.
        auto move = [&](const int (&sr)[XP], int eb) {
            WT v[XP][NB];
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                if (!SRC_LDS && k > 0 && eb + k * NT >= ne) continue;
                const int s = PK ? (sr[k] & kSortSrcNone) : sr[k];
                const int si = PK ? (s != kSortSrcNone ? s : 0) : (s > 0 ? s : 0);
                #pragma unroll
                for (int b = 0; b < NB; ++b) v[k][b] = xrow[b][si];
            }
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                if (!SRC_LDS && k > 0 && eb + k * NT >= ne) continue;
                const int e = eb + tid + k * NT;
                const int pos = PK ? (int)((unsigned)sr[k] >> kSortSrcBits) : e;
                const bool real = PK ? (sr[k] & kSortSrcNone) != kSortSrcNone : sr[k] >= 0;
                #pragma unroll
                for (int b = 0; b < NB; ++b)
                    xs[b * xs_stride + (e < ne ? pos : dump)] = (real && row_ok[b]) ? v[k][b] : WT(0);
            }
        };
        move(src, 0);
        // longer chunks: further rounds of XP elements per thread, each round's loads issued together
        const int32_t* xi = xidx + (size_t)tile_begin * BW;
        const int emax = ne > 0 ? ne - 1 : 0;
        // (from the LDS copy a thread leaves when its own elements run out: measured 0.2-0.3 us faster on dense
        // 4096x4096 at batch 2 and 4 than leaving together)
        for (int eb = XP * NT; SRC_LDS ? (eb + tid < ne) : (eb < ne); eb += XP * NT) {
            int s2[XP];
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                const int e = eb + tid + k * NT;
                s2[k] = xi[e < emax ? e : emax];
            }
            move(s2, eb);
        }
    }
};

// One batch row: the same staging with the batch loop folded away.
template <typename WT, int BW, int NT, int XP>
struct XStage<WT, BW, 1, NT, XP, false> {
    int src[XP];
    __device__ __forceinline__ void load_idx(const int32_t* xidx, int tile_begin, int ne, int tid) {
        const int32_t* xi = xidx + (size_t)tile_begin * BW;
        const int emax = ne > 0 ? ne - 1 : 0;
        #pragma unroll
        for (int k = 0; k < XP; ++k) {
            const int e = tid + k * NT;
            src[k] = xi[e < emax ? e : emax];
        }
    }
    template <bool SRC_LDS>
    __device__ __forceinline__ void gather(int batch, long long ldx, int xn_stride, int xs_stride,
                                           const int32_t* xidx, const WT* x, WT* xs,
                                           int tile_begin, int ne, int b0, int tid) {
        const bool row_ok = b0 < batch;
        const WT* xrow = SRC_LDS ? x : x + (long long)(row_ok ? b0 : 0) * ldx;
        const int dump = xs_stride - 1;
        WT v[XP];
        #pragma unroll
        for (int k = 0; k < XP; ++k) v[k] = xrow[src[k] > 0 ? src[k] : 0];
        #pragma unroll
        for (int k = 0; k < XP; ++k) {
            const int e = tid + k * NT;
            xs[e < ne ? e : dump] = (src[k] >= 0 && row_ok) ? v[k] : WT(0);
        }
        const int32_t* xi = xidx + (size_t)tile_begin * BW;
        const int emax = ne > 0 ? ne - 1 : 0;
        for (int e0 = tid + XP * NT; e0 < ne; e0 += XP * NT) {
            int s2[XP];
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                const int e = e0 + k * NT;
                s2[k] = xi[e < emax ? e : emax];
            }
            WT v2[XP];
            #pragma unroll
            for (int k = 0; k < XP; ++k) v2[k] = xrow[s2[k] > 0 ? s2[k] : 0];
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                const int e = e0 + k * NT;
                xs[e < ne ? e : dump] = (s2[k] >= 0 && row_ok) ? v2[k] : WT(0);
            }
        }
    }
};

// One batch row, vector kernel: every wavefront stages the x-segments of ITS OWN groups of tiles only (groups
// wave, wave + NW, ...: exactly those whose weights it streams), so a staged value is written and read by the
// same wavefront and no workgroup barrier stands between the gather and the first FMA.  GE = staged elements
// per group (TPL tiles of BW columns); the wavefront's e-th element belongs to its (e / GE)-th group and sits
// at staged position (wave + (e / GE) * NW) * GE + e % GE, the place the whole-workgroup form gives it.
// Lane l takes elements l, l + 64, ...; the first XP indices per lane are fetched before the weight stream.
// Loads and LDS writes are unconditional: positions past the end read a clamped index and land in the dump slot.
template <typename WT, int BW, int NW, int TPL, int XP, bool VEC4 = false>
struct XStageWave {
    static constexpr int GE = TPL * BW;
    static constexpr bool kVec = VEC4 && !(PIVOT_ABLATE & 32) && XP % 4 == 0;
    int src[XP];
    static __device__ __forceinline__ int pos_of(int e, int wave) {
        const int q = e / GE;
        return (wave + q * NW) * GE + (e - q * GE);
    }
    // Which of the wavefront's elements lane l takes in slot k of a round.  Vector form (VEC4): four consecutive
    // ones per group of four slots, so that their indices are one 16-byte load and their staged values one LDS
    // store (a 4-byte load per lane occupies the memory pipeline as long as a 16-byte one; the layer kernel gains
    // 0.03-0.15 us warm on every workload, 4096x9216 fp32 3.45 -> 3.34 us, and 0.02-0.05 us cold; the chain
    // kernel lost 0.1-0.2 us cold with it and keeps the scalar form); else l, l + 64, ...
    static __device__ __forceinline__ int elem_of(int lane, int k) {
        return kVec ? ((k >> 2) * 64 + lane) * 4 + (k & 3) : lane + k * 64;
    }
    // the source index of staged element p of the work item (ablation 32: `xidx` is the tile list's block columns)
    static __device__ __forceinline__ int index_at(const int32_t* xidx, int tile_begin, int p) {
        if constexpr ((PIVOT_ABLATE & 32) != 0) return xidx[tile_begin + p / BW] * BW + p % BW;
        else return xidx[(size_t)tile_begin * BW + p];
    }
    // the indices of one round into s[]: clamped, unconditional loads (positions past the end read the last
    // entries; index arrays carry 16 bytes of padding, so entries 0..3 are readable even for an empty item)
    static __device__ __forceinline__ void round_idx(const int32_t* xidx, int tile_begin, int ne, int wave, int lane,
                                                     int e0, int (&s)[XP]) {
        if constexpr (kVec) {
            const int32_t* xi = xidx + (size_t)tile_begin * BW;
            const int last = ne >= 4 ? ne - 4 : 0;
            #pragma unroll
            for (int q = 0; q < XP / 4; ++q) {
                const int pos = pos_of(e0 + elem_of(lane, 4 * q), wave);       // a multiple of 4: GE is one
                const int4 v = *reinterpret_cast<const int4*>(xi + (pos < last ? pos : last));
                s[4 * q] = v.x; s[4 * q + 1] = v.y; s[4 * q + 2] = v.z; s[4 * q + 3] = v.w;
            }
        } else {
            const int emax = ne > 0 ? ne - 1 : 0;
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                const int pos = pos_of(e0 + elem_of(lane, k), wave);
                s[k] = index_at(xidx, tile_begin, pos < emax ? pos : emax);
            }
        }
    }
    // the values of one round into LDS (padding columns as zero; positions past the end into the dump slots, the
    // last four elements of the 16 bytes behind the staged row)
    static __device__ __forceinline__ void round_store(WT* xs, int xs_stride, int ne, int wave, int lane, int e0,
                                                       const int (&s)[XP], const WT (&v)[XP]) {
        if constexpr (kVec) {
            typedef WT vec4 __attribute__((ext_vector_type(4)));
            #pragma unroll
            for (int q = 0; q < XP / 4; ++q) {
                const int pos = pos_of(e0 + elem_of(lane, 4 * q), wave);
                vec4 o;
                #pragma unroll
                for (int c = 0; c < 4; ++c) o[c] = (s[4 * q + c] >= 0) ? v[4 * q + c] : WT(0);
                *reinterpret_cast<vec4*>(xs + (pos < ne ? pos : xs_stride - 4)) = o;
            }
        } else {
            const int dump = xs_stride - 1;
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                const int pos = pos_of(e0 + elem_of(lane, k), wave);
                xs[pos < ne ? pos : dump] = (s[k] >= 0) ? v[k] : WT(0);
            }
        }
    }
    __device__ __forceinline__ void load_idx(const int32_t* xidx, int tile_begin, int ne, int wave, int lane) {
        round_idx(xidx, tile_begin, ne, wave, lane, 0, src);
    }
    // `x`: the row of x, in global memory or (SRC_LDS) its copy in LDS
    template <bool SRC_LDS>
    __device__ __forceinline__ void gather(const int32_t* xidx, const WT* x, WT* xs, int xs_stride,
                                           int tile_begin, int ne, int wave, int lane) {
        WT v[XP];
        #pragma unroll
        for (int k = 0; k < XP; ++k) v[k] = x[src[k] > 0 ? src[k] : 0];
        round_store(xs, xs_stride, ne, wave, lane, 0, src, v);
        // longer work items: further rounds of XP elements per lane (the condition is the same in every lane)
        for (int e0 = XP * 64; pos_of(e0, wave) < ne; e0 += XP * 64) {
            int s2[XP];
            round_idx(xidx, tile_begin, ne, wave, lane, e0, s2);
            WT v2[XP];
            #pragma unroll
            for (int k = 0; k < XP; ++k) v2[k] = x[s2[k] > 0 ? s2[k] : 0];
            round_store(xs, xs_stride, ne, wave, lane, e0, s2, v2);
        }
    }
};

// The whole of x copied into LDS with coalesced 16-byte loads that depend on
// nothing (x-resident variant): issued first, together with the gather
// indices, so that both arrive after ONE trip to memory and the gather itself
// runs LDS to LDS.  Without it the gather is a chain of two dependent trips
// (index, then x[index]) whose second leg queues behind the weight stream.
// A thread holds up to XN vectors; the launcher only picks this variant when
// NB rows of x fit (NB * xn_vecs <= XN * NT) and rows are 16-byte aligned.
// Slots past the end are switched off lane by lane.
template <typename WT, int NB, int NT, int XN = 8>
struct XRes {
    using V = typename Elem<WT>::vec;
    static constexpr int VEC = Elem<WT>::VEC;
    V v[XN];
    __device__ __forceinline__ void load(int batch, long long ldx, int xn_vecs, const void* x, int b0, int tid) {
        const int total = NB * xn_vecs;
        #pragma unroll
        for (int j = 0; j < XN; ++j) {
            // Lanes past the end load nothing: a 16-byte load per lane occupies the compute unit's memory
            // pipeline for 16 clocks per wavefront, needed or not (4096x9216 fp32, where 5 of the 8 slots are
            // used: 3.64 -> 3.47 us warm; 4096x4096 fp16 dense, 1 of 8: 9.4 -> 9.0 us cold).  Predicated per
            // lane, not skipped by a uniform branch around the slot: the branches cost 0.1 us cold.
            const int id = tid + j * NT;
            const int b = (NB == 1) ? 0 : id / xn_vecs;
            const int i = (NB == 1) ? id : id - b * xn_vecs;
            const bool ok = id < total && (b0 + b) < batch;
            const WT* row = reinterpret_cast<const WT*>(x) + (long long)(ok ? b0 + b : 0) * ldx;
            if (ok) v[j] = load16<V>(row + (size_t)i * VEC);
        }
    }
    __device__ __forceinline__ void store(int batch, int xn_vecs, WT* xn, int b0, int tid) {
        const int total = NB * xn_vecs;
        const int xn_stride = xn_vecs * VEC;
        #pragma unroll
        for (int j = 0; j < XN; ++j) {
            const int id = tid + j * NT;
            const int b = (NB == 1) ? 0 : id / xn_vecs;
            const int i = (NB == 1) ? id : id - b * xn_vecs;
            const bool ok = id < total && (b0 + b) < batch;
            if (ok) *reinterpret_cast<V*>(xn + b * xn_stride + i * VEC) = v[j];
        }
    }
};

// The work item's descriptor: loaded from the schedule, or computed when the
// schedule is uniform (balanced pruning: every block row keeps the same
// number of tiles), which takes one dependent load off the critical path.
struct Chunk { int br, tile_begin, ntiles, slot, first, nparts; };
__device__ __forceinline__ Chunk load_chunk(int uniform_ct, int uniform_parts, const int4* chunks, const int32_t* part_base) {
    Chunk c;
    if (uniform_ct > 0) {
        c.br = blockIdx.x / uniform_parts;
        c.tile_begin = blockIdx.x * uniform_ct;
        c.ntiles = uniform_ct;
        c.slot = blockIdx.x;
        c.first = c.br * uniform_parts;
        c.nparts = uniform_parts;
    } else {
        // device copy of the schedule: eight ints per chunk (block_row, tile_begin, tile_end, slot, first slot of
        // the block row, its number of pieces, 0, 0), so that the descriptor is ONE dependent load
        const int4 cd = chunks[2 * blockIdx.x];
        const int4 ce = chunks[2 * blockIdx.x + 1];
        c.br = cd.x; c.tile_begin = cd.y; c.ntiles = cd.z - cd.y; c.slot = cd.w;
        c.first = ce.x;
        c.nparts = ce.y;
        (void)part_base;
    }
    return c;
}

// Everything after the per-wave sums are in LDS `red[w*N + idx]`, idx = j*BH + r
// (j = batch column of this launch tile, r = row inside the row slice):
// hand-over between the chunks of a split block row (Section 4.1.5: tiles that
// share rows need one more reduction), bias, activation, store through P_row.
template <int BH, int NBT, int NT>
__device__ __forceinline__ void finish_rows(const FcArgs& a, const float* red, int nred, int br, int slot,
                                            int first, int nparts, const RowPre<BH, BH * NBT, NT>& rp,
                                            int b0, int tid, int* s_flag) {
    constexpr int N = BH * NBT;
    const int gy = blockIdx.y, slice = blockIdx.z, SL = gridDim.z;
    if (nparts > 1) {
        float* mine = a.partials + (((size_t)gy * a.nchunks + slot) * SL + slice) * N;
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
            // one counter per 256-byte line: counters of different rows never share a line
            uint32_t* tk = a.tickets + (((size_t)gy * a.nbr + br) * SL + slice) * kTicketStride;
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
            const float* p = a.partials + (((size_t)gy * a.nchunks + first) * SL + slice) * N + idx;
            for (int q = 0; q < nparts; ++q) s += agent_load(p + (size_t)q * SL * N);
        } else {
            for (int w = 0; w < nred; ++w) s += red[w * N + idx];
        }
        const float v = apply_act(s + rp.bias[k], a.act);
        if ((PIVOT_ABLATE & 8) && !(v == 12345.678f)) continue;      // ablation: computed, never stored
        if (rp.dst[k] >= 0) store_out(a.y, (long long)(b0 + j) * a.ldy + rp.dst[k], v, a.out_f16);
    }
}

// ---------------------------------------------------------------------------
// batch 1..4: vector-ALU kernel.  BH is the height of the row slice.  Lane l
// of a wave reads bytes [16 l, 16 l+16) of each 1 KB piece of the slice's tile
// stream, i.e. VEC columns of one tile row; LPR lanes cover a row, a wave
// covers RPW rows per load.
// ---------------------------------------------------------------------------
// XR: 0 = gather from global x; 1 = gather from an LDS copy of x; 2 = the same for irregular schedules, with
// the copy requested before the work item's descriptor has arrived (it depends on nothing); 3 = as 2 with up
// to 16 vectors of x per thread (long inputs, LDS beyond 64 KB: a gather of single elements from a long x
// moves a whole cache line per element, the copy moves every line once).
template <typename WT, int BH, int BW, int NB, int NW, int XR>
__global__ void __launch_bounds__(NW * 64) fc_gemv_kernel(PIVOT_GEMV_PARAMS, FcArgs a) {
    using V = typename Elem<WT>::vec;
    constexpr int VEC = Elem<WT>::VEC;
    constexpr int NT  = NW * 64;
    constexpr int LPR = BW / VEC;                       // lanes per tile row
    constexpr int RPW = 64 / LPR;                       // tile rows per wave-load
    constexpr int NL  = (BH >= RPW) ? BH / RPW : 1;     // wave-loads per tile
    constexpr int TPL = (BH >= RPW) ? 1 : RPW / BH;     // tiles per wave-load: a slice shorter than a wave-load takes
                                                        // the same rows of TPL consecutive tiles (BH*BW*es contiguous bytes each)
    constexpr int U   = (NL >= 8) ? 1 : 8 / NL;         // groups in flight per wave
    constexpr int N   = BH * NB;
    static_assert(BW >= VEC && LPR <= 64, "tile width not supported");

    extern __shared__ __align__(16) char smem[];
    __shared__ int s_flag;
    // LDS: [x-resident copy of x: NB rows + a dump vector][staged x-segments]; the sums reuse it afterwards
    WT* xn = reinterpret_cast<WT*>(smem);
    WT* xs = XR ? xn + NB * (int)((unsigned)q_misc >> 14) * VEC + VEC : xn;
    float* red = reinterpret_cast<float*>(smem);        // reused after the stream phase

    PIVOT_STAMP_DECL;
    PIVOT_STAMP(0);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b0 = blockIdx.y * NB, slice = blockIdx.z;
    // only the preloaded arguments are used up to the point where the weight stream has been issued
    const int q_uniform_parts = q_ct_parts >> 16, q_uniform_ct = q_uniform_parts > 0 ? (q_ct_parts & 0xFFFF) : 0;
    const int q_bh_full = q_misc & 0x7F, q_batch = (q_misc >> 7) & 0x7F, q_xn_vecs = (int)((unsigned)q_misc >> 14);
    const int q_xs_stride = (q_ct_parts & 0xFFFF) * BW + VEC;
    // one batch row: row 0 only; the LDS-copy forms are only launched on densely packed rows of x (row stride =
    // row length), so that the copy can be requested without waiting for the rest of the argument block
    const long long q_ldx = (NB == 1) ? 0 : (XR != 0) ? (long long)q_xn_vecs * VEC : a.ldx;
    // order of issue = order of arrival: (x,) gather indices, then the weights, then the epilogue operands
    XRes<WT, NB, NT, (XR == 3) ? 16 : 8> xres;
    constexpr bool kLoadX = !(PIVOT_ABLATE & (1 | 4)), kStageX = !(PIVOT_ABLATE & (1 | 2));
    if constexpr (XR >= 2 && kLoadX) xres.load(q_batch, q_ldx, q_xn_vecs, p_x, b0, tid);
    const Chunk ck = load_chunk(q_uniform_ct, q_uniform_parts, p_chunks, a.part_base);
    const int br = ck.br, tile_begin = ck.tile_begin, ntiles = ck.ntiles, slot = ck.slot;
    const int first = ck.first, nparts = ck.nparts;
    const int ngroups = (ntiles + TPL - 1) / TPL;
    const int row0 = br * q_bh_full + slice * BH;
    const int tile_elems = q_bh_full * BW;

    if constexpr (XR == 1 && kLoadX) xres.load(q_batch, q_ldx, q_xn_vecs, p_x, b0, tid);
    constexpr int XPF = (XR == 3) ? 8 : 4;              // long inputs come with long work items: 8 indices up front
    XStage<WT, BW, NB, NT, XPF> xst;                    // several batch rows: staged by the whole workgroup
    XStageWave<WT, BW, NW, TPL, XPF, true> xsw;         // one batch row: every wavefront stages for itself
    if constexpr (!kStageX) { /* ablation: no gather index */ }
    else if constexpr (NB == 1) xsw.load_idx(p_idx, tile_begin, ntiles * BW, wave, lane);
    else                        xst.load_idx(p_idx, tile_begin, ntiles * BW, tid);

    const int s  = lane / LPR;                          // row within the wave-load
    const int cg = lane % LPR;                          // column group
    const int ts = (TPL > 1) ? s / BH : 0;              // tile within the group
    const size_t gstride = (size_t)TPL * tile_elems;    // elements between groups of tiles
    const int lane_off = (TPL > 1) ? ts * tile_elems + (s % BH) * BW + cg * VEC : lane * VEC;
    const WT* vbase = reinterpret_cast<const WT*>(p_vals) + (size_t)tile_begin * tile_elems
                      + (size_t)slice * BH * BW + lane_off;

    // Loads are unconditional (group index clamped; the value array is padded by
    // one group of zeros, so even an empty chunk reads valid memory): no branch
    // sits between the loads and the compiler can wait for exactly the ones it needs (skipping the duplicates
    // of the last group with a wave-uniform branch was measured: 4096x9216 fp32 5.3 -> 5.8 us cold, 4096x4096
    // fp16 at 25-100 % kept 0.6-0.9 us slower; only the chain kernel's short later layers gain from it).
    const int gmax = ngroups > 0 ? ngroups - 1 : 0;
    V w[U][NL];
    auto issue = [&](int g0, int u0, int u1) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            if (u < u0 || u >= u1) continue;
            const int g = g0 + u * NW;
            const int gc = g < gmax ? g : gmax;
            #pragma unroll
            for (int j = 0; j < NL; ++j) w[u][j] = load16<V>(vbase + gc * gstride + j * 64 * VEC);
        }
    };
    // The forms that request the copy of x first (XR >= 2) put it into LDS after HALF of the first weight loads
    // have been issued and issue the other half behind that: issuing a wave's loads takes over a microsecond
    // (the memory pipeline takes 64 bytes per clock from the whole compute unit), and x, requested first, is
    // back long before; the regular form keeps everything in one burst (measured: config 4 layer 1 10.3 ->
    // 9.95 us, config 3 dense 9.4 -> 9.3 us cold; the regular form on config 2 would lose 0.06 us).
    constexpr int UH = (XR >= 2 && U >= 2) ? U / 2 : U;
    issue(wave, 0, UH);
    if constexpr (UH < U) {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kLoadX) xres.store(q_batch, q_xn_vecs, xn, b0, tid);
        __builtin_amdgcn_sched_barrier(0);
        issue(wave, UH, U);
    }
    RowPre<BH, N, NT> rp;
    rp.load(p_bias, p_scatter, row0, tid);
    // every load above is issued before anything below waits for one of them
    __builtin_amdgcn_sched_barrier(0);
    PIVOT_STAMP(1);
    if constexpr (XR != 0) {
        if constexpr (UH == U && kLoadX) xres.store(q_batch, q_xn_vecs, xn, b0, tid);
        PIVOT_STAMP(2);
        if constexpr (kStageX) lds_barrier();
        PIVOT_STAMP(3);
        if constexpr (!kStageX) { /* ablation: nothing staged */ }
        else if constexpr (NB == 1) xsw.template gather<true>(p_idx, xn, xs, q_xs_stride, tile_begin, ntiles * BW, wave, lane);
        else xst.template gather<true>(q_batch, q_ldx, q_xn_vecs * VEC, q_xs_stride, p_idx, xn, xs, tile_begin, ntiles * BW, b0, tid);
    } else {
        if constexpr (!kStageX) { /* ablation: nothing staged */ }
        else if constexpr (NB == 1) xsw.template gather<false>(p_idx, reinterpret_cast<const WT*>(p_x), xs, q_xs_stride, tile_begin, ntiles * BW, wave, lane);
        else xst.template gather<false>(q_batch, q_ldx, 0, q_xs_stride, p_idx, reinterpret_cast<const WT*>(p_x), xs, tile_begin, ntiles * BW, b0, tid);
    }
    // what a wavefront staged for itself only it reads: LDS operations of one wavefront complete in order
    if constexpr (NB == 1) wave_lds_sync();
    else                   lds_barrier();
    PIVOT_STAMP(4);

    float acc[NL][NB];
    #pragma unroll
    for (int j = 0; j < NL; ++j)
        #pragma unroll
        for (int b = 0; b < NB; ++b) acc[j][b] = 0.f;

    auto consume = [&](int u, int g) {
        const int tl = g * TPL + ts;
        #pragma unroll
        for (int b = 0; b < NB; ++b) {
            const V xv = *reinterpret_cast<const V*>(xs + b * q_xs_stride + tl * BW + cg * VEC);
            #pragma unroll
            for (int j = 0; j < NL; ++j) acc[j][b] = dot_vec(w[u][j], xv, acc[j][b]);
        }
    };
    // All rounds but the last: every group is complete, and each register slot is
    // refilled as soon as it has been consumed, so the wave keeps its 8 loads in
    // flight instead of draining them once per round.
    int g0 = wave;
    for (; g0 + NW * U < ngroups; g0 += NW * U) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + u * NW;
            consume(u, g);
            const int gn = g + NW * U;
            const int gc = gn < gmax ? gn : gmax;
            #pragma unroll
            for (int j = 0; j < NL; ++j) w[u][j] = load16<V>(vbase + gc * gstride + j * 64 * VEC);
        }
    }
    // last round: may be partial
    #pragma unroll
    for (int u = 0; u < U; ++u) {
        const int g = g0 + u * NW;
        if (g < ngroups && g * TPL + ts < ntiles) consume(u, g);
    }

    PIVOT_STAMP(5);
    if constexpr (PIVOT_ABLATE & 16) {                  // ablation: one value per workgroup instead of the outputs
        float t = rp.bias[0] + (float)rp.dst[0];
        #pragma unroll
        for (int j = 0; j < NL; ++j)
            #pragma unroll
            for (int b = 0; b < NB; ++b) t += acc[j][b];
        if (tid == 0) reinterpret_cast<float*>(a.y)[0] = t;
        return;
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
    PIVOT_STAMP(6);
    finish_rows<BH, NB, NT>(a, red, NW, br, slot, first, nparts, rp, b0, tid, &s_flag);
#ifdef PIVOT_TRACE
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // the stamp is taken when the stores have been acknowledged
#endif
    PIVOT_STAMP(7);
    PIVOT_STAMP_FLUSH(a, NW, wave, lane);
}

// ---------------------------------------------------------------------------
// batch >= 8, fp16 weights: matrix-core kernels.  The tile is the A operand,
// the x-segment (k x batch) the B operand, accumulation in fp32.  x must be in
// block order already ([batch][K_pad], produced by the previous layer's store,
// by the recurrent cell, or by gather_x_kernel): lane l reads its B fragment,
// 8 consecutive k of one batch row, with one 16-byte load, no LDS staging.
// KIND 0: v_mfma_f32_16x16x32_f16, slices with BH % 16 == 0, BW % 32 == 0, 16 batch columns.
//         lane l supplies A[row l%16][k 8(l/16)..+7] = 16 contiguous bytes of a BRC tile row.
// KIND 1: v_mfma_f32_32x32x16_f16, slices with BH % 32 == 0, BW % 16 == 0, 32 batch columns.
//         lane l supplies A[row l%32][k 8(l/32)..+7].
// Batch columns past `batch` read row batch-1 again; their results are never stored.
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
// KIND 2 (LDS-fed kernel only): v_mfma_f32_16x16x32_f16 over PAIRS of consecutive 16-column tiles of a block
// row, so that tiles 16 columns wide can still be cut into 16-row slices: lanes with k group 0-1 supply rows of
// the pair's first tile, groups 2-3 of its second (each tile's slice is 512 contiguous bytes); the staged
// x-segments of consecutive tiles are adjacent in LDS, so the B fragment is the same single 16-byte read.
template <> struct Mfma<2> : Mfma<0> {};

template <int KIND, int BH, int BW, int NW>
__global__ void __launch_bounds__(NW * 64) fc_mfma_kernel(PIVOT_LEAD_PARAMS, FcArgs a) {
    using MF = Mfma<KIND>;
    using acc_t = typename MF::acc_t;
    constexpr int MR = MF::MR, MK = MF::MK, NBT = MF::NBT, CV = MF::CV;
    constexpr int NT = NW * 64;
    constexpr int RB = BH / MR;                         // row blocks per tile slice
    constexpr int KS = BW / MK;                         // k steps per tile
    constexpr int LT = RB * KS;                         // 16-byte weight loads per lane per tile
    constexpr int U  = (LT >= 8) ? 1 : 8 / LT;          // tiles in flight per wave
    constexpr int N  = BH * NBT;
    constexpr int RW = NW < 4 ? NW : 4;                 // waves that hold the sums at the end
    static_assert(BH % MR == 0 && BW % MK == 0, "tile shape does not fit this MFMA");

    extern __shared__ __align__(16) char smem[];
    __shared__ int s_flag;
    float* red = reinterpret_cast<float*>(smem);        // RW * N floats

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b0 = blockIdx.y * NBT, slice = blockIdx.z;
    const Chunk ck = load_chunk(a.uniform_ct, a.uniform_parts, p_chunks, p_part_base);
    const int br = ck.br, tile_begin = ck.tile_begin, ntiles = ck.ntiles, slot = ck.slot;
    const int first = ck.first, nparts = ck.nparts;
    const int row0 = br * a.bh_full + slice * BH;

    RowPre<BH, N, NT> rp;
    rp.load(p_bias, p_scatter, row0, tid);

    const int li = lane % MR;                           // A row / B column of this lane
    const int lg = lane / MR;                           // k group of 8
    const _Float16* vbase = reinterpret_cast<const _Float16*>(p_vals) + (size_t)tile_begin * a.tile_elems
                            + (size_t)slice * BH * BW + li * BW + lg * 8;
    const int brow = (b0 + li < a.batch) ? b0 + li : a.batch - 1;
    const _Float16* xb = reinterpret_cast<const _Float16*>(p_x) + (long long)brow * a.ldx + lg * 8;
    const int32_t* ci_base = p_idx + tile_begin;    // wave-uniform: scalar loads, their own counter

    const int tmax = ntiles > 0 ? ntiles - 1 : 0;       // clamped, unconditional loads (see fc_gemv_kernel)
    f16x8 w[U][LT];
    f16x8 xv[U][KS];
    auto issue = [&](int t0) {
        int ci[U];
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * NW;
            ci[u] = ci_base[t < tmax ? t : tmax];
        }
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * NW;
            const int tc = t < tmax ? t : tmax;
            #pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                #pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    w[u][rb * KS + ks] = load16<f16x8>(vbase + (size_t)tc * a.tile_elems + rb * MR * BW + ks * MK);
        }
        #pragma unroll
        for (int u = 0; u < U; ++u)
            #pragma unroll
            for (int ks = 0; ks < KS; ++ks) xv[u][ks] = load16<f16x8>(xb + (size_t)ci[u] * BW + ks * MK);
    };

    acc_t acc[RB];
    #pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = acc_t(0);

    // One tile's loads: block column (scalar), A fragments, B fragments.
    auto fill = [&](int u, int t) {
        const int tc = t < tmax ? t : tmax;
        const int ci = ci_base[tc];
        #pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            #pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                w[u][rb * KS + ks] = load16<f16x8>(vbase + (size_t)tc * a.tile_elems + rb * MR * BW + ks * MK);
        #pragma unroll
        for (int ks = 0; ks < KS; ++ks) xv[u][ks] = load16<f16x8>(xb + (size_t)ci * BW + ks * MK);
    };
    auto consume = [&](int u) {
        #pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            #pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[rb] = MF::run(w[u][rb * KS + ks], xv[u][ks], acc[rb]);
    };

    issue(wave);
    // all rounds but the last: consume a slot and refill it at once (loads stay in flight)
    int t0 = wave;
    for (; t0 + NW * U < ntiles; t0 += NW * U) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            consume(u);
            fill(u, t0 + u * NW + NW * U);
        }
    }
    #pragma unroll
    for (int u = 0; u < U; ++u)
        if (t0 + u * NW < ntiles) consume(u);

    // waves -> one sum: rounds of (up to) 4 writers into a 4-slot LDS buffer
    auto put = [&](int w_slot) {
        #pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            #pragma unroll
            for (int v = 0; v < CV; ++v)
                red[w_slot * N + li * BH + rb * MR + MF::row_of(lane, v)] = acc[rb][v];
    };
    #pragma unroll
    for (int base = RW; base < NW; base += RW) {
        if (wave >= base && wave < base + RW) put(wave - base);
        __syncthreads();
        if (wave < RW) {
            #pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                #pragma unroll
                for (int v = 0; v < CV; ++v)
                    acc[rb][v] += red[wave * N + li * BH + rb * MR + MF::row_of(lane, v)];
        }
        __syncthreads();
    }
    if (wave < RW) put(wave);
    __syncthreads();
    finish_rows<BH, NBT, NT>(a, red, RW, br, slot, first, nparts, rp, b0, tid, &s_flag);
}

// ---------------------------------------------------------------------------
// batch 3..16, fp16 weights: matrix cores fed from LDS.  With several batch
// rows the vector kernel is bound by LDS (every 16-byte weight load needs one
// 16-byte LDS read per batch row); here a tile slice is the MFMA A operand and
// ONE 16-byte LDS read per lane supplies the B fragment for all batch rows.
// Prologue and epilogue are the vector kernel's (preloaded arguments only, the
// whole of x copied first where it fits, gather into LDS xs[b][tile*BW + c]
// for b < NBS); lane l reads B[k 8(l/MR)..+7][column l%MR] = xs[l%MR][...].
// Lanes whose column is past NBS read row 0; their accumulator columns are
// never stored.
// ---------------------------------------------------------------------------
template <int KIND, int BH, int BW, int NBS, int NW, int XR>
__global__ void __launch_bounds__(NW * 64) fc_mfma_lds_kernel(PIVOT_GEMV_PARAMS, FcArgs a) {
    using MF = Mfma<KIND>;
    using acc_t = typename MF::acc_t;
    using WT = _Float16;
    constexpr int VEC = 8;
    constexpr int MR = MF::MR, MK = MF::MK, CV = MF::CV;
    constexpr bool PAIR = (KIND == 2);                  // one MFMA step spans two consecutive tiles
    constexpr int NT = NW * 64;
    constexpr int RB = BH / MR;                         // row blocks per tile slice
    constexpr int KS = PAIR ? 1 : BW / MK;              // k steps per tile (pair)
    constexpr int LT = RB * KS;                         // 16-byte weight loads per lane per tile (pair)
    constexpr int U  = (LT >= 8) ? 1 : 8 / LT;          // tiles (pairs) in flight per wave
    constexpr int N  = BH * NBS;
    constexpr int XPAD = PAIR ? BW : 0;                 // zeroed columns after the last staged tile (odd tile count)
    static_assert(BH % MR == 0 && (PAIR ? BW * 2 == MK : BW % MK == 0), "tile shape does not fit this MFMA");
    static_assert(NBS <= MR, "more staged batch rows than MFMA columns");

    extern __shared__ __align__(16) char smem[];
    __shared__ int s_flag;
    const int q_uniform_parts = q_ct_parts >> 16, q_uniform_ct = q_uniform_parts > 0 ? (q_ct_parts & 0xFFFF) : 0;
    const int q_bh_full = q_misc & 0x7F, q_batch = (q_misc >> 7) & 0x7F, q_xn_vecs = (int)((unsigned)q_misc >> 14);
    const int q_xs_stride = (q_ct_parts & 0xFFFF) * BW + XPAD + VEC;
    WT* xn = reinterpret_cast<WT*>(smem);
    WT* xs = XR ? xn + NBS * q_xn_vecs * VEC + VEC : xn;
    float* red = reinterpret_cast<float*>(smem);        // reused after the stream phase: NW * N floats

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b0 = blockIdx.y * NBS, slice = blockIdx.z;
    const long long q_ldx = (XR != 0) ? (long long)q_xn_vecs * VEC : a.ldx;
    XRes<WT, NBS, NT> xres;
    if constexpr (XR != 0) xres.load(q_batch, q_ldx, q_xn_vecs, p_x, b0, tid);
    const Chunk ck = load_chunk(q_uniform_ct, q_uniform_parts, p_chunks, a.part_base);
    const int br = ck.br, tile_begin = ck.tile_begin, ntiles = ck.ntiles, slot = ck.slot;
    const int first = ck.first, nparts = ck.nparts;
    const int row0 = br * q_bh_full + slice * BH;
    const int tile_elems = q_bh_full * BW;

    XStage<WT, BW, NBS, NT, 4, true> xst;               // p_idx: the packed source-ordered gather lists
    xst.load_idx(p_idx, tile_begin, ntiles * BW, tid);

    const int li = lane % MR;                           // A row / B column of this lane
    const int lg = lane / MR;                           // k group of 8
    const _Float16* vbase = reinterpret_cast<const _Float16*>(p_vals) + (size_t)tile_begin * tile_elems
                            + (size_t)slice * BH * BW + li * BW + (PAIR ? (lg & 1) : lg) * 8;
    const int tmax = ntiles > 0 ? ntiles - 1 : 0;       // clamped, unconditional loads (see fc_gemv_kernel)
    const int nsteps = PAIR ? (ntiles + 1) / 2 : ntiles; // MFMA steps along the block row: tiles, or pairs of tiles
    f16x8 w[U][LT];
    auto fill = [&](int u, int t) {
        const int tt = PAIR ? 2 * t + (lg >> 1) : t;    // this lane's tile
        const int tc = tt < tmax ? tt : tmax;
        #pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            #pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                w[u][rb * KS + ks] = load16<f16x8>(vbase + (size_t)tc * tile_elems + rb * MR * BW + ks * MK);
                if (PAIR && tt >= ntiles) w[u][rb * KS + ks] = f16x8(0);   // the missing half of the last pair
            }
    };
    // with a copy of x: into LDS after half of the first weight loads, the other half behind it (see fc_gemv_kernel)
    constexpr int UH = (XR != 0 && U >= 2) ? U / 2 : U;
    #pragma unroll
    for (int u = 0; u < UH; ++u) fill(u, wave + u * NW);
    if constexpr (UH < U) {
        __builtin_amdgcn_sched_barrier(0);
        xres.store(q_batch, q_xn_vecs, xn, b0, tid);
        __builtin_amdgcn_sched_barrier(0);
        #pragma unroll
        for (int u = UH; u < U; ++u) fill(u, wave + u * NW);
    }

    RowPre<BH, N, NT> rp;
    rp.load(p_bias, p_scatter, row0, tid);
    __builtin_amdgcn_sched_barrier(0);                  // every load above is issued before anything below waits
    if constexpr (XR != 0) {
        if constexpr (UH == U) xres.store(q_batch, q_xn_vecs, xn, b0, tid);
        lds_barrier();
        xst.template gather<true>(q_batch, q_ldx, q_xn_vecs * VEC, q_xs_stride, p_idx, xn, xs, tile_begin, ntiles * BW, b0, tid);
    } else {
        xst.template gather<false>(q_batch, q_ldx, 0, q_xs_stride, p_idx, reinterpret_cast<const WT*>(p_x), xs, tile_begin, ntiles * BW, b0, tid);
    }
    if constexpr (PAIR) {
        // the columns a last, single tile's partner would have: zero weights meet zero inputs, never stale LDS
        if (tid < NBS * XPAD) xs[(tid / XPAD) * q_xs_stride + ntiles * BW + tid % XPAD] = WT(0);
    }
    lds_barrier();

    acc_t acc[RB];
    #pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = acc_t(0);
    const WT* xrow = xs + (li < NBS ? li : 0) * q_xs_stride + lg * 8;
    auto consume = [&](int u, int t) {
        #pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const f16x8 xv = *reinterpret_cast<const f16x8*>(xrow + t * (PAIR ? 2 * BW : BW) + ks * MK);
            #pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[rb] = MF::run(w[u][rb * KS + ks], xv, acc[rb]);
        }
    };
    int t0 = wave;
    for (; t0 + NW * U < nsteps; t0 += NW * U) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            consume(u, t0 + u * NW);
            fill(u, t0 + u * NW + NW * U);
        }
    }
    #pragma unroll
    for (int u = 0; u < U; ++u)
        if (t0 + u * NW < nsteps) consume(u, t0 + u * NW);

    // every wave's sums for the staged batch columns go to LDS; the epilogue adds the NW copies
    __syncthreads();                                    // xs no longer needed; red aliases it
    if (li < NBS) {
        #pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            #pragma unroll
            for (int v = 0; v < CV; ++v)
                red[wave * N + li * BH + rb * MR + MF::row_of(lane, v)] = acc[rb][v];
    }
    __syncthreads();
    finish_rows<BH, NBS, NT>(a, red, NW, br, slot, first, nparts, rp, b0, tid, &s_flag);
}

// ---------------------------------------------------------------------------
// batch 5..16, fp16 weights: matrix cores with the B fragments gathered from a
// copy of x in LDS (Listing 1: the group fetch through P_col, done where the
// fragment is formed).  Staging the x-segments of 16 batch rows element by
// element costs a work item more than streaming its weights (16 rows x tiles x
// BW two-byte loads and LDS writes, repeated by every row slice of the block
// row); here the 16 rows of x are copied into LDS whole, in natural order, with
// independent 16-byte loads, the item's gather indices are copied beside them
// as byte offsets, and the lane that supplies B[k 8g..8g+7][column n] reads
// its eight indices with two 16-byte LDS reads and its eight values with eight
// 2-byte LDS reads from row n.  Rows are 16 bytes apart from a power of two, so
// the sixteen lanes that read the same column of different rows hit different
// banks.  Index -1 (padding column) and the partner of a last, single tile
// of the paired form point at the zeroed 16 bytes behind the row.
// Needs 8 wavefronts (each copies two rows), at most 512 vectors per row and
// 8192 staged columns per work item; q_misc bit 31: rows are whole 16-byte
// vectors, 16-byte aligned and densely packed (else an element-wise copy).
// ---------------------------------------------------------------------------
template <int KIND, int BH, int BW>
__global__ void __launch_bounds__(512) fc_mfma_xrow_kernel(PIVOT_GEMV_PARAMS, FcArgs a) {
    using MF = Mfma<KIND>;
    using acc_t = typename MF::acc_t;
    using WT = _Float16;
    constexpr int NW = 8, NT = NW * 64, NBS = 16;
    constexpr int MR = MF::MR, MK = MF::MK, CV = MF::CV;
    constexpr bool PAIR = (KIND == 2);                  // one MFMA step spans two consecutive tiles
    constexpr int RB = BH / MR;                         // row blocks per tile slice
    constexpr int KS = PAIR ? 1 : BW / MK;              // k steps per tile (pair)
    constexpr int LT = RB * KS;                         // 16-byte weight loads per lane per tile (pair)
    constexpr int U  = (LT >= 8) ? 1 : 8 / LT;          // tiles (pairs) in flight per wave (16 KB: slower throughout)
    constexpr int N  = BH * NBS;
    constexpr int STEP = PAIR ? 2 * BW : BW;            // staged columns per MFMA step along the block row
    constexpr int XV = 8;                               // vectors of one row a lane copies (2 rows per wavefront)
    constexpr int IV = 4;                               // int4 of gather indices a thread copies
    static_assert(BH % MR == 0 && (PAIR ? BW * 2 == MK : BW % MK == 0), "tile shape does not fit this MFMA");

    extern __shared__ __align__(16) char smem[];
    __shared__ int s_flag;
    const int q_uniform_parts = q_ct_parts >> 16, q_uniform_ct = q_uniform_parts > 0 ? (q_ct_parts & 0xFFFF) : 0;
    const int q_bh_full = q_misc & 0x7F, q_batch = (q_misc >> 7) & 0x7F, q_xn_vecs = (q_misc >> 14) & 0x1FFFF;
    const bool q_vec_rows = q_misc < 0;
    const int row_bytes = q_xn_vecs * 16 + 16;          // a row of x and 16 zeroed bytes
    const int zero_off = q_xn_vecs * 16;
    int* xi_lds = reinterpret_cast<int*>(smem + NBS * row_bytes);
    float* red = reinterpret_cast<float*>(smem);        // reused after the stream phase: NW * N floats

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b0 = blockIdx.y * NBS, slice = blockIdx.z;

    // The copy of x, requested first: loads return in order, so behind the weights it would wait for their trip
    // to HBM (weights first: 0.6-0.9 us slower on 4096x4096 at every density; interleaved with them: 0.2-0.5 us
    // slower; twice the weights in flight: 0.6-1.0 us slower).  Wavefront w takes rows w and w + 8, lane l
    // vectors l, l + 64, ... of each.
    f16x8 xv_[2][XV];
    auto xload = [&](int k) {                           // k-th of the thread's 2 * XV vectors
        const int r = k / XV, j = k % XV;
        const int b = wave + r * NW;
        const f16x8* src = reinterpret_cast<const f16x8*>(p_x) + (long long)(b0 + b) * q_xn_vecs;
        const int i = lane + j * 64;
        if (i < q_xn_vecs && b0 + b < q_batch) xv_[r][j] = load16<f16x8>(reinterpret_cast<const WT*>(src + i));
    };
    if (q_vec_rows) {
        #pragma unroll
        for (int k = 0; k < 2 * XV; ++k) xload(k);
    }
    const Chunk ck = load_chunk(q_uniform_ct, q_uniform_parts, p_chunks, a.part_base);
    const int br = ck.br, tile_begin = ck.tile_begin, ntiles = ck.ntiles, slot = ck.slot;
    const int first = ck.first, nparts = ck.nparts;
    const int row0 = br * q_bh_full + slice * BH;
    const int tile_elems = q_bh_full * BW;
    const int nsteps = PAIR ? (ntiles + 1) / 2 : ntiles; // MFMA steps along the block row: tiles, or pairs of tiles
    const int ne = ntiles * BW, ne_pad = nsteps * STEP;

    // the item's gather indices (whole int4: a tile has at least 16 columns)
    const int4* xi4 = reinterpret_cast<const int4*>(p_idx + (size_t)tile_begin * BW);
    int4 iv[IV];
    #pragma unroll
    for (int j = 0; j < IV; ++j) {
        const int e4 = tid + j * NT;
        if (e4 * 4 < ne) iv[j] = xi4[e4];
    }

    const int li = lane % MR;                           // A row / B column of this lane
    const int lg = lane / MR;                           // k group of 8
    const _Float16* vbase = reinterpret_cast<const _Float16*>(p_vals) + (size_t)tile_begin * tile_elems
                            + (size_t)slice * BH * BW + li * BW + (PAIR ? (lg & 1) : lg) * 8;
    const int tmax = ntiles > 0 ? ntiles - 1 : 0;       // clamped, unconditional loads (see fc_gemv_kernel)
    f16x8 w[U][LT];
    auto fill = [&](int u, int t) {
        const int tt = PAIR ? 2 * t + (lg >> 1) : t;    // this lane's tile
        const int tc = tt < tmax ? tt : tmax;
        #pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            #pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                w[u][rb * KS + ks] = load16<f16x8>(vbase + (size_t)tc * tile_elems + rb * MR * BW + ks * MK);
                if (PAIR && tt >= ntiles) w[u][rb * KS + ks] = f16x8(0);   // the missing half of the last pair
            }
    };
    #pragma unroll
    for (int u = 0; u < U; ++u) fill(u, wave + u * NW);

    RowPre<BH, N, NT> rp;
    rp.load(p_bias, p_scatter, row0, tid);
    __builtin_amdgcn_sched_barrier(0);                  // every load above is issued before anything below waits

    // x and the indices into LDS (they were requested first, so they arrive first)
    if (q_vec_rows) {
        #pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int b = wave + r * NW;
            #pragma unroll
            for (int j = 0; j < XV; ++j) {
                const int i = lane + j * 64;
                if (i < q_xn_vecs && b0 + b < q_batch) *reinterpret_cast<f16x8*>(smem + b * row_bytes + i * 16) = xv_[r][j];
            }
        }
    } else {
        // rows that are not whole aligned vectors: element by element (a.xn_stride = elements per row)
        const WT* x = reinterpret_cast<const WT*>(p_x);
        for (int b = wave; b < NBS; b += NW) {
            if (b0 + b >= q_batch) continue;
            for (int c = lane; c < a.xn_stride; c += 64)
                *reinterpret_cast<WT*>(smem + b * row_bytes + c * 2) = x[(long long)(b0 + b) * a.ldx + c];
        }
    }
    if (tid < NBS * 4) *reinterpret_cast<int*>(smem + (tid >> 2) * row_bytes + zero_off + (tid & 3) * 4) = 0;
    #pragma unroll
    for (int j = 0; j < IV; ++j) {
        const int e4 = tid + j * NT;
        if (e4 * 4 < ne) {
            int4 o;
            o.x = iv[j].x >= 0 ? iv[j].x * 2 : zero_off; o.y = iv[j].y >= 0 ? iv[j].y * 2 : zero_off;
            o.z = iv[j].z >= 0 ? iv[j].z * 2 : zero_off; o.w = iv[j].w >= 0 ? iv[j].w * 2 : zero_off;
            *reinterpret_cast<int4*>(xi_lds + e4 * 4) = o;
        }
    }
    if (tid < ne_pad - ne) xi_lds[ne + tid] = zero_off;    // (paired form, odd tile count: BW <= NT entries)
    lds_barrier();

    acc_t acc[RB];
    #pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = acc_t(0);
    const char* xrow = smem + (li < NBS ? li : 0) * row_bytes;
    const int* xi_l = xi_lds + lg * 8;
    auto consume = [&](int u, int t) {
        #pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int4 i0 = *reinterpret_cast<const int4*>(xi_l + t * STEP + ks * MK);
            const int4 i1 = *reinterpret_cast<const int4*>(xi_l + t * STEP + ks * MK + 4);
            f16x8 xv;
            xv[0] = *reinterpret_cast<const WT*>(xrow + i0.x); xv[1] = *reinterpret_cast<const WT*>(xrow + i0.y);
            xv[2] = *reinterpret_cast<const WT*>(xrow + i0.z); xv[3] = *reinterpret_cast<const WT*>(xrow + i0.w);
            xv[4] = *reinterpret_cast<const WT*>(xrow + i1.x); xv[5] = *reinterpret_cast<const WT*>(xrow + i1.y);
            xv[6] = *reinterpret_cast<const WT*>(xrow + i1.z); xv[7] = *reinterpret_cast<const WT*>(xrow + i1.w);
            #pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[rb] = MF::run(w[u][rb * KS + ks], xv, acc[rb]);
        }
    };
    int t0 = wave;
    for (; t0 + NW * U < nsteps; t0 += NW * U) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            consume(u, t0 + u * NW);
            fill(u, t0 + u * NW + NW * U);
        }
    }
    #pragma unroll
    for (int u = 0; u < U; ++u)
        if (t0 + u * NW < nsteps) consume(u, t0 + u * NW);

    // every wave's sums for the staged batch columns go to LDS; the epilogue adds the NW copies
    __syncthreads();                                    // x no longer needed; red aliases it
    if (li < NBS) {
        #pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            #pragma unroll
            for (int v = 0; v < CV; ++v)
                red[wave * N + li * BH + rb * MR + MF::row_of(lane, v)] = acc[rb][v];
    }
    __syncthreads();
    finish_rows<BH, NBS, NT>(a, red, NW, br, slot, first, nparts, rp, b0, tid, &s_flag);
}

}  // namespace pivot
