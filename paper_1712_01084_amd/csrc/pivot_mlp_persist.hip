// A chain of pruned layers in ONE launch (Section 4.2: consecutive PBP layers
// whose boundary permutations are composed or eliminated).  With a launch per
// layer every boundary costs an empty-kernel turnaround plus a cold first trip
// to memory for the next layer's indices and weights.  Here workgroup g runs
// work item g of layer 0, then work item g of layer 1, and so on; the layers
// are ordered by the data itself: an intermediate activation is stored as the
// 8-byte pair (value, tag) with one device-coherent store, and the gather of
// the next layer re-reads the pairs it needs until all carry this launch's
// tag.  A workgroup requests the next layer's gather indices and weights
// before it starts waiting, so they arrive while the boundary is in flight.
//
// The tag is a launch counter kept per workgroup in device memory owned by
// the chain plan (word g is read and bumped by workgroup g alone, so every
// launch, also a replayed graph node, sees a value no earlier launch used);
// the pair buffers are owned by the plan too, hence launches of one chain plan
// must not overlap.  No fences, no atomics on floats, fixed summation order:
// results are bit-identical from run to run.  All workgroups must be resident
// at once (checked at plan time); every wait is bounded: after kSpinLimit
// polls it raises the status word, the wait ends, and the results of that
// launch are undefined.
//
// The per-layer body is the batch-1 vector kernel: 16-byte coalesced stream of
// BRC tile rows, x-segments staged in LDS, DPP lane reduction, LDS wave
// reduction, bias, activation, store through the composed boundary array.
// Restricted to BRC plans of one weight type with whole block rows per work
// item, batch 1; an fp16 chain rounds an intermediate to fp16 once, at the
// producer's store, as the launch-per-layer form does.
#include <cstdlib>

#include "pivot_fc_kernels.h"

namespace pivot {

namespace {

constexpr int kMaxChainLayers = 8;
constexpr int kChainNW = 8;                     // wavefronts per workgroup
constexpr int kChainMaxGrid = 1024;             // launch-counter words
constexpr int kChainStatus = 1024;              // index of the status word
constexpr uint32_t kChainSpinLimit = 1u << 18;
// LDS in front of the staged input: the wavefronts' partial sums, two slots used by a workgroup's items in turn.  With a
// slot of their own the sums need ONE workgroup barrier per item (all sums written -> the finishing wavefront
// reads them): a wavefront that is past it may stage the next layer's input and even write that layer's sums
// (other slot) while the finishing wavefront still reads this layer's; it reaches the slot after that only past
// the next item's barrier, which the finishing wavefront joins when it has read.
constexpr int kChainRedBytes = 2 * kChainNW * 64 * 4;

struct ChainLayer {
    const int4*    chunks;      // eight ints per chunk (irregular schedules)
    const int32_t* xidx;        // gather index of every kept tile's columns
    const void*    vals;        // tile values of the plans' weight type
    const float*   bias_p;
    const int32_t* dst;         // block-space row -> position in `out`, -1 = not stored
    const void*    in;          // layer 0: x (weight type) in natural order; later layers: pairs in this layer's block order
    void*          out;         // pairs in the next layer's block order; last layer: float y
    int nitems, slices, bhs, bh_full, uniform_ct, uniform_parts, chunk_tiles, act, k_valid;
    int xn_vecs;                // first layer, kInCopy: 16-byte vectors of x
};

struct ChainArgs {
    ChainLayer L[kMaxChainLayers];
    uint32_t*  ctl;             // [0, kChainMaxGrid): launch counter of every workgroup; [kChainStatus]: status
    int        nlayers;
    long long* trace;           // timeline builds only (PIVOT_TRACE): [layer][workgroup][wavefront][8] time stamps
};

// Timeline builds: per layer and wavefront, the 100 MHz clock at 0 item start, 1 every load issued, 2 own
// x-segments staged (tagged input: the pairs of its producers have arrived), 3 last weight consumed, 4 sums of
// all wavefronts in LDS, 5 outputs stored.
#ifdef PIVOT_TRACE
#define CHAIN_STAMP(i) do { __builtin_amdgcn_sched_barrier(0); ctr_[i] = wall_clock64(); __builtin_amdgcn_sched_barrier(0); } while (0)
#else
#define CHAIN_STAMP(i) do {} while (0)
#endif

__device__ __forceinline__ unsigned long long cld64(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void cst64(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t cld32(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void cst32(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A poll that did not succeed: pause; every 64th time look at the status word,
// and give up (raising it) at the limit.  Returns false when the wait must end.
__device__ __forceinline__ bool chain_keep_waiting(uint32_t* ctl, uint32_t& spins) {
    __builtin_amdgcn_s_sleep(4);
    if ((++spins & 63u) != 0u) return true;
    if (cld32(ctl + kChainStatus) != 0u) return false;
    if (spins >= kChainSpinLimit) { cst32(ctl + kChainStatus, 1u); return false; }
    return true;
}

// Reads the fields of a layer description from the argument block here, while the current layer's loads are in
// flight, so that they sit in the scalar cache when the next layer begins (fetched only where they are first
// used, at the start of that layer, they cost a trip of about 0.7 us with nothing else to do).
__device__ __forceinline__ void pin_layer(const ChainLayer& p) {
    asm volatile("" :: "s"(p.chunks), "s"(p.xidx), "s"(p.vals), "s"(p.bias_p), "s"(p.dst), "s"(p.in), "s"(p.out));
    asm volatile("" :: "s"(p.nitems), "s"(p.slices), "s"(p.bhs), "s"(p.bh_full), "s"(p.uniform_ct), "s"(p.uniform_parts),
                 "s"(p.chunk_tiles), "s"(p.act), "s"(p.k_valid), "s"(p.xn_vecs));
}

// One work item of one layer (see fc_gemv_kernel for the streaming scheme).
// No thread leaves early: every barrier is reached by the whole workgroup.
// XIN says where the layer's input comes from, at compile time (a run-time branch around the gather loads would
// make the compiler wait for every outstanding weight load before it issues them):
//   kInPlain  the caller's x, gathered element by element from global memory
//   kInCopy   the caller's x, first copied whole into LDS with coalesced 16-byte loads (up to 16 per thread) and
//             gathered from there: for a long x the element gather moves a whole cache line per element
//   kInTagged (value, tag) pairs of the previous layer, re-read until they carry this launch's tag
//             SHORT (a property of the whole chain, chosen by the launcher): no wavefront of any later layer
//             stages more than 64 elements, and a lane fetches ONE gather index and polls one pair per round
//             instead of four, three of which would be clamped and thrown away: a 4-byte load per lane occupies
//             the memory pipeline for as long as a 16-byte one, and at a boundary the issue of the item's first
//             loads is on the critical path (25088-4096-4096-1000: 15.6 -> 15.1-15.4 us cold, 13.05 -> 12.7
//             warm).  A template argument of the kernel, not one more case per layer: with four more
//             instantiations of the item inside one kernel the compiler copied the argument block to scratch.
// The first layer (usually the long one) fetches eight gather indices per thread up front, so that up to 4096
// staged elements need one round of dependent loads.
enum { kInPlain = 0, kInTagged = 1, kInCopy = 2 };
template <typename WT, int BH, int BW, int NW, int XIN, bool SHORT>
__device__ __forceinline__ void chain_item(const ChainLayer& P, int item, bool out_tagged,
                                           uint32_t tag, uint32_t counter, uint32_t* s_tag, uint32_t* ctl, char* smem,
                                           long long* trace, const ChainLayer& next, int red_slot) {
    using V = typename Elem<WT>::vec;
    constexpr int VEC = Elem<WT>::VEC;
    constexpr int NT  = NW * 64;
    constexpr int LPR = BW / VEC;
    constexpr int RPW = 64 / LPR;
    constexpr int NL  = (BH >= RPW) ? BH / RPW : 1;
    constexpr int TPL = (BH >= RPW) ? 1 : RPW / BH;
    constexpr int U   = (NL >= 8) ? 1 : 8 / NL;
    constexpr bool IN_TAGGED = (XIN == kInTagged);
    constexpr int XP  = IN_TAGGED ? (SHORT ? 1 : 4) : 8;
    static_assert(BH <= NT, "one thread per output row");

    // LDS: [partial sums, two slots][copy of x + a dump vector (kInCopy)][staged x-segments]
    WT* xn  = reinterpret_cast<WT*>(smem + kChainRedBytes);
    WT* xs  = (XIN == kInCopy) ? xn + (size_t)P.xn_vecs * VEC + VEC : xn;
    float* red = reinterpret_cast<float*>(smem) + red_slot * (NW * 64);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#ifdef PIVOT_TRACE
    long long ctr_[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#endif
    CHAIN_STAMP(0);
    XRes<WT, 1, NT, 16> xres;
    if constexpr (XIN == kInCopy) xres.load(1, 0, P.xn_vecs, P.in, 0, tid);
    const int chunk = item / P.slices, slice = item - chunk * P.slices;
    int br, tile_begin, ntiles;
    if (P.uniform_ct > 0) {
        br = chunk / P.uniform_parts; tile_begin = chunk * P.uniform_ct; ntiles = P.uniform_ct;
    } else {
        const int4 cd = P.chunks[2 * chunk];
        br = cd.x; tile_begin = cd.y; ntiles = cd.z - cd.y;
    }
    // Every wavefront stages the x-segments of its own groups of tiles only (see XStageWave): what it writes to
    // LDS only it reads, so no workgroup barrier stands between the staging and the first FMA, and with tagged
    // input a wavefront waits only for the producers of its own tiles.
    const int ne = ntiles * BW, emax = ne > 0 ? ne - 1 : 0;
    const int xs_stride = P.chunk_tiles * BW + VEC;     // LDS row: chunk_tiles*BW staged elements + 16 bytes (dump slot last)
    const int dump = xs_stride - 1;
    const int32_t* xi = P.xidx + (size_t)tile_begin * BW;
    using XSW = XStageWave<WT, BW, NW, TPL, XP>;
    XSW xsw;
    xsw.load_idx(P.xidx, tile_begin, ne, wave, lane);

    const int ngroups = (ntiles + TPL - 1) / TPL;
    const int gmax = ngroups > 0 ? ngroups - 1 : 0;
    const int tile_elems = P.bh_full * BW;
    const int s  = lane / LPR, cg = lane % LPR;
    const int ts = (TPL > 1) ? s / BH : 0;
    const size_t gstride = (size_t)TPL * tile_elems;
    const int lane_off = (TPL > 1) ? ts * tile_elems + (s % BH) * BW + cg * VEC : lane * VEC;
    const WT* vbase = reinterpret_cast<const WT*>(P.vals) + (size_t)tile_begin * tile_elems + (size_t)slice * BH * BW + lane_off;
    V w[U][NL];
    auto issue = [&](int u0, int u1) {
        #pragma unroll
        for (int u = 0; u < U; ++u) {
            if (u < u0 || u >= u1) continue;
            const int g = wave + u * NW;
            // later layers: no clamped duplicates of the last group (wave-uniform; whatever follows only consumes
            // groups that exist).  Their items are short, and the issue of an item's first loads is on the
            // critical path of a boundary (25088-4096-4096-1000: 15.2 -> 14.9 us cold).
            if (IN_TAGGED && g > gmax) continue;
            const int gc = g < gmax ? g : gmax;
            #pragma unroll
            for (int j = 0; j < NL; ++j) w[u][j] = load16<V>(vbase + gc * gstride + j * 64 * VEC);
        }
    };
    // with a copy of x: into LDS after half of the first weight loads, the other half behind it (see fc_gemv_kernel)
    constexpr int UH = (XIN == kInCopy && U >= 2) ? U / 2 : U;
    issue(0, UH);
    if constexpr (UH < U) {
        __builtin_amdgcn_sched_barrier(0);
        xres.store(1, P.xn_vecs, xn, 0, tid);
        __builtin_amdgcn_sched_barrier(0);
        issue(UH, U);
    }
    const int orow = br * P.bh_full + slice * BH + tid % BH;
    const float bias = P.bias_p[orow];
    const int   dst  = P.dst[orow];
    __builtin_amdgcn_sched_barrier(0);                  // every load above is issued before anything below waits
    pin_layer(next);                                    // the next layer's description: into the scalar cache
    CHAIN_STAMP(1);

    // stage the x-segments: plain loads from the caller's x, or pairs re-read until they carry this launch's tag.
    // The first round stands outside the loop so that no loop header sits between its loads and the ones above.
    if constexpr (XIN == kInCopy) {
        if constexpr (UH == U) xres.store(1, P.xn_vecs, xn, 0, tid);
        lds_barrier();
    }
    if constexpr (!IN_TAGGED) {
        if constexpr (XIN == kInCopy) xsw.template gather<true>(P.xidx, xn, xs, xs_stride, tile_begin, ne, wave, lane);
        else xsw.template gather<false>(P.xidx, reinterpret_cast<const WT*>(P.in), xs, xs_stride, tile_begin, ne, wave, lane);
    } else {
        // pairs re-read until they carry this launch's tag.  Only lanes that need a pair load one: these loads
        // are not cached, every one of them is a trip through the fabric.
        const unsigned long long* xp = reinterpret_cast<const unsigned long long*>(P.in);
        uint32_t spins = 0;
        for (int e0 = 0; XSW::pos_of(e0, wave) < ne; e0 += XP * 64) {       // the same trip count in every lane
            int sr[XP];
            if (e0 == 0) {
                #pragma unroll
                for (int k = 0; k < XP; ++k) sr[k] = xsw.src[k];
            } else {
                #pragma unroll
                for (int k = 0; k < XP; ++k) {
                    const int pos = XSW::pos_of(e0 + lane + k * 64, wave);
                    sr[k] = xi[pos < emax ? pos : emax];
                }
            }
            unsigned long long pv[XP];
            bool needed[XP];
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                const int pos = XSW::pos_of(e0 + lane + k * 64, wave);
                needed[k] = pos < ne && sr[k] >= 0 && sr[k] < P.k_valid;    // padding columns read as zero
                pv[k] = 0;
            }
            for (;;) {
                #pragma unroll
                for (int k = 0; k < XP; ++k)
                    if (needed[k] && (uint32_t)(pv[k] >> 32) != tag) pv[k] = cld64(xp + sr[k]);
                bool ok = true;
                #pragma unroll
                for (int k = 0; k < XP; ++k) ok = ok && (!needed[k] || (uint32_t)(pv[k] >> 32) == tag);
                if (!__any(!ok)) break;                                     // the whole wavefront leaves together
                if (!chain_keep_waiting(ctl, spins)) break;
            }
            #pragma unroll
            for (int k = 0; k < XP; ++k) {
                const int pos = XSW::pos_of(e0 + lane + k * 64, wave);
                xs[pos < ne ? pos : dump] = needed[k] ? WT(__uint_as_float((uint32_t)pv[k])) : WT(0);
            }
        }
    }
    wave_lds_sync();
    CHAIN_STAMP(2);

    float acc[NL];
    #pragma unroll
    for (int j = 0; j < NL; ++j) acc[j] = 0.f;
    auto consume = [&](int u, int g) {
        const int tl = g * TPL + ts;
        const V xv = *reinterpret_cast<const V*>(xs + tl * BW + cg * VEC);
        #pragma unroll
        for (int j = 0; j < NL; ++j) acc[j] = dot_vec(w[u][j], xv, acc[j]);
    };
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
    #pragma unroll
    for (int u = 0; u < U; ++u) {
        const int g = g0 + u * NW;
        if (g < ngroups && g * TPL + ts < ntiles) consume(u, g);
    }
    CHAIN_STAMP(3);
    #pragma unroll
    for (int j = 0; j < NL; ++j) {
        float v = group_sum<LPR>(acc[j]);
        if constexpr (TPL > 1) v = stride_sum<BH * LPR>(v);
        acc[j] = v;
    }
    if (cg == 0 && (TPL == 1 || s < BH)) {
        #pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int r = (TPL > 1) ? s : j * RPW + s;
            red[wave * BH + r] = acc[j];
        }
    }
    // a workgroup whose first layer is layer 0 learns its tag here: thread 0's load of the launch counter,
    // requested at kernel start, has long arrived and rides on this barrier to the other threads
    if (s_tag && tid == 0) *s_tag = counter + 1u;
    // The item's only workgroup barrier.  It orders LDS traffic only (lds_barrier): __syncthreads() would also
    // wait for every outstanding store, and the device-coherent stores of the PREVIOUS layer's outputs take about
    // a microsecond to be acknowledged; nothing in this workgroup depends on them.  Behind it every wavefront has
    // consumed its staged input, so the next item may overwrite that.
    lds_barrier();
    CHAIN_STAMP(4);
    if (s_tag) tag = *s_tag;
    if (tid < BH) {
        float sum = 0.f;
        #pragma unroll
        for (int wv = 0; wv < NW; ++wv) sum += red[wv * BH + tid];
        float v = apply_act(sum + bias, P.act);
        if (dst >= 0) {
            // an intermediate of an fp16 chain is rounded to fp16 once, here (the pair carries it as a float)
            if (out_tagged && sizeof(WT) == 2) v = (float)(_Float16)v;
            if (out_tagged)
                cst64(reinterpret_cast<unsigned long long*>(P.out) + dst,
                      ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v));
            else
                reinterpret_cast<float*>(P.out)[dst] = v;
        }
    }
    CHAIN_STAMP(5);                                     // stores issued, not yet acknowledged
#ifdef PIVOT_TRACE
    if (trace && lane == 0) {
        long long* t_ = trace + ((size_t)item * NW + wave) * 8;
        for (int i_ = 0; i_ < 8; ++i_) t_[i_] = ctr_[i_];
    }
#endif
}

// The first layer's pointers and shape come as separate leading arguments: those are preloaded into SGPRs with the
// wave (14 dwords), so the first loads of the launch do not wait for a fetch of the argument block.
// q0_ct_parts = uniform_ct | uniform_parts << 16; q0_shape = slices | bhs << 8 | bh_full << 16;
// q0_chunk_tiles = chunk_tiles | xn_vecs << 16 (xn_vecs > 0: copy x into LDS first).
template <typename WT, int BW, bool SHORT>
__global__ void __launch_bounds__(kChainNW * 64) mlp_persist_kernel(
        const int32_t* __restrict__ p0_xidx, const void* __restrict__ p0_vals, const void* __restrict__ p0_in,
        const float* __restrict__ p0_bias, const int32_t* __restrict__ p0_dst,
        int q0_ct_parts, int q0_shape, int q0_chunk_tiles, int q0_nitems, ChainArgs A) {
    extern __shared__ __align__(16) char smem[];
    __shared__ uint32_t s_tag;
    const int wg = blockIdx.x;
    // This launch's tag = the workgroup's own launch counter + 1.  Thread 0 requests the counter now; nothing
    // waits for it until the workgroup first needs the tag (layer 0: at its store; a workgroup that starts with
    // a later layer: before its first poll, where it would be waiting anyway).
    uint32_t counter = 0;
    if (threadIdx.x == 0) counter = cld32(A.ctl + wg);
    uint32_t tag = 0;
    bool have_tag = false;
    int red_slot = 0;                                   // flips with every item this workgroup runs (not with the layer:
                                                        // a workgroup may have no item in some layer)
    auto run_layer = [&](const ChainLayer& P, int l, const ChainLayer& next) {
        const bool in_tagged = l > 0, out_tagged = l + 1 < A.nlayers;
        if (!have_tag && in_tagged) {
            if (threadIdx.x == 0) s_tag = counter + 1u;
            __syncthreads();
            tag = s_tag;
            have_tag = true;
            if (threadIdx.x == 0) cst32(A.ctl + wg, tag);   // bumped by its only reader: no other workgroup touches it
        }
        uint32_t* st = have_tag ? nullptr : &s_tag;
        long long* tr = A.trace ? A.trace + (size_t)l * kChainMaxGrid * kChainNW * 8 : nullptr;
        if (in_tagged) {
            switch (P.bhs) {
                case 8:  chain_item<WT, 8, BW, kChainNW, kInTagged, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                case 16: chain_item<WT, 16, BW, kChainNW, kInTagged, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                case 32: chain_item<WT, 32, BW, kChainNW, kInTagged, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                default: chain_item<WT, 64, BW, kChainNW, kInTagged, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
            }
        } else if (P.xn_vecs > 0) {
            switch (P.bhs) {
                case 8:  chain_item<WT, 8, BW, kChainNW, kInCopy, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                case 16: chain_item<WT, 16, BW, kChainNW, kInCopy, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                case 32: chain_item<WT, 32, BW, kChainNW, kInCopy, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                default: chain_item<WT, 64, BW, kChainNW, kInCopy, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
            }
        } else {
            switch (P.bhs) {
                case 8:  chain_item<WT, 8, BW, kChainNW, kInPlain, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                case 16: chain_item<WT, 16, BW, kChainNW, kInPlain, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                case 32: chain_item<WT, 32, BW, kChainNW, kInPlain, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
                default: chain_item<WT, 64, BW, kChainNW, kInPlain, SHORT>(P, wg, out_tagged, tag, counter, st, A.ctl, smem, tr, next, red_slot); break;
            }
        }
        red_slot ^= 1;
        if (!have_tag) {                                // s_tag was set inside the item, before its barrier
            tag = s_tag;
            have_tag = true;
            if (threadIdx.x == 0) cst32(A.ctl + wg, tag);
        }
    };
    // the description of the layer after the current one is touched inside the current item (pin_layer), so that
    // it sits in the scalar cache when that layer begins
    if (wg < q0_nitems) {                               // uniform over the workgroup
        ChainLayer P0;
        P0.xidx = p0_xidx; P0.vals = p0_vals; P0.in = p0_in; P0.bias_p = p0_bias; P0.dst = p0_dst;
        P0.uniform_ct = q0_ct_parts & 0xFFFF; P0.uniform_parts = q0_ct_parts >> 16;
        P0.slices = q0_shape & 0xFF; P0.bhs = (q0_shape >> 8) & 0xFF; P0.bh_full = (q0_shape >> 16) & 0xFF;
        P0.chunk_tiles = q0_chunk_tiles & 0xFFFF; P0.xn_vecs = q0_chunk_tiles >> 16; P0.nitems = q0_nitems;
        P0.chunks = A.L[0].chunks; P0.out = A.L[0].out; P0.act = A.L[0].act; P0.k_valid = A.L[0].k_valid;
        run_layer(P0, 0, A.L[1]);                        // (a chain has at least two layers)
    }
    for (int l = 1; l < A.nlayers; ++l) {
        const ChainLayer& P = A.L[l];
        if (wg < P.nitems) run_layer(P, l, A.L[l + 1 < A.nlayers ? l + 1 : l]);   // uniform over the workgroup
    }
}

template <bool SHORT>
static const void* chain_kernel_of(int wdtype, int bw) {
    if (wdtype == PIVOT_F32) {
        switch (bw) {
            case 16: return reinterpret_cast<const void*>(&mlp_persist_kernel<float, 16, SHORT>);
            case 32: return reinterpret_cast<const void*>(&mlp_persist_kernel<float, 32, SHORT>);
            case 64: return reinterpret_cast<const void*>(&mlp_persist_kernel<float, 64, SHORT>);
            default: return nullptr;
        }
    }
    switch (bw) {
        case 16: return reinterpret_cast<const void*>(&mlp_persist_kernel<_Float16, 16, SHORT>);
        case 32: return reinterpret_cast<const void*>(&mlp_persist_kernel<_Float16, 32, SHORT>);
        case 64: return reinterpret_cast<const void*>(&mlp_persist_kernel<_Float16, 64, SHORT>);
        default: return nullptr;
    }
}

const void* chain_kernel_for(int wdtype, int bw, bool short_items) {
    return short_items ? chain_kernel_of<true>(wdtype, bw) : chain_kernel_of<false>(wdtype, bw);
}

// Row slices of a layer inside the chain kernel: the plan's own choice, lowered until a slice holds at least
// one 1 KB wave-load and 8 rows (the same rule as the layer kernel's).
int chain_slices(const HostPlan& hp) {
    return fc_row_slices(FcShape{hp.d.layout, hp.d.wdtype, hp.d.bh, hp.d.bw, hp.chunk_tiles, hp.chunk_tiles, 0, 0}, 1, hp.row_slices);
}

// True if no wavefront of an item of this layer stages more than 64 elements: its groups (wave, wave + 8, ...)
// of TPL tiles of bw columns.
static bool chain_layer_short(const HostPlan& hp) {
    const int vec = 16 / elem_size(hp.d.wdtype), lpr = hp.d.bw / vec, rpw = 64 / (lpr > 0 ? lpr : 1);
    const int bhs = hp.d.bh / chain_slices(hp);
    const int tpl = bhs >= rpw ? 1 : rpw / bhs;
    const int ct = hp.uniform_ct > 0 ? hp.uniform_ct : hp.chunk_tiles;
    const int ngroups = (ct + tpl - 1) / tpl;
    return ((ngroups + kChainNW - 1) / kChainNW) * tpl * hp.d.bw <= 64;
}
// The kernel form for a chain: SHORT when every layer behind the first is.
static bool chain_short(const std::vector<const HostPlan*>& layers) {
    for (size_t l = 1; l < layers.size(); ++l) if (!chain_layer_short(*layers[l])) return false;
    return true;
}

}  // namespace

size_t chain_persist_ctl_bytes() { return (size_t)(kChainStatus + 64) * 4; }

bool chain_persist_supported(const std::vector<const HostPlan*>& layers, int device, int* grid_out, size_t* smem_out,
                             size_t* smem_copy_out, std::string* why) {
    auto no = [&](const char* m) { if (why) *why = m; return false; };
    const int Lc = (int)layers.size();
    if (Lc < 2 || Lc > kMaxChainLayers) return no("2..8 layers");
    const int bw = layers[0]->d.bw, wdtype = layers[0]->d.wdtype;
    const int es = elem_size(wdtype), vec = 16 / es;
    if (!chain_kernel_for(wdtype, bw, false)) return no("tile width 16, 32 or 64");
    int G = 0;
    size_t smem = 0;
    for (const HostPlan* hp : layers) {
        if (hp->d.wdtype != wdtype || hp->d.layout != PIVOT_BRC) return no("BRC plans of one weight type only");
        if (hp->d.bw != bw) return no("one tile width for all layers");
        if (hp->max_parts > 1) return no("whole block rows per work item only");
        const int sl = chain_slices(*hp);
        const int bhs = hp->d.bh / sl;
        if (bhs != 8 && bhs != 16 && bhs != 32 && bhs != 64) return no("row slices of 8, 16, 32 or 64 rows");
        if (bw < vec || bw / vec > 64 || hp->d.bh > 64) return no("tile shape");
        const long long items = (long long)hp->nchunks * sl;
        if (items > kChainMaxGrid) return no("more work items than the one-launch form takes");
        G = std::max(G, (int)items);
        const int ct = hp->uniform_ct > 0 ? hp->uniform_ct : hp->chunk_tiles;
        smem = std::max(smem, ((size_t)ct * bw + vec) * es);
    }
    smem = kChainRedBytes + align_up(smem, 16);
    if (smem > 64 * 1024) return no("staged x does not fit in LDS");
    // with the first layer's x copied into LDS whole (chosen at launch if x is 16-byte aligned): 0 = not possible
    size_t smem_copy = 0;
    {
        const HostPlan& f = *layers[0];
        const int ct = f.uniform_ct > 0 ? f.uniform_ct : f.chunk_tiles;
        const size_t need = kChainRedBytes + ((size_t)f.d.K + vec) * es + ((size_t)ct * bw + vec) * es;
        const size_t item_bytes = (size_t)ct * (f.d.bh / chain_slices(f)) * bw * es;  // same threshold as the layer kernel
        // worth it when the element gather would move at least twice the bytes of the copy (a cache line per element)
        if (item_bytes >= 48 * 1024 && (size_t)ct * bw * 128 >= 2 * (size_t)f.d.K * es && f.d.K % vec == 0 &&
            f.d.K / vec <= 16 * kChainNW * 64 && need <= 150 * 1024)
            smem_copy = align_up(std::max(need, smem), 16);
    }
    if (device >= 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, chain_kernel_for(wdtype, bw, chain_short(layers)), kChainNW * 64, smem) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) {
            (void)hipGetLastError();
            return no("occupancy query failed");
        }
        if ((long long)per_cu * cus < G) return no("the work items of a layer are not all resident at once");
        // the copy takes most of a compute unit's LDS: one workgroup per compute unit
        if (smem_copy > 80 * 1024 && G > cus) smem_copy = 0;
        if (smem_copy > 0 && smem_copy <= 80 * 1024 && (long long)(160 * 1024 / smem_copy) * cus < G) smem_copy = 0;
    } else {
        smem_copy = 0;
    }
    if (grid_out) *grid_out = G;
    if (smem_out) *smem_out = smem;
    if (smem_copy_out) *smem_copy_out = smem_copy;
    return true;
}

int launch_chain_persist(const ChainPersistLaunch& C) {
    ChainArgs A{};
    const int Lc = (int)C.layers.size();
    A.nlayers = Lc;
    A.ctl = C.ctl;
    A.trace = nullptr;
#ifdef PIVOT_TRACE
    // timeline builds: [layer][1024 workgroups][8 wavefronts][8] int64 time stamps
    if (const char* e = getenv("PIVOT_CHAIN_TRACE_PTR")) A.trace = reinterpret_cast<long long*>(strtoull(e, nullptr, 0));
#endif
    bool short_items = true;
    for (int l = 0; l < Lc; ++l) {
        const ChainPersistLayer& s = C.layers[l];
        const HostPlan& hp = *s.hp;
        ChainLayer& P = A.L[l];
        const int sl = chain_slices(hp);
        P.chunks = reinterpret_cast<const int4*>(s.chunks);
        P.xidx = s.xidx; P.vals = s.vals; P.bias_p = s.bias_p; P.dst = s.dst;
        P.in = s.in; P.out = s.out;
        P.nitems = hp.nchunks * sl; P.slices = sl; P.bhs = hp.d.bh / sl; P.bh_full = hp.d.bh;
        P.uniform_ct = hp.uniform_ct; P.uniform_parts = hp.uniform_parts;
        P.chunk_tiles = hp.uniform_ct > 0 ? hp.uniform_ct : hp.chunk_tiles;
        P.act = hp.d.act; P.k_valid = hp.d.K; P.xn_vecs = 0;
        if (l > 0 && !chain_layer_short(hp)) short_items = false;
    }
    size_t smem = C.smem;
    if (C.smem_copy > 0 && (reinterpret_cast<uintptr_t>(A.L[0].in) & 15) == 0) {
        A.L[0].xn_vecs = C.layers[0].hp->d.K / (16 / elem_size(C.wdtype));
        smem = C.smem_copy;
        if (smem > 64 * 1024) {                         // more than 64 KB of dynamic LDS has to be allowed per kernel and device
            static size_t allowed[16][12] = {};
            int dev = 0;
            HIP_TRY(hipGetDevice(&dev));
            size_t& a = allowed[dev & 15][(short_items ? 6 : 0) + (C.wdtype == PIVOT_F32 ? 0 : 3) + (C.bw == 16 ? 0 : (C.bw == 32 ? 1 : 2))];
            if (smem > a) {
                HIP_TRY(hipFuncSetAttribute(chain_kernel_for(C.wdtype, C.bw, short_items), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
                a = smem;
            }
        }
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(C.stream);
    const ChainLayer& F = A.L[0];
    if (F.uniform_ct > 0xFFFF || F.uniform_parts > 0x7FFF || F.chunk_tiles > 0xFFFF || F.xn_vecs > 0x7FFF) { set_error("first layer outside the packed arguments"); return PIVOT_E_UNSUPPORTED; }
    const int32_t* p0_xidx = F.xidx; const void* p0_vals = F.vals; const void* p0_in = F.in;
    const float* p0_bias = F.bias_p; const int32_t* p0_dst = F.dst;
    int q0_ct_parts = F.uniform_ct | (F.uniform_parts << 16), q0_shape = F.slices | (F.bhs << 8) | (F.bh_full << 16);
    int q0_chunk_tiles = F.chunk_tiles | (F.xn_vecs << 16), q0_nitems = F.nitems;
    void* args[] = {&p0_xidx, &p0_vals, &p0_in, &p0_bias, &p0_dst, &q0_ct_parts, &q0_shape, &q0_chunk_tiles, &q0_nitems, &A};
    HIP_TRY(hipLaunchKernel(chain_kernel_for(C.wdtype, C.bw, short_items), dim3(C.grid), dim3(kChainNW * 64), args, smem, st));
    return PIVOT_OK;
}

int chain_persist_status_offset() { return kChainStatus * 4; }

}  // namespace pivot
