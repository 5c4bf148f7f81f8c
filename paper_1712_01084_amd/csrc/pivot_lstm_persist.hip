// Persistent recurrent kernel: the whole LSTM loop around a pruned gate matrix
// in ONE launch.  The recurrence is the PBP layer (paper Eq. 2) back to back
// with itself through a point-wise cell, so the boundary fusion of Section
// 4.2.1 applies at every step; what a launch per step adds on top of that is
// only launch latency and a re-read of the weights.  Here every wavefront keeps
// its share of the kept tiles in registers (as MFMA A fragments) for all steps,
// and the steps are ordered by the data itself instead of by kernel boundaries
// or grid-wide barriers (measured on MI355X: a barrier over 256 workgroups
// costs 1.9 us at best and 4.1 us with one shared counter, a step needs two;
// a value that carries its own "ready" mark costs one trip through memory,
// about 2.5 us here from the producer's store to the consumer's load, and
// that trip, twice per step, is what bounds the step).
//
// Work split (static, derived from row_ptr alone): with T kept tiles in
// canonical (block row, block column) order and G workgroups of 4 wavefronts,
// L = ceil(T / 4G); wavefront w owns tiles [wL, wL+L), workgroup g the 4L
// tiles [4gL, 4gL+4L).  A maximal run of tiles of one block row inside a
// workgroup's range is a "segment"; its partial sums go to the global slot
// numbered by the ordinal of the segment's last tile, so the cell phase can
// find all pieces of a block row from row_ptr: block row [b, e) has one piece
// per workgroup g in [b/4L, (e-1)/4L], slot min((g+1)4L, e) - 1.
//
// One step t:
//   phase A  every wavefront reads the B fragments (k x batch) of its tiles
//            from the block-order input of step t, one MFMA per tile
//            (v_mfma_f32_16x16x32_f16, tile 16x32 = A, accumulate in fp32),
//            flushes the accumulator to LDS whenever the block row changes;
//            the workgroup adds the pieces of each segment in wavefront order
//            and stores one partial per segment, every element as the pair
//            (value, t+1) in one 8-byte store.
//   phase B  workgroup g < K_pad/32 owns 32 block-space columns of the next
//            input, one thread per (column, batch row): for a column that is
//            a unit's h it reads the pieces of the unit's four gate rows until
//            their marks say t+1, adds them in ascending slot order plus the
//            permuted bias; the cell state stays in a register for the whole
//            sequence; h_t goes straight to its block-order position in the
//            input of step t+1 (via LDS, as whole cache lines per batch row;
//            x_{t+1} and padding columns are rewritten unchanged).
// The inputs of all steps are pre-filled with a fp16 bit pattern no finite
// value has (0xFFFF) wherever h_t will land, so a B fragment is complete when
// none of its halves is that pattern: phase A of step t+1 simply re-reads
// until it is.  Partials rotate through eight buffers; every four steps each
// workgroup publishes its progress and checks that all others are within four
// steps, so a buffer is never overwritten before all its readers are done.
//
// Everything that crosses workgroups is written with device-coherent stores
// and read with device-coherent loads; no fences, no floating-point atomics,
// fixed summation order: results are bit-identical from run to run.  All
// workgroups must be resident at once (checked at launch).  Every wait is
// bounded: after kSpinLimit polls it raises the status word and every
// workgroup leaves.
#include "pivot_fc_kernels.h"

namespace pivot {

namespace {

constexpr int kNW = 4;                  // wavefronts per workgroup
constexpr int kNT = kNW * 64;
constexpr int kBH = 16, kBW = 32;       // tile shape this kernel is written for
constexpr int kSlot = 16 * 16;          // floats per flushed accumulator in LDS: [batch column n < 16][row < 16]
constexpr uint32_t kSpinLimit = 1u << 18;  // polls before a wait gives up (a few tenths of a second)
constexpr unsigned short kNotYet = 0xFFFFu;
constexpr int kPBuf = 8;                // partial buffers in rotation
constexpr int kCellB = 8;               // batch rows the cell phase is laid out for

struct PersistArgs {
    const _Float16* vals;       // [T][16][32] BRC
    const int32_t*  col_idx;    // [T]
    const int32_t*  row_ptr;    // [nbr+1]
    const int32_t*  invprow;    // [4H] natural gate row -> block-space row
    const int32_t*  pcol_pad;   // [K_pad] block-space column -> natural input column (-1 = padding)
    const float*    bias_p;     // [M_pad]
    const _Float16* xs;         // [steps][batch][I] the caller's inputs
    _Float16*       xg;         // [steps][batch][K_pad] block-order inputs: x_t and padding placed, h_0 in step 0,
                                //   kNotYet wherever h_t (t >= 1) will land
    size_t          xg_step;    // elements between steps
    unsigned long long* partials;   // [kPBuf][T][16][batch] pairs (value, step+1), zeroed before the launch
    uint32_t*       ctl;        // [0..G) cell phases finished per workgroup; [256] status (0 ok, 1 a wait gave up)
    float*          h;          // [batch][H] h_0 in, h_steps out
    float*          c;          // [batch][H]
    float*          z_dbg;      // optional [batch][4H]
    int T, nbr, H, I, K_pad, batch, steps, L;
};

__device__ __forceinline__ float sigm(float v) { return 1.0f / (1.0f + __expf(-v)); }

__device__ __forceinline__ unsigned long long ld64(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld32(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st32(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// true if one of the four fp16 halves of the two words is the "not written yet" pattern
__device__ __forceinline__ bool not_yet(unsigned long long v) {
    const uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    return (lo & 0xFFFFu) == kNotYet || (lo >> 16) == kNotYet || (hi & 0xFFFFu) == kNotYet || (hi >> 16) == kNotYet;
}

// A poll that did not succeed: pause; every 64th time look at the status word,
// and give up (raising it) at the limit.  Returns false when the wait must end.
__device__ __forceinline__ bool keep_waiting(uint32_t* ctl, uint32_t& spins) {
    // a short pause: since a retry re-reads only what is missing, longer pauses only add to the wake-up time
    // (256 steps: 16 -> 1845 us, 8 -> 1782, 4 -> 1755, 2 -> 1741, 1 or none -> 1732)
    __builtin_amdgcn_s_sleep(1);
    if ((++spins & 63u) != 0u) return true;
    if (ld32(ctl + 256) != 0u) return false;
    if (spins >= kSpinLimit) { st32(ctl + 256, 1u); return false; }
    return true;
}

// 16 bytes another workgroup may have written during this launch.  One load
// instruction instead of two 8-byte ones: device-coherent loads are not cached,
// every instruction is a trip through the fabric for each line it touches.
// The compiler does not track the returned data; wait_frags() must follow.
__device__ __forceinline__ void frag_load(f16x8& dst, const _Float16* p) {
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(dst) : "v"(p) : "memory");
}
template <int LMAX>
__device__ __forceinline__ void wait_frags(f16x8 (&xb)[LMAX]) {
    if constexpr (LMAX == 8)
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(xb[0]), "+v"(xb[1]), "+v"(xb[2]), "+v"(xb[3]),
                                            "+v"(xb[4]), "+v"(xb[5]), "+v"(xb[6]), "+v"(xb[7]) :: "memory");
    else
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(xb[0]), "+v"(xb[1]), "+v"(xb[2]), "+v"(xb[3]),
                                            "+v"(xb[4]), "+v"(xb[5]), "+v"(xb[6]), "+v"(xb[7]),
                                            "+v"(xb[8]), "+v"(xb[9]), "+v"(xb[10]), "+v"(xb[11]),
                                            "+v"(xb[12]), "+v"(xb[13]), "+v"(xb[14]), "+v"(xb[15]) :: "memory");
}
__device__ __forceinline__ bool not_yet16(const f16x8& v) {
    unsigned long long q[2];
    __builtin_memcpy(q, &v, 16);
    return not_yet(q[0]) || not_yet(q[1]);
}

template <int LMAX>
__global__ void __launch_bounds__(kNT) lstm_persist_kernel(PersistArgs a) {
    extern __shared__ __align__(16) float s_part[];      // [4L][kSlot] accumulators flushed by the wavefronts
    __shared__ int s_row[4 * LMAX + 1];                  // block row of every tile of the workgroup's range (-1 = none)
    __shared__ int s_seg_b[4 * LMAX], s_seg_e[4 * LMAX]; // segments: tile positions [b, e) inside the range
    __shared__ int s_nseg;
    __shared__ unsigned short s_next[kCellB][kBW];       // this workgroup's 32 columns of the next input

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.x, G = gridDim.x;
    const int L = a.L, R = 4 * L;                        // tiles per wavefront / per workgroup
    const int range0 = g * R;

    // ---- static set-up -------------------------------------------------------
    // block row of each tile of the range: last i with row_ptr[i] <= t
    for (int p = tid; p <= R; p += kNT) {
        const int t = range0 + p;
        int br = -1;
        if (p < R && t < a.T) {
            int lo = 0, hi = a.nbr;                      // invariant: row_ptr[lo] <= t < row_ptr[hi]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (a.row_ptr[mid] <= t) lo = mid; else hi = mid;
            }
            br = lo;
        }
        s_row[p] = br;
    }
    __syncthreads();
    if (tid == 0) {
        int n = 0;
        for (int p = 0; p < R && s_row[p] >= 0; ) {
            int q = p + 1;
            while (q < R && s_row[q] == s_row[p]) ++q;
            s_seg_b[n] = p; s_seg_e[n] = q; ++n;
            p = q;
        }
        s_nseg = n;
    }
    __syncthreads();
    const int nseg = s_nseg;

    // this wavefront's tiles: A fragments (lane l: row l%16, k 8(l/16)..+7), block column, flush-after flag
    const int wp0 = wave * L;                            // first tile position of the wavefront inside the range
    const int li = lane & 15, lg = lane >> 4;
    f16x8 w[LMAX];
    int ci[LMAX];
    unsigned flush = 0;
    #pragma unroll
    for (int i = 0; i < LMAX; ++i) {
        const int p = wp0 + i;
        const bool have = i < L && s_row[p < R ? p : R] >= 0;
        const int t = have ? range0 + p : 0;
        w[i] = load16<f16x8>(a.vals + (size_t)t * (kBH * kBW) + li * kBW + lg * 8);
        if (!have) w[i] = f16x8(0);
        ci[i] = have ? a.col_idx[t] : 0;
        const bool last = have && (i == L - 1 || s_row[p + 1] != s_row[p]);
        flush |= (last ? 1u : 0u) << i;
    }
    // batch columns past `batch` repeat the last row: their accumulator columns are never read
    const int brow = li < a.batch ? li : a.batch - 1;

    // Cell items.  Workgroup g < K_pad/32 owns block-space columns [32g, 32g+32) of every step's input; thread
    // (column tid/8, batch row tid%8) computes one element: a unit's h, or a copy of x_{t+1}, or zero padding.
    // Eight neighbouring lanes share a column, so the eight batch values of a gate row (64 contiguous bytes)
    // come back with one request; the finished 32 columns go through LDS so that they leave as whole cache
    // lines per batch row (a write-through store of part of a line is a slow read-modify-write at the memory).
    const int cb_own = g;
    const bool cell_wg = cb_own * kBW < a.K_pad;
    const int ib = tid & (kCellB - 1), icol = cb_own * kBW + (tid >> 3);
    const bool has_item = cell_wg && ib < a.batch;
    const int src = has_item ? a.pcol_pad[icol] : -1;
    const bool is_h = src >= 0 && src < a.H;
    const int unit = is_h ? src : 0;
    const int x_off = src >= a.H ? src - a.H : -1;       // index into x_t of an input column
    int   g_first[4], g_cnt[4], g_end[4], g_rr[4];
    float g_bias[4];
    int rounds = 0;                                      // most pieces any of this thread's gate rows is cut into
    #pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = a.invprow[q * a.H + unit];
        const int br = r / kBH;
        const int b = a.row_ptr[br], en = a.row_ptr[br + 1];
        g_rr[q] = r - br * kBH;
        g_end[q] = en;
        g_first[q] = b / R;
        g_cnt[q] = (is_h && en > b) ? (en - 1) / R - b / R + 1 : 0;
        g_bias[q] = a.bias_p[r];
        rounds = g_cnt[q] > rounds ? g_cnt[q] : rounds;
    }
    float c_state = is_h ? a.c[(size_t)ib * a.H + unit] : 0.f;
    float h_state = is_h ? a.h[(size_t)ib * a.H + unit] : 0.f;
    const size_t pbuf = (size_t)a.T * 16 * a.batch;      // pairs per partial buffer: [T][16 rows][batch]

    // ---- the sequence --------------------------------------------------------
    int alive = 1;
    for (int t = 0; t < a.steps && alive; ++t) {
        const _Float16* xg = a.xg + (size_t)t * a.xg_step;
        const uint32_t mark = (uint32_t)t + 1u;
        int ok = 1;
        uint32_t spins = 0;

        // Partials rotate through kPBuf buffers.  Every kPBuf/2 steps each workgroup publishes how many cell
        // phases it has finished and checks that every workgroup is within kPBuf/2 steps, so the buffers written
        // until the next check hold only partials that all of their readers have consumed.
        const bool check = (t % (kPBuf / 2) == 0) && t >= kPBuf;
        uint32_t seen = (check && tid < G) ? ld32(a.ctl + tid) : 0xFFFFFFFFu;

        // x_{t+1} for the columns of the next input that are inputs: requested first, so that it is back with
        // the B fragments instead of costing a trip of its own in phase B
        unsigned short out = 0;                          // padding columns stay zero
        if (x_off >= 0 && t + 1 < a.steps)
            out = __builtin_bit_cast(unsigned short, a.xs[((size_t)(t + 1) * a.batch + ib) * a.I + x_off]);

        // phase A: B fragments (lane l: batch row l%16, k 8(l/16)..+7), re-read until complete
        f16x8 xb[LMAX];
        for (;;) {
            // while the input is not there yet only the first fragment is polled: 1024 wavefronts re-reading
            // everything would crowd the fabric that the producers' stores need
            for (;;) {
                frag_load(xb[0], xg + (size_t)brow * a.K_pad + ci[0] * kBW + lg * 8);
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(xb[0]) :: "memory");
                if (!not_yet16(xb[0])) break;
                if (!keep_waiting(a.ctl, spins)) { ok = 0; break; }
            }
            if (!ok) break;
            #pragma unroll
            for (int i = 0; i < LMAX; ++i) {
                if (i < L) frag_load(xb[i], xg + (size_t)brow * a.K_pad + ci[i] * kBW + lg * 8);
                else       xb[i] = f16x8(0);
            }
            wait_frags<LMAX>(xb);
            // fragments of other producers may still be missing: only those are read again (one trip per
            // retry instead of a probe and a full read; requesting everything before the probe, for the
            // wavefronts that arrive late, was measured slower)
            unsigned missing = 0;
            #pragma unroll
            for (int i = 0; i < LMAX; ++i) missing |= (i < L && not_yet16(xb[i]) ? 1u : 0u) << i;
            while (__any(missing != 0)) {
                if (!keep_waiting(a.ctl, spins)) { ok = 0; break; }
                #pragma unroll
                for (int i = 0; i < LMAX; ++i)
                    if (missing & (1u << i)) frag_load(xb[i], xg + (size_t)brow * a.K_pad + ci[i] * kBW + lg * 8);
                wait_frags<LMAX>(xb);
                unsigned still = 0;
                #pragma unroll
                for (int i = 0; i < LMAX; ++i) still |= ((missing >> i) & 1u) && not_yet16(xb[i]) ? (1u << i) : 0u;
                missing = still;
            }
            break;
        }
        f32x4 acc = f32x4(0);
        #pragma unroll
        for (int i = 0; i < LMAX; ++i) {
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(w[i], xb[i], acc, 0, 0, 0);
            if (flush & (1u << i)) {                     // wave-uniform
                // accumulator element v of lane l is C[row 4(l/16)+v][batch column l%16]
                *reinterpret_cast<f32x4*>(s_part + (wp0 + i) * kSlot + li * 16 + lg * 4) = acc;
                acc = f32x4(0);
            }
        }
        while (seen < (uint32_t)(t - kPBuf / 2)) {
            if (!keep_waiting(a.ctl, spins)) { ok = 0; break; }
            seen = ld32(a.ctl + tid);
        }
        alive = __syncthreads_and(ok);
        if (!alive) break;
        // pieces of each segment in wavefront order -> one partial per segment, [row][batch] so that the batch
        // values of a row are contiguous
        unsigned long long* pbw = a.partials + (size_t)(t % kPBuf) * pbuf;
        {
            // 16 * batch threads per segment; the thread groups take the segments in turn (a workgroup whose
            // tiles are many short block rows has a dozen segments, and the slowest workgroup sets the step)
            const int per = 16 * a.batch, ngrp = kNT / per;
            const int grp = tid / per, rest = tid - grp * per;
            const int row = rest / a.batch, n = rest - row * a.batch;
            if (grp < ngrp) {
                for (int s = grp; s < nseg; s += ngrp) {
                    const int sb = s_seg_b[s], se = s_seg_e[s];
                    float sum = 0.f;
                    #pragma unroll
                    for (int k = 0; k < kNW; ++k) {
                        const int lo = sb > k * L ? sb : k * L;
                        const int hi = se < (k + 1) * L ? se : (k + 1) * L;
                        if (lo < hi) sum += s_part[(hi - 1) * kSlot + n * 16 + row];
                    }
                    const unsigned long long pair = ((unsigned long long)mark << 32) | __builtin_bit_cast(uint32_t, sum);
                    __hip_atomic_store(pbw + ((size_t)(range0 + se - 1) * 16 + row) * a.batch + n, pair,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }

        // phase B: gates (pieces in ascending slot order), cell, the 32 columns of the next input
        if (cell_wg) {
            if (out == kNotYet) out = 0xFFFEu;           // a NaN input stays a NaN, never the mark
            float z[4] = {0.f, 0.f, 0.f, 0.f};
            // the pieces of all four gate rows are requested together, up to four per row and round (a second
            // round only for block rows cut into more than four pieces)
            for (int k0 = 0; k0 < rounds && ok; k0 += 4) {
                unsigned long long v[4][4];
                for (;;) {
                    uint32_t bad = 0;                    // no short-circuit: every load is issued before any is looked at
                    #pragma unroll
                    for (int q = 0; q < 4; ++q)
                        #pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            v[q][k] = (unsigned long long)mark << 32;            // absent piece: ready, value +0
                            if (k0 + k < g_cnt[q]) {
                                const int gi = g_first[q] + k0 + k;
                                const int slot = ((gi + 1) * R < g_end[q] ? (gi + 1) * R : g_end[q]) - 1;
                                v[q][k] = ld64(pbw + ((size_t)slot * 16 + g_rr[q]) * a.batch + ib);
                            }
                        }
                    #pragma unroll
                    for (int q = 0; q < 4; ++q)
                        #pragma unroll
                        for (int k = 0; k < 4; ++k) bad |= (uint32_t)(v[q][k] >> 32) ^ mark;
                    if (bad == 0u) break;
                    if (!keep_waiting(a.ctl, spins)) { ok = 0; break; }
                }
                #pragma unroll
                for (int q = 0; q < 4; ++q)
                    #pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (k0 + k < g_cnt[q]) z[q] += __builtin_bit_cast(float, (uint32_t)v[q][k]);
            }
            if (is_h && ok) {
                #pragma unroll
                for (int q = 0; q < 4; ++q) z[q] += g_bias[q];
                c_state = sigm(z[1]) * c_state + sigm(z[0]) * tanhf(z[2]);
                h_state = sigm(z[3]) * tanhf(c_state);
                out = __builtin_bit_cast(unsigned short, (_Float16)h_state);
                if (out == kNotYet) out = 0xFFFEu;
                if (a.z_dbg && t + 1 == a.steps) {
                    float* zd = a.z_dbg + (size_t)ib * 4 * a.H;
                    #pragma unroll
                    for (int q = 0; q < 4; ++q) zd[q * a.H + unit] = z[q];
                }
            }
            s_next[ib][tid >> 3] = out;
        }
        alive = __syncthreads_and(ok);                   // also: every thread is done reading s_part and the partials
        if (!alive) break;
        if (cell_wg && t + 1 < a.steps && tid < a.batch * (kBW / 2)) {
            // 16 lanes per batch row, one 4-byte word each: 64 contiguous bytes = one whole line per row
            const int b = tid / (kBW / 2), pr = tid - b * (kBW / 2);
            const uint32_t word = (uint32_t)s_next[b][2 * pr] | ((uint32_t)s_next[b][2 * pr + 1] << 16);
            st32(reinterpret_cast<uint32_t*>(a.xg + (size_t)(t + 1) * a.xg_step + (size_t)b * a.K_pad + cb_own * kBW) + pr, word);
        }
        if (tid == 0 && (t + 1) % (kPBuf / 2) == 0) st32(a.ctl + g, mark);   // cell phases 0..t of this workgroup are finished
    }
    if (is_h && alive) {
        a.c[(size_t)ib * a.H + unit] = c_state;
        a.h[(size_t)ib * a.H + unit] = h_state;
    }
}

}  // namespace

// Block-order inputs of all steps for the one-launch form: x_t and h_0 in place, zero in the padding
// columns, the "not yet" pattern wherever a later h_t will land.
__global__ void lstm_prepare_kernel(const _Float16* xs, const float* h0, const int32_t* pcol_pad, _Float16* xg,
                                    size_t xg_step, int H, int I, int K_pad, int batch, size_t total) {
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; idx < total; idx += stride) {
        const int c = (int)(idx % K_pad);
        const size_t tb = idx / K_pad;                   // step * batch + b
        const int b = (int)(tb % batch);
        const size_t t = tb / batch;
        const int src = pcol_pad[c];
        unsigned short v;
        if (src < 0) v = 0;
        else if (src >= H) v = __builtin_bit_cast(unsigned short, xs[tb * I + (src - H)]);
        else if (t == 0) v = __builtin_bit_cast(unsigned short, (_Float16)h0[(size_t)b * H + src]);
        else v = kNotYet;
        if (v == kNotYet && (src >= H || (src >= 0 && t == 0))) v = 0xFFFEu;   // a NaN input stays a NaN, not the mark
        reinterpret_cast<unsigned short*>(xg)[t * xg_step + (size_t)b * K_pad + c] = v;
    }
}

// Device limits looked up once per device.
static int persist_grid(int device) {
    static int cached_dev = -1, cached = 0;
    if (cached_dev == device) return cached;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
    cached = prop.multiProcessorCount;
    cached_dev = device;
    return cached;
}

bool lstm_persist_supported(const HostPlan& hp, int H, int batch, int device, int* grid_out, int* L_out) {
    if (hp.d.wdtype != PIVOT_F16 || hp.d.layout != PIVOT_BRC || hp.d.bh != kBH || hp.d.bw != kBW) return false;
    if (batch < 1 || batch > kCellB || hp.T < 1) return false;
    int cus = persist_grid(device);
    if (cus < 1) return false;
    if (cus > 256) cus = 256;
    if (hp.K_pad / kBW > cus) return false;                                // one workgroup per 32 input columns
    // Workgroups: as few as fill the eight tile slots of every wavefront (every workgroup adds uncached requests
    // to both exchanges of a step), but at least half the compute units and one per 32 input columns.  Measured
    // on 6144 tiles: 256 workgroups (6 tiles per wavefront) 2195 us for 256 steps, 224 (7) 2220 us, 192 (8)
    // 2065 us, 160 (10, the 16-slot kernel) 2660 us.
    int G = (hp.T + 4 * 8 - 1) / (4 * 8);
    G = std::max(G, std::max(hp.K_pad / kBW, cus / 2));
    G = std::min(G, cus);
    const int L = (hp.T + 4 * G - 1) / (4 * G);
    // tiles stay in registers (16 slots); with 16 tiles per wavefront the flushed accumulators alone would take
    // the 64 KB of LDS a launch gets without asking for more, so 15 is the limit
    if (L > 15) return false;
    // every workgroup must be resident at once (they wait for each other): asked once per device and L
    {
        static int fits[16][16] = {};                                     // [device & 15][L]: 0 unknown, 1 yes, -1 no
        int& f = fits[device & 15][L];
        if (f == 0) {
            int prev = -1, per_cu = 0;
            if (hipGetDevice(&prev) != hipSuccess) { (void)hipGetLastError(); return false; }
            if (prev != device && hipSetDevice(device) != hipSuccess) { (void)hipGetLastError(); return false; }
            const size_t smem = (size_t)4 * L * kSlot * 4;
            const hipError_t e = L <= 8 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, lstm_persist_kernel<8>, kNT, smem)
                                        : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, lstm_persist_kernel<16>, kNT, smem);
            if (prev != device) (void)hipSetDevice(prev);
            if (e != hipSuccess) { (void)hipGetLastError(); return false; }
            f = per_cu >= 1 ? 1 : -1;
        }
        if (f < 0) return false;
    }
    if (grid_out) *grid_out = G;
    if (L_out) *L_out = L;
    return true;
}

size_t lstm_persist_partial_bytes(const HostPlan& hp, int batch) { return align_up((size_t)kPBuf * hp.T * batch * 16 * 8, 256); }
// The part of them a sequence of `steps` steps uses (step t: buffer t % kPBuf) and that therefore has to be zero
// before the launch: a short sequence clears one buffer per step instead of all eight (6 MB each on the
// 8192x3072 workload at batch 8).
size_t lstm_persist_used_partial_bytes(const HostPlan& hp, int batch, int steps) {
    const size_t nbuf = steps < kPBuf ? (steps > 0 ? steps : 1) : kPBuf;
    return std::min(lstm_persist_partial_bytes(hp, batch), align_up(nbuf * hp.T * batch * 16 * 8, 256));
}

int launch_lstm_persist(const LstmPersistLaunch& P) {
    int G = 0, L = 0;
    if (!lstm_persist_supported(*P.hp, P.H, P.batch, P.device, &G, &L)) {
        set_error("internal: persistent recurrent kernel not available for this plan");
        return PIVOT_E_UNSUPPORTED;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(P.stream);
    {
        const size_t total = (size_t)P.steps * P.batch * P.hp->K_pad;
        const int blocks = (int)((total + 255) / 256 > 8192 ? 8192 : (total + 255) / 256);
        hipLaunchKernelGGL(lstm_prepare_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<const _Float16*>(P.xs),
                           P.h, P.pcol_pad, reinterpret_cast<_Float16*>(P.xg), P.xg_step_elems, P.H, P.I, P.hp->K_pad,
                           P.batch, total);
        HIP_TRY(hipGetLastError());
    }
    PersistArgs a;
    a.vals = reinterpret_cast<const _Float16*>(P.vals); a.col_idx = P.col_idx; a.row_ptr = P.row_ptr;
    a.invprow = P.invprow; a.pcol_pad = P.pcol_pad; a.bias_p = P.bias_p;
    a.xs = reinterpret_cast<const _Float16*>(P.xs); a.xg = reinterpret_cast<_Float16*>(P.xg); a.xg_step = P.xg_step_elems;
    a.partials = reinterpret_cast<unsigned long long*>(P.partials); a.ctl = P.ctl; a.h = P.h; a.c = P.c; a.z_dbg = P.z_dbg;
    a.T = P.hp->T; a.nbr = P.hp->nbr; a.H = P.H; a.I = P.I; a.K_pad = P.hp->K_pad; a.batch = P.batch; a.steps = P.steps; a.L = L;
    const size_t smem = (size_t)4 * L * kSlot * 4;
    // (that all workgroups fit on the device at once was checked by lstm_persist_supported)
    if (L <= 8) hipLaunchKernelGGL(lstm_persist_kernel<8>, dim3(G), dim3(kNT), smem, st, a);
    else        hipLaunchKernelGGL(lstm_persist_kernel<16>, dim3(G), dim3(kNT), smem, st, a);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

}  // namespace pivot
