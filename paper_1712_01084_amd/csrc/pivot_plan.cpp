// Host-side plan builder: the static "compile" step of the PBP form (paper
// Eq. 1 and Section 4.2.1).  Pure CPU code, integer work and bit copies only.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <numeric>

#include "pivot_internal.h"

namespace pivot {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

const char* last_error() { return g_error; }

static bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

bool device_supported(const pivot_fc_desc& d, std::string* why) {
    auto fail = [&](const char* m) { if (why) *why = m; return false; };
    if (!is_pow2(d.bh) || !is_pow2(d.bw)) return fail("tile sides must be powers of two on the device path");
    if (d.bh < 8 || d.bh > 64 || d.bw < 8 || d.bw > 64) return fail("tile sides must lie in 8..64 on the device path");
    return true;
}

int max_chunk_tiles(const pivot_fc_desc& d) {
    // the vector kernel stages up to 4 batch rows of the chunk's x-segments in LDS
    const int lds_budget = 48 * 1024;
    int per_tile = d.bw * 4 * elem_size(d.wdtype);
    return std::max(1, lds_budget / std::max(1, per_tile));
}

void choose_schedule(HostPlan& hp) {
    const pivot_fc_desc& d = hp.d;
    const size_t tile_bytes = (size_t)d.bh * d.bw * elem_size(d.wdtype);
    int max_row = 0;
    for (int i = 0; i < hp.nbr; ++i) max_row = std::max(max_row, hp.row_ptr[i + 1] - hp.row_ptr[i]);

    // Measured on MI355X (GPU-side time of back-to-back launches): a block row that
    // is cut in pieces pays about 1.2 us for the hand-over between workgroups, 16
    // wavefronts per workgroup about 0.7 us more than 4, and the best point is about
    // one workgroup per compute unit.  So: slice rows (no hand-over) until there are
    // about 256 work items, keep block rows whole unless LDS forces a cut or a work
    // item would stream 256 KB or more while compute units sit idle, and size the
    // workgroup to the bytes it streams.
    int sl = d.row_slices;
    if (sl == 0) {
        // slices of whole 1 KB wave-loads first
        const int vec = 16 / elem_size(d.wdtype);
        const int rpw = 64 / std::max(1, d.bw / vec);
        sl = 1;
        while (sl < 8 && hp.nbr * sl < 256 && d.bh / (sl * 2) >= rpw &&
               fc_row_slices(FcShape{d.layout, d.wdtype, d.bh, d.bw, 0, 0, 0, 0}, 1, sl * 2) == sl * 2) sl *= 2;
        // Still fewer work items than compute units, block rows that will stay whole (under 256 KB per work item)
        // and enough left per work item (16 KB): shorter slices, where a wave-load takes the same rows of several
        // consecutive tiles.  Measured on 4096x4096 with 64x16 fp16 tiles (64 block rows: 128 -> 256 work items):
        // cold 4.19 -> 3.94 us at 10 % kept, 5.25 -> 4.87 at 25 %, 7.20 -> 6.60 at 50 %; with 11 KB per work item
        // (1024x1024, 16x16 tiles) it costs 0.1 us, and where rows get cut anyway (dense) it costs 0.3 us cold.
        const size_t row_bytes = (size_t)max_row * tile_bytes;
        while (sl < 8 && hp.nbr * sl < 256 && row_bytes / sl < 256 * 1024 && row_bytes / (sl * 2) >= 16 * 1024 &&
               fc_row_slices(FcShape{d.layout, d.wdtype, d.bh, d.bw, 0, 0, 0, 0}, 1, sl * 2) == sl * 2) sl *= 2;
    }
    if (d.device >= 0) sl = fc_row_slices(FcShape{d.layout, d.wdtype, d.bh, d.bw, 0, 0, 0, 0}, 1, sl);
    hp.row_slices = sl;

    const size_t slice_bytes = std::max<size_t>(1, tile_bytes / sl);
    int ct = d.chunk_tiles;
    if (ct == 0) {
        const int cap = max_chunk_tiles(d);
        int parts = std::max(1, (max_row + cap - 1) / cap);
        while ((size_t)hp.nbr * sl * parts < 256 && (size_t)max_row * slice_bytes / parts >= 256 * 1024) parts *= 2;
        ct = std::max(1, (max_row + parts - 1) / parts);
        // Strongly skewed masks (the longest block row at least four times the average one): the few long rows set
        // the launch time while most work items are short, so long rows are cut in spite of the hand-over, into
        // pieces of twice the average row, kept between 32 and 96 KB per work item.  Measured with per-row counts
        // following a Zipf profile, cold, batch 1 / batch 4 (8 for fp16), whole rows -> pieces: 8192x3072 16x32
        // fp16 5.95 -> 5.6 / 12.0 -> 7.9 us (a step of the launch-per-step recurrent form 11.0 -> 8.9);
        // 4096x4096 32x32 fp32 8.7 -> 6.6 / 14.2 -> 9.1; 2048x8192 16x16 fp32 8.4 -> 7.0 / 15.8 -> 10.5;
        // 4096x9216 32x32 fp32 9.5 -> 8.4 / 16.6 -> 13.3 (pieces of 32 KB there: 11.6 / 14.4).  Warm launches at
        // batch 1 lose up to 0.7 us to the hand-over.
        if (hp.nbr > 0 && (long long)max_row * hp.nbr >= 4LL * hp.T) {
            const int lo = (int)std::max<size_t>(1, (32 * 1024) / slice_bytes), hi = (int)std::max<size_t>(1, (96 * 1024) / slice_bytes);
            const int want = std::min(hi, std::max(lo, 2 * ((hp.T + hp.nbr - 1) / hp.nbr)));
            if (want < ct) ct = want;
        }
    }
    if (d.device >= 0) ct = std::min(ct, max_chunk_tiles(d));
    build_schedule(hp, ct);

    int nw = d.wg_waves;
    if (nw == 0) {
        const size_t big = (size_t)std::min(ct, std::max(max_row, 1)) * slice_bytes;
        // (one wavefront per work item up to 8 KB: no workgroup barrier, no reduction across wavefronts; measured
        // on square block-diagonal layers of size 64-4096, warm: 2.2-2.6 -> 2.0-2.4 us up to 8 KB per work item,
        // 2.6 -> 2.75 and 2.6 -> 3.0 us at 16 KB.  Batch 1 only: other batches run such plans with 4.)
        nw = big <= 8 * 1024 ? 1 : (big <= 32 * 1024 ? 4 : (big <= 256 * 1024 ? 8 : 16));
    }
    hp.wg_waves = nw;
}

void build_schedule(HostPlan& hp, int chunk_tiles) {
    hp.chunk_tiles = chunk_tiles;
    struct C { int32_t br, b, e, slot; };
    std::vector<C> cs;
    hp.part_base.assign(hp.nbr + 1, 0);
    hp.max_parts = 1;
    for (int i = 0; i < hp.nbr; ++i) {
        int b = hp.row_ptr[i], e = hp.row_ptr[i + 1];
        int first = (int)cs.size();
        if (b == e) cs.push_back({i, b, e, (int32_t)cs.size()});
        for (int s = b; s < e; s += chunk_tiles) {
            int n = std::min(chunk_tiles, e - s);
            cs.push_back({i, s, s + n, (int32_t)cs.size()});
        }
        hp.part_base[i + 1] = (int32_t)cs.size();
        hp.max_parts = std::max(hp.max_parts, (int)cs.size() - first);
    }
    // regular schedule: same number of tiles in every block row, all chunks full
    hp.uniform_ct = hp.uniform_parts = 0;
    if (hp.nbr > 0 && hp.T > 0 && hp.T % hp.nbr == 0) {
        const int per_row = hp.T / hp.nbr;
        bool same = per_row % chunk_tiles == 0 || per_row <= chunk_tiles;
        for (int i = 0; i < hp.nbr && same; ++i) same = (hp.row_ptr[i + 1] - hp.row_ptr[i]) == per_row;
        if (same) {
            hp.uniform_ct = std::min(per_row, chunk_tiles);
            hp.uniform_parts = per_row / hp.uniform_ct;
        }
    }
    std::stable_sort(cs.begin(), cs.end(), [](const C& a, const C& b) { return (a.e - a.b) > (b.e - b.b); });
    hp.nchunks = (int)cs.size();
    hp.chunks.resize((size_t)hp.nchunks * 4);
    for (int j = 0; j < hp.nchunks; ++j) {
        hp.chunks[4 * j + 0] = cs[j].br;
        hp.chunks[4 * j + 1] = cs[j].b;
        hp.chunks[4 * j + 2] = cs[j].e;
        hp.chunks[4 * j + 3] = cs[j].slot;
    }
}

static int check_permutation(const int32_t* p, int n, const char* name, std::vector<int32_t>& inv) {
    inv.assign(n, -1);
    for (int i = 0; i < n; ++i) {
        int32_t v = p[i];
        if (v < 0 || v >= n) {
            set_error("%s[%d] = %d is outside 0..%d", name, i, v, n - 1);
            return PIVOT_E_NOT_PERMUTATION;
        }
        if (inv[v] != -1) {
            set_error("%s is not a bijection: value %d appears at %d and %d", name, v, inv[v], i);
            return PIVOT_E_NOT_PERMUTATION;
        }
        inv[v] = i;
    }
    return PIVOT_OK;
}

template <typename E>
static void pack_tiles(const HostPlan& hp, const E* W, int w_space, const int32_t* prow, const int32_t* pcol, E* out) {
    const int M = hp.d.M, K = hp.d.K, bh = hp.d.bh, bw = hp.d.bw, layout = hp.d.layout;
    const size_t T = (size_t)hp.T;
    for (int i = 0; i < hp.nbr; ++i) {
        for (int t = hp.row_ptr[i]; t < hp.row_ptr[i + 1]; ++t) {
            const int j = hp.col_idx[t];
            for (int r = 0; r < bh; ++r) {
                const int R = i * bh + r;
                const E* src_row = nullptr;
                if (R < M) src_row = W + (size_t)(w_space == PIVOT_W_PIVOTED ? R : prow[R]) * K;
                for (int c = 0; c < bw; ++c) {
                    const int C = j * bw + c;
                    E v = E(0);
                    if (src_row && C < K) v = src_row[w_space == PIVOT_W_PIVOTED ? C : pcol[C]];
                    size_t off;
                    if (layout == PIVOT_BRC)      off = ((size_t)t * bh + r) * bw + c;
                    else if (layout == PIVOT_BCR) off = ((size_t)t * bw + c) * bh + r;
                    else                          off = ((size_t)c * T + t) * bh + r;
                    out[off] = v;
                }
            }
        }
    }
}

// The gather lists of the LDS-fed matrix-core kernel (see HostPlan::xsort): per
// work item, the staged positions in ascending order of the address they read.
// Tiles of a block row are in ascending block column, so the block-order list
// is already sorted; the natural-order list is sorted here (stable, padding last).
void build_sorted_gather(HostPlan& hp) {
    const pivot_fc_desc& d = hp.d;
    hp.xsort.clear(); hp.xsort_blk.clear(); hp.sorted_ok = false;
    if (d.layout != PIVOT_BRC || mfma_kind(d.wdtype, d.bh, d.bw) < 0) return;
    if (hp.K_pad >= kSortSrcNone || (long long)hp.chunk_tiles * d.bw > (1ll << (32 - kSortSrcBits))) return;
    const size_t n = (size_t)hp.T * d.bw;
    hp.xsort.resize(n); hp.xsort_blk.resize(n);
    std::vector<int32_t> order;
    for (int j = 0; j < hp.nchunks; ++j) {
        const size_t e0 = (size_t)hp.chunks[(size_t)4 * j + 1] * d.bw, e1 = (size_t)hp.chunks[(size_t)4 * j + 2] * d.bw;
        const int ne = (int)(e1 - e0);
        order.resize(ne);
        std::iota(order.begin(), order.end(), 0);
        const int32_t* src = hp.xidx.data() + e0;
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
            const unsigned ka = src[a] < 0 ? 0xFFFFFFFFu : (unsigned)src[a], kb = src[b] < 0 ? 0xFFFFFFFFu : (unsigned)src[b];
            return ka < kb;
        });
        for (int i = 0; i < ne; ++i) {
            const int e = order[i];
            const uint32_t s = src[e] < 0 ? (uint32_t)kSortSrcNone : (uint32_t)src[e];
            hp.xsort[e0 + i] = (int32_t)(s | ((uint32_t)e << kSortSrcBits));
            const size_t g = e0 + i;                    // block order: position i reads column col_idx[t]*bw + c
            // (tiles are listed by ascending block column, so the padding columns, which only the last block
            // column has, come last here as well)
            const uint32_t col = (uint32_t)hp.col_idx[g / d.bw] * d.bw + (uint32_t)(g % d.bw);
            const uint32_t sb = col < (uint32_t)d.K ? col : (uint32_t)kSortSrcNone;
            hp.xsort_blk[g] = (int32_t)(sb | ((uint32_t)i << kSortSrcBits));
        }
    }
    hp.sorted_ok = true;
}

int build_host_plan(const pivot_fc_desc& d, const void* W, int w_space, const uint8_t* tile_mask,
                    const int32_t* prow, const int32_t* pcol, const float* bias, HostPlan& hp) {
    if (!W || !tile_mask || !prow || !pcol) { set_error("W, tile_mask, prow and pcol are required"); return PIVOT_E_NULL; }
    if (d.M <= 0 || d.K <= 0 || d.bh <= 0 || d.bw <= 0) { set_error("M, K, bh, bw must be positive"); return PIVOT_E_SHAPE; }
    if ((int64_t)d.M * d.K > (int64_t)1 << 40) { set_error("matrix too large"); return PIVOT_E_SHAPE; }
    if (d.wdtype != PIVOT_F32 && d.wdtype != PIVOT_F16) { set_error("unknown wdtype %d", d.wdtype); return PIVOT_E_UNSUPPORTED; }
    if (d.layout != PIVOT_BRC && d.layout != PIVOT_BCR && d.layout != PIVOT_CBR) { set_error("unknown layout %d", d.layout); return PIVOT_E_UNSUPPORTED; }
    if (d.act != PIVOT_ACT_NONE && d.act != PIVOT_ACT_RELU) { set_error("unknown activation %d", d.act); return PIVOT_E_UNSUPPORTED; }
    if (w_space != PIVOT_W_NATURAL && w_space != PIVOT_W_PIVOTED) { set_error("unknown weight space %d", w_space); return PIVOT_E_UNSUPPORTED; }
    if (d.chunk_tiles < 0) { set_error("chunk_tiles must be >= 0"); return PIVOT_E_SHAPE; }
    if (d.flags & ~(PIVOT_PLAN_GATHER_FROM_GLOBAL | PIVOT_PLAN_LSTM_LAUNCH_PER_STEP | PIVOT_PLAN_GATHER_FROM_LDS_COPY | PIVOT_PLAN_LSTM_ONE_LAUNCH_ALWAYS)) { set_error("unknown flags"); return PIVOT_E_UNSUPPORTED; }
    if (d.wg_waves != 0 && d.wg_waves != 1 && d.wg_waves != 4 && d.wg_waves != 8 && d.wg_waves != 16) { set_error("wg_waves must be 0, 1, 4, 8 or 16"); return PIVOT_E_UNSUPPORTED; }
    if (d.row_slices != 0 && d.row_slices != 1 && d.row_slices != 2 && d.row_slices != 4 && d.row_slices != 8) { set_error("row_slices must be 0, 1, 2, 4 or 8"); return PIVOT_E_UNSUPPORTED; }

    hp.d = d;
    hp.nbr = (d.M + d.bh - 1) / d.bh;
    hp.nbc = (d.K + d.bw - 1) / d.bw;
    hp.M_pad = hp.nbr * d.bh;
    hp.K_pad = hp.nbc * d.bw;

    int rc = check_permutation(prow, d.M, "prow", hp.invprow);
    if (rc) return rc;
    rc = check_permutation(pcol, d.K, "pcol", hp.invpcol);
    if (rc) return rc;

    try {
        hp.row_ptr.assign(hp.nbr + 1, 0);
        hp.col_idx.clear();
        for (int i = 0; i < hp.nbr; ++i) {
            for (int j = 0; j < hp.nbc; ++j)
                if (tile_mask[(size_t)i * hp.nbc + j]) hp.col_idx.push_back(j);
            if (hp.col_idx.size() > (size_t)INT32_MAX) { set_error("too many tiles"); return PIVOT_E_SHAPE; }
            hp.row_ptr[i + 1] = (int32_t)hp.col_idx.size();
        }
        hp.T = (int)hp.col_idx.size();
        size_t nvals = (size_t)hp.T * d.bh * d.bw;
        if (nvals * elem_size(d.wdtype) > ((size_t)1 << 36)) { set_error("kept tiles exceed 64 GiB"); return PIVOT_E_SHAPE; }
        hp.vals.assign(nvals * elem_size(d.wdtype), 0);
        if (d.wdtype == PIVOT_F32)
            pack_tiles<uint32_t>(hp, (const uint32_t*)W, w_space, prow, pcol, (uint32_t*)hp.vals.data());
        else
            pack_tiles<uint16_t>(hp, (const uint16_t*)W, w_space, prow, pcol, (uint16_t*)hp.vals.data());

        hp.bias_p.assign(hp.M_pad, 0.0f);
        if (bias) for (int r = 0; r < d.M; ++r) hp.bias_p[r] = bias[prow[r]];
        hp.prow_pad.assign(hp.M_pad, -1);
        std::copy(prow, prow + d.M, hp.prow_pad.begin());
        hp.pcol_pad.assign(hp.K_pad, -1);
        std::copy(pcol, pcol + d.K, hp.pcol_pad.begin());

        hp.xidx.resize((size_t)hp.T * d.bw);
        for (int t = 0; t < hp.T; ++t)
            for (int c = 0; c < d.bw; ++c) hp.xidx[(size_t)t * d.bw + c] = hp.pcol_pad[(size_t)hp.col_idx[t] * d.bw + c];

        choose_schedule(hp);
        build_sorted_gather(hp);
    } catch (const std::bad_alloc&) {
        set_error("out of host memory while building the plan");
        return PIVOT_E_ALLOC;
    }
    return PIVOT_OK;
}

}  // namespace pivot
