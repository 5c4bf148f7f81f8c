// Chooses the kernel, the row slicing and the launch shape for one layer
// application and sizes its workspace.
#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "pivot_fc_kernels.h"

namespace pivot {

// Compute units of the current device (asked once per device).
static int device_cus() {
    static int cus[16] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return 1; }
    int& c = cus[dev & 15];
    if (c == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) c = n;
        else { (void)hipGetLastError(); c = 1; }
    }
    return c;
}

// Batch rows the LDS-fed matrix-core kernel stages: 4, or 8 (batch 9..16 then runs as two launch rows of 8, each
// workgroup gathering half the rows: staging all 16 in one workgroup was measured slower at every density, 6.0 ->
// 4.7 us at 5 % kept and 13.4 -> 12.3 at 50 % on 4096x4096, where 16 rows no longer fit; four launch rows of 4
// were slower again from 10 % kept on: the weights are then streamed four times).
static int mfma_lds_rows(int batch) { return batch <= 4 ? 4 : 8; }

// Which kernel applies the layer:
//   kPathVector      batch 1-2 (and whatever the matrix cores cannot take): FMA / dot2 against x staged in LDS
//   kPathMfmaLds     fp16, batch >= 3: MFMA with the B fragments read from x staged in LDS (4 or 8 batch rows per launch row)
//   kPathMfmaGather  fp16, batch >= 8 otherwise: MFMA with B fragments read from an x in block order
// Every work item of the LDS-fed form gathers its own x-segments for all batch rows (rows * tiles * bw
// elements), the block-order form gathers x once in a launch of its own.  Measured (4096x4096, 64x16 tiles):
// at batch 3-4 the LDS-fed form beats the vector kernel at every density (LDS reads per weight load 4 -> 1).
// From batch 8 on the gather decides: read in the order of the tile list every element costs a cache line per
// batch row, and the form lost beyond a few thousand staged elements (dense, batch 8: 14.2 -> 18.6 us); read
// through the plan's source-ordered lists (neighbouring lanes, neighbouring addresses) it wins wherever the
// staged rows fit in 48 KB of LDS (batch 8: 7.6 -> 5.4 us at 10 % kept, 9.8 -> 7.4 at 25 %, 12.3 -> 10.1 at
// 50 %, 14.2 -> 12.4 dense; batch 16: 7.3 -> 6.1 at 5 %, 11.0 -> 9.5 at 25 %).  Letting it take up to 136 KB of
// LDS (one workgroup per compute unit) for 16 staged rows at 50 % and dense was measured too: 13.5 -> 13.2 us and
// 14.5 -> 15.4 us, so longer rows stay with the block-order form.
//   kPathMfmaXrow    fp16, batch 5-16: MFMA with the B fragments gathered from a copy of the rows of x in LDS
// At batch 9-16 the staging itself bounds the LDS-fed form (16 rows x staged columns two-byte gathers per work
// item, repeated by every row slice, and the weights streamed once per launch row of 8); gathering where the
// fragment is formed needs one copy of x per work item instead, whatever the number of staged columns.  The copy
// costs a work item 1.5-2.3 us (4096 columns: 128 KB through one compute unit's memory pipeline before its first
// MFMA), the gathers 0.2-0.9 us, so the form is taken from a quarter of the columns staged per work item on
// (4096x4096, 64x16 tiles, batch 16, cold: 8.3 -> 7.1 us at 25 % kept, 12.5 -> 9.1 at 50 %, 14.9 -> 12.7 dense;
// at 10 % it would lose, 6.0 -> 6.3, at 5 % 4.8 -> 6.3).  Batch 5-8 takes it under the same rule (only the rows
// that exist are copied; same matrix, batch 8: 6.5 -> 6.1 us at 25 %, 9.65 -> 8.1 at 50 %, 12.45 -> 11.7 dense,
// batch 5 the same within 0.1 us; warm 0.2 us slower at 25 %, 0.3-0.45 faster above); at batch 4 it loses
// (5.6 -> 6.0, 7.7 -> 7.9, 9.8 -> 11.1).
int fc_path(const FcShape& s, int batch) {
    const int layout = s.layout, wdtype = s.wdtype, bh = s.bh, bw = s.bw, lds_tiles = s.lds_tiles;
    // the matrix-core kernels read A fragments from row-major (BRC) tiles only
    if (layout != PIVOT_BRC || mfma_kind(wdtype, bh, bw) < 0 || batch < 3) return kPathVector;
    if (batch >= 5 && batch <= 16 && s.xrow_len > 0 && s.chunk_tiles > 0) {
        // 16 rows of x (each with 16 zeroed bytes behind it) and the work item's gather indices in LDS; a lane
        // copies at most 8 vectors of a row, a thread at most 4 int4 of indices
        const size_t vecs = ((size_t)s.xrow_len + 7) / 8;
        const size_t cols = ((size_t)s.chunk_tiles + 1) * bw;
        const size_t lds = 16 * (vecs * 16 + 16) + cols * 4;
        // "a quarter of the columns staged per work item": at batch 5-8 of the AVERAGE work item.  With a few
        // long block rows among many short ones most work items copy all of x for a handful of tiles, which the
        // 8-row LDS-fed form does not: 8192x3072, 16x32 tiles, per-row counts from 96 down to 2, batch 8, x
        // already in block order (a step of the recurrent layer): 11.0 -> 12.0 us.  (With x in natural order the
        // copy wins on that matrix too, 12.0 -> 10.4 us, and on 4096x4096 with the same profile it loses at batch
        // 16 and wins at batch 5-8; the path does not depend on where x comes from, and batch 9-16 keeps the rule
        // it was measured with.)
        const size_t rule_cols = batch <= 8 ? ((size_t)s.mean_tiles + 1) * bw : cols;
        if (vecs <= 512 && cols <= 8192 && lds <= 156 * 1024 && rule_cols * 4 >= (size_t)s.xrow_len) return kPathMfmaXrow;
    }
    if (lds_tiles > 0) {
        const int rows = mfma_lds_rows(batch);
        const size_t xs_bytes = (size_t)rows * ((size_t)lds_tiles * bw + 8 + 16) * 2;   // + the paired form's zeroed columns
        // every launch row of 8 batch rows streams the weights again and gathers its own rows: beyond two launch
        // rows the form is kept while the launch rows together stage at most 5120 columns per work item
        // (4096x4096, 64x16 tiles: batch 24 at 5 / 25 % kept 7.9 -> 5.6 us, 12.1 -> 10.7; batch 64 at 5 %
        // 9.8 -> 8.5; but batch 24 dense 16.1 -> 19.1 and batch 64 at 25 % 14.4 -> 21.0, which stay with the
        // block-order form)
        const size_t launch_rows = (size_t)(batch + rows - 1) / rows;
        if (xs_bytes <= 48 * 1024 && (launch_rows <= 2 || launch_rows * lds_tiles * bw <= 5120)) return kPathMfmaLds;
    }
    return batch >= 8 ? kPathMfmaGather : kPathVector;
}

bool fc_uses_matrix_cores(const FcShape& s, int batch) {
    return fc_path(s, batch) == kPathMfmaGather;
}

// Batch rows one launch row covers in the kernel's epilogue and in the workspace (grid.y repeats it).
int fc_batch_tile(const FcShape& s, int batch) {
    if (s.layout != PIVOT_BRC) return 1;     // the column-major kernels take one batch row per launch row
    const int path = fc_path(s, batch);
    if (path == kPathMfmaGather) return mfma_kind(s.wdtype, s.bh, s.bw) == 0 ? 16 : 32;
    if (path == kPathMfmaLds) return mfma_lds_rows(batch);
    if (path == kPathMfmaXrow) return 16;
    return batch >= 3 ? 4 : batch;
}

// Largest number of row slices <= want that the chosen kernel supports: a
// slice of the vector kernel has at least 8 rows and is a whole number of 1 KB
// wave-loads or a whole fraction of one (a wave-load then takes the same rows
// of several consecutive tiles), a slice of the matrix kernel whole MFMA row blocks.
int fc_row_slices(const FcShape& s, int batch, int want) {
    const int layout = s.layout, wdtype = s.wdtype, bh = s.bh, bw = s.bw;
    if (layout != PIVOT_BRC) return 1;       // a row slice is contiguous only in row-major tiles
    int sl = want < 1 ? 1 : want;
    // The LDS-fed matrix-core kernel beyond 8 batch rows (several launch rows of 8): every row slice of a block
    // row stages the same x-segments again, so at most two slices (4096x4096, 64x16 tiles, cold, four slices ->
    // two: 10 % kept, batch 12 / 16 / 24 / 32 / 64: 5.9 -> 5.4, 5.9 -> 5.4, 7.2 -> 6.4, 8.45 -> 7.1, 12.8 -> 10.3
    // us; 25 % kept, batch 24 / 32: 10.8 -> 9.3, 12.7 -> 10.2; one slice: 6.6 at batch 16; up to batch 8 four
    // slices are the faster, 4.9 against 5.3 us).
    if (sl > 2 && batch > 8 && fc_path(s, batch) == kPathMfmaLds) sl = 2;
    while (sl > 1) {
        bool ok = (bh % sl == 0);
        const int bhs = bh / sl;
        if (ok) {
            const int path = fc_path(s, batch);
            if (path != kPathVector) {
                // whole MFMA row blocks: 16 rows (32 for tiles 16 columns wide, except in the kernels fed from
                // LDS, which pair such tiles)
                const int mr = (mfma_kind(wdtype, bh, bw) == 0 || (path != kPathMfmaGather && bw == 16)) ? 16 : 32;
                ok = (bhs % mr == 0);
            } else {
                const int vec = 16 / elem_size(wdtype);
                const int rpw = 64 / (bw / vec > 0 ? bw / vec : 1);
                ok = bhs >= 8 && (bhs % rpw == 0 || rpw % bhs == 0);
            }
        }
        if (ok) break;
        sl /= 2;
    }
    return sl;
}

// Arrival counters of split block rows: one 256-byte line per (launch row, block row, row slice).  The region is
// sized for the largest number of launch rows any batch up to 64 can have, so that its size, and with it the
// place of everything that follows it in a workspace, does not depend on the batch of a run: counters are only
// ever touched as counters (every run leaves them at zero), never overlaid by another batch's partial sums.
// Plans without split block rows use no counters.
size_t fc_ticket_bytes(const HostPlan& hp) {
    if (hp.max_parts <= 1) return 0;
    int ngy_max = 1;
    for (int batch = 1; batch <= 64; ++batch) {
        const int nbt = fc_batch_tile(fc_shape(hp), batch);
        ngy_max = std::max(ngy_max, (batch + nbt - 1) / nbt);
    }
    // counters are sized for the plan's slice count (a launch may use fewer)
    return (size_t)4 * kTicketStride * hp.nbr * ngy_max * hp.row_slices;
}

size_t fc_partial_bytes(const HostPlan& hp, int batch) {
    if (hp.max_parts <= 1) return 0;
    const int nbt = fc_batch_tile(fc_shape(hp), batch);
    const int ngy = (batch + nbt - 1) / nbt;
    return align_up((size_t)4 * hp.nchunks * hp.d.bh * nbt * ngy, 256);
}

size_t fc_workspace_bytes(const HostPlan& hp, int batch) {
    if (batch < 1) return 0;
    return fc_ticket_bytes(hp) + fc_partial_bytes(hp, batch);
}

size_t fc_gather_bytes(const HostPlan& hp, int batch) {
    if (!fc_uses_matrix_cores(fc_shape(hp), batch)) return 0;
    return align_up((size_t)batch * hp.K_pad * elem_size(hp.d.wdtype), 256);
}

// "pivot::<kernel and template arguments>" as a profiler prints it
template <typename... A>
static std::string kernel_name(const char* fmt, A... args) {
    char buf[160];
    snprintf(buf, sizeof buf, fmt, args...);
    return std::string("pivot::") + buf;
}

int launch_fc(const FcLaunch& L, std::string* describe) {
    const FcShape shape{L.layout, L.wdtype, L.bh, L.bw, L.lds_tiles, L.chunk_tiles, L.xrow_len, mean_tiles_of(L.T, L.nchunks)};
    const int path = fc_path(shape, L.batch);
    const bool mc = path == kPathMfmaGather, ml = path == kPathMfmaLds, mx = path == kPathMfmaXrow;
    const int nbt = fc_batch_tile(shape, L.batch);
    const int ngy = (L.batch + nbt - 1) / nbt;
    const int sl = fc_row_slices(shape, L.batch, L.row_slices);
    const int bhs = L.bh / sl;
    int nw = (L.wg_waves == 16 || L.wg_waves == 8) ? L.wg_waves : 4;
    // one wavefront per work item: the vector kernel at batch 1 with the gather from global memory (tiny layers)
    const bool one_wave = L.wg_waves == 1 && L.layout == PIVOT_BRC && path == kPathVector && nbt == 1;
    if (one_wave) nw = 1;
    if (ml && nw > 8) nw = 8;                // the LDS-fed matrix-core kernel comes with 4 or 8 wavefronts
    const int es = elem_size(L.wdtype);

    FcArgs a;
    a.vals = L.vals; a.col_idx = L.col_idx; a.xidx = L.xidx; a.chunks = reinterpret_cast<const int4*>(L.chunks);
    a.part_base = L.part_base; a.bias_p = L.bias_p; a.scatter = L.scatter;
    a.x = L.x; a.y = L.y; a.partials = L.partials; a.tickets = L.tickets;
    a.ldx = L.ldx; a.ldy = L.ldy; a.batch = L.batch; a.act = L.act; a.out_f16 = L.out_f16;
    a.nchunks = L.nchunks; a.nbr = L.nbr;
    a.bh_full = L.bh; a.tile_elems = L.bh * L.bw;
    a.uniform_ct = L.uniform_ct; a.uniform_parts = L.uniform_parts;
    a.T = L.T; a.chunk_tiles = L.chunk_tiles;
    a.trace = nullptr;
#ifdef PIVOT_TRACE
    // timeline builds: where the vector kernel puts its time stamps (8 x int64 per wavefront of the launch)
    if (const char* e = getenv("PIVOT_TRACE_PTR")) a.trace = reinterpret_cast<long long*>(strtoull(e, nullptr, 0));
#endif
    dim3 grid(L.nchunks, ngy, sl);
    hipStream_t st = reinterpret_cast<hipStream_t>(L.stream);

    if (mc) {
        if (!L.x_block_order) { set_error("internal: the matrix-core kernel needs x in block order"); return PIVOT_E_UNSUPPORTED; }
        a.xs_stride = 0;
        const int rw = nw < 4 ? nw : 4;
        size_t smem = (size_t)rw * bhs * nbt * 4;
        if (describe) { *describe = kernel_name("fc_mfma_kernel<%d, %d, %d, %d>", mfma_kind(L.wdtype, L.bh, L.bw), bhs, L.bw, nw); return PIVOT_OK; }
        return launch_mfma_f16(a, mfma_kind(L.wdtype, L.bh, L.bw), bhs, L.bw, nw, grid, smem, st);
    }
    if (L.uniform_ct > 0xFFFF || L.uniform_parts > 0x7FFF) a.uniform_ct = a.uniform_parts = 0;   // packed into 16 bits each: fall back to loaded descriptors
    if (mx) {
        if (L.chunk_tiles > 0xFFFF || L.bh > 64) { set_error("shape outside the kernel's packed arguments"); return PIVOT_E_UNSUPPORTED; }
        const int xlen = L.x_block_order ? L.K_pad : L.K;
        int kind = mfma_kind(L.wdtype, L.bh, L.bw);
        if (kind == 1 && L.bw == 16 && bhs % 32 != 0) kind = 2;
        const int vecs = (xlen + 7) / 8;
        // rows copied with 16-byte loads when they are whole aligned vectors, densely packed; else element by element
        const bool vec_rows = xlen % 8 == 0 && L.ldx == xlen && (reinterpret_cast<uintptr_t>(L.x) & 15) == 0;
        a.xn_vecs = vecs | (vec_rows ? (1 << 17) : 0); a.xn_stride = xlen; a.xs_stride = 0;
        const size_t steps_cols = ((size_t)(a.uniform_ct > 0 ? a.uniform_ct : L.chunk_tiles) + 1) * L.bw;
        size_t smem = (size_t)16 * (vecs * 16 + 16) + steps_cols * 4;
        const size_t red_bytes = (size_t)8 * bhs * 16 * 4;
        smem = align_up(smem > red_bytes ? smem : red_bytes, 16);
        if (vecs > 512 || steps_cols > 8192 || smem > 158 * 1024) { set_error("internal: x does not fit the LDS copy (%zu bytes)", smem); return PIVOT_E_UNSUPPORTED; }
        if (describe) { *describe = kernel_name("fc_mfma_xrow_kernel<%d, %d, %d>", kind, bhs, L.bw); return PIVOT_OK; }
        return launch_mfma_xrow_f16(a, kind, bhs, L.bw, grid, smem, st);
    }
    // staged x: nbt rows of (tiles per chunk)*bw elements, plus 16 bytes whose last element is the dump slot
    // (the vector kernel derives the same stride from its preloaded arguments)
    // the LDS-fed matrix-core kernel takes slices that are not whole 32-row blocks of 16-column tiles as pairs
    // of tiles (16x16x32 MFMA) and keeps 16 zeroed columns after the last staged tile
    int kind = mfma_kind(L.wdtype, L.bh, L.bw);
    if (ml && kind == 1 && L.bw == 16 && bhs % 32 != 0) kind = 2;
    a.xs_stride = (a.uniform_ct > 0 ? a.uniform_ct : L.chunk_tiles) * L.bw + (ml && kind == 2 ? 16 : 0) + 16 / es;
    size_t xs_bytes = (size_t)nbt * a.xs_stride * es;
    size_t red_bytes = (size_t)nw * bhs * nbt * 4;
    // x-resident variant: every work item first copies the whole of x (nbt rows) into LDS with independent
    // coalesced loads and gathers from there.  Taken when the rows are 16-byte vectors (densely packed if there
    // is more than one: the kernel then derives the row stride from its preloaded arguments), a thread has to hold at
    // most 8 of them, everything fits in 64 KB of LDS, and the work item streams at least 32 KB of weights
    // (measured at batch 1, where the global form needs no barrier at all because every wavefront stages for
    // itself: below that the copy and its barrier cost 0.3 us warm and gain nothing cold, 1024x1024 fp32 3.19
    // either way, 4096x4096 fp32 at 10 % 4.02 / 4.03; at 40 KB they gain 0.2 us cold, 4096x4096 fp16 at 25 %
    // 4.75 -> 4.54; at 58 KB 0.3 us, 4096x9216 fp32 5.63 -> 5.27; dense 4096x4096 fp16 0.2 us).  With several batch rows the gather issues a load per element and
    // row, so there the copy is also taken as soon as it needs no more loads than the gather would
    // (4096x4096 fp16 at 10 % kept: batch 2 4.16 -> 4.02 us cold, batch 4 4.75 -> 4.43; at 25 %, batch 2:
    // 5.49 -> 4.98; at 5 %, where the gather is the shorter, the copy was 0.1 us slower; warm launches pay
    // 0.2-0.4 us for it).
    if (L.chunk_tiles > 0xFFFF || L.bh > 64 || L.batch > 64) { set_error("shape outside the vector kernel's packed arguments"); return PIVOT_E_UNSUPPORTED; }
    const int vec = 16 / es;
    const int xlen = L.x_block_order ? L.K_pad : L.K;
    int xres = 0;
    size_t xn_bytes = 0;
    const size_t item_bytes = (size_t)(a.uniform_ct > 0 ? a.uniform_ct : L.chunk_tiles) * bhs * L.bw * es;
    const size_t staged_cols = (size_t)(a.uniform_ct > 0 ? a.uniform_ct : L.chunk_tiles) * L.bw;
    if (L.layout == PIVOT_BRC && L.x_resident != 0 && !one_wave &&
        (L.x_resident == 2 || item_bytes >= 32 * 1024 || (nbt >= 2 && staged_cols * vec >= (size_t)xlen)) && xlen % vec == 0 && (nbt == 1 || L.ldx == xlen) &&
        (reinterpret_cast<uintptr_t>(L.x) & 15) == 0) {
        const size_t vectors = (size_t)nbt * (xlen / vec);
        xn_bytes = (size_t)nbt * xlen * es + 16;
        if (vectors <= (size_t)8 * nw * 64 && xn_bytes + xs_bytes <= 64 * 1024 && red_bytes <= 64 * 1024) {
            // form 1 (everything requested in one burst) for regular schedules whose work item is in flight whole
            // with the first loads (8 KB per wavefront); form 2 (x stored to LDS between the two halves of the
            // first weight loads) for irregular schedules and for longer work items, whose refills then start sooner
            xres = (a.uniform_ct > 0 && item_bytes <= (size_t)nw * 8 * 1024) ? 1 : 2;
        } else if (!ml && nbt == 1 && vectors <= (size_t)16 * 8 * 64 && xn_bytes + xs_bytes <= 144 * 1024 &&
                   (size_t)L.nchunks * sl <= (size_t)device_cus() &&
                   (L.x_resident == 2 || (size_t)(a.uniform_ct > 0 ? a.uniform_ct : L.chunk_tiles) * L.bw * 128 >= 2 * xn_bytes)) {
            // Long x (beyond 64 KB of LDS or 8 vectors per thread): 8 wavefronts hold up to 16 vectors each and
            // the workgroup takes most of the 160 KB of a compute unit, so this form is only used when every
            // work item still gets a compute unit of its own.  It replaces a gather that moves a whole cache
            // line per element by a copy that moves every line once (25088 inputs, 78 tiles per work item:
            // 320 KB of lines per work item against 100 KB), so it is taken only when the gathered lines are at
            // least twice the copy (16384 inputs, 8 tiles of 64 columns per work item: 64 KB either way, and the
            // copy was measured 0.6 us slower).
            xres = 3;
            nw = 8;
            red_bytes = (size_t)nw * bhs * nbt * 4;
        }
    }
    a.xn_vecs = xres ? xlen / vec : 0; a.xn_stride = xlen;
    size_t smem = xres ? xn_bytes + xs_bytes : xs_bytes;
    smem = align_up(smem > red_bytes ? smem : red_bytes, 16);
    if (smem > (size_t)(xres == 3 ? 150 : 64) * 1024) { set_error("chunk does not fit in LDS (%zu bytes)", smem); return PIVOT_E_UNSUPPORTED; }
    if (describe) {
        // the instantiation the per-path launchers pick for these values (they take 8 wavefronts for 16 where
        // they have no 16-wavefront form, and know one LDS-copy form where the vector kernel knows three)
        const char* wt = L.wdtype == PIVOT_F32 ? "float" : "_Float16";
        if (L.layout != PIVOT_BRC) *describe = kernel_name("fc_colmajor_kernel<%s, %d, %d, %d, %d>", wt, L.layout, L.bh, L.bw, nw >= 8 ? 8 : 4);
        else if (ml) *describe = kernel_name("fc_mfma_lds_kernel<%d, %d, %d, %d, %d, %d>", kind, bhs, L.bw, nbt, nw >= 8 ? 8 : 4, xres ? 2 : 0);
        else *describe = kernel_name("fc_gemv_kernel<%s, %d, %d, %d, %d, %d>", wt, bhs, L.bw, nbt, nw, xres);
        return PIVOT_OK;
    }
#if PIVOT_ABLATE & 32
    // ablation build without permutations: batch 1 through the vector kernel only, which then reads the tile
    // list's block columns where it otherwise reads the per-column gather index
    if (L.layout != PIVOT_BRC || ml || nbt != 1) { set_error("this ablation build runs BRC plans at batch 1 only"); return PIVOT_E_UNSUPPORTED; }
    a.xidx = L.col_idx;
#endif
    if (L.layout != PIVOT_BRC) return launch_colmajor(a, L.layout, L.wdtype, L.bh, L.bw, nw, grid, smem, st);
    if (ml) {
        if (!L.xsort) { set_error("internal: the LDS-fed matrix-core kernel needs the packed gather lists"); return PIVOT_E_UNSUPPORTED; }
        a.xidx = L.xsort;
    }
    if (ml) return launch_mfma_lds_f16(a, kind, bhs, L.bw, nbt, nw, xres, grid, smem, st);
    if (L.wdtype == PIVOT_F32) return launch_gemv_f32(a, bhs, L.bw, nbt, nw, xres, grid, smem, st);
    return launch_gemv_f16(a, bhs, L.bw, nbt, nw, xres, grid, smem, st);
}

}  // namespace pivot
