// C ABI of the library: argument checks, device upload, and the sequencing of
// kernel launches for single layers, chains and the recurrent loop.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>

#include "pivot_internal.h"

namespace pivot {
const char* last_error();
}

using namespace pivot;

#define API_HIP(expr, cleanup)                                                         \
    do {                                                                               \
        hipError_t e_ = (expr);                                                        \
        if (e_ != hipSuccess) {                                                        \
            set_error("%s failed: %s", #expr, hipGetErrorString(e_));                  \
            cleanup;                                                                   \
            return PIVOT_E_HIP;                                                        \
        }                                                                              \
    } while (0)

namespace {

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

struct Piece { const void* src; size_t bytes; void** dst; };

int upload(pivot_fc_plan_t* p) {
    HostPlan& h = p->host;
    DevPlan& d = p->dev;
    // device-only arrays: the gather index for an x already in block order, the identity scatter of chain
    // intermediates, and the schedule with each block row's piece range folded in (one load instead of two)
    std::vector<int32_t> xblk, rowid, chunks8;
    try {
        xblk.resize(h.xidx.size());
        rowid.assign(h.M_pad, -1);
        chunks8.assign((size_t)h.nchunks * 8, 0);
    } catch (const std::bad_alloc&) { set_error("out of host memory"); return PIVOT_E_ALLOC; }
    // (padding columns are -1 here too: a block-order x is never read past its K real columns, so whatever a
    // reused workspace holds there cannot reach a sum)
    for (int t = 0; t < h.T; ++t)
        for (int c = 0; c < h.d.bw; ++c) {
            const int col = h.col_idx[t] * h.d.bw + c;
            xblk[(size_t)t * h.d.bw + c] = col < h.d.K ? col : -1;
        }
    for (int r = 0; r < h.d.M; ++r) rowid[r] = r;
    for (int j = 0; j < h.nchunks; ++j) {
        for (int q = 0; q < 4; ++q) chunks8[(size_t)8 * j + q] = h.chunks[(size_t)4 * j + q];
        const int br = h.chunks[(size_t)4 * j];
        chunks8[(size_t)8 * j + 4] = h.part_base[br];
        chunks8[(size_t)8 * j + 5] = h.part_base[br + 1] - h.part_base[br];
    }
    Piece pieces[] = {
        {h.vals.data(),      h.vals.size(),                 (void**)&d.vals},
        {h.col_idx.data(),   h.col_idx.size() * 4,          (void**)&d.col_idx},
        {chunks8.data(),     chunks8.size() * 4,            (void**)&d.chunks},
        {h.part_base.data(), h.part_base.size() * 4,        (void**)&d.part_base},
        {h.bias_p.data(),    h.bias_p.size() * 4,           (void**)&d.bias_p},
        {h.prow_pad.data(),  h.prow_pad.size() * 4,         (void**)&d.prow_pad},
        {h.pcol_pad.data(),  h.pcol_pad.size() * 4,         (void**)&d.pcol_pad},
        {h.invprow.data(),   h.invprow.size() * 4,          (void**)&d.invprow},
        {h.invpcol.data(),   h.invpcol.size() * 4,          (void**)&d.invpcol},
        {h.xidx.data(),      h.xidx.size() * 4,             (void**)&d.xidx},
        {xblk.data(),        xblk.size() * 4,               (void**)&d.xidx_blk},
        {h.xsort.data(),     h.xsort.size() * 4,            (void**)&d.xsort},
        {h.xsort_blk.data(), h.xsort_blk.size() * 4,        (void**)&d.xsort_blk},
        {rowid.data(),       rowid.size() * 4,              (void**)&d.rowid_pad},
        {h.row_ptr.data(),   h.row_ptr.size() * 4,          (void**)&d.row_ptr},
    };
    size_t total = 0;
    // every array is followed by zeroed padding: 16 KB after the tile values (clamped
    // vector loads of an empty or last work item stay inside), 16 bytes after the others
    auto padded = [&](const Piece& pc) { return align_up(pc.bytes + (pc.src == (const void*)h.vals.data() ? kValsPadBytes : 16), 256); };
    for (auto& pc : pieces) total += padded(pc);
    DeviceGuard g(p->device);
    if (!g.ok) { set_error("cannot select device %d", p->device); return PIVOT_E_HIP; }
    void* base = nullptr;
    hipError_t e = hipMalloc(&base, total);
    if (e != hipSuccess) { set_error("hipMalloc(%zu) failed: %s", total, hipGetErrorString(e)); return PIVOT_E_ALLOC; }
    d.base = (char*)base;
    d.bytes = total;
    e = hipMemset(base, 0, total);
    if (e != hipSuccess) { set_error("hipMemset failed: %s", hipGetErrorString(e)); (void)hipFree(base); d = DevPlan{}; return PIVOT_E_HIP; }
    size_t off = 0;
    for (auto& pc : pieces) {
        *pc.dst = d.base + off;
        if (pc.bytes) {
            e = hipMemcpy(d.base + off, pc.src, pc.bytes, hipMemcpyHostToDevice);
            if (e != hipSuccess) {
                set_error("hipMemcpy to device failed: %s", hipGetErrorString(e));
                (void)hipFree(base);
                d = DevPlan{};
                return PIVOT_E_HIP;
            }
        }
        off += padded(pc);
    }
    return PIVOT_OK;
}

}  // namespace

extern "C" {

int pivot_version(void) { return PIVOT_VERSION; }

const char* pivot_last_error(void) { return pivot::last_error(); }

int pivot_fc_plan(const pivot_fc_desc* desc, const void* W, int w_space, const uint8_t* tile_mask,
                  const int32_t* prow, const int32_t* pcol, const float* bias, pivot_fc_plan_t** out) {
    if (out) *out = nullptr;
    if (!desc || !out) { set_error("desc and out are required"); return PIVOT_E_NULL; }
    if (desc->device >= 0) {
        std::string why;
        if (!device_supported(*desc, &why)) { set_error("%s", why.c_str()); return PIVOT_E_UNSUPPORTED; }
    }
    pivot_fc_plan_t* p = new (std::nothrow) pivot_fc_plan_t();
    if (!p) { set_error("out of host memory"); return PIVOT_E_ALLOC; }
    int rc = build_host_plan(*desc, W, w_space, tile_mask, prow, pcol, bias, p->host);
    if (rc != PIVOT_OK) { delete p; return rc; }
    p->device = desc->device;
    if (p->device >= 0) {
        rc = upload(p);
        if (rc != PIVOT_OK) { delete p; return rc; }
    }
    *out = p;
    return PIVOT_OK;
}

int pivot_fc_plan_host_view(const pivot_fc_plan_t* plan, pivot_plan_view* v) {
    if (!plan || !v) { set_error("plan and view are required"); return PIVOT_E_NULL; }
    const HostPlan& h = plan->host;
    v->M = h.d.M; v->K = h.d.K; v->bh = h.d.bh; v->bw = h.d.bw; v->wdtype = h.d.wdtype;
    v->layout = h.d.layout; v->act = h.d.act;
    v->nbr = h.nbr; v->nbc = h.nbc; v->M_pad = h.M_pad; v->K_pad = h.K_pad; v->T = h.T;
    v->chunk_tiles = h.chunk_tiles; v->wg_waves = h.wg_waves; v->row_slices = h.row_slices; v->nchunks = h.nchunks;
    v->row_ptr = h.row_ptr.data(); v->col_idx = h.col_idx.data(); v->vals = h.vals.data();
    v->bias_p = h.bias_p.data(); v->invprow = h.invprow.data(); v->invpcol = h.invpcol.data();
    v->prow_pad = h.prow_pad.data(); v->pcol_pad = h.pcol_pad.data();
    v->chunks = h.chunks.data(); v->part_base = h.part_base.data(); v->xidx = h.xidx.data();
    v->xsort = h.sorted_ok ? h.xsort.data() : nullptr; v->xsort_blk = h.sorted_ok ? h.xsort_blk.data() : nullptr;
    return PIVOT_OK;
}

int pivot_fc_plan_clone(const pivot_fc_plan_t* plan, pivot_fc_plan_t** out) {
    if (out) *out = nullptr;
    if (!plan || !out) { set_error("plan and out are required"); return PIVOT_E_NULL; }
    pivot_fc_plan_t* p = new (std::nothrow) pivot_fc_plan_t();
    if (!p) { set_error("out of host memory"); return PIVOT_E_ALLOC; }
    try {
        p->host = plan->host;
    } catch (const std::bad_alloc&) {
        delete p;
        set_error("out of host memory");
        return PIVOT_E_ALLOC;
    }
    p->device = plan->device;
    if (p->device >= 0) {
        int rc = upload(p);
        if (rc != PIVOT_OK) { delete p; return rc; }
    }
    *out = p;
    return PIVOT_OK;
}

void pivot_fc_plan_destroy(pivot_fc_plan_t* plan) {
    if (!plan) return;
    if (plan->dev.base) {
        DeviceGuard g(plan->device);
        (void)hipFree(plan->dev.base);
    }
    delete plan;
}

size_t pivot_fc_workspace_bytes(const pivot_fc_plan_t* plan, int batch) {
    if (!plan || batch < 1) return 0;
    return fc_workspace_bytes(plan->host, batch) + fc_gather_bytes(plan->host, batch);
}

int pivot_workspace_init(void* ws_dev, size_t ws_bytes, void* stream) {
    if (!ws_dev && ws_bytes) { set_error("workspace pointer is NULL"); return PIVOT_E_NULL; }
    return launch_fill_zero(ws_dev, ws_bytes, stream);
}

}  // extern "C"

namespace {

// Fills the plan-dependent part of a launch.  `tickets`: fc_ticket_bytes(plan) of arrival counters that are zero
// between runs; `partials`: fc_partial_bytes(plan, batch) of scratch (both may be NULL when the size is 0).
int prepare(const pivot_fc_plan_t* plan, int batch, void* tickets, void* partials, FcLaunch& L) {
    if (!plan) { set_error("plan is NULL"); return PIVOT_E_NULL; }
    if (plan->device < 0) { set_error("host-only plan (device = -1) cannot run"); return PIVOT_E_NO_DEVICE; }
    if (batch < 1 || batch > 64) { set_error("batch %d outside 1..64", batch); return PIVOT_E_SHAPE; }
    const HostPlan& h = plan->host;
    if ((fc_ticket_bytes(h) > 0 && !tickets) || (fc_partial_bytes(h, batch) > 0 && !partials)) { set_error("workspace missing"); return PIVOT_E_WORKSPACE; }
    if (reinterpret_cast<uintptr_t>(tickets) % 16 != 0 || reinterpret_cast<uintptr_t>(partials) % 16 != 0) { set_error("workspace must be 16-byte aligned"); return PIVOT_E_WORKSPACE; }
    const DevPlan& d = plan->dev;
    L.vals = d.vals; L.col_idx = d.col_idx; L.chunks = d.chunks; L.part_base = d.part_base; L.bias_p = d.bias_p;
    L.K = h.d.K; L.x_resident = (h.d.flags & PIVOT_PLAN_GATHER_FROM_GLOBAL) ? 0 : ((h.d.flags & PIVOT_PLAN_GATHER_FROM_LDS_COPY) ? 2 : 1);
    L.M_pad = h.M_pad; L.K_pad = h.K_pad; L.bh = h.d.bh; L.bw = h.d.bw; L.wdtype = h.d.wdtype; L.layout = h.d.layout; L.T = h.T; L.act = h.d.act;
    L.nchunks = h.nchunks; L.nbr = h.nbr; L.chunk_tiles = h.chunk_tiles; L.wg_waves = h.wg_waves;
    L.lds_tiles = h.lds_tiles(); L.xrow_len = h.xrow_len();
    L.row_slices = h.row_slices;
    L.uniform_ct = h.uniform_ct; L.uniform_parts = h.uniform_parts;
    L.batch = batch;
    L.tickets = reinterpret_cast<uint32_t*>(tickets);
    L.partials = reinterpret_cast<float*>(partials);
    return PIVOT_OK;
}

// Input side of a launch whose x is in natural order: the vector kernel
// gathers through the composed index array; the matrix-core kernel wants block
// order, so x is copied there first (`xg`: fc_gather_bytes of scratch).
int natural_input(const pivot_fc_plan_t* plan, const void* x_dev, int64_t ldx, int batch, void* xg, void* stream,
                  FcLaunch& L) {
    const HostPlan& h = plan->host;
    if (fc_uses_matrix_cores(fc_shape(h), batch)) {
        int rc = launch_gather_x(x_dev, ldx, plan->dev.pcol_pad, xg, h.K_pad, batch, h.d.wdtype, stream);
        if (rc != PIVOT_OK) return rc;
        L.x = xg; L.ldx = h.K_pad; L.xidx = plan->dev.xidx_blk; L.xsort = plan->host.sorted_ok ? plan->dev.xsort_blk : nullptr; L.x_block_order = 1;
    } else {
        L.x = x_dev; L.ldx = ldx; L.xidx = plan->dev.xidx; L.xsort = plan->host.sorted_ok ? plan->dev.xsort : nullptr; L.x_block_order = 0;
    }
    return PIVOT_OK;
}

}  // namespace

namespace pivot {

int run_layer(const pivot_fc_plan_t* plan, const void* x_dev, int64_t ldx, void* y_dev, int64_t ldy, int batch,
              void* tickets, void* partials, void* xg, void* stream) {
    FcLaunch L{};
    int rc = prepare(plan, batch, tickets, partials, L);
    if (rc != PIVOT_OK) return rc;
    if (!x_dev || !y_dev) { set_error("x_dev and y_dev are required"); return PIVOT_E_NULL; }
    if (ldx < plan->host.d.K || ldy < plan->host.d.M) { set_error("ldx/ldy smaller than K/M"); return PIVOT_E_SHAPE; }
    if (fc_gather_bytes(plan->host, batch) > 0 && !xg) { set_error("workspace missing"); return PIVOT_E_WORKSPACE; }
    rc = natural_input(plan, x_dev, ldx, batch, xg, stream, L);
    if (rc != PIVOT_OK) return rc;
    L.scatter = plan->dev.prow_pad;
    L.y = y_dev; L.ldy = ldy; L.out_f16 = 0; L.stream = stream;
    return launch_fc(L);
}

}  // namespace pivot

extern "C" {

int pivot_fc_run(const pivot_fc_plan_t* plan, const void* x_dev, int64_t ldx, void* y_dev, int64_t ldy,
                 int batch, void* ws_dev, size_t ws_bytes, void* stream) {
    if (!plan) { set_error("plan is NULL"); return PIVOT_E_NULL; }
    if (plan->device < 0) { set_error("host-only plan (device = -1) cannot run"); return PIVOT_E_NO_DEVICE; }
    if (batch < 1 || batch > 64) { set_error("batch %d outside 1..64", batch); return PIVOT_E_SHAPE; }
    const HostPlan& h = plan->host;
    const size_t nt = fc_ticket_bytes(h), np = fc_partial_bytes(h, batch), ng = fc_gather_bytes(h, batch);
    if (nt + np + ng > 0 && (!ws_dev || ws_bytes < nt + np + ng)) {
        set_error("workspace too small: need %zu bytes, got %zu", nt + np + ng, ws_dev ? ws_bytes : (size_t)0);
        return PIVOT_E_WORKSPACE;
    }
    char* ws = reinterpret_cast<char*>(ws_dev);
    return run_layer(plan, x_dev, ldx, y_dev, ldy, batch, ws, ws + nt, ws + nt + np, stream);
}

// ------------------------------------------------------------------ chains

int pivot_mlp_plan(pivot_fc_plan_t* const* layers, int Lcount, int flags, pivot_mlp_plan_t** out) {
    if (out) *out = nullptr;
    if (!layers || !out) { set_error("layers and out are required"); return PIVOT_E_NULL; }
    if (Lcount < 1) { set_error("a chain needs at least one layer"); return PIVOT_E_SHAPE; }
    if (flags & ~(PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER | PIVOT_MLP_LAUNCH_PER_LAYER)) { set_error("unknown flags"); return PIVOT_E_UNSUPPORTED; }
    for (int l = 0; l < Lcount; ++l) {
        if (!layers[l]) { set_error("layer %d is NULL", l); return PIVOT_E_NULL; }
        if (layers[l]->host.d.wdtype != layers[0]->host.d.wdtype || layers[l]->device != layers[0]->device) {
            set_error("all layers of a chain must share wdtype and device");
            return PIVOT_E_UNSUPPORTED;
        }
        if (l > 0 && layers[l]->host.d.K != layers[l - 1]->host.d.M) {
            set_error("layer %d takes %d inputs but layer %d produces %d", l, layers[l]->host.d.K, l - 1, layers[l - 1]->host.d.M);
            return PIVOT_E_SHAPE;
        }
    }
    pivot_mlp_plan_t* mp = new (std::nothrow) pivot_mlp_plan_t();
    if (!mp) { set_error("out of host memory"); return PIVOT_E_ALLOC; }
    try {
        mp->layers.assign(layers, layers + Lcount);
        mp->flags = flags;
        mp->device = layers[0]->device;
        for (int l = 0; l + 1 < Lcount; ++l) {
            const HostPlan& a = layers[l]->host;
            const HostPlan& b = layers[l + 1]->host;
            std::vector<int32_t> q(b.d.K), dst(a.M_pad, -1);
            bool ident = true;
            for (int c = 0; c < b.d.K; ++c) {            // q[c] = invprow_l[pcol_{l+1}[c]]
                q[c] = a.invprow[b.pcol_pad[c]];
                ident = ident && (q[c] == c);
            }
            for (int r = 0; r < a.d.M; ++r) dst[r] = b.invpcol[a.prow_pad[r]];
            mp->q.push_back(std::move(q));
            mp->dst.push_back(std::move(dst));
            mp->identity.push_back(ident ? 1 : 0);
        }
        for (auto& v : mp->q) mp->q_ptrs.push_back(v.data());
        for (auto& v : mp->dst) mp->dst_ptrs.push_back(v.data());
    } catch (const std::bad_alloc&) {
        delete mp;
        set_error("out of host memory");
        return PIVOT_E_ALLOC;
    }
    if (mp->device >= 0 && Lcount > 1) {
        size_t total = 0;
        for (auto& v : mp->dst) total += align_up(v.size() * 4, 256);
        DeviceGuard g(mp->device);
        // one-launch form: control words and a buffer of (value, tag) pairs per boundary, zeroed once
        std::vector<const HostPlan*> hps;
        for (int l = 0; l < Lcount; ++l) hps.push_back(&layers[l]->host);
        mp->persist_ok = !(flags & PIVOT_MLP_LAUNCH_PER_LAYER) &&
                         chain_persist_supported(hps, mp->device, &mp->persist_grid, &mp->persist_smem, &mp->persist_smem_copy, nullptr);
        const size_t persist_off = total;
        if (mp->persist_ok) {
            total += align_up(chain_persist_ctl_bytes(), 256);
            for (int l = 0; l + 1 < Lcount; ++l) total += align_up((size_t)layers[l + 1]->host.K_pad * 8, 256);
        }
        void* base = nullptr;
        hipError_t e = hipMalloc(&base, total);
        if (e != hipSuccess) { set_error("hipMalloc(%zu) failed: %s", total, hipGetErrorString(e)); delete mp; return PIVOT_E_ALLOC; }
        mp->dev_base = (char*)base;
        size_t off = 0;
        for (auto& v : mp->dst) {
            e = hipMemcpy(mp->dev_base + off, v.data(), v.size() * 4, hipMemcpyHostToDevice);
            if (e != hipSuccess) { set_error("hipMemcpy failed: %s", hipGetErrorString(e)); (void)hipFree(base); delete mp; return PIVOT_E_HIP; }
            mp->dst_dev.push_back(reinterpret_cast<int32_t*>(mp->dev_base + off));
            off += align_up(v.size() * 4, 256);
        }
        if (mp->persist_ok) {
            e = hipMemset(mp->dev_base + persist_off, 0, total - persist_off);
            if (e != hipSuccess) { set_error("hipMemset failed: %s", hipGetErrorString(e)); (void)hipFree(base); delete mp; return PIVOT_E_HIP; }
            off = persist_off;
            mp->persist_ctl = reinterpret_cast<uint32_t*>(mp->dev_base + off);
            off += align_up(chain_persist_ctl_bytes(), 256);
            for (int l = 0; l + 1 < Lcount; ++l) {
                mp->persist_pairs.push_back(reinterpret_cast<unsigned long long*>(mp->dev_base + off));
                off += align_up((size_t)layers[l + 1]->host.K_pad * 8, 256);
            }
        }
    }
    *out = mp;
    return PIVOT_OK;
}

int pivot_mlp_plan_host_view(const pivot_mlp_plan_t* plan, pivot_mlp_view* v) {
    if (!plan || !v) { set_error("plan and view are required"); return PIVOT_E_NULL; }
    v->L = (int32_t)plan->layers.size();
    v->flags = plan->flags;
    v->q = plan->q_ptrs.data();
    v->dst = plan->dst_ptrs.data();
    v->identity = plan->identity.data();
    v->one_launch = plan->persist_ok ? 1 : 0;
    return PIVOT_OK;
}

void pivot_mlp_plan_destroy(pivot_mlp_plan_t* plan) {
    if (!plan) return;
    if (plan->dev_base) {
        DeviceGuard g(plan->device);
        (void)hipFree(plan->dev_base);
    }
    delete plan;
}

}  // extern "C"

namespace {

// Workspace of a chain: [arrival counters of layer 0] [of layer 1] ... [partial sums of layer 0] ... [block-order
// copy of x (matrix path)] [intermediate 0] ...  The counters come first and their sizes do not depend on the
// batch, so they are only ever touched as counters, whatever batches the workspace is reused with (they rely on
// being zero between launches; every run leaves them so).  Every layer has its own.
// Intermediate l holds batch rows of K_pad_{l+1} elements of wdtype in the consumer's block order; its padding
// columns are never read by the kernels that stage x in LDS (their gather index is -1 there) and are cleared
// before a kernel that reads the rows directly.
struct MlpLayout { size_t gather_off, total; std::vector<size_t> inter_off, ticket_off, partial_off; };

MlpLayout mlp_layout(const pivot_mlp_plan_t* mp, int batch) {
    MlpLayout m{0, 0, {}, {}, {}};
    size_t off = 0;
    for (auto* l : mp->layers) { m.ticket_off.push_back(off); off += align_up(fc_ticket_bytes(l->host), 256); }
    for (auto* l : mp->layers) { m.partial_off.push_back(off); off += align_up(fc_partial_bytes(l->host, batch), 256); }
    m.gather_off = off;
    off += fc_gather_bytes(mp->layers[0]->host, batch);
    for (size_t l = 0; l + 1 < mp->layers.size(); ++l) {
        m.inter_off.push_back(off);
        off += align_up((size_t)batch * mp->layers[l + 1]->host.K_pad * elem_size(mp->layers[l + 1]->host.d.wdtype), 256);
    }
    m.total = off;
    return m;
}

}  // namespace

extern "C" {

size_t pivot_mlp_workspace_bytes(const pivot_mlp_plan_t* plan, int batch) {
    if (!plan || batch < 1) return 0;
    return mlp_layout(plan, batch).total;
}

int pivot_mlp_run(const pivot_mlp_plan_t* plan, const void* x_dev, int64_t ldx, void* y_dev, int64_t ldy,
                  int batch, void* ws_dev, size_t ws_bytes, void* stream) {
    if (!plan) { set_error("plan is NULL"); return PIVOT_E_NULL; }
    if (!x_dev || !y_dev) { set_error("x_dev and y_dev are required"); return PIVOT_E_NULL; }
    if (plan->device < 0) { set_error("host-only chain cannot run"); return PIVOT_E_NO_DEVICE; }
    if (batch < 1 || batch > 64) { set_error("batch %d outside 1..64", batch); return PIVOT_E_SHAPE; }
    MlpLayout m = mlp_layout(plan, batch);
    if (!ws_dev || ws_bytes < m.total) { set_error("workspace too small: need %zu bytes", m.total); return PIVOT_E_WORKSPACE; }
    const int Lc = (int)plan->layers.size();
    const bool keep = (plan->flags & PIVOT_MLP_KEEP_FINAL_BLOCK_ORDER) != 0;
    const pivot_fc_plan_t* last = plan->layers[Lc - 1];
    if (ldx < plan->layers[0]->host.d.K || ldy < (keep ? last->host.M_pad : last->host.d.M)) { set_error("ldx/ldy too small"); return PIVOT_E_SHAPE; }
    char* ws = reinterpret_cast<char*>(ws_dev);
    if (batch == 1 && plan->persist_ok) {
        // the whole chain in one launch; intermediates are the plan's own (value, tag) pairs
        ChainPersistLaunch C;
        C.ctl = plan->persist_ctl; C.grid = plan->persist_grid; C.smem = plan->persist_smem; C.smem_copy = plan->persist_smem_copy;
        C.bw = plan->layers[0]->host.d.bw; C.wdtype = plan->layers[0]->host.d.wdtype; C.stream = stream;
        for (int l = 0; l < Lc; ++l) {
            const pivot_fc_plan_t* p = plan->layers[l];
            ChainPersistLayer s{};
            s.hp = &p->host; s.vals = p->dev.vals; s.chunks = p->dev.chunks; s.bias_p = p->dev.bias_p;
            s.xidx = l == 0 ? p->dev.xidx : p->dev.xidx_blk;
            s.in = l == 0 ? x_dev : static_cast<const void*>(plan->persist_pairs[l - 1]);
            if (l + 1 < Lc) {
                s.dst = plan->identity[l] ? p->dev.rowid_pad : plan->dst_dev[l];
                s.out = plan->persist_pairs[l];
            } else {
                s.dst = keep ? p->dev.rowid_pad : p->dev.prow_pad;
                s.out = y_dev;
            }
            C.layers.push_back(s);
        }
        return launch_chain_persist(C);
    }
    for (int l = 0; l < Lc; ++l) {
        const pivot_fc_plan_t* p = plan->layers[l];
        FcLaunch L{};
        int rc = prepare(p, batch, ws + m.ticket_off[l], ws + m.partial_off[l], L);
        if (rc != PIVOT_OK) return rc;
        L.stream = stream;
        if (l == 0) {
            rc = natural_input(p, x_dev, ldx, batch, ws + m.gather_off, stream, L);
            if (rc != PIVOT_OK) return rc;
        } else {
            L.xidx = p->dev.xidx_blk; L.xsort = p->host.sorted_ok ? p->dev.xsort_blk : nullptr; L.x = ws + m.inter_off[l - 1]; L.ldx = p->host.K_pad; L.x_block_order = 1;
            // the kernel that reads its B fragments straight from the rows also reads the padding columns
            // (against zero weights): they must hold finite values, whatever the workspace held before
            if (p->host.K_pad > p->host.d.K && fc_uses_matrix_cores(fc_shape(p->host), batch) &&
                (rc = launch_zero_pad_cols(ws + m.inter_off[l - 1], p->host.d.K, p->host.K_pad, batch, elem_size(p->host.d.wdtype), stream)) != PIVOT_OK) return rc;
        }
        if (l + 1 < Lc) {
            // producer-side store through the composed boundary array; identity boundaries store contiguously
            L.scatter = plan->identity[l] ? p->dev.rowid_pad : plan->dst_dev[l];
            L.y = ws + m.inter_off[l];
            L.ldy = plan->layers[l + 1]->host.K_pad;
            L.out_f16 = (p->host.d.wdtype == PIVOT_F16);
        } else {
            L.scatter = keep ? p->dev.rowid_pad : p->dev.prow_pad;
            L.y = y_dev; L.ldy = ldy; L.out_f16 = 0;
        }
        rc = launch_fc(L);
        if (rc != PIVOT_OK) return rc;
    }
    return PIVOT_OK;
}

int pivot_mlp_status(const pivot_mlp_plan_t* plan, void* stream, int* status) {
    if (!plan || !status) { set_error("plan and status are required"); return PIVOT_E_NULL; }
    *status = 0;
    if (!plan->persist_ok) return PIVOT_OK;
    DeviceGuard g(plan->device);
    API_HIP(hipStreamSynchronize(reinterpret_cast<hipStream_t>(stream)), (void)0);
    char* word = reinterpret_cast<char*>(plan->persist_ctl) + chain_persist_status_offset();
    uint32_t st = 0;
    API_HIP(hipMemcpy(&st, word, 4, hipMemcpyDeviceToHost), (void)0);
    if (st != 0) API_HIP(hipMemset(word, 0, 4), (void)0);
    *status = (int)st;
    return PIVOT_OK;
}

int pivot_mlp_status_word(const pivot_mlp_plan_t* plan, const uint32_t** word_dev) {
    if (!plan || !word_dev) { set_error("plan and word_dev are required"); return PIVOT_E_NULL; }
    *word_dev = nullptr;
    if (!plan->persist_ok) return PIVOT_OK;
    *word_dev = reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(plan->persist_ctl) + chain_persist_status_offset());
    return PIVOT_OK;
}

// --------------------------------------------------------------- recurrence

}  // extern "C"

namespace {

// [launch-per-step form: arrival counters, partial sums][gate pre-activations][control words + partials of the
// one-launch form][inputs of all steps]
struct LstmLayout { size_t tickets, scratch, z_off, ctl_off, part_off, xg_off, xg_step, total; };

LstmLayout lstm_layout(const pivot_fc_plan_t* p, int steps, int batch) {
    LstmLayout m{};
    m.tickets = fc_ticket_bytes(p->host);
    m.scratch = align_up(fc_workspace_bytes(p->host, batch), 256);
    m.z_off = m.scratch;
    m.ctl_off = m.z_off + align_up((size_t)batch * p->host.d.M * 4, 256);
    m.part_off = m.ctl_off + kLstmCtlBytes;
    m.xg_off = m.part_off + lstm_persist_partial_bytes(p->host, batch);
    m.xg_step = align_up((size_t)batch * p->host.K_pad * elem_size(p->host.d.wdtype), 256);
    m.total = m.xg_off + m.xg_step * (size_t)(steps > 0 ? steps : 1);
    return m;
}

}  // namespace

extern "C" {

size_t pivot_lstm_workspace_bytes(const pivot_fc_plan_t* plan, int H, int I, int steps, int batch) {
    if (!plan || batch < 1 || steps < 0) return 0;
    (void)H; (void)I;
    return lstm_layout(plan, steps, batch).total;
}

int pivot_lstm_run(const pivot_fc_plan_t* plan, int H, int I, const void* xs_dev, float* h_dev, float* c_dev,
                   float* z_dbg, int steps, int batch, void* ws_dev, size_t ws_bytes, void* stream) {
    if (!plan) { set_error("plan is NULL"); return PIVOT_E_NULL; }
    if (!xs_dev || !h_dev || !c_dev) { set_error("xs_dev, h_dev and c_dev are required"); return PIVOT_E_NULL; }
    if (plan->device < 0) { set_error("host-only plan cannot run"); return PIVOT_E_NO_DEVICE; }
    const HostPlan& h = plan->host;
    if (H < 1 || I < 0 || h.d.M != 4 * H || h.d.K != H + I) { set_error("plan is %dx%d, expected 4H x (H+I) with H=%d I=%d", h.d.M, h.d.K, H, I); return PIVOT_E_SHAPE; }
    if (steps < 0 || batch < 1 || batch > 64) { set_error("bad steps/batch"); return PIVOT_E_SHAPE; }
    if (steps == 0) return PIVOT_OK;
    LstmLayout m = lstm_layout(plan, steps, batch);
    if (!ws_dev || ws_bytes < m.total) { set_error("workspace too small: need %zu bytes", m.total); return PIVOT_E_WORKSPACE; }
    char* ws = reinterpret_cast<char*>(ws_dev);
    float* z = reinterpret_cast<float*>(ws + m.z_off);
    char* xg = ws + m.xg_off;
    int rc;
    // (fewer than 4 steps: loading every tile into registers first does not pay yet)
    if (!(h.d.flags & PIVOT_PLAN_LSTM_LAUNCH_PER_STEP) && (steps >= 4 || (h.d.flags & PIVOT_PLAN_LSTM_ONE_LAUNCH_ALWAYS)) && lstm_persist_supported(h, H, batch, plan->device, nullptr, nullptr)) {
        // one launch for the whole sequence
        // control words + the partial buffers this sequence will use
        if ((rc = launch_fill_zero(ws + m.ctl_off, (m.part_off - m.ctl_off) + lstm_persist_used_partial_bytes(h, batch, steps), stream)) != PIVOT_OK) return rc;
        LstmPersistLaunch P{};
        P.hp = &h;
        P.vals = plan->dev.vals; P.col_idx = plan->dev.col_idx; P.row_ptr = plan->dev.row_ptr;
        P.invprow = plan->dev.invprow; P.invpcol = plan->dev.invpcol; P.pcol_pad = plan->dev.pcol_pad; P.bias_p = plan->dev.bias_p;
        P.xs = xs_dev; P.xg = xg; P.xg_step_elems = m.xg_step / elem_size(h.d.wdtype);
        P.partials = ws + m.part_off;
        P.ctl = reinterpret_cast<uint32_t*>(ws + m.ctl_off);
        P.h = h_dev; P.c = c_dev; P.z_dbg = z_dbg;
        P.H = H; P.I = I; P.batch = batch; P.steps = steps; P.device = plan->device; P.stream = stream;
        return launch_lstm_persist(P);
    }
    // one layer launch and one cell launch per step
    if ((rc = launch_fill_zero(ws + m.ctl_off, kLstmCtlBytes, stream)) != PIVOT_OK) return rc;
    // block-order inputs of all steps: padding zero, x_t placed once, h_0 placed into step 0
    if ((rc = launch_fill_zero(xg, m.xg_step * (size_t)steps, stream)) != PIVOT_OK) return rc;
    if (m.xg_step != (size_t)batch * h.K_pad * elem_size(h.d.wdtype)) {
        // steps are padded apart: place step by step
        for (int t = 0; t < steps; ++t) {
            const char* xs_t = reinterpret_cast<const char*>(xs_dev) + (size_t)t * batch * I * elem_size(h.d.wdtype);
            if ((rc = launch_lstm_place_inputs(xs_t, xg + m.xg_step * (size_t)t, plan->dev.invpcol, H, I, h.K_pad, 1, batch, h.d.wdtype, stream)) != PIVOT_OK) return rc;
        }
    } else {
        if ((rc = launch_lstm_place_inputs(xs_dev, xg, plan->dev.invpcol, H, I, h.K_pad, steps, batch, h.d.wdtype, stream)) != PIVOT_OK) return rc;
    }
    if ((rc = launch_lstm_place_state(h_dev, xg, plan->dev.invpcol, H, h.K_pad, batch, h.d.wdtype, stream)) != PIVOT_OK) return rc;
    for (int t = 0; t < steps; ++t) {
        FcLaunch L{};
        rc = prepare(plan, batch, ws, ws + m.tickets, L);
        if (rc != PIVOT_OK) return rc;
        L.xidx = plan->dev.xidx_blk; L.xsort = plan->host.sorted_ok ? plan->dev.xsort_blk : nullptr; L.x_block_order = 1;
        L.x = xg + m.xg_step * (size_t)t; L.ldx = h.K_pad;
        L.scatter = plan->dev.prow_pad;      // gates land in natural order for the cell
        L.y = z; L.ldy = h.d.M; L.out_f16 = 0; L.stream = stream;
        if ((rc = launch_fc(L)) != PIVOT_OK) return rc;
        LstmCellLaunch C{};
        C.z = z; C.invpcol = plan->dev.invpcol;
        C.h = h_dev; C.c = c_dev;
        C.xg_next = (t + 1 < steps) ? (void*)(xg + m.xg_step * (size_t)(t + 1)) : nullptr;
        C.z_dbg = (t + 1 == steps) ? z_dbg : nullptr;
        C.H = H; C.M_pad = h.M_pad; C.K_pad = h.K_pad; C.batch = batch; C.wdtype = h.d.wdtype; C.stream = stream;
        if ((rc = launch_lstm_cell(C)) != PIVOT_OK) return rc;
    }
    return PIVOT_OK;
}

int pivot_lstm_status(const pivot_fc_plan_t* plan, int steps, int batch, const void* ws_dev, void* stream, int* status) {
    if (!plan || !ws_dev || !status) { set_error("plan, ws_dev and status are required"); return PIVOT_E_NULL; }
    if (plan->device < 0) { set_error("host-only plan"); return PIVOT_E_NO_DEVICE; }
    LstmLayout m = lstm_layout(plan, steps, batch);
    uint32_t word = 0;
    DeviceGuard g(plan->device);
    API_HIP(hipStreamSynchronize(reinterpret_cast<hipStream_t>(stream)), (void)0);
    API_HIP(hipMemcpy(&word, reinterpret_cast<const char*>(ws_dev) + m.ctl_off + 1024, 4, hipMemcpyDeviceToHost), (void)0);
    *status = (int)word;
    return PIVOT_OK;
}

int pivot_lstm_status_word(const pivot_fc_plan_t* plan, int steps, int batch, const void* ws_dev, const uint32_t** word_dev) {
    if (!plan || !ws_dev || !word_dev) { set_error("plan, ws_dev and word_dev are required"); return PIVOT_E_NULL; }
    LstmLayout m = lstm_layout(plan, steps, batch);
    *word_dev = reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(ws_dev) + m.ctl_off + 1024);
    return PIVOT_OK;
}

int pivot_fc_kernel_name(const pivot_fc_plan_t* plan, int batch, char* buf, size_t buf_len) {
    if (!plan || !buf || buf_len == 0) { set_error("plan and buf are required"); return PIVOT_E_NULL; }
    buf[0] = 0;
    if (batch < 1 || batch > 64) { set_error("batch %d outside 1..64", batch); return PIVOT_E_SHAPE; }
    FcLaunch L{};
    const HostPlan& h = plan->host;
    L.K = h.d.K; L.x_resident = (h.d.flags & PIVOT_PLAN_GATHER_FROM_GLOBAL) ? 0 : ((h.d.flags & PIVOT_PLAN_GATHER_FROM_LDS_COPY) ? 2 : 1);
    L.M_pad = h.M_pad; L.K_pad = h.K_pad; L.bh = h.d.bh; L.bw = h.d.bw; L.wdtype = h.d.wdtype; L.layout = h.d.layout; L.T = h.T; L.act = h.d.act;
    L.nchunks = h.nchunks; L.nbr = h.nbr; L.chunk_tiles = h.chunk_tiles; L.wg_waves = h.wg_waves;
    L.lds_tiles = h.lds_tiles(); L.xrow_len = h.xrow_len(); L.row_slices = h.row_slices; L.uniform_ct = h.uniform_ct; L.uniform_parts = h.uniform_parts;
    L.batch = batch;
    // a natural-order x, 16-byte aligned, rows densely packed (what the matrix-core form reads is its own copy)
    const bool blk = fc_uses_matrix_cores(fc_shape(h), batch);
    L.x = reinterpret_cast<const void*>(uintptr_t(256)); L.ldx = blk ? h.K_pad : h.d.K; L.x_block_order = blk ? 1 : 0;
    L.xsort = h.sorted_ok ? reinterpret_cast<const int32_t*>(uintptr_t(256)) : nullptr;
    std::string name;
    int rc = launch_fc(L, &name);
    if (rc != PIVOT_OK) return rc;
    snprintf(buf, buf_len, "%s", name.c_str());
    return PIVOT_OK;
}

int pivot_null_run(void* stream) { return launch_null(stream); }

int pivot_exchange_probe_run(void* scratch_dev, size_t scratch_bytes, int rounds, void* stream) {
    if (!scratch_dev) { set_error("scratch_dev is required"); return PIVOT_E_NULL; }
    if (scratch_bytes < PIVOT_PROBE_SCRATCH_BYTES || (reinterpret_cast<uintptr_t>(scratch_dev) & 255) != 0) { set_error("the probe needs %zu bytes of scratch, 256-byte aligned", (size_t)PIVOT_PROBE_SCRATCH_BYTES); return PIVOT_E_WORKSPACE; }
    if (rounds < 1 || rounds > 100000) { set_error("rounds %d outside 1..100000", rounds); return PIVOT_E_SHAPE; }
    return launch_exchange_probe(scratch_dev, rounds, stream);
}

int pivot_stream_read_run(const void* buf_dev, size_t bytes, float* out_dev, void* stream) {
    if (!buf_dev || !out_dev) { set_error("buf_dev and out_dev are required"); return PIVOT_E_NULL; }
    if (bytes < 1024 || bytes > ((size_t)1 << 40) || (reinterpret_cast<uintptr_t>(buf_dev) & 15) != 0) { set_error("bytes must be >= 1024 and the buffer 16-byte aligned"); return PIVOT_E_SHAPE; }
    return launch_stream_read(buf_dev, bytes, out_dev, stream);
}

int pivot_csr_run(const int32_t* row_ptr_dev, const int32_t* col_dev, const void* val_dev, int wdtype, int M,
                  int64_t nnz, const void* x_dev, const float* bias_dev, float* y_dev, int act, void* stream) {
    if (!row_ptr_dev || !x_dev || !y_dev || (nnz > 0 && (!col_dev || !val_dev))) { set_error("row_ptr, col, val, x and y are required"); return PIVOT_E_NULL; }
    if (M < 1 || nnz < 0) { set_error("bad shape"); return PIVOT_E_SHAPE; }
    if (wdtype != PIVOT_F32 && wdtype != PIVOT_F16) { set_error("unknown wdtype"); return PIVOT_E_UNSUPPORTED; }
    return launch_csr(row_ptr_dev, col_dev, val_dev, wdtype, M, nnz, x_dev, bias_dev, y_dev, act, stream);
}

int pivot_dense_run(const void* W_dev, int wdtype, int M, int K, const void* x_dev, int64_t ldx,
                    const float* bias_dev, void* y_dev, int64_t ldy, int batch, int act, void* stream) {
    if (!W_dev || !x_dev || !y_dev) { set_error("W_dev, x_dev and y_dev are required"); return PIVOT_E_NULL; }
    if (M < 1 || K < 1 || ldx < K || ldy < M) { set_error("bad shape"); return PIVOT_E_SHAPE; }
    if (wdtype != PIVOT_F32 && wdtype != PIVOT_F16) { set_error("unknown wdtype"); return PIVOT_E_UNSUPPORTED; }
    return launch_dense(W_dev, wdtype, M, K, x_dev, ldx, bias_dev, y_dev, ldy, batch, act, stream);
}

}  // extern "C"
