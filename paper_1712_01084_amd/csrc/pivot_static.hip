// pivot_fc_run_static: the layer entry point for callers that can neither
// allocate device memory nor hand over a workspace (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  The scratch
// of a run (arrival counters and partial sums of split block rows, and the
// block-order copy of x that one matrix-core form reads) lives in a file-scope
// device array of fixed size instead of a caller's buffer; the kernels are the
// ones pivot_fc_run launches and take the array's address as an argument just
// as they take the workspace there.
#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>

#include "pivot_fc_kernels.h"

namespace pivot {

namespace {

// [arrival counters][partial sums, then the block-order copy of x].  The counter region is only ever used for
// counters, whatever plan runs: every run leaves its counters at zero (the last workgroup to arrive resets
// them), so no call has to clear anything for the next one, and nothing a run keeps in the second region is
// read before the same run has written it.
constexpr size_t kCounterBytes = PIVOT_STATIC_COUNTER_BYTES;
constexpr size_t kDataBytes    = PIVOT_STATIC_DATA_BYTES;
static __device__ __align__(256) unsigned char scratch[kCounterBytes + kDataBytes];

// In host code `scratch` is only a handle for the runtime, not an address a kernel could use: the address of
// each device's own copy is asked for once, with that device current, and kept here.
constexpr int kMaxDevices = 64;
std::atomic<unsigned char*> g_scratch[kMaxDevices];
std::mutex g_setup;

int scratch_of(int device, void* stream, unsigned char** out) {
    if (device < 0 || device >= kMaxDevices) { set_error("device ordinal %d outside 0..%d", device, kMaxDevices - 1); return PIVOT_E_UNSUPPORTED; }
    unsigned char* p = g_scratch[device].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_setup);
        p = g_scratch[device].load(std::memory_order_acquire);
        if (!p) {
            int prev = -1;
            HIP_TRY(hipGetDevice(&prev));
            if (prev != device) HIP_TRY(hipSetDevice(device));
            void* addr = nullptr;
            const hipError_t e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
            // the counters start at zero (the array is zero when the code object is loaded; cleared here once
            // more, by a kernel, so that a caller that is capturing its stream records no memset node)
            int rc = PIVOT_OK;
            if (e == hipSuccess && addr) rc = launch_fill_zero(addr, kCounterBytes, stream);
            if (prev != device) (void)hipSetDevice(prev);
            if (e != hipSuccess || !addr) { set_error("hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e)); return PIVOT_E_HIP; }
            if (rc != PIVOT_OK) return rc;
            p = static_cast<unsigned char*>(addr);
            g_scratch[device].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return PIVOT_OK;
}

}  // namespace

}  // namespace pivot

using namespace pivot;

extern "C" {

int pivot_fc_run_static(const pivot_fc_plan_t* plan, const void* x_dev, int64_t ldx, void* y_dev, int64_t ldy,
                        int batch, void* stream) {
    if (!plan) { set_error("plan is NULL"); return PIVOT_E_NULL; }
    if (plan->device < 0) { set_error("host-only plan (device = -1) cannot run"); return PIVOT_E_NO_DEVICE; }
    if (batch < 1 || batch > 64) { set_error("batch %d outside 1..64", batch); return PIVOT_E_SHAPE; }
    const HostPlan& h = plan->host;
    const size_t nt = fc_ticket_bytes(h), np = fc_partial_bytes(h, batch), ng = fc_gather_bytes(h, batch);
    if (nt > kCounterBytes || np + ng > kDataBytes) {
        set_error("this plan at batch %d needs %zu bytes of arrival counters and %zu bytes of partial sums and staged "
                  "input; the built-in scratch holds %zu and %zu: use pivot_fc_run with a workspace",
                  batch, nt, np + ng, kCounterBytes, kDataBytes);
        return PIVOT_E_WORKSPACE;
    }
    unsigned char* base = nullptr;
    const int rc = scratch_of(plan->device, stream, &base);
    if (rc != PIVOT_OK) return rc;
    return run_layer(plan, x_dev, ldx, y_dev, ldy, batch, base, base + kCounterBytes, base + kCounterBytes + np, stream);
}

}  // extern "C"
