// Utility kernels around the layer kernels: workspace clearing, the empty
// kernel used to measure the launch floor, the pre-gather of x for the
// matrix-core path, the dense comparator and the LSTM cell.
#include "pivot_fc_kernels.h"

namespace pivot {

// ---------------------------------------------------------------------------
// x in natural order -> block order: xg[b][c] = x[b][pcol_pad[c]] (0 in padding
// columns).  The matrix-core kernel reads its B fragments from xg; gathering
// once per launch costs K*batch loads instead of (kept tiles)*bw*batch.
// ---------------------------------------------------------------------------
template <typename WT>
__global__ void gather_x_kernel(const WT* x, long long ldx, const int32_t* pcol_pad, WT* xg, int K_pad, int batch) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    const int b = blockIdx.y;
    if (c >= K_pad) return;
    const int src = pcol_pad[c];
    xg[(size_t)b * K_pad + c] = (src >= 0) ? x[(size_t)b * ldx + src] : WT(0);
}

int launch_gather_x(const void* x, int64_t ldx, const int32_t* pcol_pad, void* xg, int K_pad, int batch,
                    int wdtype, void* stream) {
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    dim3 grid((K_pad + 255) / 256, batch);
    if (wdtype == PIVOT_F16)
        hipLaunchKernelGGL(gather_x_kernel<_Float16>, grid, dim3(256), 0, st, (const _Float16*)x, (long long)ldx, pcol_pad, (_Float16*)xg, K_pad, batch);
    else
        hipLaunchKernelGGL(gather_x_kernel<float>, grid, dim3(256), 0, st, (const float*)x, (long long)ldx, pcol_pad, (float*)xg, K_pad, batch);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

// ---------------------------------------------------------------------------
// small utility kernels
// ---------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint32_t* p, size_t nwords) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < nwords; i += stride) p[i] = 0u;
}

// columns [K, K_pad) of every row of a [batch][K_pad] buffer, in 2-byte units (es = 2 or 4 bytes per element)
__global__ void zero_pad_cols_kernel(unsigned short* buf, int first, int row_len, int batch) {
    const int n = row_len - first;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n * batch; i += gridDim.x * blockDim.x)
        buf[(size_t)(i / n) * row_len + first + i % n] = 0;
}

int launch_zero_pad_cols(void* buf, int K, int K_pad, int batch, int es, void* stream) {
    if (K_pad <= K || batch < 1) return PIVOT_OK;
    const int u = es / 2;                                  // 2-byte units per element
    const int n = (K_pad - K) * u * batch;
    hipLaunchKernelGGL(zero_pad_cols_kernel, dim3((n + 255) / 256), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<unsigned short*>(buf), K * u, K_pad * u, batch);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

__global__ void null_kernel() {}

int launch_null(void* stream) {
    hipLaunchKernelGGL(null_kernel, dim3(1), dim3(64), 0, reinterpret_cast<hipStream_t>(stream));
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

// Reads `npieces` KB once: wavefront w reads pieces [w*per, (w+1)*per), 16 bytes per lane and piece, eight
// pieces in flight, adds everything up and stores one float per wavefront.  Nothing but the read: what one
// launch of the layer kernel cannot beat for the same number of bytes.
__global__ void __launch_bounds__(512) stream_read_kernel(const f32x4* __restrict__ base, int npieces, int per_wave,
                                                           float* __restrict__ out) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int gw = blockIdx.x * (blockDim.x >> 6) + wave;
    const int last = npieces > 0 ? npieces - 1 : 0;
    float acc = 0.f;
    for (int k0 = 0; k0 < per_wave; k0 += 8) {
        f32x4 w[8];
        #pragma unroll
        for (int u = 0; u < 8; ++u) {
            int piece = gw * per_wave + k0 + u;
            piece = piece < last ? piece : last;
            w[u] = base[(size_t)piece * 64 + lane];
        }
        #pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u < per_wave && gw * per_wave + k0 + u < npieces) acc += w[u].x + w[u].y + w[u].z + w[u].w;
    }
    acc = group_sum<64>(acc);
    if (lane == 0) out[gw] = acc;
}

int launch_stream_read(const void* buf, size_t bytes, float* out, void* stream) {
    const int G = 256, W = 8;
    const int npieces = (int)(bytes / 1024);
    if (npieces < 1) { set_error("stream read needs at least 1 KB"); return PIVOT_E_SHAPE; }
    const int per_wave = (npieces + G * W - 1) / (G * W);
    hipLaunchKernelGGL(stream_read_kernel, dim3(G), dim3(W * 64), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<const f32x4*>(buf), npieces, per_wave, out);
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

// ---------------------------------------------------------------------------
// What one trip between two workgroups costs (see pivot_exchange_probe_run).
// Scratch: [8 int64 results][pad to 1 KB][256 words: XCD + 1 of every workgroup][flag words, one per 256-byte line].
// Every wait is bounded; a workgroup that gives up reports -1 and its partner runs into its own bound.
// ---------------------------------------------------------------------------
constexpr int kProbeMaxWg = 256;
constexpr unsigned kProbeMaxSpin = 1u << 20;
constexpr int kProbeTabOff = 1024, kProbeFlagOff = 4096;          // bytes

template <int SCOPE>
__device__ bool probe_bounce(unsigned* a2b, unsigned* b2a, bool is_a, int rounds) {
    for (int i = 1; i <= rounds; ++i) {
        const unsigned v = (unsigned)i;
        unsigned spins = 0;
        if (is_a) {
            __hip_atomic_store(a2b, v, __ATOMIC_RELAXED, SCOPE);
            while (__hip_atomic_load(b2a, __ATOMIC_RELAXED, SCOPE) != v) { if (++spins > kProbeMaxSpin) return false; }
        } else {
            while (__hip_atomic_load(a2b, __ATOMIC_RELAXED, SCOPE) != v) { if (++spins > kProbeMaxSpin) return false; }
            __hip_atomic_store(b2a, v, __ATOMIC_RELAXED, SCOPE);
        }
    }
    return true;
}

// plain stores (the L1 writes through to the XCD's L2), polls that invalidate the L1 first
__device__ bool probe_bounce_l2(unsigned* a2b, unsigned* b2a, bool is_a, int rounds) {
    volatile unsigned* va = a2b;
    volatile unsigned* vb = b2a;
    for (int i = 1; i <= rounds; ++i) {
        const unsigned v = (unsigned)i;
        unsigned spins = 0;
        if (is_a) {
            *va = v;
            for (;;) { asm volatile("buffer_inv sc0" ::: "memory"); if (*vb == v) break; if (++spins > kProbeMaxSpin) return false; }
        } else {
            for (;;) { asm volatile("buffer_inv sc0" ::: "memory"); if (*va == v) break; if (++spins > kProbeMaxSpin) return false; }
            *vb = v;
        }
    }
    return true;
}

__global__ void __launch_bounds__(64) exchange_probe_kernel(char* scratch, int nwg, int rounds) {
    extern __shared__ char one_per_cu[];                // sized so that a compute unit holds one workgroup
    long long* out = reinterpret_cast<long long*>(scratch);
    unsigned* tab = reinterpret_cast<unsigned*>(scratch + kProbeTabOff);
    unsigned* f = reinterpret_cast<unsigned*>(scratch + kProbeFlagOff);
    const int wg = blockIdx.x;
    if (threadIdx.x != 0) return;
    unsigned xcc = 0;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    xcc &= 0xFu;
    __hip_atomic_store(tab + wg, xcc + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // wait (bounded) until every workgroup has published, then pick the partners: the first workgroup on
    // workgroup 0's XCD and the first on another one (every workgroup computes the same two)
    bool all = false;
    for (unsigned spin = 0; spin < 4096u && !all; ++spin) {
        all = true;
        for (int i = 0; i < nwg; ++i)
            if (__hip_atomic_load(tab + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) { all = false; break; }
    }
    int pb = -1, pc = -1;
    if (all) {
        const unsigned x0 = __hip_atomic_load(tab + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int i = 1; i < nwg; ++i) {
            const unsigned xi = __hip_atomic_load(tab + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (pb < 0 && xi == x0) pb = i;
            if (pc < 0 && xi != x0) pc = i;
        }
    }
    if (!all || pb < 0 || pc < 0) { if (wg == 0) out[0] = -1; return; }
    if (wg != 0 && wg != pb && wg != pc) return;
    const bool is_a = wg == 0;
    if (wg == 0 || wg == pb) {
        long long t0 = wall_clock64();
        bool ok = probe_bounce<__HIP_MEMORY_SCOPE_AGENT>(f + 0, f + 64, is_a, rounds);
        long long t1 = wall_clock64();
        if (is_a) { out[1] = ok ? t1 - t0 : -1; out[4] = pb; }
        t0 = wall_clock64();
        ok = probe_bounce<__HIP_MEMORY_SCOPE_WORKGROUP>(f + 128, f + 192, is_a, rounds);
        t1 = wall_clock64();
        if (is_a) out[2] = ok ? t1 - t0 : -1;
        t0 = wall_clock64();
        ok = probe_bounce_l2(f + 256, f + 320, is_a, rounds);
        t1 = wall_clock64();
        if (is_a) out[6] = ok ? t1 - t0 : -1;
    }
    if (wg == 0 || wg == pc) {
        const long long t0 = wall_clock64();
        const bool ok = probe_bounce<__HIP_MEMORY_SCOPE_AGENT>(f + 384, f + 448, is_a, rounds);
        const long long t1 = wall_clock64();
        if (is_a) { out[3] = ok ? t1 - t0 : -1; out[5] = pc; }
    }
    if (is_a) out[0] = 1;
}

int launch_exchange_probe(void* scratch, int rounds, void* stream) {
    int dev = 0, cus = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int nwg = cus < kProbeMaxWg ? cus : kProbeMaxWg;
    if (nwg < 2) { set_error("the probe needs at least two compute units"); return PIVOT_E_UNSUPPORTED; }
    // 96 KB of LDS per workgroup: no two on one compute unit, so all of them are resident at once
    const size_t smem = 96 * 1024;
    static bool allowed[16] = {};
    if (!allowed[dev & 15]) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&exchange_probe_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        allowed[dev & 15] = true;
    }
    int rc = launch_fill_zero(scratch, PIVOT_PROBE_SCRATCH_BYTES, stream);
    if (rc != PIVOT_OK) return rc;
    hipLaunchKernelGGL(exchange_probe_kernel, dim3(nwg), dim3(64), smem, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<char*>(scratch), nwg, rounds);
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
// dense comparator: y = act(W x + b), W streamed once, one wave per R rows,
// UN steps of the row loop in flight.  At batch 1 two rows per wavefront and 8
// steps (4096x9216 fp32 cold: 27.7 us = 5.5 TB/s; four rows and 2 steps, half
// the wavefronts per compute unit, 32.7 us; one row and 8 steps 28.0 us).
// ---------------------------------------------------------------------------
template <typename WT, int NB, int R, int UN>
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
    #pragma unroll UN
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

template <typename WT, int NB, int R, int UN>
static int launch_dense_t(const void* W, int M, int K, const void* x, int64_t ldx, const float* bias,
                          void* y, int64_t ldy, int batch, int act, hipStream_t st) {
    int rows_per_block = 4 * R;
    dim3 grid((M + rows_per_block - 1) / rows_per_block);
    hipLaunchKernelGGL((dense_kernel<WT, NB, R, UN>), grid, dim3(256), 0, st, (const WT*)W, M, K, (const WT*)x,
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
    // from 512 MB on the form with four rows per wavefront is the faster one again (16384x16384 fp32: 178 us against 193)
    const bool huge = (size_t)M * (size_t)K * (size_t)(wdtype == PIVOT_F32 ? 4 : 2) >= ((size_t)512 << 20);
    if (wdtype == PIVOT_F32) {
        if (batch == 1 && huge) return launch_dense_t<float, 1, 4, 2>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
        if (batch == 1) return launch_dense_t<float, 1, 2, 8>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
        if (batch <= 4) return launch_dense_t<float, 4, 2, 2>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
        return launch_dense_t<float, 16, 1, 2>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
    }
    if (batch == 1 && huge) return launch_dense_t<_Float16, 1, 4, 2>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
    if (batch == 1) return launch_dense_t<_Float16, 1, 2, 8>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
    if (batch <= 4) return launch_dense_t<_Float16, 4, 2, 2>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
    return launch_dense_t<_Float16, 16, 1, 2>(W, M, K, x, ldx, bias, y, ldy, batch, act, st);
}

// ---------------------------------------------------------------------------
// generic sparse comparator: y = act(A x + b) with A in plain CSR (the kind of
// routine a pruned layer is usually handed to; Section 5.1 compares against
// one).  L lanes share a row; L is the power of two nearest the mean row length.
// ---------------------------------------------------------------------------
template <typename WT, int L>
__global__ void __launch_bounds__(256) csr_spmv_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                                                       const WT* __restrict__ val, const WT* __restrict__ x,
                                                       const float* __restrict__ bias, float* __restrict__ y, int M, int act) {
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    const int row = gid / L, sub = gid % L;
    const bool ok = row < M;
    const int b = ok ? row_ptr[row] : 0, e = ok ? row_ptr[row + 1] : 0;
    float acc = 0.f;
    for (int k = b + sub; k < e; k += L) acc = fmaf((float)val[k], (float)x[col[k]], acc);
    acc = group_sum<L>(acc);
    if (ok && sub == 0) y[row] = apply_act(acc + (bias ? bias[row] : 0.f), act);
}

template <typename WT>
static int launch_csr_t(const int32_t* row_ptr, const int32_t* col, const void* val, int M, int64_t nnz, const void* x,
                        const float* bias, float* y, int act, hipStream_t st) {
    const double mean = M > 0 ? (double)nnz / M : 0;
    int L = 1;
    while (L < 64 && L * 1.5 < mean) L *= 2;
#define CSR_CASE(L_)                                                                                                     \
    case L_: hipLaunchKernelGGL((csr_spmv_kernel<WT, L_>), dim3((unsigned)(((size_t)M * L_ + 255) / 256)), dim3(256), 0, \
                                st, row_ptr, col, (const WT*)val, (const WT*)x, bias, y, M, act); break;
    switch (L) { CSR_CASE(1) CSR_CASE(2) CSR_CASE(4) CSR_CASE(8) CSR_CASE(16) CSR_CASE(32) default: CSR_CASE(64) }
#undef CSR_CASE
    HIP_TRY(hipGetLastError());
    return PIVOT_OK;
}

int launch_csr(const int32_t* row_ptr, const int32_t* col, const void* val, int wdtype, int M, int64_t nnz, const void* x,
               const float* bias, float* y, int act, void* stream) {
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (wdtype == PIVOT_F32) return launch_csr_t<float>(row_ptr, col, val, M, nnz, x, bias, y, act, st);
    return launch_csr_t<_Float16>(row_ptr, col, val, M, nnz, x, bias, y, act, st);
}

// ---------------------------------------------------------------------------
// LSTM cell around the pruned gate matrix (gate order i,f,g,o).
// ---------------------------------------------------------------------------
__device__ __forceinline__ float sigmoidf_(float v) { return 1.0f / (1.0f + __expf(-v)); }

__global__ void lstm_cell_kernel(LstmCellLaunch L) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= L.batch * L.H) return;
    const int b = idx / L.H, j = idx - b * L.H;
    // the layer kernel scattered the gate pre-activations into natural order: coalesced reads here
    const float* z = L.z + (size_t)b * 4 * L.H;
    const float zi = z[j];
    const float zf = z[L.H + j];
    const float zg = z[2 * L.H + j];
    const float zo = z[3 * L.H + j];
    const int dstc = L.xg_next ? L.invpcol[j] : 0;
    const float c = sigmoidf_(zf) * L.c[idx] + sigmoidf_(zi) * tanhf(zg);
    const float h = sigmoidf_(zo) * tanhf(c);
    L.c[idx] = c;
    L.h[idx] = h;
    if (L.xg_next) {
        // boundary fusion (Section 4.2.1 applied to the recurrence): h_t goes straight to its
        // block-order position in the next step's input
        const size_t o = (size_t)b * L.K_pad + dstc;
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
