// Device-side helpers for the gfx950 kernels: vector types, 16-byte streaming
// loads, wave64 cross-lane reductions, LDS-only barriers, agent-scope
// loads/stores for the split-row hand-over.
#pragma once

#include <hip/hip_runtime.h>

namespace pivot {

typedef float    f32x4  __attribute__((ext_vector_type(4)));
typedef float    f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x2  __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8  __attribute__((ext_vector_type(8)));
typedef int      i32x4  __attribute__((ext_vector_type(4)));

// One 16-byte load per lane (global_load_dwordx4).
template <typename V>
__device__ __forceinline__ V load16(const void* p) {
    return *reinterpret_cast<const V*>(p);
}

// Barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load (vmcnt(0)), which would serialise the weight stream
// behind the barrier; this one leaves those loads in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Orders the LDS writes of a wavefront before its own later LDS reads (other lanes' data): the hardware
// completes one wavefront's LDS operations in order, so this only keeps the compiler from reordering them.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// v + (v from lane ^ 1), ^2 via quad permutes; 4 and 8 via row mirrors (valid
// because after the previous steps all lanes of the mirrored group agree);
// 16 and 32 through the LDS crossbar (ds_bpermute, no memory traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    int s = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false);
    return v + __builtin_bit_cast(float, s);
}

// Sum over groups of `W` adjacent lanes (W a power of two <= 64); every lane
// of a group ends up with the group's sum.  Fixed order: bit-reproducible.
template <int W>
__device__ __forceinline__ float group_sum(float v) {
    if constexpr (W >= 2)  v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    if constexpr (W >= 4)  v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    if constexpr (W >= 8)  v = dpp_add<0x141>(v);   // row_half_mirror
    if constexpr (W >= 16) v = dpp_add<0x140>(v);   // row_mirror
    if constexpr (W >= 32) v += __shfl_xor(v, 16, 64);
    if constexpr (W >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

// Sum over lanes l, l^S, l^2S, ... up to l^32 (S a power of two >= 1):
// combines lanes that differ in the bits >= log2(S).
template <int S>
__device__ __forceinline__ float stride_sum(float v) {
    #pragma unroll
    for (int m = S; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Loads and stores that are coherent across the whole device (they bypass the
// per-XCD caches), for data handed from one workgroup to another inside one
// kernel.
__device__ __forceinline__ float agent_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void agent_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float apply_act(float v, int act) {
    return (act == 1) ? fmaxf(v, 0.0f) : v;
}

}  // namespace pivot
