// Device-side helpers shared by the HIP kernels of the UBP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdint>

#include "ubp_internal.h"

namespace ubp {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return (T)v; } // round to nearest even

template <typename T, int VEC> struct VecOf { typedef T type __attribute__((ext_vector_type(VEC))); };
template <typename T> struct VecOf<T, 1> { typedef T type; };

template <typename T, int VEC>
__device__ __forceinline__ void load_row(const T *p, float (&out)[VEC]) {
    if constexpr (VEC == 1) {
        out[0] = to_f32(*p);
    } else {
        typedef typename VecOf<T, VEC>::type V;
        V v = *reinterpret_cast<const V *>(p);
#pragma unroll
        for (int t = 0; t < VEC; ++t) out[t] = to_f32((T)v[t]);
    }
}

template <typename T, int VEC>
__device__ __forceinline__ void store_row(T *p, const float (&in)[VEC]) {
    if constexpr (VEC == 1) {
        *p = from_f32<T>(in[0]);
    } else {
        typedef typename VecOf<T, VEC>::type V;
        V v;
#pragma unroll
        for (int t = 0; t < VEC; ++t) v[t] = from_f32<T>(in[t]);
        *reinterpret_cast<V *>(p) = v;
    }
}

// Epilogue on an accumulator tile of the MFMA kernels: lane 16 g + n holds 4 pixels of row
// (first row of the stripe) + n.  A uniform test keeps the plain product free of it.
__device__ __forceinline__ float epilogue_value(const Epilogue &e, float v, float b) {
    return fminf(fmaxf(v + b, e.lo), e.hi);
}
__device__ __forceinline__ float epilogue_bias(const Epilogue &e, int row, int M) {
    return (e.bias != nullptr && row < M) ? e.bias[row] : 0.f;
}
__device__ __forceinline__ void epilogue_tile(const Epilogue &e, float4v &acc, float b) {
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] = epilogue_value(e, acc[v], b);
}

template <bool BF16>
__device__ __forceinline__ float4v mfma16(short8v a, short8v b, float4v c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8v, a), __builtin_bit_cast(bf8v, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), c, 0, 0, 0);
}

// transposed 8-byte read at an absolute LDS byte address
__device__ __forceinline__ short4v lds_read_tr(uint32_t lds_addr) {
    typedef __attribute__((address_space(3))) short4v *lds_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(uintptr_t)lds_addr);
}

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base
// wave-uniform).  Written as inline assembly on purpose: the compiler then does not treat
// the load as a pending LDS write, which would make it wait for ALL outstanding vector
// memory operations before every LDS read.  Ordering against the LDS reads of the staged
// data is done by hand (wait_vmcnt, then the producer's counter of resident chunks).
__device__ __forceinline__ void load16_to_lds(const void *gbase, uint32_t lane_off, uint32_t lds_base) {
    // address = gbase (wave-uniform, in SGPRs) + lane_off (32-bit per-lane byte offset)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(gbase), "s"(lds_base));
}

__device__ __forceinline__ uint32_t lds_address(const char *p) {
    typedef __attribute__((address_space(3))) const char *lds_ptr;
    return (uint32_t)(uintptr_t)(lds_ptr)p;
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt immediate out of range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// waits until at most n vector memory operations of this wavefront are outstanding (n is
// wave-uniform; it is rounded down to the nearest available immediate, which only waits longer)
__device__ __forceinline__ void wait_vmcnt_at_most(int n) {
    if (n >= 48) wait_vmcnt<48>();
    else if (n >= 32) wait_vmcnt<32>();
    else if (n >= 24) wait_vmcnt<24>();
    else if (n >= 16) wait_vmcnt<16>();
    else if (n >= 12) wait_vmcnt<12>();
    else if (n >= 8) wait_vmcnt<8>();
    else if (n >= 6) wait_vmcnt<6>();
    else if (n >= 4) wait_vmcnt<4>();
    else if (n >= 3) wait_vmcnt<3>();
    else if (n >= 2) wait_vmcnt<2>();
    else if (n >= 1) wait_vmcnt<1>();
    else wait_vmcnt<0>();
}

__device__ __forceinline__ uint32_t flag_load(uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

constexpr int kSpinLimit = 1 << 22; // polls before a wait gives up (each poll is >= 100 cycles)

// s_barrier with only the LDS counter drained: __syncthreads() would also wait for every
// outstanding vector memory operation, i.e. for loads that are meant to stay in flight
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Raises a kernel's dynamic LDS limit to all of a CU's LDS, once per device ordinal (the limit
// belongs to the function on a device).  One instance per kernel instantiation.
struct LdsLimit {
    std::atomic<uint64_t> done{0};
    ubp_status raise(const void *fn) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) {
            (void)hipGetLastError();
            return UBP_ERR_DEVICE;
        }
        const uint64_t bit = (dev >= 0 && dev < 64) ? (uint64_t(1) << dev) : 0;
        if (bit && (done.load(std::memory_order_acquire) & bit)) return UBP_OK;
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
            (void)hipGetLastError();
            return UBP_ERR_DEVICE;
        }
        done.fetch_or(bit, std::memory_order_release);
        return UBP_OK;
    }
};

} // namespace ubp
