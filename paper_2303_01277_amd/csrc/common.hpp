// Shared host/device helpers of the gfx950 kernels (wave64 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/sylvie.h"

namespace sylvie {

constexpr int kWave = 64;

// ---- host side -------------------------------------------------------------

void set_error(const char *fmt, ...);  // api.hip
int32_t fail(int32_t code, const char *fmt, ...);

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

#define SYLVIE_HIP_LAUNCH_CHECK(name)                                                   \
    do {                                                                                \
        hipError_t e_ = hipGetLastError();                                              \
        if (e_ != hipSuccess)                                                           \
            return ::sylvie::fail(SYLVIE_ERR_HIP, "%s: %s", name, hipGetErrorString(e_)); \
    } while (0)

// ---- device side -----------------------------------------------------------

__device__ __forceinline__ int lane_id() { return static_cast<int>(threadIdx.x) & 63; }

// Wave-uniform value of a quantity that is the same in every lane (lets the
// compiler keep it, and everything derived from it, on the scalar unit).
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint32_t uniform(uint32_t v)
{
    return static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(v)));
}
__device__ __forceinline__ int64_t uniform(int64_t v)
{
    const uint32_t lo = uniform(static_cast<uint32_t>(v));
    const uint32_t hi = uniform(static_cast<uint32_t>(static_cast<uint64_t>(v) >> 32));
    return static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
}
__device__ __forceinline__ float uniform(float v)
{
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}

// Streaming accesses: data that is read or written exactly once by the launch (output rows,
// read-modify-write rows, index streams) goes past the caches' retention with the
// non-temporal hint, which on this chip lifts a write-dominated kernel from 5.4 to 6.2 TB/s and
// a read-modify-write kernel from 5.1 to 6.7 TB/s.  N floats (1, 2 or 4) per lane.
template <int N>
struct StreamVec { typedef float type __attribute__((ext_vector_type(N))); };
template <>
struct StreamVec<1> { typedef float type; };
template <int N>
__device__ __forceinline__ void stream_load(float (&o)[N], const float *p)
{
    typedef typename StreamVec<N>::type V;
    const V v = __builtin_nontemporal_load(reinterpret_cast<const V *>(p));
    __builtin_memcpy(o, &v, sizeof(V));
}
template <int N>
__device__ __forceinline__ void stream_store(float *p, const float (&o)[N])
{
    typedef typename StreamVec<N>::type V;
    V v;
    __builtin_memcpy(&v, o, sizeof(V));
    __builtin_nontemporal_store(v, reinterpret_cast<V *>(p));
}

// ---- VEC (1, 2 or 4) adjacent floats per lane ----------------------------------------------

template <int VEC>
struct Vec;
template <>
struct Vec<4> { using type = float4; };
template <>
struct Vec<2> { using type = float2; };
template <>
struct Vec<1> { using type = float; };

template <int VEC>
struct NativeVec {
    typedef float type __attribute__((ext_vector_type(VEC)));
};
template <>
struct NativeVec<1> {
    typedef float type;
};

// Every operand read through load_vec is device (global) memory; saying so keeps the load a
// global one where the pointer was reassembled from lane reads and its origin is no longer visible.
template <int VEC>
__device__ __forceinline__ void load_vec(float (&o)[VEC], const float *p)
{
    typedef typename NativeVec<VEC>::type V;
    typedef const __attribute__((address_space(1))) V *global_ptr;
    const V v = *(global_ptr)(p);
    __builtin_memcpy(o, &v, sizeof(v));
}
// The same through a wave-uniform row address and a lane's own byte offset inside the row
// (an unsigned 32-bit offset lets the load take the row address from scalar registers).
template <int VEC>
__device__ __forceinline__ void load_vec_at(float (&o)[VEC], const float *row, uint32_t byte_off)
{
    typedef typename NativeVec<VEC>::type V;
    typedef const __attribute__((address_space(1))) char *global_bytes;
    typedef const __attribute__((address_space(1))) V *global_ptr;
    const V v = *(global_ptr)((global_bytes)(row) + byte_off);
    __builtin_memcpy(o, &v, sizeof(v));
}
template <int VEC>
__device__ __forceinline__ void store_vec(float *p, const float (&o)[VEC])
{
    typename Vec<VEC>::type v;
    __builtin_memcpy(&v, o, sizeof(v));
    *reinterpret_cast<typename Vec<VEC>::type *>(p) = v;
}

// Between an LDS write by one lane and the read of that location by another lane of the SAME
// wavefront: makes the hand-off defined in the memory model (the compiler may not move either
// access across it).  A wavefront's LDS operations execute in order, so this emits no
// instruction.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Plain compare-select minimum / maximum (inputs are finite by contract).
__device__ __forceinline__ float fmin_sel(float a, float b) { return b < a ? b : a; }
__device__ __forceinline__ float fmax_sel(float a, float b) { return b > a ? b : a; }

// Minimum and maximum over the 64 lanes, returned wave-uniform.  DPP butterfly
// inside each row of 16 lanes (quad swaps, half-row mirror, row mirror), then
// row broadcasts 15 -> rows 1,3 and 31 -> rows 2,3; lane 63 ends with the full
// result.  Each step is one VALU op with the lane permutation fused in.  The
// min and max chains alternate and an s_nop separates dependent steps: a DPP
// operand needs two wait states after the VALU write that produced it, and the
// compiler does not schedule inside an asm block.
__device__ __forceinline__ void wave_minmax(float &mn, float &mx)
{
    asm volatile(
        "s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(mn), "+v"(mx));
    mn = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mn), 63));
    mx = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 63));
}

}  // namespace sylvie
