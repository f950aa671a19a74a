// Global-memory access helpers.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"

namespace chicle {

// Loads and stores through pointers that were parked in LDS: the compiler no longer knows that they
// point to HBM and would emit flat accesses, whose completion is counted together with LDS traffic.
#define CHICLE_GLOBAL __attribute__((address_space(1)))
typedef int int2_a4 __attribute__((ext_vector_type(2), aligned(4)));
typedef int int4_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef float float2_a4 __attribute__((ext_vector_type(2), aligned(4)));
typedef float float4_a4 __attribute__((ext_vector_type(4), aligned(4)));
__device__ __forceinline__ int gld(const int32_t *p) { return *(const CHICLE_GLOBAL int32_t *)p; }
__device__ __forceinline__ float gld(const float *p) { return *(const CHICLE_GLOBAL float *)p; }
__device__ __forceinline__ int2_a4 gld2(const int32_t *p) { return *(const CHICLE_GLOBAL int2_a4 *)p; }
__device__ __forceinline__ int4_a4 gld4(const int32_t *p) { return *(const CHICLE_GLOBAL int4_a4 *)p; }
__device__ __forceinline__ float2_a4 gld2(const float *p) { return *(const CHICLE_GLOBAL float2_a4 *)p; }
__device__ __forceinline__ float4_a4 gld4(const float *p) { return *(const CHICLE_GLOBAL float4_a4 *)p; }
typedef float float4_v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4_v gld_state(const RowState *p) { return *(const CHICLE_GLOBAL float4_v *)p; }
__device__ __forceinline__ void gst(float *p, float x) { *(CHICLE_GLOBAL float *)p = x; }

// Read of the private vector that bypasses the per-CU vector cache (updates reach it through atomics
// performed in L2).
__device__ __forceinline__ float ld_l2(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Index of an entry in its solver's compact private vector, with the sign bit set where no other row of the
// solver holds that column (long-row contexts): the gather of such an entry is known to be zero (the vector is
// zero at the start of a pass and nothing else writes there) and its update is a plain store, not a
// read-modify-write that fetches a whole line for four bytes.
constexpr int UNIQUE_COLUMN = (int)0x80000000;
__device__ __forceinline__ int vec_index(int c) { return c & 0x7fffffff; }
__device__ __forceinline__ float gather_entry(const float *u, int c) { return c < 0 ? 0.f : ld_l2(u + c); }
__device__ __forceinline__ void add_entry(float *u, int c, float x)
{
    if (c < 0) gst(u + vec_index(c), x);
    else unsafeAtomicAdd(u + c, x);
}

// Zeroes n 32-bit words: the small buffers (rings, progress counters) that every local pass starts from zero
// are cleared by a kernel and not by a memset node, so that a caller may capture a round in a HIP graph.
__global__ __launch_bounds__(256) void clear_words(unsigned *p, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

}  // namespace chicle
