// Device-side helpers shared by the kernel files: vector types, wave-level primitives, the orderable score maps and
// the feasibility rule of LiNR (arXiv 2407.13218) Sec. 3.1.1 over the bitmask / timestamp attributes.
#pragma once
#include "linr_internal.h"
#include <limits.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned long long u64;

#define WPB LINR_WAVES_PER_BLOCK


// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ u64 wave_ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ bool wave_any(bool p) { return wave_ballot(p) != 0ull; }

// monotone map fp32 -> uint32 (−0.0 is first folded into +0.0 so that both compare equal)
__device__ __forceinline__ uint32_t ord_f32(float s)
{
    s = s + 0.0f;
    uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unord_f32(uint32_t o)
{
    uint32_t u = (o & 0x80000000u) ? (o ^ 0x80000000u) : ~o;
    return __uint_as_float(u);
}
__device__ __forceinline__ uint32_t ord_i32(int x) { return (uint32_t)x ^ 0x80000000u; }
__device__ __forceinline__ int unord_i32(uint32_t o) { return (int)(o ^ 0x80000000u); }

__device__ __forceinline__ u64 aload64(const u64* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// read back what this wave itself stored earlier (same compute unit, same L2: no device-wide flush needed)
__device__ __forceinline__ u64 own_load64(const u64* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void own_stores_done()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}
__device__ __forceinline__ uint32_t aload32(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sec. 3.1.1 feasibility rule over the 32-bit attribute mask and the timestamp window
__device__ __forceinline__ bool filter_pass(const linr_filter& f, uint32_t mask, bool has_ts, uint32_t ts)
{
    bool ok = ((mask & f.all_bits) == f.all_bits) && ((mask & f.none_bits) == 0u);
#pragma unroll
    for (uint32_t g = 0; g < (uint32_t)LINR_MAX_ANY; ++g)
        ok = ok && (g >= f.n_any || (mask & f.any_bits[g]) != 0u);
    if (has_ts) ok = ok && (ts >= f.ts_min) && (ts <= f.ts_max);
    return ok;
}
