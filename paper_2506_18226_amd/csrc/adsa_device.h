// Device-side helpers shared by the two attention kernels (gfx950).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adsa {

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Pointers the kernel reads out of the sequence record are declared as what they are, global memory:
// the accesses then compile to global (not flat) instructions whatever else is done with the value.
#define ADSA_GLOBAL __attribute__((address_space(1)))
typedef ADSA_GLOBAL char gchar;
typedef ADSA_GLOBAL float gfloat;
typedef ADSA_GLOBAL int32_t gint;

// 16-byte streaming load: K/V rows are read once per step, so keep them out of the caches' way
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const gchar* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const ADSA_GLOBAL u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 load16(const gchar* p) {
  const u32x4 v = *reinterpret_cast<const ADSA_GLOBAL u32x4*>(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store16(gchar* p, const uint4& x) {
  u32x4 v; v.x = x.x; v.y = x.y; v.z = x.z; v.w = x.w;
  *reinterpret_cast<ADSA_GLOBAL u32x4*>(p) = v;
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// 8 consecutive fp32 values -> 8 bf16 (round to nearest even) in one 16-byte vector
__device__ __forceinline__ uint4 pack8_bf16(const gchar* f) {
  const uint4 ua = load16(f), ub = load16(f + 16);
  const float4 a = make_float4(__uint_as_float(ua.x), __uint_as_float(ua.y), __uint_as_float(ua.z), __uint_as_float(ua.w));
  const float4 b = make_float4(__uint_as_float(ub.x), __uint_as_float(ub.y), __uint_as_float(ub.z), __uint_as_float(ub.w));
  return make_uint4(f32_to_bf16_rne(a.x) | (f32_to_bf16_rne(a.y) << 16), f32_to_bf16_rne(a.z) | (f32_to_bf16_rne(a.w) << 16),
                    f32_to_bf16_rne(b.x) | (f32_to_bf16_rne(b.y) << 16), f32_to_bf16_rne(b.z) | (f32_to_bf16_rne(b.w) << 16));
}

// Demands a wave-uniform value that was just loaded in scalar registers AT THIS POINT of the program:
// its load cannot sink below the statement, into a later and then dependent round trip.  (Input only:
// the value itself, and what the compiler knows about where a pointer points, stay as they are.)
template <typename T>
__device__ __forceinline__ void pin_uniform(const T& x) { asm volatile("" : : "s"(x)); }

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// Value of lane (lane ^ X) for X in {8, 16, 32}: DPP inside a 16-lane row, register-only swaps of
// 16- and 32-lane halves beyond it (both outputs of a swap of x with itself are returned).
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <int X>
__device__ __forceinline__ float xor_sum(float x) {
  if constexpr (X == 8) return x + dpp_f<0x128>(x);            // row_ror:8
  else {
    const unsigned u = __float_as_uint(x);
    const u32x2 r = X == 16 ? __builtin_amdgcn_permlane16_swap(u, u, false, false)
                            : __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);       // one of the two is x itself, the other its partner
  }
}
template <int X>
__device__ __forceinline__ float xor_max(float x) {
  if constexpr (X == 8) return fmaxf(x, dpp_f<0x128>(x));
  else {
    const unsigned u = __float_as_uint(x);
    const u32x2 r = X == 16 ? __builtin_amdgcn_permlane16_swap(u, u, false, false)
                            : __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
  }
}

// Data handed from one workgroup to another inside a launch (chunk partials, logits) is written
// and read with device-scope atomic accesses: they go through to the level where all XCDs agree
// and are never left dirty in (or served stale from) one XCD's L2.  The order between them and the
// arrival counter is made in the kernels' split paths (completed stores, barrier, release/acquire ticket).
__device__ __forceinline__ void st_dev(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev2(float* p, float a, float b) {   // 8-byte aligned pair
  const unsigned long long v = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace adsa
