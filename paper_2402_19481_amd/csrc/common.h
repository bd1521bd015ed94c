// Shared device helpers for the gfx950 kernels: bf16 bit conversion, vector
// types, wave reductions and the launch-check macro.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include "../../include/distrifusion.h"

namespace df {

typedef unsigned short bf16_t;  // raw bfloat16 bits

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((unsigned int)v) << 16); }

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

// float -> bf16, round to nearest even, in hardware (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ unsigned int pack_bf2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(pack_bf2(f, 0.f) & 0xffffu); }

// x * sigmoid(x); the hardware reciprocal (1 ulp) replaces the multi-instruction IEEE division
__device__ __forceinline__ float silu_f(float x) {
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

// GELU in its exact (erf) form, 0.5 x (1 + erf(x / sqrt 2)).  erfc(|z|) = t (a1 + t (a2 + t (a3 + t (a4 + t a5))))
// exp(-z^2) with t = 1 / (1 + p |z|) (Abramowitz & Stegun 7.1.26: absolute error below 1.5e-7, the size of float
// rounding of the result); for negative arguments 1 + erf(z) is erfc(|z|) itself, so nothing cancels.  A dozen
// instructions per value where the library erff takes several times that; the GEGLU epilogues are otherwise bounded
// by this function.
__device__ __forceinline__ float gelu_erf(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
  float poly = fmaf(t, 1.061405429f, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  const float erfc_abs = poly * t * __builtin_amdgcn_exp2f(-z * z * 1.4426950408889634f);
  return 0.5f * x * (x >= 0.f ? 2.0f - erfc_abs : erfc_abs);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kVec = 4;  // elements per 16-byte access
  __device__ static __forceinline__ float ld(const float* p) { return *p; }
  __device__ static __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
  __device__ static __forceinline__ void st(bf16_t* p, float v) { *p = f2bf(v); }
};

// 16-byte vector load/store of kVec elements to/from float registers
__device__ __forceinline__ void ld_vec(const float* p, float* v) {
  f32x4 t = *reinterpret_cast<const f32x4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void ld_vec(const bf16_t* p, float* v) {
  u32x4 t = *reinterpret_cast<const u32x4*>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
  v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xffff0000u);
  v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xffff0000u);
}
__device__ __forceinline__ void st_vec(float* p, const float* v) {
  f32x4 t = {v[0], v[1], v[2], v[3]};
  *reinterpret_cast<f32x4*>(p) = t;
}
__device__ __forceinline__ void st_vec(bf16_t* p, const float* v) {
  u32x4 t = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]), pack_bf2(v[4], v[5]), pack_bf2(v[6], v[7])};
  *reinterpret_cast<u32x4*>(p) = t;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Kernel-selection overrides from the environment (DF_TILE, DF_SPLITK, DF_ATTN_*, ...) exist only in builds with
// -DDF_TUNING; in the library as shipped every choice is a function of the call's arguments alone.
#ifdef DF_TUNING
static inline const char* tune_env(const char* name) { return getenv(name); }
#else
static inline const char* tune_env(const char*) { return nullptr; }
#endif

// Position of row m (within its batch item) of a segmented GEMM output inside the destination buffer's batch item:
// identity, or - for a vertical strip of a token grid, pin > 0 - grid row m / pin, column m % pin of the strip, in a
// destination whose grid rows are pout tokens long (the caller's row offset selects the strip's first column).
__device__ __forceinline__ long long seg_pos(int m, int pin, int pout) {
  return pin > 0 ? (long long)(m / pin) * pout + (m % pin) : (long long)m;
}

static inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

}  // namespace df

#define DF_LAUNCH_CHECK()                          \
  do {                                             \
    if (hipGetLastError() != hipSuccess) return DF_EHIP; \
  } while (0)
