// Per-token layers that need no cross-patch data (Section 4, Sparse operations:
// they run on the fresh tokens only): LayerNorm, GEGLU gating, casts, skip
// concatenation, nearest 2x upsampling, and the sampler's element-wise update
// (Section 3, Eq. 1).  All are HBM-streaming kernels with 8/16-byte accesses.
#include "kernels.h"

namespace df {

namespace {

// one wave per row; float in, bf16 out; two passes over registers (mean, then centred variance)
template <int PER>  // float4 loads per lane: C <= 64*4*PER
__global__ __launch_bounds__(256) void layernorm_rows(const float* __restrict__ x, bf16_t* __restrict__ y,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      int M, int C, float eps) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const float* xr = x + row * C;
  f32x4 v[PER];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < C) {
      v[i] = *reinterpret_cast<const f32x4*>(xr + c);
      s += v[i].x + v[i].y + v[i].z + v[i].w;
    } else {
      v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
  const float mean = wave_sum(s) / (float)C;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < C) {
      const f32x4 d = v[i] - mean;
      q += d.x * d.x + d.y * d.y + d.z * d.z + d.w * d.w;
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)C + eps);
  bf16_t* yr = y + row * C;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < C) {
      const f32x4 g = *reinterpret_cast<const f32x4*>(gamma + c);
      const f32x4 b = *reinterpret_cast<const f32x4*>(beta + c);
      const f32x4 o = (v[i] - mean) * rstd * g + b;
      u32x2 t = {pack_bf2(o.x, o.y), pack_bf2(o.z, o.w)};
      *reinterpret_cast<u32x2*>(yr + c) = t;
    }
  }
}


// h [M, 2F] bf16 (value half, gate half) -> out [M, F] = value * gelu(gate)
__global__ __launch_bounds__(256) void geglu_kernel(const bf16_t* __restrict__ h, bf16_t* __restrict__ out, long long M,
                                                    int F) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int fv = F / 8;
  if (idx >= M * fv) return;
  const long long row = idx / fv;
  const int f0 = (int)(idx % fv) * 8;
  float a[8], g[8];
  ld_vec(h + row * 2 * F + f0, a);
  ld_vec(h + row * 2 * F + F + f0, g);
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] *= gelu_erf(g[i]);
  st_vec(out + row * F + f0, a);
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ x, bf16_t* __restrict__ y,
                                                        long long n4, int silu) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  f32x4 v = *reinterpret_cast<const f32x4*>(x + i * 4);
  if (silu) { v.x = silu_f(v.x); v.y = silu_f(v.y); v.z = silu_f(v.z); v.w = silu_f(v.w); }
  u32x2 t = {pack_bf2(v.x, v.y), pack_bf2(v.z, v.w)};
  *reinterpret_cast<u32x2*>(y + i * 4) = t;
}

__global__ __launch_bounds__(256) void cast_bf16_tail(const float* __restrict__ x, bf16_t* __restrict__ y,
                                                      long long lo, long long n, int silu) {
  const long long i = lo + (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float v = x[i];
  y[i] = f2bf(silu ? silu_f(v) : v);
}

// out[p, 0:Ca] = a[p], out[p, Ca:Ca+Cb] = b[p]; float4 granularity
// optionally also a bf16 copy (operand of the 1x1 shortcut convolution that follows)
__global__ __launch_bounds__(256) void concat_kernel(const float* __restrict__ a, int Ca4, const float* __restrict__ b,
                                                     int Cb4, float* __restrict__ out, bf16_t* __restrict__ out_bf,
                                                     long long pixels) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int C4 = Ca4 + Cb4;
  if (idx >= pixels * C4) return;
  const long long p = idx / C4;
  const int c = (int)(idx % C4);
  const f32x4 v = c < Ca4 ? *reinterpret_cast<const f32x4*>(a + (p * Ca4 + c) * 4)
                          : *reinterpret_cast<const f32x4*>(b + (p * Cb4 + (c - Ca4)) * 4);
  *reinterpret_cast<f32x4*>(out + idx * 4) = v;
  if (out_bf) {
    u32x2 t = {pack_bf2(v.x, v.y), pack_bf2(v.z, v.w)};
    *reinterpret_cast<u32x2*>(out_bf + idx * 4) = t;
  }
}

// x [B,R,W,C] float -> y [B,2R,2W,C] bf16, each pixel repeated 2x2
__global__ __launch_bounds__(256) void upsample2x_kernel(const float* __restrict__ x, bf16_t* __restrict__ y, int B,
                                                         int R, int W, int C4) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)B * 2 * R * 2 * W * C4;
  if (idx >= total) return;
  const int c = (int)(idx % C4);
  long long t = idx / C4;
  const int wo = (int)(t % (2 * W));
  t /= 2 * W;
  const int ro = (int)(t % (2 * R));
  const int b = (int)(t / (2 * R));
  const f32x4 v = *reinterpret_cast<const f32x4*>(x + ((((long long)b * R + (ro >> 1)) * W + (wo >> 1)) * C4 + c) * 4);
  u32x2 o = {pack_bf2(v.x, v.y), pack_bf2(v.z, v.w)};
  *reinterpret_cast<u32x2*>(y + idx * 4) = o;
}

__global__ __launch_bounds__(256) void axpy_kernel(float* __restrict__ x, const float* __restrict__ e, float alpha,
                                                   long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) x[i] = fmaf(alpha, e[i], x[i]);
}

inline unsigned blocks_for(long long n) { return (unsigned)((n + 255) / 256); }

}  // namespace

int launch_layernorm(const float* x, bf16_t* y, const float* gamma, const float* beta, int M, int C, float eps,
                     hipStream_t st) {
  if (C % 4 || C > 64 * 4 * 8) return DF_ESHAPE;
  dim3 grid((M + 3) / 4);
  const int per = cdiv(C, 256);
  if (per <= 1) hipLaunchKernelGGL(layernorm_rows<1>, grid, dim3(256), 0, st, x, y, gamma, beta, M, C, eps);
  else if (per <= 3) hipLaunchKernelGGL(layernorm_rows<3>, grid, dim3(256), 0, st, x, y, gamma, beta, M, C, eps);
  else if (per <= 5) hipLaunchKernelGGL(layernorm_rows<5>, grid, dim3(256), 0, st, x, y, gamma, beta, M, C, eps);
  else hipLaunchKernelGGL(layernorm_rows<8>, grid, dim3(256), 0, st, x, y, gamma, beta, M, C, eps);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

int launch_geglu(const bf16_t* h, bf16_t* out, int M, int F, hipStream_t st) {
  if (F % 8) return DF_ESHAPE;
  const long long n = (long long)M * (F / 8);
  hipLaunchKernelGGL(geglu_kernel, dim3(blocks_for(n)), dim3(256), 0, st, h, out, (long long)M, F);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

int launch_cast_bf16(const float* x, bf16_t* y, long long n, int silu, hipStream_t st) {
  const long long n4 = n / 4;
  if (n4 > 0) hipLaunchKernelGGL(cast_bf16_kernel, dim3(blocks_for(n4)), dim3(256), 0, st, x, y, n4, silu);
  if (n4 * 4 < n) hipLaunchKernelGGL(cast_bf16_tail, dim3(1), dim3(256), 0, st, x, y, n4 * 4, n, silu);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

int launch_concat(const float* a, int Ca, const float* b, int Cb, float* out, bf16_t* out_bf, long long pixels,
                  hipStream_t st) {
  if (Ca % 4 || Cb % 4) return DF_ESHAPE;
  const long long n = pixels * ((Ca + Cb) / 4);
  hipLaunchKernelGGL(concat_kernel, dim3(blocks_for(n)), dim3(256), 0, st, a, Ca / 4, b, Cb / 4, out, out_bf, pixels);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

int launch_upsample2x_bf16(const float* x, bf16_t* y, int B, int R, int W, int C, hipStream_t st) {
  if (C % 4) return DF_ESHAPE;
  const long long n = (long long)B * 4 * R * W * (C / 4);
  hipLaunchKernelGGL(upsample2x_kernel, dim3(blocks_for(n)), dim3(256), 0, st, x, y, B, R, W, C / 4);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

// Register-resident MFMA loop: what the matrix pipes deliver when nothing else is in the way (measurement support).
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* __restrict__ out, int iters) {
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(1.0f + 0.001f * (threadIdx.x & 7)); b[i] = (__bf16)(0.5f); }
  f32x16 acc[4];
  for (int k = 0; k < 4; ++k)
    for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
  }
  float s = 0.f;
  for (int k = 0; k < 4; ++k) s += acc[k][0];
  if (s == 12345.678f) out[blockIdx.x] = s;      // keeps the loop alive; never true
}

int launch_mfma_probe(float* out, int blocks, int iters, hipStream_t st) {
  if (blocks <= 0 || iters <= 0) return DF_ESHAPE;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, out, iters);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

// ---- synchronisation probe (measurement support): what it costs to make every workgroup wait for all others ----
// Three ways to run `iters` dependent phases over `blocks` workgroups, each phase = every workgroup writes 1 KB and
// then reads the 1 KB another workgroup wrote in that phase:
//   mode 0  one kernel per phase (the kernel boundary is the barrier): what the UNet step does;
//   mode 1  one persistent kernel, a counter barrier with device-scope release / acquire fences between phases;
//   mode 2  one persistent kernel, no fences: every 32-bit value travels in a 64-bit word together with the phase
//           number, written and polled with relaxed device-scope atomics (two hops: all -> reducers -> all).
// All waits are bounded (a spin limit sets the fail flag and lets every wave run to its end), and the launcher admits
// at most one workgroup per compute unit, so that all of them are resident together.
// Layout of `buf` (unsigned words): [0] fail flag, [1] barrier counter, [2] generation, [64 ..] tagged words,
// then the float payload.
typedef unsigned long long u64_t;
constexpr unsigned int kProbeSpinLimit = 1u << 20;

__global__ __launch_bounds__(256) void sync_probe_phase(float* __restrict__ pay, unsigned int* __restrict__ ctl, int it) {
  const int nb = gridDim.x, b = blockIdx.x, tid = threadIdx.x;
  if (it > 0) {
    const int ob = (b + nb / 2 + 1) % nb;
    if (pay[((size_t)((it - 1) & 1) * nb + ob) * 256 + tid] != (float)(it - 1 + ob)) ctl[0] = 2u;
  }
  pay[((size_t)(it & 1) * nb + b) * 256 + tid] = (float)(it + b);
}

__global__ __launch_bounds__(256) void sync_probe_fence(float* __restrict__ pay, unsigned int* __restrict__ ctl, int iters) {
  const int nb = gridDim.x, b = blockIdx.x, tid = threadIdx.x;
  for (int it = 0; it < iters; ++it) {
    pay[((size_t)(it & 1) * nb + b) * 256 + tid] = (float)(it + b);
    __syncthreads();
    if (tid == 0) {
      __threadfence();
      __hip_atomic_fetch_add(ctl + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      unsigned int spins = 0;
      while (__hip_atomic_load(ctl + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned int)(it + 1) * nb) {
        if (++spins > kProbeSpinLimit) { ctl[0] = 1u; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      __threadfence();
    }
    __syncthreads();
    const int ob = (b + nb / 2 + 1) % nb;
    if (ctl[0] == 0u && pay[((size_t)(it & 1) * nb + ob) * 256 + tid] != (float)(it + ob)) ctl[0] = 2u;
  }
}

__device__ __forceinline__ void probe_put(u64_t* p, float v, unsigned int tag) {
  __hip_atomic_store(p, ((u64_t)tag << 32) | (u64_t)__float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float probe_get(const u64_t* p, unsigned int tag, unsigned int* fail) {
  for (unsigned int spins = 0;; ++spins) {
    const u64_t w = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((unsigned int)(w >> 32) == tag) return __uint_as_float((unsigned int)w);
    if (spins > kProbeSpinLimit) { *fail = 1u; return 0.f; }
    __builtin_amdgcn_s_sleep(1);
  }
}

// 32 values per workgroup reach 32 reducer workgroups, whose sums reach everybody (what a single-kernel GroupNorm
// with 32 groups would exchange)
__global__ __launch_bounds__(256) void sync_probe_tagged(u64_t* __restrict__ part, u64_t* __restrict__ red,
                                                         unsigned int* __restrict__ ctl, int iters) {
  constexpr int G = 32;
  const int nb = gridDim.x, b = blockIdx.x, tid = threadIdx.x;
  __shared__ float s_v[256];
  __shared__ unsigned int s_tag;
  if (tid == 0) s_tag = ctl[2];                      // the generation is read before anything is produced
  __syncthreads();
  unsigned int tag = s_tag;
  for (int it = 0; it < iters; ++it) {
    tag += 1;
    if (tid < G) probe_put(part + (size_t)tid * nb + b, (float)(b + tid + it), tag);
    if (b < G) {
      float acc = 0.f;
      for (int k = tid; k < nb; k += 256) acc += probe_get(part + (size_t)b * nb + k, tag, ctl);
      s_v[tid] = acc;
      __syncthreads();
      if (tid == 0) {
        float t = 0.f;
        for (int k = 0; k < 256; ++k) t += s_v[k];
        probe_put(red + b, t, tag);
      }
      __syncthreads();
    }
    if (tid < G) {
      const float v = probe_get(red + tid, tag, ctl);
      const float want = (float)nb * (float)(tid + it) + (float)nb * (float)(nb - 1) * 0.5f;
      if (ctl[0] == 0u && v != want) ctl[0] = 2u;
    }
  }
  if (b == 0 && tid == 0) ctl[2] = tag;              // the next launch starts from here (visible at the kernel boundary)
}

__global__ void probe_clear(unsigned int* ctl, int n, int keep_gen) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n && !(keep_gen && i == 2)) ctl[i] = 0u;
}

size_t sync_probe_bytes(int blocks) { return 256 + (size_t)33 * blocks * 8 + 256 + (size_t)2 * blocks * 256 * 4 + 256; }

int launch_sync_probe(void* buf, int blocks, int iters, int mode, hipStream_t st) {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return DF_EHIP;
  if (blocks < 34 || blocks > cus || blocks > 1024 || iters < 1 || mode < 0 || mode > 2) return DF_ESHAPE;
  unsigned int* ctl = (unsigned int*)buf;
  u64_t* part = (u64_t*)((char*)buf + 256);
  u64_t* red = part + (size_t)32 * blocks;
  float* pay = (float*)((char*)buf + 256 + (size_t)33 * blocks * 8 + 256);
  hipLaunchKernelGGL(probe_clear, dim3(1), dim3(64), 0, st, ctl, 64, 1);
  if (mode == 0) {
    for (int it = 0; it < iters; ++it) hipLaunchKernelGGL(sync_probe_phase, dim3(blocks), dim3(256), 0, st, pay, ctl, it);
  } else if (mode == 1) {
    hipLaunchKernelGGL(sync_probe_fence, dim3(blocks), dim3(256), 0, st, pay, ctl, iters);
  } else {
    hipLaunchKernelGGL(sync_probe_tagged, dim3(blocks), dim3(256), 0, st, part, red, ctl, iters);
  }
  DF_LAUNCH_CHECK();
  return DF_OK;
}

__global__ void scale_kernel(float* __restrict__ y, const float* __restrict__ x, float alpha, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = alpha * x[i];
}

int launch_scale(float* y, const float* x, float alpha, long long n, hipStream_t st) {
  if (n <= 0) return DF_OK;
  hipLaunchKernelGGL(scale_kernel, dim3(blocks_for(n)), dim3(256), 0, st, y, x, alpha, n);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

int launch_axpy(float* x, const float* e, float alpha, long long n, hipStream_t st) {
  if (n <= 0) return DF_OK;
  hipLaunchKernelGGL(axpy_kernel, dim3(blocks_for(n)), dim3(256), 0, st, x, e, alpha, n);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

}  // namespace df
