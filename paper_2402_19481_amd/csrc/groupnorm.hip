// Corrected asynchronous GroupNorm (Section 4, Eq. 2) for channels-last patches.
//
// Three launches, the two big ones HBM-bound streaming passes with 16-byte accesses:
//   gn_stats     every block sums a strip of pixels into per-group (sum, sum of
//                squares) partials.
//   gn_finalize  one workgroup per batch item adds the partials in a fixed order,
//                emits the fresh per-patch sums, combines them with the stale sums
//                of the other patches according to the statistic mode and stores
//                mean / rstd (and refreshes the patch's slot of the cache).
//   gn_apply     y = (x - mean) * rstd * gamma + beta (+ SiLU); the second read of
//                x comes from L2 / Infinity Cache at the sizes of one patch.
// A lane keeps a fixed channel offset for its whole strip, so gamma/beta and
// the statistics are fetched once per lane.
//
// Numerics: sums are taken of x - p, p being the group's first value of the batch
// item (its "pivot"), and turned into the sums of x in double only where a group's
// totals are known: E[x^2] - E[x]^2 of float sums loses (mean / sigma)^2 ulps, which
// a tensor whose mean is far from zero cannot afford at float32 tolerance.  The
// normalisation subtracts the mean as a (high, low) float pair before scaling.
#include <cstdlib>
#include <mutex>
#include "kernels.h"

namespace df {

namespace {

constexpr int kMaxG = 64;
constexpr long long kGnGroupMaxElems = 80 * 1024;   // per (group, batch item): above this the three-kernel path

struct GnHalo {
  bf16_t* out;      // nullptr: no boundary-row copy
  int W, rpp, patch0, npatch;
  int single;       // the tensor holds exactly one patch (rpp rows): boundary rows follow from comparisons
};

// stores 4 or 8 bf16 values of pixel p (within its batch item), channels c0.., into the boundary-row state if the
// pixel lies on the first or last row of its patch
template <int V>
__device__ __forceinline__ void halo_store(const GnHalo& h, int b, long long p, int C, int c0, const float* v) {
  // (this runs per pixel and lane: no 64-bit division, and none at all for the one-patch tensors of a displaced step)
  const unsigned int pi = (unsigned int)p;
  unsigned int row, col, pr, patch;
  if (h.single) {
    const unsigned int last0 = (unsigned int)(h.rpp - 1) * (unsigned int)h.W;
    if (pi >= (unsigned int)h.W && pi < last0) return;           // an interior row
    pr = pi < (unsigned int)h.W ? 0u : (unsigned int)(h.rpp - 1);
    col = pi < (unsigned int)h.W ? pi : pi - last0;
    row = pr; patch = (unsigned int)h.patch0;
    if (h.rpp == 1) { pr = 0; col = pi; }
  } else {
    row = pi / (unsigned int)h.W; col = pi - row * (unsigned int)h.W;
    const unsigned int q = row / (unsigned int)h.rpp;
    pr = row - q * (unsigned int)h.rpp; patch = (unsigned int)h.patch0 + q;
  }
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    if ((int)pr != (which ? h.rpp - 1 : 0)) continue;
    bf16_t* o = h.out + ((((long long)b * h.npatch + patch) * 2 + which) * h.W + col) * C + c0;
    if constexpr (V == 8) {
      st_vec(o, v);
    } else {
      u32x2 t = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3])};
      *reinterpret_cast<u32x2*>(o) = t;
    }
  }
}

struct GnLayout {
  int tp;        // lanes per pixel (C / vec)
  int ppb;       // pixels per block iteration
  int threads;   // tp * ppb
  int nblk;      // blocks per segment
  int pix_per_blk;
};

template <typename Tin>
__global__ void gn_stats(const Tin* __restrict__ x, float* __restrict__ partial, int pix_seg, int C, int G, int tp,
                         int ppb, int pix_per_blk, int nseg) {
  constexpr int V = Elem<Tin>::kVec;
  __shared__ float s_sum[kMaxG], s_sq[kMaxG];
  const int blk = blockIdx.x, seg = blockIdx.y, b = blockIdx.z;
  const int nblk = gridDim.x;
  const int cg = C / G;
  const int tid = threadIdx.x;
  if (tid < G) { s_sum[tid] = 0.f; s_sq[tid] = 0.f; }
  __syncthreads();

  const int c0 = (tid % tp) * V;
  const int psub = tid / tp;
  const long long seg_base = ((long long)b * nseg + seg) * pix_seg;
  const int p_lo = blk * pix_per_blk;
  int p_hi = p_lo + pix_per_blk;
  if (p_hi > pix_seg) p_hi = pix_seg;
  float s[V], q[V], piv[V];
#pragma unroll
  for (int i = 0; i < V; ++i) {
    s[i] = 0.f; q[i] = 0.f;
    piv[i] = Elem<Tin>::ld(x + (long long)b * nseg * pix_seg * C + ((c0 + i) / cg) * cg);   // the group's pivot
  }
#pragma unroll 4
  for (int p = p_lo + psub; p < p_hi; p += ppb) {
    float v[V];
    ld_vec(x + (seg_base + p) * C + c0, v);
#pragma unroll
    for (int i = 0; i < V; ++i) { const float d = v[i] - piv[i]; s[i] += d; q[i] = fmaf(d, d, q[i]); }
  }
  // Ordered fold of the lanes' per-channel sums into groups (no atomics: the result must not depend on timing -
  // the UNet amplifies even one-ulp differences of a statistic to the level of its bf16 rounding noise).
  extern __shared__ float s_lane[];            // [2][V][blockDim.x]: per-channel-slot sums of every lane
  const int nthr = blockDim.x;
#pragma unroll
  for (int i = 0; i < V; ++i) {
    s_lane[i * nthr + tid] = s[i];
    s_lane[(V + i) * nthr + tid] = q[i];
  }
  __syncthreads();
  if (tid < G) {
    float ss = 0.f, qq = 0.f;
    for (int ch = tid * cg; ch < (tid + 1) * cg; ++ch) {
      const int tcol = ch / V, i = ch % V;
      for (int ps = 0; ps < ppb; ++ps) {
        ss += s_lane[i * nthr + ps * tp + tcol];
        qq += s_lane[(V + i) * nthr + ps * tp + tcol];
      }
    }
    s_sum[tid] = ss;
    s_sq[tid] = qq;
  }
  __syncthreads();
  float* my = partial + ((((long long)b * nseg + seg) * nblk + blk) * G) * 2;
  if (tid < G) { my[2 * tid] = s_sum[tid]; my[2 * tid + 1] = s_sq[tid]; }
}

// Sums of x from the sums of x - piv over n values (double: this is where the cancellation would happen).
__device__ __forceinline__ void gn_unshift(float s, float q, double n, float piv, double& S, double& SS) {
  const double p = (double)piv;
  S = (double)s + n * p;
  SS = (double)q + 2.0 * p * (double)s + n * p * p;
}

struct GnMoments { float mean_hi, mean_lo, rstd; };

// Mean and variance of one (batch item, group) from the fresh sums of this launch and the cached per-patch sums,
// according to the statistic mode (Section 4, Eq. 2; Section 5.3).  Runs once per group, in double.
// `st_*`: sums of the cached entries of the other patches, `own_*`: the cached entry of this patch.
__device__ __forceinline__ GnMoments gn_combine_pre(double tot_s, double tot_q, double n_loc, int nseg, int N,
                                                    int stat_mode, double st_s, double st_q, double own_s,
                                                    double own_q, float eps) {
  double mean, var;
  if (nseg > 1 || (N == 1 && stat_mode != DF_GN_STALE)) {
    // the whole image is fresh: exact statistics
    const double n = n_loc * (double)nseg;
    mean = tot_s / n;
    var = fmax(tot_q / n - mean * mean, 0.0);
  } else {
    const double n_glob = n_loc * (double)N;
    const double loc_m = tot_s / n_loc, loc_m2 = tot_q / n_loc;
    if (stat_mode == DF_GN_SUMS) {
      mean = (tot_s + st_s) / n_glob;
      var = fmax((tot_q + st_q) / n_glob - mean * mean, 0.0);
    } else if (stat_mode == DF_GN_EQ2) {
      mean = (st_s + own_s) / n_glob + (loc_m - own_s / n_loc);
      const double m2 = (st_q + own_q) / n_glob + (loc_m2 - own_q / n_loc);
      var = m2 - mean * mean;
      if (var < 0.0) var = loc_m2 - loc_m * loc_m;
    } else if (stat_mode == DF_GN_SEPARATE) {
      mean = loc_m;
      var = fmax(loc_m2 - loc_m * loc_m, 0.0);
    } else {
      mean = (st_s + own_s) / n_glob;
      var = fmax((st_q + own_q) / n_glob - mean * mean, 0.0);
    }
  }
  GnMoments m;
  m.mean_hi = (float)mean;
  m.mean_lo = (float)(mean - (double)m.mean_hi);
  m.rstd = (float)(1.0 / sqrt(var + (double)eps));
  return m;
}

__device__ __forceinline__ GnMoments gn_combine(double tot_s, double tot_q, double n_loc, int nseg, int N, int stat_mode,
                                                const float* stale, int b, int g, int B, int G, int patch_idx,
                                                float eps) {
  double st_s = 0.0, st_q = 0.0, own_s = 0.0, own_q = 0.0;
  if (!(nseg > 1 || (N == 1 && stat_mode != DF_GN_STALE))) {
    for (int j = 0; j < N; ++j) {
      const float* sp = stale + (((long long)j * B + b) * G + g) * 2;
      const float a = sp[0], c = sp[1];
      if (j == patch_idx) { own_s = a; own_q = c; } else { st_s += a; st_q += c; }
    }
  }
  return gn_combine_pre(tot_s, tot_q, n_loc, nseg, N, stat_mode, st_s, st_q, own_s, own_q, eps);
}

// The cached sums of one (batch item, group) gathered by a whole wave: lane j fetches patch j's entry (one memory
// round trip for all patches instead of a chain of N), lane order fixes the order of the additions.
__device__ __forceinline__ void gn_stale_wave(const float* stale, int b, int g, int B, int G, int N,
                                              int patch_idx, int lane, double& st_s, double& st_q, double& own_s,
                                              double& own_q) {
  st_s = st_q = own_s = own_q = 0.0;
  if (stale == nullptr) return;
  for (int j0 = 0; j0 < N; j0 += 64) {
    float a = 0.f, c = 0.f;
    if (j0 + lane < N) {
      const float* sp = stale + (((long long)(j0 + lane) * B + b) * G + g) * 2;
      a = sp[0]; c = sp[1];
    }
    const int n = N - j0 < 64 ? N - j0 : 64;
    for (int j = 0; j < n; ++j) {
      const float aj = __shfl(a, j, 64), cj = __shfl(c, j, 64);
      if (j0 + j == patch_idx) { own_s = aj; own_q = cj; } else { st_s += aj; st_q += cj; }
    }
  }
}

// One workgroup per batch item: adds the partials in a fixed order, emits the fresh per-patch sums, combines them with
// the stale sums of the other patches according to the statistic mode and stores mean / rstd.  A separate launch
// instead of a "last workgroup" epilogue: the device-scope fences that pattern needs cost more than the launch.
template <typename Tin>
__global__ __launch_bounds__(1024) void gn_finalize(const float* __restrict__ partial, float* __restrict__ meanrstd,
                                                    const float* stale, float* sums_out, const Tin* __restrict__ x,
                                                    int pix_seg, int C, int G, int nblk, int nseg, int B, int patch_idx,
                                                    int N, float eps, int stat_mode) {
  __shared__ float s_red[2][32][kMaxG];
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int cg = C / G;
  const int parts = blockDim.x / G < 32 ? blockDim.x / G : 32;
  const int g = tid % G, part = tid / G;
  double tot_s = 0.0, tot_q = 0.0;  // sums of x over all segments (valid on part == 0 lanes)
  // the partials are sums of x - pivot, the pivot being the group's first value of the batch item
  const float piv = Elem<Tin>::ld(x + (long long)b * nseg * pix_seg * C + g * cg);
  const double n_seg = (double)pix_seg * (double)cg;
  for (int sg = 0; sg < nseg; ++sg) {
    float a = 0.f, c = 0.f;
    if (part < parts) {
      const float* base = partial + (((long long)b * nseg + sg) * nblk) * G * 2;
      // 16 partials per trip are requested together (one memory round trip), then added in index order
      for (int k0 = part; k0 < nblk; k0 += 16 * parts) {
        float2 v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int k = k0 + i * parts;
          v[i] = k < nblk ? *reinterpret_cast<const float2*>(base + ((long long)k * G + g) * 2) : make_float2(0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) { a += v[i].x; c += v[i].y; }
      }
      s_red[0][part][g] = a;
      s_red[1][part][g] = c;
    }
    __syncthreads();
    if (part == 0) {
      float fs = 0.f, fq = 0.f;
      for (int k = 0; k < parts; ++k) { fs += s_red[0][k][g]; fq += s_red[1][k][g]; }
      double S, SS;
      gn_unshift(fs, fq, n_seg, piv, S, SS);
      tot_s += S; tot_q += SS;
      if (nseg > 1) {
        float* o = sums_out + (((long long)sg * B + b) * G + g) * 2;
        o[0] = (float)S; o[1] = (float)SS;
      }
    }
    __syncthreads();
  }
  // the cached sums of the other patches: thread (part, g) fetches patch part's entry of group g (one round trip for
  // all patches), thread (0, g) adds them in patch order
  const bool need_stale = !(nseg > 1 || (N == 1 && stat_mode != DF_GN_STALE));
  double st_s = 0.0, st_q = 0.0, own_s = 0.0, own_q = 0.0;
  if (need_stale) {
    for (int j0 = 0; j0 < N; j0 += parts) {
      __syncthreads();
      if (part < parts && j0 + part < N) {
        const float* sp = stale + (((long long)(j0 + part) * B + b) * G + g) * 2;
        s_red[0][part][g] = sp[0];
        s_red[1][part][g] = sp[1];
      }
      __syncthreads();
      if (part == 0) {
        const int n = N - j0 < parts ? N - j0 : parts;
        for (int j = 0; j < n; ++j) {
          const float a = s_red[0][j][g], c = s_red[1][j][g];
          if (j0 + j == patch_idx) { own_s = a; own_q = c; } else { st_s += a; st_q += c; }
        }
      }
    }
  }
  if (part != 0) return;
  const GnMoments mo = gn_combine_pre(tot_s, tot_q, n_seg, nseg, N, stat_mode, st_s, st_q, own_s, own_q, eps);
  if (nseg == 1 && sums_out != nullptr) {  // written after the stale sums were read: may alias the own slot
    float* o = sums_out + ((long long)b * G + g) * 2;
    o[0] = (float)tot_s; o[1] = (float)tot_q;
  }
  float* mr = meanrstd + ((long long)b * G + g) * 4;
  mr[0] = mo.mean_hi; mr[1] = mo.mean_lo; mr[2] = mo.rstd;
}

template <typename Tin, typename Tout>
__global__ void gn_apply(const Tin* __restrict__ x, Tout* __restrict__ y, const float* __restrict__ meanrstd,
                         const float* __restrict__ gamma, const float* __restrict__ beta, int pix_b, int C, int G,
                         int tp, int ppb, int pix_per_blk, int silu, int packed, GnHalo halo) {
  constexpr int V = Elem<Tin>::kVec;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int c0 = (tid % tp) * V;
  const int psub = tid / tp;
  const int cg = C / G;
  float sc[V], sh[V], mh[V], ml[V];
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const int c = c0 + i;
    const int g = c / cg;
    const float* mr = meanrstd + ((long long)b * G + g) * 4;
    mh[i] = mr[0]; ml[i] = mr[1];
    sc[i] = mr[2] * gamma[c];
    sh[i] = beta[c];
  }
  const long long base = (long long)b * pix_b;
  const int p_lo = blockIdx.x * pix_per_blk;
  int p_hi = p_lo + pix_per_blk;
  if (p_hi > pix_b) p_hi = pix_b;
  for (int p = p_lo + psub; p < p_hi; p += ppb) {
    float v[V];
    ld_vec(x + (base + p) * C + c0, v);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float t = fmaf((v[i] - mh[i]) - ml[i], sc[i], sh[i]);
      v[i] = silu ? silu_f(t) : t;
    }
    Tout* o = y + (base + p) * C + c0;
    if (packed) {
      // fragment-packed bf16 operand of the linear layers: pixel m = base + p is row m%32 of fragment row m/32, the
      // 8 channels from c0 & ~7 sit in slot (m%32) + 32*((c0/8)%2) of fragment column c0/16
      const long long m = base + p;
      o = y + (((m >> 5) * (C >> 4) + (c0 >> 4)) * 64 + (m & 31) + 32 * ((c0 >> 3) & 1)) * 8 + (c0 & 7);
    }
    if constexpr (sizeof(Tout) == sizeof(Tin)) {
      st_vec(o, v);
    } else {  // float in, bf16 out: 4 values = 8 bytes
      u32x2 t = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3])};
      *reinterpret_cast<u32x2*>(o) = t;
    }
    if constexpr (sizeof(Tout) == 2) {
      if (halo.out) halo_store<V>(halo, b, p, C, c0, v);
    }
  }
}

// Small tensors (the patch at the deeper levels): one workgroup per (group, batch item) does the whole GroupNorm in
// one launch - sums over the group's channels of every pixel, ordered fold, statistic combination, then the
// normalisation on a second read that hits L2.  Groups are independent, so no workgroup waits for another.
template <typename Tin, typename Tout>
__global__ __launch_bounds__(1024) void gn_group_kernel(const Tin* __restrict__ x, Tout* __restrict__ y,
                                                        const float* stale, float* sums_out,
                                                        const float* __restrict__ gamma, const float* __restrict__ beta,
                                                        int pix_seg, int C, int G, int nseg, int B, int patch_idx, int N,
                                                        float eps, int stat_mode, int silu, int packed, GnHalo halo) {
  __shared__ float s_s[1024], s_q[1024];
  __shared__ float s_mr[3];
  const int g = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63;
  const int cg = C / G, cgv = cg >> 2;              // channel vectors of 4 per group
  const int ppass = blockDim.x / cgv;               // pixels per pass
  const int cv = tid % cgv, psub = tid / cgv;
  const bool active = psub < ppass;
  const int c0 = g * cg + cv * 4;
  const float piv = Elem<Tin>::ld(x + (long long)b * nseg * pix_seg * C + g * cg);   // sums are taken of x - piv
  const double n_seg = (double)pix_seg * (double)cg;
  double tot_s = 0.0, tot_q = 0.0;
  for (int sg = 0; sg < nseg; ++sg) {
    const long long base = ((long long)b * nseg + sg) * pix_seg;
    float a = 0.f, q = 0.f;
    if (active)
      for (int p = psub; p < pix_seg; p += ppass) {
        float v[4];
        const Tin* src = x + (base + p) * C + c0;
        if constexpr (sizeof(Tin) == 4) {
          ld_vec(src, v);
        } else {
          const u32x2 t = *reinterpret_cast<const u32x2*>(src);
          v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
          v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) { const float d = v[i] - piv; a += d; q = fmaf(d, d, q); }
      }
    s_s[tid] = a; s_q[tid] = q;
    __syncthreads();
    if (tid < 64) {                                  // ordered fold: strided serial sums, then a fixed butterfly
      float fs = 0.f, fq = 0.f;
      for (int k = lane; k < (int)blockDim.x; k += 64) { fs += s_s[k]; fq += s_q[k]; }
      fs = wave_sum(fs); fq = wave_sum(fq);
      double S, SS;
      gn_unshift(fs, fq, n_seg, piv, S, SS);
      tot_s += S; tot_q += SS;
      if (nseg > 1 && lane == 0) {
        float* o = sums_out + (((long long)sg * B + b) * G + g) * 2;
        o[0] = (float)S; o[1] = (float)SS;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    const GnMoments mo = gn_combine(tot_s, tot_q, n_seg, nseg, N, stat_mode, stale, b, g, B, G, patch_idx, eps);
    if (nseg == 1 && sums_out != nullptr) {          // after the stale sums were read: may alias the own slot
      float* o = sums_out + ((long long)b * G + g) * 2;
      o[0] = (float)tot_s; o[1] = (float)tot_q;
    }
    s_mr[0] = mo.mean_hi; s_mr[1] = mo.mean_lo; s_mr[2] = mo.rstd;
  }
  __syncthreads();
  if (!active) return;
  const float mean = s_mr[0], mean_lo = s_mr[1], rstd = s_mr[2];
  float sc[4], sh[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    sc[i] = rstd * gamma[c0 + i];
    sh[i] = beta[c0 + i];
  }
  const long long pix_b = (long long)pix_seg * nseg;
  const long long base = (long long)b * pix_b;
  for (long long p = psub; p < pix_b; p += ppass) {
    float v[4];
    const Tin* src = x + (base + p) * C + c0;
    if constexpr (sizeof(Tin) == 4) {
      ld_vec(src, v);
    } else {
      const u32x2 t = *reinterpret_cast<const u32x2*>(src);
      v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
      v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float t = fmaf((v[i] - mean) - mean_lo, sc[i], sh[i]);
      v[i] = silu ? silu_f(t) : t;
    }
    const long long m = base + p;
    Tout* o = y + m * C + c0;
    if (packed) o = y + (((m >> 5) * (C >> 4) + (c0 >> 4)) * 64 + (m & 31) + 32 * ((c0 >> 3) & 1)) * 8 + (c0 & 7);
    if constexpr (sizeof(Tout) == 4) {
      st_vec(o, v);
    } else {
      u32x2 t = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3])};
      *reinterpret_cast<u32x2*>(o) = t;
      if (halo.out) halo_store<4>(halo, b, p, C, c0, v);
    }
  }
}

// The same for one segment whose share per lane is at most NV pixels: every lane requests all its pixels at once
// (one memory round trip instead of one per pass) and keeps them in registers for the normalisation, so x is read
// once.
template <typename Tin, typename Tout, int NV>
__global__ __launch_bounds__(1024) void gn_group_reg_kernel(const Tin* __restrict__ x, Tout* __restrict__ y,
                                                            const float* stale, float* sums_out,
                                                            const float* __restrict__ gamma, const float* __restrict__ beta,
                                                            int pix, int C, int G, int B, int patch_idx, int N, float eps,
                                                            int stat_mode, int silu, int packed, GnHalo halo) {
  __shared__ float s_s[1024], s_q[1024];
  __shared__ float s_mr[3];
  const int g = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63;
  const int cg = C / G, cgv = cg >> 2;
  const int ppass = blockDim.x / cgv;
  const int cv = tid % cgv, psub = tid / cgv;
  const bool active = psub < ppass;
  const int c0 = g * cg + cv * 4;
  const long long base = (long long)b * pix;
  const float piv = Elem<Tin>::ld(x + base * C + g * cg);     // sums are taken of x - piv
  // everything that does not depend on x is requested first: affine parameters and the cached sums
  float gm[4] = {0.f, 0.f, 0.f, 0.f}, bt[4] = {0.f, 0.f, 0.f, 0.f};
  if (active) { ld_vec(gamma + c0, gm); ld_vec(beta + c0, bt); }
  double st_s = 0.0, st_q = 0.0, own_s = 0.0, own_q = 0.0;
  if (tid < 64)
    gn_stale_wave((N == 1 && stat_mode != DF_GN_STALE) ? nullptr : stale, b, g, B, G, N, patch_idx, lane, st_s, st_q,
                  own_s, own_q);
  float v[NV][4];
  float a = 0.f, q = 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int p = psub + k * ppass;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[k][i] = 0.f;
    if (active && p < pix) {
      const Tin* src = x + (base + p) * C + c0;
      if constexpr (sizeof(Tin) == 4) {
        ld_vec(src, v[k]);
      } else {
        const u32x2 t = *reinterpret_cast<const u32x2*>(src);
        v[k][0] = __uint_as_float(t.x << 16); v[k][1] = __uint_as_float(t.x & 0xffff0000u);
        v[k][2] = __uint_as_float(t.y << 16); v[k][3] = __uint_as_float(t.y & 0xffff0000u);
      }
    }
  }
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    if (!(active && psub + k * ppass < pix)) continue;          // absent pixels hold zeros, not the pivot
#pragma unroll
    for (int i = 0; i < 4; ++i) { const float d = v[k][i] - piv; a += d; q = fmaf(d, d, q); }
  }
  s_s[tid] = a; s_q[tid] = q;
  __syncthreads();
  if (tid < 64) {
    float fs = 0.f, fq = 0.f;
    for (int k = lane; k < (int)blockDim.x; k += 64) { fs += s_s[k]; fq += s_q[k]; }
    fs = wave_sum(fs); fq = wave_sum(fq);
    if (tid == 0) {
      const double n_loc = (double)pix * (double)cg;
      double S, SS;
      gn_unshift(fs, fq, n_loc, piv, S, SS);
      const GnMoments mo = gn_combine_pre(S, SS, n_loc, 1, N, stat_mode, st_s, st_q, own_s, own_q, eps);
      if (sums_out != nullptr) {                     // after the stale sums were read: may alias the own slot
        float* o = sums_out + ((long long)b * G + g) * 2;
        o[0] = (float)S; o[1] = (float)SS;
      }
      s_mr[0] = mo.mean_hi; s_mr[1] = mo.mean_lo; s_mr[2] = mo.rstd;
    }
  }
  __syncthreads();
  if (!active) return;
  const float mean = s_mr[0], mean_lo = s_mr[1], rstd = s_mr[2];
  float sc[4], sh[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    sc[i] = rstd * gm[i];
    sh[i] = bt[i];
  }
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int p = psub + k * ppass;
    if (p >= pix) continue;
    float o4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float t = fmaf((v[k][i] - mean) - mean_lo, sc[i], sh[i]);
      o4[i] = silu ? silu_f(t) : t;
    }
    const long long m = base + p;
    Tout* o = y + m * C + c0;
    if (packed) o = y + (((m >> 5) * (C >> 4) + (c0 >> 4)) * 64 + (m & 31) + 32 * ((c0 >> 3) & 1)) * 8 + (c0 & 7);
    if constexpr (sizeof(Tout) == 4) {
      st_vec(o, o4);
    } else {
      u32x2 t = {pack_bf2(o4[0], o4[1]), pack_bf2(o4[2], o4[3])};
      *reinterpret_cast<u32x2*>(o) = t;
      if (halo.out) halo_store<4>(halo, b, p, C, c0, o4);
    }
  }
}

GnLayout gn_layout(int C, int vec, long long pix, int target_blocks, int max_threads) {
  GnLayout L;
  L.tp = C / vec;
  L.ppb = max_threads / L.tp;
  if (L.ppb < 1) L.ppb = 1;
  L.threads = L.tp * L.ppb;
  long long per = (pix + target_blocks - 1) / target_blocks;
  long long min_per = (long long)L.ppb * 4;
  if (per < min_per) per = min_per;
  per = (per + L.ppb - 1) / L.ppb * L.ppb;
  L.pix_per_blk = (int)per;
  L.nblk = (int)((pix + per - 1) / per);
  return L;
}

}  // namespace

size_t groupnorm_scratch_bytes(int B, int nseg, int G) {
  // partials for at most 2048 blocks per batch item + mean/rstd
  return kScratchCounterBytes + ((size_t)B * 2048 * G * 2 + (size_t)B * G * 4) * sizeof(float) + 1024;
}

int launch_groupnorm(const GnArgs& a, hipStream_t st) {
  const int vec = a.in_dtype == DF_BF16 ? 8 : 4;
  if (a.C % a.G || a.C % vec || a.G > kMaxG || a.C / vec > 1024) return DF_ESHAPE;
  if (a.in_dtype == DF_BF16 && a.out_dtype != DF_BF16) return DF_ESHAPE;
  if (a.B > 1024) return DF_ESHAPE;
  if (a.y_packed && (a.out_dtype != DF_BF16 || a.C % 16)) return DF_ESHAPE;
  const long long pix_seg = (long long)a.Rseg * a.W;
  GnHalo halo = {};
  if (a.halo_out) {
    if (a.out_dtype != DF_BF16 || a.y_packed || a.halo_rpp <= 0 || ((long long)a.Rseg * a.nseg) % a.halo_rpp ||
        a.halo_patch0 < 0 || a.halo_patch0 + (a.Rseg * a.nseg) / a.halo_rpp > a.halo_npatch || ((uintptr_t)a.halo_out % 16))
      return DF_EINVAL;
    halo.out = (bf16_t*)a.halo_out; halo.W = a.W; halo.rpp = a.halo_rpp; halo.patch0 = a.halo_patch0;
    halo.npatch = a.halo_npatch;
    halo.single = ((long long)a.Rseg * a.nseg == a.halo_rpp) ? 1 : 0;
  }
  if (pix_seg <= 0 || pix_seg * a.nseg > 0x7fffffffLL) return DF_ESHAPE;
  // small tensors: the whole GroupNorm in one launch, one workgroup per (group, batch item)
  {
    const int cg = a.C / a.G;
    const long long per_group = pix_seg * a.nseg * cg;
    static const bool no_fused = tune_env("DF_GN_3K") != nullptr;   // tuning aid
    if (!no_fused && cg % 4 == 0 && cg / 4 <= 1024 && per_group <= kGnGroupMaxElems) {
      dim3 grid(a.G, a.B);
      const int ppass = 1024 / (cg / 4);
      if (a.nseg == 1 && pix_seg <= (long long)ppass * 8) {
        // one patch, at most 8 pixels per lane: single read of x
#define DF_GN_REG(TI, TO)                                                                                             \
  hipLaunchKernelGGL((gn_group_reg_kernel<TI, TO, 8>), grid, dim3(1024), 0, st, (const TI*)a.x, (TO*)a.y, a.stale,     \
                     a.sums_out, a.gamma, a.beta, (int)pix_seg, a.C, a.G, a.B, a.patch_idx, a.N, a.eps, a.stat_mode,  \
                     a.silu, a.y_packed, halo)
        if (a.in_dtype == DF_BF16) DF_GN_REG(bf16_t, bf16_t);
        else if (a.out_dtype == DF_BF16) DF_GN_REG(float, bf16_t);
        else DF_GN_REG(float, float);
#undef DF_GN_REG
        DF_LAUNCH_CHECK();
        return DF_OK;
      }
#define DF_GN_GROUP(TI, TO)                                                                                         \
  hipLaunchKernelGGL((gn_group_kernel<TI, TO>), grid, dim3(1024), 0, st, (const TI*)a.x, (TO*)a.y, a.stale, a.sums_out, \
                     a.gamma, a.beta, (int)pix_seg, a.C, a.G, a.nseg, a.B, a.patch_idx, a.N, a.eps, a.stat_mode, a.silu, \
                     a.y_packed, halo)
      if (a.in_dtype == DF_BF16) DF_GN_GROUP(bf16_t, bf16_t);
      else if (a.out_dtype == DF_BF16) DF_GN_GROUP(float, bf16_t);
      else DF_GN_GROUP(float, float);
#undef DF_GN_GROUP
      DF_LAUNCH_CHECK();
      return DF_OK;
    }
  }
  // up to 512 partial blocks per batch item: the finalize workgroup folds them with 32 lanes per group
  int target = 512 / a.nseg;
  if (target < 1) target = 1;
  GnLayout L = gn_layout(a.C, vec, pix_seg, target, 256);
  if ((long long)L.nblk * a.nseg > 2048) return DF_ESHAPE;
  if (L.threads < a.G) return DF_ESHAPE;
  char* scr = scratch_region(a.scr, groupnorm_scratch_bytes(a.B, a.nseg, a.G));
  if (!scr) return DF_ENOMEM;
  float* meanrstd = (float*)(scr + kScratchCounterBytes);
  float* partial = meanrstd + (size_t)a.B * a.G * 4;
  dim3 gs(L.nblk, a.nseg, a.B);
  if (a.in_dtype == DF_BF16)
    hipLaunchKernelGGL(gn_stats<bf16_t>, gs, dim3(L.threads), (size_t)2 * 8 * L.threads * sizeof(float), st, (const bf16_t*)a.x, partial, (int)pix_seg, a.C, a.G,
                       L.tp, L.ppb, L.pix_per_blk, a.nseg);
  else
    hipLaunchKernelGGL(gn_stats<float>, gs, dim3(L.threads), (size_t)2 * 4 * L.threads * sizeof(float), st, (const float*)a.x, partial, (int)pix_seg, a.C, a.G,
                       L.tp, L.ppb, L.pix_per_blk, a.nseg);
  DF_LAUNCH_CHECK();
  if (a.in_dtype == DF_BF16)
    hipLaunchKernelGGL(gn_finalize<bf16_t>, dim3(a.B), dim3(1024), 0, st, partial, meanrstd, a.stale, a.sums_out,
                       (const bf16_t*)a.x, (int)pix_seg, a.C, a.G, L.nblk, a.nseg, a.B, a.patch_idx, a.N, a.eps, a.stat_mode);
  else
    hipLaunchKernelGGL(gn_finalize<float>, dim3(a.B), dim3(1024), 0, st, partial, meanrstd, a.stale, a.sums_out,
                       (const float*)a.x, (int)pix_seg, a.C, a.G, L.nblk, a.nseg, a.B, a.patch_idx, a.N, a.eps, a.stat_mode);
  DF_LAUNCH_CHECK();
  const long long pix_b = pix_seg * a.nseg;
  GnLayout A = gn_layout(a.C, vec, pix_b, 2048, 256);
  dim3 ga(A.nblk, a.B);
  if (a.in_dtype == DF_BF16) {
    hipLaunchKernelGGL((gn_apply<bf16_t, bf16_t>), ga, dim3(A.threads), 0, st, (const bf16_t*)a.x, (bf16_t*)a.y,
                       meanrstd, a.gamma, a.beta, (int)pix_b, a.C, a.G, A.tp, A.ppb, A.pix_per_blk, a.silu, a.y_packed, halo);
  } else if (a.out_dtype == DF_BF16) {
    hipLaunchKernelGGL((gn_apply<float, bf16_t>), ga, dim3(A.threads), 0, st, (const float*)a.x, (bf16_t*)a.y,
                       meanrstd, a.gamma, a.beta, (int)pix_b, a.C, a.G, A.tp, A.ppb, A.pix_per_blk, a.silu, a.y_packed, halo);
  } else {
    hipLaunchKernelGGL((gn_apply<float, float>), ga, dim3(A.threads), 0, st, (const float*)a.x, (float*)a.y, meanrstd,
                       a.gamma, a.beta, (int)pix_b, a.C, a.G, A.tp, A.ppb, A.pix_per_blk, a.silu, a.y_packed, halo);
  }
  DF_LAUNCH_CHECK();
  return DF_OK;
}

// Argument validation shared by the two GroupNorm entry points of the C ABI.
int groupnorm_entry(const void* x_fresh, void* y, const float* stale_stats, float* fresh_stats_out, const float* gamma,
                    const float* beta, int B, int R, int W, int C, int G, int patch_idx, int N, float eps, int stat_mode,
                    int fuse_silu, int dtype, const Scratch* scr, hipStream_t st) {
  if (!x_fresh || !y || !gamma || !beta || (dtype != DF_F32 && dtype != DF_BF16)) return DF_EINVAL;
  if (stat_mode < DF_GN_SUMS || stat_mode > DF_GN_STALE) return DF_EINVAL;
  if (B <= 0 || R <= 0 || W <= 0 || C <= 0 || G <= 0 || N <= 0 || patch_idx < 0 || patch_idx >= N) return DF_ESHAPE;
  if ((N > 1 || stat_mode == DF_GN_STALE) && !stale_stats) return DF_EINVAL;
  if (((uintptr_t)x_fresh % 16) || ((uintptr_t)y % 16)) return DF_EINVAL;
  GnArgs a = {};
  a.x = x_fresh; a.y = y; a.stale = stale_stats; a.sums_out = fresh_stats_out; a.gamma = gamma; a.beta = beta;
  a.B = B; a.Rseg = R; a.W = W; a.C = C; a.G = G; a.nseg = 1; a.patch_idx = patch_idx; a.N = N; a.eps = eps;
  a.stat_mode = stat_mode; a.silu = fuse_silu ? 1 : 0; a.in_dtype = dtype; a.out_dtype = dtype;
  a.scr = scr;
  return launch_groupnorm(a, st);
}

}  // namespace df

// ---- the entry point for callers that cannot allocate ----
// Its kernels take their partial sums from this array instead of an allocated region.  Every GPU the library runs on
// holds its own copy until the process ends; host code reaches it only through the address hipGetSymbolAddress
// returns for the current device.
static constexpr size_t kStaticScratchBytes = DF_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
void* g_static_scratch[64];            // per device: address of that device's copy of `scratch`
std::mutex g_static_scratch_mu;

int static_scratch_region(df::Scratch* out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DF_EHIP;
  std::lock_guard<std::mutex> lock(g_static_scratch_mu);
  if (!g_static_scratch[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return DF_EHIP; }
    g_static_scratch[dev] = ptr;
  }
  out->ptr = (char*)g_static_scratch[dev];
  out->bytes = kStaticScratchBytes;
  return DF_OK;
}
}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int df_groupnorm_stale_noalloc(const void* x_fresh, void* y, const float* stale_stats, float* fresh_stats_out,
                               const float* gamma, const float* beta, int B, int R, int W, int C, int G, int patch_idx,
                               int N, float eps, int stat_mode, int fuse_silu, int dtype, void* stream) {
  if (B <= 0 || G <= 0) return DF_ESHAPE;
  // the statistics pass keeps up to 2048 partial (sum, sum of squares) pairs per batch item and group
  if (df::groupnorm_scratch_bytes(B, 1, G) > kStaticScratchBytes) return DF_ENOMEM;
  df::Scratch region = {nullptr, 0};
  const int rc = static_scratch_region(&region);
  if (rc != DF_OK) return rc;
  // nothing in the region has to start at zero: every partial and every statistic is written before it is read
  return df::groupnorm_entry(x_fresh, y, stale_stats, fresh_stats_out, gamma, beta, B, R, W, C, G, patch_idx, N, eps,
                             stat_mode, fuse_silu, dtype, &region, (hipStream_t)stream);
}

#pragma GCC visibility pop
}  // extern "C"
