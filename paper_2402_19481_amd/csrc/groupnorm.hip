// Corrected asynchronous GroupNorm (Section 4, Eq. 2) for channels-last patches.
//
// Large tensors take two launches, both streaming passes with 16-byte accesses:
//   gn_stats     every block sums a strip of pixels into per-group (sum, sum of
//                squares) partials; one block also snapshots the cached sums.
//   gn_apply     every block first adds all partials in the same fixed order (so
//                all blocks hold bit-identical statistics without a third launch or
//                a grid-wide wait: an in-kernel barrier across the eight XCDs costs
//                more than a kernel boundary here), combines them with the stale
//                sums of the other patches according to the statistic mode, then
//                y = (x - mean) * rstd * gamma + beta (+ SiLU) on the strip it summed
//                in the first launch; block 0 also emits the fresh per-patch sums.
// Small tensors take one launch, one workgroup per (group, batch item).
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
constexpr long long kGnGroupMaxElems = 24 * 1024;   // per (group, batch item): above this the two-launch path (unless
                                                    // the patch fits the registers of one workgroup per group)
constexpr int kGnMaxPpb = 32;                      // pixels a block of that path handles per iteration, at most
constexpr int kGnMaxStrips = 256;                   // pixel strips (= blocks per launch) per batch item on that path

struct GnHalo {
  bf16_t* out;      // nullptr: no boundary-row copy
  int W, rpp, patch0, npatch;
  int single;       // the tensor holds exactly one patch (rpp rows): boundary rows follow from comparisons
  int cols, rows;   // cols != 0: vertical strips of rpp columns, the state holds boundary columns of `rows` pixels
};

// stores 4 or 8 bf16 values of pixel p (within its batch item), channels c0.., into the boundary-row state if the
// pixel lies on the first or last row of its patch
template <int V>
__device__ __forceinline__ void halo_store(const GnHalo& h, int b, long long p, int C, int c0, const float* v) {
  // (this runs per pixel and lane: no 64-bit division, and none at all for the one-patch tensors of a displaced step)
  const unsigned int pi = (unsigned int)p;
  unsigned int row, col, pr, patch;
  if (h.cols) {
    row = pi / (unsigned int)h.W; col = pi - row * (unsigned int)h.W;
    const unsigned int q = col / (unsigned int)h.rpp;
    const unsigned int pc = col - q * (unsigned int)h.rpp;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
      if ((int)pc != (which ? h.rpp - 1 : 0)) continue;
      bf16_t* o = h.out + ((((long long)b * h.npatch + (h.patch0 + q)) * 2 + which) * h.rows + row) * C + c0;
      if constexpr (V == 8) {
        st_vec(o, v);
      } else {
        u32x2 t = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3])};
        *reinterpret_cast<u32x2*>(o) = t;
      }
    }
    return;
  }
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

// NCH (template parameter of the two-launch kernels): 16-byte loads a lane keeps in flight, 1, 2, 4 or 8

// 16 bytes as loaded -> kVec float values
template <typename T>
__device__ __forceinline__ void unpack_vec(const u32x4& t, float* v) {
  if constexpr (sizeof(T) == 4) {
    v[0] = __uint_as_float(t.x); v[1] = __uint_as_float(t.y); v[2] = __uint_as_float(t.z); v[3] = __uint_as_float(t.w);
  } else {
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
    v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xffff0000u);
    v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xffff0000u);
  }
}

struct GnLayout {
  int tp;        // lanes per pixel (C / vec)
  int ppb;       // pixels per block iteration
  int threads;   // tp * ppb
  int nblk;      // blocks per segment
  int pix_per_blk;
};

template <typename Tin, int NCH>
__global__ void gn_stats(const Tin* __restrict__ x, float* __restrict__ partial, int pix_seg, int C, int G, int tp,
                         int ppb, int pix_per_blk, int nseg, const float* stale, float* __restrict__ stale_copy,
                         int stale_n) {
  constexpr int V = Elem<Tin>::kVec;
  __shared__ float s_sum[kMaxG], s_sq[kMaxG], s_piv[kMaxG];
  const int blk = blockIdx.x, seg = blockIdx.y, b = blockIdx.z;
  const int nblk = gridDim.x;
  const int cg = C / G;
  const int tid = threadIdx.x;
  const int c0 = (tid % tp) * V;
  const int psub = tid / tp;
  const long long seg_base = ((long long)b * nseg + seg) * pix_seg;
  const int p_lo = blk * pix_per_blk;
  int p_hi = p_lo + pix_per_blk;
  if (p_hi > pix_seg) p_hi = pix_seg;
  // a lane requests NCH pixels at once (a strip is usually one chunk: the whole tensor is in flight together);
  // the first chunk goes out before anything else
  u32x4 raw[NCH];
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int p = p_lo + psub + k * ppb;
    raw[k] = *reinterpret_cast<const u32x4*>(x + (seg_base + (p < p_hi ? p : p_lo)) * C + c0);
  }
  if (tid < G) s_piv[tid] = Elem<Tin>::ld(x + (long long)b * nseg * pix_seg * C + tid * cg);   // the groups' pivots
  // The second launch may overwrite the patch's own slot of the cached sums (in-place refresh) while other blocks of
  // it still need the old value: it reads this snapshot instead.
  if (stale != nullptr && blk == 0 && seg == 0 && b == 0)
    for (int i = tid; i < stale_n; i += blockDim.x) stale_copy[i] = stale[i];
  __syncthreads();

  const int ga = c0 / cg;                       // group of the lane's first channel
  float s[V], q[V], piv[V];
#pragma unroll
  for (int i = 0; i < V; ++i) {
    s[i] = 0.f; q[i] = 0.f;
    piv[i] = s_piv[cg >= V ? (c0 + i >= (ga + 1) * cg ? ga + 1 : ga) : (c0 + i) / cg];
  }
  for (int p0 = p_lo + psub; p0 < p_hi; p0 += NCH * ppb) {
    if (p0 != p_lo + psub) {
#pragma unroll
      for (int k = 0; k < NCH; ++k) {
        const int p = p0 + k * ppb;
        raw[k] = *reinterpret_cast<const u32x4*>(x + (seg_base + (p < p_hi ? p : p0)) * C + c0);
      }
    }
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      if (p0 + k * ppb >= p_hi) break;
      float v[V];
      unpack_vec<Tin>(raw[k], v);
#pragma unroll
      for (int i = 0; i < V; ++i) { const float d = v[i] - piv[i]; s[i] += d; q[i] = fmaf(d, d, q[i]); }
    }
  }
  // Ordered fold of the lanes' per-channel sums into groups (no atomics: the result must not depend on timing -
  // the UNet amplifies even one-ulp differences of a statistic to the level of its bf16 rounding noise).
  // Two levels: thread (g, ps) adds group g's channels over the lanes of pixel slot ps, then thread g adds the slots.
  extern __shared__ float s_lane[];            // fast path: float4 per lane; general path: [V][blockDim.x]
  __shared__ float s_lvl[2][kGnMaxPpb][kMaxG];
  const int nthr = blockDim.x;
  if (cg >= V) {
    // a lane's V consecutive channels touch at most two groups: it leaves (sum, sum of squares) of the part in its
    // first group and of the part in the next one
    f32x4 mine = {0.f, 0.f, 0.f, 0.f};
    const int nb = (ga + 1) * cg - c0;          // channels of the lane that belong to group ga
#pragma unroll
    for (int i = 0; i < V; ++i) {
      if (i < nb) { mine.x += s[i]; mine.y += q[i]; } else { mine.z += s[i]; mine.w += q[i]; }
    }
    reinterpret_cast<f32x4*>(s_lane)[tid] = mine;
    __syncthreads();
    for (int role = tid; role < G * ppb; role += nthr) {
      const int fg = role % G, fps = role / G;
      const int t_lo = (fg * cg) / V, t_hi = ((fg + 1) * cg - 1) / V;
      float as = 0.f, aq = 0.f;
      for (int tc = t_lo; tc <= t_hi; ++tc) {
        const f32x4 e = reinterpret_cast<const f32x4*>(s_lane)[fps * tp + tc];
        if ((tc * V) / cg == fg) { as += e.x; aq += e.y; } else { as += e.z; aq += e.w; }
      }
      s_lvl[0][fps][fg] = as;
      s_lvl[1][fps][fg] = aq;
    }
    __syncthreads();
  } else {
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
      for (int i = 0; i < V; ++i) s_lane[i * nthr + tid] = pass ? q[i] : s[i];
      __syncthreads();
      for (int role = tid; role < G * ppb; role += nthr) {
        const int fg = role % G, fps = role / G;
        float acc = 0.f;
        for (int ch = fg * cg; ch < (fg + 1) * cg; ++ch) acc += s_lane[(ch % V) * nthr + fps * tp + ch / V];
        s_lvl[pass][fps][fg] = acc;
      }
      __syncthreads();
    }
  }
  if (tid < G) {
    float ss = 0.f, qq = 0.f;
    for (int ps = 0; ps < ppb; ++ps) { ss += s_lvl[0][ps][tid]; qq += s_lvl[1][ps][tid]; }
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

// Second launch of the large path.  Every block adds the partials of its batch item in the same fixed order, combines
// them with the cached sums and normalises the strip of pixels it was given.
template <typename Tin, typename Tout, int NCH>
__global__ __launch_bounds__(1024) void gn_apply(const Tin* __restrict__ x, Tout* __restrict__ y,
                                                 const float* __restrict__ partial, const float* __restrict__ stale_copy,
                                                 float* sums_out, const float* __restrict__ gamma,
                                                 const float* __restrict__ beta, int pix_seg, int C, int G, int nblk,
                                                 int nseg, int B, int patch_idx, int N, float eps, int stat_mode, int tp,
                                                 int ppb, int pix_per_blk, int silu, int packed, GnHalo halo) {
  constexpr int V = Elem<Tin>::kVec;
  __shared__ float s_red[2][32][kMaxG];
  __shared__ float s_mom[kMaxG][3];
  const int blk = blockIdx.x, seg = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int cg = C / G;
  // The lane's first NCH pixels are requested before anything else: the fold of the partials below then runs
  // while they are on their way (usually that is the lane's whole share of the strip).
  const bool works = tid < tp * ppb;
  const int c0 = (tid % tp) * V;
  const int psub = tid / tp;
  const long long base = ((long long)b * nseg + seg) * pix_seg;     // pixels before this segment
  const int p_lo = blk * pix_per_blk;
  int p_hi = p_lo + pix_per_blk;
  if (p_hi > pix_seg) p_hi = pix_seg;
  u32x4 raw[NCH];
  if (works) {
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
      const int p = p_lo + psub + k * ppb;
      raw[k] = *reinterpret_cast<const u32x4*>(x + (base + (p < p_hi ? p : p_lo)) * C + c0);
    }
  }
  {
    const int parts = (int)blockDim.x / G < 32 ? (int)blockDim.x / G : 32;
    const int g = tid % G, part = tid / G;
    const bool folds = part < parts;
    double tot_s = 0.0, tot_q = 0.0;  // sums of x over all segments (valid where part == 0)
    // the partials are sums of x - pivot, the pivot being the group's first value of the batch item
    const float piv = folds ? Elem<Tin>::ld(x + (long long)b * nseg * pix_seg * C + g * cg) : 0.f;
    const double n_seg = (double)pix_seg * (double)cg;
    for (int sg = 0; sg < nseg; ++sg) {
      float a = 0.f, c = 0.f;
      if (folds) {
        const float* base = partial + (((long long)b * nseg + sg) * nblk) * G * 2;
        // 8 partials per trip are requested together (one memory round trip), then added in index order
        for (int k0 = part; k0 < nblk; k0 += 8 * parts) {
          float2 v[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int k = k0 + i * parts;
            v[i] = k < nblk ? *reinterpret_cast<const float2*>(base + ((long long)k * G + g) * 2) : make_float2(0.f, 0.f);
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) { a += v[i].x; c += v[i].y; }
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
        if (nseg > 1 && blk == 0 && seg == 0) {        // full image: the per-patch sums are the cache's new content
          float* o = sums_out + (((long long)sg * B + b) * G + g) * 2;
          o[0] = (float)S; o[1] = (float)SS;
        }
      }
      __syncthreads();
    }
    if (part == 0) {
      double st_s = 0.0, st_q = 0.0, own_s = 0.0, own_q = 0.0;
      if (!(nseg > 1 || (N == 1 && stat_mode != DF_GN_STALE))) {
        for (int j = 0; j < N; ++j) {                  // patch order fixes the order of the additions
          const float* sp = stale_copy + (((long long)j * B + b) * G + g) * 2;
          const float av = sp[0], cv = sp[1];
          if (j == patch_idx) { own_s = av; own_q = cv; } else { st_s += av; st_q += cv; }
        }
      }
      const GnMoments mo = gn_combine_pre(tot_s, tot_q, n_seg, nseg, N, stat_mode, st_s, st_q, own_s, own_q, eps);
      if (nseg == 1 && sums_out != nullptr && blk == 0) {   // may alias the patch's slot of the cache: every block reads
        float* o = sums_out + ((long long)b * G + g) * 2;   // the snapshot, never the cache itself
        o[0] = (float)tot_s; o[1] = (float)tot_q;
      }
      s_mom[g][0] = mo.mean_hi; s_mom[g][1] = mo.mean_lo; s_mom[g][2] = mo.rstd;
    }
    __syncthreads();
  }
  if (!works) return;
  float sc[V], sh[V], mh[V], ml[V];
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const int c = c0 + i;
    const int g = c / cg;
    mh[i] = s_mom[g][0]; ml[i] = s_mom[g][1];
    sc[i] = s_mom[g][2] * gamma[c];
    sh[i] = beta[c];
  }
  for (int p0 = p_lo + psub; p0 < p_hi; p0 += NCH * ppb) {
    if (p0 != p_lo + psub) {                   // further chunks of a long strip
#pragma unroll
      for (int k = 0; k < NCH; ++k) {
        const int p = p0 + k * ppb;
        raw[k] = *reinterpret_cast<const u32x4*>(x + (base + (p < p_hi ? p : p0)) * C + c0);
      }
    }
#pragma unroll
   for (int k = 0; k < NCH; ++k) {
    const int p = p0 + k * ppb;
    if (p >= p_hi) break;
    float v[V];
    unpack_vec<Tin>(raw[k], v);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float t = fmaf((v[i] - mh[i]) - ml[i], sc[i], sh[i]);
      v[i] = silu ? silu_f(t) : t;
    }
    const long long m = base + p;
    Tout* o = y + m * C + c0;
    if (packed) {
      // fragment-packed bf16 operand of the linear layers: pixel m is row m%32 of fragment row m/32, the
      // 8 channels from c0 & ~7 sit in slot (m%32) + 32*((c0/8)%2) of fragment column c0/16
      o = y + (((m >> 5) * (C >> 4) + (c0 >> 4)) * 64 + (m & 31) + 32 * ((c0 >> 3) & 1)) * 8 + (c0 & 7);
    }
    if constexpr (sizeof(Tout) == sizeof(Tin)) {
      st_vec(o, v);
    } else {  // float in, bf16 out: 4 values = 8 bytes
      u32x2 t = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3])};
      *reinterpret_cast<u32x2*>(o) = t;
    }
    if constexpr (sizeof(Tout) == 2) {
      if (halo.out) halo_store<V>(halo, b, (long long)seg * pix_seg + p, C, c0, v);
    }
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

// Strips of the two-launch path: as close to target_blocks strips as the pixel count allows (the chip has 256
// compute units and a strip is one block in either launch); a small tensor gets short strips and blocks with few
// pixel slots rather than few blocks.
GnLayout gn_layout(int C, int vec, long long pix, int target_blocks, int max_threads, int min_threads) {
  GnLayout L;
  L.tp = C / vec;
  long long per = (pix + target_blocks - 1) / target_blocks;
  L.ppb = max_threads / L.tp;
  if (L.ppb > kGnMaxPpb) L.ppb = kGnMaxPpb;
  if (L.ppb > per) L.ppb = (int)per;
  if (L.ppb * L.tp < min_threads) L.ppb = (min_threads + L.tp - 1) / L.tp;   // the kernels give every group a thread
  if (L.ppb < 1) L.ppb = 1;
  L.threads = L.tp * L.ppb;
  per = (per + L.ppb - 1) / L.ppb * L.ppb;
  L.pix_per_blk = (int)per;
  L.nblk = (int)((pix + per - 1) / per);
  return L;
}

}  // namespace

size_t groupnorm_scratch_bytes(int B, int nseg, int G, int N) {
  // snapshot of the cached sums + partials of at most kGnMaxStrips strips per batch item
  (void)nseg;
  return kScratchCounterBytes + ((size_t)B * kGnMaxStrips * G * 2 + (size_t)N * B * G * 2 + 64) * sizeof(float) + 1024;
}

int launch_groupnorm(const GnArgs& a, hipStream_t st) {
  const int vec = a.in_dtype == DF_BF16 ? 8 : 4;
  if (a.C % a.G || a.C % vec || a.G > kMaxG || a.C / vec > 1024) return DF_ESHAPE;
  if (a.in_dtype == DF_BF16 && a.out_dtype != DF_BF16) return DF_ESHAPE;
  if (a.B > 1024) return DF_ESHAPE;
  if (a.y_packed && (a.out_dtype != DF_BF16 || a.C % 16)) return DF_ESHAPE;
  const long long pix_seg = (long long)a.Rseg * a.W;
  GnHalo halo = {};
  if (a.halo_out && a.halo_cols) {
    if (a.out_dtype != DF_BF16 || a.y_packed || a.halo_rpp <= 0 || a.W % a.halo_rpp || a.halo_patch0 < 0 ||
        a.halo_patch0 + a.W / a.halo_rpp > a.halo_npatch || ((uintptr_t)a.halo_out % 16))
      return DF_EINVAL;
    halo.out = (bf16_t*)a.halo_out; halo.W = a.W; halo.rpp = a.halo_rpp; halo.patch0 = a.halo_patch0;
    halo.npatch = a.halo_npatch; halo.cols = 1; halo.rows = a.Rseg * a.nseg;
  } else if (a.halo_out) {
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
    const int ppass = (cg % 4 == 0 && cg / 4 <= 1024) ? 1024 / (cg / 4) : 0;
    const bool fits_regs = a.nseg == 1 && pix_seg <= (long long)ppass * 8;
    if (!no_fused && cg % 4 == 0 && cg / 4 <= 1024 && (fits_regs || per_group <= kGnGroupMaxElems)) {
      dim3 grid(a.G, a.B);
      if (fits_regs) {
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
  // Both launches use the same partition of the pixels into strips, at most kGnMaxStrips per batch item: every block
  // of the second launch reads all partials of its batch item, so their number is bounded, and a block normalises
  // the strip whose sums it (or a block on the same XCD) took, which is then still in that XCD's L2 for tensors of a
  // few MB per XCD.
  int target = kGnMaxStrips / a.nseg;
  if (target < 1) target = 1;
  GnLayout L = gn_layout(a.C, vec, pix_seg, target, 1024, a.G);
  if (L.threads > 1024 || L.ppb > kGnMaxPpb) return DF_ESHAPE;
  char* scr = scratch_region(a.scr, groupnorm_scratch_bytes(a.B, a.nseg, a.G, a.N));
  if (!scr) return DF_ENOMEM;
  const bool need_stale = !(a.nseg > 1 || (a.N == 1 && a.stat_mode != DF_GN_STALE));
  const int stale_n = need_stale ? a.N * a.B * a.G * 2 : 0;
  float* stale_copy = (float*)(scr + kScratchCounterBytes);
  float* partial = stale_copy + (((size_t)a.N * a.B * a.G * 2 + 63) / 64) * 64;
  dim3 gs(L.nblk, a.nseg, a.B);
  const size_t lds = (size_t)vec * L.threads * sizeof(float);
  const int thr_apply = L.threads < a.G ? a.G : L.threads;   // the fold needs a lane per group
  const int iters = L.pix_per_blk / L.ppb;              // pixels per lane and strip
#define DF_GN_STATS(TI, NCHV)                                                                                         \
  hipLaunchKernelGGL((gn_stats<TI, NCHV>), gs, dim3(L.threads), lds, st, (const TI*)a.x, partial, (int)pix_seg, a.C,  \
                     a.G, L.tp, L.ppb, L.pix_per_blk, a.nseg, need_stale ? a.stale : nullptr, stale_copy, stale_n)
#define DF_GN_APPLY(TI, TO, NCHV)                                                                                     \
  hipLaunchKernelGGL((gn_apply<TI, TO, NCHV>), gs, dim3(thr_apply), 0, st, (const TI*)a.x, (TO*)a.y, partial,         \
                     stale_copy, a.sums_out, a.gamma, a.beta, (int)pix_seg, a.C, a.G, L.nblk, a.nseg, a.B, a.patch_idx, \
                     a.N, a.eps, a.stat_mode, L.tp, L.ppb, L.pix_per_blk, a.silu, a.y_packed, halo)
#define DF_GN_BOTH(NCHV)                                                                                              \
  {                                                                                                                   \
    if (a.in_dtype == DF_BF16) DF_GN_STATS(bf16_t, NCHV); else DF_GN_STATS(float, NCHV);                              \
    DF_LAUNCH_CHECK();                                                                                                \
    if (a.in_dtype == DF_BF16) DF_GN_APPLY(bf16_t, bf16_t, NCHV);                                                     \
    else if (a.out_dtype == DF_BF16) DF_GN_APPLY(float, bf16_t, NCHV);                                                \
    else DF_GN_APPLY(float, float, NCHV);                                                                             \
  }
  if (iters <= 1) DF_GN_BOTH(1) else if (iters <= 2) DF_GN_BOTH(2) else if (iters <= 4) DF_GN_BOTH(4) else DF_GN_BOTH(8)
#undef DF_GN_BOTH
#undef DF_GN_APPLY
#undef DF_GN_STATS
  DF_LAUNCH_CHECK();
  return DF_OK;
}

// Per-strip sums of a full image for vertical strips (the synchronous step only: not on the hot path).  One
// workgroup per (strip, group, batch item); sums of x minus the group's pivot, ordered fold, turned into sums of x
// in double.
template <typename Tin>
__global__ __launch_bounds__(256) void gn_strip_sums_kernel(const Tin* __restrict__ x, float* __restrict__ sums, int B,
                                                            int R, int W, int C, int G, int N) {
  __shared__ float s_s[256], s_q[256];
  const int j = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int cg = C / G, Wp = W / N;
  const float piv = Elem<Tin>::ld(x + (long long)b * R * W * C + g * cg);
  const long long n = (long long)R * Wp * cg;
  float a = 0.f, q = 0.f;
  for (long long i = tid; i < n; i += 256) {
    const int ch = (int)(i % cg);
    const long long px = i / cg;
    const int c = (int)(px % Wp), r = (int)(px / Wp);
    const float d = Elem<Tin>::ld(x + (((long long)b * R + r) * W + j * Wp + c) * C + g * cg + ch) - piv;
    a += d; q = fmaf(d, d, q);
  }
  s_s[tid] = a; s_q[tid] = q;
  __syncthreads();
  if (tid == 0) {
    float fs = 0.f, fq = 0.f;
    for (int k = 0; k < 256; ++k) { fs += s_s[k]; fq += s_q[k]; }
    double S, SS;
    gn_unshift(fs, fq, (double)n, piv, S, SS);
    float* o = sums + (((long long)j * B + b) * G + g) * 2;
    o[0] = (float)S; o[1] = (float)SS;
  }
}

int launch_gn_strip_sums(const void* x, int in_dtype, float* sums, int B, int R, int W, int C, int G, int N, hipStream_t st) {
  if (B <= 0 || R <= 0 || W <= 0 || C <= 0 || G <= 0 || N <= 0 || C % G || W % N || G > 65535 || B > 65535) return DF_ESHAPE;
  dim3 grid(N, G, B);
  if (in_dtype == DF_BF16)
    hipLaunchKernelGGL(gn_strip_sums_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)x, sums, B, R, W, C, G, N);
  else
    hipLaunchKernelGGL(gn_strip_sums_kernel<float>, grid, dim3(256), 0, st, (const float*)x, sums, B, R, W, C, G, N);
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
  // the statistics pass keeps up to 256 partial (sum, sum of squares) pairs per batch item and group, plus a snapshot
  // of the cached sums
  if (N <= 0 || df::groupnorm_scratch_bytes(B, 1, G, N) > kStaticScratchBytes) return DF_ENOMEM;
  df::Scratch region = {nullptr, 0};
  const int rc = static_scratch_region(&region);
  if (rc != DF_OK) return rc;
  // nothing in the region has to start at zero: every partial and every statistic is written before it is read
  return df::groupnorm_entry(x_fresh, y, stale_stats, fresh_stats_out, gamma, beta, B, R, W, C, G, patch_idx, N, eps,
                             stat_mode, fuse_silu, dtype, &region, (hipStream_t)stream);
}

#pragma GCC visibility pop
}  // extern "C"
