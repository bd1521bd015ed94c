// Linear layers of the patch on MFMA-fragment-packed operands (Section 4, Sparse operations: linear layers act on
// the fresh tokens only).
//
// The patch's linear layers have few rows (300-1200 tokens) and short reductions, so a workgroup-tiled GEMM spends
// its time on barriers and LDS round trips, not on the matrix pipe.  Here neither operand touches LDS in the K loop:
//   - activations and weights are stored in the order the MFMA consumes them: a fragment is 32 rows x 16 k
//     = 64 lanes x 16 bytes = 1 KB contiguous, lane l holding row l%32, k = 8*(l/32) .. +7, so one
//     global_load_dwordx4 per lane fetches an operand, perfectly coalesced, straight into registers;
//   - a wave owns a (TM*32 tokens) x (TN*32 features) output tile and a 1/KSPLIT share of K; the KSPLIT waves of a
//     workgroup add their partial tiles through LDS in wave order at the end (fixed order: results are
//     reproducible), so even a 300 x 1280 output puts ~800 waves on the chip;
//   - loads run PF k-steps ahead in a register ring; there is no barrier inside the K loop.
// The product is computed transposed (weights as the A operand, tokens as the B operand), so a lane ends up with
// one token and 16 features.  Weight rows are stored with bits 2 and 3 of the in-fragment row index swapped, which
// makes those 16 features two runs of 8 consecutive ones: exactly the 16 bytes that the same lane of the *next*
// layer's activation fragment holds.  The epilogue therefore writes the next layer's packed operand with one
// 16-byte store per lane and no data exchange.
#include "kernels.h"

namespace df {

namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_w;

struct WParams {
  const bf16x8* Xp;
  const bf16x8* Wp;
  int M, N, K;          // N: rows of W that produce outputs (geglu: F value rows; the gate rows follow at row F)
  const float* bias;
  const float* ln_s;
  const float* ln_t;
  float ln_eps;
  const float* residual;
  long long ldr;
  float* out_f32;
  long long ldo;
  bf16_t* out_packed;
  bf16_t* out_rows;
  long long ld_rows;
  int geglu;
  int nseg, seg_w;
  bf16_t* seg_out[3];
  long long seg_ld[3], seg_rows_out[3], seg_row0[3];
  int seg_rows_in[3];
  int seg_tr[3];
  int seg_pin[3], seg_pout[3];
  // fused cross-attention (XA > 0): per (batch item, head) 8*XA key fragments then 4*XA value fragments
  const bf16x8* xkv;
  int xa_keys;          // valid text tokens
  long long xa_bstride; // fragments between batch items
  int xa_rows;          // token rows per batch item
  float xa_scale;
};


// XA > 0 (TM = 1, TN = 2, KSPLIT = 4, N = one head per workgroup): the 64 output features are the query of one
// attention head; cross-attention against XA 32-key tiles of packed text keys / values runs in the epilogue and the
// kernel writes the attention output (packed) instead of the projection.
#ifdef DF_TUNING
// Tuning build only: per workgroup (wave 0), the constant-rate clock at entry and exit and cycle stamps between.
__device__ long long g_wg_trace[1024 * 16];
#define DF_WTRACE(slot, expr)                                                                   \
  do {                                                                                          \
    if (threadIdx.x == 0 && blockIdx.x < 1024) g_wg_trace[blockIdx.x * 16 + (slot)] = (long long)(expr); \
  } while (0)
#else
#define DF_WTRACE(slot, expr) do {} while (0)
#endif

template <int TM, int TN, int KSPLIT, int PF, bool LN, int XA>
__global__ __launch_bounds__(64 * KSPLIT) void wgemm_kernel(WParams p) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  DF_WTRACE(0, wall_clock64());
  DF_WTRACE(1, __builtin_readcyclecounter());
  // rows of token fragments reduced per pass: as many as fit in 128 KB of LDS (the whole tile, half of it, or one row)
  constexpr int RP = (KSPLIT * TM * TN * 4 <= 128) ? TM : (TM % 2 == 0 && KSPLIT * (TM / 2) * TN * 4 <= 128) ? TM / 2 : 1;
  constexpr int U = RP * TN * 4;            // float4 units of a pass: (row, tn, jj)
  f32x4* red = reinterpret_cast<f32x4*>(smem_raw);                       // [KSPLIT][U][64], reused per pass
  float* stat = reinterpret_cast<float*>(smem_raw + KSPLIT * U * 1024);  // [KSPLIT][TM][32][2]
  u32x4* qlds = reinterpret_cast<u32x4*>(smem_raw + KSPLIT * U * 1024 + KSPLIT * TM * 32 * 2 * 4);   // [4][64] (XA)
  float* vecs = reinterpret_cast<float*>(smem_raw + KSPLIT * U * 1024 + KSPLIT * TM * 32 * 2 * 4 + (XA > 0 ? 4096 : 0));   // [4][128]
  constexpr int GP = TN >= 2 ? TN / 2 : 1;   // geglu: the tile's first GP fragments are value rows, the last GP their gates

  // Every kernel argument the prologue needs is requested here, in one batch: left to the compiler, the scalar loads
  // of arguments first used under a condition (norm vectors, bias, residual, operand pointers) are issued where that
  // code starts, and the prologue of these few-microsecond kernels became a chain of four or five dependent round
  // trips to the scalar cache.
  asm volatile("" ::"s"(p.Xp), "s"(p.Wp), "s"(p.M), "s"(p.N), "s"(p.K), "s"(p.bias), "s"(p.ln_s), "s"(p.ln_t),
               "s"(p.residual), "s"(p.ldr), "s"(p.geglu));
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: the k-walk and tile addresses stay off the vector ALU
  const int tok = lane & 31, g = lane >> 5;
  const int MT = (p.M + 31) >> 5;                      // 32-token fragments rows
  const int MG = (MT + TM - 1) / TM;                   // tile groups along M
  const int NTo = p.N >> 5;                            // 32-feature output fragments
  const int NG = p.geglu ? NTo / GP : NTo / TN;        // geglu: fragment j < GP is paired with gate fragment j + GP
  const int nwg = MG * NG;
  int t = blockIdx.x;
  {
    // workgroups go round-robin over the 8 XCDs; give each XCD a contiguous run of tiles, token tiles fastest, so
    // that the workgroups that share a weight fragment sit behind the same L2
    const int xcd = t & 7, loc = t >> 3;
    const int base = nwg >> 3, rem = nwg & 7;
    t = xcd * base + (xcd < rem ? xcd : rem) + loc;
  }
  const int mg = t % MG, ng = t / MG;
  const int KF = p.K >> 4, KFw = KF / KSPLIT;
  const int kf0 = wave * KFw;
#ifdef DF_TUNING
  asm volatile("" ::"s"(kf0), "s"(mg), "s"(ng));
#endif
  DF_WTRACE(6, __builtin_readcyclecounter());

  const bf16x8* xb[TM];
  const bf16x8* wb[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    int mt = mg * TM + i;
    if (mt > MT - 1) mt = MT - 1;                     // ragged last group: recompute the last fragment row, never stored
    xb[i] = p.Xp + ((size_t)mt * KF + kf0) * 64 + lane;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int nt = p.geglu ? (j < GP ? ng * GP + j : NTo + ng * GP + (j - GP)) : ng * TN + j;
    wb[j] = p.Wp + ((size_t)nt * KF + kf0) * 64 + lane;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  float ln_sum[TM], ln_sq[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) { ln_sum[i] = 0.f; ln_sq[i] = 0.f; }
  constexpr bool ln = LN;

  // Epilogue operands are requested before the K loop: their latency would otherwise sit, un-overlapped, at the end
  // of every one of these short kernels.  A pair unit = (token fragment row i, output fragment j, half f): 8
  // consecutive features per lane.  The tile is reduced and written in passes of RP rows; the pair units of a pass go
  // round-robin over the waves, which run the epilogue for them.
  // The per-feature vectors (norm scale / shift or bias, of the value and of the gate half) are the same for every
  // token: wave v < 4 fetches vector v for the tile's whole feature range with ONE load (<= 128 floats) and parks it
  // in LDS for the epilogue.  Fetched per unit and lane they were 8-32 extra vector-memory instructions per wave, each
  // of which costs the compute unit's load path as much as a 1 KB operand fragment.
  const int JO = p.geglu ? GP : TN;                    // output fragments per row of the tile
  const int npu = RP * JO * 2;
  static_assert(KSPLIT >= 4, "one wave per parked vector");
  f32x4 vec_pre = {0.f, 0.f, 0.f, 0.f};
  {
    const int n0 = ng * JO * 32;
    const bool gg = TN >= 2 && p.geglu;
    const float* src = nullptr;                        // (uniform)
    if (ln) src = wave == 0 ? p.ln_s + n0 : wave == 1 ? p.ln_t + n0 : (gg && wave == 2) ? p.ln_s + p.N + n0
                                                          : (gg && wave == 3) ? p.ln_t + p.N + n0 : nullptr;
    else if (p.bias) src = wave == 0 ? p.bias + n0 : (gg && wave == 2) ? p.bias + p.N + n0 : nullptr;
    if (src && lane * 4 < JO * 32) vec_pre = *reinterpret_cast<const f32x4*>(src + 4 * lane);
  }
  struct Epi { float r[8]; };
  auto load_epi = [&](int i0, int pu, Epi& e) {
    const int f = pu & 1;
    const int j = p.geglu ? (pu >> 1) % GP : (pu >> 1) % TN;          // compile-time divisors (JO is a run-time value)
    const int mt = mg * TM + i0 + (p.geglu ? (pu >> 1) / GP : (pu >> 1) / TN);
    const int m = mt * 32 + tok;
    const int n = (ng * JO + j) * 32 + 16 * f + 8 * g;
    if (p.residual && m < p.M) {
      ld_vec(p.residual + (long long)m * p.ldr + n, e.r); ld_vec(p.residual + (long long)m * p.ldr + n + 4, e.r + 4);
    }
  };
  constexpr int MAXU = (RP * TN * 2 + KSPLIT - 1) / KSPLIT;   // pair units of a pass per wave
  constexpr int NPRE = MAXU < 3 ? MAXU : 3;
  Epi epre[NPRE];
#pragma unroll
  for (int t = 0; t < NPRE; ++t)
    if (wave + t * KSPLIT < npu) load_epi(0, wave + t * KSPLIT, epre[t]);
  DF_WTRACE(7, __builtin_readcyclecounter());
  // fused cross-attention: the wave that runs it also requests the head's key fragments now
  bf16x8 xkf[XA > 0 ? XA : 1][4];
  const bf16x8* xkv_ptr = nullptr;
  if constexpr (XA > 0) {
    const int bi = (int)(((long long)mg * 32) / p.xa_rows);   // TM == 1; a fragment row never straddles batch items when
                                                              // rows % 32 == 0, otherwise the launcher requires one item
    xkv_ptr = p.xkv + (size_t)bi * p.xa_bstride + (size_t)ng * (12 * XA) * 64 + lane;
    if (wave == 0) {
#pragma unroll
      for (int kt = 0; kt < XA; ++kt)
#pragma unroll
        for (int ds = 0; ds < 4; ++ds) xkf[kt][ds] = xkv_ptr[(size_t)(kt * 4 + ds) * 64];
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  bf16x8 xr[PF][TM], wr[PF][TN];
  // The loop body is straight-line code (no branches): KFw % PF == 0 (launcher), refills past the end re-read the
  // wave's last fragment.  Every wave walks its k-range from a different starting fragment (wrapping around): the
  // streams of all waves are otherwise aligned modulo the fragment-row pitch and hit the same few L2 / memory
  // channels at any moment.  The order is a fixed function of the tile, so results stay reproducible.
  const int rot = (int)((unsigned)(mg * 7 + ng * 3 + wave * 5) % (unsigned)KFw);
  auto pos = [&](int step) {
    if (step > KFw - 1) step = KFw - 1;
    const int k = step + rot;
    return (size_t)(k < KFw ? k : k - KFw) * 64;
  };
#pragma unroll
  for (int s = 0; s < PF; ++s) {
    const size_t o = pos(s);
#pragma unroll
    for (int i = 0; i < TM; ++i) xr[s][i] = xb[i][o];
#pragma unroll
    for (int j = 0; j < TN; ++j) wr[s][j] = wb[j][o];
  }
  __builtin_amdgcn_sched_barrier(0);
  DF_WTRACE(2, __builtin_readcyclecounter());
  for (int kf = 0; kf < KFw; kf += PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[s][j], xr[s][i], acc[i][j], 0, 0, 0);
      if constexpr (ln) {
        // row sums of the tokens for the folded LayerNorm (vector ALU, beside the matrix pipe)
        const bf16x2_w ones = __builtin_bit_cast(bf16x2_w, 0x3f803f80u);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const u32x4 raw = __builtin_bit_cast(u32x4, xr[s][i]);
          const unsigned int wds[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const bf16x2_w v2 = __builtin_bit_cast(bf16x2_w, wds[q]);
            ln_sum[i] = __builtin_amdgcn_fdot2_f32_bf16(v2, ones, ln_sum[i], false);
            ln_sq[i] = __builtin_amdgcn_fdot2_f32_bf16(v2, v2, ln_sq[i], false);
          }
        }
      }
      const size_t o = pos(kf + s + PF);
#pragma unroll
      for (int i = 0; i < TM; ++i) xr[s][i] = xb[i][o];
#pragma unroll
      for (int j = 0; j < TN; ++j) wr[s][j] = wb[j][o];
      __builtin_amdgcn_sched_barrier(0);               // keep the refill here, PF steps ahead of its use
    }
  }

  DF_WTRACE(3, __builtin_readcyclecounter());
  // ---- add the KSPLIT partial tiles in wave order, one token-fragment row at a time ----
  if (ln) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const float sm = ln_sum[i] + __shfl_xor(ln_sum[i], 32, 64);   // the two lane groups hold different k
      const float sq = ln_sq[i] + __shfl_xor(ln_sq[i], 32, 64);
      if (g == 0) {
        stat[((wave * TM + i) * 32 + tok) * 2] = sm;
        stat[((wave * TM + i) * 32 + tok) * 2 + 1] = sq;
      }
    }
  }
#pragma unroll
  for (int i0 = 0; i0 < TM; i0 += RP) {
  if (i0 > 0) __syncthreads();                         // the previous pass's partial tiles have been read
#pragma unroll
  for (int il = 0; il < RP; ++il)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const f32x16& t = acc[i0 + il][j];
        const f32x4 v = {t[4 * jj], t[4 * jj + 1], t[4 * jj + 2], t[4 * jj + 3]};
        red[(wave * U + (il * TN + j) * 4 + jj) * 64 + lane] = v;
      }
  if (i0 == 0 && wave < 4 && lane * 4 < JO * 32) *reinterpret_cast<f32x4*>(vecs + wave * 128 + 4 * lane) = vec_pre;
  __syncthreads();
  DF_WTRACE(8 + 2 * (i0 / RP < 4 ? i0 / RP : 3), __builtin_readcyclecounter());

#pragma unroll
  for (int t = 0; t < MAXU; ++t) {
    const int pu = wave + t * KSPLIT;
    if (pu >= npu) break;
    const int f = pu & 1;
    const int j = p.geglu ? (pu >> 1) % GP : (pu >> 1) % TN;
    const int il = p.geglu ? (pu >> 1) / GP : (pu >> 1) / TN;
    const int i = i0 + il;
    const int mt = mg * TM + i;
    if (mt >= MT) continue;
    Epi e;
    if (t < NPRE && i0 == 0) e = epre[t < NPRE ? t : 0];   // the residual rows of the first pass were requested early
    else load_epi(i0, pu, e);
    const float* vq = vecs + j * 32 + 16 * f + 8 * g;  // this lane's 8 features in the parked vectors
    auto vec8 = [&](int which, float* o) {
      const f32x4 lo = *reinterpret_cast<const f32x4*>(vq + which * 128), hi = *reinterpret_cast<const f32x4*>(vq + which * 128 + 4);
      o[0] = lo.x; o[1] = lo.y; o[2] = lo.z; o[3] = lo.w; o[4] = hi.x; o[5] = hi.y; o[6] = hi.z; o[7] = hi.w;
    };
    float v[8], gt[8];
    {
      f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = a;
#pragma unroll
      for (int w = 0; w < KSPLIT; ++w) {
        a += red[(w * U + (il * TN + j) * 4 + 2 * f) * 64 + lane];
        b += red[(w * U + (il * TN + j) * 4 + 2 * f + 1) * 64 + lane];
      }
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    if (TN >= 2 && p.geglu) {
      f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = a;
#pragma unroll
      for (int w = 0; w < KSPLIT; ++w) {
        a += red[(w * U + (il * TN + j + GP) * 4 + 2 * f) * 64 + lane];
        b += red[(w * U + (il * TN + j + GP) * 4 + 2 * f + 1) * 64 + lane];
      }
      gt[0] = a.x; gt[1] = a.y; gt[2] = a.z; gt[3] = a.w; gt[4] = b.x; gt[5] = b.y; gt[6] = b.z; gt[7] = b.w;
    }
    const int m = mt * 32 + tok;
    const int nfrag = ng * JO + j;                     // output fragment along the feature axis
    const int n = nfrag * 32 + 16 * f + 8 * g;         // first of this lane's 8 consecutive features
    if (ln) {
      float sm = 0.f, sq = 0.f;
#pragma unroll
      for (int w = 0; w < KSPLIT; ++w) {
        sm += stat[((w * TM + i) * 32 + tok) * 2];
        sq += stat[((w * TM + i) * 32 + tok) * 2 + 1];
      }
      // hardware reciprocal and reciprocal square root (1 ulp) in place of the IEEE division and square root
      // sequences: this epilogue runs once per workgroup and is not hidden behind anything
      const float inv_k = __builtin_amdgcn_rcpf((float)p.K);
      const float mean = sm * inv_k;
      const float var = fmaxf(fmaf(sq, inv_k, -mean * mean), 0.f);
      const float rstd = __builtin_amdgcn_rsqf(var + p.ln_eps);
      float ea[8], eb[8];
      vec8(0, ea); vec8(1, eb);
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = rstd * (v[q] - mean * ea[q]) + eb[q];
      if (TN >= 2 && p.geglu) {
        vec8(2, ea); vec8(3, eb);
#pragma unroll
        for (int q = 0; q < 8; ++q) gt[q] = rstd * (gt[q] - mean * ea[q]) + eb[q];
      }
    } else if (p.bias) {
      float ea[8];
      vec8(0, ea);
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] += ea[q];
      if (TN >= 2 && p.geglu) {
        vec8(2, ea);
#pragma unroll
        for (int q = 0; q < 8; ++q) gt[q] += ea[q];
      }
    }
    if (TN >= 2 && p.geglu) {
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] *= gelu_erf(gt[q]);
    }
    if constexpr (XA > 0) {
      // this wave's 8 features x 32 tokens are the d-step 2*j + f of the head's Q^T operand
      u32x4 qv = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]), pack_bf2(v[4], v[5]), pack_bf2(v[6], v[7])};
      qlds[(2 * j + f) * 64 + lane] = qv;
      continue;
    }
    const bool row_ok = m < p.M;
    if (p.residual && row_ok) {
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] += e.r[q];
    }
    if (p.out_f32 && row_ok) {
      st_vec(p.out_f32 + (long long)m * p.ldo + n, v);
      st_vec(p.out_f32 + (long long)m * p.ldo + n + 4, v + 4);
    }
    if (p.out_packed) {
      // fragment (mt, n/16) of the [M, N] result as the next layer's activation operand; padded token rows are
      // written too (they only ever feed padded rows)
      const int KFo = p.N >> 4;
      st_vec(p.out_packed + (((size_t)mt * KFo + (n >> 4)) * 64 + lane) * 8, v);
    }
    if (row_ok) {
      if (p.nseg > 0) {
        // 8 features never straddle a segment (seg_w % 32 == 0); at most three segments, usually one batch item:
        // comparisons instead of integer divisions
        const int sg = (n >= p.seg_w ? 1 : 0) + (n >= 2 * p.seg_w ? 1 : 0);
        const int bi = m < p.seg_rows_in[sg] ? 0 : m / p.seg_rows_in[sg];
        if (p.seg_tr[sg]) {
          // feature-major output: the 32 tokens of a half wave are consecutive in memory for each feature
          bf16_t* o = p.seg_out[sg] + ((long long)bi * p.seg_w + (n - sg * p.seg_w)) * p.seg_ld[sg] + p.seg_row0[sg] +
                      seg_pos(m - bi * p.seg_rows_in[sg], p.seg_pin[sg], p.seg_pout[sg]);
#pragma unroll
          for (int q = 0; q < 8; ++q) o[q * p.seg_ld[sg]] = f2bf(v[q]);
        } else {
          const long long orow = (long long)bi * p.seg_rows_out[sg] + p.seg_row0[sg] +
                                 seg_pos(m - bi * p.seg_rows_in[sg], p.seg_pin[sg], p.seg_pout[sg]);
          st_vec(p.seg_out[sg] + orow * p.seg_ld[sg] + (n - sg * p.seg_w), v);
        }
      } else if (p.out_rows) {
        st_vec(p.out_rows + (long long)m * p.ld_rows + n, v);
      }
    }
  }
  DF_WTRACE(9 + 2 * (i0 / RP < 4 ? i0 / RP : 3), __builtin_readcyclecounter());
  }
  DF_WTRACE(4, __builtin_readcyclecounter());
  DF_WTRACE(5, wall_clock64());
  if constexpr (XA > 0) {
    __syncthreads();
    if (wave != 0) return;
    // one wave: S^T = K Q^T over XA key tiles (lane = token, 16 keys per tile in natural order thanks to the row
    // permutation of the packed keys), softmax over the valid keys, O^T = V^T P^T, packed output
    const int mt = mg;                                   // TM == 1
    const bf16x8* kv = xkv_ptr;
    bf16x8 qf[4];
#pragma unroll
    for (int ds = 0; ds < 4; ++ds) qf[ds] = __builtin_bit_cast(bf16x8, qlds[ds * 64 + lane]);
    auto& kf = xkf;
    bf16x8 vf[2][2 * XA];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int ks = 0; ks < 2 * XA; ++ks) vf[dt][ks] = kv[(size_t)(4 * XA + dt * 2 * XA + ks) * 64];
    f32x16 sa[XA];
#pragma unroll
    for (int kt = 0; kt < XA; ++kt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sa[kt][e] = 0.f;
#pragma unroll
      for (int ds = 0; ds < 4; ++ds) sa[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kt][ds], qf[ds], sa[kt], 0, 0, 0);
    }
    const float sc = p.xa_scale * 1.4426950408889634f;
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < XA; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = kt * 32 + 16 * (e >> 3) + 8 * g + (e & 7);
        if (key >= p.xa_keys) sa[kt][e] = -INFINITY;
        mx = fmaxf(mx, sa[kt][e]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sc;
    float l = 0.f;
#pragma unroll
    for (int kt = 0; kt < XA; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(sa[kt][e], sc, -mx));
        sa[kt][e] = pv;
        l += pv;
      }
    l += __shfl_xor(l, 32, 64);
    f32x16 oa[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) oa[dt][e] = 0.f;
    }
#pragma unroll
    for (int ks = 0; ks < 2 * XA; ++ks) {
      const int kt = ks >> 1, hf = ks & 1;
      u32x4 pk;
      pk.x = pack_bf2(sa[kt][8 * hf + 0], sa[kt][8 * hf + 1]);
      pk.y = pack_bf2(sa[kt][8 * hf + 2], sa[kt][8 * hf + 3]);
      pk.z = pack_bf2(sa[kt][8 * hf + 4], sa[kt][8 * hf + 5]);
      pk.w = pack_bf2(sa[kt][8 * hf + 6], sa[kt][8 * hf + 7]);
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) oa[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][ks], pf, oa[dt], 0, 0, 0);
    }
    const float inv = 1.0f / l;
    const int KFo = p.N >> 4;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int f2 = 0; f2 < 2; ++f2) {
        float o8[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) o8[q] = oa[dt][8 * f2 + q] * inv;
        st_vec(p.out_packed + (((size_t)mt * KFo + ng * 4 + dt * 2 + f2) * 64 + lane) * 8, o8);
      }
  }
}

// row-major [M, K] bf16 -> fragments [ceil(M/32)][K/16][64][8]; rows beyond M are zero
__global__ void pack_rows_kernel(const bf16_t* __restrict__ x, long long ldx, u32x4* __restrict__ out, int M, int K,
                                 long long total) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;   // one 16-byte lane slot
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const long long frag = idx >> 6;
  const int KF = K >> 4;
  const int kf = (int)(frag % KF);
  const long long mt = frag / KF;
  const long long m = mt * 32 + (lane & 31);
  u32x4 v = {0u, 0u, 0u, 0u};
  if (m < M) v = *reinterpret_cast<const u32x4*>(x + m * ldx + kf * 16 + 8 * (lane >> 5));
  out[idx] = v;
}

// [N, K] bf16 weights -> fragments [N/32][K/16][64][8] with in-fragment row i holding weight row
// (i with bits 2 and 3 swapped), optionally scaled per input channel by gamma before rounding
__global__ void pack_wfrag_kernel(const bf16_t* __restrict__ w, const float* __restrict__ gamma,
                                  u32x4* __restrict__ out, int N, int K, long long total) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const long long frag = idx >> 6;
  const int KF = K >> 4;
  const int kf = (int)(frag % KF);
  const long long nt = frag / KF;
  const int i = lane & 31;
  const int row = (i & 0x13) | ((i & 4) << 1) | ((i & 8) >> 1);
  const long long n = nt * 32 + row;
  const int k0 = kf * 16 + 8 * (lane >> 5);
  u32x4 v = *reinterpret_cast<const u32x4*>(w + n * K + k0);
  if (gamma) {
    const unsigned int wd[4] = {v.x, v.y, v.z, v.w};
    unsigned int o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float lo = __uint_as_float(wd[q] << 16) * gamma[k0 + 2 * q];
      const float hi = __uint_as_float(wd[q] & 0xffff0000u) * gamma[k0 + 2 * q + 1];
      o[q] = pack_bf2(lo, hi);
    }
    v.x = o[0]; v.y = o[1]; v.z = o[2]; v.w = o[3];
  }
  out[idx] = v;
}

template <int TM, int TN, int KSPLIT, int PFMAX>
int launch_cfg(const WParams& p, hipStream_t st);

__global__ void pack_text_kv_kernel(const bf16_t* __restrict__ kv, long long ld, u32x4* __restrict__ out, int B, int TL,
                                    int count, int C, int XA, long long total) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  long long frag = idx >> 6;
  const int heads = C / 64, per_head = 12 * XA;
  const int fr = (int)(frag % per_head); frag /= per_head;
  const int hh = (int)(frag % heads); frag /= heads;
  const int j = (int)(frag % count);
  const int b = (int)(frag / count);
  const int i = lane & 31, g = lane >> 5;
  const int sig = (i & 0x13) | ((i & 4) << 1) | ((i & 8) >> 1);
  u32x4 v = {0u, 0u, 0u, 0u};
  if (fr < 4 * XA) {
    const int kt = fr >> 2, ds = fr & 3;
    const int key = kt * 32 + sig;
    if (key < TL)
      v = *reinterpret_cast<const u32x4*>(kv + ((long long)b * TL + key) * ld + (long long)j * 2 * C + hh * 64 + ds * 16 + 8 * g);
  } else {
    const int fv = fr - 4 * XA;
    const int dt = fv / (2 * XA), ks = fv % (2 * XA);
    const int d = dt * 32 + sig;
    unsigned int e[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int key = ks * 16 + 8 * g + q;
      e[q] = key < TL ? kv[((long long)b * TL + key) * ld + (long long)j * 2 * C + C + hh * 64 + d] : 0u;
    }
    v.x = e[0] | (e[1] << 16); v.y = e[2] | (e[3] << 16); v.z = e[4] | (e[5] << 16); v.w = e[6] | (e[7] << 16);
  }
  out[idx] = v;
}

int tune_cfg() {
  static const int v = [] { const char* e = tune_env("DF_WGEMM_CFG"); return e ? atoi(e) : 0; }();
  return v;
}

template <int TM, int TN, int KSPLIT, int PF, bool LN, int XA = 0>
int launch_one(const WParams& p, hipStream_t st) {
  const int MT = (p.M + 31) / 32, MG = (MT + TM - 1) / TM;
  const int NTo = p.N / 32;
  if (!p.geglu && NTo % TN) return DF_ESHAPE;
  constexpr int GP = TN >= 2 ? TN / 2 : 1;             // (value, gate) fragment pairs of a geglu tile
  if (p.geglu && (TN % 2 || NTo % GP)) return DF_ESHAPE;
  const int NG = p.geglu ? NTo / GP : NTo / TN;
  const int KF = p.K / 16;
  if (KF % KSPLIT) return DF_ESHAPE;
  constexpr int RP = (KSPLIT * TM * TN * 4 <= 128) ? TM : (TM % 2 == 0 && KSPLIT * (TM / 2) * TN * 4 <= 128) ? TM / 2 : 1;
  constexpr int smem = KSPLIT * RP * TN * 4 * 1024 + KSPLIT * TM * 32 * 2 * 4 + (XA > 0 ? 4096 : 0) + 4 * 128 * 4;
  auto k = wgemm_kernel<TM, TN, KSPLIT, PF, LN, XA>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess) return DF_EHIP;
    attr_set = true;
  }
  hipLaunchKernelGGL(k, dim3((unsigned)(MG * NG)), dim3(64 * KSPLIT), smem, st, p);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

// prefetch depth: the largest of PFMAX (5 or 10), 4, 2, 1 that divides the k-steps of a wave
template <int TM, int TN, int KSPLIT, int PFMAX>
int launch_cfg(const WParams& p, hipStream_t st) {
  const int KF = p.K / 16;
  if (KF % KSPLIT) return DF_ESHAPE;
  const int KFw = KF / KSPLIT;
  const bool ln = p.ln_s != nullptr;
#define DF_WG(PFV)                                                                     \
  return ln ? launch_one<TM, TN, KSPLIT, PFV, true>(p, st) : launch_one<TM, TN, KSPLIT, PFV, false>(p, st)
  if (KFw % PFMAX == 0) { DF_WG(PFMAX); }
  if (KFw % 4 == 0) { DF_WG(4); }
  if (KFw % 2 == 0) { DF_WG(2); }
  DF_WG(1);
#undef DF_WG
}

}  // namespace

#ifdef DF_TUNING
// Tuning build only: copies the stamps of the last wgemm_kernel launch to host memory (synchronises).
extern "C" __attribute__((visibility("default"))) int df_tune_wgemm_trace(long long* out, int n) {
  if (!out || n <= 0 || n > 1024 * 16) return DF_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return DF_EHIP;
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(g_wg_trace), (size_t)n * sizeof(long long)) != hipSuccess) return DF_EHIP;
  return DF_OK;
}
#endif

size_t packed_text_kv_bytes(int B, int TL, int count, int C) {
  const int XA = (TL + 31) / 32;
  return (size_t)B * count * (C / 64) * 12 * XA * 1024;
}

int launch_pack_text_kv(const bf16_t* kv, long long ld, bf16_t* out, int B, int TL, int count, int C, hipStream_t st) {
  if (B <= 0 || TL <= 0 || count <= 0 || C % 64 || ld % 8 || ((uintptr_t)kv % 16) || ((uintptr_t)out % 16)) return DF_ESHAPE;
  const int XA = (TL + 31) / 32;
  const long long total = (long long)B * count * (C / 64) * 12 * XA * 64;
  hipLaunchKernelGGL(pack_text_kv_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, kv, ld, (u32x4*)out, B, TL,
                     count, C, XA, total);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

size_t packed_rows_bytes(long long M, long long K) { return (size_t)((M + 31) / 32) * 32 * K * 2; }

int launch_pack_rows(const bf16_t* x, long long ldx, bf16_t* out, int M, int K, hipStream_t st) {
  if (M <= 0 || K <= 0 || K % 16 || ldx % 8 || ((uintptr_t)x % 16) || ((uintptr_t)out % 16)) return DF_ESHAPE;
  const long long total = (long long)((M + 31) / 32) * (K / 16) * 64;
  hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, x, ldx, (u32x4*)out, M, K,
                     total);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

int launch_pack_wfrag(const bf16_t* w, const float* gamma, bf16_t* out, int N, int K, hipStream_t st) {
  if (N <= 0 || K <= 0 || N % 32 || K % 16 || ((uintptr_t)w % 16) || ((uintptr_t)out % 16)) return DF_ESHAPE;
  const long long total = (long long)(N / 32) * (K / 16) * 64;
  hipLaunchKernelGGL(pack_wfrag_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w, gamma, (u32x4*)out, N,
                     K, total);
  DF_LAUNCH_CHECK();
  return DF_OK;
}

int launch_wgemm(const WGemmArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0 || a.K % 64) return DF_ESHAPE;
  const int Nout = a.geglu ? a.geglu : a.N;
  if (a.geglu && a.N != 2 * a.geglu) return DF_ESHAPE;
  if (Nout % 32) return DF_ESHAPE;
  if (!a.Xp || !a.Wp) return DF_EINVAL;
  if (a.ln_s && (!a.ln_t || a.bias)) return DF_EINVAL;
  auto al = [](const void* ptr, int b) { return ((uintptr_t)ptr % b) == 0; };
  if (!al(a.Xp, 16) || !al(a.Wp, 16) || !al(a.bias, 16) || !al(a.ln_s, 16) || !al(a.ln_t, 16) || !al(a.residual, 16) ||
      !al(a.out_f32, 16) || !al(a.out_packed, 16) || !al(a.out_rows, 16))
    return DF_EINVAL;
  if ((a.residual && a.ldr % 4) || (a.out_f32 && a.ldo % 4) || (a.out_rows && a.ld_rows % 8)) return DF_EINVAL;
  WParams p = {};
  p.Xp = (const bf16x8*)a.Xp; p.Wp = (const bf16x8*)a.Wp; p.M = a.M; p.N = Nout; p.K = a.K;
  p.bias = a.bias; p.ln_s = a.ln_s; p.ln_t = a.ln_t; p.ln_eps = a.ln_eps; p.residual = a.residual; p.ldr = a.ldr;
  p.out_f32 = a.out_f32; p.ldo = a.ldo; p.out_packed = (bf16_t*)a.out_packed; p.out_rows = (bf16_t*)a.out_rows;
  p.ld_rows = a.ld_rows; p.geglu = a.geglu ? 1 : 0;
  if (a.nseg > 0) {
    if (a.nseg > 3 || a.seg_w % 32 || a.seg_w * a.nseg != a.N || a.geglu) return DF_ESHAPE;
    p.nseg = a.nseg; p.seg_w = a.seg_w;
    for (int i = 0; i < a.nseg; ++i) {
      if (!a.seg_out[i] || a.seg_rows_in[i] <= 0 || (!a.seg_tr[i] && (a.seg_ld[i] % 8 || !al(a.seg_out[i], 16))))
        return DF_EINVAL;
      p.seg_tr[i] = a.seg_tr[i]; p.seg_pin[i] = a.seg_pin[i]; p.seg_pout[i] = a.seg_pout[i];
      p.seg_out[i] = (bf16_t*)a.seg_out[i]; p.seg_ld[i] = a.seg_ld[i]; p.seg_rows_out[i] = a.seg_rows_out[i];
      p.seg_row0[i] = a.seg_row0[i]; p.seg_rows_in[i] = a.seg_rows_in[i];
    }
  }
  if (a.xa_kv) {
    const int XA = (a.xa_keys + 31) / 32;
    if (a.geglu || a.nseg || !a.ln_s || !a.out_packed || a.N % 64 || XA < 1 || XA > 4 || a.xa_rows <= 0 ||
        (a.M != a.xa_rows && a.xa_rows % 32) || !al(a.xa_kv, 16))
      return DF_ESHAPE;
    p.xkv = (const bf16x8*)a.xa_kv; p.xa_keys = a.xa_keys; p.xa_rows = a.xa_rows; p.xa_scale = a.xa_scale;
    p.xa_bstride = a.xa_bstride / 8;
    const int KFw = a.K / 16 / 4;
#define DF_XA(PFV)                                                             \
  switch (XA) {                                                                \
    case 1: return launch_one<1, 2, 4, PFV, true, 1>(p, st);                   \
    case 2: return launch_one<1, 2, 4, PFV, true, 2>(p, st);                   \
    case 3: return launch_one<1, 2, 4, PFV, true, 3>(p, st);                   \
    default: return launch_one<1, 2, 4, PFV, true, 4>(p, st);                  \
  }
    if (KFw % 5 == 0) { DF_XA(5) }
    if (KFw % 4 == 0) { DF_XA(4) }
    if (KFw % 2 == 0) { DF_XA(2) }
    DF_XA(1)
#undef DF_XA
  }
  switch (tune_cfg()) {                                  // DF_WGEMM_CFG: tuning aid
    case 1: return launch_cfg<1, 2, 4, 5>(p, st);
    case 2: return launch_cfg<2, 2, 4, 5>(p, st);
    case 3: return launch_cfg<1, 2, 4, 10>(p, st);
    case 5: return launch_cfg<1, 2, 8, 5>(p, st);
    case 6: return launch_cfg<2, 3, 4, 5>(p, st);
    case 9: return launch_cfg<4, 4, 4, 2>(p, st);
    default: break;
  }
  const int nfrag = Nout / 32;
  if (!p.geglu && nfrag % 2) return launch_cfg<1, 1, 4, 5>(p, st);
  // Measured on the patch step (kernel trace, cold weights).  A compute unit feeds its waves about one 1 KB operand
  // fragment per 32 cycles, whatever the L2 hit rate, so a kernel's K loop lasts (fragment loads of the busiest unit)
  // x 32 cycles, and every workgroup adds a fixed ramp and epilogue.  A wave tile of 32 tokens x 64 features keeps
  // the most waves in flight and wins while the problem has few tiles; from ~320 workgroups on, the 64 x 64 tile's
  // lower operand traffic per flop wins; and where a still larger tile (128 x 128 for the GEGLU projection, 64 x 96
  // otherwise) covers the output with at most one workgroup per unit, its traffic per flop and its single round of
  // workgroups win again, provided the reduction is long enough to amortise the row-by-row epilogue.
  const int MT = (a.M + 31) / 32;
  const long long wg12 = (long long)MT * (p.geglu ? nfrag : nfrag / 2);
  const bool long_k = a.K / 16 / 4 >= 16;
  if (wg12 >= 320 && long_k) {
    if (p.geglu && nfrag % 2 == 0 && (long long)((MT + 3) / 4) * (nfrag / 2) <= 256) return launch_cfg<4, 4, 4, 2>(p, st);
    if (!p.geglu && nfrag % 3 == 0 && (long long)((MT + 1) / 2) * (nfrag / 3) <= 256) return launch_cfg<2, 3, 4, 5>(p, st);
  }
  if (wg12 >= 320) return launch_cfg<2, 2, 4, 5>(p, st);
  return launch_cfg<1, 2, 4, 5>(p, st);
}

}  // namespace df
