// Displaced self-attention (Section 4, Sparse operations): fresh queries of one
// patch against keys/values of the whole feature map, where the patch's own
// rows are read from the fresh tensors and every other row from the stale
// buffers.  The splice happens in the tile loader; no scattered copy exists.
//
// bf16 kernel (head dim 64): flash-style, one workgroup = 4 waves x 32 queries,
// 64-key K/V tiles staged through LDS and shared by the 4 waves.  Each wave
// computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16 so that a lane owns one
// query column: the online-softmax row statistics are lane-local plus one
// exchange with lane^32.  The rows of the K tile are assigned to MFMA rows in
// a permuted order chosen so that the exponentiated accumulators are, without
// any data movement, the B operand (P^T) of O^T = V^T P^T, and the matching
// V^T operand is one 16-byte read from a transposed, XOR-swizzled V tile.
// Small query counts are spread over the chip by splitting the key range
// across workgroups; partial (O, m, l) are merged by a second kernel.
//
// f32 kernel: one wave per query, lanes stride over keys; for the small
// full-precision configuration only.
#include <cstdlib>
#include <type_traits>

#include "kernels.h"

namespace df {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

struct AttnParams {
  const void* q; const void* kf; const void* vf; const void* ks; const void* vs;
  void* out;
  float* part_o;   // [nsplit][B][heads][Lq][d] float (split mode)
  float* part_ml;  // [nsplit][B][heads][Lq][2]
  int B, Lq, L, heads;
  int own_lo, own_n;
  int own_period;  // 0: keys [own_lo, own_lo + own_n) are fresh; P > 0: key j is fresh iff j % P lies in that range
                   // (a vertical strip of a token grid with P columns) and is row (j / P) * own_n + j % P - own_lo
  long long ldq, ldkf, ldvf, ldks, ldvs, ldo;
  long long bsq, bskf, bsvf, bsks, bsvs, bso;
  float scale;
  int nsplit, keys_per_split;
  int out_packed;
  // transposed-V variant: vs is V^T [B][heads*64][vt_ld] (keys contiguous), every key comes from ks / vs
  long long vt_ld;
};

// Row of the fresh tensor that holds key j, or -1 if the key comes from the stale buffer (Section 4: the keys and
// values are the scatter output; the scatter is resolved here, key by key).
__device__ __forceinline__ long long fresh_row(int own_lo, int own_n, int period, int j) {
  if (period > 0) {
    const int r = j / period, rel = j - r * period - own_lo;
    return (rel >= 0 && rel < own_n) ? (long long)r * own_n + rel : -1;
  }
  const int rel = j - own_lo;
  return (rel >= 0 && rel < own_n) ? (long long)rel : -1;
}

__device__ __forceinline__ const bf16_t* key_row(const bf16_t* fresh, const bf16_t* stale, long long ldf, long long lds,
                                                 int own_lo, int own_n, int period, int j) {
  const long long fr = fresh_row(own_lo, own_n, period, j);
  return fr >= 0 ? fresh + fr * ldf : stale + (long long)j * lds;
}

// physical key (0..31) loaded into MFMA row rho of a 32-key block
__device__ __forceinline__ int key_of_mfma_row(int rho) {
  const int j = rho >> 3, g = (rho >> 2) & 1, r = rho & 3;
  return 16 * (j >> 1) + 8 * g + 4 * (j & 1) + r;
}

// PERIODIC: the fresh keys are a vertical strip of the token grid (own_period > 0); a separate instantiation, so that
// the contiguous split keeps its tile-level fast paths and carries none of the per-key index arithmetic.
template <bool PERIODIC>
__global__ __launch_bounds__(256, 2) void attn_bf16_d64(AttnParams p) {
  const int period = PERIODIC ? p.own_period : 0;
  constexpr int D = 64, TK = 64;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[2][TK * D];   // [key][d], 16-byte chunks XOR-swizzled by row
  __shared__ __attribute__((aligned(16))) bf16_t Vt[2][D * TK];   // [d][key], swizzled

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the query rows, hence the key ranges and the
                                                               // ragged-tile test, stay off the vector ALU
  const int g = lane >> 5, c = lane & 31;
  const int xor32 = (lane ^ 32) << 2;                          // byte index of the partner lane for ds_bpermute
  const int csig = (c & 0x13) | ((c & 4) << 1) | ((c & 8) >> 1);   // c with bits 2 and 3 swapped
  // 1-D grid; workgroups go round-robin over the 8 XCDs, so XCD x takes the x-th contiguous chunk of the
  // (query block fastest, head, batch*split) order: the query blocks that read the same K/V range share an L2
  int t = blockIdx.x;
  {
    const int nwg = gridDim.x;
    const int xcd = t & 7, loc = t >> 3;
    const int base = nwg >> 3, rem = nwg & 7;
    t = xcd * base + (xcd < rem ? xcd : rem) + loc;
  }
  const int nqb = (p.Lq + 127) / 128;
  const int qb = t % nqb;
  const int h = (t / nqb) % p.heads;
  const int zz = t / (nqb * p.heads);
  const int b = zz / p.nsplit, split = zz % p.nsplit;
  const int q0 = qb * 128 + wave * 32;
  const int kv_lo = split * p.keys_per_split;
  int kv_hi = kv_lo + p.keys_per_split;
  if (kv_hi > p.L) kv_hi = p.L;
  const int ntiles = (kv_hi - kv_lo + TK - 1) / TK;

  const bf16_t* kf = (const bf16_t*)p.kf + (long long)b * p.bskf + h * D;
  const bf16_t* vf = (const bf16_t*)p.vf + (long long)b * p.bsvf + h * D;
  const bf16_t* ks = p.ks ? (const bf16_t*)p.ks + (long long)b * p.bsks + h * D : nullptr;
  const bf16_t* vs = p.vs ? (const bf16_t*)p.vs + (long long)b * p.bsvs + h * D : nullptr;

  // Q^T operand: lane (g, c) holds Q[q0 + c][16*ks + 8*g .. +7] for ks = 0..3
  bf16x8 qreg[4];
  {
    const int qi = q0 + c;
    const bf16_t* qp = (const bf16_t*)p.q + (long long)b * p.bsq + (long long)qi * p.ldq + h * D;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4 t = {0u, 0u, 0u, 0u};
      if (qi < p.Lq) t = *reinterpret_cast<const u32x4*>(qp + 16 * s + 8 * g);
      qreg[s] = __builtin_bit_cast(bf16x8, t);
    }
  }

  // cooperative tile loads: K: lane -> (key = tid/8 (+32), chunk = tid%8); V: keys 2*kap, 2*kap+1, chunk = tid%8
  const int ld_key = tid >> 3, ld_ch = tid & 7;
  // The K/V rows come from HBM or the Infinity Cache with microseconds of latency and a tile's compute is a fraction
  // of that, so three tiles of loads are kept in flight in a register ring (slot = tile % 3, loop unrolled by 3).
  constexpr int PF = 3;
  u32x4 kreg[PF][2], vreg[PF][2];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  // a lane's row offsets inside a tile (32-bit: the launcher bounds the pitches); a tile that lies wholly in the
  // stale buffer or wholly in the fresh rows only adds a scalar base (the generic path below redoes a select and a
  // 64-bit multiply per row and tile)
  unsigned int kof_s[2], vof_s[2], kof_f[2], vof_f[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    kof_s[i] = (unsigned int)(ld_key + 32 * i) * (unsigned int)p.ldks + ld_ch * 8;
    vof_s[i] = (unsigned int)(2 * ld_key + i) * (unsigned int)p.ldvs + ld_ch * 8;
    kof_f[i] = (unsigned int)(ld_key + 32 * i) * (unsigned int)p.ldkf + ld_ch * 8;
    vof_f[i] = (unsigned int)(2 * ld_key + i) * (unsigned int)p.ldvf + ld_ch * 8;
  }
  auto load_tile = [&](int t, auto slot) {
    constexpr int S = decltype(slot)::value;
    const int base = kv_lo + t * TK;
    if (!PERIODIC && base + TK <= kv_hi) {         // (uniform) a full tile of a contiguous split
      const int rel = base - p.own_lo;
      if (rel >= 0 && rel + TK <= p.own_n) {               // all rows fresh
        const bf16_t* kb = kf + (long long)rel * p.ldkf;
        const bf16_t* vb = vf + (long long)rel * p.ldvf;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          kreg[S][i] = *reinterpret_cast<const u32x4*>(kb + kof_f[i]);
          vreg[S][i] = *reinterpret_cast<const u32x4*>(vb + vof_f[i]);
        }
        return;
      }
      if (rel + TK <= 0 || rel >= p.own_n) {               // all rows stale
        const bf16_t* kb = ks + (long long)base * p.ldks;
        const bf16_t* vb = vs + (long long)base * p.ldvs;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          kreg[S][i] = *reinterpret_cast<const u32x4*>(kb + kof_s[i]);
          vreg[S][i] = *reinterpret_cast<const u32x4*>(vb + vof_s[i]);
        }
        return;
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int jk = base + ld_key + 32 * i;
      kreg[S][i] = jk < kv_hi ? *reinterpret_cast<const u32x4*>(key_row(kf, ks, p.ldkf, p.ldks, p.own_lo, p.own_n, period, jk) + ld_ch * 8)
                              : zero4;
      const int jv = base + 2 * ld_key + i;
      vreg[S][i] = jv < kv_hi ? *reinterpret_cast<const u32x4*>(key_row(vf, vs, p.ldvf, p.ldvs, p.own_lo, p.own_n, period, jv) + ld_ch * 8)
                              : zero4;
    }
  };
  auto store_tile = [&](int buf, auto slot) {
    constexpr int S = decltype(slot)::value;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = ld_key + 32 * i;
      const int f = (row & 3) | (((row >> 3) & 1) << 2);
      *reinterpret_cast<u32x4*>(&Ks[buf][row * D + ((ld_ch ^ f) * 8)]) = kreg[S][i];
    }
    // V transposed: dword (keys 2*kap, 2*kap+1) of row d goes to chunk (kap/4) ^ (d%8) ^ (d/8), dword kap%4
    const int kap = ld_key;
    unsigned int* vt = reinterpret_cast<unsigned int*>(&Vt[buf][0]);
    const unsigned int a[4] = {vreg[S][0].x, vreg[S][0].y, vreg[S][0].z, vreg[S][0].w};
    const unsigned int bq[4] = {vreg[S][1].x, vreg[S][1].y, vreg[S][1].z, vreg[S][1].w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int d = ld_ch * 8 + e;
      const unsigned int lo = (e & 1) ? (a[e >> 1] >> 16) : (a[e >> 1] & 0xffffu);
      const unsigned int hi = (e & 1) ? (bq[e >> 1] & 0xffff0000u) : (bq[e >> 1] << 16);
      const int chunk = (kap >> 2) ^ (d & 7) ^ (d >> 3);
      vt[d * 32 + chunk * 4 + (kap & 3)] = lo | hi;
    }
  };

  f32x16 o_acc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o_acc[i][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = p.scale * kLog2e;

  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  if (ntiles > 0) load_tile(0, I0{});
  if (ntiles > 1) load_tile(1, I1{});
  if (ntiles > 2) load_tile(2, I2{});
  // one tile: ring slot -> LDS buffer t&1, barrier, refill the slot with tile t+3, compute from LDS.  A buffer is
  // rewritten two tiles later, after the barrier of the tile in between, which every wave reaches only after it has
  // finished reading it.
  auto do_tile = [&](int t, auto slot) {
    const int buf = t & 1;
    store_tile(buf, slot);
    __syncthreads();
    if (t + PF < ntiles) load_tile(t + PF, slot);
    // ---- S^T = K Q^T for two 32-key blocks ----
    f32x16 s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) s_acc[kb][e] = 0.f;
      const int row = 32 * kb + key_of_mfma_row(c);
      const int f = (row & 3) | (((row >> 3) & 1) << 2);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bf16x8 kfrag = *reinterpret_cast<const bf16x8*>(&Ks[buf][row * D + (((2 * s + g) ^ f) * 8)]);
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag, qreg[s], s_acc[kb], 0, 0, 0);
      }
    }
    // accumulator e = 4*j + r of block kb is key  base + 32*kb + 16*(j/2) + 8*g + 4*(j%2) + r  for query c
    const int tile_base = kv_lo + t * TK;
    float mx = -INFINITY;
    if (tile_base + TK > kv_hi) {   // ragged last tile: keys beyond the range get no weight
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = e >> 2, r = e & 3;
          const int key = tile_base + 32 * kb + 16 * (j >> 1) + 8 * g + 4 * (j & 1) + r;
          if (key >= kv_hi) s_acc[kb][e] = -INFINITY;
        }
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s_acc[kb][e]);
    mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_ds_bpermute(xor32, __float_as_int(mx)))) * sc;   // scale > 0
    const float m_new = fmaxf(m_run, mx);           // finite: every tile holds at least one valid key
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // exp2(-inf) = 0 on the first tile
    float rs = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][e], sc, -m_new));   // raw v_exp_f32: arguments are <= 0
        s_acc[kb][e] = pv;
        rs += pv;
      }
    rs += __int_as_float(__builtin_amdgcn_ds_bpermute(xor32, __float_as_int(rs)));
    l_run = l_run * alpha + rs;
    m_run = m_new;
    // the running maximum rarely moves after the first tiles: rescale only when some query of the wave needs it
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o_acc[i][e] *= alpha;
    }

    // ---- O^T += V^T P^T : four 16-key steps; lane supplies P for its query and key slots 8g..8g+7 ----
#pragma unroll
    for (int ts = 0; ts < 4; ++ts) {
      const int kb = ts >> 1, half = ts & 1;
      u32x4 pk;
      pk.x = pack_bf2(s_acc[kb][8 * half + 0], s_acc[kb][8 * half + 1]);
      pk.y = pack_bf2(s_acc[kb][8 * half + 2], s_acc[kb][8 * half + 3]);
      pk.z = pack_bf2(s_acc[kb][8 * half + 4], s_acc[kb][8 * half + 5]);
      pk.w = pack_bf2(s_acc[kb][8 * half + 6], s_acc[kb][8 * half + 7]);
      const bf16x8 pfrag = __builtin_bit_cast(bf16x8, pk);
      const int kchunk = 4 * kb + 2 * half + g;     // keys 32*kb + 16*half + 8*g .. +7
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        const int d = 32 * db + csig;                 // MFMA row c computes feature row sigma(c) (see the write below)
        const int chunk = kchunk ^ (d & 7) ^ (d >> 3);
        const bf16x8 vfrag = *reinterpret_cast<const bf16x8*>(&Vt[buf][d * TK + chunk * 8]);
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfrag, pfrag, o_acc[db], 0, 0, 0);
      }
    }
  };
  for (int t = 0; t < ntiles; t += PF) {
    do_tile(t, I0{});
    if (t + 1 < ntiles) do_tile(t + 1, I1{});
    if (t + 2 < ntiles) do_tile(t + 2, I2{});
  }

  // ---- write: V^T rows were taken in the order sigma (bits 2 and 3 of the row index swapped), so accumulator
  // elements 8f .. 8f+7 of lane (g, c) are O[q0 + c][32*db + 16*f + 8*g .. +7]: eight consecutive features ----
  const int qi = q0 + c;
  if (qi >= p.Lq) return;
  if (p.nsplit == 1) {
    const float inv = 1.0f / l_run;
    bf16_t* op = (bf16_t*)p.out + (long long)b * p.bso + (long long)qi * p.ldo + h * D;
    const long long m = (long long)b * p.Lq + qi;     // token row of the packed operand
    bf16_t* pp = (bf16_t*)p.out + (((m >> 5) * (long long)(p.heads * D / 16) + h * (D / 16)) * 64 + (m & 31) + 32 * g) * 8;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        u32x4 t;
        t.x = pack_bf2(o_acc[db][8 * f + 0] * inv, o_acc[db][8 * f + 1] * inv);
        t.y = pack_bf2(o_acc[db][8 * f + 2] * inv, o_acc[db][8 * f + 3] * inv);
        t.z = pack_bf2(o_acc[db][8 * f + 4] * inv, o_acc[db][8 * f + 5] * inv);
        t.w = pack_bf2(o_acc[db][8 * f + 6] * inv, o_acc[db][8 * f + 7] * inv);
        if (p.out_packed) *reinterpret_cast<u32x4*>(pp + (2 * db + f) * 512) = t;
        else *reinterpret_cast<u32x4*>(op + 32 * db + 16 * f + 8 * g) = t;
      }
  } else {
    const long long row = (((long long)split * p.B + b) * p.heads + h) * p.Lq + qi;
    float* po = p.part_o + row * D;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        f32x4 t0 = {o_acc[db][8 * f], o_acc[db][8 * f + 1], o_acc[db][8 * f + 2], o_acc[db][8 * f + 3]};
        f32x4 t1 = {o_acc[db][8 * f + 4], o_acc[db][8 * f + 5], o_acc[db][8 * f + 6], o_acc[db][8 * f + 7]};
        *reinterpret_cast<f32x4*>(po + 32 * db + 16 * f + 8 * g) = t0;
        *reinterpret_cast<f32x4*>(po + 32 * db + 16 * f + 8 * g + 4) = t1;
      }
    if (g == 0) {
      p.part_ml[row * 2] = m_run;      // in log2 units
      p.part_ml[row * 2 + 1] = l_run;
    }
  }
}

// ---- variant for the UNet step: every key row comes from the (already refreshed) stale buffers, V is stored
// transposed ([feature][key], written that way by the projection), so K and V^T tiles go global -> LDS with direct
// loads (no registers, no transposing stores) through a 3-stage ring awaited with an explicit vmcnt.  The swizzles
// of the LDS tiles are applied on the source side: LDS slot s of row r receives global chunk s ^ key(r). ----
#ifdef DF_TUNING
// Tuning build only: per workgroup (waves 0 and 5; wave 5's rows follow at +256), 32 stamps: the constant-rate clock at entry and exit, cycle stamps between.
__device__ long long g_attn_trace[512 * 32];
#define DF_ATRACE(slot, expr)                                                                             \
  do {                                                                                                    \
    const unsigned wg_ = blockIdx.x + gridDim.x * blockIdx.y;                                            \
    if ((threadIdx.x == 0 || threadIdx.x == 320) && wg_ < 256 && (slot) < 32)                             \
      g_attn_trace[(wg_ + (threadIdx.x ? 256 : 0)) * 32 + (slot)] = (long long)(expr);                    \
  } while (0)
#else
#define DF_ATRACE(slot, expr) do {} while (0)
#endif

#define DF_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define DF_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// NGR = 2: eight waves in two groups of four.  Both groups hold the same 128 queries; of every 128 consecutive keys
// group 0 takes the first 64 and group 1 the last 64, and the two running (max, sum, O) states are merged through LDS
// at the end.  A SIMD then always has two waves in different phases of their tile, so one wave's softmax (vector ALU)
// runs under the other's matrix instructions and LDS waits, which a single wave per SIMD leaves exposed.
template <int NST, int NGR>
__global__ __launch_bounds__(256 * NGR, NGR == 1 ? 2 : 1) void attn_vt_d64(AttnParams p) {
  constexpr int D = 64, TK = 64;
  constexpr int KB = TK * D * 2, STAGE = 2 * KB * NGR;     // bytes: K tiles of all groups, then their V^T tiles
  extern __shared__ __attribute__((aligned(16))) char smem[];
  DF_ATRACE(0, wall_clock64());
  DF_ATRACE(1, __builtin_readcyclecounter());
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: what depends on it (key range, masks of the
                                                               // ragged tile, LDS addresses) stays off the vector ALU
  const int grp = wave >> 2, wq = wave & 3;
  const int xor32 = (lane ^ 32) << 2;                          // byte index of the partner lane for ds_bpermute
  const int g = lane >> 5, c = lane & 31;
  const int csig = (c & 0x13) | ((c & 4) << 1) | ((c & 8) >> 1);
  int t = blockIdx.x;
  {
    const int nwg = gridDim.x;
    const int xcd = t & 7, loc = t >> 3;
    const int base = nwg >> 3, rem = nwg & 7;
    t = xcd * base + (xcd < rem ? xcd : rem) + loc;
  }
  const int nqb = (p.Lq + 127) / 128;
  const int qb = t % nqb;
  const int h = (t / nqb) % p.heads;
  const int zz = t / (nqb * p.heads);
  const int b = zz / p.nsplit, split = zz % p.nsplit;
  const int q0 = qb * 128 + wq * 32;
  const int kv_lo = split * p.keys_per_split;              // multiple of 64
  int kv_hi = kv_lo + p.keys_per_split;
  if (kv_hi > p.L) kv_hi = p.L;
  const int ntiles = (kv_hi - kv_lo + TK * NGR - 1) / (TK * NGR);   // iterations: one 64-key tile per group each

  const bf16_t* kg = (const bf16_t*)p.ks + (long long)b * p.bsks + h * D;
  const bf16_t* vg = (const bf16_t*)p.vs + (long long)b * p.bsvs + (long long)h * D * p.vt_ld;

  bf16x8 qreg[4];
  {
    const int qi = q0 + c;
    const bf16_t* qp = (const bf16_t*)p.q + (long long)b * p.bsq + (long long)qi * p.ldq + h * D;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4 tq = {0u, 0u, 0u, 0u};
      if (qi < p.Lq) tq = *reinterpret_cast<const u32x4*>(qp + 16 * s + 8 * g);
      qreg[s] = __builtin_bit_cast(bf16x8, tq);
    }
  }

  // direct loads: instruction j of a wave covers tile rows (2*wave + j)*8 + lane/8, 16-byte slot lane%8.  A lane's
  // offsets inside a tile never change (32-bit, the launcher bounds the pitches); a tile adds a scalar base.
  const int lr = lane >> 3, slot = lane & 7;
  unsigned int kofs[2], vofs[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = (2 * wave + j) * 8 + lr;               // key within the iteration's K tiles
    const int f = (row >> 1) & 7;                          // swizzle key: conflict-free 16-byte reads on 64 banks
    kofs[j] = (unsigned int)row * (unsigned int)p.ldks + (unsigned int)((slot ^ f) * 8);
    const int d = ((2 * wave + j) & 7) * 8 + lr;           // feature row of the V^T tile (waves 4-7: second group's tile)
    const int ch = slot ^ (d & 7) ^ (d >> 3);              // 8-key chunk; the buffer is padded to whole tiles
    vofs[j] = (unsigned int)d * (unsigned int)p.vt_ld + (unsigned int)(ch * 8);
  }
  auto issue = [&](int tl, int stage) {
    if (tl > ntiles - 1) tl = ntiles - 1;                  // past the end: re-read the last tile (keeps vmcnt uniform)
    const int key0 = kv_lo + tl * TK * NGR;
    char* sk = smem + stage * STAGE;
    char* sv = sk + KB * NGR;
    if (key0 + TK * NGR <= p.L) {                          // (uniform) every key row of the iteration exists
      const bf16_t* kb = kg + (long long)key0 * p.ldks;
#pragma unroll
      for (int j = 0; j < 2; ++j)
        __builtin_amdgcn_global_load_lds(DF_GPTR(kb + kofs[j]), DF_LPTR(sk + (2 * wave + j) * 1024), 16, 0, 0);
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row = (2 * wave + j) * 8 + lr;
        int key = key0 + row;
        if (key > p.L - 1) key = p.L - 1;                  // rows beyond the last key are masked below
        const int f = (row >> 1) & 7;
        __builtin_amdgcn_global_load_lds(DF_GPTR(kg + (long long)key * p.ldks + ((slot ^ f) * 8)),
                                         DF_LPTR(sk + (2 * wave + j) * 1024), 16, 0, 0);
      }
    }
    long long vkey0 = key0 + TK * grp;
    if (vkey0 > p.vt_ld - TK) vkey0 = p.vt_ld - TK;        // a tile wholly beyond the padded buffer: masked below
    const bf16_t* vb = vg + vkey0;
#pragma unroll
    for (int j = 0; j < 2; ++j)
      __builtin_amdgcn_global_load_lds(DF_GPTR(vb + vofs[j]), DF_LPTR(sv + (2 * wave + j) * 1024), 16, 0, 0);
  };

  f32x16 o_acc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o_acc[i][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = p.scale * kLog2e;

#pragma unroll
  for (int i = 0; i < NST - 1; ++i) issue(i, i);
  DF_ATRACE(2, __builtin_readcyclecounter());
  int stage = 0, nstage = NST - 1;
  for (int tl = 0; tl < ntiles; ++tl) {
    if (tl < 8) DF_ATRACE(3 + 3 * tl, __builtin_readcyclecounter());
    // tile tl has landed once at most the loads of the NST-2 younger tiles (4 each) are outstanding
    {
      constexpr int VM = 4 * (NST - 2);
      __builtin_amdgcn_s_waitcnt((VM & 0xF) | ((VM >> 4) << 14) | (0x7 << 4) | (0 << 8));   // vmcnt(VM) lgkmcnt(0)
    }
    asm volatile("" ::: "memory");
    if (tl < 8) DF_ATRACE(4 + 3 * tl, __builtin_readcyclecounter());
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (tl < 8) DF_ATRACE(5 + 3 * tl, __builtin_readcyclecounter());
    issue(tl + NST - 1, nstage);                           // the stage every wave finished reading before the barrier
    const bf16_t* Ks = reinterpret_cast<const bf16_t*>(smem + stage * STAGE + grp * KB);
    const bf16_t* Vt = reinterpret_cast<const bf16_t*>(smem + stage * STAGE + KB * NGR + grp * KB);
    const int tile_base = kv_lo + tl * TK * NGR + grp * TK;
    // The tile's work in two copies: full tiles carry no mask code at all (written as one body with a run-time flag,
    // the compiler evaluates the masks' comparisons ahead of the branch in every tile: a third of the loop's vector
    // instructions).
    auto tile = [&](auto raggedc) {
    constexpr bool ragged = decltype(raggedc)::value;
    // All LDS fragment reads of a phase are issued before its MFMAs (one read per MFMA would put an LDS round trip
    // between every pair of matrix instructions), and the V^T fragments are requested before the softmax so that
    // they arrive while the vector ALU works.
    bf16x8 kfr[2][4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int row = 32 * kb + key_of_mfma_row(c);
      const int f = (row >> 1) & 7;
#pragma unroll
      for (int s = 0; s < 4; ++s) kfr[kb][s] = *reinterpret_cast<const bf16x8*>(&Ks[row * D + (((2 * s + g) ^ f) * 8)]);
    }
    __builtin_amdgcn_sched_barrier(0);
    f32x16 s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) s_acc[kb][e] = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[kb][s], qreg[s], s_acc[kb], 0, 0, 0);
    u32x4 vfr[4][2];
#pragma unroll
    for (int ts = 0; ts < 4; ++ts) {
      const int kchunk = 4 * (ts >> 1) + 2 * (ts & 1) + g;
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        const int d = 32 * db + csig;
        vfr[ts][db] = *reinterpret_cast<const u32x4*>(&Vt[d * TK + (kchunk ^ (d & 7) ^ (d >> 3)) * 8]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (ragged) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = e >> 2, r = e & 3;
          const int key = tile_base + 32 * kb + 16 * (j >> 1) + 8 * g + 4 * (j & 1) + r;
          if (key >= kv_hi) s_acc[kb][e] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s_acc[kb][e]);
    mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_ds_bpermute(xor32, __float_as_int(mx)))) * sc;
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float rs = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][e], sc, -m_new));
        s_acc[kb][e] = pv;
        rs += pv;
      }
    rs += __int_as_float(__builtin_amdgcn_ds_bpermute(xor32, __float_as_int(rs)));
    l_run = l_run * alpha + rs;
    m_run = m_new;
    // the running maximum rarely moves after the first tiles: rescale only when some query of the wave needs it
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o_acc[i][e] *= alpha;
    }
#pragma unroll
    for (int ts = 0; ts < 4; ++ts) {
      const int kb = ts >> 1, half = ts & 1;
      u32x4 pk;
      pk.x = pack_bf2(s_acc[kb][8 * half + 0], s_acc[kb][8 * half + 1]);
      pk.y = pack_bf2(s_acc[kb][8 * half + 2], s_acc[kb][8 * half + 3]);
      pk.z = pack_bf2(s_acc[kb][8 * half + 4], s_acc[kb][8 * half + 5]);
      pk.w = pack_bf2(s_acc[kb][8 * half + 6], s_acc[kb][8 * half + 7]);
      const bf16x8 pfrag = __builtin_bit_cast(bf16x8, pk);
      const int kchunk = 4 * kb + 2 * half + g;            // keys 32*kb + 16*half + 8*g .. +7
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        u32x4 vraw = vfr[ts][db];
        if constexpr (ragged) {                            // keys beyond the range: P is 0, V must be finite
          const int key = tile_base + kchunk * 8;
          if (key + 0 >= kv_hi) vraw.x = 0u; else if (key + 1 >= kv_hi) vraw.x &= 0xffffu;
          if (key + 2 >= kv_hi) vraw.y = 0u; else if (key + 3 >= kv_hi) vraw.y &= 0xffffu;
          if (key + 4 >= kv_hi) vraw.z = 0u; else if (key + 5 >= kv_hi) vraw.z &= 0xffffu;
          if (key + 6 >= kv_hi) vraw.w = 0u; else if (key + 7 >= kv_hi) vraw.w &= 0xffffu;
        }
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vraw), pfrag, o_acc[db], 0, 0, 0);
      }
    }
    };
    if (tile_base + TK <= kv_hi) tile(std::false_type{});          // (wave-uniform branches)
    else if (tile_base < kv_hi) tile(std::true_type{});            // the last iteration may hold one tile only
    stage = (stage + 1 == NST) ? 0 : stage + 1;
    nstage = (nstage + 1 == NST) ? 0 : nstage + 1;
  }
  __builtin_amdgcn_s_waitcnt((0 & 0xF) | (0x7 << 4) | (0 << 8));     // drain the clamped tail loads
  DF_ATRACE(28, __builtin_readcyclecounter());
  DF_ATRACE(31, ntiles);

  if constexpr (NGR == 2) {
    // group 1 hands its state to group 0 (the ring is free once every wave has drained its loads)
    __syncthreads();
    float* mrg = reinterpret_cast<float*>(smem);           // [4 waves][34][64]: 32 accumulators, max, sum per lane
    if (grp == 1) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) mrg[(wq * 34 + i * 16 + e) * 64 + lane] = o_acc[i][e];
      mrg[(wq * 34 + 32) * 64 + lane] = m_run;
      mrg[(wq * 34 + 33) * 64 + lane] = l_run;
    }
    __syncthreads();
    if (grp == 1) return;
    const float m1 = mrg[(wq * 34 + 32) * 64 + lane], l1 = mrg[(wq * 34 + 33) * 64 + lane];
    const float m_new = fmaxf(m_run, m1);                  // group 0 always holds at least one key: finite
    const float a0 = __builtin_amdgcn_exp2f(m_run - m_new), a1 = __builtin_amdgcn_exp2f(m1 - m_new);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) o_acc[i][e] = o_acc[i][e] * a0 + mrg[(wq * 34 + i * 16 + e) * 64 + lane] * a1;
    l_run = l_run * a0 + l1 * a1;
    m_run = m_new;
  }

  DF_ATRACE(29, __builtin_readcyclecounter());
  DF_ATRACE(30, wall_clock64());
  const int qi = q0 + c;
  if (qi >= p.Lq) return;
  if (p.nsplit == 1) {
    const float inv = 1.0f / l_run;
    bf16_t* op = (bf16_t*)p.out + (long long)b * p.bso + (long long)qi * p.ldo + h * D;
    const long long m = (long long)b * p.Lq + qi;
    bf16_t* pp = (bf16_t*)p.out + (((m >> 5) * (long long)(p.heads * D / 16) + h * (D / 16)) * 64 + (m & 31) + 32 * g) * 8;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        u32x4 tq;
        tq.x = pack_bf2(o_acc[db][8 * f + 0] * inv, o_acc[db][8 * f + 1] * inv);
        tq.y = pack_bf2(o_acc[db][8 * f + 2] * inv, o_acc[db][8 * f + 3] * inv);
        tq.z = pack_bf2(o_acc[db][8 * f + 4] * inv, o_acc[db][8 * f + 5] * inv);
        tq.w = pack_bf2(o_acc[db][8 * f + 6] * inv, o_acc[db][8 * f + 7] * inv);
        if (p.out_packed) *reinterpret_cast<u32x4*>(pp + (2 * db + f) * 512) = tq;
        else *reinterpret_cast<u32x4*>(op + 32 * db + 16 * f + 8 * g) = tq;
      }
  } else {
    const long long row = (((long long)split * p.B + b) * p.heads + h) * p.Lq + qi;
    float* po = p.part_o + row * D;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        f32x4 t0 = {o_acc[db][8 * f], o_acc[db][8 * f + 1], o_acc[db][8 * f + 2], o_acc[db][8 * f + 3]};
        f32x4 t1 = {o_acc[db][8 * f + 4], o_acc[db][8 * f + 5], o_acc[db][8 * f + 6], o_acc[db][8 * f + 7]};
        *reinterpret_cast<f32x4*>(po + 32 * db + 16 * f + 8 * g) = t0;
        *reinterpret_cast<f32x4*>(po + 32 * db + 16 * f + 8 * g + 4) = t1;
      }
    if (g == 0) {
      p.part_ml[row * 2] = m_run;
      p.part_ml[row * 2 + 1] = l_run;
    }
  }
}

// Self-attention of a patch with few queries (the deepest level: 300-1024 query rows against the whole image's keys).
// One workgroup = one 32-query block of one head; its NW waves take contiguous runs of 64-key tiles and merge their
// (max, sum, O) states through LDS at the end, so nothing is split across workgroups and no second kernel runs.
// Nothing is shared between waves inside the loop: every wave stages its own K and V^T tiles (global -> LDS with
// direct loads, 1 KB contiguous per instruction; a wave reading its MFMA operands straight from the row-major buffers
// touches 32 cache lines per instruction and ran at a quarter of the rate) in a private 16 KB of LDS, so the loop has no
// barrier: a tile's fragments go LDS -> registers, then the next tile's loads are issued into the same LDS while the
// tile computes.  Same operand conventions and swizzles as attn_vt_d64.
template <int NW>
__global__ __launch_bounds__(64 * NW) void attn_wave_d64(AttnParams p) {
  constexpr int D = 64, TK = 64;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  DF_ATRACE(0, wall_clock64());
  DF_ATRACE(1, __builtin_readcyclecounter());
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int xor32 = (lane ^ 32) << 2;
  const int g = lane >> 5, c = lane & 31;
  const int csig = (c & 0x13) | ((c & 4) << 1) | ((c & 8) >> 1);
  // Grid (heads rounded up to a multiple of 8, query blocks, batch): workgroups go round-robin over the 8 XCDs in
  // x-fastest order, so every query block of head h runs on XCD h % 8 and the blocks of a head, which read the same
  // K / V^T, share an L2 - without any index arithmetic (the divisions of a linear index were a tenth of this kernel).
  const int h = blockIdx.x, qb = blockIdx.y, b = blockIdx.z;
  if (h >= p.heads) return;
  const int q0 = qb * 32;
  const int NT = (p.L + TK - 1) / TK;
  const int t_lo = (int)((long long)wave * NT / NW), t_hi = (int)((long long)(wave + 1) * NT / NW);

  const bf16_t* kg = (const bf16_t*)p.ks + (long long)b * p.bsks + h * D;
  const bf16_t* vg = (const bf16_t*)p.vs + (long long)b * p.bsvs + (long long)h * D * p.vt_ld;

  bf16x8 qreg[4];
  {
    const int qi = q0 + c;
    const bf16_t* qp = (const bf16_t*)p.q + (long long)b * p.bsq + (long long)qi * p.ldq + h * D;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4 tq = {0u, 0u, 0u, 0u};
      if (qi < p.Lq) tq = *reinterpret_cast<const u32x4*>(qp + 16 * s + 8 * g);
      qreg[s] = __builtin_bit_cast(bf16x8, tq);
    }
  }
  // direct loads: instruction j of the wave covers tile rows j*8 + lane/8, 16-byte slot lane%8 (swizzled on the source
  // side); a lane's offsets inside a tile never change (32-bit, the launcher bounds the pitches)
  const int lr = lane >> 3, slot = lane & 7;
  unsigned int kofs[8], vofs[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int row = j * 8 + lr;
    kofs[j] = (unsigned int)row * (unsigned int)p.ldks + (unsigned int)((slot ^ ((row >> 1) & 7)) * 8);
    vofs[j] = (unsigned int)row * (unsigned int)p.vt_ld + (unsigned int)((slot ^ (row & 7) ^ (row >> 3)) * 8);
  }
  char* sk = smem + wave * (2 * TK * D * 2);                 // this wave's K tile [key][d], then its V^T tile [d][key]
  char* sv = sk + TK * D * 2;
  auto issue = [&](int tl) {
    const int key0 = tl * TK;
    if (key0 + TK <= p.L) {                                  // (uniform) every key row of the tile exists
      const bf16_t* kb0 = kg + (long long)key0 * p.ldks;
#pragma unroll
      for (int j = 0; j < 8; ++j) __builtin_amdgcn_global_load_lds(DF_GPTR(kb0 + kofs[j]), DF_LPTR(sk + j * 1024), 16, 0, 0);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = j * 8 + lr;
        int key = key0 + row;
        if (key > p.L - 1) key = p.L - 1;                    // rows beyond the last key are masked in the tile body
        __builtin_amdgcn_global_load_lds(DF_GPTR(kg + (long long)key * p.ldks + ((slot ^ ((row >> 1) & 7)) * 8)),
                                         DF_LPTR(sk + j * 1024), 16, 0, 0);
      }
    }
    const bf16_t* vb0 = vg + key0;                           // the V^T buffer is padded to whole tiles
#pragma unroll
    for (int j = 0; j < 8; ++j) __builtin_amdgcn_global_load_lds(DF_GPTR(vb0 + vofs[j]), DF_LPTR(sv + j * 1024), 16, 0, 0);
  };
  bf16x8 kfr[2][4];
  u32x4 vfr[4][2];
  auto read_frags = [&]() {
    const bf16_t* Ks = reinterpret_cast<const bf16_t*>(sk);
    const bf16_t* Vt = reinterpret_cast<const bf16_t*>(sv);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int row = 32 * kb + key_of_mfma_row(c);
      const int f = (row >> 1) & 7;
#pragma unroll
      for (int s = 0; s < 4; ++s) kfr[kb][s] = *reinterpret_cast<const bf16x8*>(&Ks[row * D + (((2 * s + g) ^ f) * 8)]);
    }
#pragma unroll
    for (int ts = 0; ts < 4; ++ts) {
      const int kchunk = 4 * (ts >> 1) + 2 * (ts & 1) + g;
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        const int d = 32 * db + csig;
        vfr[ts][db] = *reinterpret_cast<const u32x4*>(&Vt[d * TK + (kchunk ^ (d & 7) ^ (d >> 3)) * 8]);
      }
    }
  };

  f32x16 o_acc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o_acc[i][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = p.scale * kLog2e;

  auto tile = [&](int tl, auto raggedc) {
    constexpr bool ragged = decltype(raggedc)::value;
    const int tile_base = tl * TK;
    f32x16 s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) s_acc[kb][e] = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[kb][s], qreg[s], s_acc[kb], 0, 0, 0);
    if constexpr (ragged) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = e >> 2, r = e & 3;
          const int key = tile_base + 32 * kb + 16 * (j >> 1) + 8 * g + 4 * (j & 1) + r;
          if (key >= p.L) s_acc[kb][e] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s_acc[kb][e]);
    mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_ds_bpermute(xor32, __float_as_int(mx)))) * sc;
    const float m_new = fmaxf(m_run, mx);                    // finite: a tile holds at least one key
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float rs = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][e], sc, -m_new));
        s_acc[kb][e] = pv;
        rs += pv;
      }
    l_run = l_run * alpha + rs;                              // this lane's half of the keys; the halves meet at the end
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o_acc[i][e] *= alpha;
    }
#pragma unroll
    for (int ts = 0; ts < 4; ++ts) {
      const int kb = ts >> 1, half = ts & 1;
      u32x4 pk;
      pk.x = pack_bf2(s_acc[kb][8 * half + 0], s_acc[kb][8 * half + 1]);
      pk.y = pack_bf2(s_acc[kb][8 * half + 2], s_acc[kb][8 * half + 3]);
      pk.z = pack_bf2(s_acc[kb][8 * half + 4], s_acc[kb][8 * half + 5]);
      pk.w = pack_bf2(s_acc[kb][8 * half + 6], s_acc[kb][8 * half + 7]);
      const bf16x8 pfrag = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        u32x4 vraw = vfr[ts][db];
        if constexpr (ragged) {                              // keys beyond the range: P is 0, V must be finite
          const int key = tile_base + (4 * kb + 2 * half + g) * 8;
          if (key + 0 >= p.L) vraw.x = 0u; else if (key + 1 >= p.L) vraw.x &= 0xffffu;
          if (key + 2 >= p.L) vraw.y = 0u; else if (key + 3 >= p.L) vraw.y &= 0xffffu;
          if (key + 4 >= p.L) vraw.z = 0u; else if (key + 5 >= p.L) vraw.z &= 0xffffu;
          if (key + 6 >= p.L) vraw.w = 0u; else if (key + 7 >= p.L) vraw.w &= 0xffffu;
        }
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vraw), pfrag, o_acc[db], 0, 0, 0);
      }
    }
  };
  // The query blocks of a head read the same keys; started on the same tile they would all wait for the same cache
  // lines while the rest of the head's K / V^T (cold: other patches' rows, last touched a step ago) is not even
  // requested.  Block qb therefore walks each wave's run of tiles from a different starting tile, wrapping around:
  // ten blocks keep ten tiles per wave slot in flight and find the others' tiles in L2.  The order is a fixed
  // function of the indices, so results stay reproducible.
  const int nt = t_hi - t_lo;
  const int rot = ((qb & 7) * nt) >> 3;                      // < nt, spread over the run
  auto tile_at = [&](int i) { const int k = i + rot; return t_lo + (k < nt ? k : k - nt); };
  if (nt > 0) issue(tile_at(0));
  DF_ATRACE(2, __builtin_readcyclecounter());
  for (int i = 0; i < nt; ++i) {
    const int tl = tile_at(i);
    __builtin_amdgcn_s_waitcnt((0 & 0xF) | (0x7 << 4) | (0xF << 8));   // vmcnt(0): the tile has landed in LDS
    asm volatile("" ::: "memory");
    DF_ATRACE(3 + 3 * i, __builtin_readcyclecounter());
    read_frags();
    __builtin_amdgcn_s_waitcnt((0x3F & 0xF) | ((0x3F >> 4) << 14) | (0x7 << 4) | (0 << 8));   // lgkmcnt(0): fragments in registers
    asm volatile("" ::: "memory");
    DF_ATRACE(4 + 3 * i, __builtin_readcyclecounter());
    if (i + 1 < nt) issue(tile_at(i + 1));                   // (uniform) into the LDS just read, under this tile's work
    __builtin_amdgcn_sched_barrier(0);
    if (tl * TK + TK <= p.L) tile(tl, std::false_type{});
    else tile(tl, std::true_type{});
    __builtin_amdgcn_sched_barrier(0);
    DF_ATRACE(5 + 3 * i, __builtin_readcyclecounter());
  }
  __builtin_amdgcn_s_waitcnt((0 & 0xF) | (0x7 << 4) | (0 << 8));
  l_run += __int_as_float(__builtin_amdgcn_ds_bpermute(xor32, __float_as_int(l_run)));

  // ---- merge the NW states in wave order ----
  __syncthreads();                                           // every wave is done with its tiles: the LDS is free
  float* mrg = reinterpret_cast<float*>(smem);               // [NW][34][64]: 32 accumulators, max, sum per lane
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) mrg[(wave * 34 + i * 16 + e) * 64 + lane] = o_acc[i][e];
  mrg[(wave * 34 + 32) * 64 + lane] = m_run;
  mrg[(wave * 34 + 33) * 64 + lane] = l_run;
  __syncthreads();
  DF_ATRACE(28, __builtin_readcyclecounter());
  DF_ATRACE(31, nt);
  const int qi = q0 + c;
  if (qi >= p.Lq) return;
  float mw[NW], m_all = -INFINITY;
#pragma unroll
  for (int w = 0; w < NW; ++w) { mw[w] = mrg[(w * 34 + 32) * 64 + lane]; m_all = fmaxf(m_all, mw[w]); }
  float l_all = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    mw[w] = __builtin_amdgcn_exp2f(mw[w] - m_all);           // a wave without keys has max -inf: weight 0
    l_all = fmaf(mw[w], mrg[(w * 34 + 33) * 64 + lane], l_all);
  }
  const float inv = __builtin_amdgcn_rcpf(l_all);
  // wave w finishes accumulators 4w .. 4w+3 (NW == 8) of every lane: 4 consecutive features of the lane's query
  constexpr int PER = 32 / NW;
  static_assert(PER == 4 || PER == 8, "four or eight waves");
  float o[PER];
#pragma unroll
  for (int k = 0; k < PER; ++k) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) v = fmaf(mw[w], mrg[(w * 34 + wave * PER + k) * 64 + lane], v);
    o[k] = v * inv;
  }
  const int e0 = wave * PER;                                 // accumulator index = 16 * db + 8 * f + e
  const int db = e0 >> 4, f = (e0 >> 3) & 1, eo = e0 & 7;
  bf16_t* dst;
  if (p.out_packed) {
    const long long m = (long long)b * p.Lq + qi;
    dst = (bf16_t*)p.out + (((m >> 5) * (long long)(p.heads * D / 16) + h * (D / 16)) * 64 + (m & 31) + 32 * g) * 8 +
          (2 * db + f) * 512 + eo;
  } else {
    dst = (bf16_t*)p.out + (long long)b * p.bso + (long long)qi * p.ldo + h * D + 32 * db + 16 * f + 8 * g + eo;
  }
  if constexpr (PER == 4) {
    u32x2 tq = {pack_bf2(o[0], o[1]), pack_bf2(o[2], o[3])};
    *reinterpret_cast<u32x2*>(dst) = tq;
  } else {
    u32x4 tq = {pack_bf2(o[0], o[1]), pack_bf2(o[2], o[3]), pack_bf2(o[4], o[5]), pack_bf2(o[6], o[7])};
    *reinterpret_cast<u32x4*>(dst) = tq;
  }
  DF_ATRACE(29, __builtin_readcyclecounter());
  DF_ATRACE(30, wall_clock64());
}

// merges the per-split partials: one lane per (query, 4 consecutive d)
__global__ __launch_bounds__(256) void attn_combine_d64(AttnParams p) {
  constexpr int D = 64;
  // 32-bit index arithmetic (the launcher bounds rows * 16 below 2^31): the 64-bit divisions below were a tenth of
  // this kernel's time
  const unsigned int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const unsigned int rows = (unsigned int)(p.B * p.heads * p.Lq);
  if (idx >= rows * (D / 4)) return;
  const unsigned int row = idx / (D / 4);
  const int d4 = (int)(idx % (D / 4)) * 4;
  float m = -INFINITY;
  for (int s = 0; s < p.nsplit; ++s) m = fmaxf(m, p.part_ml[((size_t)s * rows + row) * 2]);
  float l = 0.f;
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < p.nsplit; ++s) {
    const float w = __builtin_amdgcn_exp2f(p.part_ml[((size_t)s * rows + row) * 2] - m);
    l += w * p.part_ml[((size_t)s * rows + row) * 2 + 1];
    const f32x4 t = *reinterpret_cast<const f32x4*>(p.part_o + ((size_t)s * rows + row) * D + d4);
    o += t * w;
  }
  const float inv = __builtin_amdgcn_rcpf(l);
  const unsigned int bh = row / (unsigned int)p.Lq;
  const int qi = (int)(row - bh * (unsigned int)p.Lq);
  const int b = (int)(bh / (unsigned int)p.heads);
  const int h = (int)(bh - (unsigned int)b * (unsigned int)p.heads);
  bf16_t* op = (bf16_t*)p.out + (long long)b * p.bso + (long long)qi * p.ldo + h * D + d4;
  if (p.out_packed) {
    const long long m = (long long)b * p.Lq + qi;
    const int col = h * D + d4;
    op = (bf16_t*)p.out + (((m >> 5) * (long long)(p.heads * D / 16) + (col >> 4)) * 64 + (m & 31) + 32 * ((col >> 3) & 1)) * 8 + (col & 7);
  }
  u32x2 t = {pack_bf2(o.x * inv, o.y * inv), pack_bf2(o.z * inv, o.w * inv)};
  *reinterpret_cast<u32x2*>(op) = t;
}

// ---- f32: one wave per (batch, head, query); lanes stride over keys ----
template <int D>
__global__ __launch_bounds__(256) void attn_f32(AttnParams p) {
  const int lane = threadIdx.x & 63;
  const long long wid = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long total = (long long)p.B * p.heads * p.Lq;
  if (wid >= total) return;
  const int qi = (int)(wid % p.Lq);
  const int h = (int)((wid / p.Lq) % p.heads);
  const int b = (int)(wid / ((long long)p.Lq * p.heads));
  const float* qp = (const float*)p.q + (long long)b * p.bsq + (long long)qi * p.ldq + h * D;
  const float* kf = (const float*)p.kf + (long long)b * p.bskf + h * D;
  const float* vf = (const float*)p.vf + (long long)b * p.bsvf + h * D;
  const float* ks = p.ks ? (const float*)p.ks + (long long)b * p.bsks + h * D : nullptr;
  const float* vs = p.vs ? (const float*)p.vs + (long long)b * p.bsvs + h * D : nullptr;
  float qv[D];
#pragma unroll
  for (int i = 0; i < D; ++i) qv[i] = qp[i];
  float m = -INFINITY, l = 0.f, acc[D];
#pragma unroll
  for (int i = 0; i < D; ++i) acc[i] = 0.f;
  for (int j = lane; j < p.L; j += 64) {
    const long long fr = fresh_row(p.own_lo, p.own_n, p.own_period, j);
    const float* kr = fr >= 0 ? kf + fr * p.ldkf : ks + (long long)j * p.ldks;
    const float* vr = fr >= 0 ? vf + fr * p.ldvf : vs + (long long)j * p.ldvs;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < D; ++i) s = fmaf(qv[i], kr[i], s);
    s *= p.scale;
    const float mn = fmaxf(m, s);
    const float a = expf(m - mn), e = expf(s - mn);
    l = l * a + e;
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] = fmaf(acc[i], a, e * vr[i]);
    m = mn;
  }
  const float mg = wave_max(m);
  const float w = (m == -INFINITY) ? 0.f : expf(m - mg);
  l = wave_sum(l * w);
  float* op = (float*)p.out + (long long)b * p.bso + (long long)qi * p.ldo + h * D;
#pragma unroll
  for (int i = 0; i < D; ++i) {
    const float v = wave_sum(acc[i] * w);
    if (lane == (i & 63)) op[i] = v / l;
  }
}

// Number of key-range splits.  Cost model from the kernel traces of the patch step: a compute unit works through its
// workgroups' 64-key tiles at a roughly constant rate whether one or three of them are resident, so the time follows
// the most loaded unit, ceil(workgroups / 256) x (tiles per workgroup + a fixed part); the merge kernel grows with the
// number of partials.  (Plain "at least 512 workgroups" picked 800 for the 1200-query level: 768 run at once and
// the last 32 had the chip to themselves for a full workgroup lifetime, +35 %.)
int pick_splits(int B, int Lq, int L, int heads) {
  static const int forced = tune_env("DF_ATTN_SPLITS") ? atoi(tune_env("DF_ATTN_SPLITS")) : 0;   // tuning aid
  if (forced > 0) return (L / forced >= 64) ? forced : 1;
  const long long blocks = (long long)cdiv(Lq, 128) * heads * B;
  int best = 1;
  double best_cost = 1e30;
  for (int ns = 1; ns <= 16; ++ns) {
    if (ns > 1 && L / ns < 128) break;
    const int tiles = cdiv(cdiv(L, ns), 64);
    const long long per_cu = (blocks * ns + 255) / 256;
    const double cost = (double)per_cu * (tiles + 2) + (ns > 1 ? 1.0 + 0.5 * ns : 0.0);
    if (cost < best_cost - 1e-9) { best_cost = cost; best = ns; }
  }
  return best;
}

}  // namespace

#ifdef DF_TUNING
// Tuning build only: copies the stamps of the last attn_wave_d64 launch to host memory (synchronises).
extern "C" __attribute__((visibility("default"))) int df_tune_attn_trace(long long* out, int n) {
  if (!out || n <= 0 || n > 512 * 32) return DF_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return DF_EHIP;
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(g_attn_trace), (size_t)n * sizeof(long long)) != hipSuccess) return DF_EHIP;
  return DF_OK;
}
#endif

size_t attention_scratch_bytes(int B, int Lq, int L, int heads, int d) {
  const int ns = pick_splits(B, Lq, L, heads);
  if (ns == 1) return kScratchCounterBytes;
  return kScratchCounterBytes + (size_t)ns * B * heads * Lq * (d + 2) * sizeof(float) + 256;
}

int launch_attention(const AttnArgs& a, hipStream_t st) {
  if (a.B <= 0 || a.Lq <= 0 || a.L <= 0 || a.heads <= 0) return DF_ESHAPE;
  if (!(a.scale > 0.f) || !(a.scale < INFINITY)) return DF_EINVAL;   // the kernels fold the scale into exp2 arguments
  if (a.own_period < 0 || (a.own_period > 0 && (a.L % a.own_period || a.own_lo < 0 || a.own_lo + a.own_n > a.own_period)))
    return DF_ESHAPE;
  const bool own_all = a.own_lo <= 0 && a.own_lo + a.own_n >= (a.own_period > 0 ? a.own_period : a.L);
  if (!own_all && (!a.k_stale || !a.v_stale)) return DF_EINVAL;
  AttnParams p = {};
  p.q = a.q; p.kf = a.k_fresh; p.vf = a.v_fresh; p.ks = a.k_stale; p.vs = a.v_stale; p.out = a.out;
  p.B = a.B; p.Lq = a.Lq; p.L = a.L; p.heads = a.heads; p.own_lo = a.own_lo; p.own_n = a.own_n;
  p.own_period = a.own_period;
  p.ldq = a.ldq; p.ldkf = a.ldkf; p.ldvf = a.ldvf; p.ldks = a.ldks; p.ldvs = a.ldvs; p.ldo = a.ldo;
  p.bsq = a.bsq; p.bskf = a.bskf; p.bsvf = a.bsvf; p.bsks = a.bsks; p.bsvs = a.bsvs; p.bso = a.bso;
  p.scale = a.scale;
  p.nsplit = 1; p.keys_per_split = a.L;
  p.out_packed = a.out_packed;
  if (a.out_packed && (a.dtype != DF_BF16 || ((uintptr_t)a.out % 16))) return DF_EINVAL;
  if (a.dtype == DF_F32) {
    const long long waves = (long long)a.B * a.heads * a.Lq;
    dim3 grid((unsigned)((waves + 3) / 4));
    if (a.d == 32) hipLaunchKernelGGL(attn_f32<32>, grid, dim3(256), 0, st, p);
    else if (a.d == 64) hipLaunchKernelGGL(attn_f32<64>, grid, dim3(256), 0, st, p);
    else return DF_ESHAPE;
    DF_LAUNCH_CHECK();
    return DF_OK;
  }
  if (a.d != 64) return DF_ESHAPE;
  const long long lds[] = {a.ldq, a.ldkf, a.ldvf, a.ldks, a.ldvs, a.ldo, a.bsq, a.bskf, a.bsvf, a.bsks, a.bsvs, a.bso};
  for (long long v : lds) if (v % 8) return DF_EINVAL;
  const void* ptrs[] = {a.q, a.k_fresh, a.v_fresh, a.k_stale, a.v_stale, a.out};
  for (const void* q : ptrs) if ((uintptr_t)q % 16) return DF_EINVAL;
  // Few queries against many keys (the patch at the deepest level): one workgroup per 32-query block and head whose
  // waves split the keys; no partials, no merge kernel.  Each block streams the head's whole K / V^T, so this pays
  // only while the query blocks are few: a compute unit then pulls Lq / 32 x the head's keys through its load path where
  // the LDS-tiled kernel pulls Lq / 128 x.  Measured: 300 queries x 2400 keys 17.9 -> 16.6 us (both launches of the
  // split form counted), 1024 x 4096 49.2 -> 56.4 us.
  // It also wants its workgroups in one round (at most one per compute unit): two batch items of 300 queries make 400
  // workgroups, 144 units run two of them in turn, and the split form wins again (2.48 vs 3.02 ms per step).
  static const int wave_lq = tune_env("DF_ATTN_WAVE_LQ") ? atoi(tune_env("DF_ATTN_WAVE_LQ")) : 512;   // tuning aid
  if (a.v_transposed && a.Lq <= wave_lq && a.L >= 512 && (long long)cdiv(a.Lq, 32) * a.heads * a.B <= 256) {
    if (!a.k_stale || !a.v_stale || a.own_n != 0 || a.own_period != 0 || a.vt_ld % 8 || a.vt_ld < (long long)cdiv(a.L, 64) * 64) return DF_EINVAL;
    if (a.ldks <= 0 || a.ldks >= (1 << 23) || a.vt_ld >= (1 << 25)) return DF_ESHAPE;   // 32-bit offsets inside a tile
    p.vt_ld = a.vt_ld;
    if (a.B > 65535 || cdiv(a.Lq, 32) > 65535) return DF_ESHAPE;
    const dim3 grid((unsigned)(cdiv(a.heads, 8) * 8), (unsigned)cdiv(a.Lq, 32), (unsigned)a.B);
    constexpr int NW = 8;
    constexpr int smem = NW * 2 * 64 * 64 * 2;          // a K and a V^T tile per wave; the merge reuses it
    static_assert(NW * 34 * 64 * 4 <= smem, "the merge fits");
    static bool attr_set = false;
    if (!attr_set) {
      if (hipFuncSetAttribute((const void*)attn_wave_d64<NW>, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
        return DF_EHIP;
      attr_set = true;
    }
    hipLaunchKernelGGL(attn_wave_d64<NW>, grid, dim3(64 * NW), smem, st, p);
    DF_LAUNCH_CHECK();
    return DF_OK;
  }
  int ns = pick_splits(a.B, a.Lq, a.L, a.heads);
  if ((long long)a.B * ns > 65535) return DF_ESHAPE;
  if ((long long)a.B * a.heads * a.Lq * 16 >= (1LL << 31)) return DF_ESHAPE;   // the merge kernel indexes with 32 bits
  if (ns > 1) {
    const int kps = cdiv(cdiv(a.L, ns), 128) * 128;      // whole 128-key iterations of the two-group kernel
    ns = cdiv(a.L, kps);                                 // rounding up may leave the last ranges empty: drop them
    if (ns > 1) {
      char* scr = scratch_region(a.scr, attention_scratch_bytes(a.B, a.Lq, a.L, a.heads, a.d));
      if (!scr) return DF_ENOMEM;
      p.nsplit = ns;
      p.keys_per_split = kps;
      p.part_o = (float*)(scr + kScratchCounterBytes);
      p.part_ml = p.part_o + (size_t)ns * a.B * a.heads * a.Lq * 64;
    }
  }
  const long long nwg = (long long)cdiv(a.Lq, 128) * a.heads * a.B * p.nsplit;
  if (nwg > 0x7fffffffLL) return DF_ESHAPE;
  if (a.v_transposed) {
    // every key from k_stale (row-major) / v_stale (V^T, row pitch vt_ld >= L rounded up to whole 64-key tiles)
    if (!a.k_stale || !a.v_stale || a.own_n != 0 || a.own_period != 0 || a.vt_ld % 8 || a.vt_ld < (long long)cdiv(a.L, 64) * 64) return DF_EINVAL;
    if (a.ldks <= 0 || a.ldks >= (1 << 23) || a.vt_ld >= (1 << 25)) return DF_ESHAPE;   // 32-bit offsets inside a tile
    p.vt_ld = a.vt_ld;
    // Up to ~600 workgroups (at most two per compute unit): two groups of four waves and a two-stage ring (64 KB of
    // LDS); measured on the patch step, the second group gains ~9 % over one group with a three-stage ring.  Larger
    // launches keep one group and three stages (48 KB, three workgroups per unit), which is faster there (the
    // 480 x 480-latent share: 27.4 vs 31.5 ms of self-attention).  Deeper rings lose in both forms: the kernel is not
    // bound by the latency of the K / V^T stream.
    static const int forced_st = tune_env("DF_ATTN_STAGES") ? atoi(tune_env("DF_ATTN_STAGES")) : 0;   // tuning aid
    static const int forced_gr = tune_env("DF_ATTN_GROUPS") ? atoi(tune_env("DF_ATTN_GROUPS")) : 0;   // tuning aid
    static const long long g2max = tune_env("DF_ATTN_G2MAX") ? atoll(tune_env("DF_ATTN_G2MAX")) : 600;   // tuning aid
    const int ngr = forced_gr ? forced_gr : (nwg <= g2max ? 2 : 1);
    const int nst = forced_st ? forced_st : (ngr == 2 ? 2 : 3);
#define DF_ATTN_VT(NSTV, NGRV)                                                                                      \
  {                                                                                                                 \
    constexpr int smem = NSTV * 2 * 64 * 64 * 2 * NGRV;                                                             \
    static bool attr_set = false;                                                                                   \
    if (!attr_set) {                                                                                                \
      if (hipFuncSetAttribute((const void*)attn_vt_d64<NSTV, NGRV>, hipFuncAttributeMaxDynamicSharedMemorySize,     \
                              smem) != hipSuccess)                                                                  \
        return DF_EHIP;                                                                                             \
      attr_set = true;                                                                                              \
    }                                                                                                               \
    hipLaunchKernelGGL((attn_vt_d64<NSTV, NGRV>), dim3((unsigned)nwg), dim3(256 * NGRV), smem, st, p);              \
  }
    if (ngr == 2) { if (nst <= 2) DF_ATTN_VT(2, 2) else if (nst == 3) DF_ATTN_VT(3, 2) else DF_ATTN_VT(4, 2) }
    else if (nst <= 3) DF_ATTN_VT(3, 1) else if (nst == 4) DF_ATTN_VT(4, 1) else DF_ATTN_VT(6, 1)
#undef DF_ATTN_VT
  } else {
    // 32-bit row offsets inside a 64-key tile
    if (a.ldkf >= (1 << 24) || a.ldvf >= (1 << 24) || a.ldks >= (1 << 24) || a.ldvs >= (1 << 24)) return DF_ESHAPE;
    if (a.own_period > 0) hipLaunchKernelGGL(attn_bf16_d64<true>, dim3((unsigned)nwg), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(attn_bf16_d64<false>, dim3((unsigned)nwg), dim3(256), 0, st, p);
  }
  DF_LAUNCH_CHECK();
  if (ns > 1) {
    const long long n = (long long)a.B * a.heads * a.Lq * 16;
    hipLaunchKernelGGL(attn_combine_d64, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p);
    DF_LAUNCH_CHECK();
  }
  return DF_OK;
}

}  // namespace df
