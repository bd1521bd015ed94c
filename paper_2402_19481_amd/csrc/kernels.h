// Internal launch interface of the gfx950 kernels.  Every function enqueues on
// `st` and returns a DF_* code; shapes are validated by the callers in api.cpp
// and unet.cpp, so these check only what the kernels themselves assume.
#pragma once
#include "common.h"

namespace df {

// ---- device scratch ----
// Kernels that need device memory beyond their inputs and outputs (GroupNorm partial sums, split-K and split-key
// partials, the page of zeros behind the convolution's padding) take it from a Scratch region.  A UNet plan carves
// its region out of the caller's workspace, so the graphs it records only ever hold plan-owned addresses; the
// per-operation entry points use one region per device that the library allocates on first use.  That region is
// never freed or moved while the process lives: a larger request allocates a further buffer and the old one stays
// valid for anything that still holds its address.
// The first 16 KiB of a region are reserved: [0, 8 KiB) counters that every kernel leaves at zero,
// [8 KiB, 16 KiB) a page of zeros nobody writes.
struct Scratch {
  char* ptr;
  size_t bytes;
};
constexpr size_t kScratchCounterBytes = 16384;
constexpr size_t kScratchZeroPageOffset = 8192;
constexpr int kScratchNumCounters = 2048;
// Region of at least `bytes` for a launch: `given` if non-null (nullptr result if it is too small), else the
// library's per-device region.  Returns nullptr on failure.
char* scratch_region(const Scratch* given, size_t bytes);
// Zeroes the reserved head of a caller-provided region (synchronous; used once when a plan is created).
int scratch_init(const Scratch& s);

// ---- refresh.hip ----
int launch_copy_rows(void* dst, const void* src, long long rows, long long row_bytes, long long dst_stride_bytes,
                     long long src_stride_bytes, hipStream_t st);

// ---- groupnorm.hip ----
struct GnArgs {
  const void* x;        // [B, nseg*Rseg, W, C]
  void* y;              // same shape, out dtype
  const float* stale;   // [N,B,G,2] or nullptr (nseg > 1 or N == 1)
  float* sums_out;      // nseg == 1: [B,G,2] (may be null); nseg > 1: [nseg,B,G,2]
  const float* gamma;
  const float* beta;
  int B, Rseg, W, C, G;
  int nseg;             // 1: one patch (displaced); >1: full image split into nseg patches, exact statistics
  int patch_idx, N;
  float eps;
  int stat_mode, silu;
  int in_dtype, out_dtype;
  // optional copy of the boundary rows of y (bf16 output, row-major y only) into the stale state of the convolution
  // that consumes y: [B, halo_npatch, 2, W, C]; pixel row r belongs to patch halo_patch0 + r / halo_rpp and is stored
  // as that patch's first (r % halo_rpp == 0) and / or last (== halo_rpp - 1) row
  void* halo_out;
  int halo_rpp, halo_patch0, halo_npatch;
  // halo_cols != 0: the patches are vertical strips of halo_rpp columns; the state is [B, halo_npatch, 2, rows, C]
  // (first and last column of every patch, rows = Rseg * nseg) and pixel column c belongs to patch
  // halo_patch0 + c / halo_rpp
  int halo_cols;
  int y_packed;         // bf16 output in the fragment-packed layout of wgemm.hip (rows = B*rows*W pixels, K = C)
  const Scratch* scr;   // scratch region of the caller (a plan's), or nullptr: the library's per-device region
};
int launch_groupnorm(const GnArgs& a, hipStream_t st);
// Per-strip (sum, sum of squares) of a full image split into N vertical strips: x [B, R, W, C] (float or bf16) ->
// sums [N, B, G, 2], the content of the GroupNorm cache after a synchronous step on vertical strips.
int launch_gn_strip_sums(const void* x, int in_dtype, float* sums, int B, int R, int W, int C, int G, int N, hipStream_t st);
// df_groupnorm_stale's arguments, validated and launched with the given scratch region (nullptr: the library's)
int groupnorm_entry(const void* x_fresh, void* y, const float* stale_stats, float* fresh_stats_out, const float* gamma,
                    const float* beta, int B, int R, int W, int C, int G, int patch_idx, int N, float eps, int stat_mode,
                    int fuse_silu, int dtype, const Scratch* scr, hipStream_t st);
size_t groupnorm_scratch_bytes(int B, int nseg, int G, int N);

// ---- conv.hip / gemm ----
struct ConvArgs {
  const void* x;         // fresh rows [B, R, W, Cin]
  const void* halo_top;  // row above the patch [B][W*Cin] with batch stride halo_bstride elements, or nullptr (zero)
  const void* halo_bot;  // row below the patch, or nullptr
  long long halo_bstride;
  // patches that are vertical strips: the stale pixel left / right of input row r of batch item b sits at
  // halo_left + b*side_bstride + r*side_rstride (elements), nullptr = zero (image border); excludes the row halos
  const void* halo_left;
  const void* halo_right;
  long long side_bstride, side_rstride;
  const void* w;         // [Cout, 3, 3, Cin]
  const float* bias;     // [Cout] or nullptr
  const float* chan_add; // [B, Cout] added per batch item and channel (row stride chan_ld), or nullptr
  long long chan_ld;
  const float* residual; // [B, Ro, Wo, Cout] float added before the activation, or nullptr
  void* y;               // [B, Ro, Wo, Cout]
  int B, R, W, Cin, Cout, stride, act;
  int dtype;             // of x, halos and w
  int out_dtype;
  const Scratch* scr;    // see GnArgs
};
int launch_conv3x3(const ConvArgs& a, hipStream_t st);

struct GemmArgs {
  const void* A;  // [M, K] bf16, row stride lda
  const void* W;  // [N, K] bf16, row stride ldw
  const float* bias;      // [N] or nullptr
  const float* residual;  // [M, N] float, row stride ldr, or nullptr (may alias out when out is float)
  void* out;              // [M, N], row stride ldo
  int M, N, K;
  long long lda, ldw, ldr, ldo;
  int act;        // 0 none, 1 SiLU
  int out_dtype;
  // GEGLU epilogue: W holds 2F rows (F value rows, then F gate rows), N = 2F; the output is [M, F] bf16 with
  // out[m, f] = (x w_f + b_f) * gelu(x w_{F+f} + b_{F+f}).  Requires K % 64 == 0, K >= 128, F % 64 == 0.
  int geglu;
  // Segmented bf16 output (fused QKV projection): column segment s = col / seg_w is written to seg_out[s] instead of
  // `out`; input row m lands on row (m / seg_rows_in[s]) * seg_rows_out[s] + seg_row0[s] + m % seg_rows_in[s] with
  // row stride seg_ld[s].  nseg = 0: plain output.  Requires K % 64 == 0, K >= 128, no split-K (any K is accepted).
  int nseg, seg_w;
  void* seg_out[3];
  long long seg_ld[3], seg_rows_out[3], seg_row0[3];
  int seg_rows_in[3];
  // seg_tr[s] != 0: segment s is written transposed, out[(b * seg_w + col) * seg_ld[s] + seg_row0[s] + row_in_batch]
  // (feature-major, rows contiguous: the V^T layout of the attention kernel); seg_rows_out is ignored for it
  int seg_tr[3];
  // seg_pin[s] > 0: row m of a batch item is token (m / seg_pin, m % seg_pin) of a vertical strip and lands on row
  // seg_row0 + (m / seg_pin) * seg_pout + m % seg_pin of the destination's batch item (its grid rows are seg_pout long)
  int seg_pin[3], seg_pout[3];
  // W is in the tiled layout written by launch_pack_weight (requires N % 64 == 0, K % 64 == 0, K >= 128).
  int packed_w;
  // LayerNorm folded into the GEMM: A holds the un-normalised rows (bf16), W was packed with the norm scale
  // multiplied in, ln_s[n] = sum_k W'[n,k], ln_t[n] = sum_k W[n,k] beta[k] + bias[n] (bias must then be null).
  // The kernel derives each row's mean and rstd from the A tiles it streams and applies
  // out = rstd * (acc - mean * ln_s[n]) + ln_t[n].  Requires the pipelined kernel (K % 64 == 0, K >= 128).
  const float* ln_s;
  const float* ln_t;
  float ln_eps;
  // optional second output: the same values rounded to bf16, [M, N] with row stride ldo2 (plain outputs only)
  void* out2;
  long long ldo2;
  const Scratch* scr;     // see GnArgs
};
int launch_gemm_bf16(const GemmArgs& a, hipStream_t st);
// Weight re-layout for the pipelined kernel: 64x64 tiles [N/64][K/64][64][64] with the LDS swizzle baked in, optionally
// scaled per input channel by gamma[K] before rounding.  N % 64 == 0, K % 64 == 0.
int launch_pack_weight(const bf16_t* w, const float* gamma, bf16_t* out, int N, int K, hipStream_t st);
// s[n] = sum_k bf16(w[n,k] * gamma[k]); t[n] = sum_k w[n,k] * beta[k] + bias[n] (bias may be null)
int launch_fold_vectors(const bf16_t* w, const float* gamma, const float* beta, const float* bias, float* s, float* t,
                        int N, int K, hipStream_t st);
size_t gemm_scratch_bytes(long long M, long long N);  // also covers a convolution with M output pixels, N = Cout

// ---- wgemm.hip: linear layers on fragment-packed operands ----
// Packed layout of a [R, K] bf16 matrix: fragments [ceil(R/32)][K/16][64 lanes][8], lane l of fragment (rt, kf)
// holding row rt*32 + l%32, columns kf*16 + 8*(l/32) .. +7 (rows beyond R are zero).  Weights use the same layout with
// the in-fragment row i holding matrix row rt*32 + (i with bits 2 and 3 swapped).
struct WGemmArgs {
  const void* Xp;         // packed activations [M, K]
  const void* Wp;         // packed weights [N, K]
  int M, N, K;            // K % 64 == 0, N % 32 == 0
  const float* bias;      // [N] or nullptr
  const float* ln_s;      // folded LayerNorm vectors (see GemmArgs), or nullptr
  const float* ln_t;
  float ln_eps;
  const float* residual;  // row-major [M, N'] float, row stride ldr, or nullptr (may alias out_f32)
  long long ldr;
  float* out_f32;         // row-major [M, N'] float, row stride ldo, or nullptr
  long long ldo;
  void* out_packed;       // packed bf16 [M, N'] (the next layer's activation operand), or nullptr
  void* out_rows;         // row-major bf16 [M, N'], row stride ld_rows, or nullptr
  long long ld_rows;
  int geglu;              // F: W holds F value rows then F gate rows (N == 2F), N' = F; 0: N' = N
  int nseg, seg_w;        // segmented row-major bf16 output as in GemmArgs (replaces out_rows)
  void* seg_out[3];
  long long seg_ld[3], seg_rows_out[3], seg_row0[3];
  int seg_rows_in[3];
  int seg_tr[3];          // transposed segments, as in GemmArgs
  int seg_pin[3], seg_pout[3];   // strip-of-a-grid row mapping, as in GemmArgs
  // Fused cross-attention: the layer is a query projection with N = heads * 64 and a folded LayerNorm; instead of
  // the projection the kernel writes out_packed = softmax(q k^T * xa_scale) v per head, against xa_keys text tokens
  // whose keys / values were packed by launch_pack_text_kv (xa_kv: this block's fragments, batch stride
  // xa_bstride elements; xa_rows token rows per batch item, a multiple of 32 unless there is one batch item).
  const void* xa_kv;
  int xa_keys, xa_rows;
  long long xa_bstride;
  float xa_scale;
};
int launch_wgemm(const WGemmArgs& a, hipStream_t st);
size_t packed_rows_bytes(long long M, long long K);
int launch_pack_rows(const bf16_t* x, long long ldx, bf16_t* out, int M, int K, hipStream_t st);
int launch_pack_wfrag(const bf16_t* w, const float* gamma, bf16_t* out, int N, int K, hipStream_t st);
// Text keys / values of `count` transformer blocks (kv [B*TL, count*2C] row-major: per block C key then C value
// columns) -> MFMA fragments [B][count][heads][12*XA][64][8], XA = ceil(TL/32): per head 4*XA key fragments (32 keys x
// 16 d, key rows in the bit-2/3-swapped order, zero beyond TL) then 4*XA value fragments (V^T: 32 d x 16 keys).
size_t packed_text_kv_bytes(int B, int TL, int count, int C);
int launch_pack_text_kv(const bf16_t* kv, long long ld, bf16_t* out, int B, int TL, int count, int C, hipStream_t st);

// ---- attn.hip ----
struct AttnArgs {
  const void* q;        // [B, Lq, heads*d], row stride ldq, batch stride bsq
  const void* k_fresh;  // rows [own_lo, own_lo + own_n) of the key set
  const void* v_fresh;
  const void* k_stale;  // all other rows, indexed by absolute key row; may be null if own range covers everything
  const void* v_stale;
  void* out;            // [B, Lq, heads*d]
  int B, Lq, L, heads, d;
  int own_lo, own_n;    // key rows [own_lo, own_lo+own_n) come from the fresh tensors (row 0 of fresh = key own_lo)
  int own_period;       // P > 0 (vertical strip of a token grid with P columns, L % P == 0): key j is fresh iff j % P is
                        // in [own_lo, own_lo+own_n), and is then row (j / P) * own_n + j % P - own_lo of the fresh tensors
  long long ldq, ldkf, ldvf, ldks, ldvs, ldo;
  long long bsq, bskf, bsvf, bsks, bsvs, bso;  // batch strides in elements
  float scale;
  int dtype;
  int out_packed;       // bf16 output in the fragment-packed layout of wgemm.hip: rows = B*Lq tokens, K = heads*d
  // v_transposed: v_stale is V^T [B][heads*d][vt_ld] (key index contiguous, vt_ld >= L rounded up to 64, batch stride
  // bsvs) and every key is read from k_stale / v_stale (own_n must be 0; k_fresh / v_fresh are ignored); bf16, d = 64
  int v_transposed;
  long long vt_ld;
  const Scratch* scr;   // see GnArgs
};
int launch_attention(const AttnArgs& a, hipStream_t st);
size_t attention_scratch_bytes(int B, int Lq, int L, int heads, int d);

// ---- elementwise.hip ----
int launch_layernorm(const float* x, bf16_t* y, const float* gamma, const float* beta, int M, int C, float eps, hipStream_t st);
int launch_geglu(const bf16_t* h, bf16_t* out, int M, int F, hipStream_t st);  // h [M, 2F] -> out [M, F]
int launch_cast_bf16(const float* x, bf16_t* y, long long n, int silu, hipStream_t st);
int launch_concat(const float* a, int Ca, const float* b, int Cb, float* out, bf16_t* out_bf, long long pixels,
                  hipStream_t st);   // out_bf: optional bf16 copy of the result
int launch_upsample2x_bf16(const float* x, bf16_t* y, int B, int R, int W, int C, hipStream_t st);
int launch_axpy(float* x, const float* e, float alpha, long long n, hipStream_t st);
int launch_mfma_probe(float* out, int blocks, int iters, hipStream_t st);
size_t sync_probe_bytes(int blocks);
int launch_sync_probe(void* buf, int blocks, int iters, int mode, hipStream_t st);
int launch_scale(float* y, const float* x, float alpha, long long n, hipStream_t st);

}  // namespace df
