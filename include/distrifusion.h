/*
 * distrifusion.h - C ABI of the displaced-patch hot path for AMD MI355X (gfx950).
 *
 * One device's view of displaced patch parallelism (DistriFusion, Section 4):
 * the image is split into N horizontal patches; this device computes patch
 * `patch_idx` fresh, and every layer that mixes information across space takes
 * the context of the other patches from full-shape buffers of stale activations
 * left by the previous denoising step.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  Inputs are
 *     never modified; outputs are fully overwritten.  Activations are
 *     channels-last: [B, rows, W, C], equivalently [B, tokens, C].
 *   - `dtype` is DF_F32 or DF_BF16 and applies to activations and to matrix /
 *     convolution weights.  Biases, norm scale/shift and statistics are float.
 *     bf16 kernels accumulate in float.
 *   - `stream` is a hipStream_t (0 = default stream).  Calls are asynchronous
 *     on that stream and return after enqueueing.
 *   - Patches: a full tensor of H rows is split into N strips of R = H / N
 *     rows; patch i owns rows [i*R, (i+1)*R).  H % N must be 0.
 *   - Return value: DF_OK, or a negative error; arguments are checked before
 *     the first launch, so nothing has been enqueued when an argument error
 *     (DF_EINVAL, DF_ESHAPE, DF_ENOMEM) comes back.
 *   - Scratch: the per-operation entry points keep one scratch region per device
 *     (GroupNorm partial sums, split-K and split-key partials, a page of zeros).
 *     It is allocated on first use and only ever grows; growing allocates a
 *     further buffer and never frees or moves the previous one, so work that is
 *     still queued, or a graph captured around these calls, keeps valid
 *     addresses.  The allocation must not happen during stream capture: call an
 *     entry point eagerly once with the shape before capturing it.  A UNet plan
 *     does not use this region at all: its scratch is part of the workspace the
 *     caller hands to df_unet_create.
 *   - Calls on different streams must not share a scratch region concurrently:
 *     issue the library's calls for one device from one stream at a time.
 */
#ifndef DISTRIFUSION_H
#define DISTRIFUSION_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { DF_F32 = 0, DF_BF16 = 1 };

enum {
  DF_OK = 0,
  DF_EINVAL = -1, /* null pointer, bad enum value, misaligned pointer */
  DF_ESHAPE = -2, /* shape the kernels do not support (H % N, C % G, head dim, ...) */
  DF_EHIP = -3,   /* a HIP runtime call or launch failed */
  DF_ENOMEM = -4  /* scratch or workspace too small / allocation failed */
};

/* GroupNorm statistic modes (Section 4, Corrected asynchronous GroupNorm; Section 5.3, GroupNorm) */
enum {
  DF_GN_SUMS = 0,     /* statistics of the scatter output: fresh own sums + stale sums of the other patches */
  DF_GN_EQ2 = 1,      /* Eq. 2 as printed, with the negative-variance fallback to the fresh local variance */
  DF_GN_SEPARATE = 2, /* fresh patch only ("Separate GN") */
  DF_GN_STALE = 3     /* stale global statistics only ("Stale GN") */
};

enum { DF_MODE_FULL = 0, DF_MODE_DISPLACED = 1 };

/* Direction of the patch split.  Rows: N horizontal strips of H/N rows (the default of every entry point without a
 * split_axis argument).  Columns: N vertical strips of W/N columns (Section 5.1, Baselines: the naive patch split
 * alternates between the two; nothing in Section 4 depends on the direction). */
enum { DF_SPLIT_ROWS = 0, DF_SPLIT_COLS = 1 };

const char* df_strerror(int err);

/*
 * Stale-buffer refresh (Section 4: after a layer's fresh activation is known it
 * replaces this patch's region of the full-shape buffer that the next step will
 * read as stale; on several devices this is the local part of the AllGather).
 *   dst_full  [B, full_elems_per_batch]   full-shape buffer (modified: rows of the patch only)
 *   src_patch [B, full_elems_per_batch/N] the fresh patch
 * Copies src_patch[b] to dst_full[b] at element offset patch_idx * full/N.
 * full_elems_per_batch % N must be 0.  Source and destination must not overlap.
 */
int df_buffer_refresh(void* dst_full, const void* src_patch, int B, long long full_elems_per_batch,
                      int patch_idx, int N, int dtype, void* stream);

/*
 * Corrected asynchronous GroupNorm of one patch (Section 4, Eq. 2).
 *   x_fresh         [B, R, W, C]  fresh patch
 *   y               [B, R, W, C]  normalised output, same dtype
 *   stale_stats     [N, B, G, 2]  float: per patch (sum, sum of squares) cached from the previous step
 *   fresh_stats_out [B, G, 2]     float: this patch's fresh (sum, sum of squares); may be NULL.
 *                                 May point at stale_stats + patch_idx*B*G*2 to refresh in place.
 *   gamma, beta     [C]           float
 * Statistics are combined according to stat_mode (DF_GN_*), variance is biased,
 * y = (x - mean) * rsqrt(var + eps) * gamma + beta, then SiLU if fuse_silu.
 * C % G == 0; C % 8 == 0 (bf16) or C % 4 == 0 (f32).
 */
int df_groupnorm_stale(const void* x_fresh, void* y, const float* stale_stats, float* fresh_stats_out,
                       const float* gamma, const float* beta, int B, int R, int W, int C, int G,
                       int patch_idx, int N, float eps, int stat_mode, int fuse_silu, int dtype, void* stream);

/*
 * df_groupnorm_stale for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same kernels, same results, but the statistics pass keeps
 * its partial sums in a fixed array of DF_NOALLOC_SCRATCH_BYTES that is part of the library's device image (every GPU
 * the library runs on holds it until the process ends) instead of the library's allocated scratch.  The call never
 * allocates or frees.  Shapes whose partial sums do not fit (roughly B * G > 1000) return DF_ENOMEM and launch nothing.
 * All calls on one GPU share the array: calls that overlap on one GPU (different streams) race; issue them from
 * one stream at a time.  The array keeps the previous call's contents; nothing in it has to start at zero.
 */
#define DF_NOALLOC_SCRATCH_BYTES (2u << 20)
int df_groupnorm_stale_noalloc(const void* x_fresh, void* y, const float* stale_stats, float* fresh_stats_out,
                               const float* gamma, const float* beta, int B, int R, int W, int C, int G,
                               int patch_idx, int N, float eps, int stat_mode, int fuse_silu, int dtype, void* stream);

/*
 * Sparse 3x3 convolution of one patch (Section 4, Sparse operations; Section 5.3:
 * only the rows at the patch boundary come from other patches).
 *   x_fresh    [B, R, W, Cin]      fresh input rows s..e-1, R = H/N, s = patch_idx*R
 *   stale_full [B, H, W, Cin]      stale full-shape input; only rows s-1 and e are read
 *                                  (zero beyond the image).  May be NULL when N == 1.
 *   w          [Cout, 3, 3, Cin]   dtype
 *   bias       [Cout] float, may be NULL
 *   y          [B, R/stride, W/stride, Cout]
 * Zero padding 1; stride 1 or 2 (then R and W must be even; only the row above
 * the patch is needed).  act: 0 none, 1 SiLU.
 */
int df_conv3x3_halo(const void* x_fresh, const void* stale_full, const void* w, const float* bias, void* y,
                    int B, int H, int W, int Cin, int Cout, int patch_idx, int N, int stride, int act,
                    int dtype, void* stream);

/*
 * Self-attention as cross-attention of the fresh queries against the whole
 * feature map (Section 4, Sparse operations): keys/values of the patch's own
 * token rows [patch_idx*Lq, (patch_idx+1)*Lq) are read from k_fresh/v_fresh, all
 * other rows from the stale buffers.  Lq = L / N.
 *   q, k_fresh, v_fresh [B, Lq, heads*d]
 *   k_stale, v_stale    [B, L,  heads*d]   may be NULL when N == 1
 *   out                 [B, Lq, heads*d]
 * out = softmax(q k^T * scale) v per head, no mask.  d is 64 for DF_BF16, 32
 * or 64 for DF_F32.  scale must be positive and finite (DF_EINVAL otherwise).
 * Returns DF_ESHAPE for heads*d >= 2^24 (row offsets inside a key tile are
 * 32-bit), when B * (key-range splits) exceeds 65535 and when B*heads*Lq >= 2^27.
 */
int df_attn_displaced(const void* q, const void* k_fresh, const void* v_fresh, const void* k_stale,
                      const void* v_stale, void* out, int B, int L, int heads, int d, int patch_idx, int N,
                      float scale, int dtype, void* stream);

/*
 * The three spatially mixing operations for either split direction (Section 4; Section 5.1, Baselines).  With
 * DF_SPLIT_ROWS they are df_buffer_refresh / df_conv3x3_halo / df_attn_displaced.  With DF_SPLIT_COLS patch i owns
 * columns [i*W/N, (i+1)*W/N) of every row (W % N == 0):
 *   df_conv3x3_halo_axis   x_fresh [B, H, W/N, Cin], stale_full [B, H, W, Cin] (only columns s-1 and e are read; zero
 *                          beyond the image), y [B, H/stride, (W/N)/stride, Cout]; stride 2 needs H and W/N even.
 *   df_attn_displaced_axis tokens are the pixels of an H x W grid in row-major order; q, k_fresh, v_fresh
 *                          [B, H*(W/N), heads*d] hold the strip's tokens in row-major order, k_stale, v_stale
 *                          [B, H*W, heads*d]; key (r, c) is taken from the fresh tensors iff c lies in the strip.
 *   df_buffer_refresh_axis dst_full [B, H, row_elems] (row_elems = W * channels), src_patch [B, H, row_elems/N]: every
 *                          row of the full buffer receives the strip's part of that row.
 * df_groupnorm_stale needs no direction: it only sees the patch's values and the per-patch sums.
 */
int df_buffer_refresh_axis(void* dst_full, const void* src_patch, int B, int H, long long row_elems, int patch_idx,
                           int N, int dtype, int split_axis, void* stream);
int df_conv3x3_halo_axis(const void* x_fresh, const void* stale_full, const void* w, const float* bias, void* y, int B,
                         int H, int W, int Cin, int Cout, int patch_idx, int N, int stride, int act, int dtype,
                         int split_axis, void* stream);
int df_attn_displaced_axis(const void* q, const void* k_fresh, const void* v_fresh, const void* k_stale,
                           const void* v_stale, void* out, int B, int H, int W, int heads, int d, int patch_idx, int N,
                           float scale, int dtype, int split_axis, void* stream);

/*
 * Linear layer on the fresh tokens (Section 4, Sparse operations: linear layers run on the fresh region only
 * and need no data of other patches).  y[M,N] = x[M,K] w[N,K]^T + bias[N] + residual[M,N].
 *   x, w bf16; bias, residual float or NULL; y bf16 or float (out_dtype); residual may alias y when y is float.
 * K % 32 == 0.
 */
int df_linear(const void* x, const void* w, const float* bias, const float* residual, void* y, int M, int N, int K,
              int out_dtype, void* stream);

/*
 * The same linear layer on operands stored in the order the matrix instructions consume them (the layout the UNet
 * step uses internally between the layers of a transformer block; Section 4, Sparse operations).
 * Packed layout of a [R, K] bf16 matrix, K % 16 == 0: fragments [ceil(R/32)][K/16][64][8]; slot l of fragment
 * (rt, kf) holds row rt*32 + l%32, columns kf*16 + 8*(l/32) .. +7; rows beyond R are zero.  df_packed_bytes gives
 * the size.  Packed weights use the same layout with in-fragment row i holding matrix row rt*32 + sigma(i), sigma
 * swapping bits 2 and 3 of i, and may be scaled per column by gamma[K] (LayerNorm scale folded in) before rounding.
 *   df_pack_rows           x [M, K] bf16 row-major -> packed
 *   df_pack_linear_weight  w [N, K] bf16 row-major (N % 32 == 0) -> packed; gamma may be NULL
 *   df_linear_packed       y = x w^T + bias (+ residual), K % 64 == 0, N % 32 == 0.
 *     ln_s, ln_t non-NULL (then bias must be NULL): LayerNorm folded into the layer, y = rstd*(acc - mean*ln_s) +
 *     ln_t with mean / rstd of each row of x over K computed by the kernel, ln_s[n] = sum_k w'[n,k] (w' the scaled,
 *     rounded weights), ln_t[n] = sum_k w[n,k] beta[k] + bias[n].
 *     geglu != 0: w holds N/2 value rows then N/2 gate rows; y [M, N/2] = value * gelu(gate).
 *     Outputs (any subset, at least one): y_f32 row-major float (residual may alias it), y_packed packed bf16 (all
 *     ceil(M/32)*32 rows are written), y_rows row-major bf16.
 */
size_t df_packed_bytes(long long rows, long long K);
int df_pack_rows(const void* x, void* packed, int M, int K, void* stream);
int df_pack_linear_weight(const void* w, const float* gamma, void* packed, int N, int K, void* stream);
int df_linear_packed(const void* xp, const void* wp, const float* bias, const float* ln_s, const float* ln_t,
                     float ln_eps, const float* residual, float* y_f32, void* y_packed, void* y_rows, int M, int N,
                     int K, int geglu, void* stream);

/*
 * The two attention forms the UNet step runs internally, exposed for tests and measurements.
 *
 * df_attn_stale_vt: self-attention of Lq query rows against L key rows when every key already sits in the (refreshed)
 * stale buffers and the values are stored transposed (Section 4: the patch's own K / V rows are written into the
 * buffers by the projection, so no splice is left for the attention kernel).  q [B, Lq, heads*64], k [B, L, heads*64],
 * vt [B, heads*64, vt_ld] with vt[b][c][j] = v[b][j][c], vt_ld >= L rounded up to a multiple of 64 (columns beyond L
 * are never used); out [B, Lq, heads*64] row-major, or fragment-packed (rows = B*Lq; the padding rows of the last
 * fragment row are left untouched) if out_packed.  bf16, d = 64.  DF_ESHAPE for heads*64 >= 2^23 or vt_ld >= 2^25
 * (32-bit offsets inside a tile), DF_EINVAL for vt_ld % 8 != 0 or vt_ld below L rounded up to 64.
 *
 * df_cross_attn_packed: cross-attention to the text tokens fused into its query projection (Section 4: per-token
 * layers need no data of other patches).  out = softmax(q k^T * scale) v per head with q = LayerNorm(x) wq^T, the
 * norm folded as in df_linear_packed (ln_s, ln_t).  x and out are fragment-packed [B*rows_per_batch, C]; wq_packed
 * from df_pack_linear_weight; text_kv_packed from df_pack_text_kv, which re-lays the projected text keys / values
 * kv [B*text_len, count*2C] (per block C key columns then C value columns, row-major bf16) of `count` blocks as MFMA
 * fragments; `block` selects one.  text_len <= 128; rows_per_batch % 32 == 0 unless B == 1; C % 64 == 0.
 */
int df_attn_stale_vt(const void* q, const void* k, const void* vt, void* out, int B, int Lq, int L, int heads,
                     long long vt_ld, float scale, int out_packed, void* stream);
size_t df_packed_text_kv_bytes(int B, int text_len, int count, int C);
int df_pack_text_kv(const void* kv, void* packed, int B, int text_len, int count, int C, void* stream);
int df_cross_attn_packed(const void* xp, const void* wq_packed, const float* ln_s, const float* ln_t, float ln_eps,
                         const void* text_kv_packed, void* out_packed, int B, int rows_per_batch, int C, int text_len,
                         int count, int block, float scale, void* stream);

/* ---- whole UNet step --------------------------------------------------------------------- */

typedef struct df_unet_cfg {
  int H, W;          /* full latent size */
  int N;             /* number of row patches */
  int B;             /* batch */
  int in_ch;         /* latent channels */
  int n_levels;      /* <= 4 */
  int levels[4];     /* channels per level */
  int depths[4];     /* transformer depth per level (0: no attention) */
  int head_dim;      /* 64 */
  int groups;        /* GroupNorm groups */
  int emb_dim;       /* width of the conditioning embedding vector */
  int text_len, text_dim;
  int res_per_level; /* residual blocks per down level (up levels have one more) */
  int split_axis;    /* DF_SPLIT_ROWS (0): N strips of H/N rows; DF_SPLIT_COLS: N strips of W/N columns, then a
                        DISPLACED step takes x [B, H, W/N, in_ch] and the boundary state of a convolution holds the
                        first and last column of every patch, [B, N, 2, rows, Cin] */
} df_unet_cfg;

typedef struct df_unet df_unet;

/* Parameter list the plan expects, in order.  Matrices and conv kernels (ndim 2 or 4) are bf16,
 * vectors (ndim 1) are float.  Returns the count / fills one entry; DF_EINVAL if idx is out of range. */
int df_unet_num_weights(const df_unet_cfg* cfg);
int df_unet_weight_info(const df_unet_cfg* cfg, int idx, char* name, int name_cap, int* ndim, long long dims[4]);

/* Bytes of device workspace (activations of one step in either mode) and of the stale-state blob. */
size_t df_unet_workspace_bytes(const df_unet_cfg* cfg);
size_t df_unet_stale_bytes(const df_unet_cfg* cfg);

/* Builds the execution plan.  `weights[i]` are device pointers in df_unet_weight_info order and must
 * outlive the plan; `workspace` is device memory of at least df_unet_workspace_bytes, 256-byte aligned. */
int df_unet_create(df_unet** out, const df_unet_cfg* cfg, const void* const* weights, int n_weights,
                   void* workspace, size_t workspace_bytes);
void df_unet_destroy(df_unet* u);

/* Location of one named stale buffer inside the blob (tests and tools).  Names: "<conv>.in" (boundary
 * rows [B, N, 2, W, Cin] bf16: first and last input row of every patch; for vertical strips the first and last input
 * column, [B, N, 2, rows, Cin]), "<attn>.k" ([B, L, C] bf16),
 * "<attn>.v" (values stored transposed, [B, C, Lp] bf16 with Lp = L rounded up to a multiple of 64 - the key index
 * is contiguous so that the attention kernel streams V^T tiles; columns L .. Lp-1 are never written and never
 * contribute; layers whose width is not a multiple of 64 or is below 128 keep [B, L, C]),
 * "<gn>.stats" ([N, B, G, 2] float). */
int df_unet_stale_lookup(const df_unet* u, const char* name, size_t* offset, size_t* bytes);
int df_unet_num_stale(const df_unet* u);
int df_unet_stale_name(const df_unet* u, int idx, char* name, int name_cap);

/*
 * One UNet forward for one patch (Section 4; Section 3, Eq. 1: eps = eps_theta(x_t, t, c)).
 *   mode DF_MODE_FULL       x [B, H, W, in_ch] float: the synchronous first step on the whole image;
 *                           fills every stale buffer.  patch_idx is ignored.
 *   mode DF_MODE_DISPLACED  x [B, H/N, W, in_ch] float ([B, H, W/N, in_ch] for vertical strips): patch `patch_idx` with stale context; if
 *                           `refresh`, the patch's own rows of every stale buffer are overwritten.
 *   emb [B, emb_dim] float, text [B, text_len, text_dim] bf16, stale: blob of df_unet_stale_bytes,
 *   eps_out: float, same shape as x.
 */
int df_patch_unet_step(df_unet* u, const void* x, const void* emb, const void* text, void* stale,
                       void* eps_out, int patch_idx, int mode, int refresh, void* stream);

/*
 * GroupNorm statistic mode of the DISPLACED steps (Section 4, Eq. 2; Section 5.3 compares the corrected
 * asynchronous GroupNorm with "Separate GN" and "Stale GN"): one of DF_GN_*, default DF_GN_SUMS.  FULL steps always
 * use the exact statistics of the whole image.  Warm-up steps (Section 4: a few synchronous steps before the
 * displaced ones) need no entry point of their own: the caller runs DF_MODE_FULL for them.
 */
int df_unet_set_gn_mode(df_unet* u, int stat_mode);

/*
 * df_patch_unet_step records the launches of a step into a HIP graph the second time it sees the same call (mode,
 * patch, refresh, stream and all pointers equal) and replays the graph from then on (Section 5.1 uses CUDAGraph for
 * the same purpose).  Calls on the legacy default stream (stream == 0) and calls made while per-launch timing is on
 * always launch eagerly.  df_unet_set_graph(u, 0) switches the graph path off.
 */
int df_unet_set_graph(df_unet* u, int on);

/*
 * Optional per-launch timing of df_patch_unet_step (measurement support; Section 5.1 times whole runs, this
 * splits a step by kernel class).  While enabled, every kernel launch of a step is bracketed by two events on
 * the step's stream, which slows the step down; totals accumulate per class until reset.
 * df_unet_profile_read synchronises the device, then returns the class totals: elapsed ms, algorithmic flops,
 * algorithmic bytes and launch count.  Classes: 0 .. df_unet_profile_num_classes()-1, named by
 * df_unet_profile_class_name.
 */
int df_unet_profile_enable(df_unet* u, int on);
int df_unet_profile_reset(df_unet* u);
int df_unet_profile_num_classes(void);
const char* df_unet_profile_class_name(int cls);
int df_unet_profile_read(df_unet* u, int cls, double* ms, double* flops, double* bytes, long long* launches);
/* The same totals per kernel: one operation at one shape ("linear_packed 300x1280x1280", "self_attn 300x2400x1280",
 * ...), i.e. launches of one kernel instantiation with one grid.  df_unet_profile_num_kernels synchronises the device
 * and returns how many distinct kernels the profiled steps launched (or a negative error); df_unet_profile_kernel
 * fills one entry: its label, class and totals. */
int df_unet_profile_num_kernels(df_unet* u);
int df_unet_profile_kernel(df_unet* u, int idx, char* label, int label_cap, int* cls, double* ms, double* flops,
                           double* bytes, long long* launches);

/* Sampler update on the patch's latent rows (Section 3, Eq. 1; Euler step): x += (sigma_next - sigma) * eps. */
int df_euler_update(float* x, const float* eps, float sigma, float sigma_next, long long n, void* stream);

/* Input scaling of the noise predictor on the sigma ladder of the Euler sampler (Section 3, Eq. 1: the model is
 * evaluated on the current noisy latent): y = x / sqrt(sigma^2 + 1).  y may alias x. */
int df_scale_input(float* y, const float* x, float sigma, long long n, void* stream);

/* Measurement support: `blocks` workgroups of four waves each issue `iters` x 4 register-resident bf16 MFMAs
 * (32x32x16, four independent accumulators); *flops receives the operation count.  `out` needs `blocks` floats and
 * is not written.  The achieved rate is the matrix-pipe ceiling the kernels are compared with besides the nominal one. */
int df_mfma_probe(float* out, int blocks, int iters, double* flops, void* stream);

/* Measurement support: the cost of making every workgroup wait for all others, which decides between one launch per
 * layer and a persistent kernel for the step (Section 5.1 removes launch overhead with CUDAGraph; this is the
 * measurement behind this build's choice of graph-replayed separate launches).  `iters` dependent phases over `blocks`
 * workgroups (34 <= blocks <= number of compute units), each phase = write 1 KB per workgroup, then read what another
 * workgroup wrote: mode 0 one kernel per phase, mode 1 one kernel with a fenced counter barrier per phase, mode 2 one
 * kernel exchanging 32 tagged words per workgroup through relaxed device-scope atomics (no fences).  Every wait is
 * bounded.  `buf`: df_sync_probe_bytes(blocks) bytes of device memory, 256-byte aligned, zero before the first call;
 * its first word is non-zero afterwards if a wait ran out (1) or a value arrived wrong (2).  Time it with events. */
size_t df_sync_probe_bytes(int blocks);
int df_sync_probe(void* buf, int blocks, int iters, int mode, void* stream);

/* Plain device-to-device copy of `bytes` bytes with the refresh kernel (bandwidth calibration). */
int df_copy_bytes(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
