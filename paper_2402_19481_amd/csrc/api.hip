// C ABI of the layer operations: argument validation and translation into the
// internal launch structures.  No arithmetic happens here.
#include <mutex>

#include "kernels.h"

namespace df {

namespace {
struct DevScratch {
  void* ptr = nullptr;
  size_t bytes = 0;
};
DevScratch g_scratch[64];
std::mutex g_scratch_mu;
}  // namespace

int scratch_init(const Scratch& s) {
  if (!s.ptr || s.bytes < kScratchCounterBytes) return DF_ENOMEM;
  if (hipMemset(s.ptr, 0, kScratchCounterBytes) != hipSuccess || hipDeviceSynchronize() != hipSuccess) return DF_EHIP;
  return DF_OK;
}

// The per-device region of the per-operation entry points.  It only ever grows, and growing never frees: the
// previous buffer stays allocated (and its reserved head stays zero) until the process ends, because launches that
// are still queued, and graphs a caller captured around these entry points, hold its address.  Sizes double, so all
// retired buffers together are smaller than the live one.  The allocation must not happen while the calling stream
// is being captured; capture a call only after an eager call of the same shape.
char* scratch_region(const Scratch* given, size_t bytes) {
  if (given) return (given->ptr && given->bytes >= bytes) ? given->ptr : nullptr;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  DevScratch& s = g_scratch[dev];
  if (s.bytes >= bytes) return (char*)s.ptr;
  size_t want = s.bytes ? s.bytes * 2 : (size_t)8 << 20;
  if (want < bytes) want = bytes;
  want = (want + 255) / 256 * 256;
  void* p = nullptr;
  if (hipMalloc(&p, want) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  if (hipMemset(p, 0, kScratchCounterBytes) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
    (void)hipFree(p);                       // never handed out: nothing can hold its address
    return nullptr;
  }
  s.ptr = p;                                // the previous buffer is retired, not freed
  s.bytes = want;
  return (char*)p;
}

}  // namespace df

using namespace df;

static inline bool bad_dtype(int dt) { return dt != DF_F32 && dt != DF_BF16; }
static inline size_t esize(int dt) { return dt == DF_BF16 ? 2 : 4; }

extern "C" {
#pragma GCC visibility push(default)

const char* df_strerror(int err) {
  switch (err) {
    case DF_OK: return "ok";
    case DF_EINVAL: return "invalid argument (null or misaligned pointer, bad enum)";
    case DF_ESHAPE: return "unsupported shape";
    case DF_EHIP: return "HIP runtime error";
    case DF_ENOMEM: return "out of device scratch or workspace";
    default: return "unknown error";
  }
}

int df_copy_bytes(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return DF_EINVAL;
  return launch_copy_rows(dst, src, 1, (long long)bytes, (long long)bytes, (long long)bytes, (hipStream_t)stream);
}

int df_buffer_refresh(void* dst_full, const void* src_patch, int B, long long full_elems_per_batch, int patch_idx,
                      int N, int dtype, void* stream) {
  if (!dst_full || !src_patch || bad_dtype(dtype)) return DF_EINVAL;
  if (B <= 0 || N <= 0 || full_elems_per_batch < 0 || full_elems_per_batch % N) return DF_ESHAPE;
  if (patch_idx < 0 || patch_idx >= N) return DF_ESHAPE;
  const long long chunk = full_elems_per_batch / N * (long long)esize(dtype);
  const long long full = full_elems_per_batch * (long long)esize(dtype);
  char* dst = (char*)dst_full + (long long)patch_idx * chunk;
  return launch_copy_rows(dst, src_patch, B, chunk, full, chunk, (hipStream_t)stream);
}

int df_groupnorm_stale(const void* x_fresh, void* y, const float* stale_stats, float* fresh_stats_out,
                       const float* gamma, const float* beta, int B, int R, int W, int C, int G, int patch_idx, int N,
                       float eps, int stat_mode, int fuse_silu, int dtype, void* stream) {
  return groupnorm_entry(x_fresh, y, stale_stats, fresh_stats_out, gamma, beta, B, R, W, C, G, patch_idx, N, eps,
                         stat_mode, fuse_silu, dtype, nullptr, (hipStream_t)stream);
}

int df_conv3x3_halo_axis(const void* x_fresh, const void* stale_full, const void* w, const float* bias, void* y, int B,
                         int H, int W, int Cin, int Cout, int patch_idx, int N, int stride, int act, int dtype,
                         int split_axis, void* stream) {
  if (!x_fresh || !w || !y || bad_dtype(dtype)) return DF_EINVAL;
  if (act != 0 && act != 1) return DF_EINVAL;
  if (split_axis != DF_SPLIT_ROWS && split_axis != DF_SPLIT_COLS) return DF_EINVAL;
  if (B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || N <= 0) return DF_ESHAPE;
  if ((split_axis == DF_SPLIT_ROWS ? H : W) % N) return DF_ESHAPE;
  if (patch_idx < 0 || patch_idx >= N) return DF_ESHAPE;
  if (N > 1 && !stale_full) return DF_EINVAL;
  const long long row = (long long)W * Cin;
  const size_t es = esize(dtype);
  ConvArgs a = {};
  a.x = x_fresh; a.w = w; a.bias = bias; a.y = y;
  a.B = B; a.Cin = Cin; a.Cout = Cout; a.stride = stride; a.act = act;
  a.dtype = dtype; a.out_dtype = dtype;
  if (split_axis == DF_SPLIT_ROWS) {
    const int R = H / N;
    a.R = R; a.W = W;
    a.halo_bstride = (long long)H * row;
    const int s = patch_idx * R, e = s + R;
    a.halo_top = (s > 0) ? (const char*)stale_full + (size_t)(s - 1) * row * es : nullptr;
    a.halo_bot = (e < H && stride == 1) ? (const char*)stale_full + (size_t)e * row * es : nullptr;
  } else {
    // vertical strip: the patch has all H rows and W/N columns; the stale buffer supplies column s-1 and column e
    const int Wp = W / N;
    a.R = H; a.W = Wp;
    const int s = patch_idx * Wp, e = s + Wp;
    a.side_bstride = (long long)H * row;
    a.side_rstride = row;
    a.halo_left = (s > 0) ? (const char*)stale_full + (size_t)(s - 1) * Cin * es : nullptr;
    a.halo_right = (e < W && stride == 1) ? (const char*)stale_full + (size_t)e * Cin * es : nullptr;
  }
  return launch_conv3x3(a, (hipStream_t)stream);
}

int df_conv3x3_halo(const void* x_fresh, const void* stale_full, const void* w, const float* bias, void* y, int B,
                    int H, int W, int Cin, int Cout, int patch_idx, int N, int stride, int act, int dtype,
                    void* stream) {
  return df_conv3x3_halo_axis(x_fresh, stale_full, w, bias, y, B, H, W, Cin, Cout, patch_idx, N, stride, act, dtype,
                              DF_SPLIT_ROWS, stream);
}

int df_attn_displaced_axis(const void* q, const void* k_fresh, const void* v_fresh, const void* k_stale,
                           const void* v_stale, void* out, int B, int H, int W, int heads, int d, int patch_idx, int N,
                           float scale, int dtype, int split_axis, void* stream) {
  if (!q || !k_fresh || !v_fresh || !out || bad_dtype(dtype)) return DF_EINVAL;
  if (split_axis != DF_SPLIT_ROWS && split_axis != DF_SPLIT_COLS) return DF_EINVAL;
  if (B <= 0 || H <= 0 || W <= 0 || heads <= 0 || d <= 0 || N <= 0) return DF_ESHAPE;
  if ((long long)H * W > 0x7fffffffLL || (split_axis == DF_SPLIT_ROWS ? ((long long)H * W) % N : W % N)) return DF_ESHAPE;
  if (patch_idx < 0 || patch_idx >= N) return DF_ESHAPE;
  if (N > 1 && (!k_stale || !v_stale)) return DF_EINVAL;
  const int L = H * W, Lq = L / N;
  const long long C = (long long)heads * d;
  AttnArgs a = {};
  a.q = q; a.k_fresh = k_fresh; a.v_fresh = v_fresh; a.k_stale = k_stale; a.v_stale = v_stale; a.out = out;
  a.B = B; a.Lq = Lq; a.L = L; a.heads = heads; a.d = d;
  if (split_axis == DF_SPLIT_ROWS) {
    a.own_lo = patch_idx * Lq; a.own_n = Lq;           // a block of consecutive tokens
  } else {
    a.own_period = W; a.own_n = W / N; a.own_lo = patch_idx * a.own_n;   // W/N tokens of every grid row
  }
  a.ldq = a.ldkf = a.ldvf = a.ldks = a.ldvs = a.ldo = C;
  a.bsq = a.bskf = a.bsvf = a.bso = (long long)Lq * C;
  a.bsks = a.bsvs = (long long)L * C;
  a.scale = scale; a.dtype = dtype;
  return launch_attention(a, (hipStream_t)stream);
}

int df_attn_displaced(const void* q, const void* k_fresh, const void* v_fresh, const void* k_stale,
                      const void* v_stale, void* out, int B, int L, int heads, int d, int patch_idx, int N,
                      float scale, int dtype, void* stream) {
  if (L <= 0) return (!q || !k_fresh || !v_fresh || !out || bad_dtype(dtype)) ? DF_EINVAL : DF_ESHAPE;
  return df_attn_displaced_axis(q, k_fresh, v_fresh, k_stale, v_stale, out, B, 1, L, heads, d, patch_idx, N, scale,
                                dtype, DF_SPLIT_ROWS, stream);
}

int df_buffer_refresh_axis(void* dst_full, const void* src_patch, int B, int H, long long row_elems, int patch_idx,
                           int N, int dtype, int split_axis, void* stream) {
  if (!dst_full || !src_patch || bad_dtype(dtype)) return DF_EINVAL;
  if (split_axis != DF_SPLIT_ROWS && split_axis != DF_SPLIT_COLS) return DF_EINVAL;
  if (B <= 0 || H <= 0 || N <= 0 || row_elems < 0 || patch_idx < 0 || patch_idx >= N) return DF_ESHAPE;
  if (split_axis == DF_SPLIT_ROWS) {
    if (H % N) return DF_ESHAPE;
    return df_buffer_refresh(dst_full, src_patch, B, (long long)H * row_elems, patch_idx, N, dtype, stream);
  }
  if (row_elems % N) return DF_ESHAPE;
  // every row of the full buffer receives the patch's part of that row: B*H pieces of row_elems/N elements
  const long long piece = row_elems / N * (long long)esize(dtype), full = row_elems * (long long)esize(dtype);
  return launch_copy_rows((char*)dst_full + (long long)patch_idx * piece, src_patch, (long long)B * H, piece, full,
                          piece, (hipStream_t)stream);
}

int df_attn_stale_vt(const void* q, const void* k, const void* vt, void* out, int B, int Lq, int L, int heads,
                     long long vt_ld, float scale, int out_packed, void* stream) {
  if (!q || !k || !vt || !out) return DF_EINVAL;
  if (B <= 0 || Lq <= 0 || L <= 0 || heads <= 0) return DF_ESHAPE;
  const long long C = (long long)heads * 64;
  AttnArgs a = {};
  a.q = q; a.k_fresh = k; a.v_fresh = vt; a.k_stale = k; a.v_stale = vt; a.out = out;
  a.B = B; a.Lq = Lq; a.L = L; a.heads = heads; a.d = 64; a.own_lo = 0; a.own_n = 0;
  a.ldq = a.ldkf = a.ldvf = a.ldks = a.ldvs = a.ldo = C;
  a.bsq = a.bso = (long long)Lq * C; a.bskf = a.bsvf = a.bsks = (long long)L * C; a.bsvs = C * vt_ld;
  a.v_transposed = 1; a.vt_ld = vt_ld; a.out_packed = out_packed ? 1 : 0;
  a.scale = scale; a.dtype = DF_BF16;
  return launch_attention(a, (hipStream_t)stream);
}

size_t df_packed_text_kv_bytes(int B, int text_len, int count, int C) {
  return (B > 0 && text_len > 0 && count > 0 && C > 0 && C % 64 == 0) ? packed_text_kv_bytes(B, text_len, count, C) : 0;
}

int df_pack_text_kv(const void* kv, void* packed, int B, int text_len, int count, int C, void* stream) {
  if (!kv || !packed) return DF_EINVAL;
  if (text_len > 128) return DF_ESHAPE;
  return launch_pack_text_kv((const bf16_t*)kv, (long long)count * 2 * C, (bf16_t*)packed, B, text_len, count, C,
                             (hipStream_t)stream);
}

int df_cross_attn_packed(const void* xp, const void* wq_packed, const float* ln_s, const float* ln_t, float ln_eps,
                         const void* text_kv_packed, void* out_packed, int B, int rows_per_batch, int C, int text_len,
                         int count, int block, float scale, void* stream) {
  if (!xp || !wq_packed || !ln_s || !ln_t || !text_kv_packed || !out_packed) return DF_EINVAL;
  if (B <= 0 || rows_per_batch <= 0 || C <= 0 || C % 64 || text_len <= 0 || text_len > 128 || block < 0 || block >= count)
    return DF_ESHAPE;
  const int XA = (text_len + 31) / 32, heads = C / 64;
  WGemmArgs a = {};
  a.Xp = xp; a.Wp = wq_packed; a.M = B * rows_per_batch; a.N = C; a.K = C;
  a.ln_s = ln_s; a.ln_t = ln_t; a.ln_eps = ln_eps; a.out_packed = out_packed;
  a.xa_kv = (const bf16_t*)text_kv_packed + (size_t)block * heads * 12 * XA * 512;
  a.xa_keys = text_len; a.xa_rows = rows_per_batch; a.xa_scale = scale;
  a.xa_bstride = (long long)count * heads * 12 * XA * 512;
  return launch_wgemm(a, (hipStream_t)stream);
}

int df_linear(const void* x, const void* w, const float* bias, const float* residual, void* y, int M, int N, int K,
              int out_dtype, void* stream) {
  if (!x || !w || !y || bad_dtype(out_dtype)) return DF_EINVAL;
  GemmArgs g = {};
  g.A = x; g.W = w; g.bias = bias; g.residual = residual; g.out = y;
  g.M = M; g.N = N; g.K = K; g.lda = K; g.ldw = K; g.ldr = N; g.ldo = N; g.act = 0; g.out_dtype = out_dtype;
  return launch_gemm_bf16(g, (hipStream_t)stream);
}

int df_mfma_probe(float* out, int blocks, int iters, double* flops, void* stream) {
  if (!out) return DF_EINVAL;
  if (flops) *flops = (double)blocks * 4.0 * iters * 4.0 * (2.0 * 32 * 32 * 16);
  return launch_mfma_probe(out, blocks, iters, (hipStream_t)stream);
}

size_t df_sync_probe_bytes(int blocks) { return blocks > 0 ? sync_probe_bytes(blocks) : 0; }

int df_sync_probe(void* buf, int blocks, int iters, int mode, void* stream) {
  if (!buf || ((uintptr_t)buf % 256)) return DF_EINVAL;
  return launch_sync_probe(buf, blocks, iters, mode, (hipStream_t)stream);
}

int df_scale_input(float* y, const float* x, float sigma, long long n, void* stream) {
  if (!x || !y) return DF_EINVAL;
  if (n < 0) return DF_ESHAPE;
  return launch_scale(y, x, 1.0f / sqrtf(sigma * sigma + 1.0f), n, (hipStream_t)stream);
}

size_t df_packed_bytes(long long rows, long long K) { return rows > 0 && K > 0 ? packed_rows_bytes(rows, K) : 0; }

int df_pack_rows(const void* x, void* packed, int M, int K, void* stream) {
  if (!x || !packed) return DF_EINVAL;
  return launch_pack_rows((const bf16_t*)x, K, (bf16_t*)packed, M, K, (hipStream_t)stream);
}

int df_pack_linear_weight(const void* w, const float* gamma, void* packed, int N, int K, void* stream) {
  if (!w || !packed) return DF_EINVAL;
  return launch_pack_wfrag((const bf16_t*)w, gamma, (bf16_t*)packed, N, K, (hipStream_t)stream);
}

int df_linear_packed(const void* xp, const void* wp, const float* bias, const float* ln_s, const float* ln_t,
                     float ln_eps, const float* residual, float* y_f32, void* y_packed, void* y_rows, int M, int N,
                     int K, int geglu, void* stream) {
  if (!xp || !wp || (!y_f32 && !y_packed && !y_rows)) return DF_EINVAL;
  if (geglu && N % 2) return DF_ESHAPE;
  const int Nout = geglu ? N / 2 : N;
  WGemmArgs a = {};
  a.Xp = xp; a.Wp = wp; a.M = M; a.N = N; a.K = K; a.bias = bias; a.ln_s = ln_s; a.ln_t = ln_t; a.ln_eps = ln_eps;
  a.residual = residual; a.ldr = Nout; a.out_f32 = y_f32; a.ldo = Nout; a.out_packed = y_packed; a.out_rows = y_rows;
  a.ld_rows = Nout; a.geglu = geglu ? Nout : 0;
  return launch_wgemm(a, (hipStream_t)stream);
}

int df_euler_update(float* x, const float* eps, float sigma, float sigma_next, long long n, void* stream) {
  if (!x || !eps) return DF_EINVAL;
  if (n < 0) return DF_ESHAPE;
  return launch_axpy(x, eps, sigma_next - sigma, n, (hipStream_t)stream);
}

#pragma GCC visibility pop
}  // extern "C"
