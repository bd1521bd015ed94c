// One UNet denoising step for one patch under displaced patch parallelism
// (Section 4): the plan walks the SDXL-shaped block list and enqueues the layer
// kernels.  Layers that mix space (3x3 convolutions, self-attention, GroupNorm)
// take cross-patch context from the stale-state blob; per-token layers run on
// the fresh tokens only.
//
// Stale state kept per layer (what differs from a literal full-shape copy of the
// input activation is noted):
//   convolution     the first and last input row of every patch, [B, N, 2, W, Cin]
//                   bf16 - the only rows another patch can ever read (Section 5.3)
//   self-attention  projected keys and values, [B, L, C] bf16 each; projection is
//                   per token, so projecting the scattered activation equals
//                   scattering the projections
//   GroupNorm       per-patch (sum, sum of squares), [N, B, G, 2] float
//
// FULL mode is the synchronous first step: the whole image is one fresh patch and
// every buffer is filled for all N patches.  DISPLACED computes patch i and, with
// refresh, overwrites the patch's own part of each buffer (never read by itself).
//
// Precision: matrix operands bf16, accumulation float; the residual stream
// (block outputs, transformer hidden state) stays float so that rounding does
// not accumulate over the 70 transformer blocks.
#include <cstdlib>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "kernels.h"

using namespace df;

namespace {

struct WeightSpec {
  std::string name;
  int ndim;
  long long dims[4];
};

struct BlockDesc {
  enum Kind { CONV_IN, RES, XF, PUSH, DOWN, UP, OUT } kind;
  std::string name;
  int cin = 0, cout = 0, level = 0, depth = 0;
  bool concat = false;
};

inline bool fold_ok(int C) { return C % 64 == 0 && C >= 128; }

bool cfg_ok(const df_unet_cfg* c) {
  if (!c) return false;
  if (c->n_levels < 1 || c->n_levels > 4 || c->B < 1 || c->N < 1 || c->H < 1 || c->W < 1) return false;
  if (c->head_dim != 64 || c->groups < 1 || c->groups > 64 || c->in_ch < 1 || c->res_per_level < 1) return false;
  if (c->emb_dim % 32 || c->text_dim % 32 || c->text_len < 1 || c->in_ch % 4) return false;
  const int down = 1 << (c->n_levels - 1);
  if (c->split_axis != DF_SPLIT_ROWS && c->split_axis != DF_SPLIT_COLS) return false;
  const bool cols = c->split_axis == DF_SPLIT_COLS;
  if (cols ? (c->W % (c->N * down) || c->H % down) : (c->H % (c->N * down) || c->W % down)) return false;
  for (int l = 0; l < c->n_levels; ++l) {
    const int ch = c->levels[l];
    if (ch % 64 || ch % c->groups || c->depths[l] < 0) return false;
    // a stride-2 conv needs patches with an even number of rows (columns, for vertical strips)
    if (l + 1 < c->n_levels && (((cols ? c->W : c->H) >> l) / c->N) % 2) return false;
    if (cols && c->depths[l] > 0 && !fold_ok(ch)) return false;   // narrow attention layers: horizontal strips only
  }
  return true;
}

std::vector<BlockDesc> build_blocks(const df_unet_cfg& c) {
  std::vector<BlockDesc> out;
  std::vector<int> skips;
  auto add = [&](BlockDesc::Kind k, const std::string& n, int cin, int cout, int level, int depth, bool cat) {
    BlockDesc b; b.kind = k; b.name = n; b.cin = cin; b.cout = cout; b.level = level; b.depth = depth; b.concat = cat;
    out.push_back(b);
  };
  const int nl = c.n_levels;
  int cur = c.levels[0];
  add(BlockDesc::CONV_IN, "conv_in", c.in_ch, cur, 0, 0, false);
  add(BlockDesc::PUSH, "", 0, 0, 0, 0, false);
  skips.push_back(cur);
  for (int li = 0; li < nl; ++li) {
    const int ch = c.levels[li];
    for (int j = 0; j < c.res_per_level; ++j) {
      const std::string base = "down" + std::to_string(li);
      add(BlockDesc::RES, base + ".res" + std::to_string(j), cur, ch, li, 0, false);
      cur = ch;
      if (c.depths[li] > 0) add(BlockDesc::XF, base + ".xf" + std::to_string(j), ch, ch, li, c.depths[li], false);
      add(BlockDesc::PUSH, "", 0, 0, 0, 0, false);
      skips.push_back(cur);
    }
    if (li + 1 < nl) {
      add(BlockDesc::DOWN, "down" + std::to_string(li) + ".down", cur, cur, li, 0, false);
      add(BlockDesc::PUSH, "", 0, 0, 0, 0, false);
      skips.push_back(cur);
    }
  }
  const int lm = nl - 1;
  add(BlockDesc::RES, "mid.res0", cur, cur, lm, 0, false);
  if (c.depths[lm] > 0) add(BlockDesc::XF, "mid.xf", cur, cur, lm, c.depths[lm], false);
  add(BlockDesc::RES, "mid.res1", cur, cur, lm, 0, false);
  for (int li = nl - 1; li >= 0; --li) {
    const int ch = c.levels[li];
    const std::string base = "up" + std::to_string(li);
    for (int j = 0; j < c.res_per_level + 1; ++j) {
      const int sk = skips.back();
      skips.pop_back();
      add(BlockDesc::RES, base + ".res" + std::to_string(j), cur + sk, ch, li, 0, true);
      cur = ch;
      if (c.depths[li] > 0) add(BlockDesc::XF, base + ".xf" + std::to_string(j), ch, ch, li, c.depths[li], false);
    }
    if (li > 0) add(BlockDesc::UP, base + ".up", cur, cur, li, 0, false);
  }
  add(BlockDesc::OUT, "out", cur, c.in_ch, 0, 0, false);
  return out;
}

std::vector<WeightSpec> build_weight_specs(const df_unet_cfg& c) {
  std::vector<WeightSpec> s;
  auto vec = [&](const std::string& n, long long d) { s.push_back({n, 1, {d, 0, 0, 0}}); };
  auto conv = [&](const std::string& n, int cin, int cout) {
    s.push_back({n + ".w", 4, {cout, 3, 3, cin}});
    vec(n + ".b", cout);
  };
  auto norm = [&](const std::string& n, int ch) { vec(n + ".g", ch); vec(n + ".beta", ch); };
  auto lin = [&](const std::string& n, int cin, int cout, bool bias) {
    s.push_back({n + ".w", 2, {cout, cin, 0, 0}});
    if (bias) vec(n + ".b", cout);
  };
  for (const BlockDesc& b : build_blocks(c)) {
    switch (b.kind) {
      case BlockDesc::CONV_IN: conv(b.name, b.cin, b.cout); break;
      case BlockDesc::RES:
        norm(b.name + ".gn1", b.cin);
        conv(b.name + ".conv1", b.cin, b.cout);
        lin(b.name + ".emb", c.emb_dim, b.cout, true);
        norm(b.name + ".gn2", b.cout);
        conv(b.name + ".conv2", b.cout, b.cout);
        if (b.cin != b.cout) lin(b.name + ".sc", b.cin, b.cout, true);
        break;
      case BlockDesc::XF: {
        const int ch = b.cin;
        norm(b.name + ".gn", ch);
        lin(b.name + ".pin", ch, ch, true);
        for (int d = 0; d < b.depth; ++d) {
          const std::string p = b.name + ".b" + std::to_string(d);
          norm(p + ".ln1", ch);
          lin(p + ".attn1.qkv", ch, 3 * ch, false);
          lin(p + ".attn1.o", ch, ch, true);
          norm(p + ".ln2", ch);
          lin(p + ".attn2.q", ch, ch, false);
          lin(p + ".attn2.kv", c.text_dim, 2 * ch, false);
          lin(p + ".attn2.o", ch, ch, true);
          norm(p + ".ln3", ch);
          lin(p + ".ff1", ch, 8 * ch, true);
          lin(p + ".ff2", 4 * ch, ch, true);
        }
        lin(b.name + ".pout", ch, ch, true);
        break;
      }
      case BlockDesc::DOWN:
      case BlockDesc::UP: conv(b.name, b.cin, b.cout); break;
      case BlockDesc::OUT:
        norm(b.name + ".gn", b.cin);
        conv(b.name + ".conv", b.cin, b.cout);
        break;
      case BlockDesc::PUSH: break;
    }
  }
  return s;
}

struct StaleEntry {
  std::string name;
  size_t off, bytes;
};

// A linear weight the plan keeps in the tiled layout of the pipelined GEMM, optionally with the preceding
// LayerNorm folded in (scale multiplied into the weight, shift and bias collected in `t`, column sums in `s`).
struct PackSpec {
  std::string name;   // parameter name without ".w"
  int N, K;
  std::string norm;   // name of the folded norm ("" = none)
  bool has_bias;
  size_t w_off, s_off, t_off;   // byte offsets inside the packed region (s/t only with a folded norm)
  size_t f_off;                 // the same weight in the fragment layout of the wave-level GEMM
};

// Token counts up to this use the fragment-packed transformer (wave-level GEMMs); larger ones (the synchronous first
// step on the whole image) the workgroup-tiled kernels, whose operand traffic per flop is lower.
constexpr int kFragMaxRows = 2048;
inline bool frag_path() {
  static const bool off = tune_env("DF_NO_FRAG") != nullptr;   // tuning aid
  return !off;
}

inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

// Output channels of the conditioning projections of all residual blocks, in block order: one GEMM at the start of
// the step computes them all (they depend on the embedding vector only).
inline int emb_total(const std::vector<BlockDesc>& blocks) {
  int t = 0;
  for (const BlockDesc& b : blocks)
    if (b.kind == BlockDesc::RES) t += b.cout;
  return t;
}


}  // namespace

// Optional per-launch timing: when enabled every kernel launch of a step is bracketed by two
// events on the step's stream and accounted to its class with its algorithmic flops and bytes.
enum { PC_GEMM = 0, PC_CONV, PC_SELF_ATTN, PC_CROSS_ATTN, PC_GROUPNORM, PC_REFRESH, PC_LAYERNORM, PC_ELEMENTWISE, PC_COUNT };
static const char* const kProfNames[PC_COUNT] = {"gemm", "conv3x3", "self_attn", "cross_attn", "groupnorm", "refresh",
                                                 "layernorm", "elementwise"};
struct ProfRec { int cls; double flops, bytes; int kernel; };
// totals of one kernel = one operation at one shape (the launches that share a label run the same kernel
// instantiation with the same grid)
struct ProfKernel { std::string label; int cls; double ms, flops, bytes; long long launches; };
struct Prof {
  bool on = false;
  std::vector<hipEvent_t> pool;
  std::vector<ProfRec> recs;       // launch k uses events 2k, 2k+1
  double ms[PC_COUNT] = {}, flops[PC_COUNT] = {}, bytes[PC_COUNT] = {};
  long long launches[PC_COUNT] = {};
  std::vector<ProfKernel> kernels;
  std::map<std::string, int> kernel_idx;
  int kernel_of(const std::string& label, int cls) {
    auto it = kernel_idx.find(label);
    if (it != kernel_idx.end()) return it->second;
    kernels.push_back({label, cls, 0.0, 0.0, 0.0, 0});
    kernel_idx[label] = (int)kernels.size() - 1;
    return (int)kernels.size() - 1;
  }
  bool begin(int cls, double fl, double by, hipStream_t st, const std::string& label) {
    const size_t k = recs.size();
    while (pool.size() < 2 * k + 2) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return false;
      pool.push_back(e);
    }
    recs.push_back({cls, fl, by, kernel_of(label.empty() ? std::string(kProfNames[cls]) : label, cls)});
    return hipEventRecord(pool[2 * k], st) == hipSuccess;
  }
  bool end(hipStream_t st) { return hipEventRecord(pool[2 * recs.size() - 1], st) == hipSuccess; }
  bool collect() {  // after the stream has been synchronised
    for (size_t k = 0; k < recs.size(); ++k) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, pool[2 * k], pool[2 * k + 1]) != hipSuccess) return false;
      const ProfRec& r = recs[k];
      ms[r.cls] += t; flops[r.cls] += r.flops; bytes[r.cls] += r.bytes; launches[r.cls] += 1;
      ProfKernel& pk = kernels[r.kernel];
      pk.ms += t; pk.flops += r.flops; pk.bytes += r.bytes; pk.launches += 1;
    }
    recs.clear();
    return true;
  }
  void reset() {
    for (int i = 0; i < PC_COUNT; ++i) { ms[i] = flops[i] = bytes[i] = 0; launches[i] = 0; }
    recs.clear();
    kernels.clear();
    kernel_idx.clear();
  }
  ~Prof() { for (hipEvent_t e : pool) (void)hipEventDestroy(e); }
};

struct PackedW {
  const bf16_t* w = nullptr;
  const bf16_t* f = nullptr;    // fragment layout (wgemm.hip)
  const float* s = nullptr;
  const float* t = nullptr;
};

// A step captured as a HIP graph: the ~1000 launches of a step replay from one submission, which takes the host
// out of the critical path (the counterpart of the paper's CUDAGraph use, Section 5.1).  A graph is tied to the
// mode, patch, refresh flag, stream and every pointer of the call that recorded it.
struct GraphEntry {
  int mode, patch, refresh, gn_mode;
  const void *x, *emb, *text, *eps;
  void* stale;
  hipStream_t stream;
  int calls = 0;                 // eager calls seen with this key (the first one stays eager: it may still set
                                 // function attributes, which must not happen under capture)
  hipGraphExec_t exec = nullptr;
};

struct df_unet {
  df_unet_cfg cfg;
  Prof prof;
  bool use_graph = true;
  int gn_mode = DF_GN_SUMS;      // statistic mode of the DISPLACED steps (df_unet_set_gn_mode)
  std::vector<GraphEntry> graphs;
  std::map<std::string, PackedW> packed;
  std::vector<BlockDesc> blocks;
  std::map<std::string, const void*> w;
  std::vector<StaleEntry> stale;
  std::map<std::string, int> stale_idx;
  size_t stale_bytes = 0;
  char* ws = nullptr;
  size_t ws_bytes = 0;
  // text K/V projection weights of all transformer blocks of a level, concatenated along the output dimension
  // ([count * 2C, text_dim] bf16) at the start of the workspace, so that one GEMM per level projects the text
  // for every block of the step
  size_t kv_off[4] = {0, 0, 0, 0};
  int kv_count[4] = {0, 0, 0, 0};
  size_t packed_bytes = 0;
  size_t emb_w_off = 0, emb_b_off = 0;   // concatenated conditioning-projection weights / biases
  // scratch region of the step's kernels (GroupNorm partials, split-K / split-key partials, the page of zeros): part
  // of the caller's workspace, right after the plan-owned weights, so recorded graphs hold plan-owned addresses only
  Scratch scr = {nullptr, 0};
};

namespace {

// Walks the block list.  In dry mode nothing is launched: the walk only sizes the
// workspace arena, lists the stale buffers and finds the largest scratch request.
struct Exec {
  const df_unet_cfg& c;
  const std::vector<BlockDesc>& blocks;
  const std::map<std::string, const void*>* w;
  bool dry;
  int mode, patch, refresh;
  hipStream_t st;
  char* ws;
  size_t ws_cap;
  size_t top = 0, high = 0;
  char* stale_base;
  std::vector<StaleEntry>* stale_list;          // dry: appended to; live: looked up
  const std::map<std::string, int>* stale_idx;
  size_t stale_top = 0;
  size_t scratch_need = 0;
  int err = DF_OK;
  Prof* prof = nullptr;
  const std::map<std::string, PackedW>* packed = nullptr;
  int gn_mode = DF_GN_SUMS;      // GroupNorm statistic mode of a DISPLACED step
  const Scratch* scr = nullptr;  // the plan's scratch region
  const bf16_t* kv_packed[4] = {nullptr, nullptr, nullptr, nullptr};
  int kv_count[4] = {0, 0, 0, 0};
  int kv_cursor[4] = {0, 0, 0, 0};
  bf16_t* kv2_all[4] = {nullptr, nullptr, nullptr, nullptr};
  bf16_t* xkv_all[4] = {nullptr, nullptr, nullptr, nullptr};   // text keys / values as per-head MFMA fragments
  const bf16_t* emb_w_all = nullptr;     // [sum of cout, emb_dim] conditioning projections of all residual blocks
  const float* emb_b_all = nullptr;
  float* emb_all = nullptr;              // their outputs for this step, [B, emb_n]
  int emb_n = 0, emb_cursor = 0;

  // run a launch, accounted to class `cls` when per-launch timing is on
  std::string label;             // name of the next timed launch in the per-kernel totals (consumed by timed())
  static std::string dims(std::initializer_list<long long> v) {
    std::string o;
    for (long long d : v) { if (!o.empty()) o += "x"; o += std::to_string(d); }
    return o;
  }
  template <typename F>
  void timed(int cls, double fl, double by, F&& launch) {
    if (!live()) { label.clear(); return; }
    const bool p = prof && prof->on;
    if (p && !prof->begin(cls, fl, by, st, label)) { err = DF_EHIP; return; }
    label.clear();
    run(launch());
    if (p && !prof->end(st)) err = DF_EHIP;
  }

  int B() const { return c.B; }
  int N() const { return c.N; }
  bool full() const { return mode == DF_MODE_FULL; }
  bool cols() const { return c.split_axis == DF_SPLIT_COLS; }     // patches are vertical strips
  int rows(int level) const { return (full() || cols()) ? (c.H >> level) : (c.H >> level) / c.N; }
  int width(int level) const { return (full() || !cols()) ? (c.W >> level) : (c.W >> level) / c.N; }

  void* alloc(size_t bytes) {
    bytes = align256(bytes);
    size_t at = top;
    top += bytes;
    if (top > high) high = top;
    if (!dry && top > ws_cap) { err = DF_ENOMEM; return nullptr; }
    return dry ? nullptr : ws + at;
  }
  const void* weight(const std::string& n) {
    if (dry) return nullptr;
    auto it = w->find(n);
    if (it == w->end()) { err = DF_EINVAL; return nullptr; }
    return it->second;
  }
  char* stale_buf(const std::string& n, size_t bytes) {
    if (dry) {
      stale_list->push_back({n, stale_top, bytes});
      stale_top += align256(bytes);
      return nullptr;
    }
    auto it = stale_idx->find(n);
    if (it == stale_idx->end() || (*stale_list)[it->second].bytes != bytes) { err = DF_EINVAL; return nullptr; }
    return stale_base + (*stale_list)[it->second].off;
  }
  void run(int rc) { if (err == DF_OK && rc != DF_OK) err = rc; }
  bool live() const { return !dry && err == DF_OK; }

  // ---- layers ----
  void gemm(const void* A, long long lda, const std::string& wn, bool bias, const float* residual, long long ldr,
            void* out, long long ldo, int M, int Nn, int K, int out_dtype, const GemmArgs* extra = nullptr) {
    const void* W = weight(wn + ".w");
    const float* bp = bias ? (const float*)weight(wn + ".b") : nullptr;
    gemm_w(A, lda, W, bp, residual, ldr, out, ldo, M, Nn, K, out_dtype, extra);
  }
  // GEMM on a plan-packed weight; `ln` applies the folded LayerNorm of that weight (A then holds raw rows)
  void gemm_packed(const void* A, long long lda, const std::string& wn, bool bias, bool ln, const float* residual,
                   long long ldr, void* out, long long ldo, int M, int Nn, int K, int out_dtype, void* out2,
                   const GemmArgs* extra = nullptr) {
    GemmArgs g = {};
    if (extra) g = *extra;
    const float* bp = nullptr;
    const void* W = nullptr;
    if (!dry) {
      auto it = packed->find(wn);
      if (it == packed->end()) { err = DF_EINVAL; return; }
      W = it->second.w;
      g.packed_w = 1;
      if (ln) { g.ln_s = it->second.s; g.ln_t = it->second.t; g.ln_eps = 1e-5f; }
      else if (bias) bp = (const float*)weight(wn + ".b");
      static const bool no_pack = tune_env("DF_NO_PACK") != nullptr;   // tuning aid: canonical layout where no norm is folded
      if (no_pack && !ln) { W = weight(wn + ".w"); g.packed_w = 0; }
    }
    g.out2 = out2; g.ldo2 = Nn;
    gemm_w(A, lda, W, bp, residual, ldr, out, ldo, M, Nn, K, out_dtype, &g);
  }
  void gemm_w(const void* A, long long lda, const void* W, const float* bp, const float* residual, long long ldr,
              void* out, long long ldo, int M, int Nn, int K, int out_dtype, const GemmArgs* extra = nullptr) {
    {
      const size_t need = gemm_scratch_bytes(M, Nn);
      if (need > scratch_need) scratch_need = need;
    }
    if (!live()) return;
    GemmArgs g = {};
    if (extra) g = *extra;   // epilogue variant (GEGLU / segmented output) prepared by the caller
    g.A = A; g.W = W; g.bias = bp; g.residual = residual; g.out = out;
    g.M = M; g.N = Nn; g.K = K; g.lda = lda; g.ldw = K; g.ldr = ldr; g.ldo = ldo; g.act = 0; g.out_dtype = out_dtype;
    g.scr = scr;
    const double osz = out_dtype == DF_BF16 ? 2.0 : 4.0;
    label = "linear " + dims({M, Nn, K}) + (g.geglu ? " geglu" : "") + (g.ln_s ? " ln" : "");
    timed(PC_GEMM, 2.0 * M * Nn * K, 2.0 * ((double)M * K + (double)Nn * K) + osz * M * Nn,
          [&] { return launch_gemm_bf16(g, st); });
  }

  void groupnorm(const std::string& name, const void* x, int in_dtype, int level_rows, int W, int C, float eps, int silu,
                 bf16_t* y, int y_packed = 0, bf16_t* halo_entry = nullptr) {
    // level_rows: rows of x in this mode
    const int G = c.groups;
    float* entry = (float*)stale_buf(name + ".stats", (size_t)N() * B() * G * 2 * sizeof(float));
    const size_t need = groupnorm_scratch_bytes(B(), full() ? N() : 1, G, N());
    if (need > scratch_need) scratch_need = need;
    const float* gamma = (const float*)weight(name + ".g");
    const float* beta = (const float*)weight(name + ".beta");
    if (!live()) return;
    GnArgs a = {};
    a.x = x; a.y = y; a.gamma = gamma; a.beta = beta;
    a.B = B(); a.W = W; a.C = C; a.G = G; a.eps = eps; a.silu = silu; a.in_dtype = in_dtype; a.out_dtype = DF_BF16;
    a.stat_mode = gn_mode;
    a.y_packed = y_packed;
    a.scr = scr;
    if (halo_entry && (full() || refresh)) {
      // the consumer convolution's boundary-row (boundary-column) state is refreshed by this kernel's store loop
      a.halo_out = halo_entry; a.halo_npatch = N();
      a.halo_cols = cols() ? 1 : 0;
      a.halo_rpp = cols() ? (full() ? W / N() : W) : (full() ? level_rows / N() : level_rows);
      a.halo_patch0 = full() ? 0 : patch;
    }
    if (full() && cols()) {
      // vertical strips are not contiguous pixel ranges: the image is normalised as one segment and the per-strip sums
      // of the cache come from a kernel of their own (synchronous step only)
      a.nseg = 1; a.Rseg = level_rows; a.N = 1; a.patch_idx = 0; a.stale = nullptr; a.sums_out = nullptr;
      const int Bn = B(), Nn = N();
      timed(PC_GROUPNORM, 0.0, 0.0, [&] { return launch_gn_strip_sums(x, in_dtype, entry, Bn, level_rows, W, C, G, Nn, st); });
    } else if (full()) {
      a.nseg = N(); a.Rseg = level_rows / N(); a.N = 1; a.patch_idx = 0; a.stale = nullptr; a.sums_out = entry;
    } else {
      a.nseg = 1; a.Rseg = level_rows; a.N = N(); a.patch_idx = patch; a.stale = entry;
      a.sums_out = refresh ? entry + (size_t)patch * B() * G * 2 : nullptr;
    }
    const double el = (double)B() * level_rows * W * C;
    label = "groupnorm " + dims({B() * level_rows, W, C}) + (in_dtype == DF_BF16 ? " bf16" : " f32");
    timed(PC_GROUPNORM, 0.0, el * (in_dtype == DF_BF16 ? 2.0 : 4.0) + el * 2.0, [&] { return launch_groupnorm(a, st); });
  }

  // x: bf16 [B, R, W, Cin] rows of this mode; out: [B, R/stride, W/stride, Cout]
  // boundary state of a convolution: first and last input row of every patch, [B, N, 2, W, Cin]; for vertical strips
  // the first and last input column, [B, N, 2, R, Cin] (`edge` = W or R: the length of the patch's shared edge)
  bf16_t* conv_entry(const std::string& name, int edge, int Cin) {
    return (bf16_t*)stale_buf(name + ".in", (size_t)B() * N() * 2 * (size_t)edge * Cin * sizeof(bf16_t));
  }
  // `entry_in` non-null: the stale entry was looked up by the caller and the producer of x has already refreshed it
  void conv(const std::string& name, const bf16_t* x, int R, int W, int Cin, int Cout, int stride, void* out,
            int out_dtype, const float* chan_add, const float* residual, bf16_t* entry_in = nullptr,
            bool halo_done = false, long long chan_ld = 0) {
    const size_t rowe = cols() ? (size_t)R * Cin : (size_t)W * Cin;     // elements of one boundary row / column
    bf16_t* entry = halo_done ? entry_in : conv_entry(name, cols() ? R : W, Cin);
    const void* wt = weight(name + ".w");
    const float* bias = (const float*)weight(name + ".b");
    {
      const size_t need = gemm_scratch_bytes((long long)B() * (R / stride) * (W / stride), Cout);
      if (need > scratch_need) scratch_need = need;
    }
    if (!live()) return;
    ConvArgs a = {};
    a.x = x; a.w = wt; a.bias = bias; a.chan_add = chan_add; a.chan_ld = chan_ld ? chan_ld : Cout; a.residual = residual; a.y = out;
    a.B = B(); a.R = R; a.W = W; a.Cin = Cin; a.Cout = Cout; a.stride = stride; a.act = 0;
    a.dtype = DF_BF16; a.out_dtype = out_dtype; a.scr = scr;
    if (cols()) {
      a.side_bstride = (long long)N() * 2 * rowe; a.side_rstride = Cin;
      if (!full()) {
        if (patch > 0) a.halo_left = entry + ((size_t)(patch - 1) * 2 + 1) * rowe;        // last column of the strip to the left
        if (patch + 1 < N() && stride == 1) a.halo_right = entry + ((size_t)(patch + 1) * 2) * rowe;
      }
    } else {
      a.halo_bstride = (long long)N() * 2 * rowe;
      if (!full()) {
        if (patch > 0) a.halo_top = entry + ((size_t)(patch - 1) * 2 + 1) * rowe;           // last row of the patch above
        if (patch + 1 < N() && stride == 1) a.halo_bot = entry + ((size_t)(patch + 1) * 2) * rowe;  // first row of the patch below
      }
    }
    {
      const double opx = (double)B() * (R / stride) * (W / stride);
      const double halo = full() ? 0.0 : 2.0;
      label = "conv3x3 " + dims({B() * R, W, Cin}) + "->" + std::to_string(Cout) + (stride == 2 ? " stride2" : "");
      timed(PC_CONV, 2.0 * 9 * Cin * Cout * opx,
            2.0 * B() * (R + halo) * rowe + 2.0 * 9 * Cin * Cout + opx * Cout * (out_dtype == DF_BF16 ? 2.0 : 4.0),
            [&] { return launch_conv3x3(a, st); });
    }
    if (!live() || halo_done) return;
    const long long rb = (long long)rowe * sizeof(bf16_t);
    if (cols()) {
      // boundary columns: R pieces of Cin elements each, one pixel per input row (x is [B, R, W, Cin] in this mode)
      const long long cb = (long long)Cin * sizeof(bf16_t);
      const int Wp = full() ? W / N() : W;
      if (full() || refresh)
        for (int bi = 0; bi < B(); ++bi)
          for (int j = full() ? 0 : patch; j < (full() ? N() : patch + 1); ++j)
            for (int which = 0; which < 2; ++which) {
              const int col = (full() ? j * Wp : 0) + which * (Wp - 1);
              timed(PC_REFRESH, 0.0, 2.0 * rb, [&] {
                return launch_copy_rows(entry + (((size_t)bi * N() + j) * 2 + which) * rowe,
                                        x + ((size_t)bi * R * W + col) * Cin, R, cb, cb, (long long)W * cb, st);
              });
            }
      return;
    }
    if (full()) {
      const int Rp = R / N();
      for (int which = 0; which < 2; ++which)
        timed(PC_REFRESH, 0.0, 2.0 * B() * N() * rb, [&] {
          return launch_copy_rows(entry + (size_t)which * rowe, x + (size_t)which * (Rp - 1) * rowe,
                                  (long long)B() * N(), rb, 2 * rb, (long long)Rp * rb, st);
        });
    } else if (refresh) {
      // first and last row of the patch in one launch per batch item: two "rows" of the copy, (R-1) rows apart in
      // the source, adjacent in the boundary-row state
      for (int bi = 0; bi < B(); ++bi)
        timed(PC_REFRESH, 0.0, 4.0 * rb, [&] {
          return launch_copy_rows(entry + ((size_t)bi * N() + patch) * 2 * rowe, x + (size_t)bi * R * rowe, 2, rb, rb,
                                  (long long)(R - 1) * rb, st);
        });
    }
  }

  // x_bf: bf16 copy of x if the caller already has one (operand of the 1x1 shortcut), else nullptr
  void resblock(const BlockDesc& b, const float* x, const bf16_t* emb_act, float* out, const bf16_t* x_bf = nullptr) {
    const int R = rows(b.level), W = width(b.level);
    const size_t px = (size_t)B() * R * W;
    const size_t mark = top;
    bf16_t* a1 = (bf16_t*)alloc(px * b.cin * 2);
    bf16_t* h1 = (bf16_t*)alloc(px * b.cout * 2);
    bf16_t* a2 = (bf16_t*)alloc(px * b.cout * 2);
    const float* embp = emb_all ? emb_all + emb_cursor : nullptr;     // this block's columns of the hoisted projection
    emb_cursor += b.cout;
    bf16_t* e1 = conv_entry(b.name + ".conv1", cols() ? R : W, b.cin);
    bf16_t* e2 = conv_entry(b.name + ".conv2", cols() ? R : W, b.cout);
    const bool hd = dry || e1 != nullptr;      // the GroupNorm kernels refresh the boundary rows of the convolutions
    groupnorm(b.name + ".gn1", x, DF_F32, R, W, b.cin, 1e-5f, 1, a1, 0, e1);
    conv(b.name + ".conv1", a1, R, W, b.cin, b.cout, 1, h1, DF_BF16, embp, nullptr, e1, hd, emb_n);
    groupnorm(b.name + ".gn2", h1, DF_BF16, R, W, b.cout, 1e-5f, 1, a2, 0, e2);
    const float* residual = x;
    if (b.cin != b.cout) {
      const bf16_t* xb = x_bf;
      if (!xb) {
        bf16_t* xc = (bf16_t*)alloc(px * b.cin * 2);
        timed(PC_ELEMENTWISE, 0.0, 6.0 * px * b.cin, [&] { return launch_cast_bf16(x, xc, (long long)px * b.cin, 0, st); });
        xb = xc;
      }
      gemm(xb, b.cin, b.name + ".sc", true, nullptr, 0, out, b.cout, (int)px, b.cout, b.cin, DF_F32);
      residual = out;
    }
    conv(b.name + ".conv2", a2, R, W, b.cout, b.cout, 1, out, DF_F32, nullptr, residual, e2, hd);
    top = mark;
  }


  // Linear layer on fragment-packed operands (wgemm.hip); `ln` applies the folded LayerNorm of that weight.
  void wg(const bf16_t* Xp, const std::string& wn, bool bias, bool ln, const float* residual, float* out_f32,
          bf16_t* out_packed, bf16_t* out_rows, long long ld_rows, int M, int Nn, int K, const WGemmArgs* extra = nullptr) {
    if (!live()) return;
    WGemmArgs g = {};
    if (extra) g = *extra;
    auto it = packed->find(wn);
    if (it == packed->end()) { err = DF_EINVAL; return; }
    g.Xp = Xp; g.Wp = it->second.f; g.M = M; g.N = Nn; g.K = K;
    if (ln) { g.ln_s = it->second.s; g.ln_t = it->second.t; g.ln_eps = 1e-5f; }
    else if (bias) g.bias = (const float*)weight(wn + ".b");
    const int No = g.geglu ? g.geglu : Nn;
    g.residual = residual; g.ldr = No; g.out_f32 = out_f32; g.ldo = No; g.out_packed = out_packed;
    g.out_rows = out_rows; g.ld_rows = ld_rows;
    const double ob = (out_f32 ? 4.0 : 0.0) + (out_packed ? 2.0 : 0.0) + ((out_rows || g.nseg) ? 2.0 : 0.0);
    label = "linear_packed " + dims({M, Nn, K}) + (g.geglu ? " geglu" : "") + (ln ? " ln" : "") + (g.nseg ? " qkv" : "");
    timed(PC_GEMM, 2.0 * M * Nn * K, 2.0 * ((double)M * K + (double)Nn * K) + ob * M * No,
          [&] { return launch_wgemm(g, st); });
  }

  // Transformer on fragment-packed activations (patch-sized token counts): every linear layer reads its operands in
  // MFMA order straight into registers and writes the next layer's operand in that order; LayerNorms are folded into
  // the consuming layers; attention reads row-major Q/K/V and writes its output packed.
  void transformer_frag(const BlockDesc& b, const float* x, float* out, int R, int W) {
    const int C = b.cin;
    const int Lq = R * W, L = (c.H >> b.level) * (c.W >> b.level), heads = C / c.head_dim;
    const int M = B() * Lq, TL = c.text_len;
    const float scale = 1.0f / sqrtf((float)c.head_dim);
    const size_t pC = packed_rows_bytes(M, C);
    bf16_t* nbp = (bf16_t*)alloc(pC);                       // GroupNorm output
    float* h = (float*)alloc((size_t)M * C * 4);            // hidden state (residual stream), row-major
    bf16_t* hp = (bf16_t*)alloc(pC);                        // its bf16 copy, packed
    bf16_t* qkv = (bf16_t*)alloc((size_t)M * 3 * C * 2);    // row-major queries (and fresh K/V without refresh)
    bf16_t* aop = (bf16_t*)alloc(pC);                       // attention output, packed
    bf16_t* fgp = (bf16_t*)alloc(packed_rows_bytes(M, 4 * C));
    const long long Lpad = (long long)((L + 63) / 64) * 64;   // key pitch of the V^T buffers: whole 64-key tiles
    bf16_t* ks_tmp = nullptr; bf16_t* vs_tmp = nullptr;
    if (!(full() || refresh)) {
      ks_tmp = (bf16_t*)alloc((size_t)B() * L * C * 2);
      vs_tmp = (bf16_t*)alloc((size_t)B() * C * Lpad * 2);
    }
    groupnorm(b.name + ".gn", x, DF_F32, R, W, C, 1e-6f, 0, nbp, 1);
    wg(nbp, b.name + ".pin", true, false, nullptr, h, hp, nullptr, 0, M, C, C);
    for (int d = 0; d < b.depth; ++d) {
      const std::string p = b.name + ".b" + std::to_string(d);
      bf16_t* ks = (bf16_t*)stale_buf(p + ".attn1.k", (size_t)B() * L * C * 2);
      bf16_t* vs = (bf16_t*)stale_buf(p + ".attn1.v", (size_t)B() * C * Lpad * 2);   // V^T: [B, C, Lpad]
      // where the patch's tokens start in the key / value buffers: a block of Lq rows, or - vertical strips - W
      // tokens of every grid row starting at the strip's first column
      const bool strip = cols() && !full();
      const size_t row0 = full() ? 0 : (strip ? (size_t)patch * W : (size_t)patch * Lq);
      const int pin = strip ? W : 0, pout = strip ? (c.W >> b.level) : 0;
      if (!(full() || refresh)) {
        // no refresh: the patch's keys and values go into private copies of the two buffers
        if (live()) {
          timed(PC_REFRESH, 0.0, 4.0 * B() * L * C, [&] { return launch_copy_rows(ks_tmp, ks, 1, (long long)B() * L * C * 2, 0, 0, st); });
          timed(PC_REFRESH, 0.0, 4.0 * B() * C * Lpad, [&] { return launch_copy_rows(vs_tmp, vs, 1, (long long)B() * C * Lpad * 2, 0, 0, st); });
        }
        ks = ks_tmp; vs = vs_tmp;
      }
      {
        // queries to a scratch tensor, keys straight into the patch's rows of the key buffer, values transposed into
        // the patch's columns of the V^T buffer (the refresh costs nothing)
        WGemmArgs ex = {};
        ex.nseg = 3; ex.seg_w = C;
        ex.seg_out[0] = qkv; ex.seg_ld[0] = C; ex.seg_rows_in[0] = 0x7fffffff; ex.seg_rows_out[0] = 0; ex.seg_row0[0] = 0;
        ex.seg_out[1] = ks; ex.seg_ld[1] = C; ex.seg_rows_in[1] = Lq; ex.seg_rows_out[1] = L; ex.seg_row0[1] = (long long)row0;
        ex.seg_out[2] = vs; ex.seg_ld[2] = Lpad; ex.seg_rows_in[2] = Lq; ex.seg_rows_out[2] = 0; ex.seg_row0[2] = (long long)row0;
        ex.seg_tr[2] = 1;
        ex.seg_pin[1] = ex.seg_pin[2] = pin; ex.seg_pout[1] = ex.seg_pout[2] = pout;
        wg(hp, p + ".attn1.qkv", false, true, nullptr, nullptr, nullptr, nullptr, 0, M, 3 * C, C, &ex);
      }
      {
        const size_t need = attention_scratch_bytes(B(), Lq, L, heads, c.head_dim);
        if (need > scratch_need) scratch_need = need;
      }
      if (live()) {
        AttnArgs a = {};
        a.k_stale = ks; a.v_stale = vs; a.out = aop; a.q = qkv; a.out_packed = 1;
        a.k_fresh = ks; a.v_fresh = vs; a.own_lo = 0; a.own_n = 0;
        a.v_transposed = 1; a.vt_ld = Lpad;
        a.B = B(); a.Lq = Lq; a.L = L; a.heads = heads; a.d = c.head_dim;
        a.ldq = C; a.ldkf = a.ldvf = C; a.ldks = C; a.ldvs = C; a.ldo = C;
        a.bsq = (long long)Lq * C; a.bskf = a.bsvf = (long long)L * C;
        a.bsks = (long long)L * C; a.bsvs = (long long)C * Lpad; a.bso = (long long)Lq * C;
        a.scale = scale; a.dtype = DF_BF16; a.scr = scr;
        label = "self_attn " + dims({M, L, C});
        timed(PC_SELF_ATTN, 4.0 * M * L * C, 2.0 * (2.0 * M * C + 2.0 * B() * L * C),
              [&] { return launch_attention(a, st); });
      }
      wg(aop, p + ".attn1.o", true, false, h, h, hp, nullptr, 0, M, C, C);
      // cross-attention to the text tokens
      const long long kvld = (long long)kv_count[b.level] * 2 * C;
      const int kvi = kv_cursor[b.level];
      const bf16_t* kv2 = kv2_all[b.level] + (size_t)kvi * 2 * C;
      kv_cursor[b.level] += 1;
      const bool fuse_x = xkv_all[b.level] != nullptr && (B() == 1 || Lq % 32 == 0);
      if (fuse_x) {
        // a head is one 64-feature tile of the query projection: attention against the packed text keys / values
        // runs in that layer's epilogue and writes the packed attention output
        if (live()) {
          const int XA = (TL + 31) / 32;
          WGemmArgs ex = {};
          ex.xa_kv = xkv_all[b.level] + (size_t)kvi * heads * 12 * XA * 512;
          ex.xa_keys = TL; ex.xa_rows = Lq; ex.xa_scale = scale;
          ex.xa_bstride = (long long)kv_count[b.level] * heads * 12 * XA * 512;
          auto it = packed->find(p + ".attn2.q");
          if (it == packed->end()) { err = DF_EINVAL; return; }
          WGemmArgs g2 = ex;
          g2.Xp = hp; g2.Wp = it->second.f; g2.M = M; g2.N = C; g2.K = C;
          g2.ln_s = it->second.s; g2.ln_t = it->second.t; g2.ln_eps = 1e-5f; g2.out_packed = aop;
          label = "cross_attn+q_proj " + dims({M, TL, C});
          timed(PC_CROSS_ATTN, 2.0 * M * C * C + 4.0 * M * TL * C, 2.0 * ((double)M * C + (double)C * C) + 2.0 * M * C,
                [&] { return launch_wgemm(g2, st); });
        }
      } else {
        wg(hp, p + ".attn2.q", false, true, nullptr, nullptr, nullptr, qkv, C, M, C, C);
        {
          const size_t need = attention_scratch_bytes(B(), Lq, TL, heads, c.head_dim);
          if (need > scratch_need) scratch_need = need;
        }
        if (live()) {
          AttnArgs a = {};
          a.q = qkv; a.k_fresh = kv2; a.v_fresh = kv2 + C; a.out = aop; a.out_packed = 1;
          a.B = B(); a.Lq = Lq; a.L = TL; a.heads = heads; a.d = c.head_dim; a.own_lo = 0; a.own_n = TL;
          a.ldq = C; a.ldkf = a.ldvf = kvld; a.ldks = a.ldvs = kvld; a.ldo = C;
          a.bsq = (long long)Lq * C; a.bskf = a.bsvf = (long long)TL * kvld; a.bso = (long long)Lq * C;
          a.scale = scale; a.dtype = DF_BF16; a.scr = scr;
          timed(PC_CROSS_ATTN, 4.0 * M * TL * C, 2.0 * (2.0 * M * C + 2.0 * B() * TL * C),
                [&] { return launch_attention(a, st); });
        }
      }
      wg(aop, p + ".attn2.o", true, false, h, h, hp, nullptr, 0, M, C, C);
      // GEGLU feed-forward
      {
        WGemmArgs ex = {};
        ex.geglu = 4 * C;
        wg(hp, p + ".ff1", false, true, nullptr, nullptr, fgp, nullptr, 0, M, 8 * C, C, &ex);
      }
      wg(fgp, p + ".ff2", true, false, h, h, hp, nullptr, 0, M, C, 4 * C);
    }
    wg(hp, b.name + ".pout", true, false, x, out, nullptr, nullptr, 0, M, C, C);
  }

  // Transformer with every LayerNorm folded into the GEMM that consumes it: the residual GEMMs also emit a bf16 copy
  // of the hidden state, which is the A operand of the next projection; no LayerNorm, cast or GEGLU kernel is launched.
  void transformer_folded(const BlockDesc& b, const float* x, float* out, bf16_t* nb, float* h, bf16_t* qkv, bf16_t* ao,
                          bf16_t* fg, int R, int W) {
    const int C = b.cin;
    const int Lq = R * W, L = (c.H >> b.level) * (c.W >> b.level), heads = C / c.head_dim;
    const int M = B() * Lq, TL = c.text_len;
    const float scale = 1.0f / sqrtf((float)c.head_dim);
    bf16_t* hb = (bf16_t*)alloc((size_t)M * C * 2);      // bf16 copy of the hidden state
    const long long Lpad = (long long)((L + 63) / 64) * 64;   // key pitch of the V^T buffers: whole 64-key tiles
    bf16_t* ks_tmp = nullptr; bf16_t* vs_tmp = nullptr;
    if (!(full() || refresh)) {
      ks_tmp = (bf16_t*)alloc((size_t)B() * L * C * 2);
      vs_tmp = (bf16_t*)alloc((size_t)B() * C * Lpad * 2);
    }
    gemm_packed(nb, C, b.name + ".pin", true, false, nullptr, 0, h, C, M, C, C, DF_F32, hb);
    for (int d = 0; d < b.depth; ++d) {
      const std::string p = b.name + ".b" + std::to_string(d);
      bf16_t* ks = (bf16_t*)stale_buf(p + ".attn1.k", (size_t)B() * L * C * 2);
      bf16_t* vs = (bf16_t*)stale_buf(p + ".attn1.v", (size_t)B() * C * Lpad * 2);   // V^T: [B, C, Lpad]
      // where the patch's tokens start in the key / value buffers: a block of Lq rows, or - vertical strips - W
      // tokens of every grid row starting at the strip's first column
      const bool strip = cols() && !full();
      const size_t row0 = full() ? 0 : (strip ? (size_t)patch * W : (size_t)patch * Lq);
      const int pin = strip ? W : 0, pout = strip ? (c.W >> b.level) : 0;
      if (!(full() || refresh)) {
        if (live()) {
          timed(PC_REFRESH, 0.0, 4.0 * B() * L * C, [&] { return launch_copy_rows(ks_tmp, ks, 1, (long long)B() * L * C * 2, 0, 0, st); });
          timed(PC_REFRESH, 0.0, 4.0 * B() * C * Lpad, [&] { return launch_copy_rows(vs_tmp, vs, 1, (long long)B() * C * Lpad * 2, 0, 0, st); });
        }
        ks = ks_tmp; vs = vs_tmp;
      }
      {
        GemmArgs ex = {};
        ex.nseg = 3; ex.seg_w = C;
        ex.seg_out[0] = qkv; ex.seg_ld[0] = C; ex.seg_rows_in[0] = 0x7fffffff; ex.seg_rows_out[0] = 0; ex.seg_row0[0] = 0;
        ex.seg_out[1] = ks; ex.seg_ld[1] = C; ex.seg_rows_in[1] = Lq; ex.seg_rows_out[1] = L; ex.seg_row0[1] = (long long)row0;
        ex.seg_out[2] = vs; ex.seg_ld[2] = Lpad; ex.seg_rows_in[2] = Lq; ex.seg_rows_out[2] = 0; ex.seg_row0[2] = (long long)row0;
        ex.seg_tr[2] = 1;
        ex.seg_pin[1] = ex.seg_pin[2] = pin; ex.seg_pout[1] = ex.seg_pout[2] = pout;
        gemm_packed(hb, C, p + ".attn1.qkv", false, true, nullptr, 0, qkv, C, M, 3 * C, C, DF_BF16, nullptr, &ex);
      }
      {
        const size_t need = attention_scratch_bytes(B(), Lq, L, heads, c.head_dim);
        if (need > scratch_need) scratch_need = need;
      }
      if (live()) {
        AttnArgs a = {};
        a.k_stale = ks; a.v_stale = vs; a.out = ao; a.q = qkv;
        a.k_fresh = ks; a.v_fresh = vs; a.own_lo = 0; a.own_n = 0;
        a.v_transposed = 1; a.vt_ld = Lpad;
        a.B = B(); a.Lq = Lq; a.L = L; a.heads = heads; a.d = c.head_dim;
        a.ldq = C; a.ldkf = a.ldvf = C; a.ldks = C; a.ldvs = C; a.ldo = C;
        a.bsq = (long long)Lq * C; a.bskf = a.bsvf = (long long)L * C;
        a.bsks = (long long)L * C; a.bsvs = (long long)C * Lpad; a.bso = (long long)Lq * C;
        a.scale = scale; a.dtype = DF_BF16; a.scr = scr;
        label = "self_attn " + dims({M, L, C});
        timed(PC_SELF_ATTN, 4.0 * M * L * C, 2.0 * (2.0 * M * C + 2.0 * B() * L * C),
              [&] { return launch_attention(a, st); });
      }
      gemm_packed(ao, C, p + ".attn1.o", true, false, h, C, h, C, M, C, C, DF_F32, hb);
      // cross-attention to the text tokens
      gemm_packed(hb, C, p + ".attn2.q", false, true, nullptr, 0, qkv, C, M, C, C, DF_BF16, nullptr);
      const long long kvld = (long long)kv_count[b.level] * 2 * C;
      const bf16_t* kv2 = kv2_all[b.level] + (size_t)kv_cursor[b.level] * 2 * C;
      kv_cursor[b.level] += 1;
      {
        const size_t need = attention_scratch_bytes(B(), Lq, TL, heads, c.head_dim);
        if (need > scratch_need) scratch_need = need;
      }
      if (live()) {
        AttnArgs a = {};
        a.q = qkv; a.k_fresh = kv2; a.v_fresh = kv2 + C; a.out = ao;
        a.B = B(); a.Lq = Lq; a.L = TL; a.heads = heads; a.d = c.head_dim; a.own_lo = 0; a.own_n = TL;
        a.ldq = C; a.ldkf = a.ldvf = kvld; a.ldks = a.ldvs = kvld; a.ldo = C;
        a.bsq = (long long)Lq * C; a.bskf = a.bsvf = (long long)TL * kvld; a.bso = (long long)Lq * C;
        a.scale = scale; a.dtype = DF_BF16; a.scr = scr;
        timed(PC_CROSS_ATTN, 4.0 * M * TL * C, 2.0 * (2.0 * M * C + 2.0 * B() * TL * C),
              [&] { return launch_attention(a, st); });
      }
      gemm_packed(ao, C, p + ".attn2.o", true, false, h, C, h, C, M, C, C, DF_F32, hb);
      // GEGLU feed-forward
      {
        GemmArgs ex = {};
        ex.geglu = 1;
        gemm_packed(hb, C, p + ".ff1", false, true, nullptr, 0, fg, 4 * C, M, 8 * C, C, DF_BF16, nullptr, &ex);
      }
      gemm_packed(fg, 4 * C, p + ".ff2", true, false, h, C, h, C, M, C, 4 * C, DF_F32, hb);
    }
    gemm_packed(hb, C, b.name + ".pout", true, false, x, C, out, C, M, C, C, DF_F32, nullptr);
  }

  void transformer(const BlockDesc& b, const float* x, const bf16_t* text, float* out) {
    const int R = rows(b.level), W = width(b.level), C = b.cin;
    const int Lq = R * W, L = (c.H >> b.level) * (c.W >> b.level), heads = C / c.head_dim;
    const int M = B() * Lq;
    const int TL = c.text_len;
    const size_t mark = top;
    bf16_t* nb = (bf16_t*)alloc((size_t)M * C * 2);          // normalised input of the next GEMM
    float* h = (float*)alloc((size_t)M * C * 4);             // hidden state (residual stream)
    bf16_t* qkv = (bf16_t*)alloc((size_t)M * 3 * C * 2);
    bf16_t* ao = (bf16_t*)alloc((size_t)M * C * 2);          // attention output
    bf16_t* ff = (bf16_t*)alloc((size_t)M * 8 * C * 2);
    bf16_t* fg = (bf16_t*)alloc((size_t)M * 4 * C * 2);
    const float scale = 1.0f / sqrtf((float)c.head_dim);
    if (fold_ok(C) && M <= kFragMaxRows && frag_path()) {
      top = mark;
      transformer_frag(b, x, out, R, W);
      top = mark;
      return;
    }
    if (cols() && b.depth > 0 && !fold_ok(C)) { err = DF_ESHAPE; return; }   // (cfg_ok rejects such plans up front)
    groupnorm(b.name + ".gn", x, DF_F32, R, W, C, 1e-6f, 0, nb);
    if (fold_ok(C)) {
      transformer_folded(b, x, out, nb, h, qkv, ao, fg, R, W);
      top = mark;
      return;
    }
    gemm(nb, C, b.name + ".pin", true, nullptr, 0, h, C, M, C, C, DF_F32);
    for (int d = 0; d < b.depth; ++d) {
      const std::string p = b.name + ".b" + std::to_string(d);
      // --- self-attention: fresh queries against spliced fresh/stale keys and values ---
      const float* g1 = (const float*)weight(p + ".ln1.g");
      const float* b1 = (const float*)weight(p + ".ln1.beta");
      timed(PC_LAYERNORM, 0.0, 6.0 * M * C, [&] { return launch_layernorm(h, nb, g1, b1, M, C, 1e-5f, st); });
      bf16_t* ks = (bf16_t*)stale_buf(p + ".attn1.k", (size_t)B() * L * C * 2);
      bf16_t* vs = (bf16_t*)stale_buf(p + ".attn1.v", (size_t)B() * L * C * 2);
      // With refresh the projection writes the patch's keys and values straight into its rows of the stale buffers
      // (the refresh costs nothing) and attention reads every key from there; without refresh they go to a scratch
      // tensor and are spliced in by the attention loader.
      const bool fused_kv = (full() || refresh) && C % 64 == 0 && C >= 128;
      // where the patch's tokens start in the key / value buffers: a block of Lq rows, or - vertical strips - W
      // tokens of every grid row starting at the strip's first column
      const bool strip = cols() && !full();
      const size_t row0 = full() ? 0 : (strip ? (size_t)patch * W : (size_t)patch * Lq);
      const int pin = strip ? W : 0, pout = strip ? (c.W >> b.level) : 0;
      (void)pin; (void)pout;             // (vertical strips never reach this path)
      if (fused_kv) {
        GemmArgs ex = {};
        ex.nseg = 3; ex.seg_w = C;
        ex.seg_out[0] = qkv; ex.seg_ld[0] = C; ex.seg_rows_in[0] = 0x7fffffff; ex.seg_rows_out[0] = 0; ex.seg_row0[0] = 0;
        ex.seg_out[1] = ks; ex.seg_ld[1] = C; ex.seg_rows_in[1] = Lq; ex.seg_rows_out[1] = L; ex.seg_row0[1] = (long long)row0;
        ex.seg_out[2] = vs; ex.seg_ld[2] = C; ex.seg_rows_in[2] = Lq; ex.seg_rows_out[2] = L; ex.seg_row0[2] = (long long)row0;
        gemm(nb, C, p + ".attn1.qkv", false, nullptr, 0, qkv, C, M, 3 * C, C, DF_BF16, &ex);
      } else {
        gemm(nb, C, p + ".attn1.qkv", false, nullptr, 0, qkv, 3 * C, M, 3 * C, C, DF_BF16);
      }
      {
        const size_t need = attention_scratch_bytes(B(), Lq, L, heads, c.head_dim);
        if (need > scratch_need) scratch_need = need;
      }
      if (live()) {
        AttnArgs a = {};
        a.k_stale = ks; a.v_stale = vs; a.out = ao; a.q = qkv;
        a.B = B(); a.Lq = Lq; a.L = L; a.heads = heads; a.d = c.head_dim;
        a.ldks = a.ldvs = C; a.ldo = C;
        a.bsks = a.bsvs = (long long)L * C; a.bso = (long long)Lq * C;
        if (fused_kv) {
          a.k_fresh = ks; a.v_fresh = vs; a.own_lo = 0; a.own_n = 0;     // every key row comes from the refreshed buffer
          a.ldq = C; a.ldkf = a.ldvf = C; a.bsq = (long long)Lq * C; a.bskf = a.bsvf = (long long)L * C;
        } else {
          a.k_fresh = qkv + C; a.v_fresh = qkv + 2 * C;
          a.own_lo = full() ? 0 : patch * Lq; a.own_n = Lq;
          a.ldq = a.ldkf = a.ldvf = 3 * C; a.bsq = a.bskf = a.bsvf = (long long)Lq * 3 * C;
        }
        a.scale = scale; a.dtype = DF_BF16; a.scr = scr;
        label = "self_attn " + dims({M, L, C});
        timed(PC_SELF_ATTN, 4.0 * M * L * C, 2.0 * (2.0 * M * C + 2.0 * B() * L * C),
              [&] { return launch_attention(a, st); });
      }
      if (live() && !fused_kv && (full() || refresh)) {
        // narrow layers keep the separate refresh copies of the projected keys and values
        for (int bi = 0; bi < B(); ++bi) {
          timed(PC_REFRESH, 0.0, 4.0 * Lq * C, [&] {
            return launch_copy_rows(ks + ((size_t)bi * L + row0) * C, qkv + (size_t)bi * Lq * 3 * C + C, Lq, C * 2LL,
                                    C * 2LL, 3LL * C * 2, st);
          });
          timed(PC_REFRESH, 0.0, 4.0 * Lq * C, [&] {
            return launch_copy_rows(vs + ((size_t)bi * L + row0) * C, qkv + (size_t)bi * Lq * 3 * C + 2 * C, Lq,
                                    C * 2LL, C * 2LL, 3LL * C * 2, st);
          });
        }
      }
      gemm(ao, C, p + ".attn1.o", true, h, C, h, C, M, C, C, DF_F32);
      // --- cross-attention to the text tokens: per token, no cross-patch data ---
      const float* g2 = (const float*)weight(p + ".ln2.g");
      const float* b2 = (const float*)weight(p + ".ln2.beta");
      timed(PC_LAYERNORM, 0.0, 6.0 * M * C, [&] { return launch_layernorm(h, nb, g2, b2, M, C, 1e-5f, st); });
      gemm(nb, C, p + ".attn2.q", false, nullptr, 0, qkv, C, M, C, C, DF_BF16);
      // keys/values of the text tokens: projected for all blocks of the level at the start of the step
      const long long kvld = (long long)kv_count[b.level] * 2 * C;
      const bf16_t* kv2 = kv2_all[b.level] + (size_t)kv_cursor[b.level] * 2 * C;
      kv_cursor[b.level] += 1;
      {
        const size_t need = attention_scratch_bytes(B(), Lq, TL, heads, c.head_dim);
        if (need > scratch_need) scratch_need = need;
      }
      if (live()) {
        AttnArgs a = {};
        a.q = qkv; a.k_fresh = kv2; a.v_fresh = kv2 + C; a.out = ao;
        a.B = B(); a.Lq = Lq; a.L = TL; a.heads = heads; a.d = c.head_dim; a.own_lo = 0; a.own_n = TL;
        a.ldq = C; a.ldkf = a.ldvf = kvld; a.ldks = a.ldvs = kvld; a.ldo = C;
        a.bsq = (long long)Lq * C; a.bskf = a.bsvf = (long long)TL * kvld; a.bso = (long long)Lq * C;
        a.scale = scale; a.dtype = DF_BF16; a.scr = scr;
        timed(PC_CROSS_ATTN, 4.0 * M * TL * C, 2.0 * (2.0 * M * C + 2.0 * B() * TL * C),
              [&] { return launch_attention(a, st); });
      }
      gemm(ao, C, p + ".attn2.o", true, h, C, h, C, M, C, C, DF_F32);
      // --- GEGLU feed-forward ---
      const float* g3 = (const float*)weight(p + ".ln3.g");
      const float* b3 = (const float*)weight(p + ".ln3.beta");
      timed(PC_LAYERNORM, 0.0, 6.0 * M * C, [&] { return launch_layernorm(h, nb, g3, b3, M, C, 1e-5f, st); });
      if (C % 64 == 0 && C >= 128) {
        GemmArgs ex = {};
        ex.geglu = 1;                    // value * gelu(gate) in the epilogue: the [M, 8C] tensor never exists
        gemm(nb, C, p + ".ff1", true, nullptr, 0, fg, 4 * C, M, 8 * C, C, DF_BF16, &ex);
      } else {
        gemm(nb, C, p + ".ff1", true, nullptr, 0, ff, 8 * C, M, 8 * C, C, DF_BF16);
        timed(PC_ELEMENTWISE, 0.0, 24.0 * M * C, [&] { return launch_geglu(ff, fg, M, 4 * C, st); });
      }
      gemm(fg, 4 * C, p + ".ff2", true, h, C, h, C, M, C, 4 * C, DF_F32);
    }
    timed(PC_ELEMENTWISE, 0.0, 6.0 * M * C, [&] { return launch_cast_bf16(h, nb, (long long)M * C, 0, st); });
    gemm(nb, C, b.name + ".pout", true, x, C, out, C, M, C, C, DF_F32);
    top = mark;
  }

  int step(const float* x_in, const float* emb, const bf16_t* text, float* eps_out) {
    std::vector<const float*> skips;
    std::vector<int> skip_c;
    const float* cur = x_in;
    int cur_c = c.in_ch;
    bf16_t* emb_act = (bf16_t*)alloc((size_t)B() * c.emb_dim * 2);
    timed(PC_ELEMENTWISE, 0.0, 6.0 * B() * c.emb_dim, [&] { return launch_cast_bf16(emb, emb_act, (long long)B() * c.emb_dim, 1, st); });
    emb_n = emb_total(blocks);
    emb_cursor = 0;
    emb_all = (float*)alloc((size_t)B() * emb_n * 4);
    gemm_w(emb_act, c.emb_dim, emb_w_all, emb_b_all, nullptr, 0, emb_all, emb_n, B(), emb_n, c.emb_dim, DF_F32);
    for (int lv = 0; lv < c.n_levels; ++lv) {
      kv_cursor[lv] = 0;
      if (kv_count[lv] == 0) continue;
      const int Nkv = kv_count[lv] * 2 * c.levels[lv];
      kv2_all[lv] = (bf16_t*)alloc((size_t)B() * c.text_len * Nkv * 2);
      GemmArgs ex = {};
      ex.packed_w = (c.text_dim % 64 == 0 && c.text_dim >= 128) ? 1 : 0;
      gemm_w(text, c.text_dim, kv_packed[lv], nullptr, nullptr, 0, kv2_all[lv], Nkv, B() * c.text_len, Nkv, c.text_dim,
             DF_BF16, &ex);
      // the same keys / values as MFMA fragments per head, for the cross-attention fused into the query projection
      xkv_all[lv] = nullptr;
      if (fold_ok(c.levels[lv]) && c.text_len <= 128 && c.head_dim == 64) {
        xkv_all[lv] = (bf16_t*)alloc(packed_text_kv_bytes(B(), c.text_len, kv_count[lv], c.levels[lv]));
        if (live()) {
          bf16_t* dst = xkv_all[lv];
          const bf16_t* src = kv2_all[lv];
          const int cnt = kv_count[lv], Cl = c.levels[lv];
          timed(PC_ELEMENTWISE, 0.0, 4.0 * B() * c.text_len * Nkv,
                [&] { return launch_pack_text_kv(src, Nkv, dst, B(), c.text_len, cnt, Cl, st); });
        }
      }
    }
    for (const BlockDesc& b : blocks) {
      if (err != DF_OK) break;
      const int R = rows(b.level), W = width(b.level);
      const size_t px = (size_t)B() * R * W;
      switch (b.kind) {
        case BlockDesc::CONV_IN: {
          float* out = (float*)alloc(px * b.cout * 4);
          const size_t mark = top;
          bf16_t* xb = (bf16_t*)alloc(px * b.cin * 2);
          timed(PC_ELEMENTWISE, 0.0, 6.0 * px * b.cin, [&] { return launch_cast_bf16(cur, xb, (long long)px * b.cin, 0, st); });
          conv(b.name, xb, R, W, b.cin, b.cout, 1, out, DF_F32, nullptr, nullptr);
          top = mark;
          cur = out; cur_c = b.cout;
          break;
        }
        case BlockDesc::PUSH:
          skips.push_back(cur);
          skip_c.push_back(cur_c);
          break;
        case BlockDesc::RES: {
          float* out = (float*)alloc(px * b.cout * 4);
          const size_t mark = top;
          const float* xin = cur;
          const bf16_t* xin_bf = nullptr;
          if (b.concat) {
            const float* sk = skips.back();
            const int sc = skip_c.back();
            skips.pop_back();
            skip_c.pop_back();
            float* cat = (float*)alloc(px * (size_t)(cur_c + sc) * 4);
            bf16_t* catb = (bf16_t*)alloc(px * (size_t)(cur_c + sc) * 2);   // the shortcut's operand, written by the same kernel
            timed(PC_ELEMENTWISE, 0.0, 10.0 * px * (cur_c + sc),
                  [&] { return launch_concat(cur, cur_c, sk, sc, cat, catb, (long long)px, st); });
            xin = cat;
            xin_bf = dry ? nullptr : catb;
          }
          resblock(b, xin, emb_act, out, xin_bf);
          top = mark;
          cur = out; cur_c = b.cout;
          break;
        }
        case BlockDesc::XF: {
          float* out = (float*)alloc(px * b.cout * 4);
          transformer(b, cur, text, out);
          cur = out;
          break;
        }
        case BlockDesc::DOWN: {
          const size_t opx = (size_t)B() * (R / 2) * (W / 2);
          float* out = (float*)alloc(opx * b.cout * 4);
          const size_t mark = top;
          bf16_t* xb = (bf16_t*)alloc(px * b.cin * 2);
          timed(PC_ELEMENTWISE, 0.0, 6.0 * px * b.cin, [&] { return launch_cast_bf16(cur, xb, (long long)px * b.cin, 0, st); });
          conv(b.name, xb, R, W, b.cin, b.cout, 2, out, DF_F32, nullptr, nullptr);
          top = mark;
          cur = out;
          break;
        }
        case BlockDesc::UP: {
          float* out = (float*)alloc(px * 4 * b.cout * 4);
          const size_t mark = top;
          bf16_t* xb = (bf16_t*)alloc(px * 4 * b.cin * 2);
          timed(PC_ELEMENTWISE, 0.0, 12.0 * px * b.cin, [&] { return launch_upsample2x_bf16(cur, xb, B(), R, W, b.cin, st); });
          conv(b.name, xb, 2 * R, 2 * W, b.cin, b.cout, 1, out, DF_F32, nullptr, nullptr);
          top = mark;
          cur = out;
          break;
        }
        case BlockDesc::OUT: {
          const size_t mark = top;
          bf16_t* a = (bf16_t*)alloc(px * b.cin * 2);
          groupnorm(b.name + ".gn", cur, DF_F32, R, W, b.cin, 1e-5f, 1, a);
          conv(b.name + ".conv", a, R, W, b.cin, b.cout, 1, eps_out, DF_F32, nullptr, nullptr);
          top = mark;
          break;
        }
      }
    }
    return err;
  }
};

std::vector<PackSpec> build_pack_specs(const df_unet_cfg& c, const std::vector<BlockDesc>& blocks, size_t base,
                                       size_t* end) {
  std::vector<PackSpec> v;
  size_t off = base;
  auto add = [&](const std::string& name, int N, int K, const std::string& norm, bool has_bias) {
    PackSpec sp{name, N, K, norm, has_bias, 0, 0, 0, 0};
    sp.w_off = off; off += align256((size_t)N * K * sizeof(bf16_t));
    sp.f_off = off; off += align256((size_t)N * K * sizeof(bf16_t));
    if (!norm.empty()) {
      sp.s_off = off; off += align256((size_t)N * sizeof(float));
      sp.t_off = off; off += align256((size_t)N * sizeof(float));
    }
    v.push_back(sp);
  };
  for (const BlockDesc& b : blocks) {
    if (b.kind != BlockDesc::XF || !fold_ok(b.cin)) continue;
    const int C = b.cin;
    add(b.name + ".pin", C, C, "", true);
    for (int d = 0; d < b.depth; ++d) {
      const std::string p = b.name + ".b" + std::to_string(d);
      add(p + ".attn1.qkv", 3 * C, C, p + ".ln1", false);
      add(p + ".attn1.o", C, C, "", true);
      add(p + ".attn2.q", C, C, p + ".ln2", false);
      add(p + ".attn2.o", C, C, "", true);
      add(p + ".ff1", 8 * C, C, p + ".ln3", true);
      add(p + ".ff2", C, 4 * C, "", true);
    }
    add(b.name + ".pout", C, C, "", true);
  }
  *end = off;
  return v;
}

struct DryResult {
  size_t ws_bytes, stale_bytes, scratch, packed_bytes;
  size_t emb_w_off, emb_b_off;
  size_t kv_off[4];
  int kv_count[4];
  std::vector<StaleEntry> stale;
};

DryResult dry_run(const df_unet_cfg& c, const std::vector<BlockDesc>& blocks) {
  DryResult r = {};
  for (int pass = 0; pass < 3; ++pass) {   // FULL; DISPLACED with refresh; DISPLACED without (private K / V^T copies)
    const int mode = pass == 0 ? 0 : 1;
    std::vector<StaleEntry> list;
    Exec e{c, blocks, nullptr, true, mode, 0, pass == 2 ? 0 : 1, nullptr, nullptr, 0};
    for (const BlockDesc& b : blocks)
      if (b.kind == BlockDesc::XF) e.kv_count[b.level] += b.depth;
    e.stale_base = nullptr;
    e.stale_list = &list;
    e.stale_idx = nullptr;
    e.step(nullptr, nullptr, nullptr, nullptr);
    if (e.high > r.ws_bytes) r.ws_bytes = e.high;
    if (e.scratch_need > r.scratch) r.scratch = e.scratch_need;
    if (mode == 0) { r.stale = list; r.stale_bytes = e.stale_top; }
  }
  for (int lv = 0; lv < 4; ++lv) { r.kv_off[lv] = 0; r.kv_count[lv] = 0; }
  for (const BlockDesc& b : blocks)
    if (b.kind == BlockDesc::XF) r.kv_count[b.level] += b.depth;
  size_t off = 0;
  for (int lv = 0; lv < c.n_levels; ++lv) {
    r.kv_off[lv] = off;
    off += align256((size_t)r.kv_count[lv] * 2 * c.levels[lv] * c.text_dim * sizeof(bf16_t));
  }
  size_t end = off;
  build_pack_specs(c, blocks, off, &end);
  r.emb_w_off = end;
  end += align256((size_t)emb_total(blocks) * c.emb_dim * sizeof(bf16_t));
  r.emb_b_off = end;
  end += align256((size_t)emb_total(blocks) * sizeof(float));
  r.packed_bytes = end;
  if (r.scratch < kScratchCounterBytes) r.scratch = kScratchCounterBytes;
  r.scratch = align256(r.scratch);
  r.ws_bytes += end + r.scratch + 256;
  return r;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int df_unet_num_weights(const df_unet_cfg* cfg) {
  if (!cfg_ok(cfg)) return DF_ESHAPE;
  return (int)build_weight_specs(*cfg).size();
}

int df_unet_weight_info(const df_unet_cfg* cfg, int idx, char* name, int name_cap, int* ndim, long long dims[4]) {
  if (!cfg_ok(cfg)) return DF_ESHAPE;
  if (!name || !ndim || !dims || name_cap < 1) return DF_EINVAL;
  const std::vector<WeightSpec> s = build_weight_specs(*cfg);
  if (idx < 0 || idx >= (int)s.size()) return DF_EINVAL;
  std::strncpy(name, s[idx].name.c_str(), (size_t)name_cap - 1);
  name[name_cap - 1] = 0;
  *ndim = s[idx].ndim;
  for (int i = 0; i < 4; ++i) dims[i] = s[idx].dims[i];
  return DF_OK;
}

size_t df_unet_workspace_bytes(const df_unet_cfg* cfg) {
  if (!cfg_ok(cfg)) return 0;
  return dry_run(*cfg, build_blocks(*cfg)).ws_bytes;
}

size_t df_unet_stale_bytes(const df_unet_cfg* cfg) {
  if (!cfg_ok(cfg)) return 0;
  return dry_run(*cfg, build_blocks(*cfg)).stale_bytes;
}

int df_unet_create(df_unet** out, const df_unet_cfg* cfg, const void* const* weights, int n_weights, void* workspace,
                   size_t workspace_bytes) {
  if (!out || !weights || !workspace) return DF_EINVAL;
  if (!cfg_ok(cfg)) return DF_ESHAPE;
  if ((uintptr_t)workspace % 256) return DF_EINVAL;
  const std::vector<WeightSpec> specs = build_weight_specs(*cfg);
  if (n_weights != (int)specs.size()) return DF_EINVAL;
  df_unet* u = new df_unet();
  u->cfg = *cfg;
  u->blocks = build_blocks(*cfg);
  for (size_t i = 0; i < specs.size(); ++i) {
    if (!weights[i] || ((uintptr_t)weights[i] % 16)) { delete u; return DF_EINVAL; }
    u->w[specs[i].name] = weights[i];
  }
  DryResult d = dry_run(u->cfg, u->blocks);
  if (workspace_bytes < d.ws_bytes) { delete u; return DF_ENOMEM; }
  u->stale = d.stale;
  for (size_t i = 0; i < u->stale.size(); ++i) u->stale_idx[u->stale[i].name] = (int)i;
  u->stale_bytes = d.stale_bytes;
  u->ws = (char*)workspace;
  u->ws_bytes = workspace_bytes;
  u->packed_bytes = d.packed_bytes;
  {
    int cursor[4] = {0, 0, 0, 0};
    for (int lv = 0; lv < 4; ++lv) { u->kv_off[lv] = d.kv_off[lv]; u->kv_count[lv] = d.kv_count[lv]; }
    for (const BlockDesc& b : u->blocks) {
      if (b.kind != BlockDesc::XF) continue;
      const size_t one = (size_t)2 * b.cin * cfg->text_dim * sizeof(bf16_t);
      for (int dd = 0; dd < b.depth; ++dd) {
        const void* src = u->w[b.name + ".b" + std::to_string(dd) + ".attn2.kv.w"];
        char* dst = u->ws + u->kv_off[b.level] + (size_t)cursor[b.level] * one;
        if (hipMemcpy(dst, src, one, hipMemcpyDeviceToDevice) != hipSuccess) { delete u; return DF_EHIP; }
        cursor[b.level] += 1;
      }
    }
    const bool pack_kv = cfg->text_dim % 64 == 0 && cfg->text_dim >= 128;
    if (pack_kv) {
      // re-tile the concatenated text K/V weights in place of the plain copies made above: pack each block's
      // weight from its original tensor (its rows are whole 64-row tiles of the concatenation)
      int cur2[4] = {0, 0, 0, 0};
      for (const BlockDesc& b : u->blocks) {
        if (b.kind != BlockDesc::XF) continue;
        const size_t one = (size_t)2 * b.cin * cfg->text_dim;
        for (int dd = 0; dd < b.depth; ++dd) {
          const bf16_t* src = (const bf16_t*)u->w[b.name + ".b" + std::to_string(dd) + ".attn2.kv.w"];
          bf16_t* dst = (bf16_t*)(u->ws + u->kv_off[b.level]) + (size_t)cur2[b.level] * one;
          if (launch_pack_weight(src, nullptr, dst, 2 * b.cin, cfg->text_dim, 0) != DF_OK) { delete u; return DF_EHIP; }
          cur2[b.level] += 1;
        }
      }
    }
    size_t end = 0;
    size_t base = 0;
    for (int lv = 0; lv < cfg->n_levels; ++lv)
      base = u->kv_off[lv] + align256((size_t)u->kv_count[lv] * 2 * cfg->levels[lv] * cfg->text_dim * sizeof(bf16_t));
    for (const PackSpec& sp : build_pack_specs(u->cfg, u->blocks, base, &end)) {
      PackedW pw;
      bf16_t* dst = (bf16_t*)(u->ws + sp.w_off);
      const bf16_t* src = (const bf16_t*)u->w[sp.name + ".w"];
      const float* gamma = sp.norm.empty() ? nullptr : (const float*)u->w[sp.norm + ".g"];
      if (launch_pack_weight(src, gamma, dst, sp.N, sp.K, 0) != DF_OK) { delete u; return DF_EHIP; }
      pw.w = dst;
      {
        bf16_t* fdst = (bf16_t*)(u->ws + sp.f_off);
        if (launch_pack_wfrag(src, gamma, fdst, sp.N, sp.K, 0) != DF_OK) { delete u; return DF_EHIP; }
        pw.f = fdst;
      }
      if (!sp.norm.empty()) {
        float* sv = (float*)(u->ws + sp.s_off);
        float* tv = (float*)(u->ws + sp.t_off);
        const float* beta = (const float*)u->w[sp.norm + ".beta"];
        const float* bias = sp.has_bias ? (const float*)u->w[sp.name + ".b"] : nullptr;
        if (launch_fold_vectors(src, gamma, beta, bias, sv, tv, sp.N, sp.K, 0) != DF_OK) { delete u; return DF_EHIP; }
        pw.s = sv; pw.t = tv;
      }
      u->packed[sp.name] = pw;
    }
    {
      u->emb_w_off = d.emb_w_off; u->emb_b_off = d.emb_b_off;
      size_t row = 0;
      for (const BlockDesc& b : u->blocks) {
        if (b.kind != BlockDesc::RES) continue;
        const void* wsrc = u->w[b.name + ".emb.w"];
        const void* bsrc = u->w[b.name + ".emb.b"];
        if (hipMemcpy(u->ws + u->emb_w_off + row * cfg->emb_dim * sizeof(bf16_t), wsrc,
                      (size_t)b.cout * cfg->emb_dim * sizeof(bf16_t), hipMemcpyDeviceToDevice) != hipSuccess ||
            hipMemcpy(u->ws + u->emb_b_off + row * sizeof(float), bsrc, (size_t)b.cout * sizeof(float),
                      hipMemcpyDeviceToDevice) != hipSuccess) { delete u; return DF_EHIP; }
        row += b.cout;
      }
    }
    if (hipDeviceSynchronize() != hipSuccess) { delete u; return DF_EHIP; }
  }
  u->scr.ptr = u->ws + d.packed_bytes;
  u->scr.bytes = d.scratch;
  if (scratch_init(u->scr) != DF_OK) { delete u; return DF_EHIP; }
  *out = u;
  return DF_OK;
}

void df_unet_destroy(df_unet* u) {
  if (!u) return;
  for (GraphEntry& g : u->graphs)
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
  delete u;
}

int df_unet_num_stale(const df_unet* u) { return u ? (int)u->stale.size() : DF_EINVAL; }

int df_unet_stale_name(const df_unet* u, int idx, char* name, int name_cap) {
  if (!u || !name || name_cap < 1 || idx < 0 || idx >= (int)u->stale.size()) return DF_EINVAL;
  std::strncpy(name, u->stale[idx].name.c_str(), (size_t)name_cap - 1);
  name[name_cap - 1] = 0;
  return DF_OK;
}

int df_unet_stale_lookup(const df_unet* u, const char* name, size_t* offset, size_t* bytes) {
  if (!u || !name || !offset || !bytes) return DF_EINVAL;
  auto it = u->stale_idx.find(name);
  if (it == u->stale_idx.end()) return DF_EINVAL;
  *offset = u->stale[it->second].off;
  *bytes = u->stale[it->second].bytes;
  return DF_OK;
}

int df_patch_unet_step(df_unet* u, const void* x, const void* emb, const void* text, void* stale, void* eps_out,
                       int patch_idx, int mode, int refresh, void* stream) {
  if (!u || !x || !emb || !text || !stale || !eps_out) return DF_EINVAL;
  if (mode != DF_MODE_FULL && mode != DF_MODE_DISPLACED) return DF_EINVAL;
  if (mode == DF_MODE_DISPLACED && (patch_idx < 0 || patch_idx >= u->cfg.N)) return DF_ESHAPE;
  if (((uintptr_t)x % 16) || ((uintptr_t)text % 16) || ((uintptr_t)stale % 256) || ((uintptr_t)eps_out % 16))
    return DF_EINVAL;
  Exec e{u->cfg, u->blocks, &u->w, false, mode, mode == DF_MODE_FULL ? 0 : patch_idx, refresh ? 1 : 0,
         (hipStream_t)stream, u->ws + u->packed_bytes + u->scr.bytes, u->ws_bytes - u->packed_bytes - u->scr.bytes};
  e.scr = &u->scr;
  for (int lv = 0; lv < 4; ++lv) {
    e.kv_count[lv] = u->kv_count[lv];
    e.kv_packed[lv] = (const bf16_t*)(u->ws + u->kv_off[lv]);
  }
  e.packed = &u->packed;
  e.gn_mode = u->gn_mode;
  e.emb_w_all = (const bf16_t*)(u->ws + u->emb_w_off);
  e.emb_b_all = (const float*)(u->ws + u->emb_b_off);
  e.stale_base = (char*)stale;
  e.stale_list = &u->stale;
  e.stale_idx = &u->stale_idx;
  e.prof = &u->prof;
  hipStream_t st = (hipStream_t)stream;
  // the legacy default stream cannot be captured; per-launch timing needs the events between the launches
  if (!u->use_graph || u->prof.on || st == nullptr)
    return e.step((const float*)x, (const float*)emb, (const bf16_t*)text, (float*)eps_out);
  GraphEntry* ge = nullptr;
  for (GraphEntry& g : u->graphs)
    if (g.mode == mode && g.patch == e.patch && g.refresh == e.refresh && g.gn_mode == e.gn_mode && g.x == x && g.emb == emb && g.text == text &&
        g.eps == eps_out && g.stale == stale && g.stream == st) { ge = &g; break; }
  if (!ge) {
    if (u->graphs.size() >= 64) {   // bound the cache: drop the oldest entry
      if (u->graphs.front().exec) (void)hipGraphExecDestroy(u->graphs.front().exec);
      u->graphs.erase(u->graphs.begin());
    }
    GraphEntry g;
    g.mode = mode; g.patch = e.patch; g.refresh = e.refresh; g.gn_mode = e.gn_mode; g.x = x; g.emb = emb; g.text = text; g.eps = eps_out;
    g.stale = stale; g.stream = st;
    u->graphs.push_back(g);
    ge = &u->graphs.back();
  }
  if (ge->exec) return hipGraphLaunch(ge->exec, st) == hipSuccess ? DF_OK : DF_EHIP;
  if (ge->calls == 0) {
    ge->calls = 1;
    return e.step((const float*)x, (const float*)emb, (const bf16_t*)text, (float*)eps_out);
  }
  if (hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal) != hipSuccess) {
    (void)hipGetLastError();
    return e.step((const float*)x, (const float*)emb, (const bf16_t*)text, (float*)eps_out);
  }
  const int rc = e.step((const float*)x, (const float*)emb, (const bf16_t*)text, (float*)eps_out);
  hipGraph_t graph = nullptr;
  const hipError_t ec = hipStreamEndCapture(st, &graph);
  if (rc != DF_OK || ec != hipSuccess || !graph) {
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipGetLastError();
    return rc != DF_OK ? rc : DF_EHIP;
  }
  hipGraphExec_t exec = nullptr;
  const hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (ei != hipSuccess || !exec) return DF_EHIP;
  ge->exec = exec;
  return hipGraphLaunch(exec, st) == hipSuccess ? DF_OK : DF_EHIP;
}

int df_unet_set_gn_mode(df_unet* u, int stat_mode) {
  if (!u || stat_mode < DF_GN_SUMS || stat_mode > DF_GN_STALE) return DF_EINVAL;
  u->gn_mode = stat_mode;
  return DF_OK;
}

int df_unet_set_graph(df_unet* u, int on) {
  if (!u) return DF_EINVAL;
  u->use_graph = on != 0;
  return DF_OK;
}

int df_unet_profile_enable(df_unet* u, int on) {
  if (!u) return DF_EINVAL;
  u->prof.on = on != 0;
  return DF_OK;
}

int df_unet_profile_reset(df_unet* u) {
  if (!u) return DF_EINVAL;
  u->prof.reset();
  return DF_OK;
}

int df_unet_profile_num_classes(void) { return PC_COUNT; }

const char* df_unet_profile_class_name(int cls) { return (cls >= 0 && cls < PC_COUNT) ? kProfNames[cls] : ""; }

int df_unet_profile_num_kernels(df_unet* u) {
  if (!u) return DF_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return DF_EHIP;
  if (!u->prof.collect()) return DF_EHIP;
  return (int)u->prof.kernels.size();
}

int df_unet_profile_kernel(df_unet* u, int idx, char* label, int label_cap, int* cls, double* ms, double* flops,
                           double* bytes, long long* launches) {
  if (!u || !label || label_cap < 1 || !cls || !ms || !flops || !bytes || !launches) return DF_EINVAL;
  if (idx < 0 || idx >= (int)u->prof.kernels.size()) return DF_EINVAL;
  const ProfKernel& k = u->prof.kernels[idx];
  std::strncpy(label, k.label.c_str(), (size_t)label_cap - 1);
  label[label_cap - 1] = 0;
  *cls = k.cls; *ms = k.ms; *flops = k.flops; *bytes = k.bytes; *launches = k.launches;
  return DF_OK;
}

int df_unet_profile_read(df_unet* u, int cls, double* ms, double* flops, double* bytes, long long* launches) {
  if (!u || cls < 0 || cls >= PC_COUNT || !ms || !flops || !bytes || !launches) return DF_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return DF_EHIP;
  if (!u->prof.collect()) return DF_EHIP;
  *ms = u->prof.ms[cls]; *flops = u->prof.flops[cls]; *bytes = u->prof.bytes[cls]; *launches = u->prof.launches[cls];
  return DF_OK;
}

#pragma GCC visibility pop
}  // extern "C"
