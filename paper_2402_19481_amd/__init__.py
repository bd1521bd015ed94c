"""Thin Python binding of libdistrifusion.so (hand-written HIP for MI355X / gfx950).

Argument marshalling only: every function takes torch tensors that already
live on the GPU, passes their device pointers and the current HIP stream to
the C entry point of the same name, and raises on a non-zero return code.
PyTorch provides device memory and streams, nothing else.  There is no
fallback: if the shared library is missing or not built, importing a function
raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdistrifusion.so")

DF_F32, DF_BF16 = 0, 1
GN_SUMS, GN_EQ2, GN_SEPARATE, GN_STALE = 0, 1, 2, 3
SPLIT_ROWS, SPLIT_COLS = 0, 1
MODE_FULL, MODE_DISPLACED = 0, 1

_lib = None


class DfError(RuntimeError):
    pass


class UNetCfgC(ctypes.Structure):
    _fields_ = [("H", ctypes.c_int), ("W", ctypes.c_int), ("N", ctypes.c_int), ("B", ctypes.c_int),
                ("in_ch", ctypes.c_int), ("n_levels", ctypes.c_int), ("levels", ctypes.c_int * 4),
                ("depths", ctypes.c_int * 4), ("head_dim", ctypes.c_int), ("groups", ctypes.c_int),
                ("emb_dim", ctypes.c_int), ("text_len", ctypes.c_int), ("text_dim", ctypes.c_int),
                ("res_per_level", ctypes.c_int), ("split_axis", ctypes.c_int)]


def lib():
    """Loads the shared library once; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise DfError(f"{LIB_PATH} not found: run `python -c 'import __graft_entry__ as g; g.build()'` first")
    L = ctypes.CDLL(LIB_PATH)
    vp, i, f, ll, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_longlong, ctypes.c_size_t
    L.df_strerror.restype = ctypes.c_char_p
    L.df_strerror.argtypes = [i]
    L.df_copy_bytes.argtypes = [vp, vp, sz, vp]
    L.df_buffer_refresh.argtypes = [vp, vp, i, ll, i, i, i, vp]
    L.df_groupnorm_stale.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, i, i, i, vp]
    L.df_conv3x3_halo.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, vp]
    if hasattr(L, "df_groupnorm_stale_noalloc"):
        L.df_groupnorm_stale_noalloc.argtypes = L.df_groupnorm_stale.argtypes
        L.df_groupnorm_stale_noalloc.restype = i
    L.df_attn_displaced.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, f, i, vp]
    L.df_buffer_refresh_axis.argtypes = [vp, vp, i, i, ll, i, i, i, i, vp]
    L.df_conv3x3_halo_axis.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, vp]
    L.df_attn_displaced_axis.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, i, i, vp]
    for name in ("df_buffer_refresh_axis", "df_conv3x3_halo_axis", "df_attn_displaced_axis"):
        getattr(L, name).restype = i
    L.df_euler_update.argtypes = [vp, vp, f, f, ll, vp]
    L.df_linear.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, vp]
    L.df_scale_input.argtypes = [vp, vp, f, ll, vp]
    L.df_mfma_probe.argtypes = [vp, i, i, ctypes.POINTER(ctypes.c_double), vp]
    L.df_sync_probe_bytes.argtypes = [i]
    L.df_sync_probe_bytes.restype = sz
    L.df_sync_probe.argtypes = [vp, i, i, i, vp]
    L.df_sync_probe.restype = i
    L.df_attn_stale_vt.argtypes = [vp, vp, vp, vp, i, i, i, i, ll, f, i, vp]
    L.df_packed_text_kv_bytes.restype = sz
    L.df_packed_text_kv_bytes.argtypes = [i, i, i, i]
    L.df_pack_text_kv.argtypes = [vp, vp, i, i, i, i, vp]
    L.df_cross_attn_packed.argtypes = [vp, vp, vp, vp, f, vp, vp, i, i, i, i, i, i, f, vp]
    L.df_packed_bytes.restype = sz
    L.df_packed_bytes.argtypes = [ll, ll]
    L.df_pack_rows.argtypes = [vp, vp, i, i, vp]
    L.df_pack_linear_weight.argtypes = [vp, vp, vp, i, i, vp]
    L.df_linear_packed.argtypes = [vp, vp, vp, vp, vp, f, vp, vp, vp, vp, i, i, i, i, vp]
    cfgp = ctypes.POINTER(UNetCfgC)
    if not hasattr(L, "df_patch_unet_step"):
        raise DfError("libdistrifusion.so is stale: rebuild it")
    L.df_unet_num_weights.argtypes = [cfgp]
    L.df_unet_weight_info.argtypes = [cfgp, i, ctypes.c_char_p, i, ctypes.POINTER(i), ctypes.POINTER(ll)]
    L.df_unet_workspace_bytes.restype = sz
    L.df_unet_workspace_bytes.argtypes = [cfgp]
    L.df_unet_stale_bytes.restype = sz
    L.df_unet_stale_bytes.argtypes = [cfgp]
    L.df_unet_create.argtypes = [ctypes.POINTER(vp), cfgp, ctypes.POINTER(vp), i, vp, sz]
    L.df_unet_destroy.restype = None
    L.df_unet_destroy.argtypes = [vp]
    L.df_unet_stale_lookup.argtypes = [vp, ctypes.c_char_p, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.df_unet_num_stale.argtypes = [vp]
    L.df_unet_stale_name.argtypes = [vp, i, ctypes.c_char_p, i]
    L.df_patch_unet_step.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, vp]
    L.df_unet_profile_enable.argtypes = [vp, i]
    L.df_unet_set_graph.argtypes = [vp, i]
    L.df_unet_set_gn_mode.argtypes = [vp, i]
    L.df_unet_profile_reset.argtypes = [vp]
    L.df_unet_profile_num_classes.argtypes = []
    L.df_unet_profile_class_name.argtypes = [i]
    L.df_unet_profile_class_name.restype = ctypes.c_char_p
    dp = ctypes.POINTER(ctypes.c_double)
    L.df_unet_profile_read.argtypes = [vp, i, dp, dp, dp, ctypes.POINTER(ll)]
    L.df_unet_profile_num_kernels.argtypes = [vp]
    L.df_unet_profile_num_kernels.restype = i
    L.df_unet_profile_kernel.argtypes = [vp, i, ctypes.c_char_p, i, ctypes.POINTER(i), dp, dp, dp, ctypes.POINTER(ll)]
    L.df_unet_profile_kernel.restype = i
    for name in ("df_copy_bytes", "df_buffer_refresh", "df_groupnorm_stale", "df_conv3x3_halo", "df_attn_displaced",
                 "df_euler_update", "df_linear", "df_unet_set_gn_mode", "df_scale_input", "df_mfma_probe", "df_attn_stale_vt", "df_packed_text_kv_bytes", "df_pack_text_kv",
                 "df_cross_attn_packed", "df_packed_bytes", "df_pack_rows", "df_pack_linear_weight", "df_linear_packed", "df_unet_num_weights", "df_unet_weight_info", "df_unet_create",
                 "df_unet_stale_lookup", "df_unet_num_stale", "df_unet_stale_name", "df_patch_unet_step",
                 "df_unet_profile_enable", "df_unet_set_graph", "df_unet_profile_reset", "df_unet_profile_num_classes",
                 "df_unet_profile_read"):
        getattr(L, name).restype = i
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise DfError(f"libdistrifusion: {lib().df_strerror(rc).decode()} ({rc})")


def _dt(t):
    if t.dtype == torch.float32:
        return DF_F32
    if t.dtype == torch.bfloat16:
        return DF_BF16
    raise DfError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise DfError("tensors must be contiguous and on the GPU")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def copy_bytes(dst, src):
    _check(lib().df_copy_bytes(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream()))


def buffer_refresh(dst_full, src_patch, patch_idx, N):
    """dst_full [B, ...full...] <- src_patch [B, ...full/N...] at the patch's region (in place)."""
    B = dst_full.shape[0]
    _check(lib().df_buffer_refresh(_ptr(dst_full), _ptr(src_patch), B, dst_full.numel() // B, patch_idx, N,
                                   _dt(dst_full), _stream()))
    return dst_full


def groupnorm_stale(x_fresh, stale_stats, gamma, beta, G, patch_idx, N, eps=1e-5, stat_mode=GN_SUMS,
                    fuse_silu=False, fresh_stats_out=None):
    """Returns (y, fresh_stats [B,G,2])."""
    B, R, W, C = x_fresh.shape
    y = torch.empty_like(x_fresh)
    if fresh_stats_out is None:
        fresh_stats_out = torch.empty(B, G, 2, dtype=torch.float32, device=x_fresh.device)
    _check(lib().df_groupnorm_stale(_ptr(x_fresh), _ptr(y), _ptr(stale_stats), _ptr(fresh_stats_out), _ptr(gamma),
                                    _ptr(beta), B, R, W, C, G, patch_idx, N, eps, stat_mode, int(fuse_silu),
                                    _dt(x_fresh), _stream()))
    return y, fresh_stats_out


def groupnorm_stale_noalloc(x_fresh, stale_stats, gamma, beta, G, patch_idx, N, y, fresh_stats_out, eps=1e-5,
                            stat_mode=GN_SUMS, fuse_silu=False):
    """df_groupnorm_stale_noalloc: the caller passes every buffer (y, fresh_stats_out); nothing is allocated."""
    B, R, W, C = x_fresh.shape
    _check(lib().df_groupnorm_stale_noalloc(_ptr(x_fresh), _ptr(y), _ptr(stale_stats), _ptr(fresh_stats_out),
                                            _ptr(gamma), _ptr(beta), B, R, W, C, G, patch_idx, N, eps, stat_mode,
                                            int(fuse_silu), _dt(x_fresh), _stream()))
    return y, fresh_stats_out


def conv3x3_halo(x_fresh, stale_full, w, bias, patch_idx, N, stride=1, act=0):
    B, R, W, Cin = x_fresh.shape
    Cout = w.shape[0]
    H = R * N
    y = torch.empty(B, R // stride, W // stride, Cout, dtype=x_fresh.dtype, device=x_fresh.device)
    _check(lib().df_conv3x3_halo(_ptr(x_fresh), _ptr(stale_full), _ptr(w), _ptr(bias), _ptr(y), B, H, W, Cin, Cout,
                                 patch_idx, N, stride, act, _dt(x_fresh), _stream()))
    return y


def attn_displaced(q, k_fresh, v_fresh, k_stale, v_stale, heads, patch_idx, N, scale=None, out=None):
    B, Lq, C = q.shape
    d = C // heads
    L = Lq * N
    if scale is None:
        scale = d ** -0.5
    if out is None:
        out = torch.empty_like(q)
    _check(lib().df_attn_displaced(_ptr(q), _ptr(k_fresh), _ptr(v_fresh), _ptr(k_stale), _ptr(v_stale), _ptr(out), B,
                                   L, heads, d, patch_idx, N, scale, _dt(q), _stream()))
    return out


def buffer_refresh_cols(dst_full, src_patch, patch_idx, N):
    """dst_full [B, H, W, ...] <- src_patch [B, H, W/N, ...] at the patch's columns (in place)."""
    B, H = dst_full.shape[:2]
    _check(lib().df_buffer_refresh_axis(_ptr(dst_full), _ptr(src_patch), B, H, dst_full.numel() // (B * H), patch_idx, N,
                                        _dt(dst_full), SPLIT_COLS, _stream()))
    return dst_full


def conv3x3_halo_cols(x_fresh, stale_full, w, bias, patch_idx, N, stride=1, act=0):
    """Vertical strip: x_fresh [B, H, W/N, Cin], stale_full [B, H, W, Cin]."""
    B, H, Wp, Cin = x_fresh.shape
    Cout = w.shape[0]
    y = torch.empty(B, H // stride, Wp // stride, Cout, dtype=x_fresh.dtype, device=x_fresh.device)
    _check(lib().df_conv3x3_halo_axis(_ptr(x_fresh), _ptr(stale_full), _ptr(w), _ptr(bias), _ptr(y), B, H, Wp * N, Cin,
                                      Cout, patch_idx, N, stride, act, _dt(x_fresh), SPLIT_COLS, _stream()))
    return y


def attn_displaced_cols(q, k_fresh, v_fresh, k_stale, v_stale, heads, H, W, patch_idx, N, scale=None):
    """Vertical strip of an H x W token grid: q, k_fresh, v_fresh [B, H*W/N, C], k_stale, v_stale [B, H*W, C]."""
    B, Lq, C = q.shape
    d = C // heads
    if scale is None:
        scale = d ** -0.5
    out = torch.empty_like(q)
    _check(lib().df_attn_displaced_axis(_ptr(q), _ptr(k_fresh), _ptr(v_fresh), _ptr(k_stale), _ptr(v_stale), _ptr(out),
                                        B, H, W, heads, d, patch_idx, N, scale, _dt(q), SPLIT_COLS, _stream()))
    return out


def linear(x, w, bias=None, residual=None, out_dtype=torch.bfloat16, out=None):
    """x [M,K] bf16, w [N,K] bf16 -> [M,N] (+ bias + residual)."""
    M, K = x.shape
    N = w.shape[0]
    if out is None:
        out = torch.empty(M, N, dtype=out_dtype, device=x.device)
    _check(lib().df_linear(_ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(out), M, N, K, _dt(out), _stream()))
    return out


def attn_stale_vt(q, k, vt, heads, L, scale=None, packed=False):
    """q [B,Lq,C], k [B,L,C], vt [B,C,vt_ld] (values transposed) -> attention output, row-major [B,Lq,C] or packed."""
    B, Lq, C = q.shape
    if scale is None:
        scale = 64 ** -0.5
    if packed:
        out = torch.empty(lib().df_packed_bytes(B * Lq, C) // 2, dtype=torch.bfloat16, device=q.device)
    else:
        out = torch.empty_like(q)
    _check(lib().df_attn_stale_vt(_ptr(q), _ptr(k), _ptr(vt), _ptr(out), B, Lq, L, heads, vt.shape[2], scale,
                                  1 if packed else 0, _stream()))
    return out


def pack_text_kv(kv, B, text_len, count, C):
    """kv [B*text_len, count*2C] bf16 (projected text keys / values of `count` blocks) -> per-head MFMA fragments."""
    out = torch.empty(lib().df_packed_text_kv_bytes(B, text_len, count, C) // 2, dtype=torch.bfloat16, device=kv.device)
    _check(lib().df_pack_text_kv(_ptr(kv), _ptr(out), B, text_len, count, C, _stream()))
    return out


def cross_attn_packed(xp, wq_packed, ln_s, ln_t, text_kv_packed, B, rows_per_batch, C, text_len, count, block,
                      ln_eps=1e-5, scale=None):
    """Cross-attention fused into its LayerNorm-folded query projection; returns the packed output [B*rows, C]."""
    if scale is None:
        scale = 64 ** -0.5
    out = torch.empty(lib().df_packed_bytes(B * rows_per_batch, C) // 2, dtype=torch.bfloat16, device=xp.device)
    _check(lib().df_cross_attn_packed(_ptr(xp), _ptr(wq_packed), _ptr(ln_s), _ptr(ln_t), ln_eps, _ptr(text_kv_packed),
                                      _ptr(out), B, rows_per_batch, C, text_len, count, block, scale, _stream()))
    return out


def mfma_probe(blocks=2048, iters=4096):
    """Launches the register-resident MFMA loop; returns its flop count (time it with events)."""
    out = torch.empty(blocks, dtype=torch.float32, device="cuda")
    fl = ctypes.c_double()
    _check(lib().df_mfma_probe(_ptr(out), blocks, iters, ctypes.byref(fl), _stream()))
    return fl.value


def sync_probe(buf, blocks, iters, mode):
    """Runs the synchronisation probe (see the header); buf: zero-initialised uint8 tensor of sync_probe_bytes(blocks)."""
    _check(lib().df_sync_probe(_ptr(buf), blocks, iters, mode, _stream()))


def sync_probe_bytes(blocks):
    return lib().df_sync_probe_bytes(blocks)


def scale_input(x, sigma, out=None):
    """x / sqrt(sigma^2 + 1): the sampler's scaling of the model input."""
    if out is None:
        out = torch.empty_like(x)
    _check(lib().df_scale_input(_ptr(out), _ptr(x), float(sigma), x.numel(), _stream()))
    return out


def pack_rows(x):
    """x [M,K] bf16 row-major -> fragment-packed copy (int16 tensor of df_packed_bytes/2 elements)."""
    M, K = x.shape
    out = torch.empty(lib().df_packed_bytes(M, K) // 2, dtype=torch.bfloat16, device=x.device)
    _check(lib().df_pack_rows(_ptr(x), _ptr(out), M, K, _stream()))
    return out


def pack_linear_weight(w, gamma=None):
    """w [N,K] bf16 -> fragment-packed weights (rows permuted inside each 32-row fragment, optional column scale)."""
    N, K = w.shape
    out = torch.empty(N * K, dtype=torch.bfloat16, device=w.device)
    _check(lib().df_pack_linear_weight(_ptr(w), _ptr(gamma), _ptr(out), N, K, _stream()))
    return out


def linear_packed(xp, wp, M, N, K, bias=None, ln_s=None, ln_t=None, ln_eps=1e-5, residual=None, geglu=False,
                  want=("f32",)):
    """Linear layer on packed operands; returns a dict of the requested outputs: "f32" [M,N'] float row-major,
    "packed" packed bf16, "rows" [M,N'] bf16 row-major (N' = N/2 with geglu)."""
    No = N // 2 if geglu else N
    dev = xp.device
    outs = {}
    if "f32" in want:
        outs["f32"] = torch.empty(M, No, dtype=torch.float32, device=dev)
    if "packed" in want:
        outs["packed"] = torch.empty(lib().df_packed_bytes(M, No) // 2, dtype=torch.bfloat16, device=dev)
    if "rows" in want:
        outs["rows"] = torch.empty(M, No, dtype=torch.bfloat16, device=dev)
    _check(lib().df_linear_packed(_ptr(xp), _ptr(wp), _ptr(bias), _ptr(ln_s), _ptr(ln_t), ln_eps, _ptr(residual),
                                  _ptr(outs.get("f32")), _ptr(outs.get("packed")), _ptr(outs.get("rows")), M, N, K,
                                  1 if geglu else 0, _stream()))
    return outs


def euler_update(x, eps, sigma, sigma_next):
    _check(lib().df_euler_update(_ptr(x), _ptr(eps), sigma, sigma_next, x.numel(), _stream()))
    return x


def make_cfg(cfg, B=1, split_axis=SPLIT_ROWS):
    """df_inputs.unet_table.UNetCfg (or anything with the same fields) -> C struct."""
    c = UNetCfgC()
    c.H, c.W, c.N, c.B, c.in_ch = cfg.H, cfg.W, cfg.N, B, cfg.in_ch
    c.n_levels = len(cfg.levels)
    for k in range(c.n_levels):
        c.levels[k] = cfg.levels[k]
        c.depths[k] = cfg.depths[k]
    c.head_dim, c.groups, c.emb_dim = cfg.head_dim, cfg.groups, cfg.emb_dim
    c.text_len, c.text_dim, c.res_per_level = cfg.text_len, cfg.text_dim, cfg.res_per_level
    c.split_axis = split_axis
    return c


def unet_weight_specs(ccfg):
    """[(name, shape)] of the parameters the plan expects, in order."""
    L = lib()
    n = L.df_unet_num_weights(ctypes.byref(ccfg))
    if n < 0:
        _check(n)
    out = []
    buf = ctypes.create_string_buffer(128)
    nd = ctypes.c_int()
    dims = (ctypes.c_longlong * 4)()
    for k in range(n):
        _check(L.df_unet_weight_info(ctypes.byref(ccfg), k, buf, 128, ctypes.byref(nd), dims))
        out.append((buf.value.decode(), tuple(int(dims[j]) for j in range(nd.value))))
    return out


class PatchUNet:
    """Owns the plan, its workspace and the stale-state blob of one UNet on one GPU."""

    def __init__(self, cfg, weights, B=1, device="cuda:0", split_axis=SPLIT_ROWS):
        """weights: list of device tensors in `unet_weight_specs` order (bf16 matrices, float vectors).
        split_axis: SPLIT_ROWS (horizontal strips) or SPLIT_COLS (vertical strips)."""
        L = lib()
        self.cfg, self.ccfg, self.B, self.split_axis = cfg, make_cfg(cfg, B, split_axis), B, split_axis
        self.device = torch.device(device)
        self.weights = list(weights)
        specs = unet_weight_specs(self.ccfg)
        if len(specs) != len(self.weights):
            raise DfError("wrong number of weight tensors")
        for (name, shape), w in zip(specs, self.weights):
            want = torch.bfloat16 if len(shape) > 1 else torch.float32
            if tuple(w.shape) != shape or w.dtype != want or not w.is_cuda or not w.is_contiguous():
                raise DfError(f"weight {name}: expected {shape} {want}, got {tuple(w.shape)} {w.dtype}")
        ws = L.df_unet_workspace_bytes(ctypes.byref(self.ccfg))
        ss = L.df_unet_stale_bytes(ctypes.byref(self.ccfg))
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=self.device)
        self.stale = torch.zeros(ss, dtype=torch.uint8, device=self.device)
        arr = (ctypes.c_void_p * len(self.weights))(*[w.data_ptr() for w in self.weights])
        h = ctypes.c_void_p()
        _check(L.df_unet_create(ctypes.byref(h), ctypes.byref(self.ccfg), arr, len(self.weights),
                                self.workspace.data_ptr(), ws))
        self.handle = h

    def step(self, x, emb, text, patch_idx=0, mode=MODE_DISPLACED, refresh=True, out=None):
        if out is None:
            out = torch.empty_like(x)
        _check(lib().df_patch_unet_step(self.handle, _ptr(x), _ptr(emb), _ptr(text), self.stale.data_ptr(), _ptr(out),
                                        patch_idx, mode, int(refresh), _stream()))
        return out

    def set_gn_mode(self, stat_mode):
        """GroupNorm statistic mode of the displaced steps (GN_SUMS default, GN_EQ2, GN_SEPARATE, GN_STALE)."""
        _check(lib().df_unet_set_gn_mode(self.handle, int(stat_mode)))

    def _loop_buffer(self, key, shape):
        """Persistent float buffers of the sampling loop: the step's graph cache is keyed on its pointers, so the
        scaled input and the eps output must live at the same addresses in every step for the graph to replay."""
        bufs = self.__dict__.setdefault("_loop_bufs", {})
        k = (key, tuple(shape))
        if k not in bufs:
            bufs[k] = torch.empty(shape, dtype=torch.float32, device=self.device)
        return bufs[k]

    def sample_patch(self, x_full, emb, text, sigmas, patch_idx, n_warmup=1):
        """Euler sampling loop of one device: `n_warmup` synchronous steps on the whole latent (they fill the stale
        state; the paper runs the first steps this way), then displaced steps that advance the rows of patch
        `patch_idx` only and refresh its slots of the stale state.  x_full [B,H,W,4] float is updated in place (all rows
        during warm-up, then the patch's rows); every arithmetic step runs in the library.  Returns the list of the
        per-step eps tensors (full image for warm-up steps, patch rows afterwards).  The scaled input and the eps
        output of the displaced steps sit in buffers the object keeps, so from the third displaced step on the whole
        UNet step is one HIP-graph replay."""
        B, H, W, C = x_full.shape
        if self.split_axis == SPLIT_COLS:
            Wp = W // self.cfg.N
            region = (slice(None), slice(None), slice(patch_idx * Wp, (patch_idx + 1) * Wp))
            pshape = (B, H, Wp, C)
        else:
            R = H // self.cfg.N
            region = (slice(None), slice(patch_idx * R, (patch_idx + 1) * R))
            pshape = (B, R, W, C)
        eps_all = []
        xin_full, eps_full = self._loop_buffer("xin_full", x_full.shape), self._loop_buffer("eps_full", x_full.shape)
        xin, eps_p = self._loop_buffer("xin", pshape), self._loop_buffer("eps", pshape)
        xp = x_full[region]
        own = xp.is_contiguous()                       # B == 1, horizontal strips: the patch is one block of x_full
        if not own:
            xp = self._loop_buffer("xp", pshape)
            xp.copy_(x_full[region])
        for k in range(len(sigmas) - 1):
            s0, s1 = float(sigmas[k]), float(sigmas[k + 1])
            if k < n_warmup:
                eps = self.step(scale_input(x_full, s0, out=xin_full), emb, text, 0, MODE_FULL, True, out=eps_full)
                euler_update(x_full, eps, s0, s1)
                if not own:
                    xp.copy_(x_full[region])
            else:
                eps = self.step(scale_input(xp, s0, out=xin), emb, text, patch_idx, MODE_DISPLACED, True, out=eps_p)
                euler_update(xp, eps, s0, s1)
                if not own and self.split_axis == SPLIT_COLS:
                    buffer_refresh_cols(x_full, xp, patch_idx, self.cfg.N)
                elif not own:
                    buffer_refresh(x_full, xp, patch_idx, self.cfg.N)
            eps_all.append(eps.clone())
        return eps_all

    def set_graph(self, on):
        """Switches HIP-graph replay of repeated steps on (default) or off."""
        _check(lib().df_unet_set_graph(self.handle, int(on)))

    def profile(self, on):
        """Switches per-launch event timing of the steps on or off (resets the totals)."""
        _check(lib().df_unet_profile_enable(self.handle, int(on)))
        _check(lib().df_unet_profile_reset(self.handle))

    def profile_read(self):
        """{class name: dict(ms, flops, bytes, launches)} accumulated since profiling was switched on."""
        L = lib()
        out = {}
        for k in range(L.df_unet_profile_num_classes()):
            ms, fl, by, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_double(), ctypes.c_longlong()
            _check(L.df_unet_profile_read(self.handle, k, ctypes.byref(ms), ctypes.byref(fl), ctypes.byref(by),
                                          ctypes.byref(n)))
            out[L.df_unet_profile_class_name(k).decode()] = dict(ms=ms.value, flops=fl.value, bytes=by.value,
                                                                 launches=n.value)
        return out

    def profile_kernels(self):
        """[dict(label, cls, ms, flops, bytes, launches)] per kernel (one operation at one shape) since profiling was
        switched on."""
        L = lib()
        n = L.df_unet_profile_num_kernels(self.handle)
        if n < 0:
            _check(n)
        out = []
        buf = ctypes.create_string_buffer(160)
        for k in range(n):
            cls, ms, fl, by, cnt = (ctypes.c_int(), ctypes.c_double(), ctypes.c_double(), ctypes.c_double(),
                                    ctypes.c_longlong())
            _check(L.df_unet_profile_kernel(self.handle, k, buf, 160, ctypes.byref(cls), ctypes.byref(ms),
                                            ctypes.byref(fl), ctypes.byref(by), ctypes.byref(cnt)))
            out.append(dict(label=buf.value.decode(), cls=L.df_unet_profile_class_name(cls.value).decode(),
                            ms=ms.value, flops=fl.value, bytes=by.value, launches=cnt.value))
        return out

    def stale_names(self):
        L = lib()
        buf = ctypes.create_string_buffer(128)
        out = []
        for k in range(L.df_unet_num_stale(self.handle)):
            _check(L.df_unet_stale_name(self.handle, k, buf, 128))
            out.append(buf.value.decode())
        return out

    def stale_view(self, name):
        """uint8 view of one named stale buffer inside the blob."""
        off, nb = ctypes.c_size_t(), ctypes.c_size_t()
        _check(lib().df_unet_stale_lookup(self.handle, name.encode(), ctypes.byref(off), ctypes.byref(nb)))
        return self.stale[off.value:off.value + nb.value]

    def close(self):
        if getattr(self, "handle", None):
            lib().df_unet_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
