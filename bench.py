#!/usr/bin/env python3
"""Benchmark of the displaced-patch UNet step on one MI355X.

A step is one pass of the whole hot path for one patch: df_patch_unet_step in
DISPLACED mode with refresh (GroupNorm with stale statistics, 3x3 convolutions
with stale halo rows, self-attention against spliced fresh/stale K/V, all
per-token layers, and the refresh of the patch's rows of every stale buffer).
Workload: SDXL-shaped UNet, 1280x1920 image (160x240 latent), N=8 row patches,
patch 3, batch 1, bf16 with float accumulation, seeded synthetic inputs and
random-init weights.  The stale state is left by one untimed FULL step.

Prints one JSON line: metric, value (ms per step), roofline of the dominant kernel class, per-class breakdown,
and the CPU oracle's time for the same step.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


TRAFFIC_PROFILE = os.path.join("profiles", "unet_step_cfg4_hbm_traffic.md")


def traffic_from_profile(cls=None, kernel=None):
    """HBM bytes of a kernel class per step, or of one kernel per launch, as the committed rocprofv3 --pmc summary of
    this command states them (FETCH_SIZE + WRITE_SIZE, calibrated with `bench.py --calibrate-copy`), or None.  Counter
    runs are separate profiler runs by nature, so this is never a measurement of the present run and is labelled so."""
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_PROFILE)):
            f = line.split()
            if cls and len(f) == 3 and f[0] == "traffic_per_step_bytes" and f[1] == cls:
                return float(f[2])
            if kernel and len(f) > 2 and f[0] == "traffic_per_launch_bytes" and " ".join(f[2:]) == kernel:
                return float(f[1])
    except OSError:
        pass
    return None


def calibrate_copy(df, torch, mib, reps):
    """Plain copies of a known size through the library's copy kernel (df_copy_bytes), for calibrating the
    FETCH_SIZE / WRITE_SIZE counters: run under `rocprofv3 --pmc FETCH_SIZE` (then WRITE_SIZE) and divide the
    counter's KiB per dispatch of `copy_rows_vec16` by the KiB this prints."""
    n = mib << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    dst = torch.empty_like(src)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        df.copy_bytes(dst, src)
        st.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(reps):
            df.copy_bytes(dst, src)
        e1.record(st)
        e1.synchronize()
    assert torch.equal(dst, src)
    us = e0.elapsed_time(e1) * 1e3 / reps
    print(json.dumps({"op": "calibrate_copy", "kernel": "copy_rows_vec16", "dispatches": reps + 1,
                      "read_KiB_per_dispatch": n // 1024, "written_KiB_per_dispatch": n // 1024,
                      "us_per_dispatch": round(us, 2), "gbs": round(2.0 * n / us / 1e3, 1)}), flush=True)


def run_loop(df, torch, net, cfg, patch, steps, emb, text, workload):
    """The multi-step configuration: `steps` Euler steps on a fixed sigma ladder, step 0 FULL on the whole latent,
    then DISPLACED + refresh on the patch's rows (Section 4: the first step is synchronous), the scaled input and the
    eps output at fixed addresses so that the displaced steps replay one HIP graph.  Per-step times from HIP events
    on the stream the steps run on; one untimed pass of the loop first (it records the graph)."""
    sig = [14.6 * (0.03 / 14.6) ** (k / steps) for k in range(steps + 1)]
    R = cfg.H // cfg.N
    g = torch.Generator(device="cuda:0").manual_seed(41)
    x0 = torch.randn(1, cfg.H, cfg.W, cfg.in_ch, generator=g, device="cuda:0") * sig[0]
    st = torch.cuda.Stream()
    times = None
    with torch.cuda.stream(st):
        for rep in range(2):
            x_full = x0.clone()
            xp = x_full[:, patch * R:(patch + 1) * R]
            xin_full, eps_full = torch.empty_like(x_full), torch.empty_like(x_full)
            if rep == 0:
                xin, eps = torch.empty_like(xp), torch.empty_like(xp)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            st.synchronize()
            t0 = time.perf_counter()
            for k in range(steps):
                ev[k].record(st)
                if k == 0:
                    net.step(df.scale_input(x_full, sig[0], out=xin_full), emb, text, 0, df.MODE_FULL, True, out=eps_full)
                    df.euler_update(x_full, eps_full, sig[0], sig[1])
                else:
                    net.step(df.scale_input(xp, sig[k], out=xin), emb, text, patch, df.MODE_DISPLACED, True, out=eps)
                    df.euler_update(xp, eps, sig[k], sig[k + 1])
            ev[steps].record(st)
            st.synchronize()
            wall = (time.perf_counter() - t0) * 1e3
            times = [ev[k].elapsed_time(ev[k + 1]) for k in range(steps)]
        assert bool(torch.isfinite(x_full).all())
    disp = times[1:]
    from df_inputs import unet_table as ut
    tflop = 2.0 * ut.count_macs(cfg)["total"] / 1e12
    print(json.dumps({
        "metric": "ms per patch UNet step (1 MI355X), multi-step loop", "value": round(sum(disp) / len(disp), 4),
        "unit": "ms", "n_gpus": 1, "steps": steps, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload + ", %d-step Euler loop (step 0 FULL, then DISPLACED + refresh)" % steps},
        "ms_per_step_list": [round(t, 3) for t in times], "full_first_step_ms": round(times[0], 3),
        "displaced_step_ms_mean": round(sum(disp) / len(disp), 4), "displaced_step_ms_max": round(max(disp), 4),
        "loop_wall_ms": round(wall, 3), "tflop_per_displaced_step": round(tflop, 4),
        "displaced_tflops": round(tflop / (sum(disp) / len(disp) * 1e-3), 2)}), flush=True)


def make_weights(df, torch, ccfg, seed):
    g = torch.Generator(device="cuda:0").manual_seed(seed)
    out = []
    for name, shape in df.unet_weight_specs(ccfg):
        x = torch.randn(shape, generator=g, device="cuda:0", dtype=torch.float32)
        if name.endswith(".w"):
            fan_in = 1
            for d in shape[1:]:
                fan_in *= d
            out.append((x * fan_in ** -0.5).to(torch.bfloat16).contiguous())
        elif name.endswith(".g"):
            out.append(1.0 + 0.1 * x)
        elif name.endswith(".beta"):
            out.append(0.1 * x)
        else:
            out.append(0.02 * x)
    return out


def cpu_baseline(cfg, weights_dev, specs, inputs, patch):
    """Times the CPU oracle (as it stands) on one DISPLACED step of the same configuration."""
    import numpy as np
    import torch
    from df_inputs import unet_table as ut
    from oracle import unet as ounet

    named = []
    for (name, _), w in zip(specs, weights_dev):
        if w.dtype == torch.bfloat16:
            named.append((name, w.view(torch.int16).cpu().numpy().view(np.uint16)))
        else:
            named.append((name, w.cpu().numpy()))
    P = ounet.Params(named)
    bl = ut.blocks(cfg)
    # zero-filled stale buffers of the right shapes (their content does not change the work done)
    stale = {}
    G, N = cfg.groups, cfg.N
    for b in bl:
        k = b[0]
        if k == "conv_in":
            stale[b[1] + ".in"] = np.zeros((1, cfg.H, cfg.W, b[2]))
        elif k == "res":
            _, nm, cin, cout, lv, _ = b
            h, w = cfg.level_hw(lv)
            stale[nm + ".conv1.in"] = np.zeros((1, h, w, cin))
            stale[nm + ".conv2.in"] = np.zeros((1, h, w, cout))
            stale[nm + ".gn1.stats"] = np.ones((N, 1, G, 2))
            stale[nm + ".gn2.stats"] = np.ones((N, 1, G, 2))
        elif k == "xf":
            _, nm, c, depth, lv = b
            h, w = cfg.level_hw(lv)
            stale[nm + ".gn.stats"] = np.ones((N, 1, G, 2))
            for d in range(depth):
                stale[f"{nm}.b{d}.attn1.k"] = np.zeros((1, h * w, c))
                stale[f"{nm}.b{d}.attn1.v"] = np.zeros((1, h * w, c))
        elif k == "down":
            h, w = cfg.level_hw(b[3])
            stale[b[1] + ".in"] = np.zeros((1, h, w, b[2]))
        elif k == "up":
            h, w = cfg.level_hw(b[3] - 1)
            stale[b[1] + ".in"] = np.zeros((1, h, w, b[2]))
        elif k == "out":
            stale[b[1] + ".gn.stats"] = np.ones((N, 1, G, 2))
            stale[b[1] + ".conv.in"] = np.zeros((1, cfg.H, cfg.W, b[2]))
    x, emb, text = inputs
    t0 = time.perf_counter()
    ounet.unet_step(cfg, bl, P, x, emb, text, stale, patch, ounet.DISPLACED, refresh=True)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    return dict(value=round(dt * 1e3, 1), unit="ms", cores=int(cores), kind="oracle",
                sample="one DISPLACED step of the same configuration (float64 numpy oracle, zero-filled stale buffers)")


def measured_mfma_peak(df, torch):
    """TFLOP/s of the library's register-resident bf16 MFMA loop, timed with events on a side stream."""
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        df.mfma_probe(2048, 2048)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        fl = df.mfma_probe(2048, 8192)
        e1.record(st)
        e1.synchronize()
    return round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)


def run_tile_sweep(df, torch):
    """Every tile shape / ring depth of the LDS-tiled MFMA kernel on convolution and linear shapes of the larger
    workloads (2048x2048 and 3840x3840 shares, the synchronous full-image step), no split along K.  Needs the tuning
    build (python -m paper_2402_19481_amd.build --tuning): the library proper has no override switches.  One JSON
    line per shape: microseconds and TFLOP/s per tile configuration ("auto" = the library's own choice)."""
    import math
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(1)
    bf = lambda t: t.to(torch.bfloat16).contiguous()
    rn = lambda *s: torch.randn(*s, generator=g, device=dev)
    stream = torch.cuda.Stream()

    def timed(fn, rep=20):
        with torch.cuda.stream(stream):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            stream.synchronize()
            e0.record(stream)
            for _ in range(rep):
                fn()
            e1.record(stream)
            e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / rep

    tiles = ["", "64x64x2", "64x64x3", "64x64x7", "64x64x6", "128x64x3", "128x64x7", "64x128x2", "128x128x2", "128x128x3", "128x128x7", "128x128x6"]
    convs = [("conv 32x128 320->320 (configuration 3)", 32, 128, 320, 320), ("conv 64x256 320->320", 64, 256, 320, 320),
             ("conv 64x256 960->320", 64, 256, 960, 320), ("conv 32x128 640->640", 32, 128, 640, 640),
             ("conv 32x128 1920->640", 32, 128, 1920, 640), ("conv 16x64 1280->1280", 16, 64, 1280, 1280),
             ("conv 160x240 320->320 (full image)", 160, 240, 320, 320)]
    gemms = [("linear 4096x640x640", 4096, 640, 640), ("linear 4096x1920x640", 4096, 1920, 640),
             ("linear 4096x640x2560", 4096, 640, 2560), ("linear 4096x5120x640", 4096, 5120, 640),
             ("linear 9600x640x640 (full image)", 9600, 640, 640), ("linear 2400x1280x1280 (full image)", 2400, 1280, 1280),
             ("linear 2400x1280x5120 (full image)", 2400, 1280, 5120), ("linear 38400x320x960 (full image)", 38400, 320, 960)]
    os.environ["DF_TUNE"] = "1"

    def sweep(name, flops, fn):
        rec = {"op": name, "gflop": round(flops / 1e9, 2)}
        for t in tiles:
            if t:
                os.environ["DF_TILE"] = t
            else:
                os.environ.pop("DF_TILE", None)
            us = timed(fn)
            rec[t or "auto"] = {"us": round(us, 1), "tflops": round(flops / us / 1e6)}
        print(json.dumps(rec), flush=True)

    for name, R, W, Cin, Cout in convs:
        x, st = bf(rn(1, R, W, Cin)), bf(rn(1, R * 4, W, Cin))
        w, b = bf(rn(Cout, 3, 3, Cin) / math.sqrt(9 * Cin)), rn(Cout)
        sweep(name, 2.0 * 9 * Cin * Cout * R * W, lambda: df.conv3x3_halo(x, st, w, b, 1, 4))
    for name, M, N, K in gemms:
        x, w, b = bf(rn(M, K)), bf(rn(N, K) / math.sqrt(K)), rn(N)
        sweep(name, 2.0 * M * N * K, lambda: df.linear(x, w, b))


def run_timeline(df, torch, tune_path):
    """In-kernel timelines from the tuning build (cycle stamps written by the kernels themselves): where a k-slab of the
    LDS-tiled MFMA kernel spends its cycles, and how a wave-level linear layer of the patch step divides into
    prologue, K loop and reduction + epilogue.  One JSON line per case."""
    import ctypes
    import math
    import statistics
    lib = ctypes.CDLL(tune_path)
    dev = "cuda:0"
    g = torch.Generator(device="cpu").manual_seed(1)
    rn = lambda *s: torch.randn(*s, generator=g).to(dev)
    bf = lambda t: t.to(torch.bfloat16)
    os.environ["DF_TUNE"] = "1"

    def pipe(name, fn, tile, KT):
        os.environ["DF_TILE"] = tile
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        n = 8 + 4 * KT
        buf = (ctypes.c_longlong * n)()
        if lib.df_tune_pipe_trace(buf, n) != 0:
            raise RuntimeError("df_tune_pipe_trace failed")
        t = list(buf)
        ph = [(t[8 + 4 * k + 1] - t[8 + 4 * k], t[8 + 4 * k + 2] - t[8 + 4 * k + 1], t[8 + 4 * k + 3] - t[8 + 4 * k + 2],
               (t[8 + 4 * (k + 1)] if k + 1 < KT else t[2]) - t[8 + 4 * k + 3]) for k in range(KT)]
        mid = ph[3:-2] if KT > 8 else ph
        m = [round(statistics.mean(x[i] for x in mid)) for i in range(4)]
        print(json.dumps({"kernel": "mfma_pipe_kernel", "op": name, "tile": tile, "k_slabs": KT,
                          "cycles_before_first_slab": t[8] - t[0], "cycles_k_loop": t[2] - t[8],
                          "per_slab_cycles": {"wait_own_loads": m[0], "barrier": m[1], "issue_loads_and_lds_reads": m[2],
                                              "mfma": m[3], "total": sum(m)},
                          "note": "each of the four stamps of a slab costs ~90 cycles itself"}), flush=True)

    M, N, K = 2400, 1280, 5120
    x, w, b = bf(rn(M, K)), bf(rn(N, K) / math.sqrt(K)), rn(N)
    for tile in ("64x64x2", "128x128x3", "128x128x7"):
        pipe("linear 2400x1280x5120", lambda: df.linear(x, w, b), tile, K // 64)
    R, W, Cin, Cout = 64, 256, 960, 320
    x2, st = bf(rn(1, R, W, Cin)), bf(rn(1, R * 4, W, Cin))
    w2, b2 = bf(rn(Cout, 3, 3, Cin) / math.sqrt(9 * Cin)), rn(Cout)
    for tile in ("64x64x3", "128x128x7"):
        pipe("conv 64x256 960->320", lambda: df.conv3x3_halo(x2, st, w2, b2, 1, 4), tile, 9 * Cin // 64)
    os.environ.pop("DF_TILE", None)

    def wgemm(name, fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        n = 1024 * 16
        buf = (ctypes.c_longlong * n)()
        if lib.df_tune_wgemm_trace(buf, n) != 0:
            raise RuntimeError("df_tune_wgemm_trace failed")
        t = [list(buf[i * 16:(i + 1) * 16]) for i in range(1024)]
        smax = max(r[0] for r in t)
        t = [r for r in t if r[0] > smax - 100000 and r[5] >= r[0]]   # this launch's workgroups (100 MHz clock: 1 ms)
        s0 = min(r[0] for r in t)
        mean = lambda v: round(statistics.mean(v))
        print(json.dumps({"kernel": "wgemm_kernel", "op": name, "workgroups": len(t),
                          "first_start_to_last_end_us": round((max(r[5] for r in t) - s0) / 100.0, 2),
                          "last_start_us": round((max(r[0] for r in t) - s0) / 100.0, 2),
                          "cycles": {"prologue": mean([r[2] - r[1] for r in t]),
                                     "prologue_tile_indices": mean([r[6] - r[1] for r in t]),
                                     "prologue_epilogue_operand_requests": mean([r[7] - r[6] for r in t]),
                                     "prologue_first_operand_requests": mean([r[2] - r[7] for r in t]),
                                     "k_loop": mean([r[3] - r[2] for r in t]),
                                     "reduce_and_epilogue": mean([r[4] - r[3] for r in t]),
                                     # passes of the epilogue: partial tiles to LDS + barrier, then the wave's units
                                     "epilogue_pass0_to_lds": mean([r[8] - r[3] for r in t]),
                                     "epilogue_pass0_units": mean([r[9] - r[8] for r in t]),
                                     "epilogue_later_passes": mean([r[4] - r[9] for r in t])}}), flush=True)

    M = 300
    for name, N, K, geglu, ln in (("linear_packed 300x10240x1280 geglu ln", 10240, 1280, True, True),
                                  ("linear_packed 300x1280x5120", 1280, 5120, False, False),
                                  ("linear_packed 300x1280x1280", 1280, 1280, False, False),
                                  ("linear_packed 300x3840x1280 ln", 3840, 1280, False, True)):
        xw, ww, bw = bf(rn(M, K)), bf(rn(N, K) / math.sqrt(K)), rn(N)
        xp, wp = df.pack_rows(xw), df.pack_linear_weight(ww)
        kw = dict(geglu=geglu, want=("packed",))
        if ln:
            kw.update(ln_s=rn(N), ln_t=rn(N))
        else:
            kw.update(bias=bw)
        wgemm(name, lambda: df.linear_packed(xp, wp, M, N, K, **kw))

    # self-attention of the deepest level (300 queries x 2400 keys x 20 heads): waves 0 and 5 of every workgroup
    B, Lq, L, heads = 1, 300, 2400, 20
    q, k = bf(rn(B, Lq, heads * 64)), bf(rn(B, L, heads * 64))
    vt = bf(rn(B, heads * 64, (L + 63) // 64 * 64))
    for _ in range(4):
        df.attn_stale_vt(q, k, vt, heads, L, packed=True)
    torch.cuda.synchronize()
    n = 512 * 32
    buf = (ctypes.c_longlong * n)()
    if lib.df_tune_attn_trace(buf, n) != 0:
        raise RuntimeError("df_tune_attn_trace failed")
    mean = lambda v: round(statistics.mean(v))
    for wv, off in ((0, 0), (5, 256)):
        t = [r for r in (list(buf[(off + i) * 32:(off + i + 1) * 32]) for i in range(256)) if r[31] > 0 and r[30] > 0]
        s0 = min(r[0] for r in t)
        tiles = []
        for i in range(max(r[31] for r in t)):
            rows = [r for r in t if r[31] > i]
            prev = (lambda r: r[2]) if i == 0 else (lambda r, i=i: r[5 + 3 * (i - 1)])
            tiles.append({"wait_loads": mean([r[3 + 3 * i] - prev(r) for r in rows]),
                          "lds_to_registers": mean([r[4 + 3 * i] - r[3 + 3 * i] for r in rows]),
                          "issue_next_and_compute": mean([r[5 + 3 * i] - r[4 + 3 * i] for r in rows])})
        print(json.dumps({"kernel": "attn_wave_d64", "op": "self_attn 300x2400x1280", "wave": wv, "workgroups": len(t),
                          "first_start_to_last_end_us": round((max(r[30] for r in t) - s0) / 100.0, 2),
                          "cycles": {"prologue": mean([r[2] - r[1] for r in t]), "tiles": tiles,
                                     "wait_for_slowest_wave": mean([r[28] - r[5 + 3 * (r[31] - 1)] for r in t]),
                                     "merge_and_store": mean([r[29] - r[28] for r in t]),
                                     "total": mean([r[29] - r[1] for r in t])}}), flush=True)

    # self-attention of the middle level (1200 queries x 9600 keys x 10 heads): the LDS-shared kernel, wave 0 of the
    # first 256 workgroups, first eight iterations (128 keys each: one 64-key tile per wave group)
    B, Lq, L, heads = 1, 1200, 9600, 10
    q, k = bf(rn(B, Lq, heads * 64)), bf(rn(B, L, heads * 64))
    vt = bf(rn(B, heads * 64, (L + 63) // 64 * 64))
    for _ in range(4):
        df.attn_stale_vt(q, k, vt, heads, L, packed=True)
    torch.cuda.synchronize()
    if lib.df_tune_attn_trace(buf, n) != 0:
        raise RuntimeError("df_tune_attn_trace failed")
    t = [r for r in (list(buf[i * 32:(i + 1) * 32]) for i in range(256)) if r[31] > 0 and r[30] > 0]
    s0 = min(r[0] for r in t)
    its = min(8, t[0][31])
    print(json.dumps({"kernel": "attn_vt_d64<2, 2>", "op": "self_attn 1200x9600x640", "workgroups_traced": len(t),
                      "iterations_per_workgroup": t[0][31],
                      "first_start_to_last_traced_end_us": round((max(r[30] for r in t) - s0) / 100.0, 2),
                      "cycles": {"prologue": mean([r[2] - r[1] for r in t]),
                                 "per_iteration": {
                                     "wait_own_loads": mean([r[4 + 3 * i] - r[3 + 3 * i] for r in t for i in range(1, its)]),
                                     "barrier": mean([r[5 + 3 * i] - r[4 + 3 * i] for r in t for i in range(1, its)]),
                                     "tile_body": mean([r[3 + 3 * (i + 1)] - r[5 + 3 * i] for r in t for i in range(1, its - 1)])},
                                 "to_loop_end": mean([r[28] - r[1] for r in t]),
                                 "merge_of_the_two_groups": mean([r[29] - r[28] for r in t])}}), flush=True)


def run_ops(df, torch):
    """Single operations at the shapes of configurations 2, 3 and 5 plus the two ceilings (register-resident MFMA
    loop, plain copy).  Every case runs REP times back to back on a side stream; the time is the HIP-event span divided
    by REP, so cases shorter than ~10 us are bounded by the host's launch rate - the committed rocprofv3 kernel trace
    of this command has the per-kernel durations.  One JSON line per case."""
    import math
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(2)
    rn = lambda *sh, std=1.0: torch.randn(*sh, generator=g, device=dev) * std
    bf = lambda t: t.to(torch.bfloat16).contiguous()
    stream = torch.cuda.Stream()
    REP = 20

    def timed(name, fn, flops=None, nbytes=None, note=None):
        with torch.cuda.stream(stream):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            stream.synchronize()
            e0.record(stream)
            for _ in range(REP):
                fn()
            e1.record(stream)
            e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / REP
        rec = {"op": name, "us": round(us, 2)}
        if flops:
            rec["tflops"] = round(flops / us / 1e6, 2)
            rec["frac_of_bf16_mfma_peak"] = round(flops / us / 1e6 / 2500.0, 4)
        if nbytes:
            rec["gbs"] = round(nbytes / us / 1e3, 1)
            rec["frac_of_hbm_peak"] = round(nbytes / us / 1e3 / 8000.0, 4)
        if note:
            rec["note"] = note
        print(json.dumps(rec), flush=True)

    # ceilings
    fl = [0.0]
    def probe():
        fl[0] = df.mfma_probe(2048, 8192)
    probe()
    timed("mfma_probe_register_resident", probe, flops=fl[0])
    # what a grid-wide wait costs: kernel boundary vs fenced in-kernel barrier vs fence-free tagged exchange
    nblk, iters = 256, 200
    pbuf = torch.zeros(df.sync_probe_bytes(nblk), dtype=torch.uint8, device=dev)
    for mode, nm in ((0, "kernel_boundary_per_phase_graph_replay"), (1, "in_kernel_barrier_with_fences"),
                     (2, "in_kernel_tagged_exchange_no_fences")):
        with torch.cuda.stream(stream):
            df.sync_probe(pbuf, nblk, iters, mode)
            stream.synchronize()
            graph = None
            if mode == 0:                 # the step replays its launches from a HIP graph: time the boundaries that way
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    df.sync_probe(pbuf, nblk, iters, mode)
                graph.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            stream.synchronize()
            e0.record(stream)
            if graph is not None:
                graph.replay()
            else:
                df.sync_probe(pbuf, nblk, iters, mode)
            e1.record(stream)
            e1.synchronize()
        flag = int(pbuf[:4].view(torch.int32).item())
        print(json.dumps({"op": "sync_probe_" + nm, "workgroups": nblk, "phases": iters,
                          "us_per_phase": round(e0.elapsed_time(e1) * 1e3 / iters, 2), "fail_flag": flag}), flush=True)
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    big2 = torch.empty_like(big)
    timed("copy_1GiB", lambda: df.copy_bytes(big2, big), nbytes=2.0 * big.numel())
    del big, big2

    # configuration 2: displaced self-attention layer, N=4, 1024 fresh of 4096 tokens, 10 heads x 64
    Lq, L, C, heads = 1024, 4096, 640, 10
    hid = bf(rn(1, Lq, C))
    wq, wk, wv, wo = (bf(rn(C, C, std=1 / math.sqrt(C))) for _ in range(4))
    ks, vs = bf(rn(1, L, C)), bf(rn(1, L, C))
    q, kf, vf = bf(rn(1, Lq, C)), bf(rn(1, Lq, C)), bf(rn(1, Lq, C))
    timed("cfg2_attention_core", lambda: df.attn_displaced(q, kf, vf, ks, vs, heads, 1, 4),
          flops=4.0 * Lq * L * C, nbytes=2.0 * (2 * Lq * C + 2 * L * C))
    def layer():
        h2 = hid.view(Lq, C)
        qq = df.linear(h2, wq).view(1, Lq, C)
        kk = df.linear(h2, wk).view(1, Lq, C)
        vv = df.linear(h2, wv).view(1, Lq, C)
        o = df.attn_displaced(qq, kk, vv, ks, vs, heads, 1, 4)
        return df.linear(o.view(Lq, C), wo)
    timed("cfg2_self_attention_layer", layer, flops=4.0 * Lq * L * C + 2.0 * Lq * C * C * 4,
          note="Q, K, V, out projections + attention core: 5 launches through the per-op entry points")

    # configuration 3: GroupNorm -> conv3x3 -> SiLU on a 32-row patch of 128x128x320, N=4
    R, H, W, Cc, G = 32, 128, 128, 320, 32
    xg = bf(rn(1, R, W, Cc))
    stats = rn(4, 1, G, 2).abs() * 1000
    gam, bet = 1 + 0.1 * rn(Cc), 0.1 * rn(Cc)
    wc = bf(rn(Cc, 3, 3, Cc, std=math.sqrt(2.0 / (9 * Cc))))
    bc = 0.02 * rn(Cc)
    stale_full = bf(rn(1, H, W, Cc))
    timed("cfg3_groupnorm", lambda: df.groupnorm_stale(xg, stats, gam, bet, G, 1, 4), nbytes=2.0 * xg.numel() * 2)
    timed("cfg3_conv3x3", lambda: df.conv3x3_halo(xg, stale_full, wc, bc, 1, 4, act=1),
          flops=2.0 * 9 * Cc * Cc * R * W, nbytes=2.0 * ((R + 2) * W * Cc + 9 * Cc * Cc + R * W * Cc))
    timed("cfg3_gn_conv_silu_chain",
          lambda: df.conv3x3_halo(df.groupnorm_stale(xg, stats, gam, bet, G, 1, 4)[0], stale_full, wc, bc, 1, 4, act=1),
          flops=2.0 * 9 * Cc * Cc * R * W)

    # configuration 5: the largest GroupNorm (64 x 256 x 960 bf16 = 31.5 MB) and one step's K/V refresh volume
    x5 = bf(rn(1, 64, 256, 960))
    st5 = rn(4, 1, G, 2).abs() * 1000
    g5, b5 = 1 + 0.1 * rn(960), 0.1 * rn(960)
    timed("cfg5_groupnorm_31MB", lambda: df.groupnorm_stale(x5, st5, g5, b5, G, 1, 4), nbytes=2.0 * x5.numel() * 2)
    full = torch.empty(1, 4 * 52_428_800, dtype=torch.bfloat16, device=dev)     # 0.42 GB: K/V of one step, one patch of 4
    part = torch.empty(1, 52_428_800, dtype=torch.bfloat16, device=dev)
    timed("cfg5_refresh_105MB_slice", lambda: df.buffer_refresh(full, part, 1, 4), nbytes=2.0 * part.numel() * 2)
    # level-2 patch GEMMs of configuration 4 on packed operands
    for (M, N, K, gg) in [(300, 1280, 1280, False), (300, 3840, 1280, False), (300, 1280, 5120, False), (300, 10240, 1280, True)]:
        wp = df.pack_linear_weight(bf(rn(N, K, std=1 / math.sqrt(K))))
        xp = df.pack_rows(bf(rn(M, K)))
        timed("cfg4_linear_packed_%dx%dx%d%s" % (M, N, K, "_geglu" if gg else ""),
              lambda: df.linear_packed(xp, wp, M, N, K, geglu=gg, want=("packed",)), flops=2.0 * M * N * K,
              nbytes=2.0 * (M * K + N * K + M * (N // 2 if gg else N)), note="weights stay hot in L2 / Infinity Cache")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--profile-steps", type=int, default=3, help="extra steps with per-launch event timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch every step eagerly (no HIP graph replay)")
    ap.add_argument("--small", action="store_true", help="reduced-width UNet (plumbing check, not the benchmark)")
    ap.add_argument("--workload", choices=["cfg4", "3840", "2048"], default="cfg4",
                    help="cfg4: the headline workload (1280x1920, N=8); 3840: one of 8 row patches of a 3840x3840 image "
                         "(480x480 latent), the paper's best-scaling resolution; 2048: one of 4 row patches of a 2048x2048 "
                         "image (256x256 latent), the shape of the multi-step configuration - further workloads, not the "
                         "headline")
    ap.add_argument("--batch", type=int, default=1,
                    help="batch items through the same step (2 = both classifier-free-guidance branches); the headline is 1")
    ap.add_argument("--split-axis", choices=["rows", "cols"], default="rows",
                    help="direction of the patch split (cols: vertical strips; the latent width must divide by 4N, so "
                         "not for the headline workload)")
    ap.add_argument("--full-step", action="store_true",
                    help="time and profile the synchronous full-image step (the first step of a sampling run) instead of "
                         "the displaced patch step; a secondary measurement, not the headline")
    ap.add_argument("--loop", type=int, default=0,
                    help="run the multi-step configuration's loop with this many Euler steps (step 0 FULL, the rest "
                         "DISPLACED + refresh) on the chosen workload and print per-step times; --workload 2048 --loop 10 "
                         "is that configuration as stated")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="only run plain copies of this many MiB through the library's copy kernel (counter calibration)")
    ap.add_argument("--all-kernels", action="store_true", help="list every kernel of the step in `top_kernels`, not the top 8")
    ap.add_argument("--tile-sweep", action="store_true",
                    help="tile-shape sweep of the LDS-tiled MFMA kernel on large shapes (needs the tuning build)")
    ap.add_argument("--timeline", action="store_true",
                    help="in-kernel cycle stamps of the tiled MFMA kernel and the wave-level linear layers (needs the tuning build)")
    ap.add_argument("--ops", action="store_true",
                    help="single-operation measurements at the shapes of the other configurations instead of the step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2402_19481_amd as df
    from df_inputs import unet_table as ut

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.tile_sweep or args.timeline:
        tune = os.path.join(os.path.dirname(df.LIB_PATH), "libdistrifusion_tune.so")
        if not os.path.exists(tune):
            print("bench.py --tile-sweep / --timeline: build the tuning library first: python -m paper_2402_19481_amd.build --tuning",
                  file=sys.stderr)
            sys.exit(1)
        df.LIB_PATH = tune
        if args.timeline:
            run_timeline(df, torch, tune)
        else:
            run_tile_sweep(df, torch)
        return
    if args.ops:
        run_ops(df, torch)
        return
    if args.calibrate_copy:
        calibrate_copy(df, torch, args.calibrate_copy, max(args.steps, 1))
        return
    if args.small:
        cfg = ut.UNetCfg(H=32, W=16, N=4, **ut.SMALL)
        patch = 1
        workload = "reduced-width UNet 32x16 latent, N=4 (plumbing check)"
    elif args.workload == "3840":
        cfg = ut.UNetCfg(H=480, W=480, N=8, **ut.SDXL)
        patch = 3
        workload = ("SDXL-shaped UNet step for one patch: 3840x3840 image (480x480x4 latent), N=8 row patches "
                    "(60 latent rows), patch 3, DISPLACED + refresh")
    elif args.workload == "2048":
        cfg = ut.UNetCfg(H=256, W=256, N=4, **ut.SDXL)
        patch = 1
        workload = ("SDXL-shaped UNet step for one patch: 2048x2048 image (256x256x4 latent), N=4 row patches "
                    "(64 latent rows), patch 1, DISPLACED + refresh")
    else:
        cfg = ut.UNetCfg(H=160, W=240, N=8, **ut.SDXL)
        patch = 3
        workload = ("SDXL-shaped UNet step for one patch: 1280x1920 image (160x240x4 latent), N=8 row patches "
                    "(20 latent rows), patch 3, DISPLACED + refresh")
    ccfg = df.make_cfg(cfg)
    specs = df.unet_weight_specs(ccfg)
    weights = make_weights(df, torch, ccfg, seed=4)
    Bn = args.batch
    cols = args.split_axis == "cols"
    if cols:
        workload = workload.replace("row patches", "column patches (vertical strips)").replace("latent rows)", "latent columns)")
    net = df.PatchUNet(cfg, weights, B=Bn, split_axis=df.SPLIT_COLS if cols else df.SPLIT_ROWS)
    if args.no_graph:
        net.set_graph(False)
    if args.loop:
        gl = torch.Generator(device="cuda:0").manual_seed(40)
        emb_l = torch.randn(1, cfg.emb_dim, generator=gl, device="cuda:0")
        text_l = torch.randn(1, cfg.text_len, cfg.text_dim, generator=gl, device="cuda:0").to(torch.bfloat16)
        run_loop(df, torch, net, cfg, patch, args.loop, emb_l, text_l, workload.replace(", DISPLACED + refresh", ""))
        net.close()
        return
    g = torch.Generator(device="cuda:0").manual_seed(40)
    x_prev = torch.randn(Bn, cfg.H, cfg.W, cfg.in_ch, generator=g, device="cuda:0")
    R = cfg.H // cfg.N
    x = x_prev + 0.02 * torch.randn(x_prev.shape, generator=g, device="cuda:0")
    if cols:
        Wp = cfg.W // cfg.N
        x = x[:, :, patch * Wp:(patch + 1) * Wp].contiguous()
    else:
        x = x[:, patch * R:(patch + 1) * R].contiguous()
    emb = torch.randn(Bn, cfg.emb_dim, generator=g, device="cuda:0")
    text = torch.randn(Bn, cfg.text_len, cfg.text_dim, generator=g, device="cuda:0").to(torch.bfloat16)
    eps = torch.empty_like(x)

    # everything runs on one side stream (the library replays repeated steps as a HIP graph, which the legacy default
    # stream does not allow)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        # the synchronous first step fills every stale buffer (outside the timed region); its second run is timed for
        # context: what the first step of a sampling run costs
        net.step(x_prev, emb, text, mode=df.MODE_FULL)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        net.step(x_prev, emb, text, mode=df.MODE_FULL)
        torch.cuda.synchronize()
        full_ms = (time.perf_counter() - t1) * 1e3

        if args.full_step:
            eps = torch.empty_like(x_prev)
            workload = workload.split(" for one patch")[0] + ", synchronous step on the full image" + \
                workload.split(" for one patch")[1].split(", N=")[0]

            def one():
                net.step(x_prev, emb, text, mode=df.MODE_FULL, out=eps)
        else:
            def one():
                net.step(x, emb, text, patch_idx=patch, mode=df.MODE_DISPLACED, refresh=True, out=eps)

        for _ in range(max(args.warmup, 2)):      # the first call is eager, the second records the graph
            one()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        assert bool(torch.isfinite(eps).all())

        # per-launch event timing over further steps of the same work, on the stream the kernels run on
        net.profile(True)
        for _ in range(args.profile_steps):
            one()
        prof = net.profile_read()
        kernels = net.profile_kernels()
        net.profile(False)
    # Every launch of a profiled step sits between two events, and an event costs the stream a few microseconds that
    # a graph-replayed step does not pay.  That per-launch cost is measured, not assumed: the event intervals of a
    # step must add up to the graph-replayed step time, so overhead = (sum of intervals - step time) / launches, and
    # it is taken off every launch.  The resulting per-kernel averages agree with the rocprofv3 kernel trace of the
    # same command.
    n_launch = sum(v["launches"] for v in prof.values()) / max(args.profile_steps, 1)
    raw_ms = sum(v["ms"] for v in prof.values()) / max(args.profile_steps, 1)
    ev_over_ms = max(0.0, (raw_ms - ms) / n_launch) if (n_launch and not args.no_graph) else 0.0
    breakdown = {}
    for k, v in prof.items():
        if v["launches"] == 0:
            continue
        v["event_ms"] = v["ms"]
        v["ms"] = max(v["ms"] - ev_over_ms * v["launches"], 1e-6)
        per_step_ms = v["ms"] / args.profile_steps
        breakdown[k] = dict(ms_per_step=round(per_step_ms, 4), launches_per_step=v["launches"] // args.profile_steps,
                            tflops=round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["flops"] else None,
                            gbs=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1),
                            event_ms_per_step=round(v["event_ms"] / args.profile_steps, 4))
    # The roofline object is that of the single dominant KERNEL: one operation at one shape, i.e. the launches of one
    # kernel instantiation with one grid (the library's profile keeps totals per such kernel).  The class it belongs
    # to (all linear layers, all convolutions, ...) is reported beside it.
    for kr in kernels:
        kr["ms"] = max(kr["ms"] - ev_over_ms * kr["launches"], 1e-6)
    kd = max(kernels, key=lambda kr: kr["ms"])
    dom = kd["cls"]
    d = prof[dom]

    def roof(rec, name, extra):
        if rec["flops"] > 0:
            ach = rec["flops"] / (rec["ms"] * 1e-3) / 1e12
            out = dict(bound="mfma", kernel=name, achieved=round(ach, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                       frac=round(ach / PEAK_BF16_TFLOPS, 4), traffic=None,
                       flops_per_launch=rec["flops"] / rec["launches"])
        else:
            ach = rec["bytes"] / (rec["ms"] * 1e-3) / 1e9
            out = dict(bound="hbm", kernel=name, achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                       frac=round(ach / PEAK_HBM_GBS, 4), traffic=None)
        out["algorithmic_bytes_per_launch"] = round(rec["bytes"] / rec["launches"])
        out["avg_launch_us"] = round(rec["ms"] * 1e3 / rec["launches"], 3)
        out["launches_per_step"] = rec["launches"] // args.profile_steps
        out["ms_per_step"] = round(rec["ms"] / args.profile_steps, 4)
        out.update(extra)
        return out

    roofline = roof(kd, kd["label"], {})
    roofline["share_of_step"] = round(kd["ms"] / args.profile_steps / ms, 4)
    cls_roof = roof(d, dom, {})
    headline = not (args.small or args.workload != "cfg4" or args.batch != 1 or args.full_step)
    tr = traffic_from_profile(cls=dom) if headline else None
    trk = traffic_from_profile(kernel=kd["label"]) if headline else None
    # Counters cannot be read in a timed run: `traffic` is the bytes per launch that the committed counter profile of
    # this same command states (two separate rocprofv3 --pmc runs), not a measurement of the present run.
    if trk is not None:
        roofline["traffic"] = round(trk)
        roofline["traffic_source"] = TRAFFIC_PROFILE + " (separate rocprofv3 --pmc runs of this command)"
    if tr is not None:
        cls_roof["traffic"] = round(tr / (d["launches"] / args.profile_steps))
        cls_roof["traffic_source"] = TRAFFIC_PROFILE + " (separate rocprofv3 --pmc runs of this command)"
    roofline["kernel_class"] = cls_roof
    top = sorted(kernels, key=lambda kr: -kr["ms"])[:(None if args.all_kernels else 8)]
    top_kernels = [dict(kernel=kr["label"], ms_per_step=round(kr["ms"] / args.profile_steps, 4),
                        launches_per_step=kr["launches"] // args.profile_steps,
                        tflops=round(kr["flops"] / (kr["ms"] * 1e-3) / 1e12, 1) if kr["flops"] else None,
                        gbs=round(kr["bytes"] / (kr["ms"] * 1e-3) / 1e9, 1)) for kr in top]

    macs = ut.count_macs(cfg)
    tflop = 2.0 * macs["total"] / 1e12 * Bn * (cfg.N if args.full_step else 1)
    out = {
        "metric": "ms per patch UNet step (1 MI355X)", "value": round(ms, 4), "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload, "batch": Bn, "patch_idx": patch, "n_patches": cfg.N,
                   "tflop_per_step": round(tflop, 4)},
        "tflops": round(tflop / (ms * 1e-3), 2),
        "mfma_util_frac_of_bf16_peak": round(tflop / (ms * 1e-3) / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
        # ceiling measured in this run: register-resident MFMA loop (nominal dense bf16 peak is 2500 TFLOP/s)
        "mfma_peak_measured_tflops": measured_mfma_peak(df, torch),
        # the other parts of the headline metric: MFMA utilisation of attention and convolution, GroupNorm / refresh GB/s
        "attn_mfma_util_frac": round((breakdown.get("self_attn", {}).get("tflops") or 0.0) / PEAK_BF16_TFLOPS, 4),
        "conv_mfma_util_frac": round((breakdown.get("conv3x3", {}).get("tflops") or 0.0) / PEAK_BF16_TFLOPS, 4),
        "groupnorm_hbm_gbs": breakdown.get("groupnorm", {}).get("gbs"),
        "refresh_hbm_gbs": breakdown.get("refresh", {}).get("gbs"),
        "breakdown": breakdown,
        "top_kernels": top_kernels,
        "event_overhead_us_per_launch": round(ev_over_ms * 1e3, 2),
        # the synchronous full-image step of the same latent (first step of a run; eager launches), for context
        "full_image_step_ms": round(full_ms, 3),
    }
    if not args.no_cpu_baseline and args.workload == "cfg4" and Bn == 1 and not args.full_step:
        xin = x.cpu().numpy()
        out["cpu_baseline"] = cpu_baseline(cfg, weights, specs, (xin, emb.cpu().numpy(), text.float().cpu().numpy()), patch)
    else:
        out["cpu_baseline"] = None
    net.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
