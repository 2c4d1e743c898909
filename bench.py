#!/usr/bin/env python3
"""Benchmark of the block-sparse layer hot path on one MI355X.

A step is one pass of the whole path over benchmark configuration 2 (256x256x128 fp16, ~1 % blob edit,
16x16 blocks): difference mask + block lists (3x3 and 1x1 geometry), then gather(GN+SiLU) ->
conv3x3 -> scatter and gather -> conv1x1 -> scatter, inputs resident in HBM, replayed as one HIP
graph (block counts stay on the device).  `value` is the algorithmic bytes of one step divided by
its wall time.  The line also carries
  roofline      - the kernel that moves 91 % of the step's bytes and takes as long as any other in it
                  (the difference-mask stream: HBM bound),
  roofline_mfma - the step's MFMA-bound kernel (the 3x3 convolution on the active blocks),
both timed live with events on the launch stream, the CPU oracle timed on the host cores, and
`supplement`: per-call times, gather / scatter / difference-mask bandwidth on a 1024x1024x128
tensor with every block active (footprint far beyond the 256 MB Infinity Cache), convolution
throughput with every block active, sparse-query attention, the synthetic DDPM-style UNet step
(benchmark configuration 3) sparse at ~1.2 % and 15.5 % edit versus dense, and the synthetic latent-diffusion
style UNet step (benchmark configuration 4) at 1 / 5 / 20 % edit versus dense, and the synthetic SPADE-style
generator (benchmark configuration 5) over ten successive ~1 % label edits versus dense.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per launch from hardware counters (two rocprofv3 --pmc runs of `bench.py --probe`: FETCH_SIZE
# scaled by 2.0, WRITE_SIZE by 1.0, the factors a plain 128 MiB copy gives; see profiles/hbm_traffic_pmc.md)
PMC_TRAFFIC_DIFF_MASK_CONFIG2 = 16425 * 2 * 1024 + 64 * 1024
PMC_TRAFFIC_FUSED_CONV_CONFIG2 = 2586 * 2 * 1024 + 576 * 1024
HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"f16": 2500.0, "bf16": 2500.0, "f32": 157.3}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-supplement", action="store_true", help="only the headline step and rooflines")
    ap.add_argument("--no-unet", action="store_true", help="skip the UNet step in the supplement")
    ap.add_argument("--probe", action="store_true",
                    help="launch each kernel of interest a few times and exit (for rocprofv3 --pmc runs)")
    ap.add_argument("--three-calls", action="store_true",
                    help="gather, conv, scatter as three kernels per convolution instead of the fused one")
    return ap.parse_args()


def next_pow2(n):
    p = 1
    while p < n:
        p *= 2
    return p


def time_calls(fn, iters, warm=20):
    """Average duration of fn() in microseconds, HIP events on the current stream."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters


def time_graphed(fn, per_graph=20, replays=15):
    """Average duration of one fn() in microseconds with the host launch path taken out: per_graph
    calls are captured in a HIP graph (launched back to back by the GPU's command processor) and the
    replays are timed with events on the stream."""
    import torch
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        for _ in range(3):
            fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(per_graph):
            fn()
    torch.cuda.synchronize()
    return time_calls(g.replay, replays, 3) / per_graph


class Layer2:
    """Config 2 on the device: caches from a first all-active pass, then the sparse step.  The step
    is captured once in a HIP graph: every kernel takes the block count from device memory and the
    launches are sized by a capacity chosen after the first reduction of an edit, so a replay needs
    no host round trip."""

    def __init__(self, cfg, fused, device="cuda"):
        import torch
        from paper_2211_02048_amd import api
        from paper_2211_02048_amd.layers import BlockList, SigeConv, Workspace
        self.api, self.cfg, self.fused = api, cfg, fused
        H, W, C, Cs = cfg["H"], cfg["W"], cfg["Cin"], cfg["Cs"]
        self.a_o, self.a_e = cfg["a_orig"].to(device), cfg["a_edit"].to(device)
        self.main = SigeConv(cfg["w"].to(device), cfg["bias"], H, W, cfg["block"], 1, 1)
        self.short = SigeConv(cfg["w_s"].to(device), cfg["bias_s"], H, W, cfg["block"], 1, 0)
        self.ws = Workspace(device)
        self.bl3 = BlockList(self.main.g, device)
        self.bl1 = BlockList(self.short.g, device)
        self.mask = torch.zeros((H, W), dtype=torch.uint8, device=device)
        G = cfg["groups"]
        self.mean, self.var = torch.zeros(G, device=device), torch.zeros(G, device=device)
        self.scale, self.shift = torch.zeros(C, device=device), torch.zeros(C, device=device)
        # pre-computation pass on the original input: statistics and F(A_orig) for both convs
        api.sige_gn_stats(self.a_o, G, self.mean, self.var, gamma=cfg["gamma"].to(device),
                          beta=cfg["beta"].to(device), eps=cfg["eps"], scale=self.scale, shift=self.shift)
        self.y_main = torch.empty((H, W, C), dtype=self.a_o.dtype, device=device)
        self.y_short = torch.empty((H, W, Cs), dtype=self.a_o.dtype, device=device)
        full3, full1 = BlockList(self.main.g, device).all_active(), BlockList(self.short.g, device).all_active()
        self.main.forward(self.a_o, self.y_main, full3, self.ws, scale=self.scale, shift=self.shift,
                          act=api.ACT_SILU)
        self.short.forward(self.a_o, self.y_short, full1, self.ws)
        torch.cuda.synchronize()

    def reduce(self):
        # one pass over both activations marks the blocks of both geometries (3x3 and 1x1 tiles)
        from paper_2211_02048_amd.layers import BlockList
        c = self.cfg
        BlockList.reduce_together([self.bl3, self.bl1], a_orig=self.a_o, a_edit=self.a_e, tau=c["tau"],
                                  mask_out=self.mask, dilate=c["dilate"])

    def mark(self):
        # the marking half of the reduction: the layer's launch builds the lists from the flags
        from paper_2211_02048_amd.layers import BlockList
        c = self.cfg
        BlockList.mark_together([self.bl3, self.bl1], a_orig=self.a_o, a_edit=self.a_e, tau=c["tau"],
                                mask_out=self.mask, dilate=c["dilate"])

    def layer(self, marked=False):
        api = self.api
        if self.fused:   # both convolutions read a_e and are independent: handed over together (one launch)
            c3, _ = self.main.fused_call(self.a_e, self.y_main, self.bl3, self.ws, scale=self.scale, shift=self.shift,
                                         act=api.ACT_SILU, tag="main")
            c1, _ = self.short.fused_call(self.a_e, self.y_short, self.bl1, self.ws, tag="short")
            if marked:
                api.sige_fused_conv_pair_marked(c3, c1, [self.bl3.desc(), self.bl1.desc()])
            else:
                api.sige_fused_conv_pair(c3, c1)
            return
        self.main.forward(self.a_e, self.y_main, self.bl3, self.ws, scale=self.scale, shift=self.shift,
                          act=api.ACT_SILU, fused=self.fused)
        self.short.forward(self.a_e, self.y_short, self.bl1, self.ws, fused=self.fused)

    def step_eager(self):
        self.reduce()
        self.bl3.sync_count()   # one readback per edit and list sizes the launches exactly
        self.bl1.sync_count()
        self.layer()

    def capture(self):
        """Size the lists for this edit (one readback), then capture reduce + layer in a graph."""
        import torch
        from paper_2211_02048_amd.layers import BlockList
        self.reduce()
        n3, n1 = self.bl3.sync_count(), self.bl1.sync_count()
        cap = max(8, next_pow2(n3))
        self.capacity = cap
        self.bl3 = BlockList(self.main.g, self.a_o.device, max_blocks=cap)
        self.bl1 = BlockList(self.short.g, self.a_o.device, max_blocks=cap)

        def body():
            if self.fused:     # two launches: difference + block flags, then lists + both convolutions
                self.mark()
                self.layer(marked=True)
            else:
                self.reduce()
                self.layer()   # n_host = -1: counts are read on the device
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            for _ in range(3):
                body()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            body()
        torch.cuda.synchronize()
        return n3, n1

    def step(self):
        self.graph.replay()

    def bytes_per_step(self, n3, n1):
        c = self.cfg
        s, C, Cs, b = 2, c["Cin"], c["Cs"], c["block"]
        t = b + 2
        diff = 2 * c["H"] * c["W"] * C * s + c["H"] * c["W"]
        lists = 8 * (n3 + n1) + 8      # the mask is written by the difference pass and not read again
        if self.fused:   # tile read once, output block written once
            main = n3 * (t * t * C * s + b * b * C * s) + 9 * C * C * s
            short = n1 * (b * b * C * s + b * b * Cs * s) + C * Cs * s
        else:            # gather r+w, conv r+w, scatter r+w
            main = n3 * (2 * t * t * C * s + 2 * b * b * C * s + t * t * C * s + b * b * C * s) + 9 * C * C * s
            short = n1 * (2 * b * b * C * s + 2 * b * b * Cs * s + b * b * C * s + b * b * Cs * s) + C * Cs * s
        return diff + lists + main + short, diff

    def flops_per_step(self, n3, n1):
        c = self.cfg
        b = c["block"]
        return 2 * b * b * (n3 * 9 * c["Cin"] * c["Cout"] + n1 * c["Cin"] * c["Cs"])


def cpu_baseline(cfg, n_bytes):
    """The oracle as it stands, timed on the host cores: the whole config-2 step (difference
    mask, block lists, dense GN+SiLU+3x3 layer, dense 1x1 layer, block selection), repeated
    until about 10 s have passed."""
    import numpy as np
    import torch

    import oracle
    f64 = lambda t: t.to(torch.float64).numpy()
    a_o32, a_e32 = cfg["a_orig"].float().numpy(), cfg["a_edit"].float().numpy()
    a_o, a_e = f64(cfg["a_orig"]), f64(cfg["a_edit"])
    w, b, ws, bs = f64(cfg["w"]), f64(cfg["bias"]), f64(cfg["w_s"]), f64(cfg["bias_s"])
    mean, var = oracle.gn_stats(a_o, cfg["groups"])
    scale, shift = oracle.fold_gn(f64(cfg["gamma"]), f64(cfg["beta"]), mean, var, cfg["eps"])
    H, W, blk = cfg["H"], cfg["W"], cfg["block"]
    cache3 = np.zeros((H, W, cfg["Cout"]))
    cache1 = np.zeros((H, W, cfg["Cs"]))
    cores = oracle.get_max_threads()
    times = []
    t_all = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        m = oracle.diff_mask(a_o32, a_e32, cfg["tau"])
        b3 = oracle.active_blocks(m, H, W, blk, blk, 3, 1, 1)
        b1 = oracle.active_blocks(m, H, W, blk, blk, 1, 1, 0)
        oracle.sige_layer(a_e, cache3, b3, blk, blk, w, b, 1, 1, scale, shift, oracle.ACT_SILU)
        oracle.sige_layer(a_e, cache1, b1, blk, blk, ws, bs, 1, 0)
        times.append(time.perf_counter() - t0)
        if time.perf_counter() - t_all > 10.0 or len(times) >= 10:
            break
    t = float(np.median(times))
    return {"value": round(n_bytes / t / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"whole config-2 step (dense GN+SiLU+3x3 and 1x1 layers on the edited input, then "
                      f"block selection), median of {len(times)} runs", "s_per_step": round(t, 4)}


def supplement(L, with_unet):
    """Per-call times at config 2 and bandwidth / throughput points in regimes where they show."""
    import torch
    from paper_2211_02048_amd import api, inputs
    from paper_2211_02048_amd.layers import BlockList, SigeConv
    out = {}
    c = L.cfg
    n3, n1 = L.bl3.n_host, L.bl1.n_host
    # ---- per-call times at config 2 (exact host block count, eager launches)
    g3, ws = L.main.g, L.ws
    tiles = ws.get("tiles", L.main.tiles_numel(max(n3, 1)), L.a_e.dtype)
    ot = ws.get("out_t", L.main.out_numel(max(n3, 1)), L.a_e.dtype)
    per = {}
    per["reduce_mask_from_activations_us"] = time_calls(
        lambda: L.bl3.reduce(a_orig=L.a_o, a_edit=L.a_e, tau=c["tau"], mask_out=L.mask), 200)
    per["reduce_mask_from_mask_us"] = time_calls(lambda: L.bl1.reduce(mask_in=L.mask), 200)
    L.bl3.n_host, L.bl1.n_host = n3, n1
    per["gather_fused_gn_silu_us"] = time_calls(
        lambda: api.sige_gather(L.a_e, g3, L.bl3.indices, L.bl3.count, tiles, n_blocks=n3, scale=L.scale,
                                shift=L.shift, act=api.ACT_SILU, max_blocks=max(n3, 1)), 200)
    per["conv3x3_us"] = time_calls(
        lambda: api.sige_conv(tiles, g3, c["Cin"], c["Cout"], L.main.packed, L.main.bias, L.bl3.count, ot,
                              n_blocks=n3, max_blocks=max(n3, 1)), 200)
    per["scatter_us"] = time_calls(
        lambda: api.sige_scatter(ot, g3, L.bl3.indices, L.bl3.count, L.y_main, n_blocks=n3, Cout=c["Cout"],
                                 max_blocks=max(n3, 1)), 200)
    per["fused_conv3x3_us"] = time_calls(
        lambda: L.main.forward(L.a_e, L.y_main, L.bl3, ws, scale=L.scale, shift=L.shift, act=api.ACT_SILU,
                               fused=True), 200)
    out["config2_calls_eager"] = {k: round(v, 2) for k, v in per.items()}
    out["config2_calls_eager"]["note"] = "eager single calls include the host launch path (a few us each)"

    # ---- dense comparator: the same kernels with every block active
    full3 = BlockList(g3, "cuda").all_active()
    full1 = BlockList(L.short.g, "cuda").all_active()
    y3, y1 = torch.empty_like(L.y_main), torch.empty_like(L.y_short)

    def both(ya, yb, la, lb):
        # the two convolutions as the step runs them: handed over together (one launch where the
        # library can, i.e. with few active blocks)
        if L.fused:
            ca, _ = L.main.fused_call(L.a_e, ya, la, ws, scale=L.scale, shift=L.shift, act=api.ACT_SILU, tag="main")
            cb, _ = L.short.fused_call(L.a_e, yb, lb, ws, tag="short")
            api.sige_fused_conv_pair(ca, cb)
        else:
            L.main.forward(L.a_e, ya, la, ws, scale=L.scale, shift=L.shift, act=api.ACT_SILU)
            L.short.forward(L.a_e, yb, lb, ws)

    def dense():
        both(y3, y1, full3, full1)

    def sparse():
        both(L.y_main, L.y_short, L.bl3, L.bl1)
    dense_us = time_calls(dense, 50, 5)
    sparse_us = time_calls(sparse, 200, 5)
    nfull = g3.grid_blocks
    tl = ws.get("tiles", L.main.tiles_numel(nfull), L.a_e.dtype)
    of = ws.get("out_t", L.main.out_numel(nfull), L.a_e.dtype)
    api.sige_gather(L.a_e, g3, full3.indices, full3.count, tl, n_blocks=nfull, scale=L.scale, shift=L.shift,
                    act=api.ACT_SILU, max_blocks=nfull)
    conv_us = time_calls(lambda: api.sige_conv(tl, g3, c["Cin"], c["Cout"], L.main.packed, L.main.bias, full3.count,
                                               of, n_blocks=nfull, max_blocks=nfull), 50, 5)
    fl = 2.0 * c["H"] * c["W"] * 9 * c["Cin"] * c["Cout"]
    out["config2_all_blocks_active"] = {
        "both_convs_us": round(dense_us, 1), "both_convs_sparse_us": round(sparse_us, 1),
        "sparse_over_dense_speedup": round(dense_us / sparse_us, 2),
        "conv3x3_us": round(conv_us, 1), "conv3x3_tflops": round(fl / conv_us / 1e6, 1),
        "conv3x3_frac_mfma_peak": round(fl / conv_us / 1e6 / MFMA_PEAK_TFLOPS["f16"], 4)}

    # ---- latency against edited area (Sec. 4.2 "Large edits"): both convs of config 2 on blob masks
    import numpy as np
    rng = np.random.Generator(np.random.PCG64(2002))
    sweep = []
    for frac in (0.01, 0.05, 0.15, 0.30, 0.50, 0.75):
        m = inputs.blob_mask(rng, c["H"], c["W"], int(frac * c["H"] * c["W"]), 3 + int(20 * frac),
                             (5.0, 12.0), tol=0.1)
        md = torch.from_numpy(m).cuda()
        b3, b1 = BlockList(g3, "cuda"), BlockList(L.short.g, "cuda")
        b3.reduce(mask_in=md)
        b1.reduce(mask_in=md)
        k3, k1 = b3.sync_count(), b1.sync_count()

        def run():
            both(y3, y1, b3, b1)
        us = time_graphed(run, per_graph=10, replays=10)
        sweep.append({"edited_area": frac, "active_blocks_3x3": k3, "active_blocks_1x1": k1,
                      "both_convs_us": round(us, 1)})
    dense_g = time_graphed(dense, per_graph=10, replays=10)
    out["config2_latency_vs_edited_area"] = {"points": sweep, "all_blocks_active_us": round(dense_g, 1),
                                             "note": "graph-batched launches; break-even against the all-active "
                                                     "launch is where both_convs_us crosses all_blocks_active_us "
                                                     "(the paper reports 65-75 % on RTX 3090, Sec. 4.2)"}

    # ---- config 1 (3x3, 64->64, 64x64, fp32, 6x6 blocks, ~5 % rectangle): whole step
    c1 = inputs.config1()
    conv1 = SigeConv(c1["w"].cuda(), c1["bias"], 64, 64, 6, 1, 1)
    bl1c = BlockList(conv1.g, "cuda")
    ao1, ae1 = c1["a_orig"].cuda(), c1["a_edit"].cuda()
    m1 = torch.zeros((64, 64), dtype=torch.uint8, device="cuda")
    y1c = torch.zeros((64, 64, 64), dtype=torch.float32, device="cuda")
    bl1c.reduce(a_orig=ao1, a_edit=ae1, tau=c1["tau"], mask_out=m1)
    n1c = bl1c.sync_count()
    bl1c.n_host = -1
    bl1c.max_blocks = max(8, next_pow2(n1c))

    def step1():
        bl1c.reduce(a_orig=ao1, a_edit=ae1, tau=c1["tau"], mask_out=m1)
        bl1c.n_host = -1
        conv1.forward(ae1, y1c, bl1c, ws, fused=L.fused)
    out["config1_fp32_step"] = {"active_blocks": n1c, "of_blocks": conv1.g.grid_blocks,
                                "step_us": round(time_graphed(step1, per_graph=10, replays=10), 1)}

    # ---- bandwidth regime: 1024x1024x128 fp16 (256 MiB per tensor), all 4096 blocks active
    H2 = 1024
    C = c["Cin"]
    x = torch.randn((H2, H2, C), dtype=torch.float16, device="cuda")
    x2 = x.clone()
    big = SigeConv(c["w"].cuda(), c["bias"], H2, H2, 16, 1, 1)
    bl = BlockList(big.g, "cuda").all_active()
    nb = bl.n_host
    t2 = torch.empty(big.tiles_numel(nb), dtype=torch.float16, device="cuda")
    o2 = torch.empty(big.out_numel(nb), dtype=torch.float16, device="cuda")
    y2 = torch.empty((H2, H2, C), dtype=torch.float16, device="cuda")
    sc, sh = L.scale, L.shift
    g_us = time_calls(lambda: api.sige_gather(x, big.g, bl.indices, bl.count, t2, n_blocks=nb, scale=sc, shift=sh,
                                              act=api.ACT_SILU, max_blocks=nb), 20, 3)
    gp_us = time_calls(lambda: api.sige_gather(x, big.g, bl.indices, bl.count, t2, n_blocks=nb, max_blocks=nb),
                       20, 3)
    s_us = time_calls(lambda: api.sige_scatter(o2, big.g, bl.indices, bl.count, y2, n_blocks=nb, Cout=C,
                                               max_blocks=nb), 20, 3)
    c_us = time_calls(lambda: api.sige_conv(t2, big.g, C, C, big.packed, big.bias, bl.count, o2, n_blocks=nb,
                                            max_blocks=nb), 10, 2)
    mask_o = torch.zeros((H2, H2), dtype=torch.uint8, device="cuda")
    d_us = time_calls(lambda: api.sige_reduce_mask(big.g, None, None, a_orig=x, a_edit=x2, tau=0.0,
                                                   mask_out=mask_o), 20, 2)
    gb = nb * 2 * 18 * 18 * C * 2
    sb = nb * 2 * 16 * 16 * C * 2
    db = 2 * H2 * H2 * C * 2 + H2 * H2
    cf = 2.0 * nb * 256 * 9 * C * C
    out["bandwidth_1024x1024x128_all_blocks"] = {
        "active_blocks": nb,
        "gather_plain_us": round(gp_us, 1), "gather_plain_GBs": round(gb / gp_us / 1e3, 1),
        "gather_plain_frac_hbm_peak": round(gb / gp_us / 1e3 / HBM_PEAK_GBS, 4),
        "gather_fused_gn_silu_us": round(g_us, 1), "gather_fused_gn_silu_GBs": round(gb / g_us / 1e3, 1),
        "gather_fused_gn_silu_frac_hbm_peak": round(gb / g_us / 1e3 / HBM_PEAK_GBS, 4),
        "scatter_us": round(s_us, 1), "scatter_GBs": round(sb / s_us / 1e3, 1),
        "scatter_frac_hbm_peak": round(sb / s_us / 1e3 / HBM_PEAK_GBS, 4),
        "diff_mask_us": round(d_us, 1), "diff_mask_GBs": round(db / d_us / 1e3, 1),
        "diff_mask_frac_hbm_peak": round(db / d_us / 1e3 / HBM_PEAK_GBS, 4),
        "conv3x3_us": round(c_us, 1), "conv3x3_tflops": round(cf / c_us / 1e6, 1),
        "conv3x3_frac_mfma_peak": round(cf / c_us / 1e6 / MFMA_PEAK_TFLOPS["f16"], 4)}
    del x, x2, t2, o2, y2

    # ---- sparse-query attention at the Stable-Diffusion 64x64 level (bf16, 8 heads x 40)
    att = {}
    T, heads, d = 4096, 8, 40
    for frac, nq in (("1pct", 96), ("5pct", 400), ("20pct", 1200), ("all_queries", 4096)):
        cs = inputs.attention_case(7, T, heads, d, nq, "bf16")
        q, k, v = cs["q"].cuda(), cs["k"].cuda(), cs["v"].cuda()
        o = torch.empty_like(q)
        nbytes = api.sige_sparse_attn_workspace_bytes(nq, T, heads, d)
        wsb = torch.empty(max(nbytes // 4, 1), dtype=torch.float32, device="cuda") if nbytes else None
        us = time_calls(lambda: api.sige_sparse_attn(q, k, v, o, cs["scale"], workspace=wsb), 50, 5)
        att[frac] = {"n_q": nq, "us": round(us, 1), "tflops": round(4.0 * nq * T * heads * d / us / 1e6, 2)}
    att["all_over_1pct_speedup"] = round(att["all_queries"]["us"] / att["1pct"]["us"], 2)
    out["sparse_attention_T4096_h8_d40_bf16"] = att

    # ---- the synthetic DDPM-style UNet step (benchmark configuration 3)
    if with_unet:
        from paper_2211_02048_amd.unet import SigeUNet
        net = SigeUNet()
        un = {"config": "256x256x3, channels 128/128/256/256/512/512, 2 ResBlocks per level, attention at "
                        "16x16, fp16, 16x16 blocks, dilation 1, sparse layers at resolution >= 64",
              "dense_gmacs": round(net.macs() / 1e9, 1)}
        for name, frac in (("edit_1.2pct", 0.012), ("edit_15.5pct", 0.155)):
            io, ie, mask = inputs.unet_images(1003, 256, frac)
            io, ie = io.cuda(), ie.cuda()
            md = torch.from_numpy(mask).cuda()
            gd = net.capture_dense(io)      # a plain dense model: every block, statistics on the fly, one graph
            gd.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                gd.replay()
            torch.cuda.synchronize()
            dense_ms = (time.perf_counter() - t0) / 10 * 1e3
            del gd
            net.precompute(io)              # the pre-computation pass: caches, statistics, activated copies
            counts = net.set_edit(md, exact=False)
            g = net.capture(ie)
            for _ in range(5):
                g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(50):
                g.replay()
            torch.cuda.synchronize()
            sparse_ms = (time.perf_counter() - t0) / 50 * 1e3
            un[name] = {"edited_px": int(mask.sum()), "dense_step_ms": round(dense_ms, 3),
                        "sparse_step_ms": round(sparse_ms, 3), "speedup": round(dense_ms / sparse_ms, 2),
                        "sparse_gmacs": round(net.macs(counts) / 1e9, 1),
                        "macs_reduction": round(net.macs() / net.macs(counts), 2)}
        un["note"] = ("dense = the same kernels with every block active and group statistics computed on the "
                      "fly, one HIP graph replay; sparse = one HIP graph replay, cached statistics, activated "
                      "copies written by the producing layers, device-side block counts")
        out["unet_step_config3"] = un
        del net
        torch.cuda.empty_cache()

        # ---- the synthetic latent-diffusion style UNet step (benchmark configuration 4)
        net = SigeUNet(64, (320, 640, 1280, 1280), (64, 32, 16), 8, dtype="bf16", seed=1004, block=8, dilate=1,
                       min_sparse_res=16, in_ch=4, attn_kind="xfmr", ctx=(77, 768))
        sd = {"config": "64x64x4 latent, channels 320/640/1280/1280, 2 ResBlocks per level each followed by a "
                        "transformer block (self-attention 8 heads of 40/80/160, cross-attention over 77x768 text "
                        "embeddings, gated-GELU feed-forward) at 64/32/16, bf16, 8x8 blocks, dilation 1, sparse "
                        "layers at resolution >= 16",
              "dense_gmacs": round(net.macs() / 1e9, 1)}
        for name, frac in (("edit_1pct", 0.01), ("edit_5pct", 0.05), ("edit_20pct", 0.20)):
            io, ie, mask = inputs.unet_images(1004, 64, frac, "bf16", in_ch=4)
            io, ie = io.cuda(), ie.cuda()
            md = torch.from_numpy(mask).cuda()
            gd = net.capture_dense(io)
            gd.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                gd.replay()
            torch.cuda.synchronize()
            dense_ms = (time.perf_counter() - t0) / 5 * 1e3
            del gd
            net.precompute(io)
            counts = net.set_edit(md, exact=True)      # the attention calls are sized by the host counts
            g = net.capture(ie)
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                g.replay()
            torch.cuda.synchronize()
            sparse_ms = (time.perf_counter() - t0) / 20 * 1e3
            b0 = net.layers["down0.0.attn"]["list"][1]
            sd[name] = {"edited_latent_px": int(mask.sum()),
                        "active_tokens_64x64": b0.n_host * b0.g.block_h * b0.g.block_w,
                        "dense_step_ms": round(dense_ms, 3), "sparse_step_ms": round(sparse_ms, 3),
                        "speedup": round(dense_ms / sparse_ms, 2), "sparse_gmacs": round(net.macs(counts) / 1e9, 1),
                        "macs_reduction": round(net.macs() / net.macs(counts), 2)}
        sd["note"] = ("dense = the same kernels with every block active (all queries) and group statistics computed "
                      "on the fly, one HIP graph replay; sparse = one HIP graph replay with the block counts of the edit baked in; only "
                      "the active tokens' queries are recomputed, keys and values overwritten in their caches")
        out["unet_step_config4"] = sd
        del net
        torch.cuda.empty_cache()

        # ---- the synthetic SPADE-style conditional generator (benchmark configuration 5): ten successive
        # label edits of ~1 % each, every one reusing and updating the caches of the previous one
        from paper_2211_02048_amd.spade import SigeSpade
        net = SigeSpade()
        sizes = [(8 << i, 16 << i) for i in range(6)]
        onehot = lambda lab: {k: v.cuda() for k, v in inputs.one_hot_pyramid(lab, sizes, 35, 48).items()}
        lab = inputs.label_map(1005, 256, 512)
        seg = onehot(lab)
        net.precompute(seg)
        net.precompute(seg)
        torch.cuda.synchronize()
        gd = torch.cuda.CUDAGraph()         # the dense pass as one graph, like the sparse steps
        with torch.cuda.graph(gd):
            net.precompute(seg)
        gd.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            gd.replay()
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - t0) / 5 * 1e3
        del gd
        gen = {"config": "output 256x512 from a constant 8x16x1024 start, 7 SPADE residual blocks (1024, 1024, 1024, 512, "
                         "256, 128, 64 channels) with x2 up-sampling in between, modulation from a 35-class one-hot "
                         "label map (128 hidden channels), fp16, 16x16 blocks, dilation 1, instance-norm statistics "
                         "cached above 16x32, sparse layers above 8x16",
               "dense_gmacs": round(net.macs() / 1e9, 1), "dense_step_ms": round(dense_ms, 3), "edits": []}
        tot = 0.0
        for e in range(10):
            new = inputs.relabel(2000 + e, lab, 0.01)
            t0 = time.perf_counter()
            counts = net.set_edit(onehot(new), exact=False)
            torch.cuda.synchronize()
            g = net.capture()          # capture runs the step (warm-up + capture): the caches now hold edit e
            t0 = time.perf_counter()
            for _ in range(20):        # replays recompute the same edit on the already updated caches
                g.replay()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) / 20 * 1e3
            tot += ms
            gen["edits"].append({"changed_px": int((new != lab).sum()), "active_blocks_256x512": counts[(256, 512)],
                                 "sparse_step_ms": round(ms, 3),
                                 "macs_reduction": round(net.macs() / net.macs(counts), 2)})
            lab = new
        gen["mean_sparse_step_ms"] = round(tot / 10, 3)
        gen["speedup"] = round(dense_ms / (tot / 10), 2)
        gen["note"] = ("each edit relabels ~1 % of the pixels of the CURRENT label map; its mask is the difference "
                       "against the current one-hot map, the caches are updated in place and serve the next edit")
        out["generator_step_config5"] = gen
    return out


def probe():
    """A short, fixed sequence of launches for counter collection: a plain device copy of known size
    (the yardstick FETCH_SIZE / WRITE_SIZE are scaled by), then the kernels the rooflines quote."""
    import torch
    from paper_2211_02048_amd import api, inputs
    from paper_2211_02048_amd.layers import BlockList, SigeConv, Workspace
    cfg = inputs.config2()
    L = Layer2(cfg, fused=True)
    n3, n1 = L.capture()
    src = torch.randn(64 * 1024 * 1024, dtype=torch.float16, device="cuda")   # 128 MiB
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)                                   # yardstick 1 (runtime's copy kernel): 128 MiB each way
    for _ in range(3):
        torch.neg(src, out=dst)                          # yardstick 2 (16-byte vector loads): 128 MiB each way
    for _ in range(3):
        api.sige_reduce_mask(L.main.g, None, None, a_orig=L.a_o, a_edit=L.a_e, tau=cfg["tau"], mask_out=L.mask)
    L.bl3.sync_count(), L.bl1.sync_count()
    for _ in range(3):
        L.main.forward(L.a_e, L.y_main, L.bl3, L.ws, scale=L.scale, shift=L.shift, act=api.ACT_SILU, fused=True)
    for _ in range(3):
        L.main.forward(L.a_e, L.y_main, L.bl3, L.ws, scale=L.scale, shift=L.shift, act=api.ACT_SILU, fused=False)
    H2, C = 1024, cfg["Cin"]
    x = torch.randn((H2, H2, C), dtype=torch.float16, device="cuda")
    x2 = x.clone()
    big = SigeConv(cfg["w"].cuda(), cfg["bias"], H2, H2, 16, 1, 1)
    bl = BlockList(big.g, "cuda").all_active()
    nb = bl.n_host
    t2 = torch.empty(big.tiles_numel(nb), dtype=torch.float16, device="cuda")
    o2 = torch.empty(big.out_numel(nb), dtype=torch.float16, device="cuda")
    y2 = torch.empty((H2, H2, C), dtype=torch.float16, device="cuda")
    mask_o = torch.zeros((H2, H2), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        api.sige_reduce_mask(big.g, None, None, a_orig=x, a_edit=x2, tau=0.0, mask_out=mask_o)
        api.sige_gather(x, big.g, bl.indices, bl.count, t2, n_blocks=nb, max_blocks=nb)
        api.sige_gather(x, big.g, bl.indices, bl.count, t2, n_blocks=nb, scale=L.scale, shift=L.shift,
                        act=api.ACT_SILU, max_blocks=nb)
        api.sige_conv(t2, big.g, C, C, big.packed, big.bias, bl.count, o2, n_blocks=nb, max_blocks=nb)
        api.sige_scatter(o2, big.g, bl.indices, bl.count, y2, n_blocks=nb, Cout=C, max_blocks=nb)
    torch.cuda.synchronize()
    print(json.dumps({"probe": "done", "copy_bytes_each_way": src.numel() * 2, "active_blocks_config2": n3,
                      "blocks_1024": nb}))


def main():
    args = parse()
    if args.probe:
        probe()
        return
    if args.gpus != 1:
        print(f"bench.py: this build measures one MI355X; --gpus {args.gpus} is not supported "
              "(one GPU per box, no collectives in this path)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2211_02048_amd import api, inputs
    api.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = inputs.config2()
    L = Layer2(cfg, fused=not args.three_calls)
    n3, n1 = L.capture()

    for _ in range(args.warmup):
        L.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        L.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    assert (L.bl3.sync_count(), L.bl1.sync_count()) == (n3, n1) and n3 <= L.capacity
    n_bytes, diff_bytes = L.bytes_per_step(n3, n1)
    eager_us = time_calls(L.step_eager, 100)
    L.bl3.sync_count(), L.bl1.sync_count()

    # MFMA roofline: the 3x3 convolution on the active blocks
    if L.fused:
        conv_call = lambda: L.main.forward(L.a_e, L.y_main, L.bl3, L.ws, scale=L.scale, shift=L.shift,
                                           act=api.ACT_SILU, fused=True)
    else:
        tl = L.ws.get("tiles", L.main.tiles_numel(n3), L.a_e.dtype)
        ot = L.ws.get("out_main", L.main.out_numel(n3), L.a_e.dtype)
        conv_call = lambda: api.sige_conv(tl, L.main.g, cfg["Cin"], cfg["Cout"], L.main.packed, L.main.bias,
                                          L.bl3.count, ot, n_blocks=n3, max_blocks=n3)
    conv_us = time_graphed(conv_call)
    conv_fl = 2.0 * n3 * cfg["block"] ** 2 * 9 * cfg["Cin"] * cfg["Cout"]
    roof = {"bound": "mfma", "kernel": "conv_kernel (sige_fused_conv)" if L.fused else "conv_kernel (sige_conv)",
            "achieved": round(conv_fl / conv_us / 1e6, 2), "peak": MFMA_PEAK_TFLOPS["f16"], "unit": "TFLOP/s",
            "frac": round(conv_fl / conv_us / 1e6 / MFMA_PEAK_TFLOPS["f16"], 5),
            "traffic": PMC_TRAFFIC_FUSED_CONV_CONFIG2 if L.fused else None,
            "flop_per_launch": conv_fl, "avg_launch_us": round(conv_us, 2),
            "timing": "20 launches per HIP graph, replays timed with events on the stream",
            "note": f"{n3} active 16x16 blocks, 3x3, 128->128, fp16: {conv_fl / 1e9:.2f} GFLOP per launch - far too "
                    "little work to fill 256 CUs; the supplement has the same kernel with every block active"}

    # HBM roofline (the dominant kernel of a bandwidth metric): the difference-mask stream, both
    # activations read once.
    # Rotated over distinct buffer pairs (> 256 MB in total) so that the Infinity Cache cannot serve them.
    pairs = [(L.a_o.clone(), L.a_e.clone()) for _ in range(10)]
    it = [0]

    def diff_cold():
        a, e = pairs[it[0] % len(pairs)]
        it[0] += 1
        api.sige_reduce_mask(L.main.g, None, None, a_orig=a, a_edit=e, tau=cfg["tau"], mask_out=L.mask)
    diff_us = time_graphed(diff_cold, per_graph=20)   # 20 launches per graph = two passes over the 10 pairs
    diff_warm_us = time_graphed(lambda: api.sige_reduce_mask(L.main.g, None, None, a_orig=L.a_o, a_edit=L.a_e,
                                                             tau=cfg["tau"], mask_out=L.mask))
    roof_hbm = {"bound": "hbm", "kernel": "diff_mask_pow2 (sige_reduce_mask, mask only)",
                "achieved": round(diff_bytes / diff_us / 1e3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(diff_bytes / diff_us / 1e3 / HBM_PEAK_GBS, 4),
                "traffic": PMC_TRAFFIC_DIFF_MASK_CONFIG2,
                "bytes_per_launch": diff_bytes, "avg_launch_us": round(diff_us, 2),
                "same_buffers_every_launch_us": round(diff_warm_us, 2),
                "note": "inputs rotated over 10 buffer pairs (335 MB); 20 launches per HIP graph, replays timed with "
                        "events on the stream"}
    del pairs

    res = {"metric": "sparse-conv gather/scatter GB/s", "value": round(n_bytes / (ms_per_step * 1e-3) / 1e9, 2),
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f16", "data": "synthetic",
           "config": {"workload": "benchmark configuration 2: GN(32, cached stats)+SiLU+3x3 conv 128->128 and 1x1 shortcut "
                                  "128->256, 256x256 fp16, ~1% blob edit, 16x16 blocks; step = diff mask + block "
                                  "lists + gather/conv/scatter for both convs",
                      "launch": f"one HIP graph per step, device-side block counts, capacity {L.capacity} blocks, "
                                + ("fused gather-conv-scatter calls of both convolutions in one launch" if L.fused else "gather, conv, scatter kernels"),
                      "eager_step_ms_with_count_readback": round(eager_us / 1e3, 4),
                      "active_blocks_3x3": n3, "active_blocks_1x1": n1, "grid_blocks": L.main.g.grid_blocks,
                      "algorithmic_bytes_per_step": n_bytes, "mfma_flop_per_step": L.flops_per_step(n3, n1)},
           "roofline": roof_hbm, "roofline_mfma": roof}
    if not args.no_supplement:
        res["supplement"] = supplement(L, not args.no_unet)
    res["cpu_baseline"] = None if args.no_cpu else cpu_baseline(cfg, n_bytes)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
