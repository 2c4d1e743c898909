"""GPU parity of a whole UNet step (pre-computation pass, then the sparse edit pass) against the
step-by-step dense-then-select oracle, on a 64x64 replica of the benchmark configuration 3 network (same
topology, six levels, two ResBlocks per level, attention at the fifth level, narrower channels so
the CPU oracle finishes in seconds)."""
import numpy as np
import pytest
import torch

from helpers import f64, round_to
from paper_2211_02048_amd import api, inputs
from paper_2211_02048_amd.unet import SigeUNet

pytestmark = pytest.mark.gpu

RES, CH, ATT, HEADS, BLOCK, MIN_SPARSE = 64, (32, 32, 64, 64, 128, 128), (4,), 4, 8, 16


def rel_err(got, want):
    rms = np.sqrt(np.mean(want * want)) + 1e-30
    return np.abs(got - want).max() / rms, np.sqrt(np.mean((got - want) ** 2)) / rms


@pytest.fixture(scope="module", params=["f16", "f32"])
def setup(request):
    import oracle
    from oracle import unet as ounet
    dtype = request.param
    att = ATT
    bufs, ops = inputs.unet_topology(RES, 3, CH, att, HEADS)
    P = inputs.unet_params(1003, ops, dtype)
    img_o, img_e, mask = inputs.unet_images(1003, RES, 0.03, dtype)
    trace_d, trace_e = [], []
    cache, stats = ounet.unet_pass(bufs, ops, P, f64(img_o), storage=dtype, block=BLOCK, trace=trace_d)
    edit, blocks = ounet.unet_pass(bufs, ops, P, f64(img_e), storage=dtype, block=BLOCK, cache=cache,
                                   stats=stats, mask=mask, dilate=1, min_sparse_res=MIN_SPARSE, trace=trace_e)
    net = SigeUNet(RES, CH, att, HEADS, dtype=dtype, block=BLOCK, dilate=1, min_sparse_res=MIN_SPARSE, params=P)
    return dict(dtype=dtype, bufs=bufs, ops=ops, img_o=img_o, img_e=img_e, mask=mask, cache=cache, edit=edit,
                blocks=blocks, net=net, oracle=oracle, stats=stats, trace_d=trace_d, trace_e=trace_e)


def teacher_forced(s, inner=False):
    """Both passes of a network under teacher forcing (see teacher.py): every library call of every layer
    gets the oracle's tensors as input and is compared with the oracle's output at the per-layer
    tolerance.  Returns the two reports."""
    from teacher import UNetTeacher
    net, td = s["net"], inputs.DTYPES[s["dtype"]]
    zeros = {n: np.zeros(shape) for n, shape in s["bufs"].items()}
    zeros["image"] = f64(s["img_o"])
    t_d = UNetTeacher(net, td, s["trace_d"], zeros)
    net.hook = t_d
    try:
        net.precompute(s["img_o"].cuda())
        torch.cuda.synchronize()
        # the statistics the pre-computation pass leaves behind, from the oracle's tensors
        for n, L in net.layers.items():
            if "scale" in L:
                sc, sh = s["stats"][n]
                np.testing.assert_allclose(f64(L["scale"]), sc, rtol=5e-5, atol=1e-6, err_msg=n)
                np.testing.assert_allclose(f64(L["shift"]), sh, rtol=0, atol=2e-4 * max(1.0, np.abs(sh).max()), err_msg=n)
        start = {n: a.copy() for n, a in s["cache"].items()}
        start["image"] = f64(s["img_e"])
        t_e = UNetTeacher(net, td, s["trace_e"], start, stats=s["stats"], inner_cache=s["cache"])
        net.hook = None
        net.set_edit(torch.from_numpy(s["mask"]).cuda(), exact=True)
        t_e.prepare_edit(dict(s["trace_d"]) if inner else None)
        net.hook = t_e
        net.step(s["img_e"].cuda())
        torch.cuda.synchronize()
    finally:
        net.hook = None
    return t_d.rep, t_e.rep


def test_unet_every_layer_teacher_forced(setup):
    """The per-layer bar inside the network: 1e-2 (fp16) / 1e-4 (fp32), element-wise, for every stored
    tensor of the pre-computation pass and of the sparse step, each computed by the GPU from the
    oracle's own inputs in the kernel shape the network selects."""
    rep_d, rep_e = teacher_forced(setup)
    rep_d.assert_clean(min_checked=70)
    rep_e.assert_clean(min_checked=70)


@pytest.mark.parametrize("area", [0.012, 0.155])
def test_unet_full_size_every_layer_teacher_forced(area):
    """Benchmark configuration 3 at FULL size (256x256 image, channels 128/128/256/256/512/512, two
    ResBlocks per level, attention at 16x16, fp16, 16x16 blocks, blob edits of ~1.2 % and 15.5 % - the two
    edited areas of the paper's showcased DDPM example, Tab. 2 - sparse layers at
    resolution >= 64): both passes under teacher forcing, every stored tensor of every layer compared
    element by element at 1e-2 with the oracle, which computes each layer densely on the whole map.
    This reaches the kernel selections of the real step (the launch shared by a ResBlock's first
    convolution and its shortcut, the eight-wave whole-Cin shapes of the 512-channel layers, the K split
    over workgroups with its second kernel, the few-row 1x1 kernel, attention at T = 256), which the
    64x64 replica does not.  Block lists bit for bit."""
    from oracle import unet as ounet
    dtype, res, ch, block = "f16", 256, (128, 128, 256, 256, 512, 512), 16
    bufs, ops = inputs.unet_topology(res, 3, ch, (16,), 4)
    P = inputs.unet_params(1003, ops, dtype)
    img_o, img_e, mask = inputs.unet_images(1003, res, area, dtype)
    trace_d, trace_e = [], []
    print("oracle: dense pass on the original image", flush=True)
    cache, stats = ounet.unet_pass(bufs, ops, P, f64(img_o), storage=dtype, block=block, trace=trace_d)
    print("oracle: edit pass", flush=True)
    edit, blocks = ounet.unet_pass(bufs, ops, P, f64(img_e), storage=dtype, block=block, cache=cache, stats=stats,
                                   mask=mask, dilate=1, min_sparse_res=64, trace=trace_e)
    net = SigeUNet(res, ch, (16,), 4, dtype=dtype, block=block, dilate=1, min_sparse_res=64, params=P)
    s = dict(dtype=dtype, bufs=bufs, ops=ops, img_o=img_o, img_e=img_e, mask=mask, cache=cache, edit=edit,
             blocks=blocks, net=net, stats=stats, trace_d=trace_d, trace_e=trace_e)
    print("GPU: both passes under teacher forcing", flush=True)
    rep_d, rep_e = teacher_forced(s)
    n_sparse = 0
    for n, L in net.layers.items():
        if L["sparse"] and L["op"]["kind"] == "conv" and L["op"]["scatter"]:
            bl = L["list"][1]
            assert np.array_equal(bl.indices[:bl.n_host].cpu().numpy(), blocks[n]), n
            assert 0 < bl.n_host < bl.g.grid_blocks
            n_sparse += 1
    assert n_sparse >= 20
    # which kernels the sparse step selected, by layer sizes
    td, seen = inputs.DTYPES[dtype], set()
    for n, L in net.layers.items():
        if "conv" not in L:
            continue
        c, bl = L["conv"], L["list"][1 if L["sparse"] else 0]
        key = (c.g.H_in, c.g.k, c.g.stride, c.Cin, c.Cout)
        if key in seen:
            continue
        seen.add(key)
        nb = max(bl.n_host, 1)
        nbytes = api.sige_conv_workspace_bytes(td, c.g, c.Cin, c.Cout, nb)
        print(f"{c.g.H_in}x{c.g.W_in} {c.g.k}x{c.g.k}/{c.g.stride} {c.Cin}->{c.Cout}, {nb} blocks: "
              f"{api.sige_conv_plan(td, c.g, c.Cin, c.Cout, nb, workspace_bytes=nbytes)!r}")
    print(f"worst error / bound: pre-computation pass {rep_d.worst:.3f}, sparse step {rep_e.worst:.3f}")
    rep_d.assert_clean(min_checked=80)
    rep_e.assert_clean(min_checked=80)


def test_unet_precompute_and_sparse_step(setup):
    s = setup
    net, td = s["net"], inputs.DTYPES[s["dtype"]]
    # SECOND check, on the free-running chain (the per-layer bar is held by the teacher-forced test
    # above): along ~80 stored layers the two implementations' rounding decisions drift apart, which
    # is asserted as a drift bound - the per-layer bar on the rms error, a modest growth factor on the
    # maximum
    tol = 1e-4 if s["dtype"] == "f32" else 1e-2
    net.precompute(s["img_o"].cuda())
    torch.cuda.synchronize()
    gpu_cache = {n: b.clone() for n, b in net.B.items()}
    for n, want in s["cache"].items():
        if n == "image":
            continue
        mx, rms = rel_err(f64(net.B[n]), round_to(want, td))
        assert rms <= tol and mx <= 8 * tol, ("precompute", n, mx, rms)

    counts = net.set_edit(torch.from_numpy(s["mask"]).cuda())
    # block lists: bit-exact against the oracle, for every sparse layer
    for n, L in net.layers.items():
        if L["sparse"] and L["op"]["kind"] == "conv" and L["op"]["scatter"]:
            bl = L["list"][1]
            assert np.array_equal(bl.indices[:bl.n_host].cpu().numpy(), s["blocks"][n]), n
    assert all(0 < c for c in counts.values())
    net.step(s["img_e"].cuda())
    torch.cuda.synchronize()
    for n, want in s["edit"].items():
        if n == "image":
            continue
        mx, rms = rel_err(f64(net.B[n]), round_to(want, td))
        assert rms <= tol and mx <= 8 * tol, ("edit", n, mx, rms)
    # on sparse layers everything outside the active blocks is the cache, bit for bit
    checked = 0
    for n, L in net.layers.items():
        op = L["op"]
        if not (L["sparse"] and op["kind"] == "conv" and op["scatter"]):
            continue
        g = L["conv"].g
        keep = np.ones((g.H_out, g.W_out), bool)
        for y0, x0 in s["blocks"][n]:
            keep[y0:y0 + g.block_h, x0:x0 + g.block_w] = False
        if not keep.any():
            continue
        # a later op may write the same view in place (none does at sparse levels here), so compare
        # the view this op wrote
        k = torch.from_numpy(keep).cuda()
        now = net.view(op["y"])[k]
        before = gpu_cache[op["y"][0]][:, :, op["y"][1]:op["y"][1] + op["y"][2]][k]
        assert torch.equal(now, before), n
        checked += 1
    assert checked >= 20
    # the edit really changed the output, and only moderately many blocks were touched
    assert not torch.equal(net.B["out"], gpu_cache["out"])
    # the three-call path (gather with Scale+Shift and SiLU, conv, scatter; no activated copies) gives
    # the same bits as the fused calls with the copies written by the producing layers
    fused_run = {n: b.clone() for n, b in net.B.items()}
    net.fused = False
    for n in gpu_cache:                      # same caches, same cached statistics
        net.B[n].copy_(gpu_cache[n])
    net.step(s["img_e"].cuda())
    torch.cuda.synchronize()
    net.fused = True
    # (without residuals the two paths write the same bits; a layer with a residual rounds once in the
    # fused call and twice in the three calls, where the output tiles are a stored tensor)
    n_same = 0
    for n in fused_run:
        mx, rms = rel_err(f64(net.B[n]), f64(fused_run[n]))
        assert rms <= tol and mx <= 8 * tol, ("fused vs three calls", n, mx, rms)
        n_same += bool(torch.equal(net.B[n], fused_run[n]))
    assert n_same >= 3
    # and the copies hold exactly what a fused gather would compute from the tensors they mirror
    net.precompute(s["img_o"].cuda())
    net.step(s["img_e"].cuda())
    n_copies = 0
    for n, L in net.layers.items():
        if "pre" not in L or L["op"]["x"] == L["op"].get("y"):
            continue            # (an attention block overwrites its input in place: nothing left to compare with)
        x = net.view(L["op"]["x"])
        keep = L["pre"].clone()
        act = api.ACT_SILU if (L["op"]["kind"] == "conv" and L["op"]["act"]) else api.ACT_NONE
        net._fill_copy(L, x, L["scale"], L["shift"], act)
        assert torch.equal(L["pre"], keep), ("activated copy", n)
        n_copies += 1
    assert n_copies >= 20


def test_unet_zero_edit_and_graph_replay(setup):
    s = setup
    net = s["net"]
    net.precompute(s["img_o"].cuda())
    torch.cuda.synchronize()
    ref = {n: b.clone() for n, b in net.B.items()}
    # no edit: empty mask, original image -> sparse layers touch nothing, dense layers recompute the same
    net.set_edit(torch.zeros((RES, RES), dtype=torch.uint8, device="cuda"))
    net.step(s["img_o"].cuda())
    torch.cuda.synchronize()
    for n in ref:
        assert torch.equal(net.B[n], ref[n]), n
    # eager sparse step vs graph replays of the same step (device-side counts, capacity-sized launches)
    for n in ref:
        net.B[n].copy_(ref[n])
    net.set_edit(torch.from_numpy(s["mask"]).cuda(), exact=True)
    net.step(s["img_e"].cuda())
    torch.cuda.synchronize()
    eager = {n: b.clone() for n, b in net.B.items()}
    for n in ref:
        net.B[n].copy_(ref[n])
    net.set_edit(torch.from_numpy(s["mask"]).cuda(), exact=False)
    img_e = s["img_e"].cuda()
    g = net.capture(img_e)
    for rep in range(3):
        for n in ref:                          # eager work between the replays resets the caches
            net.B[n].copy_(ref[n])
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for n in eager:
            assert torch.equal(net.B[n], eager[n]), (rep, n)


# ---------------------------------------------------------------------------------------------
# Latent-diffusion style replica (benchmark configuration 4 at small size): transformer blocks with
# self-attention on the active tokens only, cross-attention over text embeddings, gated-GELU
# feed-forward; 16x16x4 latent, channels 32/64/64/64, attention at 16/8/4, 7 text tokens of width 32.
# ---------------------------------------------------------------------------------------------
SD = dict(res=16, in_ch=4, channels=(32, 64, 64, 64), attn_res=(16, 8, 4), heads=2, block=4, min_sparse=4,
          ctx=(7, 32))


@pytest.fixture(scope="module", params=["bf16", "f16"])
def sd_setup(request):
    import oracle
    from oracle import unet as ounet
    dtype = request.param
    bufs, ops = inputs.unet_topology(SD["res"], SD["in_ch"], SD["channels"], SD["attn_res"], SD["heads"],
                                     attn_kind="xfmr", ctx=SD["ctx"])
    P = inputs.unet_params(1004, ops, dtype, in_ch=SD["in_ch"])
    img_o, img_e, mask = inputs.unet_images(1004, SD["res"], 0.06, dtype, in_ch=SD["in_ch"])
    trace_d, trace_e = [], []
    cache, stats = ounet.unet_pass(bufs, ops, P, f64(img_o), storage=dtype, block=SD["block"], trace=trace_d)
    edit, blocks = ounet.unet_pass(bufs, ops, P, f64(img_e), storage=dtype, block=SD["block"], cache=cache,
                                   stats=stats, mask=mask, dilate=1, min_sparse_res=SD["min_sparse"], trace=trace_e)
    net = SigeUNet(SD["res"], SD["channels"], SD["attn_res"], SD["heads"], dtype=dtype, block=SD["block"], dilate=1,
                   min_sparse_res=SD["min_sparse"], params=P, in_ch=SD["in_ch"], attn_kind="xfmr", ctx=SD["ctx"])
    return dict(dtype=dtype, bufs=bufs, ops=ops, img_o=img_o, img_e=img_e, mask=mask, cache=cache, edit=edit,
                blocks=blocks, net=net, stats=stats, trace_d=trace_d, trace_e=trace_e)


def inner_tensor(L, part):
    """A transformer block's cached tensor by the oracle's name: its keys and values are the last
    two thirds of the cached queries | keys | values."""
    if part == "kv":
        return L["qkv"][:, :, L["op"]["C"]:]
    return L[part]


def test_latent_unet_every_call_teacher_forced(sd_setup):
    """The per-layer bar inside the latent-diffusion replica: 1e-2 element-wise (fp16 and bf16) for
    every stored tensor of both passes - convolutions, and inside the transformer blocks every
    library call (token norms, projections, both attentions, gated-GELU feed-forward, the residual
    scatters) - each computed by the GPU from the oracle's own inputs."""
    rep_d, rep_e = teacher_forced(sd_setup, inner=True)
    rep_d.assert_clean(min_checked=200)
    rep_e.assert_clean(min_checked=200)


def test_latent_unet_transformer_blocks(sd_setup):
    """SECOND check, on the free-running chain (the per-layer bar is held by the teacher-forced test
    above).  Whole pre-computation pass and sparse step against the step-by-step oracle; across ~150 stored tensors the two
    implementations' rounding decisions drift apart (each stored tensor is rounded to the storage
    type, unit roundoff u = 2^-11 for fp16, 2^-8 for bf16), and the drift measured along the chain
    grows smoothly to about 4 u rms.  The chain is therefore asserted at rms <= 10 u and
    max <= 80 u of the tensor's rms (fp16: 4.9e-3 / 3.9e-2, bf16: 3.9e-2 / 0.31), block lists bit for
    bit, everything outside the active blocks bit for bit."""
    s = sd_setup
    net, td = s["net"], inputs.DTYPES[s["dtype"]]
    tol = 10.0 * (2.0 ** -8 if s["dtype"] == "bf16" else 2.0 ** -11)
    net.precompute(s["img_o"].cuda())
    torch.cuda.synchronize()
    names = [n for n in s["cache"] if n != "image" and n in net.B]
    for n in names:
        mx, rms = rel_err(f64(net.B[n]), round_to(s["cache"][n], td))
        assert rms <= tol and mx <= 8 * tol, ("precompute", n, mx, rms)
    # the internal tensors of every transformer block, too (caches of the method)
    for n, L in net.layers.items():
        if L["op"]["kind"] == "xfmr":
            for part in ("h0", "kv", "h1", "h2", "h3"):
                mx, rms = rel_err(f64(inner_tensor(L, part)), round_to(s["cache"][f"{n}.{part}"], td))
                assert rms <= tol and mx <= 8 * tol, ("precompute", n, part, mx, rms)
    gpu_cache = {n: b.clone() for n, b in net.B.items()}
    copies = {n: L["pre"].clone() for n, L in net.layers.items() if "pre" in L}   # activated copies: caches too
    assert len(copies) >= 10
    inner = {(n, part): L[part].clone() for n, L in net.layers.items() if L["op"]["kind"] == "xfmr"
             for part in ("h0", "qkv", "h1", "h2", "h3")}
    counts = net.set_edit(torch.from_numpy(s["mask"]).cuda(), exact=True)
    assert all(0 < c for c in counts.values())
    n_sparse_x = 0
    for n, L in net.layers.items():
        if L["sparse"] and L["op"]["kind"] == "xfmr":
            bl = L["list"][1]
            assert np.array_equal(bl.indices[:bl.n_host].cpu().numpy(), s["blocks"][n]), n
            assert bl.n_host < bl.g.grid_blocks or bl.g.grid_blocks <= 4
            n_sparse_x += 1
    assert n_sparse_x >= 8
    net.step(s["img_e"].cuda())
    torch.cuda.synchronize()
    for n in names:
        mx, rms = rel_err(f64(net.B[n]), round_to(s["edit"][n], td))
        assert rms <= tol and mx <= 8 * tol, ("edit", n, mx, rms)
    for n, L in net.layers.items():
        if L["op"]["kind"] != "xfmr":
            continue
        g1 = L["g1"]
        keep = np.ones((g1.H_out, g1.W_out), bool)
        for y0, x0 in s["blocks"][n]:
            keep[y0:y0 + g1.block_h, x0:x0 + g1.block_w] = False
        k = torch.from_numpy(keep).cuda()
        for part in ("h0", "kv", "h1", "h2", "h3"):
            mx, rms = rel_err(f64(inner_tensor(L, part)), round_to(s["edit"][f"{n}.{part}"], td))
            assert rms <= tol and mx <= 8 * tol, ("edit", n, part, mx, rms)
        for part in ("h0", "qkv", "h1", "h2", "h3"):
            # tokens outside the active blocks: the caches, bit for bit (queries, keys and values included)
            assert torch.equal(L[part][k], inner[(n, part)][k]), (n, part)
    assert not torch.equal(net.B["out"], gpu_cache["out"])
    # zero edit: nothing moves
    for n in gpu_cache:
        net.B[n].copy_(gpu_cache[n])
    for (n, part), t in inner.items():
        net.layers[n][part].copy_(t)
    for n, t in copies.items():
        net.layers[n]["pre"].copy_(t)
    net.set_edit(torch.zeros((SD["res"], SD["res"]), dtype=torch.uint8, device="cuda"), exact=True)
    net.step(s["img_o"].cuda())
    torch.cuda.synchronize()
    for n in gpu_cache:
        assert torch.equal(net.B[n], gpu_cache[n]), n


# ---------------------------------------------------------------------------------------------
# Benchmark configuration 4 at FULL layer sizes, one resolution level at a time: a one-level network
# with the channel count, resolution, head size, text-embedding shape and block size of that level of
# the latent-diffusion step (conv-in, two ResBlocks each followed by a transformer block, two
# ResBlocks in the middle, two ResBlocks on cat(h, skip) each followed by a transformer block,
# conv-out), ~1 % edit, bf16.  Every library call of both passes is compared under teacher forcing
# with the oracle, which computes each layer on the whole map; the kernel every convolution selects
# is reported.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("res,C,area", [(64, 320, 0.01), (32, 640, 0.02), (16, 1280, 0.03)])
def test_latent_unet_full_size_level_teacher_forced(res, C, area):
    from oracle import unet as ounet
    dtype, block, heads, ctx = "bf16", 8, 8, (77, 768)
    bufs, ops = inputs.unet_topology(res, 4, (C,), (res,), heads, attn_kind="xfmr", ctx=ctx)
    P = inputs.unet_params(1004 + res, ops, dtype, in_ch=4)
    img_o, img_e, mask = inputs.unet_images(1004 + res, res, area, dtype, in_ch=4)
    trace_d, trace_e = [], []
    cache, stats = ounet.unet_pass(bufs, ops, P, f64(img_o), storage=dtype, block=block, trace=trace_d)
    edit, blocks = ounet.unet_pass(bufs, ops, P, f64(img_e), storage=dtype, block=block, cache=cache, stats=stats,
                                   mask=mask, dilate=1, min_sparse_res=16, trace=trace_e)
    net = SigeUNet(res, (C,), (res,), heads, dtype=dtype, block=block, dilate=1, min_sparse_res=16, params=P, in_ch=4,
                   attn_kind="xfmr", ctx=ctx)
    s = dict(dtype=dtype, bufs=bufs, ops=ops, img_o=img_o, img_e=img_e, mask=mask, cache=cache, edit=edit,
             blocks=blocks, net=net, stats=stats, trace_d=trace_d, trace_e=trace_e)
    rep_d, rep_e = teacher_forced(s, inner=True)
    # block lists bit for bit; the transformer blocks really were sparse
    n_tok = {}
    for n, L in net.layers.items():
        if L["sparse"] and n in blocks:        # (a shortcut branch runs on its ResBlock's list)
            bl = L["list"][1]
            assert np.array_equal(bl.indices[:bl.n_host].cpu().numpy(), blocks[n]), n
            if L["op"]["kind"] == "xfmr":
                n_tok[n] = bl.n_host * block * block
                assert 0 < bl.n_host < bl.g.grid_blocks
    assert len(n_tok) == 4
    # which kernels ran (sparse pass): the plan of every convolution, by its sizes
    td = inputs.DTYPES[dtype]
    seen = set()
    for n, L in net.layers.items():
        convs = [L["conv"]] if "conv" in L else [L[p] for p in ("in", "qkv1", "o1", "q2", "o2", "ff1", "ff2", "out")]
        nb = L["list"][1].n_host
        for c in convs:
            key = (c.g.k, c.Cin, c.Cout)
            if key in seen:
                continue
            seen.add(key)
            nbytes = api.sige_conv_workspace_bytes(td, c.g, c.Cin, c.Cout, max(nb, 1))
            print(f"{res}x{res} C={C} {nb} blocks, {c.g.k}x{c.g.k} {c.Cin}->{c.Cout}: "
                  f"{api.sige_conv_plan(td, c.g, c.Cin, c.Cout, max(nb, 1), workspace_bytes=nbytes)!r}")
    print(f"attention: T={res * res}, {heads} heads of {C // heads}, active tokens {sorted(set(n_tok.values()))}")
    rep_d.assert_clean(min_checked=70)
    rep_e.assert_clean(min_checked=70)


@pytest.mark.parametrize("area", [0.01, 0.2])
def test_latent_unet_full_size_whole_step_teacher_forced(area):
    """Benchmark configuration 4 at FULL size and as a whole (the ends of its edit sweep, 1 % and 20 %): latent 64x64x4, channels 320/640/1280/1280, two
    ResBlocks per level each followed by a transformer block (8 heads of 40/80/160, T = 4096/1024/256,
    cross-attention over 77x768 text embeddings, gated-GELU feed-forward) at 64/32/16, bf16, 8x8 blocks, ~1 %
    edit.  Both passes under teacher forcing: every stored tensor of every library call - convolutions, token
    norms, projections, both attentions, feed-forward layers, residual scatters, inside all twelve transformer
    blocks - compared element by element at 1e-2 with the oracle, which computes each layer on the whole map
    (about a minute of CPU time per pass).  Block lists bit for bit."""
    from oracle import unet as ounet
    dtype, res, ch, att, heads, block, ctx = "bf16", 64, (320, 640, 1280, 1280), (64, 32, 16), 8, 8, (77, 768)
    bufs, ops = inputs.unet_topology(res, 4, ch, att, heads, attn_kind="xfmr", ctx=ctx)
    P = inputs.unet_params(1004, ops, dtype, in_ch=4)
    img_o, img_e, mask = inputs.unet_images(1004, res, area, dtype, in_ch=4)
    trace_d, trace_e = [], []
    print("oracle: dense pass on the original latent", flush=True)
    cache, stats = ounet.unet_pass(bufs, ops, P, f64(img_o), storage=dtype, block=block, trace=trace_d)
    print("oracle: edit pass", flush=True)
    edit, blocks = ounet.unet_pass(bufs, ops, P, f64(img_e), storage=dtype, block=block, cache=cache, stats=stats,
                                   mask=mask, dilate=1, min_sparse_res=16, trace=trace_e)
    net = SigeUNet(res, ch, att, heads, dtype=dtype, block=block, dilate=1, min_sparse_res=16, params=P, in_ch=4,
                   attn_kind="xfmr", ctx=ctx)
    s = dict(dtype=dtype, bufs=bufs, ops=ops, img_o=img_o, img_e=img_e, mask=mask, cache=cache, edit=edit,
             blocks=blocks, net=net, stats=stats, trace_d=trace_d, trace_e=trace_e)
    print("GPU: both passes under teacher forcing", flush=True)
    rep_d, rep_e = teacher_forced(s, inner=True)
    n_x = 0
    for n, L in net.layers.items():
        if L["sparse"] and n in blocks:
            bl = L["list"][1]
            assert np.array_equal(bl.indices[:bl.n_host].cpu().numpy(), blocks[n]), n
            if L["op"]["kind"] == "xfmr":
                assert 0 < bl.n_host <= bl.g.grid_blocks
                n_x += 1
    assert n_x == 12
    print(f"worst error / bound: pre-computation pass {rep_d.worst:.3f}, sparse step {rep_e.worst:.3f}; "
          f"{rep_d.n_checked} + {rep_e.n_checked} tensors compared")
    rep_d.assert_clean(min_checked=220)
    rep_e.assert_clean(min_checked=220)
