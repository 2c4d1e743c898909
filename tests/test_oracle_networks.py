"""Pins for the multi-layer oracles (oracle/unet.py: unet_pass and its transformer block;
oracle/spade.py: spade_pass), none of which has a closed form (Sec. 3, Fig. "method"; Sec. 3.2
"Pre-computing normalization parameters", "Extension to attention layers"; Sec. 4.1
"Implementation details").

What fixes them, on tiny networks and with no storage rounding (storage="f64"):
 (i)   the pass on the original input equals an independent network written HERE in the usual
       way - NCHW torch tensors, a stack of skips, torch.cat, F.conv2d / F.group_norm / F.silu /
       F.layer_norm / F.gelu / F.softmax / F.instance_norm / F.interpolate in float64 - that never
       looks at the op list the oracle interprets;
 (ii)  an edit pass with the original input and an empty mask returns the cache bit for bit;
 (iii) an edit pass with every block active equals that independent network run on the EDITED
       input with the normalisation statistics of the ORIGINAL input (the cached ones);
 (iv)  the active blocks of every layer equal a set-based definition written here (pooling
       factor, dilation, tile footprint; the 1x1 shortcut on its ResBlock's list; up-sampled inputs);
       outside them a sparse layer's output is the cache bit for bit, and the first layer - whose
       mask is the true support of the change - equals the dense result everywhere;
 (v)   planted mistakes in the op list (a swapped skip, a dropped residual, a shortcut left out,
       fresh instead of cached statistics) make (i) or (iii) fail.
"""
import copy
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2211_02048_amd import inputs

GROUPS, EPS = 4, 1e-5


def nchw(a):      # numpy [H, W, C] -> torch [1, C, H, W] float64
    return torch.from_numpy(np.ascontiguousarray(a)).double().permute(2, 0, 1)[None].contiguous()


def nhwc(t):      # torch [1, C, H, W] -> numpy [H, W, C]
    return t[0].permute(1, 2, 0).contiguous().numpy()


def p64(P, name):
    return P[name].double()


# ------------------------------------------------------------------------------------------------
# An independent UNet, written the way such a network is usually written.
# ------------------------------------------------------------------------------------------------
class RefUNet:
    """conv-in; per level two ResBlocks (+ attention where listed), then a stride-2 convolution;
    two ResBlocks in the middle; per level on the way up two ResBlocks on cat(h, skip) (+ attention),
    then nearest x2 and a convolution; GroupNorm + SiLU + conv-out.  `stats` None: group
    statistics computed on the fly and recorded; otherwise the recorded ones are used."""

    def __init__(self, P, res, channels, attn_res, heads, kind, stats=None):
        self.P, self.res, self.ch, self.attn_res, self.heads, self.kind = P, res, channels, attn_res, heads, kind
        self.replay = stats is not None
        self.stats = {} if stats is None else stats
        self.seen = {}

    def conv(self, name, x, stride=1):
        w = p64(self.P, name + ".w")
        return F.conv2d(x, w, p64(self.P, name + ".b"), stride=stride, padding=w.shape[-1] // 2)

    def gn(self, name, x):
        g, b = p64(self.P, name + ".gamma"), p64(self.P, name + ".beta")
        if not self.replay:
            xs = x.reshape(1, GROUPS, -1)
            self.stats[name] = (xs.mean(-1), xs.var(-1, unbiased=False))
            return F.group_norm(x, GROUPS, g, b, EPS)
        mean, var = self.stats[name]
        C = x.shape[1]
        mean = mean.repeat_interleave(C // GROUPS, 1)[:, :, None, None]
        var = var.repeat_interleave(C // GROUPS, 1)[:, :, None, None]
        return (x - mean) / torch.sqrt(var + EPS) * g[None, :, None, None] + b[None, :, None, None]

    def resblock(self, name, x, cout):
        h = self.conv(name + ".conv1", F.silu(self.gn(name + ".conv1", x)))
        h = self.conv(name + ".conv2", F.silu(self.gn(name + ".conv2", h)))
        return h + (x if x.shape[1] == cout else self.conv(name + ".short", x))

    def mha(self, q, k, v):   # [T, C] each (k, v may have another T) -> [T, C]
        d = q.shape[1] // self.heads
        qh, kh, vh = (t.reshape(t.shape[0], self.heads, d).transpose(0, 1) for t in (q, k, v))
        p = F.softmax(qh @ kh.transpose(1, 2) / math.sqrt(d), dim=-1)
        return (p @ vh).transpose(0, 1).reshape(q.shape[0], -1)

    def lin(self, name, t):   # token rows [T, Cin] -> [T, Cout]
        return F.linear(t, p64(self.P, name + ".w")[:, :, 0, 0], p64(self.P, name + ".b"))

    def attn(self, name, x):
        _, C, H, W = x.shape
        rows = lambda t: t[0].reshape(t.shape[1], -1).T
        if self.kind == "attn":
            z = rows(self.gn(name, x))
            a = self.mha(self.lin(name + ".q", z), self.lin(name + ".k", z), self.lin(name + ".v", z))
            y = self.lin(name + ".o", a)
            return x + y.T.reshape(1, C, H, W)
        ln = lambda part, t: F.layer_norm(t, (C,), p64(self.P, f"{name}.{part}.gamma"), p64(self.P, f"{name}.{part}.beta"), 1e-5)
        h = self.lin(name + ".in", rows(self.gn(name, x)))
        t = ln("ln1", h)
        h = h + self.lin(name + ".o1", self.mha(self.lin(name + ".q1", t), self.lin(name + ".k1", t), self.lin(name + ".v1", t)))
        ctx = p64(self.P, "ctx")
        t = ln("ln2", h)
        h = h + self.lin(name + ".o2", self.mha(self.lin(name + ".q2", t), self.lin(name + ".k2", ctx), self.lin(name + ".v2", ctx)))
        u = self.lin(name + ".ff1", ln("ln3", h))
        h = h + self.lin(name + ".ff2", u[:, :4 * C] * F.gelu(u[:, 4 * C:]))
        return x + self.lin(name + ".out", h).T.reshape(1, C, H, W)

    def __call__(self, image):
        ch, nl = self.ch, len(self.ch)
        h = self.conv("conv_in", image)
        self.seen["in"] = h
        skips = []
        for l in range(nl):
            for i in range(2):
                h = self.resblock(f"down{l}.{i}", h, ch[l])
                if self.res >> l in self.attn_res:
                    h = self.attn(f"down{l}.{i}.attn", h)
                skips.append(h)
            if l + 1 < nl:
                h = self.conv(f"down{l}.downsample", h, stride=2)
        h = self.resblock("mid.0", h, ch[-1])
        h = self.resblock("mid.1", h, ch[-1])
        for l in reversed(range(nl)):
            for j in range(2):
                h = self.resblock(f"up{l}.{j}", torch.cat([h, skips.pop()], 1), ch[l])
                if self.res >> l in self.attn_res:
                    h = self.attn(f"up{l}.{j}.attn", h)
            if l > 0:
                h = self.conv(f"up{l}.upsample", F.interpolate(h, scale_factor=2, mode="nearest"))
        self.seen["last"] = h
        return self.conv("conv_out", F.silu(self.gn("conv_out", h)))


UNETS = {
    "attn": dict(res=16, channels=(8, 8, 16), attn_res=(4,), heads=2, kind="attn", ctx=(5, 12), block=4, min_sparse=8),
    "xfmr": dict(res=16, channels=(8, 16), attn_res=(16, 8), heads=2, kind="xfmr", ctx=(5, 12), block=4, min_sparse=8),
}


def make_unet(cfg, seed=11):
    bufs, ops = inputs.unet_topology(cfg["res"], 3, cfg["channels"], cfg["attn_res"], cfg["heads"], in_pad=4,
                                     attn_kind=cfg["kind"], ctx=cfg["ctx"])
    P = inputs.unet_params(seed, ops, "f32", GROUPS, in_ch=3, in_pad=4)
    img_o, img_e, mask = inputs.unet_images(seed, cfg["res"], 0.04, "f32", in_ch=3, in_pad=4, n_blobs=1)
    return bufs, ops, P, img_o.double().numpy(), img_e.double().numpy(), mask


def oracle_dense(bufs, ops, P, img, cfg):
    from oracle import unet as ounet
    return ounet.unet_pass(bufs, ops, P, img, storage="f64", groups=GROUPS, eps=EPS, block=cfg["block"])


def oracle_edit(bufs, ops, P, img, cfg, cache, stats, mask, dilate=1):
    from oracle import unet as ounet
    return ounet.unet_pass(bufs, ops, P, img, storage="f64", groups=GROUPS, eps=EPS, block=cfg["block"], cache=cache,
                           stats=stats, mask=mask, dilate=dilate, min_sparse_res=cfg["min_sparse"])


def ref_unet(P, cfg, img, stats=None):
    net = RefUNet(P, cfg["res"], cfg["channels"], cfg["attn_res"], cfg["heads"], cfg["kind"], stats)
    return nhwc(net(nchw(img))), net


@pytest.mark.parametrize("kind", ["attn", "xfmr"])
def test_unet_dense_pass_equals_an_independent_network(oracle, kind):
    cfg = UNETS[kind]
    bufs, ops, P, img_o, img_e, mask = make_unet(cfg)
    B, stats = oracle_dense(bufs, ops, P, img_o, cfg)
    want, net = ref_unet(P, cfg, img_o)
    np.testing.assert_allclose(B["out"], want, rtol=0, atol=1e-10)
    np.testing.assert_allclose(B["in"], nhwc(net.seen["in"]), rtol=0, atol=1e-12)
    np.testing.assert_allclose(B["up0.out"], nhwc(net.seen["last"]), rtol=0, atol=1e-10)
    assert np.abs(want).max() > 0.05 and np.abs(want[:, :, 3]).max() == 0.0    # three real channels, one padding
    # the recorded group statistics agree with the oracle's folded scale / shift
    for name, (scale, shift) in stats.items():
        mean, var = net.stats[name]
        g, b = p64(P, name + ".gamma").numpy(), p64(P, name + ".beta").numpy()
        C = len(g)
        m, v = np.repeat(mean[0].numpy(), C // GROUPS), np.repeat(var[0].numpy(), C // GROUPS)
        np.testing.assert_allclose(scale, g / np.sqrt(v + EPS), rtol=1e-10)
        np.testing.assert_allclose(shift, b - m * g / np.sqrt(v + EPS), rtol=0, atol=1e-10)


@pytest.mark.parametrize("kind", ["attn", "xfmr"])
def test_unet_zero_edit_returns_the_cache_bitwise(oracle, kind):
    cfg = UNETS[kind]
    bufs, ops, P, img_o, img_e, mask = make_unet(cfg)
    cache, stats = oracle_dense(bufs, ops, P, img_o, cfg)
    B, blocks = oracle_edit(bufs, ops, P, img_o, cfg, cache, stats, np.zeros_like(mask))
    for n in cache:
        assert np.array_equal(B[n], cache[n]), n
    assert all(len(b) == 0 for n, b in blocks.items() if _is_sparse(n, ops, bufs, cfg))


def _is_sparse(name, ops, bufs, cfg):
    op = next(o for o in ops if o["name"] == name)
    return bufs[op["x"][0]][0] >= cfg["min_sparse"]


@pytest.mark.parametrize("kind", ["attn", "xfmr"])
def test_unet_all_blocks_active_equals_dense_with_cached_statistics(oracle, kind):
    cfg = UNETS[kind]
    bufs, ops, P, img_o, img_e, mask = make_unet(cfg)
    cache, stats = oracle_dense(bufs, ops, P, img_o, cfg)
    B, blocks = oracle_edit(bufs, ops, P, img_e, cfg, cache, stats, np.ones_like(mask))
    _, net_o = ref_unet(P, cfg, img_o)                       # records the original's statistics
    want, _ = ref_unet(P, cfg, img_e, stats=net_o.stats)     # edited input, cached statistics
    np.testing.assert_allclose(B["out"], want, rtol=0, atol=1e-10)
    # with fresh statistics the result differs: the statistics really are the cached ones
    fresh, _ = ref_unet(P, cfg, img_e)
    assert np.abs(fresh - want).max() > 1e-6
    for n, b in blocks.items():
        op = next(o for o in ops if o["name"] == n)
        r = bufs[op["y"][0]][0] if op.get("y") else None
        if r is not None:
            assert len(b) == (-(-r // min(cfg["block"], r))) ** 2, n


def brute_blocks(mask, Hin, k, stride, pad, b, dilate):
    """Active output blocks by sets: the image mask pooled to Hin x Hin (any marked pixel under a
    cell), grown by `dilate` in the Chebyshev metric, then a block is active iff one of its output
    pixels reads a marked cell."""
    f = mask.shape[0] // Hin
    cells = {(y // f, x // f) for y, x in zip(*np.nonzero(mask))}
    grown = {(y + dy, x + dx) for (y, x) in cells for dy in range(-dilate, dilate + 1) for dx in range(-dilate, dilate + 1)
             if 0 <= y + dy < Hin and 0 <= x + dx < Hin}
    Hout = (Hin + 2 * pad - k) // stride + 1
    out = []
    for by in range(0, Hout, b):
        for bx in range(0, Hout, b):
            reads = {(y * stride + ky - pad, x * stride + kx - pad) for y in range(by, min(by + b, Hout))
                     for x in range(bx, min(bx + b, Hout)) for ky in range(k) for kx in range(k)}
            # the footprint rule takes the whole tile of the block, also where the block is cut by the border
            reads |= {(y * stride + ky - pad, x * stride + kx - pad) for y in range(by, by + b)
                      for x in range(bx, bx + b) for ky in range(k) for kx in range(k)}
            if reads & grown:
                out.append((by, bx))
    return out


@pytest.mark.parametrize("kind", ["attn", "xfmr"])
def test_unet_sparse_pass_blocks_and_selection(oracle, kind):
    cfg = UNETS[kind]
    bufs, ops, P, img_o, img_e, mask = make_unet(cfg)
    assert 0 < mask.sum() < 0.2 * mask.size
    cache, stats = oracle_dense(bufs, ops, P, img_o, cfg)
    B, blocks = oracle_edit(bufs, ops, P, img_e, cfg, cache, stats, mask, dilate=1)
    n_sparse = n_partial = 0
    for op in ops:
        n = op["name"]
        if n not in blocks:
            continue
        r_in = bufs[op["x"][0]][0]
        if op["kind"] == "conv":
            Hin = r_in * (2 if op["up"] else 1)
            k, s = (3, 1) if op["k"] == 1 else (op["k"], op["stride"])   # a shortcut runs on its ResBlock's 3x3 list
            Hout = (Hin + 2 * (op["k"] // 2) - op["k"]) // op["stride"] + 1
        else:
            Hin, k, s, Hout = r_in, 3, 1, r_in                           # the blocks of the 3x3 convolution before it
        b = min(cfg["block"], Hout)
        if r_in >= cfg["min_sparse"]:
            want = brute_blocks(mask, Hin, k, s, 1, b, 1)
            n_sparse += 1
        else:
            want = [(y, x) for y in range(0, Hout, b) for x in range(0, Hout, b)]
        assert [tuple(t) for t in blocks[n]] == want, n
        if op["kind"] == "xfmr" and r_in >= cfg["min_sparse"]:
            # the block's internal caches (residual stages, keys | values): untouched outside the active tokens
            keep = np.ones((Hout, Hout), bool)
            for y0, x0 in want:
                keep[y0:y0 + b, x0:x0 + b] = False
            for part in ("h0", "h1", "h2", "h3", "kv"):
                assert np.array_equal(B[f"{n}.{part}"][keep], cache[f"{n}.{part}"][keep]), (n, part)
                assert not np.array_equal(B[f"{n}.{part}"][~keep], cache[f"{n}.{part}"][~keep]), (n, part)
        if op["kind"] in ("conv", "xfmr") and op["y"] is not None and r_in >= cfg["min_sparse"]:
            keep = np.ones((Hout, Hout), bool)
            for y0, x0 in want:
                keep[y0:y0 + b, x0:x0 + b] = False
            v = lambda D: D[op["y"][0]][:, :, op["y"][1]:op["y"][1] + op["y"][2]]
            assert np.array_equal(v(B)[keep], v(cache)[keep]), n
            n_partial += bool(keep.any() and not keep.all())
    assert n_sparse >= 8 and n_partial >= 5
    # the first layer sees the true support of the change: sparse == dense everywhere (Sec. 3.1)
    _, net_e = ref_unet(P, cfg, img_e)
    np.testing.assert_allclose(B["in"], nhwc(net_e.seen["in"]), rtol=0, atol=1e-12)
    assert not np.array_equal(B["out"], cache["out"])


@pytest.mark.parametrize("kind,mutation", [("attn", "swap_skips"), ("attn", "drop_residual"), ("attn", "drop_shortcut"),
                                           ("xfmr", "drop_residual"), ("attn", "fresh_stats")])
def test_unet_planted_mistakes_are_caught(oracle, kind, mutation):
    cfg = UNETS[kind]
    bufs, ops, P, img_o, img_e, mask = make_unet(cfg)
    ops = copy.deepcopy(ops)
    want, net_o = ref_unet(P, cfg, img_o)
    if mutation == "swap_skips":        # the two up ResBlocks of level 0 read each other's concat buffer
        a = next(o for o in ops if o["name"] == "up0.0.conv1")
        b = next(o for o in ops if o["name"] == "up0.1.conv1")
        assert bufs[a["x"][0]] == bufs[b["x"][0]]
        # the skip halves of the two buffers hold down0.1 and down0.0: exchange which one each consumer reads
        for o in ops:
            if o["kind"] == "conv" and o["y"] is not None and o["y"][0] in (a["x"][0], b["x"][0]) and o["y"][1] > 0:
                o["y"] = (b["x"][0] if o["y"][0] == a["x"][0] else a["x"][0],) + tuple(o["y"][1:])
    elif mutation == "drop_residual":
        o = next(o for o in ops if o["kind"] == "conv" and o["residual"] is not None)
        o["residual"] = None
    elif mutation == "drop_shortcut":
        o = next(o for o in ops if o["kind"] == "conv" and o["shortcut"] is not None)
        o["shortcut"] = None
    if mutation == "fresh_stats":
        cache, stats = oracle_dense(bufs, ops, P, img_o, cfg)
        _, stats_e = oracle_dense(bufs, ops, P, img_e, cfg)          # the wrong ones: the edited input's own
        B, _ = oracle_edit(bufs, ops, P, img_e, cfg, cache, stats_e, np.ones_like(mask))
        want_e, _ = ref_unet(P, cfg, img_e, stats=net_o.stats)
        assert np.abs(B["out"] - want_e).max() > 1e-6
        return
    B, _ = oracle_dense(bufs, ops, P, img_o, cfg)
    assert np.abs(B["out"] - want).max() > 1e-6, mutation


# ------------------------------------------------------------------------------------------------
# An independent SPADE-style generator.
# ------------------------------------------------------------------------------------------------
SP = dict(out_hw=(32, 64), start_hw=(1, 2), channels=(8, 8, 8, 8, 4, 4, 4), n_labels=3, label_pad=4, hidden=4,
          stats_cached_above=(2, 4))
SP_BLOCK, SP_MIN = 4, (1, 2)
SP_SIZES = [(1 << i, 2 << i) for i in range(6)]


class RefSpade:
    def __init__(self, P, labels_onehot, stats=None, cached_above=2):
        self.P, self.seg, self.cached_above = P, labels_onehot, cached_above
        self.replay = stats is not None
        self.stats = {} if stats is None else stats

    def conv(self, name, x):
        w = p64(self.P, name + ".w")
        return F.conv2d(x, w, p64(self.P, name + ".b"), padding=w.shape[-1] // 2)

    def spade(self, name, x):
        h, w = x.shape[2:]
        seg = nchw(self.seg[(h, w)])
        gb = self.conv(name + ".gb", F.relu(self.conv(name + ".shared", seg)))
        C = x.shape[1]
        if self.replay and h > self.cached_above:
            mean, var = self.stats[name]
            n = (x - mean) / torch.sqrt(var + 1e-5)
        else:
            self.stats[name] = (x.mean((2, 3), keepdim=True), x.var((2, 3), unbiased=False, keepdim=True))
            n = F.instance_norm(x, eps=1e-5)
        return n * (1 + gb[:, :C]) + gb[:, C:]

    def block(self, name, x, cout):
        cin = x.shape[1]
        h = self.conv(name + ".conv0", F.leaky_relu(self.spade(name + ".conv0", x), 0.2))
        h = self.conv(name + ".conv1", F.leaky_relu(self.spade(name + ".conv1", h), 0.2))
        return h + (x if cin == cout else self.conv(name + ".short", self.spade(name + ".short", x)))

    def __call__(self):
        x = nchw(p64(self.P, "z").numpy())
        ups = (0, 1, 0, 1, 1, 1, 1)
        for i, cout in enumerate(SP["channels"]):
            if ups[i]:
                x = F.interpolate(x, scale_factor=2, mode="nearest")
            x = self.block(f"block{i}", x, cout)
        return self.conv("conv_img", F.leaky_relu(x, 0.2))


def make_spade(seed=21):
    bufs, ops = inputs.spade_topology(**SP)
    P = inputs.spade_params(seed, bufs, ops, "f32", n_labels=SP["n_labels"])
    lab0 = inputs.label_map(seed, 32, 64, SP["n_labels"], 6)
    lab1 = inputs.relabel(seed + 1, lab0, 0.03, SP["n_labels"], n_blobs=1)
    seg = lambda lab: {k: v.double().numpy() for k, v in
                       inputs.one_hot_pyramid(lab, SP_SIZES, SP["n_labels"], SP["label_pad"], "f32").items()}
    return bufs, ops, P, lab0, lab1, seg(lab0), seg(lab1)


def spade_oracle(bufs, ops, P, seg, **kw):
    from oracle import spade as osp
    return osp.spade_pass(bufs, ops, P, seg, storage="f64", block=SP_BLOCK, min_sparse=SP_MIN, **kw)


def test_spade_dense_pass_equals_an_independent_generator(oracle):
    bufs, ops, P, lab0, lab1, seg0, seg1 = make_spade()
    B, stats = spade_oracle(bufs, ops, P, seg0)
    want = nhwc(RefSpade(P, seg0)())
    np.testing.assert_allclose(B["out"], want, rtol=0, atol=1e-10)
    assert np.abs(want[:, :, :3]).max() > 0.05 and np.abs(want[:, :, 3:]).max() == 0.0


def test_spade_zero_edit_all_active_and_blocks(oracle):
    bufs, ops, P, lab0, lab1, seg0, seg1 = make_spade()
    cache, stats = spade_oracle(bufs, ops, P, seg0)
    mask = (lab0 != lab1).astype(np.uint8)
    assert 0 < mask.sum() < 0.2 * mask.size
    # (ii) nothing changed, empty mask: the cache, bit for bit
    B, _ = spade_oracle(bufs, ops, P, seg0, cache=cache, stats=stats, mask=np.zeros_like(mask), dilate=1)
    for n in cache:
        assert np.array_equal(B[n], cache[n]), n
    # (iii) every block active on the edited labels: the independent generator with the cached
    # statistics above the caching resolution and fresh ones at or below it
    ref0 = RefSpade(P, seg0)
    ref0()
    want = nhwc(RefSpade(P, seg1, stats=ref0.stats)())
    B, _ = spade_oracle(bufs, ops, P, seg1, cache=cache, stats=stats, mask=np.ones_like(mask), dilate=1)
    np.testing.assert_allclose(B["out"], want, rtol=0, atol=1e-10)
    fresh = nhwc(RefSpade(P, seg1)())
    assert np.abs(fresh - want).max() > 1e-7
    # (iv) the real edit: block lists by sets (one mask, pooled per resolution, dilation 1, 3x3 tiles),
    # outputs outside the blocks untouched
    B, blocks = spade_oracle(bufs, ops, P, seg1, cache=cache, stats=stats, mask=mask, dilate=1)
    n_sparse = 0
    for op in ops:
        h, w = op["hw"]
        b = min(SP_BLOCK, h)
        if h <= SP_MIN[0]:
            want_b = [(y, x) for y in range(0, h, b) for x in range(0, w, b)]
        else:
            f = mask.shape[0] // h
            cells = {(y // f, x // f) for y, x in zip(*np.nonzero(mask))}
            grown = {(y + dy, x + dx) for (y, x) in cells for dy in (-1, 0, 1) for dx in (-1, 0, 1)}
            want_b = [(by, bx) for by in range(0, h, b) for bx in range(0, w, b)
                      if {(y, x) for y in range(by - 1, by + b + 1) for x in range(bx - 1, bx + b + 1)
                          if 0 <= y < h and 0 <= x < w} & grown]
            n_sparse += 1
            if op.get("y") is not None:
                keep = np.ones((h, w), bool)
                for y0, x0 in want_b:
                    keep[y0:y0 + b, x0:x0 + b] = False
                assert np.array_equal(B[op["y"]][keep], cache[op["y"]][keep]), op["name"]
        assert [tuple(t) for t in blocks[op["name"]]] == want_b, op["name"]
    assert n_sparse >= 30
    assert not np.array_equal(B["out"], cache["out"])


@pytest.mark.parametrize("mutation", ["drop_residual", "drop_shortcut", "wrong_modulation"])
def test_spade_planted_mistakes_are_caught(oracle, mutation):
    bufs, ops, P, lab0, lab1, seg0, seg1 = make_spade()
    ops = copy.deepcopy(ops)
    want = nhwc(RefSpade(P, seg0)())
    if mutation == "drop_residual":
        next(o for o in ops if o.get("residual") is not None)["residual"] = None
    elif mutation == "drop_shortcut":
        next(o for o in ops if o.get("shortcut") is not None)["shortcut"] = None
    else:   # a modulated layer reads another layer's gamma | beta
        mods = [o for o in ops if o.get("spade") and bufs[o["spade"]["mod"]] == bufs[ops[2]["spade"]["mod"]]]
        mods[0]["spade"], mods[1]["spade"] = mods[1]["spade"], mods[0]["spade"]
    B, _ = spade_oracle(bufs, ops, P, seg0)
    assert np.abs(B["out"] - want).max() > 1e-6, mutation
