"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

Only random draws, shapes and masks live here: none of the method's arithmetic
(no normalisation statistics, no convolution, no block reduction).  The inputs
stand in for the paper's edit benchmarks (localised strokes, pasted objects and
circular inpainting masks; Sec. 4.1 "Datasets", App. B), which cannot be shipped:
only their shapes, edit-area statistics and structure are borrowed.

Every tensor is a CPU torch tensor, batch 1, NHWC ([H, W, C]), already in its
storage dtype, drawn from numpy's PCG64 with an explicit seed.
"""
from __future__ import annotations

import math

import numpy as np
import torch

DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _t(a: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dtype).contiguous()


def rect_mask(rng, H: int, W: int, area_frac: float) -> np.ndarray:
    """One axis-aligned rectangle of about area_frac of the image."""
    lo, hi = max(1, H // 8), max(2, (3 * H) // 8)
    h = int(rng.integers(lo, hi + 1))
    w = max(1, min(W, int(round(area_frac * H * W / h))))
    y0 = int(rng.integers(0, H - h + 1))
    x0 = int(rng.integers(0, W - w + 1))
    m = np.zeros((H, W), dtype=np.uint8)
    m[y0:y0 + h, x0:x0 + w] = 1
    return m


def blob_mask(rng, H: int, W: int, target_px: int, n_blobs: int = 3, axes=(5.0, 12.0),
              tol: float = 0.05) -> np.ndarray:
    """Union of n_blobs filled ellipses (random centres, semi-axes, rotation), all
    rescaled by one factor found by bisection so the union covers target_px pixels
    within +-tol (relative)."""
    cy = rng.uniform(0, H, n_blobs)
    cx = rng.uniform(0, W, n_blobs)
    a = rng.uniform(axes[0], axes[1], n_blobs)
    b = rng.uniform(axes[0], axes[1], n_blobs)
    th = rng.uniform(0, math.pi, n_blobs)
    yy, xx = np.mgrid[0:H, 0:W].astype(np.float64)

    def draw(s: float) -> np.ndarray:
        m = np.zeros((H, W), dtype=bool)
        for i in range(n_blobs):
            dy, dx = yy - cy[i], xx - cx[i]
            u = (dx * math.cos(th[i]) + dy * math.sin(th[i])) / (a[i] * s)
            v = (-dx * math.sin(th[i]) + dy * math.cos(th[i])) / (b[i] * s)
            m |= (u * u + v * v) <= 1.0
        return m

    lo, hi = 0.01, 1.0
    while draw(hi).sum() < target_px and hi < 1e3:
        hi *= 2.0
    m = draw(hi)
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        m = draw(mid)
        n = int(m.sum())
        if abs(n - target_px) <= tol * target_px:
            break
        if n < target_px:
            lo = mid
        else:
            hi = mid
    return m.astype(np.uint8)


def edited_pair(rng, H, W, C, mask: np.ndarray, sigma_edit: float, dtype: torch.dtype):
    """A_orig ~ N(0,1); A_edit equals A_orig bit for bit outside the mask and is
    A_orig + N(0, sigma_edit^2) on every channel inside it."""
    a_o = rng.standard_normal((H, W, C), dtype=np.float32)
    noise = rng.standard_normal((H, W, C), dtype=np.float32) * np.float32(sigma_edit)
    a_o_t = _t(a_o, dtype)
    a_e_t = _t(a_o + noise, dtype)
    m = torch.from_numpy(mask.astype(bool))[:, :, None]
    a_e_t = torch.where(m, a_e_t, a_o_t).contiguous()
    return a_o_t, a_e_t


def conv_params(rng, Cout: int, Cin: int, k: int, dtype: torch.dtype, bias_sigma: float = 0.1):
    """W ~ N(0, 1/fan_in) in OIHW, bias ~ N(0, bias_sigma^2) in fp32."""
    w = rng.standard_normal((Cout, Cin, k, k), dtype=np.float32) / np.float32(math.sqrt(Cin * k * k))
    b = rng.standard_normal((Cout,), dtype=np.float32) * np.float32(bias_sigma)
    return _t(w, dtype), torch.from_numpy(b)


def config1(seed: int = 1001, H: int = 64, W: int = 64, C: int = 64, area_frac: float = 0.05):
    """Single 3x3 conv, stride 1, pad 1, fp32, 64x64x64; one rectangle edit of ~5 %
    area with N(0,1) noise; output block 6x6 (8x8 input tiles); tau = 1e-6."""
    rng = _rng(seed)
    mask = rect_mask(rng, H, W, area_frac)
    a_o, a_e = edited_pair(rng, H, W, C, mask, 1.0, torch.float32)
    w, b = conv_params(rng, C, C, 3, torch.float32)
    return dict(name="config1", dtype="f32", H=H, W=W, Cin=C, Cout=C, k=3, stride=1, pad=1,
                block=6, tau=1e-6, dilate=0, mask=mask, a_orig=a_o, a_edit=a_e, w=w, bias=b)


def config2(seed: int = 1002, H: int = 256, W: int = 256, C: int = 128, Cs: int = 256,
            area_frac: float = 0.01, dtype: str = "f16", block: int = 16, n_blobs: int = 3,
            axes=(5.0, 12.0)):
    """Fused GroupNorm(32 groups, cached statistics) + SiLU + 3x3 conv C->C, plus a
    1x1 shortcut conv C->Cs on the same mask; edit = union of elliptical blobs of
    about area_frac of the image, perturbation N(0, 0.5) (variance)."""
    rng = _rng(seed)
    td = DTYPES[dtype]
    mask = blob_mask(rng, H, W, int(round(area_frac * H * W)), n_blobs, axes)
    a_o, a_e = edited_pair(rng, H, W, C, mask, math.sqrt(0.5), td)
    gamma = torch.from_numpy((1.0 + math.sqrt(0.1) * rng.standard_normal(C)).astype(np.float32))
    beta = torch.from_numpy((math.sqrt(0.1) * rng.standard_normal(C)).astype(np.float32))
    w, b = conv_params(rng, C, C, 3, td)
    ws, bs = conv_params(rng, Cs, C, 1, td)
    return dict(name="config2", dtype=dtype, H=H, W=W, Cin=C, Cout=C, Cs=Cs, k=3, stride=1, pad=1,
                block=block, tau=0.0, dilate=0, groups=32, eps=1e-5, mask=mask, a_orig=a_o,
                a_edit=a_e, gamma=gamma, beta=beta, w=w, bias=b, w_s=ws, bias_s=bs)


def attention_case(seed: int, T: int, heads: int, d: int, n_q: int, dtype: str = "bf16"):
    """q [n_q, heads, d], k and v [T, heads, d], all N(0,1) in the storage dtype."""
    rng = _rng(seed)
    td = DTYPES[dtype]
    q = _t(rng.standard_normal((n_q, heads, d), dtype=np.float32), td)
    k = _t(rng.standard_normal((T, heads, d), dtype=np.float32), td)
    v = _t(rng.standard_normal((T, heads, d), dtype=np.float32), td)
    return dict(q=q, k=k, v=v, T=T, heads=heads, d=d, n_q=n_q, dtype=dtype,
                scale=1.0 / math.sqrt(d))


def token_mask(seed: int, Ht: int, Wt: int, area_frac: float, n_blobs: int = 3) -> np.ndarray:
    """Blob mask on a token grid (latent resolution) covering about area_frac."""
    rng = _rng(seed)
    s = min(Ht, Wt) / 64.0
    return blob_mask(rng, Ht, Wt, max(1, int(round(area_frac * Ht * Wt))), n_blobs,
                     (2.0 * s + 0.5, 6.0 * s + 0.5), tol=0.15)


# ----------------------------------------------------------------------------------------
# Synthetic DDPM-style UNet denoiser (benchmark configuration 3).  The topology is plain data: a list
# of operations over named buffers, consumed by the HIP harness and, separately, by the CPU
# oracle.  Views are (buffer, first channel, channels); buffers are NHWC [res, res, Ctot].
# ----------------------------------------------------------------------------------------

def unet_topology(res: int = 256, in_ch: int = 3, channels=(128, 128, 256, 256, 512, 512),
                  attn_res=(16,), heads: int = 4, in_pad: int = 16, attn_kind: str = "attn", ctx=(77, 768)):
    """Returns (buffers, ops).  conv-in; per level two ResBlocks (GN+SiLU+3x3 twice, 1x1 shortcut
    iff the channel count changes) and a stride-2 3x3 conv; two ResBlocks in the middle; on the way
    up per level two ResBlocks on concat(h, skip) and nearest-x2 + 3x3 conv; self-attention after
    every ResBlock at the listed resolutions; GN+SiLU+3x3 conv-out.  Skips are the outputs of the
    down-path ResBlocks, consumed in reverse order.  attn_kind "attn": a plain self-attention block
    (GN, q/k/v, attention, projection, residual); "xfmr": a latent-diffusion style transformer block
    (GN + 1x1 in; layer norm + self-attention; layer norm + cross-attention over ctx = (tokens, width)
    text embeddings; layer norm + gated-GELU feed-forward; 1x1 out + residual)."""
    bufs, ops = {}, []
    nl = len(channels)
    R = [res >> i for i in range(nl)]

    def buf(name, r, c):
        bufs[name] = (r, r, c)
        return name

    def conv(name, x, y, lvl_in, k=3, stride=1, up=0, gn=True, act=True, residual=None, shortcut=None,
             scatter=True):
        ops.append(dict(kind="conv", name=name, x=x, y=y, level=lvl_in, k=k, stride=stride, up=up, gn=gn,
                        act=act, residual=residual, shortcut=shortcut, scatter=scatter))

    def resblock(name, x, y, lvl):
        cin, cout = x[2], y[2]
        h1 = (buf(name + ".h1", R[lvl], cout), 0, cout)
        conv(name + ".conv1", x, h1, lvl)
        if cin != cout:
            conv(name + ".short", x, None, lvl, k=1, gn=False, act=False, scatter=False)
            conv(name + ".conv2", h1, y, lvl, shortcut=name + ".short")
        else:
            conv(name + ".conv2", h1, y, lvl, residual=x)

    def attn(name, x, y, lvl):
        c = x[2]
        op = dict(kind=attn_kind, name=name, x=x, y=y, level=lvl, heads=heads, C=c)
        if attn_kind == "xfmr":
            op.update(n_ctx=ctx[0], d_ctx=ctx[1])
        ops.append(op)

    img = (buf("image", res, in_pad), 0, in_pad)   # the 3 image channels, zero padded to in_pad
    h = (buf("in", res, channels[0]), 0, channels[0])
    conv("conv_in", img, h, 0, gn=False, act=False)
    skips = []
    # each down ResBlock writes straight into the first... second half of the concat buffer that the
    # matching up ResBlock reads (its own slot), so the concat is never materialised
    for l in range(nl):
        c = channels[l]
        for i in range(2):
            # the up ResBlock that consumes this skip reads concat(h_up, skip): h_up has the channel
            # count of the tensor arriving there (see the up path below)
            slot = f"cat{l}.{i}"
            skips.append((l, i, slot))
    # channel count of the tensor entering each up ResBlock
    up_in = {}
    hc = channels[-1]
    for l in reversed(range(nl)):
        for j in range(2):
            i = 1 - j                       # skips are consumed in reverse order
            up_in[(l, i)] = hc
            hc = channels[l]
        # the up-conv keeps the channel count
    for l in range(nl):
        c = channels[l]
        for i in range(2):
            slot = f"cat{l}.{i}"
            ctot = up_in[(l, i)] + c
            buf(slot, R[l], ctot)
            y = (slot, up_in[(l, i)], c)
            resblock(f"down{l}.{i}", h, y, l)
            h = y
            if R[l] in attn_res:
                # attention output replaces the skip in place (reads and writes the same view)
                attn(f"down{l}.{i}.attn", h, h, l)
        if l + 1 < nl:
            hn = (buf(f"down{l}.ds", R[l + 1], c), 0, c)
            conv(f"down{l}.downsample", h, hn, l, stride=2, gn=False, act=False)
            h = hn
    c = channels[-1]
    m1 = (buf("mid.0", R[-1], c), 0, c)
    resblock("mid.0", h, m1, nl - 1)
    # mid.1 writes into the h half of the first concat buffer of the up path
    first = f"cat{nl - 1}.1"
    h = (first, 0, up_in[(nl - 1, 1)])
    resblock("mid.1", m1, h, nl - 1)
    for l in reversed(range(nl)):
        c = channels[l]
        for j in range(2):
            i = 1 - j
            slot = f"cat{l}.{i}"
            x = (slot, 0, bufs[slot][2])
            # destination: the h half of the next concat buffer, or a plain buffer before an up-conv
            if j == 0:
                nxt = f"cat{l}.0"
                y = (nxt, 0, up_in[(l, 0)])
            else:
                y = (buf(f"up{l}.out", R[l], c), 0, c)
            resblock(f"up{l}.{j}", x, y, l)
            h = y
            if R[l] in attn_res:
                attn(f"up{l}.{j}.attn", h, h, l)
        if l > 0:
            nxt = f"cat{l - 1}.1"
            y = (nxt, 0, up_in[(l - 1, 1)])
            conv(f"up{l}.upsample", h, y, l, up=1, gn=False, act=False)   # input level l, output l-1
            h = y
    out = (buf("out", res, in_pad), 0, in_pad)
    conv("conv_out", h, out, 0)
    return bufs, ops


def unet_params(seed: int, ops, dtype: str = "f16", groups: int = 32, in_ch: int = 3, in_pad: int = 16):
    """Random-init parameters for every op: W ~ N(0, 1/fan_in), bias ~ N(0, 0.01) (a fixed time
    embedding is thought of as folded into the biases), gamma ~ N(1, 0.1), beta ~ N(0, 0.1)."""
    rng = _rng(seed)
    td = DTYPES[dtype]
    P = {}

    def gn(name, c):
        P[name + ".gamma"] = torch.from_numpy((1.0 + math.sqrt(0.1) * rng.standard_normal(c)).astype(np.float32))
        P[name + ".beta"] = torch.from_numpy((math.sqrt(0.1) * rng.standard_normal(c)).astype(np.float32))

    for op in ops:
        n = op["name"]
        if op["kind"] == "conv":
            cin = op["x"][2]
            cout = op["y"][2] if op["y"] is not None else None
            if cout is None:   # shortcut conv: output channels of the ResBlock
                cout = next(o["y"][2] for o in ops if o.get("shortcut") == n)
            w, b = conv_params(rng, cout, cin, op["k"], td)
            if n == "conv_in":    # padded input channels carry zeros; keep their weights zero too
                w[:, in_ch:] = 0
            if n == "conv_out":   # padded output channels produce exactly zero
                w[in_ch:] = 0
                b[in_ch:] = 0
            P[n + ".w"], P[n + ".b"] = w, b
            if op["gn"]:
                gn(n, cin)
        elif op["kind"] == "attn":
            c = op["C"]
            gn(n, c)
            for part in ("q", "k", "v", "o"):
                w, b = conv_params(rng, c, c, 1, td)
                P[f"{n}.{part}.w"], P[f"{n}.{part}.b"] = w, b
        else:   # transformer block
            c, dc = op["C"], op["d_ctx"]
            gn(n, c)
            for ln in ("ln1", "ln2", "ln3"):
                gn(f"{n}.{ln}", c)
            shapes = {"in": (c, c), "q1": (c, c), "k1": (c, c), "v1": (c, c), "o1": (c, c), "q2": (c, c),
                      "k2": (c, dc), "v2": (c, dc), "o2": (c, c), "ff1": (8 * c, c), "ff2": (c, 4 * c), "out": (c, c)}
            for part, (co, ci) in shapes.items():
                w, b = conv_params(rng, co, ci, 1, td)
                P[f"{n}.{part}.w"], P[f"{n}.{part}.b"] = w, b
            if "ctx" not in P:   # the text embeddings: one set for the whole network
                P["ctx"] = torch.from_numpy(rng.standard_normal((op["n_ctx"], dc)).astype(np.float32)).to(td)
    return P


def unet_images(seed: int, res: int, area_frac: float, dtype: str = "f16", in_ch: int = 3, in_pad: int = 16,
                n_blobs: int = 3):
    """Original and edited input image (N(0,1), zero padded to in_pad channels) and the image-level
    difference mask: blobs covering about area_frac, inside which all channels get N(0,1) noise."""
    rng = _rng(seed)
    td = DTYPES[dtype]
    s = res / 256.0
    mask = blob_mask(rng, res, res, max(1, int(round(area_frac * res * res))), n_blobs,
                     (5.0 * s + 0.5, 12.0 * s + 0.5), tol=0.1)
    a_o, a_e = edited_pair(rng, res, res, in_ch, mask, 1.0, td)
    pad = torch.zeros((res, res, in_pad - in_ch), dtype=td)
    return torch.cat([a_o, pad], 2).contiguous(), torch.cat([a_e, pad], 2).contiguous(), mask


# ----------------------------------------------------------------------------------------
# Synthetic SPADE-style conditional generator (benchmark configuration 5): a constant start tensor,
# seven spatially-adaptive residual blocks with nearest x2 up-sampling in between, modulation
# computed from a one-hot label map.  Again plain data: buffers (H, W, C) and a list of ops.
#   up   : y = nearest x2 of x
#   conv : y = conv(act(mod(x))) (+ residual / shortcut tiles); "spade" names the label map, the
#          two modulation convolutions' buffers and whether the instance-norm statistics of x are
#          cached from the pre-computation pass (Sec. 4.1: only above 16x32) or recomputed
# ----------------------------------------------------------------------------------------

def spade_topology(out_hw=(256, 512), start_hw=(8, 16), channels=(1024, 1024, 1024, 512, 256, 128, 64),
                   n_labels: int = 35, label_pad: int = 48, hidden: int = 128, out_pad: int = 16,
                   stats_cached_above=(16, 32)):
    """Blocks: head at the start size; middle 0 (after x2) and middle 1; then four blocks each after
    x2 (7 blocks, 5 up-samplings: start * 32 = output).  A block fin -> fout: main branch
    spade+leaky+3x3 (fin -> fmid), spade+leaky+3x3 (fmid -> fout); shortcut spade+1x1 (no
    activation) iff fin != fout, else identity.  Every spade layer has its own 3x3 label
    convolution (labels -> hidden, ReLU) and 3x3 modulation convolution (hidden -> gamma | beta)."""
    bufs, ops = {}, []
    ups = (0, 1, 0, 1, 1, 1, 1)
    assert len(channels) == 7 and start_hw[0] * 32 == out_hw[0] and start_hw[1] * 32 == out_hw[1]

    def buf(name, hw, c):
        bufs[name] = (hw[0], hw[1], c)
        return name

    def spade_conv(name, x, y, hw, cin, cout, k, act, residual=None, shortcut=None, scatter=True):
        seg = f"seg{hw[0]}"
        if seg not in bufs:
            buf(seg, hw, label_pad)
        actv = buf(name + ".actv", hw, hidden)
        mod = buf(name + ".mod", hw, 2 * cin)
        cached = hw[0] > stats_cached_above[0]
        ops.append(dict(kind="conv", name=name + ".shared", x=seg, y=actv, hw=hw, cin=label_pad, cout=hidden, k=3,
                        act=None, spade=None, residual=None, shortcut=None, scatter=True))
        ops.append(dict(kind="conv", name=name + ".gb", x=actv, y=mod, hw=hw, cin=hidden, cout=2 * cin, k=3,
                        act="relu", spade=None, residual=None, shortcut=None, scatter=True))
        ops.append(dict(kind="conv", name=name, x=x, y=y, hw=hw, cin=cin, cout=cout, k=k, act=act,
                        spade=dict(mod=mod, cached=cached), residual=residual, shortcut=shortcut, scatter=scatter))

    hw = tuple(start_hw)
    x = buf("z", hw, channels[0])
    cin = channels[0]
    for i, cout in enumerate(channels):
        name = f"block{i}"
        if ups[i]:
            hw = (hw[0] * 2, hw[1] * 2)
            xu = buf(name + ".in", hw, cin)
            ops.append(dict(kind="up", name=name + ".up", x=x, y=xu, hw=hw, cin=cin))
            x = xu
        fmid = min(cin, cout)
        h = buf(name + ".h", hw, fmid)
        y = buf(name + ".out", hw, cout)
        spade_conv(name + ".conv0", x, h, hw, cin, fmid, 3, "leaky")
        if cin != cout:
            spade_conv(name + ".short", x, None, hw, cin, cout, 1, None, scatter=False)
            spade_conv(name + ".conv1", h, y, hw, fmid, cout, 3, "leaky", shortcut=name + ".short")
        else:
            spade_conv(name + ".conv1", h, y, hw, fmid, cout, 3, "leaky", residual=x)
        x, cin = y, cout
    out = buf("out", hw, out_pad)
    ops.append(dict(kind="conv", name="conv_img", x=x, y=out, hw=hw, cin=cin, cout=out_pad, k=3, act="leaky",
                    spade=None, residual=None, shortcut=None, scatter=True))
    return bufs, ops


def spade_params(seed: int, bufs, ops, dtype: str = "f16", out_ch: int = 3, n_labels: int = 35):
    """W ~ N(0, 1/fan_in), bias ~ N(0, 0.01) (none on the 1x1 shortcuts); the modulation
    convolutions are scaled down (x 0.25) so that 1 + gamma stays near one; the constant start
    tensor ~ N(0,1); label-map weights of the padded label channels are zero."""
    rng = _rng(seed)
    td = DTYPES[dtype]
    P = {}
    for op in ops:
        if op["kind"] != "conv":
            continue
        n = op["name"]
        w, b = conv_params(rng, op["cout"], op["cin"], op["k"], td)
        if n.endswith(".shared"):
            w[:, n_labels:] = 0
        if n.endswith(".gb"):
            w, b = (w.float() * 0.25).to(td), b * 0.25
        if n.endswith(".short"):
            b = torch.zeros_like(b)
        if n == "conv_img":
            w[out_ch:] = 0
            b[out_ch:] = 0
        P[n + ".w"], P[n + ".b"] = w, b
    zs = bufs["z"]
    P["z"] = _t(rng.standard_normal(zs, dtype=np.float32), td)
    return P


def label_map(seed: int, H: int, W: int, n_labels: int = 35, n_regions: int = 40) -> np.ndarray:
    """A piecewise-constant label map: nearest-seed (Voronoi) regions with random classes."""
    rng = _rng(seed)
    cy, cx = rng.uniform(0, H, n_regions), rng.uniform(0, W, n_regions)
    cls = rng.integers(0, n_labels, n_regions)
    yy, xx = np.mgrid[0:H, 0:W]
    d = (yy[None] - cy[:, None, None]) ** 2 + (xx[None] - cx[:, None, None]) ** 2
    return cls[np.argmin(d, axis=0)].astype(np.int32)


def relabel(seed: int, labels: np.ndarray, area_frac: float, n_labels: int = 35, n_blobs: int = 3) -> np.ndarray:
    """An edit: inside a few elliptical blobs covering about area_frac every pixel gets one new class
    different from the class most common there (so that labels really change)."""
    rng = _rng(seed)
    H, W = labels.shape
    s = H / 256.0
    m = blob_mask(rng, H, W, max(1, int(round(area_frac * H * W))), n_blobs, (5.0 * s + 0.5, 12.0 * s + 0.5), tol=0.1)
    out = labels.copy()
    common = np.bincount(labels[m.astype(bool)], minlength=n_labels).argmax()
    new = int((common + 1 + rng.integers(0, n_labels - 1)) % n_labels)
    out[m.astype(bool)] = new
    return out


def one_hot_pyramid(labels: np.ndarray, sizes, n_labels: int, label_pad: int, dtype: str = "f16"):
    """The label map at every listed (H, W) by nearest subsampling, one-hot, zero-padded to label_pad."""
    td = DTYPES[dtype]
    H, W = labels.shape
    out = {}
    for (h, w) in sizes:
        sy, sx = H // h, W // w
        sub = labels[::sy, ::sx][:h, :w]
        oh = np.zeros((h, w, label_pad), dtype=np.float32)
        oh[np.arange(h)[:, None], np.arange(w)[None, :], sub] = 1.0
        out[(h, w)] = torch.from_numpy(oh).to(td).contiguous()
    return out
