"""CPU oracle (test infrastructure) for one pass of a SPADE-style conditional generator under
spatially sparse inference.

As for the UNet: the method across layers, written densely and step by step.  The first pass
runs on the original label map and keeps every layer's output and the instance-normalisation
statistics of every modulated layer's input; an edit pass computes each layer densely from the
current tensors, with the cached statistics where the method caches them (Sec. 3.2
"Pre-computing normalization parameters"; Sec. 4.1: for the GAN only above 16x32, recomputed
below), and keeps the new values on the active blocks of that layer's resolution (Fig.
"pipeline" (b)).  The difference mask is where the label map changed; per resolution it is
max-pooled and dilated.  Layers at or below min_sparse (Sec. 4.1) run with every block active.
Every stored tensor is rounded once to the storage type.
"""
from __future__ import annotations

import numpy as np

from . import sige_oracle as so
from .unet import all_blocks, level_blocks

ACTS = {None: so.ACT_NONE, "relu": so.ACT_RELU, "leaky": so.ACT_LEAKY_RELU}


def _p64(P, name):
    return P[name].detach().cpu().double().numpy()


def instance_stats(x, eps: float):
    """Per-channel mean and biased variance over the pixels, folded into scale / shift."""
    x = np.asarray(x, dtype=np.float64)
    mean = x.mean(axis=(0, 1))
    var = ((x - mean) ** 2).mean(axis=(0, 1))
    scale = 1.0 / np.sqrt(var + eps)
    return scale, -mean * scale


def spade_pass(bufs, ops, P, seg, *, storage: str, eps: float = 1e-5, block: int = 16, cache=None, stats=None,
               mask=None, dilate: int = 1, min_sparse=(8, 16), trace=None):
    """seg: {(h, w): one-hot label map [h, w, label_pad]} for every resolution.  cache None: the
    pass on the original label map, returns (buffers, stats); otherwise the edit pass over copies
    of the cached buffers, returns (buffers, blocks per op).  trace (a list, optional) receives one
    (op name, {"y": copy of the buffer the operation wrote} or {"short": a shortcut branch's full
    output, "t": the modulated and activated input}) entry per operation, in order."""
    rnd = lambda a: so.round_storage(a, storage)
    dense = cache is None
    B = {n: np.zeros(s) for n, s in bufs.items()} if dense else {n: a.copy() for n, a in cache.items()}
    for n, s in bufs.items():
        if n.startswith("seg"):
            B[n] = np.asarray(seg[(s[0], s[1])], dtype=np.float64).copy()
    B["z"] = _p64(P, "z")
    stats_out = {} if dense else dict(stats)
    used, short = {}, {}
    for op in ops:
        n, (h, w) = op["name"], op["hw"]
        b = min(block, h)
        if dense or h <= min_sparse[0]:
            blocks = all_blocks(h, w, b) if h == w else np.array(
                [(y, x) for y in range(0, h, b) for x in range(0, w, b)], np.int32)
        else:
            lvl = int(np.log2(mask.shape[0] // h))
            m = so.level_mask(mask, lvl, dilate)
            blocks = so.active_blocks(m, h, w, b, b, 3, 1, 1)
        used[n] = blocks
        x = B[op["x"]]
        if op["kind"] == "up":
            y = x.repeat(2, axis=0).repeat(2, axis=1)
            B[op["y"]] = so.select_blocks(y, B[op["y"]], blocks, b, b)
            if trace is not None:
                trace.append((n, {"y": B[op["y"]].copy()}))
            continue
        act = ACTS[op["act"]]
        if op["spade"] is not None:
            if dense or not op["spade"]["cached"]:
                stats_out[n] = instance_stats(x, eps)       # the current tensor's statistics
            scale, shift = stats_out[n]
            mod = B[op["spade"]["mod"]]
            C = op["cin"]
            t = rnd(so.modulate(x, scale, shift, mod[:, :, :C], mod[:, :, C:], act))
        else:
            t = rnd(so.activation(x, act))
        k = op["k"]
        # a layer's stored output is the convolution plus its residuals (Scatter with Block Residual,
        # App. A.2), rounded once; a shortcut branch's output is a stored tensor itself
        y = so.conv2d(t, _p64(P, n + ".w"), _p64(P, n + ".b"), 1, k // 2)
        if not op["scatter"]:
            y = rnd(y)
            short[n] = y
            if trace is not None:
                trace.append((n, {"short": y.copy()}))
            continue
        if op["shortcut"] is not None:
            y = y + short[op["shortcut"]]
        if op["residual"] is not None:
            y = y + B[op["residual"]]
        y = rnd(y)
        B[op["y"]] = so.select_blocks(y, B[op["y"]], blocks, b, b)
        if trace is not None:
            trace.append((n, {"y": B[op["y"]].copy()}))
    return (B, stats_out) if dense else (B, used)
