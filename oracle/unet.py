"""CPU oracle (test infrastructure) for a whole UNet step of spatially sparse inference.

The method across layers, written densely and step by step (Sec. 3, Fig. "method"):
a first pass on the original image stores every wrapped layer's output and the group
statistics of every normalisation input; the edit pass computes each layer densely on
the whole current tensor with the CACHED statistics (Sec. 3.2 "Pre-computing
normalization parameters") and keeps the new values only on the active blocks of that
layer's resolution, the cached originals elsewhere (Fig. "pipeline" (b)).  Layers below
the sparse resolutions run with every block active (Sec. 4.1 "Implementation details").

The network itself is data (a list of operations over named buffers, see the workload
generator); this module only interprets it with the oracle's dense primitives.  Every
stored tensor (gathered activation, convolution output, layer output) is rounded once to
the storage type.
"""
from __future__ import annotations

import numpy as np

from . import sige_oracle as so


def _view(B, v):
    return B[v[0]][:, :, v[1]:v[1] + v[2]]


def _p64(P, name):
    return P[name].detach().cpu().double().numpy()


def level_blocks(mask, lvl_mask: int, dilate: int, Hout, Wout, b, k, stride, pad):
    m = so.level_mask(mask, lvl_mask, dilate)
    return so.active_blocks(m, Hout, Wout, b, b, k, stride, pad)


def all_blocks(Hout, Wout, b):
    return np.array([(y, x) for y in range(0, Hout, b) for x in range(0, Wout, b)], np.int32)


def unet_pass(bufs, ops, P, image, *, storage: str, groups: int = 32, eps: float = 1e-5, block: int = 16,
              cache=None, stats=None, mask=None, dilate: int = 1, min_sparse_res: int = 64):
    """One forward pass.  cache is None: dense pass on the original image, returns (buffers, stats).
    Otherwise: the edit pass over copies of the cached buffers, returns (buffers, blocks_per_op)."""
    rnd = lambda a: so.round_storage(a, storage)
    dense = cache is None
    B = {n: np.zeros(s) for n, s in bufs.items()} if dense else {n: a.copy() for n, a in cache.items()}
    B["image"] = np.asarray(image, dtype=np.float64).copy()
    stats_out = {} if dense else stats
    used_blocks = {}
    short = {}
    for op in ops:
        n = op["name"]
        x = _view(B, op["x"])
        r_in = x.shape[0]
        if op["kind"] == "conv":
            k, s, up = op["k"], op["stride"], op["up"]
            pad = k // 2
            xin = x.repeat(2, axis=0).repeat(2, axis=1) if up else x
            Hin = xin.shape[0]
            Hout = so.conv_out_size(Hin, k, s, pad)
            b = min(block, Hout)
            scale = shift = None
            if op["gn"]:
                if dense:
                    mean, var = so.gn_stats(x, groups)
                    stats_out[n] = so.fold_gn(_p64(P, n + ".gamma"), _p64(P, n + ".beta"), mean, var, eps)
                scale, shift = stats_out[n]
            act = so.ACT_SILU if op["act"] else so.ACT_NONE
            y = rnd(so.dense_layer(xin, _p64(P, n + ".w"), _p64(P, n + ".b"), s, pad, scale, shift, act,
                                   storage=storage))
            if not op["scatter"]:
                short[n] = y          # shortcut branch: added by the consumer on its blocks
                continue
            if op["shortcut"] is not None:
                y = rnd(y + short[op["shortcut"]])
            if op["residual"] is not None:
                y = rnd(y + _view(B, op["residual"]))
            yv = _view(B, op["y"])
            if dense or r_in < min_sparse_res:
                blocks = all_blocks(Hout, Hout, b)
            else:
                # the mask lives at the convolution's input resolution (after up-sampling, if any)
                lvl_mask = int(np.log2(mask.shape[0] // Hin))
                blocks = level_blocks(mask, lvl_mask, dilate, Hout, Hout, b, 3 if k == 1 else k, s,
                                      1 if k == 1 else pad)
            used_blocks[n] = blocks
            yv[...] = so.select_blocks(y, yv, blocks, b, b)
        else:  # self-attention block: GN -> q, k, v (1x1) -> attention -> proj (1x1) -> + x
            C, heads = op["C"], op["heads"]
            d = C // heads
            T = r_in * r_in
            if dense:
                mean, var = so.gn_stats(x, groups)
                stats_out[n] = so.fold_gn(_p64(P, n + ".gamma"), _p64(P, n + ".beta"), mean, var, eps)
            scale, shift = stats_out[n]
            z = rnd(so.scale_shift_act(x, scale, shift, so.ACT_NONE))
            q, kk, v = [rnd(so.conv2d(z, _p64(P, f"{n}.{p}.w"), _p64(P, f"{n}.{p}.b"))) for p in "qkv"]
            a = rnd(so.attention(q.reshape(T, heads, d), kk.reshape(T, heads, d), v.reshape(T, heads, d),
                                 1.0 / np.sqrt(d))).reshape(r_in, r_in, C)
            y = rnd(so.conv2d(a, _p64(P, n + ".o.w"), _p64(P, n + ".o.b")))
            y = rnd(y + x)
            assert dense or r_in < min_sparse_res, "attention is only wrapped at all-active resolutions here"
            _view(B, op["y"])[...] = y
    return (B, stats_out) if dense else (B, used_blocks)
