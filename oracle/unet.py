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
stored tensor (gathered activation, shortcut tiles, layer output = convolution plus its
residuals) is rounded once to the storage type.
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


def _transformer_block(op, B, P, x, rnd, dense, stats, used_blocks, mask, dilate, block, min_sparse_res,
                       groups, eps, rec=None):
    """A latent-diffusion style transformer block under the method (Sec. 3.2 "Extension to attention
    layers", Fig. "sige-attention"), written densely: every stage is computed for all tokens from the
    current tensors and kept only on the tokens of the active blocks; the self-attention keys and
    values are caches whose active tokens are overwritten before the attention runs.  Stages: group
    norm (cached statistics) + 1x1 in; layer norm + self-attention + residual; layer norm +
    cross-attention over the text embeddings + residual; layer norm + gated-GELU feed-forward +
    residual; 1x1 out + the block's input.  Every stored tensor is rounded once to the storage type.
    rec (a dict, optional) receives a copy of every stored tensor of the block, whole, under the
    names used below."""
    n, C, heads = op["name"], op["C"], op["heads"]
    note = (lambda name, a: rec.__setitem__(name, np.array(a, copy=True))) if rec is not None else (lambda name, a: None)
    d = C // heads
    r = x.shape[0]
    T = r * r
    b = min(block, r)
    lin = lambda z, part: so.conv2d(z, _p64(P, f"{n}.{part}.w"), _p64(P, f"{n}.{part}.b"))
    ln = lambda z, part: so.layer_norm(z, _p64(P, f"{n}.{part}.gamma"), _p64(P, f"{n}.{part}.beta"), 1e-5)
    if dense:
        mean, var = so.gn_stats(x, groups)
        stats[n] = so.fold_gn(_p64(P, n + ".gamma"), _p64(P, n + ".beta"), mean, var, eps)
        for name in ("h0", "h1", "h2", "h3"):
            B[f"{n}.{name}"] = np.zeros((r, r, C))
        B[f"{n}.kv"] = np.zeros((r, r, 2 * C))
    if dense or r < min_sparse_res:
        blocks = all_blocks(r, r, b)
    else:   # the tokens that changed are the output blocks of the 3x3 convolution before this block
        lvl_mask = int(np.log2(mask.shape[0] // r))
        blocks = level_blocks(mask, lvl_mask, dilate, r, r, b, 3, 1, 1)
    used_blocks[n] = blocks
    keep = lambda new, name: B.__setitem__(name, so.select_blocks(new, B[name], blocks, b, b))
    scale, shift = stats[n]
    x_in = x.copy()
    keep(rnd(lin(rnd(so.scale_shift_act(x, scale, shift, so.ACT_NONE)), "in")), f"{n}.h0")
    h0 = B[f"{n}.h0"]
    note("h0", h0)
    # self-attention
    tn = rnd(ln(h0, "ln1"))
    note("tn1", tn)
    q = rnd(lin(tn, "q1"))
    note("q1", q)
    kv = np.concatenate([rnd(lin(tn, "k1")), rnd(lin(tn, "v1"))], axis=2)
    keep(kv, f"{n}.kv")
    kv = B[f"{n}.kv"]
    note("kv", kv)
    a = rnd(so.attention(q.reshape(T, heads, d), kv[:, :, :C].reshape(T, heads, d),
                         kv[:, :, C:].reshape(T, heads, d), 1.0 / np.sqrt(d))).reshape(r, r, C)
    note("a1", a)
    keep(rnd(lin(a, "o1") + h0), f"{n}.h1")
    h1 = B[f"{n}.h1"]
    note("h1", h1)
    # cross-attention over the text embeddings
    ctx = _p64(P, "ctx")[None]                       # [1, n_ctx, d_ctx] as a one-row image
    kc, vc = rnd(lin(ctx, "k2"))[0], rnd(lin(ctx, "v2"))[0]
    note("kc", np.concatenate([kc, vc], axis=1))
    tn = rnd(ln(h1, "ln2"))
    note("tn2", tn)
    q = rnd(lin(tn, "q2"))
    note("q2", q)
    nc = kc.shape[0]
    a = rnd(so.attention(q.reshape(T, heads, d), kc.reshape(nc, heads, d), vc.reshape(nc, heads, d),
                         1.0 / np.sqrt(d))).reshape(r, r, C)
    note("a2", a)
    keep(rnd(lin(a, "o2") + h1), f"{n}.h2")
    h2 = B[f"{n}.h2"]
    note("h2", h2)
    # gated-GELU feed-forward
    tn = rnd(ln(h2, "ln3"))
    note("tn3", tn)
    # the first feed-forward layer and its gated GELU are one layer with one stored tensor
    gg = rnd(so.geglu(lin(tn, "ff1")))
    note("gg", gg)
    keep(rnd(lin(gg, "ff2") + h2), f"{n}.h3")
    h3 = B[f"{n}.h3"]
    note("h3", h3)
    y = rnd(lin(h3, "out") + x_in)
    yv = _view(B, op["y"])
    yv[...] = so.select_blocks(y, yv, blocks, b, b)
    note("y", B[op["y"][0]])


def unet_pass(bufs, ops, P, image, *, storage: str, groups: int = 32, eps: float = 1e-5, block: int = 16,
              cache=None, stats=None, mask=None, dilate: int = 1, min_sparse_res: int = 64, trace=None):
    """One forward pass.  cache is None: dense pass on the original image, returns (buffers, stats).
    Otherwise: the edit pass over copies of the cached buffers, returns (buffers, blocks_per_op).
    trace (a list, optional) receives one (op name, {tensor name: copy}) entry per operation, in order:
    "y" = the whole buffer the operation wrote, as it stands right after it ("short" = the full output
    of a shortcut branch, which is kept in no buffer), plus the inner tensors of an attention block."""
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
            # a layer's stored output is the convolution plus its residuals (Scatter with Block
            # Residual, App. A.2), rounded once; a shortcut branch's output is a stored tensor itself
            y = so.dense_layer(xin, _p64(P, n + ".w"), _p64(P, n + ".b"), s, pad, scale, shift, act,
                               storage=storage)
            if not op["scatter"]:
                y = rnd(y)
                short[n] = y          # shortcut branch: added by the consumer on its blocks
                if trace is not None:
                    trace.append((n, {"short": y.copy()}))
                continue
            if op["shortcut"] is not None:
                y = y + short[op["shortcut"]]
            if op["residual"] is not None:
                y = y + _view(B, op["residual"])
            y = rnd(y)
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
            if trace is not None:
                trace.append((n, {"y": B[op["y"][0]].copy()}))
        elif op["kind"] == "xfmr":
            rec = {} if trace is not None else None
            _transformer_block(op, B, P, x, rnd, dense, stats_out, used_blocks, mask, dilate, block,
                               min_sparse_res, groups, eps, rec)
            if trace is not None:
                trace.append((n, rec))
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
            y = rnd(so.conv2d(a, _p64(P, n + ".o.w"), _p64(P, n + ".o.b")) + x)
            assert dense or r_in < min_sparse_res, "attention is only wrapped at all-active resolutions here"
            _view(B, op["y"])[...] = y
            used_blocks[n] = all_blocks(r_in, r_in, min(block, r_in))
            if trace is not None:
                trace.append((n, {"qkv": np.concatenate([q, kk, v], axis=2), "a": a.copy(), "y": B[op["y"][0]].copy()}))
    return (B, stats_out) if dense else (B, used_blocks)
