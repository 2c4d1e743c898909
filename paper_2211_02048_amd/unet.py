"""A synthetic DDPM-style UNet denoiser driven entirely through the C-ABI calls.

Two passes (Sec. 3 of the paper): `precompute` runs every layer with all blocks active on the
original image, computes the group statistics of every normalisation input on the fly and leaves
every layer's output in its buffer (the cache); `set_edit` reduces the image-level difference mask to
one block list per resolution and layer geometry (Sec. 3.2, once per edit); `step` then updates
only the active blocks, in place, with the cached statistics.  Layers whose input resolution is
below `min_sparse_res` keep every block active (Sec. 4.1 "Implementation details").

Nothing here computes: buffers, views, weight packing and the order of the library calls only.
A concat is never materialised - producers scatter straight into channel slices of the buffer
the consumer gathers from.
"""
from __future__ import annotations

import math

import torch

from . import api, inputs
from .layers import BlockList, SigeConv, Workspace


def _next_pow2(n: int) -> int:
    p = 1
    while p < n:
        p *= 2
    return p


class SigeUNet:
    def __init__(self, res=256, channels=(128, 128, 256, 256, 512, 512), attn_res=(16,), heads=4,
                 dtype="f16", seed=1003, device="cuda", block=16, groups=32, eps=1e-5, dilate=1,
                 min_sparse_res=64, params=None, fused=True):
        self.res, self.device, self.td = res, device, inputs.DTYPES[dtype]
        self.block, self.groups, self.eps, self.dilate, self.min_sparse_res = block, groups, eps, dilate, min_sparse_res
        self.bufs_shape, self.ops = inputs.unet_topology(res, 3, channels, attn_res, heads)
        P = params if params is not None else inputs.unet_params(seed, self.ops, dtype, groups)
        self.B = {n: torch.zeros(s, dtype=self.td, device=device) for n, s in self.bufs_shape.items()}
        self.ws = Workspace(device)
        self.lists = {}        # (H_in, k, stride) -> [all-active list, sparse list]
        self.layers = {}
        self.graph = None
        # True: one fused gather-conv-scatter call per convolution instead of three; "lowres": only
        # for the layers below min_sparse_res (all blocks active, few of them, many channels)
        self.fused = fused
        f32 = lambda t: t.to(device, torch.float32).contiguous()
        for op in self.ops:
            n, C = op["name"], op["x"][2]
            r_in = self.bufs_shape[op["x"][0]][0]
            L = dict(op=op, sparse=r_in >= min_sparse_res)
            if op["kind"] == "conv":
                Hin = r_in * (2 if op["up"] else 1)
                Hout = (Hin + 2 * (op["k"] // 2) - op["k"]) // op["stride"] + 1
                b = min(block, Hout)
                L["conv"] = SigeConv(P[n + ".w"].to(device), P[n + ".b"], Hin, Hin, b, op["stride"], op["k"] // 2,
                                     up=op["up"])
                kk = 3 if op["k"] == 1 else op["k"]          # a 1x1 shortcut runs on its ResBlock's 3x3 list
                L["list"] = self._lists(Hin, kk, op["stride"], b)
            else:
                b = min(block, r_in)
                wqkv = torch.cat([P[f"{n}.{p}.w"] for p in "qkv"], 0).to(device)
                bqkv = torch.cat([P[f"{n}.{p}.b"] for p in "qkv"], 0)
                L["qkv"] = SigeConv(wqkv, bqkv, r_in, r_in, b, 1, 0)
                L["proj"] = SigeConv(P[n + ".o.w"].to(device), P[n + ".o.b"], r_in, r_in, b, 1, 0)
                L["list"] = self._lists(r_in, 3, 1, b)
                T = r_in * r_in
                L["qkv_buf"] = torch.zeros((r_in, r_in, 3 * C), dtype=self.td, device=device)
                L["att_buf"] = torch.zeros((r_in, r_in, C), dtype=self.td, device=device)
                nb = api.sige_sparse_attn_workspace_bytes(T, T, op["heads"], C // op["heads"])
                L["att_ws"] = torch.zeros(max(nb // 4, 1), dtype=torch.float32, device=device) if nb else None
                assert not L["sparse"], "attention is wrapped at all-active resolutions only"
            if op["kind"] == "attn" or op["gn"]:
                L["gamma"], L["beta"] = f32(P[n + ".gamma"]), f32(P[n + ".beta"])
                L["mean"] = torch.zeros(groups, device=device)
                L["var"] = torch.zeros(groups, device=device)
                L["scale"] = torch.zeros(C, device=device)
                L["shift"] = torch.zeros(C, device=device)
            self.layers[n] = L

    # ------------------------------------------------------------------ plumbing
    def _lists(self, Hin, k, stride, b):
        key = (Hin, k, stride, b)
        if key not in self.lists:
            g = api.geom(Hin, Hin, b, k, stride, k // 2)
            self.lists[key] = [BlockList(g, self.device).all_active(), BlockList(g, self.device)]
        return self.lists[key]

    def view(self, v):
        return self.B[v[0]][:, :, v[1]:v[1] + v[2]]

    # ------------------------------------------------------------------ passes
    def set_edit(self, mask_image: torch.Tensor, exact: bool = True):
        """Image-level difference mask (u8 [res, res], device) -> one block list per geometry that a
        sparse layer uses.  exact=True reads every count back once and sizes later launches exactly;
        exact=False keeps the counts on the device and sizes launches by a capacity (power of two
        above the count), which is what a captured graph needs."""
        used = {id(L["list"][1]): L["list"][1] for L in self.layers.values() if L["sparse"]}
        by_res = {}
        for bl in used.values():
            bl.max_blocks = bl.indices.shape[0]
            by_res.setdefault(bl.g.H_in, []).append(bl)
        for H_in, group in by_res.items():       # one call per resolution: its geometries share the mask
            pool = int(math.log2(self.res // H_in))
            for i in range(0, len(group), 4):
                BlockList.reduce_together(group[i:i + 4], mask_in=mask_image, pool_log2=pool, dilate=self.dilate)
        counts = {}
        for bl in used.values():
            n = bl.sync_count()
            counts[(bl.g.H_in, bl.g.k, bl.g.stride)] = n
            if not exact:
                bl.n_host = -1
                bl.max_blocks = min(bl.indices.shape[0], max(8, _next_pow2(n)))
        return counts

    def _run(self, image, dense: bool):
        self.B["image"].copy_(image)
        shortcut_tiles = {}
        for n, L in self.layers.items():
            op = L["op"]
            fused = self.fused is True or (self.fused == "lowres" and not L["sparse"])
            bl = L["list"][0 if (dense or not L["sparse"]) else 1]
            x = self.view(op["x"])
            scale = shift = None
            if "scale" in L:
                scale, shift = L["scale"], L["shift"]
                if dense:   # statistics of the original activation, computed where a dense model would
                    api.sige_gn_stats(x, self.groups, L["mean"], L["var"], gamma=L["gamma"], beta=L["beta"],
                                      eps=self.eps, scale=scale, shift=shift, C=op["x"][2])
            if op["kind"] == "conv":
                act = api.ACT_SILU if op["act"] else api.ACT_NONE
                if not op["scatter"]:
                    shortcut_tiles[n] = L["conv"].forward(x, None, bl, self.ws, scatter=False, tag="short",
                                                          fused=fused)
                    continue
                res_t = shortcut_tiles.get(op["shortcut"]) if op["shortcut"] else None
                res_f = self.view(op["residual"]) if op["residual"] is not None else None
                L["conv"].forward(x, self.view(op["y"]), bl, self.ws, scale=scale, shift=shift, act=act,
                                  residual_tiles=res_t, residual=res_f, tag="main", fused=fused)
            else:
                C, heads = op["C"], op["heads"]
                T = x.shape[0] * x.shape[1]
                L["qkv"].forward(x, L["qkv_buf"], bl, self.ws, scale=scale, shift=shift, tag="main",
                                 fused=fused)
                qkv = L["qkv_buf"].view(T, 3 * C)
                api.sige_sparse_attn(qkv[:, :C], qkv[:, C:2 * C], qkv[:, 2 * C:], L["att_buf"].view(T, C),
                                     1.0 / math.sqrt(C // heads), Nq=T, workspace=L["att_ws"], heads=heads,
                                     d=C // heads, q_ld=3 * C, kv_ld=3 * C, o_ld=C)
                L["proj"].forward(L["att_buf"], self.view(op["y"]), bl, self.ws, residual=x, tag="main",
                                  fused=fused)
        return self.B["out"]

    def precompute(self, image):
        """Dense pass on the original image: fills every cache and the normalisation statistics."""
        return self._run(image, dense=True)

    def step(self, image_edit):
        """Sparse pass on the edited image (after set_edit): updates the caches in place."""
        return self._run(image_edit, dense=False)

    def capture(self, image_edit):
        """Captures step(image_edit) in a HIP graph (lists sized by capacity, counts on the device)."""
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            for _ in range(2):
                self.step(image_edit)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.step(image_edit)
        torch.cuda.synchronize()
        return g

    def macs(self, counts=None):
        """Multiply-accumulates of one pass: dense (counts None) or with the given active-block counts."""
        total = 0
        for n, L in self.layers.items():
            op = L["op"]
            if op["kind"] != "conv":
                C, r = op["C"], self.bufs_shape[op["x"][0]][0]
                total += r * r * C * C * 4 + 2 * (r * r) ** 2 * C
                continue
            c = L["conv"]
            g = c.g
            nblk = g.grid_blocks
            if counts is not None and L["sparse"]:
                kk = 3 if g.k == 1 else g.k
                nblk = counts[(g.H_in, kk, g.stride)]
            total += nblk * g.block_h * g.block_w * g.k * g.k * c.Cin * c.Cout
        return total
