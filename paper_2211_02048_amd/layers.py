"""Orchestration of the library calls for one wrapped convolution (Fig. "method"):
reduce -> gather -> conv -> scatter.  No arithmetic happens here; the class only owns
device buffers (packed weight, block list, tile workspaces) and issues the C-ABI calls
in order on torch's current stream.
"""
from __future__ import annotations

import torch

from . import api


class Workspace:
    """Tile buffers shared by layers that run one after another on one stream."""

    def __init__(self, device):
        self.device = device
        self._buf = {}

    def get(self, name: str, numel: int, dtype) -> torch.Tensor:
        key = (name, dtype)
        b = self._buf.get(key)
        if b is None or b.numel() < numel:
            b = torch.empty(max(numel, 1), dtype=dtype, device=self.device)
            self._buf[key] = b
        return b[:numel]


class BlockList:
    """Device-side ordered list of active blocks for one (resolution, block, kernel)."""

    def __init__(self, g: api.Geom, device, max_blocks=None, use_workspace=True):
        self.g = g
        self.max_blocks = g.grid_blocks if max_blocks is None else max_blocks
        self.indices = torch.zeros((max(self.max_blocks, 1), 2), dtype=torch.int32, device=device)
        self.count = torch.zeros(1, dtype=torch.int32, device=device)
        self.n_host = -1
        # per-block flag scratch for the reduction; starts zero and every call leaves it zero
        self.scratch = torch.zeros(api.sige_reduce_mask_workspace_bytes(g), dtype=torch.uint8,
                                   device=device) if use_workspace else None

    def reduce(self, *, a_orig=None, a_edit=None, tau=0.0, mask_in=None, mask_out=None, pool_log2=0,
               dilate=0):
        api.sige_reduce_mask(self.g, self.indices, self.count, a_orig=a_orig, a_edit=a_edit, tau=tau,
                             mask_in=mask_in, mask_out=mask_out, pool_log2=pool_log2, dilate=dilate,
                             max_blocks=self.max_blocks, workspace=self.scratch)
        self.n_host = -1

    @staticmethod
    def reduce_together(lists, *, a_orig=None, a_edit=None, tau=0.0, mask_in=None, mask_out=None,
                        pool_log2=0, dilate=0):
        """One call for the lists of several layer geometries at one resolution (same mask)."""
        api.sige_reduce_mask_lists([(b.g, b.indices, b.count, b.max_blocks, b.scratch) for b in lists],
                                   a_orig=a_orig, a_edit=a_edit, tau=tau, mask_in=mask_in, mask_out=mask_out,
                                   pool_log2=pool_log2, dilate=dilate)
        for b in lists:
            b.n_host = -1

    @staticmethod
    def mark_together(lists, **kw):
        """The marking half of reduce_together: the lists stay marked for api.sige_fused_conv_pair_marked."""
        api.sige_mark_blocks([b.desc() for b in lists], **kw)
        for b in lists:
            b.n_host = -1

    def desc(self):
        return (self.g, self.indices, self.count, self.max_blocks, self.scratch)

    def all_active(self):
        """Every block of the grid, row-major: the dense / pre-computation pass."""
        g = self.g
        ys = torch.arange(0, g.H_out, g.block_h, dtype=torch.int32)
        xs = torch.arange(0, g.W_out, g.block_w, dtype=torch.int32)
        idx = torch.stack(torch.meshgrid(ys, xs, indexing="ij"), dim=-1).reshape(-1, 2)
        n = idx.shape[0]
        assert n <= self.max_blocks
        self.indices[:n].copy_(idx)
        self.count.fill_(n)
        self.n_host = n
        return self

    def sync_count(self) -> int:
        """One device->host readback of the block count (once per edit and list)."""
        n = int(self.count.item())
        if n > self.max_blocks:
            raise api.SigeError(3, f"{n} active blocks exceed max_blocks={self.max_blocks}")
        self.n_host = n
        return n


class SigeConv:
    """One convolution wrapped for sparse update: packed weight + geometry."""

    def __init__(self, w_oihw: torch.Tensor, bias, H_in: int, W_in: int, block, stride: int = 1,
                 pad=None, up: int = 0):
        self.Cout, self.Cin, k, _ = w_oihw.shape
        self.g = api.geom(H_in, W_in, block, k, stride, pad)
        self.dtype = w_oihw.dtype
        self.device = w_oihw.device
        self.packed = api.sige_pack_weight(w_oihw)
        self.bias = None if bias is None else bias.to(self.device, torch.float32).contiguous()
        self.up = up
        self._split_bytes = {}     # capacity -> workspace bytes that allow every K split

    def tiles_numel(self, n):
        return n * self.g.tile_h * self.g.tile_w * self.Cin

    def out_numel(self, n):
        return n * self.g.block_h * self.g.block_w * self.Cout

    def fused_call(self, x, y, blocks: BlockList, ws: Workspace, *, scale=None, shift=None, act=api.ACT_NONE,
                   residual_tiles=None, residual=None, scatter=True, tag="t", split_k=True, act_outs=None):
        """The arguments of this layer's fused call as a struct for api.sige_fused_conv_pair (which runs
        two independent layers in one launch when it can).  Returns (call, out_tiles or None)."""
        g, n = self.g, blocks.n_host
        cap = blocks.max_blocks if n < 0 else max(n, 1)
        split = None
        if split_k:
            nb = self._split_bytes.get(cap)
            if nb is None:
                nb = self._split_bytes[cap] = api.sige_conv_workspace_bytes(self.dtype, g, self.Cin, self.Cout, cap)
            if nb:
                split = ws.get("split_k_" + tag, nb // 4, torch.float32)   # its own: the partner may run beside it
        out_tiles = None if scatter else ws.get("out_" + tag, self.out_numel(cap), self.dtype)
        call = api.fused_conv_call(x, g, blocks.indices, blocks.count, self.Cin, self.Cout, self.packed, self.bias,
                                   y=y if scatter else None, out_tiles=out_tiles, n_blocks=n, max_blocks=cap,
                                   scale=scale, shift=shift, act=act, up=self.up, residual_tiles=residual_tiles,
                                   residual=residual, workspace=split, act_outs=act_outs if scatter else None)
        return call, out_tiles

    def forward(self, x, y, blocks: BlockList, ws: Workspace, *, scale=None, shift=None,
                act=api.ACT_NONE, residual_tiles=None, residual=None, scatter=True, tag="t", fused=False,
                split_k=True, mod=None, act_outs=None):
        """gather(x) -> conv -> scatter into y (in place), as three calls or as the one fused call
        (a modulated gather, mod given, stays a call of its own; fused then folds the scatter into
        the convolution).  act_outs: activated copies of
        the output for the layers that normalise it next (the fused call only).
        Returns the output tiles (None when the fused call scattered them directly)."""
        g, n = self.g, blocks.n_host
        cap = blocks.max_blocks if n < 0 else max(n, 1)
        split = None
        if split_k:
            nb = self._split_bytes.get(cap)
            if nb is None:
                nb = self._split_bytes[cap] = api.sige_conv_workspace_bytes(self.dtype, g, self.Cin, self.Cout, cap)
            if nb:
                split = ws.get("split_k", nb // 4, torch.float32)
        if fused and mod is None:
            out_tiles = None if scatter else ws.get("out_" + tag, self.out_numel(cap), self.dtype)
            api.sige_fused_conv(x, g, blocks.indices, blocks.count, self.Cin, self.Cout, self.packed, self.bias,
                                y=y if scatter else None, out_tiles=out_tiles, n_blocks=n, max_blocks=cap,
                                scale=scale, shift=shift, act=act, up=self.up, residual_tiles=residual_tiles,
                                residual=residual, workspace=split, act_outs=act_outs if scatter else None)
            return out_tiles
        assert not act_outs, "activated copies are written by the fused call only"
        tiles = ws.get("tiles", self.tiles_numel(cap), self.dtype)
        out_tiles = ws.get("out_" + tag, self.out_numel(cap), self.dtype)
        if mod is None:
            api.sige_gather(x, g, blocks.indices, blocks.count, tiles, n_blocks=n, scale=scale, shift=shift,
                            act=act, up=self.up, C=self.Cin, max_blocks=cap)
        else:   # spatially-adaptive normalisation: per-pixel gamma | beta beside the cached statistics
            api.sige_gather_modulated(x, g, blocks.indices, blocks.count, tiles, mod, n_blocks=n, scale=scale,
                                      shift=shift, act=act, up=self.up, C=self.Cin, max_blocks=cap)
        if scatter and fused:     # a modulated gather, then the convolution with the scatter folded in
            api.sige_conv_scatter(tiles, g, blocks.indices, blocks.count, self.Cin, self.Cout, self.packed, self.bias,
                                  y, n_blocks=n, max_blocks=cap, residual_tiles=residual_tiles, residual=residual,
                                  workspace=split)
            return None
        api.sige_conv(tiles, g, self.Cin, self.Cout, self.packed, self.bias, blocks.count, out_tiles,
                      n_blocks=n, max_blocks=cap, workspace=split)
        if scatter:
            api.sige_scatter(out_tiles, g, blocks.indices, blocks.count, y, n_blocks=n,
                             residual_tiles=residual_tiles, residual=residual, Cout=self.Cout,
                             max_blocks=cap)
        return out_tiles
