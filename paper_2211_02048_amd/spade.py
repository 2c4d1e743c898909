"""A synthetic SPADE-style conditional generator driven entirely through the C-ABI calls.

The edited input is the label map.  `precompute` runs every layer with all blocks active on the
original label map and caches every layer's output (the modulation tensors included) and the
instance-norm statistics of every modulated layer's input; `set_edit` thresholds the difference
of the one-hot label maps into the image-level mask and reduces it to one block list per
resolution; `step` updates the active blocks in place.  Statistics are cached only above 16x32
and recomputed below, layers at or below `min_sparse` keep every block active (Sec. 4.1
"Implementation details").  Successive edits reuse the caches: each step leaves them equal to a
pass on the current label map (up to the method's approximation), so the next edit's mask is the
difference against the current label map.

Nothing here computes: buffers, weight packing and the order of the library calls only.
"""
from __future__ import annotations

import math

import torch

from . import api, inputs
from .layers import BlockList, SigeConv, Workspace

ACTS = {None: api.ACT_NONE, "relu": api.ACT_RELU, "leaky": api.ACT_LEAKY_RELU}


class SigeSpade:
    def __init__(self, topo=None, dtype="f16", seed=1005, device="cuda", block=16, eps=1e-5, dilate=1,
                 min_sparse=(8, 16), params=None, n_labels=35, merge_label_convs=True):
        topo = topo or {}
        self.device, self.td = device, inputs.DTYPES[dtype]
        self.block, self.eps, self.dilate, self.min_sparse = block, eps, dilate, min_sparse
        self.bufs_shape, self.ops = inputs.spade_topology(**topo)
        P = params if params is not None else inputs.spade_params(seed, self.bufs_shape, self.ops, dtype,
                                                                  n_labels=n_labels)
        self.B = {n: torch.zeros(s, dtype=self.td, device=device) for n, s in self.bufs_shape.items()}
        self.B["z"].copy_(P["z"])
        self.seg_sizes = sorted({(s[0], s[1]) for n, s in self.bufs_shape.items() if n.startswith("seg")})
        self.out_hw = self.bufs_shape["out"][:2]
        self.ws = Workspace(device)
        self.lists, self.layers = {}, {}
        self.mask = torch.zeros(self.out_hw, dtype=torch.uint8, device=device)
        # Optional observer for tests: hook(when, name, layer, tensors), when = "pre" before an operation's
        # calls are issued and "post" after them; it may read and overwrite buffers (after synchronising).
        self.hook = None
        for op in self.ops:
            n, (h, w) = op["name"], op["hw"]
            b = min(block, h)
            L = dict(op=op, sparse=h > min_sparse[0], list=self._lists(h, w, b))
            if op["kind"] == "conv":
                L["conv"] = SigeConv(P[n + ".w"].to(device), P[n + ".b"], h, w, b, 1, op["k"] // 2)
                if op["spade"] is not None:
                    C = op["cin"]
                    L["mean"], L["var"] = torch.zeros(C, device=device), torch.zeros(C, device=device)
                    L["scale"], L["shift"] = torch.zeros(C, device=device), torch.zeros(C, device=device)
            else:
                L["g1"] = api.geom(h, w, b, 1, 1, 0)
            self.layers[n] = L
        if merge_label_convs:
            self._merge_label_convs(P)

    def _merge_label_convs(self, P):
        """The label-map convolutions of one residual block (one per modulated layer: two or three)
        read the same label map through the same block list, so they run as ONE convolution whose
        output channels are theirs side by side; each hidden tensor becomes a channel slice of the
        joint buffer (the modulation convolutions read it through its pixel stride).  Same
        arithmetic per output channel, fewer launches."""
        groups = {}
        for n, L in self.layers.items():
            op = L["op"]
            if op["kind"] == "conv" and n.endswith(".shared"):
                groups.setdefault((n.split(".")[0], op["hw"]), []).append(n)
        for (blk, (h, w)), names in groups.items():
            if len(names) < 2:
                continue
            ops = [self.layers[n]["op"] for n in names]
            hidden = [o["cout"] for o in ops]
            joint = torch.zeros((h, w, sum(hidden)), dtype=self.td, device=self.device)
            c0 = 0
            for o, c in zip(ops, hidden):
                self.B[o["y"]] = joint[:, :, c0:c0 + c]
                c0 += c
            first = self.layers[names[0]]
            b = first["conv"].g.block_h
            first["conv"] = SigeConv(torch.cat([P[n + ".w"] for n in names], 0).to(self.device),
                                     torch.cat([P[n + ".b"] for n in names], 0), h, w, b, 1, 1)
            first["joint"] = joint
            for n in names[1:]:
                self.layers[n]["merged"] = True

    def _lists(self, h, w, b):
        key = (h, w, b)
        if key not in self.lists:
            g = api.geom(h, w, b, 3, 1, 1)
            self.lists[key] = [BlockList(g, self.device).all_active(), BlockList(g, self.device)]
        return self.lists[key]

    def load_labels(self, seg):
        """seg: {(h, w): one-hot label map} for every resolution the network reads."""
        for (h, w) in self.seg_sizes:
            self.B[f"seg{h}"].copy_(seg[(h, w)])

    def set_edit(self, seg_new, exact: bool = True):
        """Difference mask of the full-resolution one-hot label maps (current vs new), then one block
        list per resolution; loads the new label maps.  Returns the block counts."""
        full = self.out_hw
        cur = self.B[f"seg{full[0]}"]
        new = seg_new[full].to(self.device)
        lists = {k: v[1] for k, v in self.lists.items() if k[0] > self.min_sparse[0]}
        top = lists[(full[0], full[1], min(self.block, full[0]))]
        top.max_blocks = top.indices.shape[0]
        top.reduce(a_orig=cur, a_edit=new, tau=0.0, mask_out=self.mask, dilate=self.dilate)
        for (h, w, b), bl in lists.items():
            if bl is top:
                continue
            bl.max_blocks = bl.indices.shape[0]
            bl.reduce(mask_in=self.mask, pool_log2=int(math.log2(full[0] // h)), dilate=self.dilate)
        counts = {}
        for (h, w, b), bl in lists.items():
            n = bl.sync_count()
            counts[(h, w)] = n
            if not exact:
                bl.n_host = -1
                bl.max_blocks = min(bl.indices.shape[0], max(8, 1 << max(0, (n - 1).bit_length())))
        self.load_labels(seg_new)
        return counts

    def _run(self, dense: bool):
        short = {}
        for n, L in self.layers.items():
            op = L["op"]
            if L.get("merged"):       # computed by the block's joint label-map convolution
                continue
            bl = L["list"][0 if (dense or not L["sparse"]) else 1]
            x = self.B[op["x"]]
            if self.hook:
                self.hook("pre", n, L, dict(dense=dense, blocks=bl))
            if op["kind"] == "up":
                g1 = L["g1"]
                nb, cap = bl.n_host, (bl.max_blocks if bl.n_host < 0 else max(bl.n_host, 1))
                t = self.ws.get("up_t", cap * g1.block_h * g1.block_w * op["cin"], self.td)
                api.sige_gather(x, g1, bl.indices, bl.count, t, n_blocks=nb, up=1, C=op["cin"], max_blocks=cap)
                api.sige_scatter(t, g1, bl.indices, bl.count, self.B[op["y"]], n_blocks=nb, Cout=op["cin"],
                                 max_blocks=cap)
                if self.hook:
                    self.hook("post", n, L, dict(dense=dense, blocks=bl))
                continue
            scale = shift = mod = None
            if op["spade"] is not None:
                scale, shift, mod = L["scale"], L["shift"], self.B[op["spade"]["mod"]]
                if dense or not op["spade"]["cached"]:   # instance norm = one group per channel
                    api.sige_gn_stats(x, op["cin"], L["mean"], L["var"], eps=self.eps, scale=scale, shift=shift,
                                      C=op["cin"])
            act = ACTS[op["act"]]
            if not op["scatter"]:
                short[n] = L["conv"].forward(x, None, bl, self.ws, scale=scale, shift=shift, act=act, mod=mod,
                                             scatter=False, tag="short")
                if self.hook:
                    self.hook("post", n, L, dict(dense=dense, blocks=bl, tiles=short[n]))
                continue
            res_t = short.get(op["shortcut"]) if op["shortcut"] else None
            res_f = self.B[op["residual"]] if op["residual"] is not None else None
            L["conv"].forward(x, L.get("joint", self.B[op["y"]]), bl, self.ws, scale=scale, shift=shift, act=act,
                              mod=mod, residual_tiles=res_t, residual=res_f, tag="main", fused=True)
            if self.hook:
                self.hook("post", n, L, dict(dense=dense, blocks=bl))
        return self.B["out"]

    def precompute(self, seg):
        self.load_labels(seg)
        return self._run(dense=True)

    def step(self):
        """Sparse pass on the label maps loaded by set_edit: updates the caches in place."""
        return self._run(dense=False)

    def capture(self):
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            for _ in range(2):
                self.step()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.step()
        torch.cuda.synchronize()
        return g

    def macs(self, counts=None):
        total = 0
        for n, L in self.layers.items():
            op = L["op"]
            if op["kind"] != "conv":
                continue
            g = L["conv"].g
            nblk = g.grid_blocks
            if counts is not None and L["sparse"]:
                nblk = counts[op["hw"]]
            total += nblk * g.block_h * g.block_w * op["k"] ** 2 * op["cin"] * op["cout"]
        return total
