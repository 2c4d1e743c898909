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
                 min_sparse_res=64, params=None, fused=True, in_ch=3, attn_kind="attn", ctx=(77, 768),
                 act_copies=True):
        self.res, self.device, self.td = res, device, inputs.DTYPES[dtype]
        self.block, self.groups, self.eps, self.dilate, self.min_sparse_res = block, groups, eps, dilate, min_sparse_res
        self.bufs_shape, self.ops = inputs.unet_topology(res, in_ch, channels, attn_res, heads, attn_kind=attn_kind,
                                                         ctx=ctx)
        P = params if params is not None else inputs.unet_params(seed, self.ops, dtype, groups, in_ch=in_ch)
        self.B = {n: torch.zeros(s, dtype=self.td, device=device) for n, s in self.bufs_shape.items()}
        self.ws = Workspace(device)
        self.lists = {}        # (H_in, k, stride) -> [all-active list, sparse list]
        self.layers = {}
        self.graph = None
        # Optional observer for tests: hook(when, name, layer, tensors) is called with when = "pre" before
        # an operation's calls are issued, "stage" after each call inside an attention block (tensors
        # names what that call just wrote) and "post" after the operation's last call.  It may read and
        # overwrite buffers (after synchronising); the orchestration itself never looks at what it does.
        self.hook = None
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
            elif op["kind"] == "xfmr":
                b = min(block, r_in)
                assert r_in % b == 0, "token blocks must tile the map exactly"
                Cx, nc, dc = op["C"], op["n_ctx"], op["d_ctx"]
                lin = lambda part: SigeConv(P[f"{n}.{part}.w"].to(device), P[f"{n}.{part}.b"], r_in, r_in, b, 1, 0)
                for part in ("in", "o1", "q2", "o2", "ff2", "out"):
                    L[part] = lin(part)
                # the first feed-forward layer carries the gated GELU in its epilogue: values and gates
                # interleaved in groups of 8 (a row permutation of the weight, no arithmetic)
                rows = api.geglu_rows(4 * Cx)
                L["ff1"] = SigeConv(P[f"{n}.ff1.w"][rows].to(device), P[f"{n}.ff1.b"][rows], r_in, r_in, b, 1, 0)
                # self-attention: queries, keys and values from one convolution, into one cached tensor
                L["qkv1"] = SigeConv(torch.cat([P[f"{n}.{p}1.w"] for p in "qkv"], 0).to(device),
                                     torch.cat([P[f"{n}.{p}1.b"] for p in "qkv"], 0), r_in, r_in, b, 1, 0)
                # keys and values of the text embeddings: a 1 x n_ctx "image", one block
                L["kv2"] = SigeConv(torch.cat([P[f"{n}.k2.w"], P[f"{n}.v2.w"]], 0).to(device),
                                    torch.cat([P[f"{n}.k2.b"], P[f"{n}.v2.b"]], 0), 1, nc, (1, nc), 1, 0)
                L["ctx"] = P["ctx"].to(device).contiguous()
                L["kc"] = torch.zeros((nc, 2 * Cx), dtype=self.td, device=device)
                for part in ("ln1", "ln2", "ln3"):
                    L[part + ".g"], L[part + ".b"] = f32(P[f"{n}.{part}.gamma"]), f32(P[f"{n}.{part}.beta"])
                for name in ("h0", "h1", "h2", "h3"):
                    L[name] = torch.zeros((r_in, r_in, Cx), dtype=self.td, device=device)
                L["qkv"] = torch.zeros((r_in, r_in, 3 * Cx), dtype=self.td, device=device)
                L["g1"] = L["in"].g
                L["list"] = self._lists(r_in, 3, 1, b)
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
            if op["kind"] in ("attn", "xfmr") or op["gn"]:
                L["gamma"], L["beta"] = f32(P[n + ".gamma"]), f32(P[n + ".beta"])
                L["mean"] = torch.zeros(groups, device=device)
                L["var"] = torch.zeros(groups, device=device)
                L["scale"] = torch.zeros(C, device=device)
                L["shift"] = torch.zeros(C, device=device)
            self.layers[n] = L
        # Activated copies (Sec. 3.2 "Pre-computing normalization parameters": with cached statistics
        # the next layer's Scale+Shift is a constant per channel): the layer that produces a tensor
        # also writes act(scale * v + shift) for every layer that normalises it, so that those gather
        # a plain tensor.  Needs the fused call (its epilogue writes the copies).
        self.act_copies = bool(act_copies) and fused is True
        self._copies_valid = False
        if self.act_copies:
            self._plan_act_copies()

    def _plan_act_copies(self):
        order = list(self.layers.items())
        specs = {}
        for i, (n, L) in enumerate(order):
            op = L["op"]
            if "scale" not in L:
                continue
            bufname, off, C = op["x"]
            latest = [None] * C                    # the last layer before this one that writes each input channel
            for pn, PL in order[:i]:
                yv = PL["op"].get("y")
                if yv is None or yv[0] != bufname:
                    continue
                lo, hi = max(yv[1], off), min(yv[1] + yv[2], off + C)
                if lo >= hi:
                    continue
                assert (lo, hi) == (yv[1], yv[1] + yv[2]), "a producer's output lies wholly inside the normalised view"
                latest[lo - off:hi - off] = [pn] * (hi - lo)
            if any(p is None for p in latest):
                continue                           # fed from outside the network: stays fused into the gather
            H = self.bufs_shape[bufname][0]
            L["pre"] = torch.zeros((H, H, C), dtype=self.td, device=self.device)
            act = api.ACT_SILU if (op["kind"] == "conv" and op["act"]) else api.ACT_NONE
            for pn in dict.fromkeys(latest):
                yv = self.layers[pn]["op"]["y"]
                o = yv[1] - off
                specs.setdefault(pn, []).append((L["pre"][:, :, o:o + yv[2]], L["scale"][o:o + yv[2]],
                                                 L["shift"][o:o + yv[2]], act))
        for pn, spec in specs.items():
            assert len(spec) <= 3, (pn, len(spec))
            self.layers[pn]["act_spec"] = spec                 # keeps the views alive
            self.layers[pn]["act_outs"] = api.act_out_array(spec)

    def _fill_copy(self, L, x, scale, shift, act):
        """Dense pass: the activated copy of a whole tensor, once its statistics are known."""
        H, C = x.shape[0], x.shape[2]
        b = min(self.block, H)
        bl = self._lists(H, 1, 1, b)[0]
        n = bl.n_host
        t = self.ws.get("fill", n * b * b * C, self.td).view(n, b, b, C)
        api.sige_gather(x, bl.g, bl.indices, bl.count, t, n_blocks=n, scale=scale, shift=shift, act=act, C=C,
                        max_blocks=n)
        api.sige_scatter(t, bl.g, bl.indices, bl.count, L["pre"], n_blocks=n, Cout=C, max_blocks=n)

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

    def _run(self, image, dense: bool, fill_copies: bool = True):
        self.B["image"].copy_(image)
        shortcut_tiles = {}
        use_copies = self.act_copies and self.fused is True
        names = list(self.layers)
        paired = set()              # shortcut convolutions already issued together with their ResBlock's first one
        for i, n in enumerate(names):
            if n in paired:
                continue
            L = self.layers[n]
            op = L["op"]
            fused = self.fused is True or (self.fused == "lowres" and not L["sparse"])
            bl = L["list"][0 if (dense or not L["sparse"]) else 1]
            if self.hook:
                self.hook("pre", n, L, dict(dense=dense, blocks=bl))
            x = self.view(op["x"])
            xn = x                  # what the normalising layer gathers: x, or its activated copy
            scale = shift = None
            act = api.ACT_SILU if (op["kind"] == "conv" and op["act"]) else api.ACT_NONE
            if "scale" in L:
                scale, shift = L["scale"], L["shift"]
                if dense:   # statistics of the original activation, computed where a dense model would
                    api.sige_gn_stats(x, self.groups, L["mean"], L["var"], gamma=L["gamma"], beta=L["beta"],
                                      eps=self.eps, scale=scale, shift=shift, C=op["x"][2])
                if "pre" in L and use_copies and (fill_copies or not dense):
                    if dense:
                        self._fill_copy(L, x, scale, shift, act)
                    xn, scale, shift, act = L["pre"], None, None, api.ACT_NONE
            # the sparse pass keeps the copies of its output up to date; the dense pass fills them where
            # they are consumed (the statistics are not known before)
            ao = L.get("act_outs") if (use_copies and not dense) else None
            if op["kind"] == "conv":
                if not op["scatter"]:
                    shortcut_tiles[n] = L["conv"].forward(x, None, bl, self.ws, scatter=False, tag="short",
                                                          fused=fused)
                    if self.hook:
                        self.hook("post", n, L, dict(dense=dense, blocks=bl, tiles=shortcut_tiles[n]))
                    continue
                res_t = shortcut_tiles.get(op["shortcut"]) if op["shortcut"] else None
                res_f = self.view(op["residual"]) if op["residual"] is not None else None
                nxt = self.layers[names[i + 1]] if i + 1 < len(names) else None
                if (fused and self.fused is True and nxt is not None and nxt["op"]["kind"] == "conv" and
                        not nxt["op"]["scatter"] and nxt["op"]["x"] == op["x"] and op["k"] == 3 and
                        nxt["op"]["k"] == 1):
                    # a ResBlock's first convolution and its 1x1 shortcut read the same tensor: handed
                    # over together (one launch when both have few active blocks)
                    ca, _ = L["conv"].fused_call(xn, self.view(op["y"]), bl, self.ws, scale=scale, shift=shift,
                                                 act=act, residual_tiles=res_t, residual=res_f, tag="main",
                                                 act_outs=ao)
                    bls = nxt["list"][0 if (dense or not nxt["sparse"]) else 1]
                    cb, tiles = nxt["conv"].fused_call(x, None, bls, self.ws, scatter=False, tag="short")
                    api.sige_fused_conv_pair(ca, cb)
                    shortcut_tiles[names[i + 1]] = tiles
                    paired.add(names[i + 1])
                    if self.hook:
                        self.hook("post", n, L, dict(dense=dense, blocks=bl))
                        self.hook("post", names[i + 1], nxt, dict(dense=dense, blocks=bls, tiles=tiles))
                    continue
                L["conv"].forward(xn, self.view(op["y"]), bl, self.ws, scale=scale, shift=shift, act=act,
                                  residual_tiles=res_t, residual=res_f, tag="main", fused=fused, act_outs=ao)
            elif op["kind"] == "xfmr":
                self._transformer(L, x, xn, self.view(op["y"]), bl, dense, scale, shift, ao, name=n)
            else:
                C, heads = op["C"], op["heads"]
                T = x.shape[0] * x.shape[1]
                L["qkv"].forward(xn, L["qkv_buf"], bl, self.ws, scale=scale, shift=shift, tag="main",
                                 fused=fused)
                if self.hook:
                    self.hook("stage", n, L, dict(dense=dense, blocks=bl, qkv=L["qkv_buf"]))
                qkv = L["qkv_buf"].view(T, 3 * C)
                api.sige_sparse_attn(qkv[:, :C], qkv[:, C:2 * C], qkv[:, 2 * C:], L["att_buf"].view(T, C),
                                     1.0 / math.sqrt(C // heads), Nq=T, workspace=L["att_ws"], heads=heads,
                                     d=C // heads, q_ld=3 * C, kv_ld=3 * C, o_ld=C)
                if self.hook:
                    self.hook("stage", n, L, dict(dense=dense, blocks=bl, a=L["att_buf"]))
                L["proj"].forward(L["att_buf"], self.view(op["y"]), bl, self.ws, residual=x, tag="main",
                                  fused=fused, act_outs=ao)
            if self.hook:
                self.hook("post", n, L, dict(dense=dense, blocks=bl))
        if dense:
            self._copies_valid = use_copies and fill_copies
        elif not use_copies:
            self._copies_valid = False          # a pass that does not maintain them leaves them stale
        return self.B["out"]

    def _transformer(self, L, x, xn, y, bl, dense, scale, shift, act_outs=None, name=None):
        """A transformer block on the tokens of the active blocks (Fig. "sige-attention"): gather,
        token-wise layers and 1x1 convolutions on the stacked tiles, keys and values scattered into
        their caches, attention for the gathered queries only, result scattered back with the
        residual.  Needs the block count on the host (it sizes the attention call)."""
        op = L["op"]
        C, heads, g1, ws = op["C"], op["heads"], L["g1"], self.ws
        d = C // heads
        nb = bl.n_host
        assert nb >= 0, "transformer blocks need exact block counts (set_edit(exact=True))"
        if nb == 0:
            return
        idx, cnt = bl.indices, bl.count
        tpb = g1.block_h * g1.block_w
        rows, T = nb * tpb, g1.H_in * g1.W_in
        sm = 1.0 / math.sqrt(d)

        def tiles(tag, ch):
            return ws.get(tag, rows * ch, self.td).view(nb, g1.block_h, g1.block_w, ch)

        def conv(layer, src, tag):
            out = tiles(tag, layer.Cout)
            nbytes = api.sige_conv_workspace_bytes(self.td, layer.g, layer.Cin, layer.Cout, nb)
            split = ws.get("split_k", nbytes // 4, torch.float32) if nbytes else None
            api.sige_conv(src, layer.g, layer.Cin, layer.Cout, layer.packed, layer.bias, cnt, out, n_blocks=nb,
                          max_blocks=nb, workspace=split)
            return out

        def normed(src_full, part):      # gather with the token norm folded in
            tn = tiles("x_n", C)
            api.sige_gather_token_norm(src_full, g1, idx, cnt, tn, C, n_blocks=nb, max_blocks=nb,
                                       gamma=L[part + ".g"], beta=L[part + ".b"], eps=1e-5)
            return tn

        def attend(q, k, v, Tk, kv_ld, q_full=None):
            o = tiles("x_o", C)
            nbytes = api.sige_sparse_attn_workspace_bytes(rows, Tk, heads, d)
            aws = ws.get("attn_ws", nbytes // 4, torch.float32) if nbytes else None
            if q_full is not None:      # the queries of the active tokens, read from the cached tensor by block list
                api.sige_sparse_attn_blocks(q_full, g1, idx, nb, k, v, o.view(rows, C), sm, heads=heads, d=d,
                                            workspace=aws, q_ld=kv_ld, kv_ld=kv_ld, o_ld=C)
            else:
                api.sige_sparse_attn(q.view(rows, C), k, v, o.view(rows, C), sm, Nq=rows, workspace=aws,
                                     heads=heads, d=d, q_ld=C, kv_ld=kv_ld, o_ld=C)
            return o

        def back(layer, src, dst, residual=None):      # convolution with the scatter folded in
            nbytes = api.sige_conv_workspace_bytes(self.td, layer.g, layer.Cin, layer.Cout, nb)
            split = ws.get("split_k", nbytes // 4, torch.float32) if nbytes else None
            api.sige_conv_scatter(src, layer.g, idx, cnt, layer.Cin, layer.Cout, layer.packed, layer.bias, dst,
                                  n_blocks=nb, max_blocks=nb, residual=residual, workspace=split)

        def seen(**tensors):      # a call has just written these (tiles: stacked rows of the active blocks)
            if self.hook:
                self.hook("stage", name, L, dict(dense=dense, blocks=bl, **tensors))

        if dense:   # keys and values of the text embeddings do not depend on the image
            one = torch.ones(1, dtype=torch.int32, device=self.device)
            kv2 = L["kv2"]
            api.sige_conv(L["ctx"].view(1, 1, -1, kv2.Cin), kv2.g, kv2.Cin, kv2.Cout, kv2.packed, kv2.bias, one,
                          L["kc"].view(1, 1, -1, 2 * C), n_blocks=1, max_blocks=1)
            seen(kc=L["kc"])
        L["in"].forward(xn, L["h0"], bl, ws, scale=scale, shift=shift, fused=True)
        seen(h0=L["h0"])
        # self-attention: only the active tokens' queries; their queries, keys and values go into the
        # cache first, in one convolution
        tn = normed(L["h0"], "ln1")
        seen(tn1=tn)
        back(L["qkv1"], tn, L["qkv"])
        seen(qkv=L["qkv"])
        qkv = L["qkv"].view(T, 3 * C)
        o = attend(None, qkv[:, C:2 * C], qkv[:, 2 * C:], T, 3 * C, q_full=qkv)
        seen(a1=o)
        back(L["o1"], o, L["h1"], L["h0"])
        seen(h1=L["h1"])
        # cross-attention over the text embeddings
        tn = normed(L["h1"], "ln2")
        seen(tn2=tn)
        q = conv(L["q2"], tn, "x_q")
        seen(q2=q)
        o = attend(q, L["kc"][:, :C], L["kc"][:, C:], L["kc"].shape[0], 2 * C)
        seen(a2=o)
        back(L["o2"], o, L["h2"], L["h1"])
        seen(h2=L["h2"])
        # gated-GELU feed-forward
        tn = normed(L["h2"], "ln3")
        seen(tn3=tn)
        gg = tiles("x_g", 4 * C)
        api.sige_conv_geglu(tn, L["ff1"].g, C, 4 * C, L["ff1"].packed, L["ff1"].bias, cnt, gg, n_blocks=nb,
                            max_blocks=nb)
        seen(gg=gg)
        back(L["ff2"], gg, L["h3"], L["h2"])
        seen(h3=L["h3"])
        L["out"].forward(L["h3"], y, bl, ws, residual=x, fused=True, act_outs=act_outs)

    def precompute(self, image, fill_copies: bool = True):
        """Dense pass on the original image: fills every cache and the normalisation statistics (and,
        unless fill_copies is False - a plain dense model, for timing - the activated copies)."""
        return self._run(image, dense=True, fill_copies=fill_copies)

    def step(self, image_edit):
        """Sparse pass on the edited image (after set_edit): updates the caches in place."""
        assert not (self.act_copies and self.fused is True) or self._copies_valid, \
            "the activated copies are stale: run precompute(image) first"
        return self._run(image_edit, dense=False)

    def capture_dense(self, image):
        """Captures a plain dense pass (statistics on the fly, no copies) in a HIP graph, for timing."""
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            for _ in range(2):
                self.precompute(image, fill_copies=False)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.precompute(image, fill_copies=False)
        torch.cuda.synchronize()
        return g

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
            if op["kind"] == "attn":
                C, r = op["C"], self.bufs_shape[op["x"][0]][0]
                total += r * r * C * C * 4 + 2 * (r * r) ** 2 * C
                continue
            if op["kind"] == "xfmr":   # linear layers + both attention maps, on the active tokens only
                C, r, nc = op["C"], self.bufs_shape[op["x"][0]][0], op["n_ctx"]
                g1 = L["g1"]
                ntok = r * r
                if counts is not None and L["sparse"]:
                    ntok = counts[(g1.H_in, 3, 1)] * g1.block_h * g1.block_w
                total += ntok * C * C * (2 + 4 + 2 + 12) + 2 * ntok * (r * r) * C + 2 * ntok * nc * C
                continue
            c = L["conv"]
            g = c.g
            nblk = g.grid_blocks
            if counts is not None and L["sparse"]:
                kk = 3 if g.k == 1 else g.k
                nblk = counts[(g.H_in, kk, g.stride)]
            total += nblk * g.block_h * g.block_w * g.k * g.k * c.Cin * c.Cout
        return total
