"""Teacher-forced comparison of a network pass on the GPU with the step-by-step oracle.

The oracle's pass records every stored tensor (its `trace`).  The GPU pass then runs with an
observer that, before every operation, overwrites the GPU buffers with the ORACLE's state at that
point (values already rounded to the storage type, so the copy is exact), and after every library
call compares what the call wrote with the oracle's tensor element by element at the per-layer
tolerance (1e-4 fp32, 1e-2 fp16 / bf16, relative to max(|ref|, rms(ref))) and replaces it by the
oracle's.  No error is carried from one layer into the next, so every layer of the network - in
the kernel shape the network really selects for it - is held to the same bar as a single call.
Failures are collected and reported together.
"""
import numpy as np
import torch

from helpers import TOL, f64, round_to


def _dev(a64, dtype, like=None):
    t = torch.from_numpy(np.ascontiguousarray(a64)).to(dtype)
    return t.cuda() if like is None else t.to(like.device)


class Report:
    def __init__(self, dtype):
        self.dtype, self.tol = dtype, TOL[dtype]
        self.bad, self.n_checked, self.worst = [], 0, 0.0

    def check(self, what, got: torch.Tensor, want64: np.ndarray):
        ref = round_to(want64, self.dtype)
        g = f64(got)
        assert g.shape == ref.shape, (what, g.shape, ref.shape)
        self.n_checked += 1
        if ref.size == 0:
            return
        rms = float(np.sqrt(np.mean(ref * ref)))
        bound = self.tol * np.maximum(np.abs(ref), rms)
        err = np.abs(g - ref)
        ok = err <= bound
        ratio = float(np.nanmax(err / (bound + 1e-300))) if bound.max() > 0 else float(err.max() > 0)
        if not np.isfinite(g).all():
            ratio = float("inf")
        self.worst = max(self.worst, ratio)
        if not ok.all():
            self.bad.append((what, int((~ok).sum()), ref.size, ratio))

    def assert_clean(self, min_checked):
        assert self.n_checked >= min_checked, f"only {self.n_checked} tensors were compared"
        assert not self.bad, (f"{len(self.bad)} of {self.n_checked} teacher-forced tensors beyond {self.tol} "
                              f"(name, elements off, of, worst err / bound): {self.bad[:12]}")


def tiles_of(full64, blocks, bh, bw):
    """[n, bh, bw, C] stacked blocks of a full [H, W, C] tensor (blocks inside the map)."""
    return np.stack([full64[y0:y0 + bh, x0:x0 + bw] for y0, x0 in blocks]) if len(blocks) else \
        np.zeros((0, bh, bw, full64.shape[2]))


def block_rows(bl):
    n = bl.n_host if bl.n_host >= 0 else int(bl.count.item())
    return bl.indices[:n].cpu().numpy()


class UNetTeacher:
    """Drives SigeUNet.precompute / step under teacher forcing from an oracle trace."""

    def __init__(self, net, dtype, trace, start_state, stats=None, inner_cache=None):
        self.net, self.dtype, self.rep = net, dtype, Report(dtype)
        self.trace = dict(trace)
        assert len(self.trace) == len(trace)
        self.state = {n: a.copy() for n, a in start_state.items()}
        self.dirty = None
        self.stats = stats                # oracle's folded scale / shift per normalising op (edit pass)
        self.inner_cache = inner_cache    # oracle's caches inside the transformer blocks (edit pass)

    # -- forcing
    def _force_buffers(self):
        # only what the GPU pass has written since the last time (an operation writes its own output
        # buffer and nothing else), everything the first time
        for n in (self.dirty if self.dirty is not None else list(self.net.B)):
            if n in self.state:
                self.net.B[n].copy_(_dev(self.state[n], self.dtype))
        self.dirty = set()

    def prepare_edit(self, kc_from):
        """Before the edit pass: every cache the GPU pass reads takes the oracle's value."""
        net = self.net
        self._force_buffers()
        for n, L in net.layers.items():
            if "scale" in L and n in self.stats:
                sc, sh = self.stats[n]
                L["scale"].copy_(torch.from_numpy(sc).float())
                L["shift"].copy_(torch.from_numpy(sh).float())
            if L["op"]["kind"] == "xfmr":
                C = L["op"]["C"]
                for part in ("h0", "h1", "h2", "h3"):
                    L[part].copy_(_dev(self.inner_cache[f"{n}.{part}"], self.dtype))
                L["qkv"][:, :, C:].copy_(_dev(self.inner_cache[f"{n}.kv"], self.dtype))
                L["kc"].copy_(_dev(kc_from[n]["kc"], self.dtype))
        net._copies_valid = True
        torch.cuda.synchronize()

    # -- the observer
    def __call__(self, when, name, L, t):
        net, op = self.net, L["op"]
        torch.cuda.synchronize()
        rec = self.trace[name]
        bl = t["blocks"]
        if when == "pre":
            self._force_buffers()
            if not t["dense"] and "pre" in L and net.act_copies:
                from paper_2211_02048_amd import api
                act = api.ACT_SILU if (op["kind"] == "conv" and op["act"]) else api.ACT_NONE
                net._fill_copy(L, net.view(op["x"]), L["scale"], L["shift"], act)
            torch.cuda.synchronize()
            return
        g = bl.g
        blocks = block_rows(bl)
        if when == "stage":
            for key, ten in t.items():
                if key in ("dense", "blocks"):
                    continue
                if key == "qkv" and op["kind"] == "xfmr":
                    C = op["C"]
                    act = np.zeros(ten.shape[:2], bool)
                    for y0, x0 in blocks:
                        act[y0:y0 + g.block_h, x0:x0 + g.block_w] = True
                    a_t = torch.from_numpy(act).cuda()
                    self.rep.check(f"{name}.q1", ten[:, :, :C][a_t], rec["q1"][act])
                    self.rep.check(f"{name}.kv", ten[:, :, C:], rec["kv"])
                    ten[:, :, :C].copy_(_dev(rec["q1"], self.dtype))
                    ten[:, :, C:].copy_(_dev(rec["kv"], self.dtype))
                elif ten.dim() == 4:          # stacked tiles of the active blocks
                    want = tiles_of(rec[key], blocks, g.block_h, g.block_w)
                    self.rep.check(f"{name}.{key}", ten[:len(blocks)], want)
                    if len(blocks):
                        ten[:len(blocks)].copy_(_dev(want, self.dtype))
                else:
                    self.rep.check(f"{name}.{key}", ten, rec[key])
                    ten.copy_(_dev(rec[key], self.dtype))
            torch.cuda.synchronize()
            return
        # post
        if "tiles" in t:              # a shortcut branch: its tiles, against the full tensor the oracle computed
            n = len(blocks)
            Cout = L["conv"].Cout
            got = t["tiles"][:n * g.block_h * g.block_w * Cout].view(n, g.block_h, g.block_w, Cout)
            full = rec["short"]
            H, W = full.shape[:2]
            want = np.zeros((n, g.block_h, g.block_w, Cout))
            valid = np.zeros((n, g.block_h, g.block_w), bool)
            for i, (y0, x0) in enumerate(blocks):
                hh, ww = min(g.block_h, H - y0), min(g.block_w, W - x0)
                want[i, :hh, :ww] = full[y0:y0 + hh, x0:x0 + ww]
                valid[i, :hh, :ww] = True
            v_t = torch.from_numpy(valid).cuda()
            self.rep.check(f"{name} (tiles)", got[v_t], want[valid])
            if n:
                got[v_t] = _dev(want[valid], self.dtype)
            torch.cuda.synchronize()
            return
        bufname, off, C = op["y"]
        self.rep.check(name, net.B[bufname][:, :, off:off + C], rec["y"][:, :, off:off + C])
        self.state[bufname] = rec["y"]
        self.dirty.add(bufname)


class SpadeTeacher:
    """The same for SigeSpade.precompute / step."""

    def __init__(self, net, dtype, trace, start_state, stats=None):
        self.net, self.dtype, self.rep = net, dtype, Report(dtype)
        self.trace = dict(trace)
        self.state = {n: a.copy() for n, a in start_state.items()}
        self.stats = stats
        self.dirty = None

    def _force_buffers(self):
        # only what the GPU pass has written since the last time (an operation writes its own output
        # buffer and nothing else), everything the first time
        for n in (self.dirty if self.dirty is not None else list(self.net.B)):
            if n in self.state:
                self.net.B[n].copy_(_dev(self.state[n], self.dtype))
        self.dirty = set()

    def __call__(self, when, name, L, t):
        net, op = self.net, L["op"]
        torch.cuda.synchronize()
        if when == "pre":
            self._force_buffers()
            if not t["dense"] and self.stats is not None and op.get("spade") and op["spade"]["cached"]:
                sc, sh = self.stats[name]
                L["scale"].copy_(torch.from_numpy(sc).float())
                L["shift"].copy_(torch.from_numpy(sh).float())
            torch.cuda.synchronize()
            return
        bl = t["blocks"]
        g = bl.g
        blocks = block_rows(bl)
        if "tiles" in t:
            rec = self.trace[name]
            n = len(blocks)
            Cout = L["conv"].Cout
            got = t["tiles"][:n * g.block_h * g.block_w * Cout].view(n, g.block_h, g.block_w, Cout)
            full = rec["short"]
            H, W = full.shape[:2]
            want = np.zeros((n, g.block_h, g.block_w, Cout))
            valid = np.zeros((n, g.block_h, g.block_w), bool)
            for i, (y0, x0) in enumerate(blocks):
                hh, ww = min(g.block_h, H - y0), min(g.block_w, W - x0)
                want[i, :hh, :ww] = full[y0:y0 + hh, x0:x0 + ww]
                valid[i, :hh, :ww] = True
            v_t = torch.from_numpy(valid).cuda()
            self.rep.check(f"{name} (tiles)", got[v_t], want[valid])
            if n:
                got[v_t] = _dev(want[valid], self.dtype)
            torch.cuda.synchronize()
            return
        # an operation that stands for several (the joint label-map convolution of a residual block)
        names = [name]
        if "joint" in L:
            blk, hw = name.split(".")[0], op["hw"]
            names = [m for m, M in net.layers.items() if m.endswith(".shared") and m.split(".")[0] == blk and
                     M["op"]["hw"] == hw]
        for m in names:
            y = net.layers[m]["op"]["y"]
            self.rep.check(m, net.B[y], self.trace[m]["y"])
            self.state[y] = self.trace[m]["y"]
            self.dirty.add(y)
