"""Thin ctypes binding of libsige_hip.so: the same entry points as include/sige.h.

Argument marshalling only.  Tensors are torch CUDA tensors used purely as device
memory; every call enqueues on torch's current stream and returns at once.  There
is no fallback: if the library has not been built, or a call is refused, a
:class:`SigeError` is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsige_hip.so")

SIGE_F32, SIGE_F16, SIGE_BF16 = 0, 1, 2
ACT_NONE, ACT_SILU, ACT_RELU, ACT_LEAKY_RELU = 0, 1, 2, 3
_DT = {torch.float32: SIGE_F32, torch.float16: SIGE_F16, torch.bfloat16: SIGE_BF16}
STATUS = {0: "SIGE_OK", 1: "SIGE_ERR_INVALID_ARG", 2: "SIGE_ERR_UNSUPPORTED", 3: "SIGE_ERR_CAPACITY",
          4: "SIGE_ERR_HIP"}

EXPORTS = ["sige_reduce_mask", "sige_reduce_mask_workspace_bytes", "sige_reduce_mask_lists", "sige_gather", "sige_gather_modulated", "sige_conv", "sige_conv_workspace_bytes", "sige_conv_geglu", "sige_conv_scatter", "sige_scatter", "sige_fused_conv", "sige_fused_conv_pair", "sige_sparse_attn", "sige_sparse_attn_blocks",
           "sige_sparse_attn_workspace_bytes", "sige_token_norm", "sige_gather_token_norm", "sige_geglu", "sige_packed_weight_bytes", "sige_pack_weight",
           "sige_gn_stats", "sige_last_error", "sige_version", "sige_set_knob", "sige_get_knob", "sige_conv_plan", "sige_reduce_mask_noalloc", "sige_mark_blocks",
           "sige_fused_conv_pair_marked"]

# sige_knob of the header
KNOBS = {"CONV_CFG": 0, "CONV_KC": 1, "CONV_SPLIT": 2, "CONV_HALF": 3, "CONV_SPLIT_WGS": 4, "CONV_POINTWISE": 5,
         "CONV_POINTWISE_W4": 6, "CONV_PAIR_WGS": 7, "ATTN_WGS": 8, "DIFF_LOADS": 9, "DIFF_WGS": 10, "CONV_LDS_PAD": 12,
         "CONV_DIRECT": 11}


class SigeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


class Geom(ctypes.Structure):
    """Mirror of sige_geom."""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("H_in", "W_in", "H_out", "W_out", "block_h", "block_w", "k", "stride", "pad")]

    @property
    def tile_h(self):
        return (self.block_h - 1) * self.stride + self.k

    @property
    def tile_w(self):
        return (self.block_w - 1) * self.stride + self.k

    @property
    def grid_blocks(self):
        return -(-self.H_out // self.block_h) * -(-self.W_out // self.block_w)


class BlockListDesc(ctypes.Structure):
    """Mirror of sige_block_list."""
    _fields_ = [("g", Geom), ("indices", ctypes.c_void_p), ("max_blocks", ctypes.c_int32),
                ("count", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


class ConvPlanInfo(ctypes.Structure):
    """Mirror of sige_conv_plan_info."""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("kernel", "shape", "patch_m", "patch_n", "k_steps_per_chunk", "ksplit", "workgroups", "threads",
                 "lds_bytes")]

    def __repr__(self):
        kind = "few-row 1x1" if self.kernel else "tiled"
        return (f"{kind} kernel, shape {self.shape} ({self.patch_m}x{self.patch_n}), {self.k_steps_per_chunk} K steps "
                f"per chunk, ksplit {self.ksplit}, {self.workgroups} workgroups of {self.threads}, {self.lds_bytes} B LDS")


def geom(H_in, W_in, block, k=3, stride=1, pad=None) -> Geom:
    pad = k // 2 if pad is None else pad
    bh, bw = (block, block) if isinstance(block, int) else block
    return Geom(H_in, W_in, (H_in + 2 * pad - k) // stride + 1, (W_in + 2 * pad - k) // stride + 1,
                bh, bw, k, stride, pad)


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the HIP library; raises if it has not been built (no CPU fallback)."""
    global _lib
    if _recording is not None:
        return _recording
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SigeError(-1, f"{LIB_PATH} is missing: run `python -m paper_2211_02048_amd.build` "
                                "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(LIB_PATH)
        L.sige_last_error.restype = ctypes.c_char_p
        L.sige_packed_weight_bytes.restype = ctypes.c_size_t
        L.sige_sparse_attn_workspace_bytes.restype = ctypes.c_size_t
        vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        gp = ctypes.POINTER(Geom)
        L.sige_reduce_mask.argtypes = [vp, vp, i32, i32, i32, i32, f32, vp, i32, i32, gp, vp, vp, i32, vp, vp, sz,
                                       vp]
        L.sige_reduce_mask_noalloc.argtypes = [vp, vp, i32, i32, i32, i32, f32, vp, i32, i32, gp, vp, vp, i32, vp, vp]
        L.sige_reduce_mask_lists.argtypes = [vp, vp, i32, i32, i32, i32, f32, vp, i32, i32,
                                             ctypes.POINTER(BlockListDesc), i32, vp, vp]
        L.sige_mark_blocks.argtypes = L.sige_reduce_mask_lists.argtypes
        L.sige_reduce_mask_workspace_bytes.restype = ctypes.c_size_t
        L.sige_reduce_mask_workspace_bytes.argtypes = [gp]
        L.sige_gather.argtypes = [vp, i32, i32, i32, i32, gp, vp, vp, i32, i32, vp, vp, i32, vp, vp]
        L.sige_gather_modulated.argtypes = [vp, i32, i32, i32, i32, gp, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp, vp]
        L.sige_conv.argtypes = [vp, i32, gp, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp]
        L.sige_conv_geglu.argtypes = [vp, i32, gp, i32, i32, vp, vp, vp, i32, i32, vp, vp]
        L.sige_conv_scatter.argtypes = [vp, i32, gp, i32, i32, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp, i32, vp, sz, vp]
        L.sige_conv_workspace_bytes.restype = ctypes.c_size_t
        L.sige_conv_workspace_bytes.argtypes = [i32, gp, i32, i32, i32]
        L.sige_fused_conv.argtypes = [vp, i32, i32, i32, i32, gp, vp, vp, i32, i32, vp, vp, i32, i32, vp, vp, vp, vp,
                                      i32, vp, i32, vp, vp, i32, vp, sz, vp]
        L.sige_fused_conv_pair.argtypes = [ctypes.POINTER(FusedConvCall), ctypes.POINTER(FusedConvCall), vp]
        L.sige_fused_conv_pair_marked.argtypes = [ctypes.POINTER(FusedConvCall), ctypes.POINTER(FusedConvCall),
                                                  ctypes.POINTER(BlockListDesc), vp]
        L.sige_scatter.argtypes = [vp, i32, gp, i32, vp, vp, i32, i32, vp, vp, i32, vp, i32, vp]
        L.sige_sparse_attn.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp, i32, vp, sz, vp]
        L.sige_sparse_attn_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.sige_sparse_attn_blocks.argtypes = [vp, i32, gp, vp, i32, vp, vp, i32, i32, i32, i32, i32, f32, vp, i32, vp, sz, vp]
        L.sige_packed_weight_bytes.argtypes = [i32, i32, i32, i32]
        L.sige_pack_weight.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        L.sige_token_norm.argtypes = [vp, i32, i32, i32, vp, i32, i32, i32, vp, vp, f32, vp, i32, vp]
        L.sige_gather_token_norm.argtypes = [vp, i32, i32, i32, gp, vp, vp, i32, i32, vp, vp, f32, vp, vp]
        L.sige_geglu.argtypes = [vp, i32, i32, i32, vp, i32, i32, i32, vp, i32, vp]
        L.sige_gn_stats.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, f32, vp, vp, vp, vp, vp]
        L.sige_conv_plan.argtypes = [i32, gp, i32, i32, i32, i32, i32, sz, ctypes.POINTER(ConvPlanInfo)]
        L.sige_set_knob.argtypes = [i32, i32]
        L.sige_get_knob.argtypes = [i32]
        L.sige_get_knob.restype = i32
        _lib = L
    return _lib


# ---- prepared calls ---------------------------------------------------------------------------------
# A step that is a few kernels of a few microseconds each is bound by what the host does per launch.
# `record()` runs a piece of code once and keeps every library call it made together with its marshalled
# arguments; `CallList.run()` then repeats exactly those calls (same pointers, same sizes, same stream)
# without building the arguments again.  Marshalling only: each run still goes through the C entry
# points, which validate, plan and launch as always.
_QUERIES = ("sige_last_error", "sige_packed_weight_bytes", "sige_sparse_attn_workspace_bytes",
            "sige_reduce_mask_workspace_bytes", "sige_conv_workspace_bytes", "sige_conv_plan", "sige_set_knob",
            "sige_get_knob")


class CallList:
    """Library calls recorded by `record()`.  The tensors they name must outlive the list; the calls run
    on the stream that was current while they were recorded."""

    def __init__(self):
        self.calls = []

    def run(self):
        for fn, args in self.calls:
            rc = fn(*args)
            if rc != 0:
                _check(rc)

    def __len__(self):
        return len(self.calls)


class _RecordingLib:
    def __init__(self, real, calls):
        self._real, self._calls = real, calls

    def __getattr__(self, name):
        fn = getattr(self._real, name)
        if not name.startswith("sige_") or name in _QUERIES:
            return fn

        def call(*args):
            self._calls.append((fn, args))
            return fn(*args)
        return call


_recording = None


class record:
    """with api.record() as calls: ...   (the calls are made as usual and kept in `calls`)"""

    def __enter__(self):
        global _recording
        assert _recording is None, "api.record() does not nest"
        self.list = CallList()
        _recording = _RecordingLib(lib(), self.list.calls)
        return self.list

    def __exit__(self, *exc):
        global _recording
        _recording = None
        return False


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int):
    if rc != 0:
        raise SigeError(rc, lib().sige_last_error().decode())


def sige_reduce_mask_workspace_bytes(g: Geom) -> int:
    return int(lib().sige_reduce_mask_workspace_bytes(ctypes.byref(g)))


def sige_reduce_mask(g: Geom, indices, count, *, a_orig=None, a_edit=None, tau=0.0, mask_in=None,
                     mask_out=None, pool_log2=0, dilate=0, max_blocks=None, workspace=None):
    """Difference mask -> pooled, dilated mask -> ordered active-block list (device)."""
    if a_orig is not None:
        Hm, Wm, C = a_orig.shape
        dt = _DT[a_orig.dtype]
    else:
        Hm, Wm = mask_in.shape
        C, dt = 0, SIGE_F32
    mb = (indices.shape[0] if indices is not None else 0) if max_blocks is None else max_blocks
    _check(lib().sige_reduce_mask(_ptr(a_orig), _ptr(a_edit), dt, Hm, Wm, C, tau, _ptr(mask_in), pool_log2,
                                  dilate, ctypes.byref(g), _ptr(mask_out), _ptr(indices), mb, _ptr(count),
                                  _ptr(workspace), 0 if workspace is None else workspace.numel() *
                                  workspace.element_size(), _stream()))


NOALLOC_MAX_BLOCKS = 65536


def sige_reduce_mask_noalloc(g: Geom, indices, count, *, a_orig=None, a_edit=None, tau=0.0, mask_in=None,
                             mask_out=None, pool_log2=0, dilate=0, max_blocks=None):
    """sige_reduce_mask with the block flags in the library's built-in scratch: allocates nothing."""
    if a_orig is not None:
        Hm, Wm, C = a_orig.shape
        dt = _DT[a_orig.dtype]
    else:
        Hm, Wm = mask_in.shape
        C, dt = 0, SIGE_F32
    mb = indices.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_reduce_mask_noalloc(_ptr(a_orig), _ptr(a_edit), dt, Hm, Wm, C, tau, _ptr(mask_in), pool_log2,
                                          dilate, ctypes.byref(g), _ptr(mask_out), _ptr(indices), mb, _ptr(count),
                                          _stream()))


def sige_reduce_mask_lists(lists, *, a_orig=None, a_edit=None, tau=0.0, mask_in=None, mask_out=None,
                           pool_log2=0, dilate=0, mark_only=False):
    """One mask, several layer geometries: lists = [(g, indices, count, max_blocks, workspace), ...]."""
    if a_orig is not None:
        Hm, Wm, C = a_orig.shape
        dt = _DT[a_orig.dtype]
    else:
        Hm, Wm = mask_in.shape
        C, dt = 0, SIGE_F32
    arr = block_list_array(lists)
    fn = lib().sige_mark_blocks if mark_only else lib().sige_reduce_mask_lists
    _check(fn(_ptr(a_orig), _ptr(a_edit), dt, Hm, Wm, C, tau, _ptr(mask_in), pool_log2, dilate, arr, len(lists),
              _ptr(mask_out), _stream()))


def sige_mark_blocks(lists, **kw):
    """The first half of sige_reduce_mask_lists: mask and per-block flags, no lists (sige_fused_conv_pair_marked
    builds them)."""
    sige_reduce_mask_lists(lists, mark_only=True, **kw)


def block_list_array(lists):
    """[(g, indices, count, max_blocks, workspace), ...] as a host array of sige_block_list."""
    arr = (BlockListDesc * max(len(lists), 1))()
    for d, (g, indices, count, mb, ws) in zip(arr, lists):
        d.g = g
        d.indices, d.count = indices.data_ptr(), count.data_ptr()
        d.max_blocks = indices.shape[0] if mb is None else mb
        d.workspace = None if ws is None else ws.data_ptr()
        d.workspace_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    arr._keep = lists
    return arr


def sige_gather(x, g: Geom, indices, count, tiles, *, n_blocks=-1, scale=None, shift=None, act=ACT_NONE,
                up=0, C=None, x_ld=None, max_blocks=None):
    """tiles[n] = act(scale * x[tile n] + shift), zero outside the image."""
    C = x.shape[-1] if C is None else C
    x_ld = x.stride(-2) if x_ld is None else x_ld
    mb = tiles.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_gather(_ptr(x), _DT[x.dtype], C, x_ld, up, ctypes.byref(g), _ptr(indices), _ptr(count),
                             mb, n_blocks, _ptr(scale), _ptr(shift), act, _ptr(tiles), _stream()))


def sige_gather_modulated(x, g: Geom, indices, count, tiles, mod, *, n_blocks=-1, scale=None, shift=None,
                          act=ACT_NONE, up=0, C=None, x_ld=None, mod_ld=None, max_blocks=None):
    """tiles[n] = act((scale * x + shift) * (1 + gamma) + beta) with per-pixel gamma | beta in mod [H, W, >=2C]."""
    C = x.shape[-1] if C is None else C
    x_ld = x.stride(-2) if x_ld is None else x_ld
    mod_ld = mod.stride(-2) if mod_ld is None else mod_ld
    mb = tiles.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_gather_modulated(_ptr(x), _DT[x.dtype], C, x_ld, up, ctypes.byref(g), _ptr(indices), _ptr(count),
                                       mb, n_blocks, _ptr(scale), _ptr(shift), _ptr(mod), mod_ld, act, _ptr(tiles),
                                       _stream()))


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def sige_conv_workspace_bytes(dtype, g: Geom, Cin, Cout, max_blocks) -> int:
    return int(lib().sige_conv_workspace_bytes(_DT[dtype], ctypes.byref(g), Cin, Cout, max_blocks))


def sige_conv_plan(dtype, g: Geom, Cin, Cout, n_blocks, *, staged_math=False, up=0, workspace_bytes=0) -> ConvPlanInfo:
    """Which kernel and launch shape a convolution call with these arguments would take (host only)."""
    info = ConvPlanInfo()
    _check(lib().sige_conv_plan(_DT[dtype], ctypes.byref(g), Cin, Cout, n_blocks, int(bool(staged_math)), up,
                                workspace_bytes, ctypes.byref(info)))
    return info


def sige_conv(tiles, g: Geom, Cin, Cout, packed_weight, bias, count, out_tiles, *, n_blocks=-1,
              max_blocks=None, workspace=None):
    """out_tiles[n] = valid conv of tiles[n] with the packed weight, plus bias."""
    mb = tiles.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_conv(_ptr(tiles), _DT[tiles.dtype], ctypes.byref(g), Cin, Cout, _ptr(packed_weight),
                           _ptr(bias), _ptr(count), mb, n_blocks, _ptr(out_tiles), _ptr(workspace),
                           _nbytes(workspace), _stream()))


def geglu_rows(n_out: int) -> torch.Tensor:
    """Row order sige_conv_geglu expects of a [2*n_out, ...] weight / bias whose first n_out rows are the
    values and whose last n_out rows are the gates: groups of 8 values followed by their 8 gates."""
    j = torch.arange(n_out).view(-1, 8)
    return torch.cat([j, j + n_out], dim=1).reshape(-1)


def sige_conv_geglu(tiles, g: Geom, Cin, Cout, packed_weight, bias, count, out_tiles, *, n_blocks=-1,
                    max_blocks=None):
    """out_tiles[n] = value * gelu(gate) of the 2*Cout-channel convolution of tiles[n] (weight rows in
    geglu_rows order)."""
    mb = tiles.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_conv_geglu(_ptr(tiles), _DT[tiles.dtype], ctypes.byref(g), Cin, Cout, _ptr(packed_weight),
                                 _ptr(bias), _ptr(count), mb, n_blocks, _ptr(out_tiles), _stream()))


def sige_conv_scatter(tiles, g: Geom, indices, count, Cin, Cout, packed_weight, bias, y, *, n_blocks=-1,
                      max_blocks=None, residual_tiles=None, residual=None, res_ld=None, y_ld=None, workspace=None):
    """conv on stacked tiles -> scatter in one call: y[block n] = conv(tiles[n]) (+ residuals), in place."""
    y_ld = y.stride(-2) if y_ld is None else y_ld
    if residual is not None and res_ld is None:
        res_ld = residual.stride(-2)
    mb = tiles.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_conv_scatter(_ptr(tiles), _DT[tiles.dtype], ctypes.byref(g), Cin, Cout, _ptr(packed_weight),
                                   _ptr(bias), _ptr(indices), _ptr(count), mb, n_blocks, _ptr(residual_tiles),
                                   _ptr(residual), res_ld or 0, _ptr(y), y_ld, _ptr(workspace), _nbytes(workspace),
                                   _stream()))


def sige_scatter(out_tiles, g: Geom, indices, count, y, *, n_blocks=-1, residual_tiles=None, residual=None,
                 Cout=None, y_ld=None, res_ld=None, max_blocks=None):
    """y[block n] = out_tiles[n] (+ residual_tiles[n]) (+ residual[block n]); y is updated in place."""
    Cout = out_tiles.shape[-1] if Cout is None else Cout
    y_ld = y.stride(-2) if y_ld is None else y_ld
    if residual is not None and res_ld is None:
        res_ld = residual.stride(-2)
    mb = out_tiles.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_scatter(_ptr(out_tiles), _DT[out_tiles.dtype], ctypes.byref(g), Cout, _ptr(indices),
                              _ptr(count), mb, n_blocks, _ptr(residual_tiles), _ptr(residual), res_ld or 0,
                              _ptr(y), y_ld, _stream()))


class ActOut(ctypes.Structure):
    """Mirror of sige_act_out."""
    _fields_ = [("y", ctypes.c_void_p), ("y_ld", ctypes.c_int32), ("scale", ctypes.c_void_p),
                ("shift", ctypes.c_void_p), ("act", ctypes.c_int32)]


class FusedConvCall(ctypes.Structure):
    """The arguments of one sige_fused_conv call (sige_fused_conv_call in the header)."""
    _fields_ = [("x", ctypes.c_void_p), ("dt", ctypes.c_int32), ("Cin", ctypes.c_int32), ("x_ld", ctypes.c_int32),
                ("up", ctypes.c_int32), ("g", ctypes.POINTER(Geom)), ("indices", ctypes.c_void_p),
                ("count", ctypes.c_void_p), ("max_blocks", ctypes.c_int32), ("n_blocks", ctypes.c_int32),
                ("scale", ctypes.c_void_p), ("shift", ctypes.c_void_p), ("act", ctypes.c_int32),
                ("Cout", ctypes.c_int32), ("packed_weight", ctypes.c_void_p), ("bias", ctypes.c_void_p),
                ("residual_tiles", ctypes.c_void_p), ("residual", ctypes.c_void_p), ("res_ld", ctypes.c_int32),
                ("y", ctypes.c_void_p), ("y_ld", ctypes.c_int32), ("out_tiles", ctypes.c_void_p),
                ("act_outs", ctypes.c_void_p), ("n_act_outs", ctypes.c_int32), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t)]


def act_out_array(act_outs):
    """[(y, scale, shift, act), ...] (device tensors; y a [H, W, >=Cout] view) -> a ctypes array of sige_act_out."""
    arr = (ActOut * len(act_outs))()
    for a, (y, scale, shift, act) in zip(arr, act_outs):
        a.y, a.y_ld, a.scale, a.shift, a.act = _ptr(y), y.stride(-2), _ptr(scale), _ptr(shift), act
    return arr


def sige_fused_conv(x, g: Geom, indices, count, Cin, Cout, packed_weight, bias, *, y=None, out_tiles=None,
                    n_blocks=-1, max_blocks=None, scale=None, shift=None, act=ACT_NONE, up=0, x_ld=None,
                    residual_tiles=None, residual=None, res_ld=None, y_ld=None, workspace=None, act_outs=None):
    """gather -> conv -> scatter in one kernel; y is updated in place (or out_tiles receives the tiles).
    act_outs: [(y, scale, shift, act), ...] or a prepared act_out_array - activated copies of the output."""
    if act_outs is not None and not isinstance(act_outs, ctypes.Array):
        act_outs = act_out_array(act_outs)
    n_ao = 0 if act_outs is None else len(act_outs)
    x_ld = x.stride(-2) if x_ld is None else x_ld
    if y is not None and y_ld is None:
        y_ld = y.stride(-2)
    if residual is not None and res_ld is None:
        res_ld = residual.stride(-2)
    mb = indices.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_fused_conv(_ptr(x), _DT[x.dtype], Cin, x_ld, up, ctypes.byref(g), _ptr(indices), _ptr(count),
                                 mb, n_blocks, _ptr(scale), _ptr(shift), act, Cout, _ptr(packed_weight), _ptr(bias),
                                 _ptr(residual_tiles), _ptr(residual), res_ld or 0, _ptr(y), y_ld or 0,
                                 _ptr(out_tiles), act_outs if n_ao else None, n_ao, _ptr(workspace),
                                 _nbytes(workspace), _stream()))


def fused_conv_call(x, g: Geom, indices, count, Cin, Cout, packed_weight, bias, *, y=None, out_tiles=None,
                    n_blocks=-1, max_blocks=None, scale=None, shift=None, act=ACT_NONE, up=0, x_ld=None,
                    residual_tiles=None, residual=None, res_ld=None, y_ld=None, workspace=None, act_outs=None):
    """The arguments of sige_fused_conv as a FusedConvCall (keeps the tensors alive alongside)."""
    if act_outs is not None and not isinstance(act_outs, ctypes.Array):
        act_outs = act_out_array(act_outs)
    n_ao = 0 if act_outs is None else len(act_outs)
    if y is not None and y_ld is None:
        y_ld = y.stride(-2)
    if residual is not None and res_ld is None:
        res_ld = residual.stride(-2)
    p = lambda t: None if t is None else t.data_ptr()
    c = FusedConvCall(p(x), _DT[x.dtype], Cin, x.stride(-2) if x_ld is None else x_ld, up, ctypes.pointer(g),
                      p(indices), p(count), indices.shape[0] if max_blocks is None else max_blocks, n_blocks,
                      p(scale), p(shift), act, Cout, p(packed_weight), p(bias), p(residual_tiles), p(residual),
                      res_ld or 0, p(y), y_ld or 0, p(out_tiles),
                      ctypes.cast(act_outs, ctypes.c_void_p) if n_ao else None, n_ao, p(workspace),
                      _nbytes(workspace))
    c._keep = (x, g, indices, count, scale, shift, packed_weight, bias, residual_tiles, residual, y, out_tiles,
               act_outs, workspace)
    return c


def sige_fused_conv_pair(first: FusedConvCall, second: FusedConvCall):
    """Two independent fused calls; one launch when both take the few-block kernel shape."""
    _check(lib().sige_fused_conv_pair(ctypes.byref(first), ctypes.byref(second), _stream()))


def sige_fused_conv_pair_marked(first: FusedConvCall, second: FusedConvCall, marked):
    """sige_fused_conv_pair on lists that sige_mark_blocks left marked (marked: the two lists as for
    sige_reduce_mask_lists); the launch builds the ordered lists itself when it can."""
    arr = marked if isinstance(marked, ctypes.Array) else block_list_array(marked)
    _check(lib().sige_fused_conv_pair_marked(ctypes.byref(first), ctypes.byref(second), arr, _stream()))


def sige_token_norm(x, y, C, *, n_rows=-1, count=None, rows_per_count=0, max_rows=None, gamma=None, beta=None,
                    eps=1e-5, x_ld=None, y_ld=None):
    """y[r] = layer_norm(x[r]) * gamma + beta for the token rows of stacked tiles (x, y: [rows, >=C])."""
    x2, y2 = x.reshape(-1, x.shape[-1]), y.reshape(-1, y.shape[-1])
    mr = x2.shape[0] if max_rows is None else max_rows
    _check(lib().sige_token_norm(_ptr(x), _DT[x.dtype], C, x2.stride(0) if x_ld is None else x_ld, _ptr(count),
                                 rows_per_count, mr, n_rows, _ptr(gamma), _ptr(beta), eps, _ptr(y),
                                 y2.stride(0) if y_ld is None else y_ld, _stream()))


def sige_gather_token_norm(x, g: Geom, indices, count, tiles, C, *, n_blocks=-1, max_blocks=None, gamma=None,
                           beta=None, eps=1e-5, x_ld=None):
    """tiles[n] = layer_norm over the channels of every pixel of block n of x (gather and token norm in one)."""
    mb = tiles.shape[0] if max_blocks is None else max_blocks
    _check(lib().sige_gather_token_norm(_ptr(x), _DT[x.dtype], C, x.stride(-2) if x_ld is None else x_ld,
                                        ctypes.byref(g), _ptr(indices), _ptr(count), mb, n_blocks, _ptr(gamma),
                                        _ptr(beta), eps, _ptr(tiles), _stream()))


def sige_geglu(x, y, C, *, n_rows=-1, count=None, rows_per_count=0, max_rows=None, x_ld=None, y_ld=None):
    """y[r, c] = x[r, c] * gelu(x[r, C + c]) for the token rows of stacked tiles."""
    x2, y2 = x.reshape(-1, x.shape[-1]), y.reshape(-1, y.shape[-1])
    mr = x2.shape[0] if max_rows is None else max_rows
    _check(lib().sige_geglu(_ptr(x), _DT[x.dtype], C, x2.stride(0) if x_ld is None else x_ld, _ptr(count),
                            rows_per_count, mr, n_rows, _ptr(y), y2.stride(0) if y_ld is None else y_ld, _stream()))


def sige_sparse_attn_workspace_bytes(Nq, T, heads, d) -> int:
    return int(lib().sige_sparse_attn_workspace_bytes(Nq, T, heads, d))


def sige_sparse_attn(q, k, v, o, scale, *, Nq=None, workspace=None, heads=None, d=None, q_ld=None,
                     kv_ld=None, o_ld=None):
    """o[i, h] = softmax(scale * q[i, h] . k[:, h]) v[:, h] for the Nq edited query tokens."""
    heads = q.shape[1] if heads is None else heads
    d = q.shape[2] if d is None else d
    Nq = q.shape[0] if Nq is None else Nq
    T = k.shape[0]
    q_ld = q.stride(0) if q_ld is None else q_ld
    kv_ld = k.stride(0) if kv_ld is None else kv_ld
    o_ld = o.stride(0) if o_ld is None else o_ld
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sige_sparse_attn(_ptr(q), q_ld, _ptr(k), _ptr(v), kv_ld, _DT[q.dtype], Nq, T, heads, d,
                                  scale, _ptr(o), o_ld, _ptr(workspace), wsb, _stream()))


def sige_sparse_attn_blocks(q_full, g: Geom, indices, n_blocks, k, v, o, scale, *, heads, d, workspace=None,
                            q_ld=None, kv_ld=None, o_ld=None):
    """The same with the queries read from a full tensor by block list: query i is pixel
    i % (block_h*block_w) of block i / (block_h*block_w); o holds the stacked rows."""
    T = k.shape[0]
    q_ld = q_full.stride(-2) if q_ld is None else q_ld
    kv_ld = k.stride(0) if kv_ld is None else kv_ld
    o_ld = o.stride(0) if o_ld is None else o_ld
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sige_sparse_attn_blocks(_ptr(q_full), q_ld, ctypes.byref(g), _ptr(indices), n_blocks, _ptr(k),
                                         _ptr(v), kv_ld, _DT[q_full.dtype], T, heads, d, scale, _ptr(o), o_ld,
                                         _ptr(workspace), wsb, _stream()))


def sige_packed_weight_bytes(dtype, Cout, Cin, k) -> int:
    return int(lib().sige_packed_weight_bytes(_DT[dtype], Cout, Cin, k))


def sige_pack_weight(w_oihw):
    """Returns the weight re-laid for sige_conv (a new device buffer owned by the caller)."""
    Cout, Cin, k, _ = w_oihw.shape
    nbytes = sige_packed_weight_bytes(w_oihw.dtype, Cout, Cin, k)
    if nbytes == 0:
        raise SigeError(2, f"sige_pack_weight: unsupported shape {tuple(w_oihw.shape)} for {w_oihw.dtype}")
    packed = torch.empty(nbytes // w_oihw.element_size(), dtype=w_oihw.dtype, device=w_oihw.device)
    w = w_oihw.contiguous()
    _check(lib().sige_pack_weight(_ptr(w), _DT[w.dtype], Cout, Cin, k, _ptr(packed), _stream()))
    return packed


def sige_gn_stats(x, groups, mean, var, *, gamma=None, beta=None, eps=1e-5, scale=None, shift=None,
                  C=None, x_ld=None):
    """Group mean / biased variance of a full tensor and the folded per-channel scale / shift."""
    H, W = x.shape[0], x.shape[1]
    C = x.shape[2] if C is None else C
    x_ld = x.stride(1) if x_ld is None else x_ld
    _check(lib().sige_gn_stats(_ptr(x), _DT[x.dtype], H, W, C, x_ld, groups, _ptr(gamma), _ptr(beta), eps,
                               _ptr(mean), _ptr(var), _ptr(scale), _ptr(shift), _stream()))


def sige_version() -> int:
    return int(lib().sige_version())


def sige_set_knob(name: str, value: int) -> None:
    """Overrides one launch heuristic (value < 0: automatic again); see sige_knob in the header."""
    _check(lib().sige_set_knob(KNOBS[name], value))


def sige_get_knob(name: str) -> int:
    return int(lib().sige_get_knob(KNOBS[name]))


class knobs:
    """with api.knobs(CONV_CFG=3, CONV_KC=16): ... - overrides for the duration of the block."""

    def __init__(self, **kv):
        self.kv = kv

    def __enter__(self):
        self.prev = {k: sige_get_knob(k) for k in self.kv}
        for k, v in self.kv.items():
            sige_set_knob(k, -1 if v is None else int(v))
        return self

    def __exit__(self, *exc):
        for k, v in self.prev.items():
            sige_set_knob(k, v)
        return False
