"""ctypes front end and paper-level compositions of the CPU oracle.

TEST INFRASTRUCTURE ONLY: a slow, obviously-correct double-precision statement
of the method, independent of the HIP library (no shared code, tables or
helpers).  Tensors are numpy arrays, batch 1, NHWC ([H, W, C]); floating data
is float64 holding storage-dtype values exactly; masks are uint8; block lists
are int32 [N, 2] = (y0, x0) of the output block.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sige_oracle.c")
_SO = os.path.join(_HERE, "libsige_oracle.so")

ACT_NONE, ACT_SILU, ACT_RELU, ACT_LEAKY_RELU = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP over output rows)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
             _SRC, "-o", _SO, "-lm"])
    return _SO


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def set_threads(n: int) -> None:
    """Number of OpenMP threads the C loops use (for the timed CPU baseline)."""
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def get_max_threads() -> int:
    return int(ctypes.CDLL("libgomp.so.1").omp_get_max_threads())


# ---------------------------------------------------------------- masks (integer, exact)

def diff_mask(a_orig, a_edit, tau: float) -> np.ndarray:
    """Sec. 3.1 "Structured sparsity": per-pixel any-channel |A_edit - A_orig| > tau,
    evaluated in single precision on exactly converted inputs."""
    a_o = np.ascontiguousarray(a_orig, dtype=np.float32)
    a_e = np.ascontiguousarray(a_edit, dtype=np.float32)
    H, W, C = a_o.shape
    m = np.zeros((H, W), dtype=np.uint8)
    _L().oracle_diff_mask(_p(a_o, ctypes.c_float), _p(a_e, ctypes.c_float), H, W, C,
                          ctypes.c_float(tau), _p(m, ctypes.c_uint8))
    return m


def downsample(m: np.ndarray) -> np.ndarray:
    """Sec. 3.2: one 2x2 / stride-2 max-pool level (ceil mode) of the mask."""
    m = np.ascontiguousarray(m, dtype=np.uint8)
    H, W = m.shape
    out = np.zeros(((H + 1) // 2, (W + 1) // 2), dtype=np.uint8)
    _L().oracle_downsample(_p(m, ctypes.c_uint8), H, W, _p(out, ctypes.c_uint8))
    return out


def dilate(m: np.ndarray, r: int) -> np.ndarray:
    """Sec. 3.2: dilation of the mask by r pixels (square window, clipped)."""
    m = np.ascontiguousarray(m, dtype=np.uint8)
    H, W = m.shape
    out = np.zeros_like(m)
    _L().oracle_dilate(_p(m, ctypes.c_uint8), H, W, int(r), _p(out, ctypes.c_uint8))
    return out


def level_mask(m: np.ndarray, levels: int, r: int) -> np.ndarray:
    """Sec. 3.2: mask at a feature-map scale = dilate(downsample^levels(m), r)."""
    for _ in range(levels):
        m = downsample(m)
    return dilate(m, r)


def active_blocks(m, Hout, Wout, bh, bw, k, stride, pad) -> np.ndarray:
    """Sec. 3.2 / Fig. "method": row-major list of the output blocks whose input
    footprint meets the mask.  m is at the conv's INPUT resolution."""
    m = np.ascontiguousarray(m, dtype=np.uint8)
    Hin, Win = m.shape
    nmax = -(-Hout // bh) * -(-Wout // bw)
    idx = np.zeros((nmax, 2), dtype=np.int32)
    n = _L().oracle_active_blocks(_p(m, ctypes.c_uint8), Hin, Win, Hout, Wout, bh, bw, k,
                                  stride, pad, _p(idx, ctypes.c_int32))
    return idx[:n].copy()


def block_pixels(blocks, bh, bw, H, W) -> np.ndarray:
    """In-image pixels of the listed blocks: list order, then row-major inside a
    block (Fig. "sige-attention": the N*h*w query tokens)."""
    out = []
    for y0, x0 in np.asarray(blocks).reshape(-1, 2):
        for y in range(y0, min(y0 + bh, H)):
            for x in range(x0, min(x0 + bw, W)):
                out.append((y, x))
    return np.asarray(out, dtype=np.int32).reshape(-1, 2)


# ---------------------------------------------------------------- normalisation

def gn_stats(x, groups: int):
    """Sec. 3.2 "Pre-computing normalization parameters": per-group mean and biased
    variance of a full [H, W, C] tensor."""
    x = _f64(x)
    H, W, C = x.shape
    mean = np.zeros(groups)
    var = np.zeros(groups)
    _L().oracle_gn_stats(_p(x, ctypes.c_double), H, W, C, groups, _p(mean, ctypes.c_double),
                         _p(var, ctypes.c_double))
    return mean, var


def fold_gn(gamma, beta, mean, var, eps: float):
    """GroupNorm with fixed (cached) statistics as a per-channel Scale+Shift:
    scale_c = gamma_c / sqrt(var_g + eps), shift_c = beta_c - mean_g * scale_c."""
    gamma = _f64(gamma)
    beta = _f64(beta)
    C, G = gamma.shape[0], len(mean)
    g = np.arange(C) // (C // G)
    scale = gamma / np.sqrt(np.asarray(var, dtype=np.float64)[g] + eps)
    shift = beta - np.asarray(mean, dtype=np.float64)[g] * scale
    return scale, shift


def scale_shift_act(x, scale, shift, act: int) -> np.ndarray:
    """Sec. 3.2 "Kernel fusion": Scale+Shift then the nonlinearity, on a full tensor."""
    x = _f64(x)
    H, W, C = x.shape
    z = np.empty_like(x)
    sc = _f64(scale) if scale is not None else None
    sh = _f64(shift) if shift is not None else None
    _L().oracle_scale_shift_act(_p(x, ctypes.c_double), H, W, C, _p(sc, ctypes.c_double),
                                _p(sh, ctypes.c_double), int(act), _p(z, ctypes.c_double))
    return z


def activation(v, act: int) -> np.ndarray:
    v = _f64(v)
    if act == ACT_SILU:
        return v / (1.0 + np.exp(-v))
    if act == ACT_RELU:
        return np.maximum(v, 0.0)
    if act == ACT_LEAKY_RELU:
        return np.where(v > 0.0, v, 0.2 * v)
    return v


def modulate(x, scale, shift, gamma_map, beta_map, act: int) -> np.ndarray:
    """A spatially-adaptive normalisation layer with cached statistics (the conditional-GAN
    generator of Sec. 4.1; Sec. 3.2 "Pre-computing normalization parameters"): the instance-norm
    statistics of the original activation are folded into per-channel scale / shift, the
    per-pixel gamma and beta come from the label map:  act((scale x + shift)(1 + gamma) + beta)."""
    n = _f64(x)
    if scale is not None:
        n = n * _f64(scale) + _f64(shift)
    return activation(n * (1.0 + _f64(gamma_map)) + _f64(beta_map), act)


# ---------------------------------------------------------------- convolution

def conv_out_size(n_in: int, k: int, stride: int, pad: int) -> int:
    return (n_in + 2 * pad - k) // stride + 1


def conv2d(z, w_oihw, bias, stride: int = 1, pad: int = 0, pixels=None) -> np.ndarray:
    """Sec. 3.1: F(A) = W * A + b, direct zero-padded convolution of the whole
    tensor (or of the listed output pixels only: result [npix, Cout])."""
    z = _f64(z)
    w = _f64(w_oihw)
    Hin, Win, Cin = z.shape
    Cout, Cin2, k, k2 = w.shape
    assert Cin == Cin2 and k == k2
    b = _f64(bias) if bias is not None else None
    Hout, Wout = conv_out_size(Hin, k, stride, pad), conv_out_size(Win, k, stride, pad)
    if pixels is not None:
        px = np.ascontiguousarray(pixels, dtype=np.int32).reshape(-1, 2)
        y = np.empty((px.shape[0], Cout))
        _L().oracle_conv2d(_p(z, ctypes.c_double), Hin, Win, Cin, _p(w, ctypes.c_double),
                           _p(b, ctypes.c_double), Cout, k, stride, pad, Hout, Wout,
                           _p(px, ctypes.c_int32), px.shape[0], _p(y, ctypes.c_double))
        return y
    y = np.empty((Hout, Wout, Cout))
    _L().oracle_conv2d(_p(z, ctypes.c_double), Hin, Win, Cin, _p(w, ctypes.c_double),
                       _p(b, ctypes.c_double), Cout, k, stride, pad, Hout, Wout, None, 0,
                       _p(y, ctypes.c_double))
    return y


def round_storage(a, storage: str) -> np.ndarray:
    """Round-to-nearest-even of float64 values to a storage type ("f32", "f16", "bf16"; "f64" = as is),
    returned as float64; half types are reached through single precision, the type the
    element-wise work is done in.  Fig. "method": the gathered blocks are a stored tensor
    of the model's dtype that the convolution then reads."""
    a = _f64(a)
    if storage == "f64":          # no rounding: the mathematical statement of a pass, for the oracle's own pins
        return a
    if storage == "f32":
        return a.astype(np.float32).astype(np.float64)
    if storage == "f16":
        return a.astype(np.float32).astype(np.float16).astype(np.float64)
    if storage == "bf16":
        bits = a.astype(np.float32).view(np.uint32)
        bits = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
        return bits.view(np.float32).astype(np.float64)
    raise ValueError(storage)


def dense_layer(x, w_oihw, bias, stride=1, pad=0, scale=None, shift=None, act=ACT_NONE,
                pixels=None, storage=None) -> np.ndarray:
    """One wrapped layer on a whole tensor: Scale+Shift (cached statistics),
    nonlinearity, then the convolution; padding is applied to the activated tensor.
    storage: when given, the activated tensor (what Gather hands to the convolution)
    is rounded once to that storage type, as a stored tensor of the model would be."""
    fused = scale is not None or act != ACT_NONE
    z = scale_shift_act(x, scale, shift, act) if fused else _f64(x)
    if fused and storage is not None:
        z = round_storage(z, storage)
    return conv2d(z, w_oihw, bias, stride, pad, pixels)


def select_blocks(y_new, y_cache, blocks, bh, bw) -> np.ndarray:
    """Fig. "pipeline" (b): cached output with the active blocks replaced."""
    y_new = _f64(y_new)
    y_cache = _f64(y_cache)
    H, W, C = y_cache.shape
    idx = np.ascontiguousarray(blocks, dtype=np.int32).reshape(-1, 2)
    out = np.empty_like(y_cache)
    _L().oracle_select_blocks(_p(y_new, ctypes.c_double), _p(y_cache, ctypes.c_double), H, W, C,
                              _p(idx, ctypes.c_int32), idx.shape[0], bh, bw,
                              _p(out, ctypes.c_double))
    return out


def sige_layer(x_edit, y_cache, blocks, bh, bw, w_oihw, bias, stride=1, pad=0, scale=None,
               shift=None, act=ACT_NONE, storage=None) -> np.ndarray:
    """Fig. "pipeline" (b), written densely: compute the layer on the whole edited
    input, keep the new values on active blocks and the cache elsewhere."""
    y = dense_layer(x_edit, w_oihw, bias, stride, pad, scale, shift, act, storage=storage)
    return select_blocks(y, y_cache, blocks, bh, bw)


def pipeline_a(x_orig, x_edit, y_cache, blocks, bh, bw, w_oihw, stride=1, pad=0) -> np.ndarray:
    """Fig. "pipeline" (a): convolve the difference without bias, keep it on the
    active blocks of a zero tensor, add the cached F(A_orig) (Sec. 3.1 identity)."""
    delta = _f64(x_edit) - _f64(x_orig)
    d = conv2d(delta, w_oihw, None, stride, pad)
    zero = np.zeros_like(d)
    return select_blocks(d, zero, blocks, bh, bw) + _f64(y_cache)


# ---------------------------------------------------------------- token-wise layers

def layer_norm(x, gamma=None, beta=None, eps: float = 1e-5) -> np.ndarray:
    """Per-token layer normalisation over the last axis (biased variance), the textbook
    operator of a transformer block; the token-wise layers between Gather and Scatter of
    an attention block (Sec. 3.2 "Extension to attention layers") use it."""
    x = _f64(x)
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    y = (x - mean) / np.sqrt(var + eps)
    if gamma is not None:
        y = y * _f64(gamma)
    if beta is not None:
        y = y + _f64(beta)
    return y


def geglu(x) -> np.ndarray:
    """Gated GELU of a feed-forward layer: x[..., :C] * gelu(x[..., C:]) with the exact
    gelu(g) = g/2 * (1 + erf(g / sqrt 2))."""
    from math import sqrt

    from scipy.special import erf          # the library's double-precision error function, element-wise
    x = _f64(x)
    C = x.shape[-1] // 2
    g = x[..., C:]
    phi = 0.5 * (1.0 + erf(g / sqrt(2.0)))
    return x[..., :C] * g * phi


# ---------------------------------------------------------------- attention

def attention(q, k, v, scale: float) -> np.ndarray:
    """Sec. 3.2 "Extension to attention layers": softmax(q K^T * scale) V for the
    given query tokens against all T keys.  q: [Nq, heads, d]; k, v: [T, heads, d]."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    Nq, heads, d = q.shape
    T = k.shape[0]
    o = np.empty_like(q)
    _L().oracle_attention(_p(q, ctypes.c_double), _p(k, ctypes.c_double), _p(v, ctypes.c_double),
                          Nq, T, heads, d, ctypes.c_double(scale), _p(o, ctypes.c_double))
    return o


def sige_attention_layer(x_edit, out_cache, blocks, bh, bw, wq, wk, wv, wo, bq, bk, bv, bo,
                         heads: int, scale: float, k_cache=None, v_cache=None) -> np.ndarray:
    """Fig. "sige-attention", written densely.  Q, K, V are 1x1 projections of the
    whole edited input (or, when caches are given, cached K/V with the active
    tokens overwritten); attention runs for the active tokens only; the Out
    projection of those rows replaces the cached output at the active tokens."""
    x = _f64(x_edit)
    H, W, C = x.shape
    tok = block_pixels(blocks, bh, bw, H, W)
    q_full = conv2d(x, wq, bq)
    k_new = conv2d(x, wk, bk)
    v_new = conv2d(x, wv, bv)
    Ch = q_full.shape[2]
    if k_cache is not None:
        k_full = _f64(k_cache).copy()
        v_full = _f64(v_cache).copy()
        for (y, xx) in tok:
            k_full[y, xx] = k_new[y, xx]
            v_full[y, xx] = v_new[y, xx]
    else:
        k_full, v_full = k_new, v_new
    d = Ch // heads
    q_act = np.stack([q_full[y, xx] for (y, xx) in tok]).reshape(-1, heads, d) if len(tok) else \
        np.zeros((0, heads, d))
    a = attention(q_act, k_full.reshape(H * W, heads, d), v_full.reshape(H * W, heads, d), scale)
    out = _f64(out_cache).copy()
    if len(tok):
        proj = conv2d(a.reshape(len(tok), 1, Ch), wo, bo)  # 1x1 conv over the token list
        for i, (y, xx) in enumerate(tok):
            out[y, xx] = proj[i, 0]
    return out
