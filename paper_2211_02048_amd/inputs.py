"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

Only random draws, shapes and masks live here: none of the method's arithmetic
(no normalisation statistics, no convolution, no block reduction).  The inputs
stand in for the paper's edit benchmarks (localised strokes, pasted objects and
circular inpainting masks; Sec. 4.1 "Datasets", App. B), which cannot be shipped:
only their shapes, edit-area statistics and structure are borrowed.

Every tensor is a CPU torch tensor, batch 1, NHWC ([H, W, C]), already in its
storage dtype, drawn from numpy's PCG64 with an explicit seed.
"""
from __future__ import annotations

import math

import numpy as np
import torch

DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _t(a: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dtype).contiguous()


def rect_mask(rng, H: int, W: int, area_frac: float) -> np.ndarray:
    """One axis-aligned rectangle of about area_frac of the image."""
    lo, hi = max(1, H // 8), max(2, (3 * H) // 8)
    h = int(rng.integers(lo, hi + 1))
    w = max(1, min(W, int(round(area_frac * H * W / h))))
    y0 = int(rng.integers(0, H - h + 1))
    x0 = int(rng.integers(0, W - w + 1))
    m = np.zeros((H, W), dtype=np.uint8)
    m[y0:y0 + h, x0:x0 + w] = 1
    return m


def blob_mask(rng, H: int, W: int, target_px: int, n_blobs: int = 3, axes=(5.0, 12.0),
              tol: float = 0.05) -> np.ndarray:
    """Union of n_blobs filled ellipses (random centres, semi-axes, rotation), all
    rescaled by one factor found by bisection so the union covers target_px pixels
    within +-tol (relative)."""
    cy = rng.uniform(0, H, n_blobs)
    cx = rng.uniform(0, W, n_blobs)
    a = rng.uniform(axes[0], axes[1], n_blobs)
    b = rng.uniform(axes[0], axes[1], n_blobs)
    th = rng.uniform(0, math.pi, n_blobs)
    yy, xx = np.mgrid[0:H, 0:W].astype(np.float64)

    def draw(s: float) -> np.ndarray:
        m = np.zeros((H, W), dtype=bool)
        for i in range(n_blobs):
            dy, dx = yy - cy[i], xx - cx[i]
            u = (dx * math.cos(th[i]) + dy * math.sin(th[i])) / (a[i] * s)
            v = (-dx * math.sin(th[i]) + dy * math.cos(th[i])) / (b[i] * s)
            m |= (u * u + v * v) <= 1.0
        return m

    lo, hi = 0.01, 1.0
    while draw(hi).sum() < target_px and hi < 1e3:
        hi *= 2.0
    m = draw(hi)
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        m = draw(mid)
        n = int(m.sum())
        if abs(n - target_px) <= tol * target_px:
            break
        if n < target_px:
            lo = mid
        else:
            hi = mid
    return m.astype(np.uint8)


def edited_pair(rng, H, W, C, mask: np.ndarray, sigma_edit: float, dtype: torch.dtype):
    """A_orig ~ N(0,1); A_edit equals A_orig bit for bit outside the mask and is
    A_orig + N(0, sigma_edit^2) on every channel inside it."""
    a_o = rng.standard_normal((H, W, C), dtype=np.float32)
    noise = rng.standard_normal((H, W, C), dtype=np.float32) * np.float32(sigma_edit)
    a_o_t = _t(a_o, dtype)
    a_e_t = _t(a_o + noise, dtype)
    m = torch.from_numpy(mask.astype(bool))[:, :, None]
    a_e_t = torch.where(m, a_e_t, a_o_t).contiguous()
    return a_o_t, a_e_t


def conv_params(rng, Cout: int, Cin: int, k: int, dtype: torch.dtype, bias_sigma: float = 0.1):
    """W ~ N(0, 1/fan_in) in OIHW, bias ~ N(0, bias_sigma^2) in fp32."""
    w = rng.standard_normal((Cout, Cin, k, k), dtype=np.float32) / np.float32(math.sqrt(Cin * k * k))
    b = rng.standard_normal((Cout,), dtype=np.float32) * np.float32(bias_sigma)
    return _t(w, dtype), torch.from_numpy(b)


def config1(seed: int = 1001, H: int = 64, W: int = 64, C: int = 64, area_frac: float = 0.05):
    """Single 3x3 conv, stride 1, pad 1, fp32, 64x64x64; one rectangle edit of ~5 %
    area with N(0,1) noise; output block 6x6 (8x8 input tiles); tau = 1e-6."""
    rng = _rng(seed)
    mask = rect_mask(rng, H, W, area_frac)
    a_o, a_e = edited_pair(rng, H, W, C, mask, 1.0, torch.float32)
    w, b = conv_params(rng, C, C, 3, torch.float32)
    return dict(name="config1", dtype="f32", H=H, W=W, Cin=C, Cout=C, k=3, stride=1, pad=1,
                block=6, tau=1e-6, dilate=0, mask=mask, a_orig=a_o, a_edit=a_e, w=w, bias=b)


def config2(seed: int = 1002, H: int = 256, W: int = 256, C: int = 128, Cs: int = 256,
            area_frac: float = 0.01, dtype: str = "f16", block: int = 16, n_blobs: int = 3,
            axes=(5.0, 12.0)):
    """Fused GroupNorm(32 groups, cached statistics) + SiLU + 3x3 conv C->C, plus a
    1x1 shortcut conv C->Cs on the same mask; edit = union of elliptical blobs of
    about area_frac of the image, perturbation N(0, 0.5) (variance)."""
    rng = _rng(seed)
    td = DTYPES[dtype]
    mask = blob_mask(rng, H, W, int(round(area_frac * H * W)), n_blobs, axes)
    a_o, a_e = edited_pair(rng, H, W, C, mask, math.sqrt(0.5), td)
    gamma = torch.from_numpy((1.0 + math.sqrt(0.1) * rng.standard_normal(C)).astype(np.float32))
    beta = torch.from_numpy((math.sqrt(0.1) * rng.standard_normal(C)).astype(np.float32))
    w, b = conv_params(rng, C, C, 3, td)
    ws, bs = conv_params(rng, Cs, C, 1, td)
    return dict(name="config2", dtype=dtype, H=H, W=W, Cin=C, Cout=C, Cs=Cs, k=3, stride=1, pad=1,
                block=block, tau=0.0, dilate=0, groups=32, eps=1e-5, mask=mask, a_orig=a_o,
                a_edit=a_e, gamma=gamma, beta=beta, w=w, bias=b, w_s=ws, bias_s=bs)


def attention_case(seed: int, T: int, heads: int, d: int, n_q: int, dtype: str = "bf16"):
    """q [n_q, heads, d], k and v [T, heads, d], all N(0,1) in the storage dtype."""
    rng = _rng(seed)
    td = DTYPES[dtype]
    q = _t(rng.standard_normal((n_q, heads, d), dtype=np.float32), td)
    k = _t(rng.standard_normal((T, heads, d), dtype=np.float32), td)
    v = _t(rng.standard_normal((T, heads, d), dtype=np.float32), td)
    return dict(q=q, k=k, v=v, T=T, heads=heads, d=d, n_q=n_q, dtype=dtype,
                scale=1.0 / math.sqrt(d))


def token_mask(seed: int, Ht: int, Wt: int, area_frac: float, n_blobs: int = 3) -> np.ndarray:
    """Blob mask on a token grid (latent resolution) covering about area_frac."""
    rng = _rng(seed)
    s = min(Ht, Wt) / 64.0
    return blob_mask(rng, Ht, Wt, max(1, int(round(area_frac * Ht * Wt))), n_blobs,
                     (2.0 * s + 0.5, 6.0 * s + 0.5), tol=0.15)
