"""Shared test plumbing: tensor conversion, the tolerance rule, and oracle-side
expected values.  No arithmetic of the method lives here except calls into oracle/."""
import numpy as np
import torch

TOL = {torch.float32: 1e-4, torch.float16: 1e-2, torch.bfloat16: 1e-2}


def f64(t: torch.Tensor) -> np.ndarray:
    """Storage-dtype tensor -> float64 numpy (exact)."""
    return t.detach().cpu().to(torch.float64).numpy()


def dev(t, device="cuda"):
    return t.to(device).contiguous()


def round_to(a: np.ndarray, dtype: torch.dtype) -> np.ndarray:
    """Oracle value rounded once to the storage dtype (round-to-nearest-even)."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).to(torch.float64).numpy()


def assert_close(got: torch.Tensor, want64: np.ndarray, dtype: torch.dtype, what: str = "", tol=None):
    """Element-wise |y - y_ref| <= tol * max(|y_ref|, rms(y_ref)); y_ref = oracle rounded to dtype.
    tol: 1e-4 for fp32, 1e-2 for fp16 / bf16."""
    tol = TOL[dtype] if tol is None else tol
    ref = round_to(want64, dtype)
    g = f64(got)
    assert g.shape == ref.shape, (what, g.shape, ref.shape)
    if ref.size == 0:
        return
    rms = float(np.sqrt(np.mean(ref * ref)))
    bound = tol * np.maximum(np.abs(ref), rms)
    err = np.abs(g - ref)
    bad = ~(err <= bound)  # NaN counts as bad
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {ref.size} elements off; worst err "
                           f"{np.nanmax(err):.3e} at bound {bound.flat[np.nanargmax(err / (bound + 1e-300))]:.3e}")


def expected_tiles(oracle, x64, blocks, th, tw, stride, pad, scale, shift, act):
    """Gathered tiles by definition: activated full tensor, zero padded, sliced."""
    z = oracle.scale_shift_act(x64, scale, shift, act) if (scale is not None or act) else x64
    H, W, C = z.shape
    out = np.zeros((len(blocks), th, tw, C))
    for n, (y0, x0) in enumerate(np.asarray(blocks).reshape(-1, 2)):
        for i in range(th):
            for j in range(tw):
                y, x = y0 * stride - pad + i, x0 * stride - pad + j
                if 0 <= y < H and 0 <= x < W:
                    out[n, i, j] = z[y, x]
    return out


def outside_blocks_mask(blocks, bh, bw, H, W) -> np.ndarray:
    m = np.ones((H, W), bool)
    for y0, x0 in np.asarray(blocks).reshape(-1, 2):
        m[y0:y0 + bh, x0:x0 + bw] = False
    return m


def assert_mostly_close(got, want64, dtype, what, frac=0.9999, loose=2.0):
    """Against the oracle WITHOUT intermediate storage rounding: at least `frac` of the elements
    within the stated tolerance and every element within `loose` times it (the remainder is the
    rounding of the activated tile to a half type before it reaches the matrix cores)."""
    tol = TOL[dtype]
    ref = round_to(want64, dtype)
    g = f64(got)
    rms = float(np.sqrt(np.mean(ref * ref)))
    bound = tol * np.maximum(np.abs(ref), rms)
    err = np.abs(g - ref)
    ok = err <= bound
    assert ok.mean() >= frac, f"{what}: only {ok.mean():.6f} of the elements within {tol}"
    assert (err <= loose * bound).all(), f"{what}: an element beyond {loose}x the tolerance"
