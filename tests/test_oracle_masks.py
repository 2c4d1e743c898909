"""Pins for the oracle's integer steps (difference mask, downsample, dilate, block
reduction): brute force against set-based definitions written here, closed forms
and the counting example the paper prints."""
import itertools
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_active(mask_set, Hin, Win, Hout, Wout, b, k, s, p):
    """Definition by sets: block (by, bx) is active iff some marked input pixel is
    read by some output pixel of the block."""
    out = []
    for by in range(-(-Hout // b)):
        for bx in range(-(-Wout // b)):
            outs = [(y, x) for y in range(by * b, by * b + b) for x in range(bx * b, bx * b + b)]
            reads = {(y * s + ky - p, x * s + kx - p) for (y, x) in outs
                     for ky in range(k) for kx in range(k)}
            if reads & mask_set:
                out.append((by * b, bx * b))
    return out


@pytest.mark.parametrize("b,k,s,p", [(2, 3, 1, 1), (3, 3, 1, 1), (2, 1, 1, 0), (2, 3, 2, 1)])
def test_active_blocks_all_masks_small(oracle, b, k, s, p):
    # every mask of a 3x4 input: 4096 cases
    Hin, Win = 3, 4
    Hout, Wout = (Hin + 2 * p - k) // s + 1, (Win + 2 * p - k) // s + 1
    cells = [(y, x) for y in range(Hin) for x in range(Win)]
    for bits in range(1 << len(cells)):
        ms = {c for i, c in enumerate(cells) if bits >> i & 1}
        m = np.zeros((Hin, Win), np.uint8)
        for (y, x) in ms:
            m[y, x] = 1
        got = [tuple(r) for r in oracle.active_blocks(m, Hout, Wout, b, b, k, s, p)]
        assert got == brute_active(ms, Hin, Win, Hout, Wout, b, k, s, p), (bits, b, k, s, p)


def test_active_blocks_random(oracle):
    rng = np.random.default_rng(7)
    for _ in range(200):
        Hin, Win = int(rng.integers(1, 17)), int(rng.integers(1, 17))
        k = int(rng.choice([1, 3, 5]))
        s = int(rng.choice([1, 2])) if k > 1 else 1   # k >= stride: the tile has no unread gaps
        p = k // 2
        b = int(rng.integers(1, 8))
        Hout, Wout = (Hin + 2 * p - k) // s + 1, (Win + 2 * p - k) // s + 1
        m = (rng.random((Hin, Win)) < rng.choice([0.02, 0.1, 0.5])).astype(np.uint8)
        ms = {(int(y), int(x)) for y, x in zip(*np.nonzero(m))}
        got = [tuple(r) for r in oracle.active_blocks(m, Hout, Wout, b, b, k, s, p)]
        assert got == brute_active(ms, Hin, Win, Hout, Wout, b, k, s, p)


def test_active_blocks_closed_forms(oracle):
    H = W = 20
    b = 6
    empty = np.zeros((H, W), np.uint8)
    assert oracle.active_blocks(empty, H, W, b, b, 3, 1, 1).shape == (0, 2)
    full = np.ones((H, W), np.uint8)
    got = oracle.active_blocks(full, H, W, b, b, 3, 1, 1)
    want = [(y, x) for y in range(0, H, b) for x in range(0, W, b)]  # ceil(20/6)^2 = 16, row-major
    assert [tuple(r) for r in got] == want and len(want) == 16
    # one marked pixel, 3x3 / stride 1 / pad 1: per axis the block row floor(y/b), plus the
    # previous one iff y mod b == 0, plus the next one iff y mod b == b-1 (clipped to the grid)
    nb = -(-H // b)
    for y in range(H):
        for x in range(W):
            m = np.zeros((H, W), np.uint8)
            m[y, x] = 1

            def axis(v):
                r = {v // b}
                if v % b == 0:
                    r.add(v // b - 1)
                if v % b == b - 1:
                    r.add(v // b + 1)
                return sorted(i for i in r if 0 <= i < nb)
            want = [(i * b, j * b) for i in axis(y) for j in axis(x)]
            got = [tuple(r) for r in oracle.active_blocks(m, H, W, b, b, 3, 1, 1)]
            assert got == want
            assert len(got) in (1, 2, 4)
            # 1x1 conv: exactly the block holding the pixel
            got1 = [tuple(r) for r in oracle.active_blocks(m, H, W, 4, 4, 1, 1, 0)]
            assert got1 == [(y // 4 * 4, x // 4 * 4)]


def test_dilate_and_downsample_bruteforce(oracle):
    rng = np.random.default_rng(11)
    for _ in range(100):
        H, W = int(rng.integers(1, 14)), int(rng.integers(1, 14))
        m = (rng.random((H, W)) < 0.15).astype(np.uint8)
        ms = {(int(y), int(x)) for y, x in zip(*np.nonzero(m))}
        r = int(rng.integers(0, 4))
        want = np.zeros((H, W), np.uint8)
        for y in range(H):
            for x in range(W):
                if any(max(abs(y - yy), abs(x - xx)) <= r for (yy, xx) in ms):  # Chebyshev ball
                    want[y, x] = 1
        assert np.array_equal(oracle.dilate(m, r), want)
        want = np.zeros(((H + 1) // 2, (W + 1) // 2), np.uint8)
        for (yy, xx) in ms:
            want[yy // 2, xx // 2] = 1
        assert np.array_equal(oracle.downsample(m), want)
    # dilation by r twice == dilation by 2r (square windows compose)
    m = (rng.random((17, 13)) < 0.05).astype(np.uint8)
    assert np.array_equal(oracle.dilate(oracle.dilate(m, 1), 2), oracle.dilate(m, 3))
    # a chain of n pool levels marks pixel (y, x) iff the 2^n window has a marked pixel
    m = (rng.random((37, 29)) < 0.02).astype(np.uint8)
    lv = oracle.level_mask(m, 3, 0)
    want = np.zeros((5, 4), np.uint8)
    for yy, xx in zip(*np.nonzero(m)):
        want[yy // 8, xx // 8] = 1
    assert np.array_equal(lv, want)


def test_diff_mask_definition(oracle):
    rng = np.random.default_rng(3)
    a = rng.standard_normal((9, 7, 5)).astype(np.float32)
    e = a.copy()
    e[2, 3, 4] += 1.0          # clearly changed
    e[5, 1, 0] += 5e-7         # below tau = 1e-6 (|a| small enough that the sum is exact enough)
    a[5, 1, 0] = e[5, 1, 0] = 0.0
    e[5, 1, 0] = 5e-7
    e[6, 6, 2] = np.nan        # NaN counts as changed
    e[0, 0, 1] = a[0, 0, 1] + np.float32(4e-6)
    m = oracle.diff_mask(a, e, 1e-6)
    want = np.zeros((9, 7), np.uint8)
    want[2, 3] = want[6, 6] = 1
    d = np.float32(e[0, 0, 1]) - np.float32(a[0, 0, 1])
    want[0, 0] = 1 if abs(d) > np.float32(1e-6) else 0
    assert np.array_equal(m, want)
    # strict comparison: a difference exactly equal to tau is not marked
    a2 = np.zeros((1, 1, 1), np.float32)
    e2 = np.full((1, 1, 1), 0.5, np.float32)
    assert oracle.diff_mask(a2, e2, 0.5)[0, 0] == 0
    assert oracle.diff_mask(a2, e2, np.nextafter(np.float32(0.5), np.float32(0)))[0, 0] == 1
    # tau = 0: bitwise-different values only; +0 and -0 are equal
    e3 = np.array([[[-0.0]]], np.float32)
    assert oracle.diff_mask(a2, e3, 0.0)[0, 0] == 0


def test_query_count_matches_paper_example(oracle):
    """Sec. 4.2 "Model efficiency": a 64x128-token layer whose attention map shrinks
    from 8192 to 672 query rows; with 4x4 token blocks (Sec. 4.1 "Implementation
    details") that is 42 full blocks."""
    vals = {}
    with open(os.path.join(GOLDEN, "attention_map_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split("=")
                vals[k.strip()] = int(v)
    Ht, Wt, b = vals["token_rows"], vals["token_cols"], vals["block_1x1"]
    assert Ht * Wt == vals["tokens"]
    n_blocks = vals["edited_queries"] // (b * b)
    assert n_blocks * b * b == vals["edited_queries"]
    # mark exactly n_blocks distinct 4x4 blocks with one pixel each
    rng = np.random.default_rng(0)
    ids = rng.choice((Ht // b) * (Wt // b), n_blocks, replace=False)
    m = np.zeros((Ht, Wt), np.uint8)
    for i in ids:
        m[(i // (Wt // b)) * b + 1, (i % (Wt // b)) * b + 2] = 1
    blocks = oracle.active_blocks(m, Ht, Wt, b, b, 1, 1, 0)
    tok = oracle.block_pixels(blocks, b, b, Ht, Wt)
    assert len(blocks) == n_blocks == 42
    assert len(tok) == vals["edited_queries"]
    assert vals["tokens"] // len(tok) == vals["shrink_factor_floor"]
    # block list is row-major and unique
    keys = [int(y) * Wt + int(x) for y, x in blocks]
    assert keys == sorted(set(keys))
