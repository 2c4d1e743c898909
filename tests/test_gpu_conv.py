"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by
element.  Masks, block lists and pure copies bit-exact; floating results within
1e-4 (fp32) / 1e-2 (fp16, bf16) of the oracle, relative to max(|ref|, rms(ref))."""

import numpy as np
import pytest
import torch

from helpers import assert_close, assert_mostly_close, dev, expected_tiles, f64, outside_blocks_mask, round_to
from paper_2211_02048_amd import api, inputs
from paper_2211_02048_amd.layers import BlockList, SigeConv, Workspace

pytestmark = pytest.mark.gpu
DT = inputs.DTYPES


def run_reduce(g, *, a_orig=None, a_edit=None, tau=0.0, mask=None, pool_log2=0, dilate=0, max_blocks=None,
               use_workspace=True):
    bl = BlockList(g, "cuda", max_blocks, use_workspace)
    bl.indices.fill_(-7)
    mask_out = None
    if a_orig is not None:
        mask_out = torch.full(a_orig.shape[:2], 9, dtype=torch.uint8, device="cuda")
    bl.reduce(a_orig=a_orig, a_edit=a_edit, tau=tau, mask_in=mask, mask_out=mask_out, pool_log2=pool_log2,
              dilate=dilate)
    torch.cuda.synchronize()
    return bl, mask_out


# ------------------------------------------------------------------ a1-a3: mask and block list

@pytest.mark.parametrize("seed", range(1001, 1021))
def test_reduce_mask_config1_bit_exact(oracle, seed):
    cfg = inputs.config1(seed=seed)
    g = api.geom(64, 64, cfg["block"], 3, 1, 1)
    bl, mask = run_reduce(g, a_orig=dev(cfg["a_orig"]), a_edit=dev(cfg["a_edit"]), tau=cfg["tau"])
    want_mask = oracle.diff_mask(cfg["a_orig"].numpy(), cfg["a_edit"].numpy(), cfg["tau"])
    want = oracle.active_blocks(want_mask, 64, 64, 6, 6, 3, 1, 1)
    assert np.array_equal(mask.cpu().numpy(), want_mask)
    n = int(bl.count.item())
    assert n == len(want) and 0 < n < 121
    assert np.array_equal(bl.indices[:n].cpu().numpy(), want)
    assert (bl.indices[n:] == -7).all()  # rows beyond the count are untouched


@pytest.mark.parametrize("dtype,C", [("f16", 128), ("bf16", 320), ("f32", 3), ("f16", 8), ("f32", 256),
                                     ("bf16", 512), ("f16", 24)])
def test_diff_mask_channel_paths(oracle, dtype, C):
    rng = np.random.default_rng(C)
    H, W = 37, 53
    a = torch.from_numpy(rng.standard_normal((H, W, C)).astype(np.float32)).to(DT[dtype])
    e = a.clone()
    ys, xs = rng.integers(0, H, 40), rng.integers(0, W, 40)
    cs = rng.integers(0, C, 40)
    for y, x, c in zip(ys, xs, cs):
        e[y, x, c] = e[y, x, c] + 1.0
    e[0, 0, C - 1] = float("nan")
    e[H - 1, W - 1, 0] = e[H - 1, W - 1, 0] + 2.0
    g = api.geom(H, W, 5, 3, 1, 1)
    for tau in (0.0, 1e-6, 1.5):
        bl, mask = run_reduce(g, a_orig=dev(a), a_edit=dev(e), tau=tau)
        want_mask = oracle.diff_mask(a.float().numpy(), e.float().numpy(), tau)
        assert np.array_equal(mask.cpu().numpy(), want_mask), (dtype, C, tau)
        want = oracle.active_blocks(want_mask, H, W, 5, 5, 3, 1, 1)
        n = int(bl.count.item())
        assert n == len(want) and np.array_equal(bl.indices[:n].cpu().numpy(), want)


def test_block_list_pool_dilate_geometries(oracle):
    rng = np.random.default_rng(42)
    cases = 0
    for Hm, Wm in [(100, 76), (64, 64), (33, 47), (256, 256)]:
        for pool in (0, 1, 2, 3):
            Hin, Win = -(-Hm // (1 << pool)), -(-Wm // (1 << pool))
            for (k, s, p) in [(3, 1, 1), (1, 1, 0), (3, 2, 1)]:
                for b in (4, 6, 16):
                    for r in (0, 1, 5):
                        if Hin + 2 * p < k or Win + 2 * p < k:
                            continue
                        m = (rng.random((Hm, Wm)) < rng.choice([0.0005, 0.005, 0.05])).astype(np.uint8)
                        g = api.geom(Hin, Win, b, k, s, p)
                        bl, _ = run_reduce(g, mask=torch.from_numpy(m).cuda(), pool_log2=pool, dilate=r,
                                           use_workspace=(cases % 2 == 0))  # both kernels, alternating
                        lv = oracle.level_mask(m, pool, r)
                        want = oracle.active_blocks(lv, g.H_out, g.W_out, b, b, k, s, p)
                        n = int(bl.count.item())
                        assert n == len(want), (Hm, Wm, pool, k, s, b, r)
                        assert np.array_equal(bl.indices[:n].cpu().numpy(), want)
                        cases += 1
    assert cases > 300


def test_block_list_degenerate_and_overflow(oracle):
    H = W = 50
    g = api.geom(H, W, 6, 3, 1, 1)
    empty = torch.zeros((H, W), dtype=torch.uint8, device="cuda")
    bl, _ = run_reduce(g, mask=empty)
    assert int(bl.count.item()) == 0 and (bl.indices == -7).all()
    full = torch.ones((H, W), dtype=torch.uint8, device="cuda")
    bl, _ = run_reduce(g, mask=full)
    want = np.array([(y, x) for y in range(0, H, 6) for x in range(0, W, 6)], np.int32)
    assert int(bl.count.item()) == 81 and np.array_equal(bl.indices.cpu().numpy(), want)
    # capacity smaller than the number of active blocks: true count, first rows only, no overrun
    bl, _ = run_reduce(g, mask=full, max_blocks=10)
    assert int(bl.count.item()) == 81
    assert np.array_equal(bl.indices.cpu().numpy(), want[:10])
    with pytest.raises(api.SigeError):
        bl.sync_count()
    # a grid larger than one compaction pass, with and without the workspace; the workspace
    # is reused by back-to-back calls (its ticket returns to zero each time)
    Hb = 300
    gb = api.geom(Hb, Hb, 4, 1, 1, 0)
    m = (np.random.default_rng(0).random((Hb, Hb)) < 0.01).astype(np.uint8)
    want = oracle.active_blocks(m, Hb, Hb, 4, 4, 1, 1, 0)
    for use_ws in (True, False):
        bl, _ = run_reduce(gb, mask=torch.from_numpy(m).cuda(), use_workspace=use_ws)
        assert gb.grid_blocks == 5625 and int(bl.count.item()) == len(want)
        assert np.array_equal(bl.indices[:len(want)].cpu().numpy(), want)
        for rep in range(3):
            bl.indices.fill_(-7)
            bl.reduce(mask_in=torch.from_numpy(m).cuda())
            assert int(bl.count.item()) == len(want)
            assert np.array_equal(bl.indices[:len(want)].cpu().numpy(), want)
        if use_ws:
            assert not bl.scratch.any()  # the flags are left cleared


@pytest.mark.parametrize("mode", ["activations", "mask"])
@pytest.mark.parametrize("pool_log2,dilate", [(0, 0), (0, 1), (1, 1), (2, 2)])
def test_reduce_mask_lists_one_pass_several_geometries(oracle, mode, pool_log2, dilate):
    """Four layer geometries of one resolution from one pass: every list bit-exact against the oracle
    (hence equal to four separate calls); flags left clean; capacity clipping per list."""
    rng = np.random.default_rng(77 + 10 * pool_log2 + dilate)
    Hm, Wm, C = 90, 122, 64
    H, W = -(-Hm // (1 << pool_log2)), -(-Wm // (1 << pool_log2))
    geoms = [api.geom(H, W, 8, 3, 1, 1), api.geom(H, W, 8, 1, 1, 0), api.geom(H, W, 4, 3, 2, 1),
             api.geom(H, W, (6, 5), 5, 1, 2)]
    m = inputs.blob_mask(rng, Hm, Wm, int(0.03 * Hm * Wm)).astype(np.float32)
    a_o = rng.standard_normal((Hm, Wm, C)).astype(np.float32)
    a_e = a_o + m[:, :, None] * rng.standard_normal((Hm, Wm, C)).astype(np.float32)
    lists = [BlockList(g, "cuda", max_blocks=(2 if i == 1 else None)) for i, g in enumerate(geoms)]
    for b in lists:
        b.indices.fill_(-7)
    for rep in range(2):      # the second call reuses the workspaces the first one left zero
        if mode == "activations":
            mask_out = torch.full((Hm, Wm), 9, dtype=torch.uint8, device="cuda")
            BlockList.reduce_together(lists, a_orig=dev(torch.from_numpy(a_o).half()),
                                      a_edit=dev(torch.from_numpy(a_e).half()), tau=0.0, mask_out=mask_out,
                                      pool_log2=pool_log2, dilate=dilate)
            want_mask = oracle.diff_mask(torch.from_numpy(a_o).half().double().numpy(),
                                         torch.from_numpy(a_e).half().double().numpy(), 0.0)
            assert np.array_equal(mask_out.cpu().numpy(), want_mask)
        else:
            want_mask = m.astype(np.uint8)
            BlockList.reduce_together(lists, mask_in=torch.from_numpy(want_mask).cuda(), pool_log2=pool_log2,
                                      dilate=dilate)
        torch.cuda.synchronize()
        lvl = oracle.level_mask(want_mask, pool_log2, dilate)
        for i, (b, g) in enumerate(zip(lists, geoms)):
            want = oracle.active_blocks(lvl, g.H_out, g.W_out, g.block_h, g.block_w, g.k, g.stride, g.pad)
            n = int(b.count.item())
            assert n == len(want) and n > 0, (i, n, len(want))
            keep = min(n, b.max_blocks)
            assert np.array_equal(b.indices[:keep].cpu().numpy(), want[:keep]), i
            assert (b.indices[keep:] == -7).all()
            assert not b.scratch.any()
    assert int(lists[1].count.item()) > 2        # the clipped list really was clipped
    # error paths: shared workspace, missing workspace, too many lists
    with pytest.raises(api.SigeError):
        api.sige_reduce_mask_lists([(geoms[0], lists[0].indices, lists[0].count, None, lists[0].scratch),
                                    (geoms[0], lists[1].indices, lists[1].count, None, lists[0].scratch)],
                                   mask_in=torch.from_numpy(want_mask).cuda(), pool_log2=pool_log2, dilate=dilate)
    with pytest.raises(api.SigeError):
        api.sige_reduce_mask_lists([(geoms[0], lists[0].indices, lists[0].count, None, None)],
                                   mask_in=torch.from_numpy(want_mask).cuda(), pool_log2=pool_log2, dilate=dilate)
    with pytest.raises(api.SigeError):
        api.sige_reduce_mask_lists([(g, b.indices, b.count, None, b.scratch) for g, b in zip(geoms, lists)] +
                                   [(geoms[0], lists[0].indices, lists[0].count, None, lists[0].scratch)],
                                   mask_in=torch.from_numpy(want_mask).cuda(), pool_log2=pool_log2, dilate=dilate)


# ------------------------------------------------------------------ a4 / a6: gather and scatter

def random_blocks(rng, g, n):
    ids = rng.choice(g.grid_blocks, size=min(n, g.grid_blocks), replace=False)
    ids.sort()
    nbx = -(-g.W_out // g.block_w)
    return np.array([((i // nbx) * g.block_h, (i % nbx) * g.block_w) for i in ids], np.int32)


@pytest.mark.parametrize("dtype,C,H,W,b,k,s", [
    ("f32", 64, 64, 64, 6, 3, 1), ("f16", 128, 70, 90, 16, 3, 1), ("bf16", 320, 33, 31, 4, 1, 1),
    ("f16", 64, 64, 48, 8, 3, 2), ("f32", 8, 20, 20, 6, 5, 1), ("f16", 24, 41, 29, 6, 3, 1),
    ("f16", 2560, 12, 10, 4, 1, 1)])     # more than 256 16-byte vectors per pixel
def test_gather_unfused_bit_exact_and_fused(oracle, dtype, C, H, W, b, k, s):
    rng = np.random.default_rng(C + H)
    td = DT[dtype]
    g = api.geom(H, W, b, k, s, k // 2)
    x = torch.from_numpy(rng.standard_normal((H, W, C)).astype(np.float32)).to(td)
    blocks = random_blocks(rng, g, 13)
    # make sure corner blocks (zero padding on two sides, partial blocks) are included
    nby, nbx = -(-g.H_out // b), -(-g.W_out // b)
    corners = np.array([(0, 0), ((nby - 1) * b, (nbx - 1) * b)], np.int32)
    blocks = np.unique(np.concatenate([blocks, corners]), axis=0)
    n = len(blocks)
    idx = torch.from_numpy(blocks).cuda()
    cnt = torch.tensor([n], dtype=torch.int32, device="cuda")
    th, tw = g.tile_h, g.tile_w
    tiles = torch.full((n + 2, th, tw, C), 3.0, dtype=td, device="cuda")
    api.sige_gather(dev(x), g, idx, cnt, tiles, n_blocks=n)
    want = expected_tiles(oracle, f64(x), blocks, th, tw, s, k // 2, None, None, 0)
    assert np.array_equal(f64(tiles[:n]), want)
    assert (tiles[n:] == 3.0).all()  # tiles beyond the count are untouched
    # device-side count (launch sized by capacity) gives the same bytes
    tiles2 = torch.full((n + 2, th, tw, C), 3.0, dtype=td, device="cuda")
    api.sige_gather(dev(x), g, idx, cnt, tiles2, n_blocks=-1)
    assert torch.equal(tiles, tiles2)
    # fused Scale+Shift + SiLU / ReLU
    scale = torch.from_numpy(rng.uniform(0.5, 1.5, C).astype(np.float32))
    shift = torch.from_numpy(rng.uniform(-0.5, 0.5, C).astype(np.float32))
    for act in (api.ACT_SILU, api.ACT_RELU, api.ACT_NONE):
        api.sige_gather(dev(x), g, idx, cnt, tiles, n_blocks=n, scale=dev(scale), shift=dev(shift), act=act)
        want = expected_tiles(oracle, f64(x), blocks, th, tw, s, k // 2, f64(scale), f64(shift), act)
        assert_close(tiles[:n], want, td, f"gather act={act}")
        # padding is exactly zero (not act(shift))
        assert (f64(tiles[:n])[want == 0.0] == 0.0).all()
    api.sige_gather(dev(x), g, idx, cnt, tiles, n_blocks=n, act=api.ACT_SILU)  # activation without scale
    want = expected_tiles(oracle, f64(x), blocks, th, tw, s, k // 2, None, None, api.ACT_SILU)
    assert_close(tiles[:n], want, td, "gather silu only")


def test_gather_strided_source_and_upsample(oracle):
    rng = np.random.default_rng(5)
    td = torch.float16
    H, W, C, LD = 24, 32, 32, 96
    buf = torch.from_numpy(rng.standard_normal((H, W, LD)).astype(np.float32)).to(td).cuda()
    x = buf[:, :, 32:64]  # channel slice of a wider buffer
    g = api.geom(H, W, 8, 3, 1, 1)
    blocks = random_blocks(rng, g, 5)
    idx = torch.from_numpy(blocks).cuda()
    cnt = torch.tensor([len(blocks)], dtype=torch.int32, device="cuda")
    tiles = torch.zeros((len(blocks), 10, 10, C), dtype=td, device="cuda")
    api.sige_gather(x, g, idx, cnt, tiles, n_blocks=len(blocks), C=C, x_ld=LD)
    want = expected_tiles(oracle, f64(x), blocks, 10, 10, 1, 1, None, None, 0)
    assert np.array_equal(f64(tiles), want)
    # nearest-neighbour x2 up-sampling folded into the gather address
    src = torch.from_numpy(rng.standard_normal((H // 2, W // 2, C)).astype(np.float32)).to(td).cuda()
    api.sige_gather(src, g, idx, cnt, tiles, n_blocks=len(blocks), up=1)
    up = f64(src).repeat(2, axis=0).repeat(2, axis=1)
    want = expected_tiles(oracle, up, blocks, 10, 10, 1, 1, None, None, 0)
    assert np.array_equal(f64(tiles), want)


@pytest.mark.parametrize("dtype,C,H,W,b", [("f32", 64, 64, 64, 6), ("f16", 128, 70, 90, 16),
                                           ("bf16", 256, 33, 31, 4), ("f16", 8, 19, 23, 5)])
def test_scatter_bit_exact_and_untouched_outside(oracle, dtype, C, H, W, b):
    rng = np.random.default_rng(H * W)
    td = DT[dtype]
    g = api.geom(H, W, b, 3, 1, 1)
    blocks = random_blocks(rng, g, 11)
    nby, nbx = -(-H // b), -(-W // b)
    blocks = np.unique(np.concatenate([blocks, np.array([((nby - 1) * b, (nbx - 1) * b)], np.int32)]), axis=0)
    n = len(blocks)
    idx = torch.from_numpy(blocks).cuda()
    cnt = torch.tensor([n], dtype=torch.int32, device="cuda")
    out_tiles = torch.from_numpy(rng.standard_normal((n + 1, b, b, C)).astype(np.float32)).to(td).cuda()
    cache = torch.from_numpy(rng.standard_normal((H, W, C)).astype(np.float32)).to(td).cuda()
    y = cache.clone()
    api.sige_scatter(out_tiles, g, idx, cnt, y, n_blocks=n)
    # Fig. "pipeline" (b): active blocks replaced, everything else is the cache bit for bit
    new_full = np.zeros((H, W, C))
    ot = f64(out_tiles)
    for i, (y0, x0) in enumerate(blocks):
        hh, ww = min(b, H - y0), min(b, W - x0)
        new_full[y0:y0 + hh, x0:x0 + ww] = ot[i, :hh, :ww]
    want = oracle.select_blocks(new_full, f64(cache), blocks, b, b)
    assert np.array_equal(f64(y), want)
    # zero blocks: nothing changes
    y2 = cache.clone()
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.sige_scatter(out_tiles, g, idx, zero, y2, n_blocks=-1)
    api.sige_scatter(out_tiles, g, idx, zero, y2, n_blocks=0)
    assert torch.equal(y2, cache)
    # residual tiles + full residual are added in fp32 and rounded once
    res_t = torch.from_numpy(rng.standard_normal((n + 1, b, b, C)).astype(np.float32)).to(td).cuda()
    res_f = torch.from_numpy(rng.standard_normal((H, W, C)).astype(np.float32)).to(td).cuda()
    y3 = cache.clone()
    api.sige_scatter(out_tiles, g, idx, cnt, y3, n_blocks=-1, residual_tiles=res_t, residual=res_f)
    rt = f64(res_t)
    for i, (y0, x0) in enumerate(blocks):
        hh, ww = min(b, H - y0), min(b, W - x0)
        new_full[y0:y0 + hh, x0:x0 + ww] = ot[i, :hh, :ww] + rt[i, :hh, :ww] + f64(res_f)[y0:y0 + hh, x0:x0 + ww]
    want = oracle.select_blocks(new_full, f64(cache), blocks, b, b)
    assert_close(y3, want, td, "scatter+residual", tol=1e-6 if td == torch.float32 else 2e-3)
    out = outside_blocks_mask(blocks, b, b, H, W)
    assert torch.equal(y3[torch.from_numpy(out).cuda()], cache[torch.from_numpy(out).cuda()])


# ------------------------------------------------------------------ a5: convolution on tiles

@pytest.mark.parametrize("dtype,Cin,Cout,b,k,s,n", [
    ("f32", 64, 64, 6, 3, 1, 9), ("f16", 128, 128, 16, 3, 1, 5), ("f16", 128, 256, 16, 1, 1, 5),
    ("bf16", 320, 320, 4, 1, 1, 7), ("f16", 64, 128, 8, 3, 2, 6), ("f32", 8, 3, 6, 3, 1, 4),
    ("bf16", 48, 40, 5, 3, 1, 11), ("f16", 16, 100, 32, 3, 1, 2), ("f16", 256, 64, 16, 3, 1, 3),
    ("f16", 96, 64, 16, 3, 1, 3), ("f32", 24, 16, 8, 3, 1, 4)])      # chunks of three K steps
def test_conv_on_tiles(oracle, dtype, Cin, Cout, b, k, s, n):
    rng = np.random.default_rng(Cin * 7 + Cout)
    td = DT[dtype]
    g = api.geom(64 * s, 64 * s, b, k, s, k // 2)
    th, tw = g.tile_h, g.tile_w
    tiles = torch.from_numpy(rng.standard_normal((n, th, tw, Cin)).astype(np.float32)).to(td)
    w, bias = inputs.conv_params(rng, Cout, Cin, k, td)
    want = np.stack([oracle.conv2d(f64(tiles[i]), f64(w), f64(bias), s, 0) for i in range(n)])
    assert want.shape == (n, b, b, Cout)
    packed = api.sige_pack_weight(dev(w))
    cnt = torch.tensor([n], dtype=torch.int32, device="cuda")
    for cfg in (None, 0, 1, 2, 3):        # the automatic choice, then every workgroup shape forced in turn
        if cfg is not None and b > (128 if cfg in (0, 1) else 64):
            continue
        with api.knobs(CONV_CFG=cfg):
            out = torch.full((n + 1, b, b, Cout), 5.0, dtype=td, device="cuda")
            try:
                api.sige_conv(dev(tiles), g, Cin, Cout, packed, dev(bias), cnt, out, n_blocks=n, max_blocks=n)
            except api.SigeError as e:
                # the K-split shape needs Cin to be a multiple of four K steps
                assert cfg == 3 and e.code == 2 and Cin % (64 if td != torch.float32 else 32) != 0
                continue
            assert_close(out[:n], want, td, f"conv cfg={cfg}")
            assert (out[n:] == 5.0).all()
            out2 = torch.full((n + 1, b, b, Cout), 5.0, dtype=td, device="cuda")
            big = torch.cat([dev(tiles), torch.zeros((3, th, tw, Cin), dtype=td, device="cuda")])
            api.sige_conv(big, g, Cin, Cout, packed, None, cnt, out2, n_blocks=-1, max_blocks=n + 1)
            want_nb = want - f64(bias)[None, None, None, :]
            assert_close(out2[:n], want_nb, td, f"conv no-bias device-count cfg={cfg}")
            assert (out2[n:] == 5.0).all()
    assert api.sige_get_knob("CONV_CFG") == -1


@pytest.mark.parametrize("dtype,Cin,Cout,b,k", [("f16", 128, 128, 16, 3), ("bf16", 64, 72, 8, 1), ("f32", 32, 40, 6, 3)])
def test_conv_epilogue_from_registers_equals_the_one_through_lds(oracle, dtype, Cin, Cout, b, k):
    """The shapes whose waves do not split K send whole channel runs straight from the accumulator
    registers (a lane owns a pixel); forced through LDS instead (the path ragged channel counts, the
    gated GELU and K splits over workgroups take) they write the same bits: tiles, scatter with both
    residuals, activated copies; and both match the oracle."""
    rng = np.random.default_rng(Cin + Cout + b)
    td = DT[dtype]
    res = 5 * b - 2                               # ragged edge blocks
    x = torch.from_numpy(rng.standard_normal((res, res, Cin)).astype(np.float32)).to(td).cuda()
    w, bias = inputs.conv_params(rng, Cout, Cin, k, td)
    conv = SigeConv(dev(w), bias, res, res, b, 1, k // 2)
    bl = BlockList(conv.g, "cuda").all_active()
    n = bl.n_host
    resid = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td).cuda()
    rt = torch.from_numpy(rng.standard_normal((n, b, b, Cout)).astype(np.float32)).to(td).cuda()
    sc = torch.from_numpy(rng.uniform(0.5, 1.5, Cout).astype(np.float32)).cuda()
    sh = torch.from_numpy(rng.uniform(-0.5, 0.5, Cout).astype(np.float32)).cuda()
    ws = Workspace("cuda")
    want = oracle.conv2d(f64(x), f64(w), f64(bias), 1, k // 2)
    rt_full = np.zeros((res, res, Cout))
    for i, (y0, x0) in enumerate(bl.indices[:n].cpu().numpy()):
        h, wd = min(b, res - y0), min(b, res - x0)
        rt_full[y0:y0 + h, x0:x0 + wd] = f64(rt[i])[:h, :wd]
    for cfg in (0, 1, 2):
        if b * b > (128 if cfg < 2 else 64) and b > (128 if cfg < 2 else 64):
            continue
        outs = []
        for direct in (None, 0):
            with api.knobs(CONV_CFG=cfg, CONV_DIRECT=direct):
                y = torch.full((res, res, Cout), float("nan"), dtype=td, device="cuda")
                copy = torch.full((res, res, Cout), float("nan"), dtype=td, device="cuda")
                conv.forward(x, y, bl, ws, residual_tiles=rt, residual=resid, fused=True,
                             act_outs=[(copy, sc, sh, api.ACT_SILU)])
                tiles = conv.forward(x, None, bl, ws, scatter=False, fused=True).clone()
                outs.append((y, copy, tiles))
        for a_, b_ in zip(*outs):
            assert torch.equal(a_, b_), f"shape {cfg}: registers and LDS epilogues differ"
        assert_close(outs[0][0], want + rt_full + f64(resid), td, f"shape {cfg}: convolution + both residuals")
        z = oracle.scale_shift_act(f64(outs[0][0]), f64(sc), f64(sh), oracle.ACT_SILU)
        assert_close(outs[0][1], z, td, f"shape {cfg}: activated copy")


@pytest.mark.parametrize("dtype,Cin,Cout,res,b,k", [
    ("f16", 512, 96, 8, 8, 3), ("bf16", 384, 136, 16, 16, 3), ("f32", 192, 32, 8, 8, 3),
    ("f16", 384, 64, 8, 4, 1), ("f16", 512, 33, 12, 8, 3),
    # the whole of Cin (or half) staged at once, waves split K: 320 (four waves), 640, 2 x 640
    ("bf16", 320, 72, 16, 8, 3), ("f16", 640, 40, 16, 8, 3), ("bf16", 1280, 64, 8, 8, 3),
    ("f16", 320, 64, 10, 4, 3), ("f32", 160, 32, 12, 8, 3), ("f32", 320, 40, 8, 8, 3)])
def test_conv_k_split_over_workgroups(oracle, dtype, Cin, Cout, res, b, k):
    """Few blocks, many input channels: with a workspace the call is cut along K over several
    workgroups and a second kernel adds the shares.  Against the oracle; the workspace is poisoned
    (no state is assumed); three calls and the fused call agree bit for bit; residuals included."""
    rng = np.random.default_rng(Cin + Cout + res)
    td = DT[dtype]
    x = torch.from_numpy(rng.standard_normal((res, res, Cin)).astype(np.float32)).to(td)
    w, bias = inputs.conv_params(rng, Cout, Cin, k, td)
    resid = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td)
    conv = SigeConv(dev(w), bias, res, res, b, 1, k // 2)
    g = conv.g
    nb = api.sige_conv_workspace_bytes(td, g, Cin, Cout, g.grid_blocks)
    assert nb > 0 and nb % 4 == 0, "this shape is meant to split"
    ws = Workspace("cuda")
    ws.get("split_k", nb // 4, torch.float32).fill_(float("nan"))
    bl = BlockList(g, "cuda").all_active()
    want = oracle.conv2d(f64(x), f64(w), f64(bias), 1, k // 2)
    three_calls = Cout % 8 == 0      # the scatter call needs 16-byte channel runs; the fused call does not
    for device_count in (False, True):
        bl.n_host = -1 if device_count else g.grid_blocks
        y_f = torch.full((res, res, Cout), float("nan"), dtype=td, device="cuda")
        conv.forward(dev(x), y_f, bl, ws, residual=dev(resid), fused=True)
        if three_calls:
            # the three calls store the output tiles (rounded once) before the scatter adds the residual ...
            y = torch.full((res, res, Cout), float("nan"), dtype=td, device="cuda")
            conv.forward(dev(x), y, bl, ws, residual=dev(resid))
            assert_close(y, round_to(want, td) + f64(resid), td, "gather + conv + scatter under a K split, residual")
            # ... and without a residual they and the fused call write the same bits
            y0 = torch.full((res, res, Cout), float("nan"), dtype=td, device="cuda")
            conv.forward(dev(x), y0, bl, ws)
            y0f = torch.full((res, res, Cout), float("nan"), dtype=td, device="cuda")
            conv.forward(dev(x), y0f, bl, ws, fused=True)
            assert torch.equal(y0, y0f), "fused call differs from gather + conv + scatter under a K split"
        # the fused call adds the residual to the fp32 sums and rounds once
        assert_close(y_f, want + f64(resid), td, "k-split + residual")
    # without a workspace: the unsplit kernel; same values up to the rounding order of the fp32 sum
    y_n = torch.full((res, res, Cout), float("nan"), dtype=td, device="cuda")
    conv.forward(dev(x), y_n, bl, ws, split_k=False, fused=True)
    y_s = torch.full((res, res, Cout), float("nan"), dtype=td, device="cuda")
    conv.forward(dev(x), y_s, bl, ws, fused=True)
    assert_close(y_n, want, td, "unsplit")
    assert_close(y_s, want, td, "k-split")
    # a partial list: only some blocks active, the rest of y untouched
    if g.grid_blocks >= 2:
        blp = BlockList(g, "cuda")
        m = np.zeros((res, res), np.uint8)
        m[0, 0] = 1
        blp.reduce(mask_in=torch.from_numpy(m).cuda())
        n = blp.sync_count()
        assert 0 < n < g.grid_blocks
        cache = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td)
        y = dev(cache).clone()
        conv.forward(dev(x), y, blp, ws, fused=not three_calls)
        blocks = blp.indices[:n].cpu().numpy()
        assert_close(y, oracle.select_blocks(want, f64(cache), blocks, b, b), td, "k-split sparse")
        out = torch.from_numpy(outside_blocks_mask(blocks, b, b, res, res)).cuda()
        assert torch.equal(y[out], dev(cache)[out])


@pytest.mark.parametrize("dtype,Cin,Cout,res,b,n", [
    ("bf16", 320, 320, 22, 5, 9), ("bf16", 1280, 200, 16, 8, 4), ("f16", 512, 100, 16, 16, 1),
    ("f32", 192, 72, 20, 6, 11), ("f16", 2560, 64, 8, 8, 1), ("bf16", 640, 36, 13, 4, 16)])
def test_conv_pointwise_few_rows(oracle, dtype, Cin, Cout, res, b, n):
    """1x1 convolutions on few rows with a long K take the kernel whose waves split K (no workspace,
    no second kernel): stacked tiles and the fused call, one and two output-channel tiles per
    workgroup, ragged rows (blocks of 25 or 36 pixels, blocks that stick out of the image), channel
    counts that are no multiple of 8, both count paths, both residuals."""
    rng = np.random.default_rng(Cin + Cout + res)
    td = DT[dtype]
    x = torch.from_numpy(rng.standard_normal((res, res, Cin)).astype(np.float32)).to(td)
    w, bias = inputs.conv_params(rng, Cout, Cin, 1, td)
    resid = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td)
    cache = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td)
    conv = SigeConv(dev(w), bias, res, res, b, 1, 0)
    g = conv.g
    bl = BlockList(g, "cuda", max_blocks=max(g.grid_blocks, n + 2)).all_active()
    pick = np.sort(rng.permutation(g.grid_blocks)[:n])
    if g.grid_blocks - 1 not in pick:
        pick[-1] = g.grid_blocks - 1          # the bottom-right block: partly outside when b does not divide res
    blocks = bl.indices[torch.from_numpy(pick).cuda()].clone()
    bl.indices.fill_(0)
    bl.indices[:n].copy_(blocks)
    bl.count.fill_(n)
    blocks = blocks.cpu().numpy()
    want_full = oracle.conv2d(f64(x), f64(w), f64(bias), 1, 0)
    want = oracle.select_blocks(want_full + f64(resid), f64(cache), blocks, b, b)
    out_mask = torch.from_numpy(outside_blocks_mask(blocks, b, b, res, res)).cuda()
    ws = Workspace("cuda")
    for mode in (None, "1", "2", "3", "2 with four waves"):
        # the automatic choice, then every patch of the few-row kernel forced in turn; the last is the
        # 64 x 64 shape as it runs when there are more patches than compute units
        kn = dict(CONV_POINTWISE=None if mode is None else int(mode[0]), CONV_POINTWISE_W4=1 if mode and len(mode) > 1 else None)
        with api.knobs(**kn):
            for device_count in (False, True):
                bl.n_host = -1 if device_count else n
                bl.max_blocks = n + 2 if device_count else g.grid_blocks
                y = dev(cache).clone()
                conv.forward(dev(x), y, bl, ws, residual=dev(resid), fused=True)
                assert_close(y, want, td, f"pointwise fused mode={mode} device_count={device_count}")
                assert torch.equal(y[out_mask], dev(cache)[out_mask])
            # stacked tiles (what the token-wise layers of a transformer block call), bias only
            bl.n_host, bl.max_blocks = n, g.grid_blocks
            tiles = torch.from_numpy(rng.standard_normal((n, b, b, Cin)).astype(np.float32)).to(td)
            want_t = np.stack([oracle.conv2d(f64(tiles[i]), f64(w), f64(bias), 1, 0) for i in range(n)])
            out = torch.full((n + 1, b, b, Cout), 5.0, dtype=td, device="cuda")
            api.sige_conv(dev(tiles), g, Cin, Cout, conv.packed, conv.bias, bl.count, out, n_blocks=n, max_blocks=n)
            assert_close(out[:n], want_t, td, f"pointwise tiles mode={mode}")
            assert (out[n:] == 5.0).all()
            if Cout % 8 == 0:
                # tile residual through the fused call (one rounding of convolution + residuals) and through
                # the three calls (the output tiles are stored, hence rounded, before the scatter adds)
                rt = out[:n].contiguous()
                rt_full = np.zeros((res, res, Cout))
                for i, (y0, x0) in enumerate(blocks):
                    h, wd = min(b, res - y0), min(b, res - x0)
                    rt_full[y0:y0 + h, x0:x0 + wd] = f64(rt[i])[:h, :wd]
                y3 = dev(cache).clone()
                conv.forward(dev(x), y3, bl, ws, residual_tiles=rt, residual=dev(resid))
                yf = dev(cache).clone()
                conv.forward(dev(x), yf, bl, ws, residual_tiles=rt, residual=dev(resid), fused=True)
                assert_close(yf, oracle.select_blocks(want_full + rt_full + f64(resid), f64(cache), blocks, b, b), td,
                             f"fused, both residuals mode={mode}")
                assert_close(y3, oracle.select_blocks(round_to(want_full, td) + rt_full + f64(resid), f64(cache), blocks,
                                                      b, b), td, f"three calls, both residuals mode={mode}")
    # the tiled kernel on the same call: same values up to the order of the fp32 sums
    with api.knobs(CONV_POINTWISE=0):
        y0 = dev(cache).clone()
        conv.forward(dev(x), y0, bl, ws, residual=dev(resid), fused=True)
        assert_close(y0, want, td, "tiled kernel on the same call")


@pytest.mark.parametrize("dtype,Cin,Cout,res,b,k,n", [
    ("bf16", 320, 320, 22, 5, 1, 9), ("f16", 1280, 64, 16, 8, 1, 3), ("f16", 128, 128, 40, 16, 3, 4),
    ("f16", 512, 96, 16, 8, 3, 4), ("f32", 64, 40, 20, 6, 3, 7)])
def test_conv_scatter(oracle, dtype, Cin, Cout, res, b, k, n):
    """The convolution on stacked tiles with the scatter folded into its epilogue: bit for bit what
    sige_conv followed by sige_scatter give (few-row kernel, tiled kernel, K split with a workspace),
    residuals included, both count paths; against the oracle; y outside the blocks untouched."""
    rng = np.random.default_rng(Cin + Cout + res + k)
    td = DT[dtype]
    w, bias = inputs.conv_params(rng, Cout, Cin, k, td)
    conv = SigeConv(dev(w), bias, res, res, b, 1, k // 2)
    g = conv.g
    nby = -(-res // b)
    pick = np.unique(np.append(rng.permutation(nby * nby)[:n - 1], nby * nby - 1))
    blocks = np.array([((i // nby) * b, (i % nby) * b) for i in pick], np.int32)
    n = len(blocks)
    idx = torch.from_numpy(blocks).cuda()
    cnt = torch.tensor([n], dtype=torch.int32, device="cuda")
    tiles = torch.from_numpy(rng.standard_normal((n + 1, g.tile_h, g.tile_w, Cin)).astype(np.float32)).to(td).cuda()
    resid = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td).cuda()
    rtiles = torch.from_numpy(rng.standard_normal((n + 1, b, b, Cout)).astype(np.float32)).to(td).cuda()
    cache = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td).cuda()
    nbytes = api.sige_conv_workspace_bytes(td, g, Cin, Cout, n + 1)
    split = torch.full((max(nbytes // 4, 1),), float("nan"), device="cuda") if nbytes else None
    out_mask = torch.from_numpy(outside_blocks_mask(blocks, b, b, res, res)).cuda()
    vec = Cout % (4 if dtype == "f32" else 8) == 0       # sige_scatter needs 16-byte channel runs
    for nb, mb in ((n, n), (-1, n + 1)):
        for rt, rf in ((None, None), (rtiles, resid)):
            y = cache.clone()
            api.sige_conv_scatter(tiles, g, idx, cnt, Cin, Cout, conv.packed, conv.bias, y, n_blocks=nb, max_blocks=mb,
                                  residual_tiles=rt, residual=rf, workspace=split)
            assert torch.equal(y[out_mask], cache[out_mask])
            if vec:
                o = torch.empty((n + 1, b, b, Cout), dtype=td, device="cuda")
                api.sige_conv(tiles, g, Cin, Cout, conv.packed, conv.bias, cnt, o, n_blocks=nb, max_blocks=mb, workspace=split)
                y2 = cache.clone()
                api.sige_scatter(o, g, idx, cnt, y2, n_blocks=nb, residual_tiles=rt, residual=rf, max_blocks=mb)
                if rt is None:
                    assert torch.equal(y, y2), "conv + scatter folded differs from the two calls"
            want_t = np.stack([oracle.conv2d(f64(tiles[i]), f64(w), f64(bias), 1, 0) for i in range(n)])
            want = f64(cache)
            for i, (y0, x0) in enumerate(blocks):
                h, wd = min(b, res - y0), min(b, res - x0)
                blk = want_t[i][:h, :wd]              # convolution plus residuals, rounded once
                if rt is not None:
                    blk = blk + f64(rtiles[i])[:h, :wd] + f64(resid)[y0:y0 + h, x0:x0 + wd]
                want[y0:y0 + h, x0:x0 + wd] = blk
            assert_close(y, want, td, f"conv_scatter n_blocks={nb} residuals={rt is not None}")


@pytest.mark.parametrize("dtype,Cin,Cout,res,b,k,n", [
    ("f16", 128, 128, 40, 16, 3, 4), ("bf16", 320, 64, 22, 5, 1, 9), ("f16", 512, 96, 16, 8, 3, 4),
    ("f32", 64, 40, 20, 6, 3, 7)])
def test_fused_conv_activated_copies(oracle, dtype, Cin, Cout, res, b, k, n):
    """Activated copies of the output (the next layers' Scale+Shift and nonlinearity applied by the
    producing layer): y is what the call gives without copies; inside the active blocks every copy is
    bit for bit what a fused gather of y with the same scale, shift and activation reads, and within
    tolerance of the oracle's; outside the blocks the copies are untouched.  Tiled kernel, few-row
    kernel and K split; residual included."""
    rng = np.random.default_rng(Cin + Cout + res + k)
    td = DT[dtype]
    x = torch.from_numpy(rng.standard_normal((res, res, Cin)).astype(np.float32)).to(td).cuda()
    w, bias = inputs.conv_params(rng, Cout, Cin, k, td)
    conv = SigeConv(dev(w), bias, res, res, b, 1, k // 2)
    g = conv.g
    g1 = api.geom(res, res, b, 1, 1, 0)
    nby = -(-res // b)
    pick = np.unique(np.append(rng.permutation(nby * nby)[:n - 1], nby * nby - 1))
    blocks = np.array([((i // nby) * b, (i % nby) * b) for i in pick], np.int32)
    n = len(blocks)
    bl = BlockList(g, "cuda", max_blocks=n + 1)
    bl.indices[:n].copy_(torch.from_numpy(blocks))
    bl.count.fill_(n)
    resid = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td).cuda()
    cache = torch.from_numpy(rng.standard_normal((res, res, Cout)).astype(np.float32)).to(td).cuda()
    ws = Workspace("cuda")
    acts = [api.ACT_SILU, api.ACT_NONE, api.ACT_RELU]
    wide = torch.full((res, res, 2 * Cout + 16), 3.0, dtype=td, device="cuda")     # two copies share a wider buffer
    lone = torch.full((res, res, Cout), 3.0, dtype=td, device="cuda")
    scales = [torch.from_numpy(rng.uniform(0.5, 1.5, Cout).astype(np.float32)).cuda() for _ in acts]
    shifts = [torch.from_numpy(rng.uniform(-0.5, 0.5, Cout).astype(np.float32)).cuda() for _ in acts]
    copies = [wide[:, :, :Cout], wide[:, :, Cout + 16:], lone]
    spec = [(copies[0], scales[0], shifts[0], acts[0]), (copies[1], scales[1], shifts[1], acts[1]),
            (copies[2], None, None, acts[2])]
    out_mask = torch.from_numpy(outside_blocks_mask(blocks, b, b, res, res)).cuda()
    for nb in (n, -1):
        bl.n_host = nb
        y0 = cache.clone()
        conv.forward(x, y0, bl, ws, residual=resid, fused=True)
        y = cache.clone()
        wide.fill_(3.0)
        lone.fill_(3.0)
        conv.forward(x, y, bl, ws, residual=resid, fused=True, act_outs=spec)
        assert torch.equal(y, y0)
        idx = bl.indices[:n].contiguous()
        cnt = bl.count
        for j, c in enumerate(copies):
            assert (c[out_mask] == 3.0).all()
            got = torch.empty((n, b, b, Cout), dtype=td, device="cuda")
            api.sige_gather(c, g1, idx, cnt, got, n_blocks=n, C=Cout)
            ref = torch.empty((n, b, b, Cout), dtype=td, device="cuda")
            api.sige_gather(y, g1, idx, cnt, ref, n_blocks=n, C=Cout, scale=spec[j][1], shift=spec[j][2], act=acts[j])
            # rows of blocks that stick out of the image are zero padding in both gathers
            assert torch.equal(got, ref), f"copy {j} differs from a fused gather of y"
            want = expected_tiles(oracle, f64(y), blocks, b, b, 1, 0,
                                  None if spec[j][1] is None else f64(spec[j][1]),
                                  None if spec[j][2] is None else f64(spec[j][2]), acts[j])
            assert_close(got, want, td, f"activated copy {j}")
        assert (wide[:, :, Cout:Cout + 16] == 3.0).all()


# ------------------------------------------------------------------ the whole layer

def sparse_layer(cfg, *, fused, shortcut=False, device_count=False, cache=None):
    """reduce -> gather -> conv -> scatter through the library; returns (y, blocks, extras)."""
    td = DT[cfg["dtype"]]
    H, W = cfg["H"], cfg["W"]
    conv = SigeConv(dev(cfg["w"]), cfg["bias"], H, W, cfg["block"], cfg["stride"], cfg["pad"])
    ws = Workspace("cuda")
    bl = BlockList(conv.g, "cuda")
    mask_out = torch.zeros((H, W), dtype=torch.uint8, device="cuda")
    a_o, a_e = dev(cfg["a_orig"]), dev(cfg["a_edit"])
    bl.reduce(a_orig=a_o, a_edit=a_e, tau=cfg["tau"], mask_out=mask_out, dilate=cfg["dilate"])
    if not device_count:
        bl.sync_count()
    y = dev(cache).clone()
    scale = shift = None
    act = api.ACT_NONE
    if fused:
        mean = torch.zeros(cfg["groups"], device="cuda")
        var = torch.zeros(cfg["groups"], device="cuda")
        scale = torch.zeros(cfg["Cin"], device="cuda")
        shift = torch.zeros(cfg["Cin"], device="cuda")
        # statistics of the ORIGINAL activation (Sec. 3.2 "Pre-computing normalization parameters")
        api.sige_gn_stats(a_o, cfg["groups"], mean, var, gamma=dev(cfg["gamma"]), beta=dev(cfg["beta"]),
                          eps=cfg["eps"], scale=scale, shift=shift)
        act = api.ACT_SILU
    conv.forward(a_e, y, bl, ws, scale=scale, shift=shift, act=act)
    # the fused call (gather -> LDS -> MFMA -> scatter in one kernel) must give the same bits
    y_f = dev(cache).clone()
    conv.forward(a_e, y_f, bl, ws, scale=scale, shift=shift, act=act, fused=True)
    torch.cuda.synchronize()
    assert torch.equal(y, y_f), "fused call differs from gather + conv + scatter"
    n = int(bl.count.item())
    return y, bl.indices[:n].cpu().numpy(), mask_out.cpu().numpy()


@pytest.mark.parametrize("seed", [1001, 1002, 1003, 1004])
@pytest.mark.parametrize("device_count", [False, True])
def test_layer_config1(oracle, seed, device_count):
    cfg = inputs.config1(seed=seed)
    a_o, a_e, w, b = f64(cfg["a_orig"]), f64(cfg["a_edit"]), f64(cfg["w"]), f64(cfg["bias"])
    cache64 = oracle.conv2d(a_o, w, b, 1, 1)
    cache = torch.from_numpy(cache64).to(torch.float32)
    y, blocks, mask = sparse_layer(cfg, fused=False, device_count=device_count, cache=cache)
    want_blocks = oracle.active_blocks(oracle.diff_mask(cfg["a_orig"].numpy(), cfg["a_edit"].numpy(), cfg["tau"]),
                                       64, 64, 6, 6, 3, 1, 1)
    assert np.array_equal(blocks, want_blocks)
    want = oracle.sige_layer(a_e, f64(cache), blocks, 6, 6, w, b, 1, 1)
    assert_close(y, want, torch.float32, "config1 layer")
    # with the true difference mask the sparse result is the dense layer on the edited input
    assert_close(y, oracle.conv2d(a_e, w, b, 1, 1), torch.float32, "config1 == dense")
    out = torch.from_numpy(outside_blocks_mask(blocks, 6, 6, 64, 64)).cuda()
    assert torch.equal(y[out], cache.cuda()[out])  # outside the active blocks: the cache, bit for bit


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_layer_config2_small_fused(oracle, dtype):
    cfg = inputs.config2(seed=7, H=96, W=80, C=64, Cs=128, area_frac=0.02, dtype=dtype, axes=(3.0, 8.0))
    td = DT[dtype]
    a_o, a_e = f64(cfg["a_orig"]), f64(cfg["a_edit"])
    w, b = f64(cfg["w"]), f64(cfg["bias"])
    mean, var = oracle.gn_stats(a_o, cfg["groups"])
    scale, shift = oracle.fold_gn(f64(cfg["gamma"]), f64(cfg["beta"]), mean, var, cfg["eps"])
    cache64 = oracle.dense_layer(a_o, w, b, 1, 1, scale, shift, oracle.ACT_SILU)
    cache = torch.from_numpy(cache64).to(td)
    y, blocks, mask = sparse_layer(cfg, fused=True, cache=cache)
    m = oracle.diff_mask(cfg["a_orig"].float().numpy(), cfg["a_edit"].float().numpy(), cfg["tau"])
    assert np.array_equal(mask, m)
    assert np.array_equal(blocks, oracle.active_blocks(m, 96, 80, 16, 16, 3, 1, 1))
    # element-wise bar against the oracle whose gathered (activated) tensor is a stored tensor of
    # the layer's dtype; and against the oracle with no intermediate rounding at all
    want = oracle.sige_layer(a_e, f64(cache), blocks, 16, 16, w, b, 1, 1, scale, shift, oracle.ACT_SILU,
                             storage=dtype)
    assert_close(y, want, td, "config2 small")
    want = oracle.sige_layer(a_e, f64(cache), blocks, 16, 16, w, b, 1, 1, scale, shift, oracle.ACT_SILU)
    assert_mostly_close(y, want, td, "config2 small vs unrounded oracle")
    out = torch.from_numpy(outside_blocks_mask(blocks, 16, 16, 96, 80)).cuda()
    assert torch.equal(y[out], cache.cuda()[out])
    # the statistics really are the cached ones: with statistics of the EDITED tensor the oracle differs
    mean_e, var_e = oracle.gn_stats(a_e, cfg["groups"])
    assert np.abs(mean_e - mean).max() > 0


def test_layer_config2_shortcut_and_residual(oracle):
    """1x1 shortcut conv on the same mask (its own k=1 list) and a ResBlock-style tail:
    scatter(main + shortcut tiles)."""
    cfg = inputs.config2(seed=11, H=64, W=64, C=64, Cs=64, area_frac=0.03, dtype="f16", axes=(3.0, 8.0))
    td = torch.float16
    a_o, a_e = f64(cfg["a_orig"]), f64(cfg["a_edit"])
    ws_, bs_ = f64(cfg["w_s"]), f64(cfg["bias_s"])
    m = oracle.diff_mask(cfg["a_orig"].float().numpy(), cfg["a_edit"].float().numpy(), 0.0)
    # shortcut alone, with its own list
    sc = SigeConv(dev(cfg["w_s"]), cfg["bias_s"], 64, 64, 16, 1, 0)
    bl1 = BlockList(sc.g, "cuda")
    bl1.reduce(mask_in=torch.from_numpy(m).cuda())
    n1 = bl1.sync_count()
    want1 = oracle.active_blocks(m, 64, 64, 16, 16, 1, 1, 0)
    assert n1 == len(want1) and np.array_equal(bl1.indices[:n1].cpu().numpy(), want1)
    cache_s = torch.from_numpy(oracle.conv2d(a_o, ws_, bs_, 1, 0)).to(td)
    y = dev(cache_s).clone()
    wsp = Workspace("cuda")
    sc.forward(dev(cfg["a_edit"]), y, bl1, wsp)
    want = oracle.sige_layer(a_e, f64(cache_s), want1, 16, 16, ws_, bs_, 1, 0)
    assert_close(y, want, td, "shortcut 1x1")
    assert_close(y, oracle.conv2d(a_e, ws_, bs_, 1, 0), td, "shortcut == dense")
    # main 3x3 + shortcut on the 3x3 list, summed in the scatter
    main = SigeConv(dev(cfg["w"]), cfg["bias"], 64, 64, 16, 1, 1)
    bl3 = BlockList(main.g, "cuda")
    bl3.reduce(mask_in=torch.from_numpy(m).cuda())
    bl3.sync_count()
    blocks3 = bl3.indices[:bl3.n_host].cpu().numpy()
    sc3 = SigeConv(dev(cfg["w_s"]), cfg["bias_s"], 64, 64, 16, 1, 0)
    w, b = f64(cfg["w"]), f64(cfg["bias"])
    dense_sum = lambda a: oracle.conv2d(a, w, b, 1, 1) + oracle.conv2d(a, ws_, bs_, 1, 0)
    cache_sum = torch.from_numpy(dense_sum(a_o)).to(td)
    y = dev(cache_sum).clone()
    res_tiles = sc3.forward(dev(cfg["a_edit"]), None, bl3, wsp, scatter=False, tag="s")
    main.forward(dev(cfg["a_edit"]), y, bl3, wsp, residual_tiles=res_tiles, tag="m")
    want = oracle.select_blocks(dense_sum(a_e), f64(cache_sum), blocks3, 16, 16)
    assert_close(y, want, td, "main + shortcut")
    y_f = dev(cache_sum).clone()
    res_f = sc3.forward(dev(cfg["a_edit"]), None, bl3, wsp, scatter=False, tag="sf", fused=True)
    assert torch.equal(res_f, res_tiles)
    full_res = dev(cfg["a_orig"])[:, :, :64].contiguous()
    main.forward(dev(cfg["a_edit"]), y_f, bl3, wsp, residual_tiles=res_f, tag="mf", fused=True)
    # the fused call adds the shortcut tiles to the fp32 sums and rounds once; the three calls round the
    # stored output tiles first: each against the oracle's statement of what it computes
    short_rounded = round_to(oracle.conv2d(a_e, ws_, bs_, 1, 0), td)            # the shortcut tiles are a stored tensor
    main_e = oracle.conv2d(a_e, w, b, 1, 1)
    assert_close(y_f, oracle.select_blocks(main_e + short_rounded, f64(cache_sum), blocks3, 16, 16), td,
                 "fused main + shortcut tiles")
    assert_close(y, oracle.select_blocks(round_to(main_e, td) + short_rounded, f64(cache_sum), blocks3, 16, 16), td,
                 "three calls, main + shortcut tiles")
    # both residual kinds at once, three calls and fused
    y1, y2 = dev(cache_sum).clone(), dev(cache_sum).clone()
    main.forward(dev(cfg["a_edit"]), y1, bl3, wsp, residual_tiles=res_tiles, residual=full_res, tag="m")
    main.forward(dev(cfg["a_edit"]), y2, bl3, wsp, residual_tiles=res_f, residual=full_res, tag="mf", fused=True)
    both = short_rounded + f64(full_res)
    assert_close(y2, oracle.select_blocks(main_e + both, f64(cache_sum), blocks3, 16, 16), td, "fused, both residuals")
    assert_close(y1, oracle.select_blocks(round_to(main_e, td) + both, f64(cache_sum), blocks3, 16, 16), td,
                 "three calls, both residuals")


def test_layer_all_active_equals_dense_and_zero_blocks(oracle):
    cfg = inputs.config2(seed=3, H=40, W=56, C=32, Cs=32, area_frac=0.05, dtype="f16", axes=(2.0, 5.0))
    td = torch.float16
    conv = SigeConv(dev(cfg["w"]), cfg["bias"], 40, 56, 16, 1, 1)
    ws = Workspace("cuda")
    bl = BlockList(conv.g, "cuda").all_active()
    y = torch.full((40, 56, 32), float("nan"), dtype=td, device="cuda")  # every element must be written
    conv.forward(dev(cfg["a_edit"]), y, bl, ws)
    want = oracle.conv2d(f64(cfg["a_edit"]), f64(cfg["w"]), f64(cfg["bias"]), 1, 1)
    assert_close(y, want, td, "all active == dense")
    y_f = torch.full((40, 56, 32), float("nan"), dtype=td, device="cuda")
    conv.forward(dev(cfg["a_edit"]), y_f, bl, ws, fused=True)
    assert torch.equal(y, y_f)
    # no active block: y untouched bitwise, through both count paths
    poison = torch.from_numpy(np.random.default_rng(1).standard_normal((40, 56, 32)).astype(np.float32)).to(td).cuda()
    y = poison.clone()
    bl.reduce(mask_in=torch.zeros((40, 56), dtype=torch.uint8, device="cuda"))
    conv.forward(dev(cfg["a_edit"]), y, bl, ws)
    conv.forward(dev(cfg["a_edit"]), y, bl, ws, fused=True)
    bl.sync_count()
    conv.forward(dev(cfg["a_edit"]), y, bl, ws)
    conv.forward(dev(cfg["a_edit"]), y, bl, ws, fused=True)
    torch.cuda.synchronize()
    assert torch.equal(y, poison)


def test_layer_stride2_and_upsample(oracle):
    rng = np.random.default_rng(21)
    td = torch.float16
    H, W, C = 64, 48, 32
    mask = inputs.blob_mask(rng, H, W, 60, 2, (2.0, 5.0))
    a_o, a_e = inputs.edited_pair(rng, H, W, C, mask, 1.0, td)
    w, b = inputs.conv_params(rng, 64, C, 3, td)
    # stride-2 down-sampling conv
    conv = SigeConv(dev(w), b, H, W, 8, 2, 1)
    bl = BlockList(conv.g, "cuda")
    bl.reduce(mask_in=torch.from_numpy(mask).cuda())
    n = bl.sync_count()
    want_blocks = oracle.active_blocks(mask, 32, 24, 8, 8, 3, 2, 1)
    assert np.array_equal(bl.indices[:n].cpu().numpy(), want_blocks) and 0 < n < 12
    cache = torch.from_numpy(oracle.conv2d(f64(a_o), f64(w), f64(b), 2, 1)).to(td)
    y = dev(cache).clone()
    conv.forward(dev(a_e), y, bl, Workspace("cuda"))
    assert_close(y, oracle.conv2d(f64(a_e), f64(w), f64(b), 2, 1), td, "stride 2 == dense")
    y_f = dev(cache).clone()
    conv.forward(dev(a_e), y_f, bl, Workspace("cuda"), fused=True)
    assert torch.equal(y, y_f)
    # nearest x2 up-sampling followed by a 3x3 conv, mask taken at the output resolution
    up_o = f64(a_o).repeat(2, axis=0).repeat(2, axis=1)
    up_e = f64(a_e).repeat(2, axis=0).repeat(2, axis=1)
    mask_up = mask.repeat(2, axis=0).repeat(2, axis=1)
    convu = SigeConv(dev(w), b, 2 * H, 2 * W, 16, 1, 1, up=1)
    blu = BlockList(convu.g, "cuda")
    blu.reduce(mask_in=torch.from_numpy(mask_up).cuda())
    blu.sync_count()
    cache = torch.from_numpy(oracle.conv2d(up_o, f64(w), f64(b), 1, 1)).to(td)
    y = dev(cache).clone()
    convu.forward(dev(a_e), y, blu, Workspace("cuda"))
    assert_close(y, oracle.conv2d(up_e, f64(w), f64(b), 1, 1), td, "upsample+conv == dense")
    y_f = dev(cache).clone()
    convu.forward(dev(a_e), y_f, blu, Workspace("cuda"), fused=True)
    assert torch.equal(y, y_f)


@pytest.mark.parametrize("area_frac", [0.01, 0.155])
def test_layer_config2_full_size(oracle, area_frac):
    """benchmark configuration 2 at full size (256x256x128 fp16, 16x16 blocks; ~1 % blobs, and the 15.5 %
    edit of the paper's micro-benchmark, Sec. 3.2), in the launch configuration the benchmark times;
    the oracle evaluates EVERY pixel of every active block.  The cache is an arbitrary seeded tensor:
    what must hold is 'dense layer on active blocks, cache bit for bit elsewhere'."""
    cfg = inputs.config2(area_frac=area_frac, n_blobs=3 if area_frac < 0.05 else 6, axes=(5.0, 12.0))
    td = torch.float16
    H = W = 256
    a_o, a_e = f64(cfg["a_orig"]), f64(cfg["a_edit"])
    mean, var = oracle.gn_stats(a_o, 32)
    scale, shift = oracle.fold_gn(f64(cfg["gamma"]), f64(cfg["beta"]), mean, var, cfg["eps"])
    rng = np.random.default_rng(99)
    cache = torch.from_numpy(rng.standard_normal((H, W, 128)).astype(np.float32)).to(td)
    y, blocks, mask = sparse_layer(cfg, fused=True, cache=cache)
    m = oracle.diff_mask(cfg["a_orig"].float().numpy(), cfg["a_edit"].float().numpy(), 0.0)
    target = area_frac * H * W
    assert np.array_equal(mask, m) and abs(int(m.sum()) - target) <= 0.05 * target
    want_blocks = oracle.active_blocks(m, H, W, 16, 16, 3, 1, 1)
    assert np.array_equal(blocks, want_blocks) and (3 <= len(blocks) <= 40 if area_frac < 0.05 else 40 <= len(blocks) <= 250)
    # which kernel ran: few blocks take the 64x32 shape whose four waves split K, the 15.5 % edit a
    # larger patch without a K split (the shape is chosen by how many workgroups the blocks make)
    plan = api.sige_conv_plan(td, api.geom(H, W, 16, 3, 1, 1), 128, 128, len(blocks), staged_math=True)
    assert plan.kernel == 0 and (plan.shape == 3 if area_frac < 0.05 else plan.shape in (0, 1, 2)), plan
    print(f"config 2 at {area_frac:.3f}: {len(blocks)} active blocks, {plan!r}")
    out = outside_blocks_mask(blocks, 16, 16, H, W)
    out_t = torch.from_numpy(out).cuda()
    assert torch.equal(y[out_t], cache.cuda()[out_t])
    # every pixel of every active block
    px = oracle.block_pixels(blocks, 16, 16, H, W)
    assert len(px) == 256 * len(blocks)
    got = y[torch.from_numpy(px[:, 0]).long().cuda(), torch.from_numpy(px[:, 1]).long().cuda()]
    want = oracle.dense_layer(a_e, f64(cfg["w"]), f64(cfg["bias"]), 1, 1, scale, shift, oracle.ACT_SILU, pixels=px,
                              storage="f16")
    assert_close(got, want, td, "config2 full size, all active pixels")
    # (second, informative check against the oracle that never rounds the activated tile)
    want = oracle.dense_layer(a_e, f64(cfg["w"]), f64(cfg["bias"]), 1, 1, scale, shift, oracle.ACT_SILU, pixels=px)
    assert_mostly_close(got, want, td, "config2 full size vs unrounded oracle")


def test_sequential_edits_incremental_cache(oracle):
    """Sec. 4.2 "Sequential edits", incremental pre-computation: after each edit the sparse pass has
    updated the cache in place, and the next edit is reduced against the previous edited input.  With
    true difference masks the cache equals the dense layer on the current input after every edit."""
    rng = np.random.default_rng(31)
    td = torch.float16
    H, W, C = 80, 64, 32
    w, b = inputs.conv_params(rng, C, C, 3, td)
    cur = torch.from_numpy(rng.standard_normal((H, W, C)).astype(np.float32)).to(td)
    conv = SigeConv(dev(w), b, H, W, 16, 1, 1)
    ws = Workspace("cuda")
    bl = BlockList(conv.g, "cuda")
    y = torch.from_numpy(oracle.conv2d(f64(cur), f64(w), f64(b), 1, 1)).to(td).cuda()
    mask_out = torch.zeros((H, W), dtype=torch.uint8, device="cuda")
    touched = 0
    for edit in range(5):
        m = inputs.blob_mask(rng, H, W, 40 + 30 * edit, 2, (2.0, 5.0), tol=0.2)
        nxt = torch.where(torch.from_numpy(m.astype(bool))[:, :, None],
                          cur + torch.from_numpy(rng.standard_normal((H, W, C)).astype(np.float32)).to(td), cur)
        bl.reduce(a_orig=dev(cur), a_edit=dev(nxt), tau=0.0, mask_out=mask_out)
        n = bl.sync_count()
        want_m = oracle.diff_mask(cur.float().numpy(), nxt.float().numpy(), 0.0)
        assert np.array_equal(mask_out.cpu().numpy(), want_m)
        assert np.array_equal(bl.indices[:n].cpu().numpy(), oracle.active_blocks(want_m, H, W, 16, 16, 3, 1, 1))
        conv.forward(dev(nxt), y, bl, ws, fused=(edit % 2 == 1))
        touched += n
        assert_close(y, oracle.conv2d(f64(nxt), f64(w), f64(b), 1, 1), td, f"cache after edit {edit}")
        cur = nxt
    assert 5 <= touched < 5 * conv.g.grid_blocks


@pytest.mark.parametrize("dtype,C,H,W,b,up,act", [("f16", 64, 40, 56, 16, 0, "leaky"), ("f32", 32, 24, 24, 6, 1, "none"),
                                                  ("bf16", 128, 32, 64, 8, 1, "leaky"), ("f16", 24, 20, 20, 5, 0, "relu")])
def test_gather_modulated(oracle, dtype, C, H, W, b, up, act):
    """Gather of a spatially-adaptive normalisation layer: per-channel scale/shift (cached statistics),
    per-pixel gamma | beta from a modulation tensor with a wider pixel stride, the activation, zero
    padding after everything; also through the x2 up-sampled view."""
    rng = np.random.default_rng(C + H + up)
    td = DT[dtype]
    code = {"none": (api.ACT_NONE, oracle.ACT_NONE), "relu": (api.ACT_RELU, oracle.ACT_RELU),
            "leaky": (api.ACT_LEAKY_RELU, oracle.ACT_LEAKY_RELU)}[act]
    hs, wsrc = (H >> up), (W >> up)
    x = torch.from_numpy(rng.standard_normal((hs, wsrc, C)).astype(np.float32)).to(td)
    ld = 2 * C + (8 if dtype != "f32" else 4)
    modbuf = torch.from_numpy((rng.standard_normal((H, W, ld)) * 0.4).astype(np.float32)).to(td)
    scale = torch.from_numpy(rng.uniform(0.5, 1.5, C).astype(np.float32))
    shift = torch.from_numpy(rng.uniform(-0.5, 0.5, C).astype(np.float32))
    g = api.geom(H, W, b, 3, 1, 1)
    blocks = random_blocks(rng, g, 7)
    n = len(blocks)
    idx = torch.from_numpy(blocks).cuda()
    cnt = torch.tensor([n], dtype=torch.int32, device="cuda")
    tiles = torch.full((n + 1, g.tile_h, g.tile_w, C), 5.0, dtype=td, device="cuda")
    api.sige_gather_modulated(dev(x), g, idx, cnt, tiles, dev(modbuf), n_blocks=n, scale=dev(scale), shift=dev(shift),
                              act=code[0], up=up, C=C, max_blocks=n)
    xin = f64(x).repeat(2, axis=0).repeat(2, axis=1) if up else f64(x)
    z = oracle.modulate(xin, f64(scale), f64(shift), f64(modbuf[:, :, :C]), f64(modbuf[:, :, C:2 * C]), code[1])
    want = expected_tiles(oracle, z, blocks, g.tile_h, g.tile_w, 1, 1, None, None, 0)   # z is already activated
    assert_close(tiles[:n], want, td, "modulated gather")
    assert (tiles[n:] == 5.0).all()
    # padding is zero after modulation and activation (beta would otherwise leak into it)
    pad_rows = [i for i, (y0, x0) in enumerate(blocks) if y0 == 0]
    if pad_rows:
        assert (tiles[pad_rows[0], 0] == 0).all()
    with pytest.raises(api.SigeError):
        api.sige_gather_modulated(dev(x), g, idx, cnt, tiles, dev(modbuf[:, :, :C]).contiguous(), n_blocks=n, C=C,
                                  up=up, max_blocks=n)          # modulation tensor narrower than 2C


@pytest.mark.parametrize("dtype,Cin,C3,C1,res,b,n", [
    ("f16", 128, 128, 256, 64, 16, 5),      # the two convolutions of benchmark configuration 2: one launch
    ("bf16", 64, 40, 72, 40, 8, 7),         # chunks of four K steps, output widths that are no multiples of 32
    ("f32", 64, 64, 32, 30, 6, 9),          # fp32, ragged blocks
    ("f16", 512, 64, 64, 16, 8, 2)])        # the 3x3 call takes another kernel shape: run one after the other
def test_fused_conv_pair(oracle, dtype, Cin, C3, C1, res, b, n):
    """A 3x3 convolution (fused GN+SiLU gather, residual) and a 1x1 convolution on the same input,
    handed over together: bit for bit what the two separate fused calls write, for a host and a
    device block count, and the 3x3 result against the oracle; an empty first list still runs the
    second call."""
    rng = np.random.default_rng(Cin + C3 + C1 + res)
    td = DT[dtype]
    x = torch.from_numpy(rng.standard_normal((res, res, Cin)).astype(np.float32)).to(td)
    w3, b3 = inputs.conv_params(rng, C3, Cin, 3, td)
    w1, b1 = inputs.conv_params(rng, C1, Cin, 1, td)
    scale = torch.from_numpy(rng.uniform(0.5, 1.5, Cin).astype(np.float32))
    shift = torch.from_numpy(rng.uniform(-0.5, 0.5, Cin).astype(np.float32))
    resid = torch.from_numpy(rng.standard_normal((res, res, C3)).astype(np.float32)).to(td)
    cache3 = torch.from_numpy(rng.standard_normal((res, res, C3)).astype(np.float32)).to(td)
    cache1 = torch.from_numpy(rng.standard_normal((res, res, C1)).astype(np.float32)).to(td)
    conv3 = SigeConv(dev(w3), b3, res, res, b, 1, 1)
    conv1 = SigeConv(dev(w1), b1, res, res, b, 1, 0)
    blocks = random_blocks(rng, conv3.g, n)
    n = len(blocks)
    bl3, bl1 = BlockList(conv3.g, "cuda", max_blocks=n + 3), BlockList(conv1.g, "cuda", max_blocks=n + 3)
    for bl in (bl3, bl1):
        bl.indices[:n].copy_(torch.from_numpy(blocks))
        bl.count.fill_(n)
    bl1.count.fill_(n - 1)                  # the lists need not be equal
    ws = Workspace("cuda")
    xd, sc, sh, rd = dev(x), dev(scale), dev(shift), dev(resid)
    for device_count in (False, True):
        bl3.n_host, bl1.n_host = (-1, -1) if device_count else (n, n - 1)
        ya, yb = dev(cache3).clone(), dev(cache1).clone()
        conv3.forward(xd, ya, bl3, ws, scale=sc, shift=sh, act=api.ACT_SILU, residual=rd, fused=True)
        conv1.forward(xd, yb, bl1, ws, fused=True)
        y3, y1 = dev(cache3).clone(), dev(cache1).clone()
        c3, _ = conv3.fused_call(xd, y3, bl3, ws, scale=sc, shift=sh, act=api.ACT_SILU, residual=rd, tag="p3")
        c1, _ = conv1.fused_call(xd, y1, bl1, ws, tag="p1")
        api.sige_fused_conv_pair(c3, c1)
        torch.cuda.synchronize()
        assert torch.equal(y3, ya) and torch.equal(y1, yb), f"pair differs from the two calls (device_count={device_count})"
    want = oracle.dense_layer(f64(x), f64(w3), f64(b3), 1, 1, f64(scale), f64(shift), oracle.ACT_SILU, storage=dtype)
    want = oracle.select_blocks(want + f64(resid), f64(cache3), blocks, b, b)
    assert_close(y3, want, td, "3x3 call of the pair")
    # an empty first list: the second call still runs
    bl3.count.fill_(0)
    bl3.n_host, bl1.n_host = 0, n - 1
    y3, y1 = dev(cache3).clone(), dev(cache1).clone()
    c3, _ = conv3.fused_call(xd, y3, bl3, ws, scale=sc, shift=sh, act=api.ACT_SILU, residual=rd, tag="p3")
    c1, _ = conv1.fused_call(xd, y1, bl1, ws, tag="p1")
    api.sige_fused_conv_pair(c3, c1)
    torch.cuda.synchronize()
    assert torch.equal(y3, dev(cache3)) and torch.equal(y1, yb)
    c1.Cin = Cin + 1                        # argument errors of either call are reported
    with pytest.raises(api.SigeError):
        api.sige_fused_conv_pair(c3, c1)


@pytest.mark.parametrize("dtype,Cin,C3,C1,res,b,frac", [
    ("f16", 128, 128, 256, 256, 16, 0.01),   # benchmark configuration 2: the launch builds the lists itself
    ("bf16", 64, 40, 72, 100, 8, 0.03),      # 169 blocks of 8x8 on a ragged grid
    ("f32", 64, 64, 32, 62, 6, 0.10),        # fp32, 11 x 11 ragged blocks, lists longer than their capacity
    ("f16", 64, 64, 64, 300, 8, 0.01),       # 1444 blocks: beyond what a workgroup scans, the compaction pass runs
    ("f16", 512, 64, 64, 32, 8, 0.05)])      # the 3x3 call takes another kernel shape: compaction pass, two launches
def test_fused_conv_pair_on_marked_lists(oracle, dtype, Cin, C3, C1, res, b, frac):
    """Marking pass + the pair call that builds the lists from the flags, against the reduction with its
    compaction pass + the plain pair call: lists and counts bit for bit, outputs bit for bit, flags and
    ticket counter zero afterwards - over successive edits through the same workspaces (a growing, a
    shrinking and an empty one), and once more replayed from a HIP graph."""
    rng = np.random.default_rng(Cin + C3 + res)
    td = DT[dtype]
    x = torch.from_numpy(rng.standard_normal((res, res, Cin)).astype(np.float32)).to(td)
    w3, b3 = inputs.conv_params(rng, C3, Cin, 3, td)
    w1, b1 = inputs.conv_params(rng, C1, Cin, 1, td)
    conv3 = SigeConv(dev(w3), b3, res, res, b, 1, 1)
    conv1 = SigeConv(dev(w1), b1, res, res, b, 1, 0)
    cap = 8 if dtype == "f32" else 64
    ws = Workspace("cuda")
    xd = dev(x)
    cache3 = torch.from_numpy(rng.standard_normal((res, res, C3)).astype(np.float32)).to(td).cuda()
    cache1 = torch.from_numpy(rng.standard_normal((res, res, C1)).astype(np.float32)).to(td).cuda()
    ref = [BlockList(conv3.g, "cuda", max_blocks=cap), BlockList(conv1.g, "cuda", max_blocks=cap)]
    got = [BlockList(conv3.g, "cuda", max_blocks=cap), BlockList(conv1.g, "cuda", max_blocks=cap)]
    ya, yb = cache3.clone(), cache1.clone()
    y3, y1 = cache3.clone(), cache1.clone()
    mask_d = torch.zeros((res, res), dtype=torch.uint8, device="cuda")

    def reference():
        BlockList.reduce_together(ref, mask_in=mask_d, dilate=1)
        ca, _ = conv3.fused_call(xd, ya, ref[0], ws, act=api.ACT_SILU, tag="r3")
        cb, _ = conv1.fused_call(xd, yb, ref[1], ws, tag="r1")
        api.sige_fused_conv_pair(ca, cb)

    def marked():
        BlockList.mark_together(got, mask_in=mask_d, dilate=1)
        c3, _ = conv3.fused_call(xd, y3, got[0], ws, act=api.ACT_SILU, tag="p3")
        c1, _ = conv1.fused_call(xd, y1, got[1], ws, tag="p1")
        api.sige_fused_conv_pair_marked(c3, c1, [bl.desc() for bl in got])

    def check(what):
        torch.cuda.synchronize()
        for r, g_ in zip(ref, got):
            n = int(r.count.item())
            assert int(g_.count.item()) == n, what
            assert torch.equal(g_.indices[:min(n, cap)], r.indices[:min(n, cap)]), what
            ws_ = g_.scratch
            half = (ws_.numel() - 16) // 2
            ph = int(ws_[2 * half:2 * half + 4].view(torch.int32).item())
            clean = ws_[(ph & 1) * half:(ph & 1) * half + half]       # the half the next marking pass uses
            assert int(clean.sum().item()) == 0, f"{what}: flags left set for the next pass"
        assert torch.equal(y3, ya) and torch.equal(y1, yb), what
        return int(ref[0].count.item())

    counts = []
    for i, f in enumerate((frac, 2 * frac, 0.5 * frac, 0.0)):
        m = np.zeros((res, res), dtype=np.uint8)
        if f > 0:
            m = inputs.blob_mask(np.random.Generator(np.random.PCG64(900 + i)), res, res, max(1, int(f * res * res)), 2,
                                 (3.0, 8.0), tol=0.5)
        mask_d.copy_(torch.from_numpy(m))
        for y in (ya, y3):
            y.copy_(cache3)
        for y in (yb, y1):
            y.copy_(cache1)
        reference()
        marked()
        counts.append(check(f"edit {i}"))
    assert counts[0] > 0 and counts[3] == 0
    if dtype == "f32":
        assert max(counts) > cap, "a list longer than its capacity is part of this case"
    # replayed from a graph: three replays on changing masks, eager work and synchronisation in between
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        marked()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        marked()
    for i in range(3):
        m = inputs.blob_mask(np.random.Generator(np.random.PCG64(950 + i)), res, res, max(1, int(frac * res * res)), 1,
                             (3.0, 8.0), tol=0.5)
        mask_d.copy_(torch.from_numpy(m))
        for y in (ya, y3):
            y.copy_(cache3)
        for y in (yb, y1):
            y.copy_(cache1)
        reference()
        g.replay()
        check(f"replay {i}")
    # argument errors: the call must read the list its marked list describes; the count is not a host value
    c3, _ = conv3.fused_call(xd, y3, got[0], ws, act=api.ACT_SILU, tag="p3")
    c1, _ = conv1.fused_call(xd, y1, got[1], ws, tag="p1")
    with pytest.raises(api.SigeError):
        api.sige_fused_conv_pair_marked(c3, c1, [got[1].desc(), got[0].desc()])
    got[0].n_host = 3
    c3h, _ = conv3.fused_call(xd, y3, got[0], ws, act=api.ACT_SILU, tag="p3")
    got[0].n_host = -1
    with pytest.raises(api.SigeError):
        api.sige_fused_conv_pair_marked(c3h, c1, [bl.desc() for bl in got])


def test_config2_full_size_step_as_benchmarked(oracle):
    """Benchmark configuration 2 at full size exactly as the benchmark's step runs it: one
    difference pass that fills the lists of both geometries (device-side counts, capacity 16),
    then both convolutions handed over together (one launch).  Lists bit for bit; both outputs
    equal to the cache outside the active blocks and to the separate fused calls everywhere;
    every pixel of every active block of both convolutions against the oracle."""
    cfg = inputs.config2()
    td = torch.float16
    H = W = 256
    C, Cs, b = cfg["Cin"], cfg["Cs"], cfg["block"]
    a_o, a_e = dev(cfg["a_orig"]), dev(cfg["a_edit"])
    main = SigeConv(dev(cfg["w"]), cfg["bias"], H, W, b, 1, 1)
    short = SigeConv(dev(cfg["w_s"]), cfg["bias_s"], H, W, b, 1, 0)
    cap = 16
    bl3, bl1 = BlockList(main.g, "cuda", max_blocks=cap), BlockList(short.g, "cuda", max_blocks=cap)
    mask = torch.zeros((H, W), dtype=torch.uint8, device="cuda")
    mean, var = torch.zeros(32, device="cuda"), torch.zeros(32, device="cuda")
    scale, shift = torch.zeros(C, device="cuda"), torch.zeros(C, device="cuda")
    api.sige_gn_stats(a_o, 32, mean, var, gamma=dev(cfg["gamma"]), beta=dev(cfg["beta"]), eps=cfg["eps"],
                      scale=scale, shift=shift)
    rng = np.random.default_rng(7)
    cache3 = torch.from_numpy(rng.standard_normal((H, W, C)).astype(np.float32)).to(td).cuda()
    cache1 = torch.from_numpy(rng.standard_normal((H, W, Cs)).astype(np.float32)).to(td).cuda()
    ws = Workspace("cuda")
    BlockList.reduce_together([bl3, bl1], a_orig=a_o, a_edit=a_e, tau=cfg["tau"], mask_out=mask, dilate=cfg["dilate"])
    y3, y1 = cache3.clone(), cache1.clone()
    c3, _ = main.fused_call(a_e, y3, bl3, ws, scale=scale, shift=shift, act=api.ACT_SILU, tag="main")
    c1, _ = short.fused_call(a_e, y1, bl1, ws, tag="short")
    assert c3.n_blocks == -1 and c1.n_blocks == -1 and c3.max_blocks == cap
    api.sige_fused_conv_pair(c3, c1)
    torch.cuda.synchronize()
    m = oracle.diff_mask(cfg["a_orig"].float().numpy(), cfg["a_edit"].float().numpy(), 0.0)
    assert np.array_equal(mask.cpu().numpy(), m)
    n3, n1 = int(bl3.count.item()), int(bl1.count.item())
    blocks3, blocks1 = bl3.indices[:n3].cpu().numpy(), bl1.indices[:n1].cpu().numpy()
    assert np.array_equal(blocks3, oracle.active_blocks(m, H, W, b, b, 3, 1, 1)) and n3 <= cap
    assert np.array_equal(blocks1, oracle.active_blocks(m, H, W, b, b, 1, 1, 0)) and 0 < n1 <= n3
    # the separate fused calls write the same bits
    z3, z1 = cache3.clone(), cache1.clone()
    main.forward(a_e, z3, bl3, ws, scale=scale, shift=shift, act=api.ACT_SILU, fused=True)
    short.forward(a_e, z1, bl1, ws, fused=True)
    assert torch.equal(y3, z3) and torch.equal(y1, z1)
    for y, cache, blocks in ((y3, cache3, blocks3), (y1, cache1, blocks1)):
        out = torch.from_numpy(outside_blocks_mask(blocks, b, b, H, W)).cuda()
        assert torch.equal(y[out], cache[out])
    om, ov = oracle.gn_stats(f64(cfg["a_orig"]), 32)
    osc, osh = oracle.fold_gn(f64(cfg["gamma"]), f64(cfg["beta"]), om, ov, cfg["eps"])

    def sample(blocks):
        return oracle.block_pixels(blocks, b, b, H, W)
    # which kernels the shared launch stands for: both calls plan the 64x32 shape whose four waves split K
    p3 = api.sige_conv_plan(td, main.g, C, C, cap, staged_math=True)
    p1 = api.sige_conv_plan(td, short.g, C, Cs, cap)
    assert (p3.kernel, p3.shape, p1.kernel, p1.shape) == (0, 3, 0, 3) and p3.k_steps_per_chunk == p1.k_steps_per_chunk
    px = sample(blocks3)
    got = y3[torch.from_numpy(px[:, 0]).long().cuda(), torch.from_numpy(px[:, 1]).long().cuda()]
    want = oracle.dense_layer(f64(cfg["a_edit"]), f64(cfg["w"]), f64(cfg["bias"]), 1, 1, osc, osh, oracle.ACT_SILU,
                              pixels=px, storage="f16")
    assert_close(got, want, td, "3x3 convolution of the step (all active pixels)")
    px = sample(blocks1)
    got = y1[torch.from_numpy(px[:, 0]).long().cuda(), torch.from_numpy(px[:, 1]).long().cuda()]
    want = oracle.dense_layer(f64(cfg["a_edit"]), f64(cfg["w_s"]), f64(cfg["bias_s"]), 1, 0, pixels=px)
    assert_close(got, want, td, "1x1 shortcut of the step (all active pixels)")


@pytest.mark.gpu
def test_recorded_calls_repeat_the_step():
    """api.record keeps the marshalled arguments of the calls made under it; run() repeats them on the
    tensors' current contents: same lists and outputs as fresh calls, bit for bit, also after the input
    has changed, and an error of a repeated call is raised like a fresh call's."""
    res, C, Co, cap = 64, 32, 32, 16
    td = torch.float16
    rng = np.random.Generator(np.random.PCG64(77))
    conv = SigeConv(torch.from_numpy(rng.standard_normal((Co, C, 3, 3)).astype(np.float32) * 0.1).to(td).cuda(),
                    torch.from_numpy(rng.standard_normal(Co).astype(np.float32)), res, res, 16, 1, 1)
    ws = Workspace("cuda")
    a_o = torch.from_numpy(rng.standard_normal((res, res, C)).astype(np.float32)).to(td).cuda()
    a_e = a_o.clone()
    cache = torch.from_numpy(rng.standard_normal((res, res, Co)).astype(np.float32)).to(td).cuda()
    y_rec, y_new = cache.clone(), cache.clone()
    bl_rec, bl_new = BlockList(conv.g, "cuda", max_blocks=cap), BlockList(conv.g, "cuda", max_blocks=cap)
    mask = torch.zeros((res, res), dtype=torch.uint8, device="cuda")

    def step(bl, y):
        BlockList.reduce_together([bl], a_orig=a_o, a_edit=a_e, tau=0.0, mask_out=mask, dilate=1)
        conv.forward(a_e, y, bl, ws, act=api.ACT_SILU, fused=True)

    a_e[5:9, 40:44] += 1.0
    with api.record() as calls:
        step(bl_rec, y_rec)
    assert len(calls) >= 2
    for edit in range(3):
        a_e.copy_(a_o)
        if edit < 2:
            a_e[20 * edit + 3:20 * edit + 9, 10:30] += 1.0
        y_rec.copy_(cache)
        y_new.copy_(cache)
        calls.run()
        step(bl_new, y_new)
        torch.cuda.synchronize()
        n = int(bl_new.count.item())
        assert int(bl_rec.count.item()) == n and (n > 0) == (edit < 2)
        assert torch.equal(bl_rec.indices[:n], bl_new.indices[:n])
        assert torch.equal(y_rec, y_new)
    fn, args = calls.calls[0]
    calls.calls[0] = (fn, args[:2] + (99,) + args[3:])          # an unknown dtype
    with pytest.raises(api.SigeError):
        calls.run()
