"""GPU parity of the sparse-query attention and of the group-statistics helper."""
import math

import numpy as np
import pytest
import torch

from helpers import round_to, expected_tiles, assert_close, dev, f64
from paper_2211_02048_amd import api, inputs

pytestmark = pytest.mark.gpu
DT = inputs.DTYPES


def attn_close(got, want64, dtype, what):
    """Element-wise at the stated tolerance: 1e-2 (fp16, bf16) or 1e-4 (fp32) of max(|ref|, rms(ref))."""
    assert_close(got, want64, dtype, what)


def run_attn(c, use_ws=True, n_q=None):
    q, k, v = dev(c["q"]), dev(c["k"]), dev(c["v"])
    n_q = q.shape[0] if n_q is None else n_q
    o = torch.full_like(q, 7.0)
    ws = None
    if use_ws:
        nb = api.sige_sparse_attn_workspace_bytes(n_q, c["T"], c["heads"], c["d"])
        if nb:
            ws = torch.empty(nb // 4, dtype=torch.float32, device="cuda")
    api.sige_sparse_attn(q, k, v, o, c["scale"], Nq=n_q, workspace=ws)
    torch.cuda.synchronize()
    return o, ws is not None


@pytest.mark.parametrize("T,heads,d,n_q,dtype", [
    (4096, 8, 40, 96, "bf16"),      # SD 64x64 level, ~1 % edit: key range split over workgroups
    (4096, 8, 40, 400, "bf16"),     # ~5-10 % edit
    (1024, 8, 80, 50, "bf16"),      # ragged query count
    (256, 8, 160, 256, "bf16"),     # every token active
    (77, 8, 40, 130, "bf16"),       # cross-attention over 77 text tokens (ragged key tail)
    (77, 8, 160, 33, "f16"),
    (100, 2, 64, 1, "f16"),         # a single query
    (31, 1, 8, 5, "f16"),           # fewer keys than one chunk, smallest head
    (512, 3, 256, 70, "bf16"),      # largest head dimension
    (2048, 4, 96, 200, "f16"),
    # single precision (the precision of the paper's experiments): its own kernel, 1e-4
    (4096, 8, 40, 96, "f32"), (1024, 8, 80, 50, "f32"), (256, 8, 160, 256, "f32"), (77, 8, 40, 130, "f32"),
    (31, 1, 4, 5, "f32"), (512, 3, 256, 70, "f32"), (300, 2, 100, 129, "f32"), (100, 2, 64, 1, "f32"),
])
def test_sparse_attention_matches_oracle(oracle, T, heads, d, n_q, dtype):
    c = inputs.attention_case(100 + T + d, T, heads, d, n_q, dtype)
    want = oracle.attention(f64(c["q"]), f64(c["k"]), f64(c["v"]), c["scale"])
    splits = []
    for use_ws in (True, False):
        o, split = run_attn(c, use_ws)
        splits.append(split)
        attn_close(o, want, DT[dtype], f"attention T={T} d={d} nq={n_q} split={split}")
    if T >= 2048 and n_q <= 128:
        assert splits == [True, False]  # the small-query cases do exercise the split + merge path


@pytest.mark.parametrize("dtype,res,b,heads,d,n", [("bf16", 32, 8, 8, 40, 3), ("f16", 16, 4, 4, 64, 16),
                                                   ("bf16", 20, 8, 2, 24, 4), ("f16", 64, 8, 8, 40, 1),
                                                   ("f32", 20, 8, 2, 24, 4), ("f32", 32, 8, 8, 40, 3)])
def test_sparse_attention_queries_by_block_list(oracle, dtype, res, b, heads, d, n):
    """Queries, keys and values are three channel ranges of one full tensor; the queries of the
    call are the pixels of the listed blocks, taken from it by the attention kernel.  Against the
    oracle's attention on the rows gathered by hand, and bit for bit against the call that is
    handed those rows; a block that sticks out of the map (20 = 2.5 blocks of 8) reads the clamped
    pixels; n_blocks == 0 enqueues nothing."""
    td = DT[dtype]
    C, T = heads * d, res * res
    rng = np.random.default_rng(res + d + n)
    qkv = torch.from_numpy(rng.standard_normal((res, res, 3 * C)).astype(np.float32)).to(td)
    g = api.geom(res, res, b, 1, 1, 0)
    gb_y, gb_x = -(-res // b), -(-res // b)
    pick = np.sort(rng.permutation(gb_y * gb_x)[:n])
    pick[-1] = gb_y * gb_x - 1                 # the bottom-right block: partly outside when b does not divide res
    blocks = np.stack([(pick // gb_x) * b, (pick % gb_x) * b], 1).astype(np.int32)
    ys = np.minimum(blocks[:, 0, None, None] + np.arange(b)[None, :, None], res - 1)
    xs = np.minimum(blocks[:, 1, None, None] + np.arange(b)[None, None, :], res - 1)
    tok = (ys * res + xs).reshape(-1)          # token of every query row, block by block, row-major inside
    flat = qkv.view(T, 3 * C)
    q_rows = flat[torch.from_numpy(tok)][:, :C].contiguous()
    scale = 1.0 / math.sqrt(d)
    want = oracle.attention(f64(q_rows).reshape(-1, heads, d), f64(flat[:, C:2 * C]).reshape(T, heads, d),
                            f64(flat[:, 2 * C:]).reshape(T, heads, d), scale).reshape(-1, C)
    qkv_d = dev(qkv).view(T, 3 * C)
    idx = torch.from_numpy(blocks).cuda()
    rows = n * b * b
    nb = api.sige_sparse_attn_workspace_bytes(rows, T, heads, d)
    for use_ws in (True, False):
        ws = torch.empty(nb // 4, dtype=torch.float32, device="cuda") if (use_ws and nb) else None
        o = torch.full((rows + 1, C), 7.0, dtype=td, device="cuda")
        api.sige_sparse_attn_blocks(qkv_d, g, idx, n, qkv_d[:, C:2 * C], qkv_d[:, 2 * C:], o, scale, heads=heads,
                                    d=d, workspace=ws, q_ld=3 * C, kv_ld=3 * C, o_ld=C)
        o2 = torch.full((rows + 1, C), 7.0, dtype=td, device="cuda")
        api.sige_sparse_attn(dev(q_rows), qkv_d[:, C:2 * C], qkv_d[:, 2 * C:], o2, scale, Nq=rows, workspace=ws,
                             heads=heads, d=d, q_ld=C, kv_ld=3 * C, o_ld=C)
        torch.cuda.synchronize()
        attn_close(o[:rows], want, td, f"attention by block list, workspace={use_ws}")
        assert torch.equal(o, o2), "queries by block list differ from the same queries handed over as rows"
        assert (o[rows] == 7.0).all()
    o = torch.full((rows, C), 7.0, dtype=td, device="cuda")
    api.sige_sparse_attn_blocks(qkv_d, g, idx, 0, qkv_d[:, C:2 * C], qkv_d[:, 2 * C:], o, scale, heads=heads, d=d,
                                q_ld=3 * C, kv_ld=3 * C, o_ld=C)
    torch.cuda.synchronize()
    assert (o == 7.0).all()
    with pytest.raises(api.SigeError):        # the geometry of a 3x3 layer has tiles larger than its blocks
        api.sige_sparse_attn_blocks(qkv_d, api.geom(res, res, b, 3, 1, 1), idx, n, qkv_d[:, C:2 * C],
                                    qkv_d[:, 2 * C:], o, scale, heads=heads, d=d, q_ld=3 * C, kv_ld=3 * C, o_ld=C)


def test_sparse_attention_edge_cases(oracle):
    c = inputs.attention_case(5, 300, 4, 40, 64, "bf16")
    # Nq smaller than the buffer: rows beyond Nq are untouched
    o, _ = run_attn(c, n_q=37)
    want = oracle.attention(f64(c["q"][:37]), f64(c["k"]), f64(c["v"]), c["scale"])
    attn_close(o[:37], want, torch.bfloat16, "attention Nq prefix")
    assert (o[37:] == 7.0).all()
    # Nq = 0: nothing enqueued
    o0 = torch.full_like(dev(c["q"]), 7.0)
    api.sige_sparse_attn(dev(c["q"]), dev(c["k"]), dev(c["v"]), o0, c["scale"], Nq=0)
    assert (o0 == 7.0).all()
    # large logits: the running max keeps exp() finite; result equals the dominant value row
    big = dict(c)
    big["q"] = c["q"] * 30
    big["k"] = c["k"] * 30
    o, _ = run_attn(big)
    want = oracle.attention(f64(big["q"]), f64(big["k"]), f64(big["v"]), c["scale"])
    assert torch.isfinite(o).all()
    attn_close(o, want, torch.bfloat16, "attention large logits")
    # strided q / k / v / o: heads*d columns inside wider rows (e.g. a fused QKV buffer)
    T, heads, d, nq = 200, 2, 40, 48
    rng = np.random.default_rng(8)
    kv = torch.from_numpy(rng.standard_normal((T, 3 * heads * d)).astype(np.float32)).to(torch.float16).cuda()
    qb = torch.from_numpy(rng.standard_normal((nq, 2 * heads * d)).astype(np.float32)).to(torch.float16).cuda()
    k = kv[:, heads * d:2 * heads * d]
    v = kv[:, 2 * heads * d:]
    q = qb[:, :heads * d]
    ob = torch.zeros((nq, 2 * heads * d), dtype=torch.float16, device="cuda")
    o = ob[:, heads * d:]
    api.sige_sparse_attn(q, k, v, o, 0.2, Nq=nq, heads=heads, d=d, q_ld=2 * heads * d, kv_ld=3 * heads * d,
                         o_ld=2 * heads * d)
    want = oracle.attention(f64(q).reshape(nq, heads, d), f64(k).reshape(T, heads, d),
                            f64(v).reshape(T, heads, d), 0.2)
    attn_close(o.reshape(nq, heads, d), want, torch.float16, "attention strided")
    assert (ob[:, :heads * d] == 0).all()


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_sparse_attention_peaked_rows(oracle, dtype):
    """Rows whose softmax is dominated by one or two keys (large logits): the probabilities that enter
    the second product are rounded to the storage type, and the row is normalised by the sum of those
    same rounded values, so a dominated row returns (a mix of) the value rows at the stated tolerance."""
    T, heads, d, nq = 640, 4, 40, 200
    c = inputs.attention_case(77, T, heads, d, nq, dtype)
    rng = np.random.default_rng(3)
    q = c["q"].float().numpy() * rng.uniform(1.0, 6.0, (nq, heads, 1)).astype(np.float32)   # temperature per row
    c["q"] = torch.from_numpy(q).to(DT[dtype])
    want = oracle.attention(f64(c["q"]), f64(c["k"]), f64(c["v"]), c["scale"])
    for use_ws in (True, False):
        o, _ = run_attn(c, use_ws)
        attn_close(o, want, DT[dtype], f"peaked rows {dtype} workspace={use_ws}")


def test_sparse_attention_token_selection_counts(oracle):
    """Fig. "sige-attention": the queries are the tokens of the active 4x4 blocks; the map is
    Nq x T instead of T x T."""
    Ht = Wt = 64
    m = inputs.token_mask(3, Ht, Wt, 0.01)
    g = api.geom(Ht, Wt, 4, 1, 1, 0)
    idx = torch.zeros((g.grid_blocks, 2), dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.sige_reduce_mask(g, idx, cnt, mask_in=torch.from_numpy(m).cuda())
    n = int(cnt.item())
    want = oracle.active_blocks(m, Ht, Wt, 4, 4, 1, 1, 0)
    assert np.array_equal(idx[:n].cpu().numpy(), want)
    tok = oracle.block_pixels(want, 4, 4, Ht, Wt)
    assert len(tok) == 16 * n and 16 * n < 0.06 * Ht * Wt


@pytest.mark.parametrize("dtype,H,W,C,G,ld", [("f16", 64, 64, 128, 32, 128), ("bf16", 37, 21, 320, 32, 320),
                                              ("f32", 16, 16, 64, 32, 64), ("f16", 32, 32, 64, 8, 192),
                                              ("f16", 24, 24, 24, 3, 24), ("f16", 40, 40, 384, 32, 384),
                                              ("f16", 8, 8, 2560, 32, 2560), ("f32", 9, 9, 1024, 16, 1024),
                                              # one group per channel (instance norm), small: the one-kernel path
                                              ("f16", 16, 32, 1024, 1024, 1024), ("bf16", 5, 7, 64, 64, 64),
                                              # too many pixels for it: the streaming pass with atomics
                                              ("f16", 128, 96, 128, 32, 128), ("f16", 100, 100, 320, 32, 320)])
def test_gn_stats_and_fold(oracle, dtype, H, W, C, G, ld):
    rng = np.random.default_rng(C)
    td = DT[dtype]
    buf = torch.from_numpy((rng.standard_normal((H, W, ld)) * 1.7 + 0.4).astype(np.float32)).to(td).cuda()
    x = buf[:, :, ld - C:]
    gamma = torch.from_numpy(rng.uniform(0.5, 1.5, C).astype(np.float32))
    beta = torch.from_numpy(rng.uniform(-0.5, 0.5, C).astype(np.float32))
    mean = torch.empty(G, device="cuda")
    var = torch.empty(G, device="cuda")
    scale = torch.empty(C, device="cuda")
    shift = torch.empty(C, device="cuda")
    api.sige_gn_stats(x, G, mean, var, gamma=dev(gamma), beta=dev(beta), eps=1e-5, scale=scale, shift=shift,
                      C=C, x_ld=ld)
    wm, wv = oracle.gn_stats(f64(x), G)
    ws, wsh = oracle.fold_gn(f64(gamma), f64(beta), wm, wv, 1e-5)
    np.testing.assert_allclose(f64(mean), wm, rtol=0, atol=2e-5)
    np.testing.assert_allclose(f64(var), wv, rtol=2e-5)
    np.testing.assert_allclose(f64(scale), ws, rtol=2e-5)
    np.testing.assert_allclose(f64(shift), wsh, rtol=0, atol=5e-5)


def test_sige_attention_layer_sparse_queries(oracle):
    """Fig. "sige-attention" end to end through the library: gather the active 4x4 token blocks, run
    the Q, K, V 1x1 convolutions on them, scatter ONLY K and V into the cached K/V, attend with the
    gathered queries against all cached keys/values, run the Out convolution on the attended tiles
    and scatter it into the cached output.  Compared with the oracle's dense statement of the layer."""
    from paper_2211_02048_amd.layers import BlockList, SigeConv, Workspace
    rng = np.random.default_rng(77)
    td, dtype = torch.bfloat16, "bf16"
    H = W = 32
    C, heads = 128, 4
    d = C // heads
    scale = 1.0 / math.sqrt(d)
    mask = inputs.token_mask(9, H, W, 0.04)
    x_o, x_e = inputs.edited_pair(rng, H, W, C, mask, 1.0, td)
    ws_, bs_ = zip(*[inputs.conv_params(rng, C, C, 1, td) for _ in range(4)])
    w64 = [f64(w) for w in ws_]
    b64 = [f64(b) for b in bs_]
    # caches from the original input, computed by the oracle and rounded to the storage type
    xo64 = f64(x_o)
    k_cache = torch.from_numpy(oracle.conv2d(xo64, w64[1], b64[1])).to(td)
    v_cache = torch.from_numpy(oracle.conv2d(xo64, w64[2], b64[2])).to(td)
    all_blocks = np.array([(y, x) for y in range(0, H, 4) for x in range(0, W, 4)], np.int32)
    out_cache64 = oracle.sige_attention_layer(xo64, np.zeros((H, W, C)), all_blocks, 4, 4, *w64, *b64, heads, scale)
    out_cache = torch.from_numpy(out_cache64).to(td)

    convs = [SigeConv(dev(w), b, H, W, 4, 1, 0) for w, b in zip(ws_, bs_)]
    wsp = Workspace("cuda")
    bl = BlockList(convs[0].g, "cuda")
    bl.reduce(mask_in=torch.from_numpy(mask).cuda())
    n = bl.sync_count()
    blocks = bl.indices[:n].cpu().numpy()
    assert np.array_equal(blocks, oracle.active_blocks(mask, H, W, 4, 4, 1, 1, 0)) and 0 < n < 24
    xe = dev(x_e)
    kc, vc, oc = dev(k_cache).clone(), dev(v_cache).clone(), dev(out_cache).clone()
    q_tiles = convs[0].forward(xe, None, bl, wsp, scatter=False, tag="q").clone()
    convs[1].forward(xe, kc, bl, wsp, tag="k")          # K and V of the edited tokens overwrite the caches
    convs[2].forward(xe, vc, bl, wsp, tag="v")
    nq = n * 16
    att = torch.zeros((nq, heads, d), dtype=td, device="cuda")
    nb = api.sige_sparse_attn_workspace_bytes(nq, H * W, heads, d)
    wsb = torch.empty(max(nb // 4, 1), dtype=torch.float32, device="cuda") if nb else None
    api.sige_sparse_attn(q_tiles.view(nq, heads, d), kc.view(H * W, heads, d), vc.view(H * W, heads, d), att, scale,
                         workspace=wsb)
    # the Out convolution reads the attended tokens as tiles [n, 4, 4, C] and scatters into the cache
    out_tiles = wsp.get("out_o", convs[3].out_numel(n), td)
    api.sige_conv(att.view(n, 4, 4, C), convs[3].g, C, C, convs[3].packed, convs[3].bias, bl.count, out_tiles,
                  n_blocks=n, max_blocks=n)
    api.sige_scatter(out_tiles, convs[3].g, bl.indices, bl.count, oc, n_blocks=n, Cout=C, max_blocks=n)
    torch.cuda.synchronize()

    want = oracle.sige_attention_layer(f64(x_e), f64(out_cache), blocks, 4, 4, *w64, *b64, heads, scale,
                                       f64(k_cache), f64(v_cache))
    act = np.zeros((H, W), bool)
    for y0, x0 in blocks:
        act[y0:y0 + 4, x0:x0 + 4] = True
    a_t = torch.from_numpy(act).cuda()
    assert torch.equal(oc[~a_t], dev(out_cache)[~a_t])      # unedited tokens keep the cached output
    # call by call at the stated tolerance, each against the oracle's result from the oracle's own
    # (rounded) inputs: queries, attended values, output projection
    xe64 = f64(x_e)
    q64 = round_to(oracle.conv2d(xe64, w64[0], b64[0]), td)
    tok = oracle.block_pixels(blocks, 4, 4, H, W)
    q_rows = np.stack([q64[y, x] for y, x in tok])
    assert_close(q_tiles.view(nq, C), q_rows, td, "queries of the active tokens")
    k_full, v_full = f64(kc), f64(vc)               # the caches as the library left them (checked below)
    a_want = oracle.attention(f64(q_tiles).reshape(nq, heads, d), k_full.reshape(H * W, heads, d),
                              v_full.reshape(H * W, heads, d), scale)
    assert_close(att, a_want, td, "attention of the active tokens")
    o_rows = oracle.conv2d(f64(att).reshape(nq, 1, C), w64[3], b64[3])[:, 0]
    o_want = np.zeros((H, W, C))
    for i, (y, x) in enumerate(tok):                # token order of the call -> the tokens' places in the map
        o_want[y, x] = o_rows[i]
    assert_close(oc[a_t], o_want[act], td, "output projection scattered into the cache")
    # and the whole layer against the oracle's dense statement of it (no intermediate forced): the
    # layer's three stored intermediates each add a rounding, so this second check is a drift bound
    drift = np.abs(f64(oc[a_t]) - round_to(want[act], td)).max() / np.sqrt(np.mean(want[act] ** 2))
    assert drift < 4e-2, f"whole layer drifted {drift:.3e} of the rms from the oracle's layer"
    # K/V caches: edited tokens overwritten, the rest bit-identical
    assert torch.equal(kc[~a_t], dev(k_cache)[~a_t]) and torch.equal(vc[~a_t], dev(v_cache)[~a_t])
    assert_close(kc[a_t], oracle.conv2d(f64(x_e), w64[1], b64[1])[act], td, "K overwrite")


@pytest.mark.parametrize("dtype,C,rows", [("bf16", 320, 37), ("f16", 1280, 70), ("f32", 64, 9), ("bf16", 2560, 5),
                                          ("f16", 8, 130)])
def test_token_norm_and_geglu(oracle, dtype, C, rows):
    """Token-wise layers on stacked tiles: layer norm over channels and the gated GELU, against the
    oracle; host row count and device count (count * tokens per block), rows beyond untouched, wider
    row strides, in-place normalisation."""
    rng = np.random.default_rng(C + rows)
    td = DT[dtype]
    ld = C + (16 if dtype == "f32" else 32)
    buf = torch.from_numpy((rng.standard_normal((rows + 4, ld)) * 2.0 + 0.5).astype(np.float32)).to(td).cuda()
    x = buf[:, :C]
    gamma = torch.from_numpy(rng.uniform(0.5, 1.5, C).astype(np.float32))
    beta = torch.from_numpy(rng.uniform(-0.5, 0.5, C).astype(np.float32))
    want = oracle.layer_norm(f64(x[:rows]), f64(gamma), f64(beta), 1e-5)
    y = torch.full((rows + 4, C), 7.0, dtype=td, device="cuda")
    api.sige_token_norm(x, y, C, n_rows=rows, gamma=dev(gamma), beta=dev(beta), eps=1e-5, x_ld=ld)
    assert_close(y[:rows], want, td, "token norm")
    assert (y[rows:] == 7.0).all()
    # device-side count: rows = count * rows_per_count, capped by max_rows
    if rows % 5 == 0:
        cnt = torch.tensor([rows // 5], dtype=torch.int32, device="cuda")
        y2 = torch.full((rows + 4, C), 7.0, dtype=td, device="cuda")
        api.sige_token_norm(x, y2, C, n_rows=-1, count=cnt, rows_per_count=5, max_rows=rows + 4, gamma=dev(gamma),
                            beta=dev(beta), eps=1e-5, x_ld=ld)
        assert torch.equal(y2, y)
        cnt.fill_(1000)
        api.sige_token_norm(x, y2, C, n_rows=-1, count=cnt, rows_per_count=5, max_rows=rows, gamma=dev(gamma),
                            beta=dev(beta), eps=1e-5, x_ld=ld)
        assert torch.equal(y2, y)          # capped at max_rows
    # in place, no affine part
    z = x[:rows].contiguous()
    api.sige_token_norm(z, z, C, n_rows=rows, eps=1e-5)
    assert_close(z, oracle.layer_norm(f64(x[:rows]), eps=1e-5), td, "token norm in place")
    # gated GELU: input rows of 2*Ch channels
    if C % 2 == 0 and (C // 2) * (4 if dtype == "f32" else 2) % 16 == 0:
        Ch = C // 2
        o = torch.full((rows + 4, Ch), 7.0, dtype=td, device="cuda")
        api.sige_geglu(x, o, Ch, n_rows=rows, x_ld=ld)
        assert_close(o[:rows], oracle.geglu(f64(x[:rows])), td, "geglu")
        assert (o[rows:] == 7.0).all()
    with pytest.raises(api.SigeError):
        api.sige_token_norm(x, y, C, n_rows=rows + 100, x_ld=ld)          # more rows than max_rows
    with pytest.raises(api.SigeError):
        api.sige_token_norm(x, y, C, n_rows=-1, x_ld=ld)                  # no count


@pytest.mark.parametrize("dtype,C,res,b,n", [("bf16", 320, 22, 4, 9), ("f16", 1280, 16, 8, 3), ("f32", 64, 13, 5, 6)])
def test_gather_token_norm(oracle, dtype, C, res, b, n):
    """The gather with the token norm folded in: against the oracle's layer norm of the gathered
    pixels (a pixel outside the tensor is a row of zeros), bit for bit against gather + token norm,
    both count paths, a wider pixel stride, tiles beyond the count untouched, geometry errors."""
    rng = np.random.default_rng(C + res)
    td = DT[dtype]
    ld = C + (16 if dtype == "f32" else 32)
    buf = torch.from_numpy((rng.standard_normal((res, res, ld)) * 2.0 + 0.5).astype(np.float32)).to(td).cuda()
    x = buf[:, :, :C]
    g = api.geom(res, res, b, 1, 1, 0)
    nby = -(-res // b)
    pick = np.sort(rng.permutation(nby * nby)[:n])
    pick[-1] = nby * nby - 1                      # the bottom-right block sticks out when b does not divide res
    blocks = np.array([((i // nby) * b, (i % nby) * b) for i in np.unique(pick)], np.int32)
    n = len(blocks)
    idx = torch.from_numpy(blocks).cuda()
    cnt = torch.tensor([n], dtype=torch.int32, device="cuda")
    gamma = torch.from_numpy(rng.uniform(0.5, 1.5, C).astype(np.float32))
    beta = torch.from_numpy(rng.uniform(-0.5, 0.5, C).astype(np.float32))
    tiles = torch.full((n + 2, b, b, C), 7.0, dtype=td, device="cuda")
    api.sige_gather_token_norm(x, g, idx, cnt, tiles, C, n_blocks=n, gamma=dev(gamma), beta=dev(beta), eps=1e-5)
    gathered = expected_tiles(oracle, f64(x), blocks, b, b, 1, 0, None, None, 0)
    want = oracle.layer_norm(gathered.reshape(-1, C), f64(gamma), f64(beta), 1e-5).reshape(n, b, b, C)
    assert_close(tiles[:n], want, td, "gather + token norm")
    assert (tiles[n:] == 7.0).all()
    t0 = torch.full((n + 2, b, b, C), 7.0, dtype=td, device="cuda")
    api.sige_gather(x, g, idx, cnt, t0, n_blocks=n, C=C)
    api.sige_token_norm(t0, t0, C, n_rows=n * b * b, gamma=dev(gamma), beta=dev(beta), eps=1e-5)
    assert torch.equal(t0, tiles), "the folded call differs from gather followed by token norm"
    t1 = torch.full((n + 2, b, b, C), 7.0, dtype=td, device="cuda")
    api.sige_gather_token_norm(x, g, idx, cnt, t1, C, n_blocks=-1, gamma=dev(gamma), beta=dev(beta), eps=1e-5)
    assert torch.equal(t1, tiles)
    with pytest.raises(api.SigeError):
        api.sige_gather_token_norm(x, api.geom(res, res, b, 3, 1, 1), idx, cnt, tiles, C, n_blocks=n)


@pytest.mark.parametrize("dtype,Cin,Cg,b,n", [("bf16", 320, 1280, 8, 10), ("f16", 64, 24, 4, 5), ("f32", 32, 16, 3, 7),
                                               ("bf16", 1280, 512, 8, 2), ("f16", 128, 2560, 8, 1)])
def test_conv_geglu(oracle, dtype, Cin, Cg, b, n):
    """The feed-forward layer with the gated GELU folded into its epilogue (one layer, one stored
    tensor): against the oracle's convolution (fp64, unrounded) followed by its gated GELU; tiled and
    few-row kernels (chosen by size); both count paths; tiles beyond the count untouched.  The two
    calls it replaces are each held to the same bar on their own inputs."""
    rng = np.random.default_rng(Cin + Cg + b)
    td = DT[dtype]
    g = api.geom(8 * b, 8 * b, b, 1, 1, 0)
    tiles = torch.from_numpy(rng.standard_normal((n, b, b, Cin)).astype(np.float32)).to(td)
    w, bias = inputs.conv_params(rng, 2 * Cg, Cin, 1, td)
    u = np.stack([oracle.conv2d(f64(tiles[i]), f64(w), f64(bias), 1, 0) for i in range(n)])     # [n, b, b, 2Cg]
    want = oracle.geglu(u.reshape(-1, 2 * Cg)).reshape(n, b, b, Cg)
    rows = api.geglu_rows(Cg)
    packed = api.sige_pack_weight(dev(w[rows].contiguous()))
    cnt = torch.tensor([n], dtype=torch.int32, device="cuda")
    for nb, mb in ((n, n), (-1, n + 1)):
        out = torch.full((n + 1, b, b, Cg), 5.0, dtype=td, device="cuda")
        big = torch.cat([dev(tiles), torch.zeros((1, b, b, Cin), dtype=td, device="cuda")])
        api.sige_conv_geglu(big, g, Cin, Cg, packed, dev(bias[rows].contiguous()), cnt, out, n_blocks=nb, max_blocks=mb)
        assert_close(out[:n], want, td, f"conv + gated GELU n_blocks={nb}")
        assert (out[n:] == 5.0).all()
    # the two calls it replaces: convolution (stored, rounded), then sige_geglu
    o2 = torch.empty((n, b, b, 2 * Cg), dtype=td, device="cuda")
    api.sige_conv(dev(tiles), g, Cin, 2 * Cg, api.sige_pack_weight(dev(w)), dev(bias), cnt, o2, n_blocks=n, max_blocks=n)
    y2 = torch.empty((n, b, b, Cg), dtype=td, device="cuda")
    api.sige_geglu(o2, y2, Cg, n_rows=n * b * b)
    # each call against the oracle on that call's own input (the intermediate is a stored tensor)
    assert_close(o2, u, td, "the convolution alone")
    assert_close(y2, oracle.geglu(f64(o2).reshape(-1, 2 * Cg)).reshape(n, b, b, Cg), td, "sige_geglu of the stored intermediate")
    with pytest.raises(api.SigeError):
        api.sige_conv_geglu(dev(tiles), g, Cin, Cg + 4, packed, None, cnt, out, n_blocks=n, max_blocks=n)
