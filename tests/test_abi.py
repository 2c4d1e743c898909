"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the public header declares, and refuses bad arguments synchronously with the
documented codes (nothing is enqueued on those paths)."""
import ctypes
import os
import re

import pytest

from paper_2211_02048_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x10000)  # never dereferenced: every call below fails validation first


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(api.LIB_PATH):
        from paper_2211_02048_amd import build
        build.build()
    return api.lib()


def test_exports_match_header(L):
    hdr = open(os.path.join(ROOT, "include", "sige.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = sorted(set(re.findall(r"\b(sige_[a-z0-9_]+)\s*\(", hdr)))
    assert declared == sorted(api.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert L.sige_version() >= 1


def good_geom():
    return api.geom(64, 64, 6, 3, 1, 1)


def err(L):
    return L.sige_last_error().decode()


def test_geometry_errors(L):
    g = good_geom()
    g.block_h = 0
    assert L.sige_gather(FAKE, 0, 64, 64, 0, ctypes.byref(g), FAKE, FAKE, 8, -1, None, None, 0, FAKE, None) == 1
    assert "block" in err(L)
    g = good_geom()
    g.k = 2
    assert L.sige_conv(FAKE, 0, ctypes.byref(g), 64, 64, FAKE, None, FAKE, 8, -1, FAKE, None, 0, None) == 1
    assert "odd" in err(L)
    g = good_geom()
    g.H_out = 63
    assert L.sige_scatter(FAKE, 0, ctypes.byref(g), 64, FAKE, FAKE, 8, -1, None, None, 0, FAKE, 64, None) == 1
    assert L.sige_gather(FAKE, 0, 64, 64, 0, None, FAKE, FAKE, 8, -1, None, None, 0, FAKE, None) == 1


def test_pointer_and_capacity_errors(L):
    g = good_geom()
    gp = ctypes.byref(g)
    # required pointer missing
    assert L.sige_gather(None, 0, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, FAKE, None) == 1
    # host n_blocks beyond the capacity
    assert L.sige_gather(FAKE, 0, 64, 64, 0, gp, FAKE, FAKE, 8, 9, None, None, 0, FAKE, None) == 3
    assert "exceeds" in err(L)
    assert L.sige_conv(FAKE, 0, gp, 64, 64, FAKE, None, FAKE, 8, 9, FAKE, None, 0, None) == 3
    assert L.sige_scatter(FAKE, 0, gp, 64, FAKE, FAKE, 8, 9, None, None, 0, FAKE, 64, None) == 3
    # neither a host count nor a device count
    assert L.sige_conv(FAKE, 0, gp, 64, 64, FAKE, None, None, 8, -1, FAKE, None, 0, None) == 1
    # channel counts the vector kernels do not cover are refused, never silently handled
    assert L.sige_gather(FAKE, 0, 3, 3, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, FAKE, None) == 2
    assert L.sige_conv(FAKE, 1, gp, 24, 64, FAKE, None, FAKE, 8, -1, FAKE, None, 0, None) == 2
    assert L.sige_conv(FAKE, 0, gp, 4, 64, FAKE, None, FAKE, 8, -1, FAKE, None, 0, None) == 2
    # fused call: exactly one destination
    assert L.sige_fused_conv(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, 64, FAKE, None, None, None, 0,
                             FAKE, 64, FAKE, None, 0, None, 0, None) == 1
    assert L.sige_fused_conv(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, 64, FAKE, None, None, None, 0,
                             None, 0, None, None, 0, None, 0, None) == 1
    assert L.sige_fused_conv(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, 64, FAKE, None, FAKE, None, 0,
                             None, 0, FAKE, None, 0, None, 0, None) == 1       # residuals need y
    assert L.sige_fused_conv(FAKE, 1, 24, 24, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, 64, FAKE, None, None, None, 0,
                             FAKE, 64, None, None, 0, None, 0, None) == 2
    assert L.sige_fused_conv(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, 9, None, None, 0, 64, FAKE, None, None, None, 0,
                             FAKE, 64, None, None, 0, None, 0, None) == 3
    # activated copies: at most SIGE_MAX_ACT_OUTS, scatter mode only, a list when the count is positive
    assert L.sige_fused_conv(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, 64, FAKE, None, None, None, 0,
                             FAKE, 64, None, None, 4, None, 0, None) == 1
    assert L.sige_fused_conv(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, 64, FAKE, None, None, None, 0,
                             FAKE, 64, None, None, 1, None, 0, None) == 1
    ao = (api.ActOut * 1)()
    ao[0].y, ao[0].y_ld, ao[0].act = FAKE, 64, 0
    assert L.sige_fused_conv(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, 64, FAKE, None, None, None, 0,
                             None, 0, FAKE, ao, 1, None, 0, None) == 1      # copies need y
    ao[0].y_ld = 60                                                            # narrower than Cout
    assert L.sige_fused_conv(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, 64, FAKE, None, None, None, 0,
                             FAKE, 64, None, ao, 1, None, 0, None) == 1
    # convolution with the gated GELU folded in: output channels in groups of 8
    assert L.sige_conv_geglu(FAKE, 1, gp, 64, 12, FAKE, None, FAKE, 8, -1, FAKE, None) == 2
    assert L.sige_conv_geglu(FAKE, 1, gp, 64, 16, FAKE, None, FAKE, 8, -1, None, None) == 1
    # convolution with the scatter folded in, gather with the token norm folded in
    assert L.sige_conv_scatter(FAKE, 1, gp, 64, 64, FAKE, None, None, FAKE, 8, -1, None, None, 0, FAKE, 64, None, 0, None) == 1
    assert L.sige_conv_scatter(FAKE, 1, gp, 64, 64, FAKE, None, FAKE, FAKE, 8, -1, None, None, 0, FAKE, 32, None, 0, None) == 1
    assert L.sige_gather_token_norm(FAKE, 1, 64, 64, gp, FAKE, FAKE, 8, -1, None, None, 1e-5, FAKE, None) == 2   # k = 3 geometry
    assert L.sige_gather_token_norm(FAKE, 1, 64, 64, gp, None, FAKE, 8, -1, None, None, 1e-5, FAKE, None) == 1
    # scale without shift
    assert L.sige_gather(FAKE, 0, 64, 64, 0, gp, FAKE, FAKE, 8, -1, FAKE, None, 0, FAKE, None) == 1
    # unknown dtype
    assert L.sige_gather(FAKE, 7, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, 0, FAKE, None) == 1
    # zero blocks on the host: accepted, nothing to do
    assert L.sige_gather(FAKE, 0, 64, 64, 0, gp, FAKE, FAKE, 8, 0, None, None, 0, FAKE, None) == 0
    assert err(L) == ""


def test_reduce_mask_errors(L):
    g = good_geom()
    gp = ctypes.byref(g)
    f = ctypes.c_float(1e-6)
    # both sources / neither source
    assert L.sige_reduce_mask(FAKE, FAKE, 0, 64, 64, 64, f, FAKE, 0, 0, gp, FAKE, FAKE, 121, FAKE, None, 0, None) == 1
    assert L.sige_reduce_mask(None, None, 0, 64, 64, 64, f, None, 0, 0, gp, FAKE, FAKE, 121, FAKE, None, 0, None) == 1
    assert "either" in err(L)
    # activation mode needs mask_out
    assert L.sige_reduce_mask(FAKE, FAKE, 0, 64, 64, 64, f, None, 0, 0, gp, None, FAKE, 121, FAKE, None, 0, None) == 1
    # pooled mask size must match the conv input
    assert L.sige_reduce_mask(None, None, 0, 100, 64, 0, f, FAKE, 0, 0, gp, None, FAKE, 121, FAKE, None, 0, None) == 1
    # block grid beyond the stated maximum
    big = api.geom(2048, 2048, 4, 1, 1, 0)
    assert L.sige_reduce_mask(None, None, 0, 2048, 2048, 0, f, FAKE, 0, 0, ctypes.byref(big), None, FAKE, 8,
                              FAKE, None, 0, None) == 3
    assert L.sige_reduce_mask_workspace_bytes(gp) == 2 * 128 + 16  # two halves of 121 block flags rounded up to 16, then the phase words


def test_attention_and_helper_errors(L):
    f = ctypes.c_float(0.1)
    assert L.sige_sparse_attn(FAKE, 320, FAKE, FAKE, 320, 0, 16, 64, 8, 38, f, FAKE, 320, None, 0, None) == 2   # fp32: d % 4
    assert L.sige_sparse_attn(FAKE, 322, FAKE, FAKE, 320, 0, 16, 64, 8, 40, f, FAKE, 320, None, 0, None) == 2   # fp32: stride % 4
    assert L.sige_sparse_attn(FAKE, 320, FAKE, FAKE, 320, 5, 16, 64, 8, 40, f, FAKE, 320, None, 0, None) == 1   # unknown dtype
    assert L.sige_sparse_attn(FAKE, 320, FAKE, FAKE, 320, 2, 16, 64, 8, 36, f, FAKE, 320, None, 0, None) == 2
    assert L.sige_sparse_attn(FAKE, 100, FAKE, FAKE, 320, 2, 16, 64, 8, 40, f, FAKE, 320, None, 0, None) == 1
    assert L.sige_sparse_attn(None, 320, FAKE, FAKE, 320, 2, 16, 64, 8, 40, f, FAKE, 320, None, 0, None) == 1
    assert L.sige_sparse_attn(None, 320, None, None, 320, 2, 0, 64, 8, 40, f, None, 320, None, 0, None) == 0
    # queries by block list: a 1x1 geometry, a host block count, indices
    g1 = api.geom(64, 64, 8, 1, 1, 0)
    g3 = api.geom(64, 64, 8, 3, 1, 1)
    blk = lambda g, idx, n, d=40: L.sige_sparse_attn_blocks(FAKE, 960, ctypes.byref(g), idx, n, FAKE, FAKE, 960, 2,
                                                            4096, 8, d, f, FAKE, 320, None, 0, None)
    assert blk(g3, FAKE, 2) == 2 and "1x1" in err(L)
    assert blk(g1, FAKE, -1) == 1
    assert blk(g1, None, 2) == 1
    assert blk(g1, FAKE, 2, 36) == 2
    assert blk(g1, None, 0) == 0
    assert L.sige_packed_weight_bytes(1, 128, 128, 3) == 128 * 128 * 9 * 2
    assert L.sige_packed_weight_bytes(0, 3, 64, 3) == 32 * 64 * 9 * 4  # Cout padded to 32
    assert L.sige_packed_weight_bytes(1, 128, 24, 3) == 0
    assert L.sige_pack_weight(FAKE, 1, 128, 24, 3, FAKE, None) == 2
    assert L.sige_gn_stats(FAKE, 1, 16, 16, 30, 32, 4, None, None, f, FAKE, FAKE, None, None, None) == 1
    assert L.sige_sparse_attn_workspace_bytes(16384, 4096, 8, 40) == 0     # enough queries: no split
    assert L.sige_sparse_attn_workspace_bytes(64, 4096, 8, 40) > 0


def test_token_layer_modulated_gather_and_list_errors(L):
    f = ctypes.c_float(1e-5)
    g = good_geom()
    gp = ctypes.byref(g)
    # token-wise layers: row protocol and alignment
    assert L.sige_token_norm(FAKE, 1, 320, 320, None, 0, 64, 65, None, None, f, FAKE, 320, None) == 3   # n_rows > max_rows
    assert L.sige_token_norm(FAKE, 1, 320, 320, None, 0, 64, -1, None, None, f, FAKE, 320, None) == 1   # -1 without count
    assert L.sige_token_norm(FAKE, 1, 324, 324, None, 0, 64, 8, None, None, f, FAKE, 324, None) == 2    # C not 16-byte
    assert L.sige_token_norm(FAKE, 1, 8192, 8192, None, 0, 64, 8, None, None, f, FAKE, 8192, None) == 2  # > 8 KiB/token
    assert L.sige_token_norm(FAKE, 1, 320, 320, None, 0, 64, 0, None, None, f, FAKE, 320, None) == 0    # nothing to do
    assert L.sige_geglu(FAKE, 1, 320, 320, None, 0, 64, 8, FAKE, 320, None) == 1                        # x rows hold 2C
    assert L.sige_geglu(None, 1, 320, 640, None, 0, 64, 8, FAKE, 320, None) == 1
    # modulated gather: the modulation tensor is required and holds gamma | beta
    assert L.sige_gather_modulated(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, None, 0, 3, FAKE, None) == 1
    assert L.sige_gather_modulated(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, FAKE, 64, 3, FAKE, None) == 2
    assert L.sige_gather_modulated(FAKE, 1, 64, 64, 0, gp, FAKE, FAKE, 8, -1, None, None, FAKE, 128, 4, FAKE, None) == 1
    # several lists per call: 1..4 lists, each with a workspace of its own
    lst = (api.BlockListDesc * 5)()
    for d in lst:
        d.g = g
        d.indices, d.count, d.max_blocks = 0x10000, 0x10000, 121
        d.workspace, d.workspace_bytes = 0x20000, 2 * 128 + 16
    fz = ctypes.c_float(0.0)
    assert L.sige_reduce_mask_lists(None, None, 0, 64, 64, 0, fz, FAKE, 0, 0, lst, 5, None, None) == 1
    assert L.sige_reduce_mask_lists(None, None, 0, 64, 64, 0, fz, FAKE, 0, 0, lst, 0, None, None) == 1
    assert L.sige_reduce_mask_lists(None, None, 0, 64, 64, 0, fz, FAKE, 0, 0, lst, 2, None, None) == 1   # shared workspace
    assert "share" in err(L)
    lst[1].workspace = None
    assert L.sige_reduce_mask_lists(None, None, 0, 64, 64, 0, fz, FAKE, 0, 0, lst, 2, None, None) == 1   # no workspace
    # convolution workspace query: a layer that never splits, one that does
    assert L.sige_conv_workspace_bytes(1, gp, 64, 64, 121) == 0
    small = api.geom(8, 8, 8, 3, 1, 1)
    assert L.sige_conv_workspace_bytes(1, ctypes.byref(small), 512, 512, 1) > 0


def test_knobs_are_explicit_state(L):
    """The launch-heuristic overrides are set and read through the ABI (no environment variables),
    default to automatic, and an unknown knob is refused."""
    for name, k in api.KNOBS.items():
        assert L.sige_get_knob(k) == -1, name
    assert L.sige_set_knob(api.KNOBS["CONV_CFG"], 3) == 0 and L.sige_get_knob(api.KNOBS["CONV_CFG"]) == 3
    assert L.sige_set_knob(api.KNOBS["CONV_CFG"], -5) == 0 and L.sige_get_knob(api.KNOBS["CONV_CFG"]) == -1
    assert L.sige_set_knob(len(api.KNOBS), 1) == 1 and "knob" in err(L)
    assert L.sige_get_knob(99) == -1
    with api.knobs(ATTN_WGS=64, CONV_KC=4):
        assert api.sige_get_knob("ATTN_WGS") == 64 and api.sige_get_knob("CONV_KC") == 4
        # fewer workgroups to aim for -> fewer key splits -> a smaller workspace
        small = L.sige_sparse_attn_workspace_bytes(64, 4096, 8, 40)
    assert api.sige_get_knob("ATTN_WGS") == -1 and api.sige_get_knob("CONV_KC") == -1
    assert 0 < small < L.sige_sparse_attn_workspace_bytes(64, 4096, 8, 40)
    hdr = open(os.path.join(ROOT, "include", "sige.h")).read()
    for name, k in api.KNOBS.items():
        assert re.search(rf"SIGE_KNOB_{name}\s*=\s*{k}\b", hdr), name
    for src in os.listdir(os.path.join(ROOT, "paper_2211_02048_amd", "csrc")):
        if src.endswith((".hip", ".h")):
            assert "getenv" not in open(os.path.join(ROOT, "paper_2211_02048_amd", "csrc", src)).read(), src


def test_conv_plans_respect_the_lds_of_a_compute_unit(L):
    """Every plan, whatever the block size and channel count, fits the 160 KiB of LDS of a compute
    unit INCLUDING the kernel's static LDS (the block origins), and the shapes that promise two
    resident workgroups fit twice; a layer no shape covers is refused cleanly.  Also: what the plan
    query reports for the layers of the benchmark configurations."""
    import torch
    n_plans = 0
    for dtype in (torch.float16, torch.float32):
        for k in (1, 3):
            for b in (4, 6, 8, 16, 22, 32, 48, 64, 96, 128):
                for cin in (16, 48, 64, 128, 320, 512, 640, 1024, 1280):
                    for nb in (1, 9, 300):
                        g = api.geom(256, 256, b, k, 1, k // 2)
                        for staged in (False, True):
                            try:
                                p = api.sige_conv_plan(dtype, g, cin, 128, nb, staged_math=staged, workspace_bytes=1 << 30)
                            except api.SigeError as e:
                                assert e.code == 2
                                continue
                            n_plans += 1
                            assert p.lds_bytes <= 160 * 1024, (dtype, k, b, cin, nb, p)
                            if p.kernel == 0 and p.shape <= 3 and p.k_steps_per_chunk == 8:
                                assert 2 * p.lds_bytes <= 160 * 1024, (dtype, k, b, cin, nb, p)   # two per compute unit
                            assert p.workgroups >= 1 and p.threads in (256, 512)
    assert n_plans > 1000
    f16 = torch.float16
    # benchmark configuration 2: both convolutions with few blocks take the 64x32 four-wave K-split shape
    g3, g1 = api.geom(256, 256, 16, 3, 1, 1), api.geom(256, 256, 16, 1, 1, 0)
    p3, p1 = api.sige_conv_plan(f16, g3, 128, 128, 16, staged_math=True), api.sige_conv_plan(f16, g1, 128, 256, 16)
    assert (p3.kernel, p3.shape, p3.patch_m, p3.patch_n) == (0, 3, 64, 32) and (p1.kernel, p1.shape) == (0, 3)
    # every block active: the 128x128 shape
    pa = api.sige_conv_plan(f16, g3, 128, 128, 256, staged_math=True)
    assert (pa.kernel, pa.shape, pa.k_steps_per_chunk) == (0, 0, 8)
    # a transformer block's feed-forward layers on 640 tokens of the latent-diffusion step: the few-row kernel
    gt = api.geom(64, 64, 8, 1, 1, 0)
    assert api.sige_conv_plan(torch.bfloat16, gt, 1280, 320, 10).kernel == 1
    with api.knobs(CONV_POINTWISE=0):
        assert api.sige_conv_plan(torch.bfloat16, gt, 1280, 320, 10).kernel == 0
    with pytest.raises(api.SigeError):
        api.sige_conv_plan(f16, g3, 24, 128, 4)            # Cin not a multiple of the K step
    with pytest.raises(api.SigeError):
        api.sige_conv_plan(f16, g3, 128, 128, 0)


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(api, "_lib", None)
    monkeypatch.setattr(api, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(api.SigeError):
        api.sige_version()


def test_struct_layouts_match_the_header(tmp_path):
    """The ctypes mirrors of the header's structs have the C compiler's sizes and field offsets
    (the header is plain C: compiled here with gcc, no GPU toolchain involved)."""
    import subprocess
    src = tmp_path / "layout.c"
    fields = {"sige_geom": ("Geom", ["H_in", "W_out", "block_w", "pad"]),
              "sige_conv_plan_info": ("ConvPlanInfo", [f for f, _ in api.ConvPlanInfo._fields_]),
              "sige_act_out": ("ActOut", ["y", "y_ld", "scale", "shift", "act"]),
              "sige_block_list": ("BlockListDesc", ["g", "indices", "max_blocks", "count", "workspace",
                                                    "workspace_bytes"]),
              "sige_fused_conv_call": ("FusedConvCall", [f for f, _ in api.FusedConvCall._fields_])}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "sige.h"', "int main(void) {"]
    for cname, (_, fs) in fields.items():
        lines.append(f'    printf("{cname} %zu\\n", sizeof({cname}));')
        for f in fs:
            lines.append(f'    printf("{cname}.{f} %zu\\n", offsetof({cname}, {f}));')
    lines += ["    return 0;", "}"]
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    out = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, (pyname, fs) in fields.items():
        cls = getattr(api, pyname)
        assert ctypes.sizeof(cls) == int(out[cname]), cname
        for f in fs:
            assert getattr(cls, f).offset == int(out[f"{cname}.{f}"]), (cname, f)
