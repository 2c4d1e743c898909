"""The seeded workload generators reproduce the stated recipes."""
import numpy as np
import torch

from paper_2211_02048_amd import inputs


def test_config1_recipe():
    c = inputs.config1()
    m = c["mask"]
    assert m.shape == (64, 64) and abs(m.sum() / 4096 - 0.05) < 0.01
    ys, xs = np.nonzero(m)
    assert m[ys.min():ys.max() + 1, xs.min():xs.max() + 1].all()  # one rectangle
    same = (c["a_orig"] == c["a_edit"]).all(dim=2).numpy()
    assert np.array_equal(~same, m.astype(bool))  # bit-identical outside, changed inside
    c2 = inputs.config1()
    assert torch.equal(c["a_edit"], c2["a_edit"]) and torch.equal(c["w"], c2["w"])  # seeded


def test_config2_recipe():
    c = inputs.config2(H=128, W=128, C=32, Cs=64, area_frac=0.01 * 4)  # same blob area in px
    m = c["mask"]
    assert abs(int(m.sum()) - 655) <= 33
    assert c["a_orig"].dtype == torch.float16 and c["w"].shape == (32, 32, 3, 3)
    assert c["w_s"].shape == (64, 32, 1, 1)
    same = (c["a_orig"] == c["a_edit"]).all(dim=2).numpy()
    assert not (~same & ~m.astype(bool)).any()      # nothing changes outside the mask
    assert (~same).sum() >= 0.99 * m.sum()          # (fp16 rounding may swallow a rare change)


def test_token_mask_fraction():
    for frac in (0.01, 0.05, 0.2):
        m = inputs.token_mask(3, 64, 64, frac)
        assert abs(m.mean() - frac) <= 0.2 * frac + 1 / 4096
