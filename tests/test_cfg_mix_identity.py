"""The guidance mix commutes with the projection (it is linear and has no bias): the checker's mixed logits equal
the projection of the mixed hidden rows exactly, and rounding the mixed rows to bf16 - the one thing the library's
hidden-row mix adds - moves them by a few 1e-3 of a row's largest |g| at the paper's guidance scales."""
import numpy as np
import pytest

from oracle import verify_oracle as vo
from paper_2605_07230_amd import workloads as wl


def _rows(seed, n=24, h=512, v=2048):
    rng = np.random.default_rng(seed)
    hc = wl.round_bf16(rng.standard_normal((n, h)).astype(np.float32))
    hu = wl.round_bf16(hc + 0.5 * rng.standard_normal((n, h)).astype(np.float32))   # correlated, as guidance rows are
    w = wl.round_bf16((0.02 * rng.standard_normal((v, h))).astype(np.float32))
    return hc, hu, w


@pytest.mark.parametrize("scale", [0.0, 1.0, 3.0, 5.0, 7.5])
def test_mixing_hidden_rows_is_the_same_definition(scale):
    hc, hu, w = _rows(1)
    g, _, _, _ = vo.lmhead_cfg(hc, hu, w, scale, 0.9, 0)
    mixed = hu.astype(np.float64) + scale * (hc.astype(np.float64) - hu.astype(np.float64))
    g1, _, _, _ = vo.lmhead_cfg(mixed, None, w, 1.0, 0.9, 0)
    np.testing.assert_allclose(g1, g, rtol=0, atol=1e-12 * max(1.0, scale))


@pytest.mark.parametrize("scale,bar", [(3.0, 3e-3), (5.0, 4e-3), (7.5, 6e-3)])
def test_one_bf16_rounding_of_the_mixed_rows_stays_far_inside_the_bar(scale, bar):
    hc, hu, w = _rows(2, n=32, h=4096, v=1024)
    g, _, _, lse = vo.lmhead_cfg(hc, hu, w, scale, 1.0, 0)
    mixed = wl.round_bf16(hu + np.float32(scale) * (hc - hu))
    g1, _, _, lse1 = vo.lmhead_cfg(mixed, None, w, 1.0, 1.0, 0)
    rel = (np.abs(g1 - g).max(axis=1) / np.abs(g).max(axis=1)).max()
    assert 0.0 < rel <= bar, rel                      # bf16 results are held to 2e-2
    assert np.abs(lse1 - lse).max() <= 2e-2
