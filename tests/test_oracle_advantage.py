"""Pins for the advantage oracle (Sec. 3.2; App. "On Advantage Normalization").  CPU only."""
import numpy as np

from oracle import fast, pods_oracle as po
from paper_2504_13818_amd import inputs


def test_hand_worked():
    r = np.array([[0, 1, 0, 1, 1, 0]], dtype=np.float32)
    sel = np.array([[0, 2, 1, 3]], dtype=np.int32)          # kept rewards 0,0,1,1: mu=.5 sigma=.5
    assert np.array_equal(po.advantage(r, sel), [[-1, -1, 1, 1]])
    r = np.array([[2, 4, 4, 4, 5, 5, 7, 9]], dtype=np.float32)   # textbook: mean 5, sigma 2
    sel = np.arange(8, dtype=np.int32)[None]
    assert np.allclose(po.advantage(r, sel), (r - 5) / 2, rtol=0, atol=1e-15)


def test_zero_sum_unit_variance_and_degenerate_groups():
    for cfg in (0, 1, 2, 4):
        r = inputs.rewards(cfg)
        m = inputs.CONFIGS[cfg]["m"]
        sel, _ = po.select_batch(r, m)
        a = po.advantage(r, sel)
        kept = np.take_along_axis(r, sel, axis=1)
        flat = kept.max(axis=1) == kept.min(axis=1)
        assert np.all(a[flat] == 0.0)
        assert np.allclose(a.sum(axis=1), 0.0, atol=1e-12)          # total advantage 0
        assert np.allclose((a[~flat] ** 2).mean(axis=1), 1.0, atol=1e-12)
        assert np.allclose(fast.advantage(r, sel), a, rtol=0, atol=1e-14)


def test_std_eps():
    r = np.array([[0, 0, 1, 1]], dtype=np.float32)
    sel = np.arange(4, dtype=np.int32)[None]
    assert np.allclose(po.advantage(r, sel, std_eps=0.5), [[-.5, -.5, .5, .5]])
    assert np.allclose(fast.advantage(r, sel, std_eps=0.5), [[-.5, -.5, .5, .5]])
