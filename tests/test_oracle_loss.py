"""Pins for the token-loss oracle (objective of Sec. 3.1 / 3.2).  CPU only."""
import math

import numpy as np
import pytest
import torch
from scipy.special import log_softmax

from oracle import pods_oracle as po


def _problem(seed, R=3, T=5, d=4, V=7, sigma=0.3, ragged=True):
    g = np.random.default_rng(seed)
    h = g.standard_normal((R, T, d))
    w = g.standard_normal((V, d)) * 0.7
    y = g.integers(0, V, (R, T)).astype(np.int32)
    lens = g.integers(1, T + 1, R).astype(np.int32) if ragged else np.full(R, T, np.int32)
    adv = g.standard_normal(R)
    cur = np.take_along_axis(log_softmax(h @ w.T, axis=-1), y[..., None].astype(np.int64), axis=-1)[..., 0]
    old = cur + g.normal(0, sigma, cur.shape)
    return h, w, y, old, adv, lens


def test_closed_form_two_token_vocabulary():
    """V=2, d=1, one rollout of one token: p(y=0) = sigmoid(h (w0 - w1))."""
    h = np.array([[[2.0]]]); w = np.array([[0.5], [-0.25]]); y = np.array([[0]], np.int32)
    p0 = 1.0 / (1.0 + math.exp(-2.0 * 0.75))
    for old_p, a, eps in ((0.9, 1.5, 0.2), (0.5, 1.5, 0.2), (0.5, -2.0, 0.2), (0.95, -2.0, 0.1)):
        rho = p0 / old_p
        want = min(rho * a, min(max(rho, 1 - eps), 1 + eps) * a)
        out = po.grpo_token_loss(h, w, y, np.array([[math.log(old_p)]]), np.array([a]), None, eps)
        assert out["loss"] == pytest.approx(-want, rel=1e-14)
        assert out["logp"][0, 0] == pytest.approx(math.log(p0), rel=1e-14)
        active = not ((a > 0 and rho > 1 + eps) or (a < 0 and rho < 1 - eps))
        # d loss / d h = -a * rho * (1 - p0) * (w0 - w1) when the unclipped term is selected
        want_dh = -a * rho * (1 - p0) * 0.75 if active else 0.0
        assert out["d_hidden"][0, 0, 0] == pytest.approx(want_dh, rel=1e-13, abs=1e-300)
        want_dw0 = -a * rho * (1 - p0) * 2.0 if active else 0.0
        assert out["d_w"][0, 0] == pytest.approx(want_dw0, rel=1e-13, abs=1e-300)
        assert out["d_w"][1, 0] == pytest.approx(-want_dw0, rel=1e-13, abs=1e-300)


def test_rho_one_reduces_to_weighted_nll_autograd():
    """With old_logp equal to the current log-prob every ratio is 1, nothing clips, the
    objective is the mean advantage, and its gradient is that of the advantage-weighted
    log-likelihood, which torch's log_softmax + autograd provide independently."""
    h, w, y, _, adv, lens = _problem(1)
    R, T, _ = h.shape
    cur = np.take_along_axis(log_softmax(h @ w.T, axis=-1), y[..., None].astype(np.int64), axis=-1)[..., 0]
    out = po.grpo_token_loss(h, w, y, cur, adv, lens, 0.2)
    assert out["loss"] == pytest.approx(-adv.mean(), rel=1e-12)
    ht = torch.tensor(h, requires_grad=True); wt = torch.tensor(w, requires_grad=True)
    lp = torch.log_softmax(ht @ wt.T, dim=-1).gather(-1, torch.tensor(y, dtype=torch.int64)[..., None])[..., 0]
    mask = torch.arange(T)[None, :] < torch.tensor(lens)[:, None]
    weight = torch.tensor(adv)[:, None] / (R * torch.tensor(lens, dtype=torch.float64)[:, None])
    (-(weight * lp * mask).sum()).backward()
    assert np.allclose(out["d_hidden"], ht.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(out["d_w"], wt.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(out["logp"][mask.numpy()], lp.detach().numpy()[mask.numpy()], rtol=1e-12)


@pytest.mark.parametrize("seed", [2, 3])
def test_finite_differences(seed):
    h, w, y, old, adv, lens = _problem(seed, sigma=0.3)
    eps = 0.2
    out = po.grpo_token_loss(h, w, y, old, adv, lens, eps, grad_scale=3.0)
    f = lambda hh, ww: po.grpo_token_loss(hh, ww, y, old, adv, lens, eps, want_dw=False)["loss"]
    step = 1e-6
    g = np.random.default_rng(seed)
    for _ in range(25):
        i, t, k = g.integers(0, h.shape[0]), g.integers(0, h.shape[1]), g.integers(0, h.shape[2])
        hp, hm = h.copy(), h.copy(); hp[i, t, k] += step; hm[i, t, k] -= step
        fd = 3.0 * (f(hp, w) - f(hm, w)) / (2 * step)
        assert out["d_hidden"][i, t, k] == pytest.approx(fd, rel=2e-6, abs=1e-8)
        v, k = g.integers(0, w.shape[0]), g.integers(0, w.shape[1])
        wp, wm = w.copy(), w.copy(); wp[v, k] += step; wm[v, k] -= step
        fd = 3.0 * (f(h, wp) - f(h, wm)) / (2 * step)
        assert out["d_w"][v, k] == pytest.approx(fd, rel=2e-6, abs=1e-8)


def test_definition_by_plain_loops():
    """The objective spelled token by token with scipy's log_softmax."""
    h, w, y, old, adv, lens = _problem(4)
    R = h.shape[0]; eps = 0.2
    total = 0.0
    for i in range(R):
        acc = 0.0
        for t in range(lens[i]):
            lp = log_softmax(w @ h[i, t])[y[i, t]]
            rho = math.exp(lp - old[i, t])
            acc += min(rho * adv[i], min(max(rho, 1 - eps), 1 + eps) * adv[i])
        total += acc / lens[i]
    assert po.grpo_token_loss(h, w, y, old, adv, lens, eps)["loss"] == pytest.approx(-total / R, rel=1e-12)


def test_clip_branches_and_zero_rows():
    """Slow to adopt, quick to abandon: a>0 with rho>1+eps and a<0 with rho<1-eps give no
    gradient; a<0 with rho>1+eps does."""
    g = np.random.default_rng(9)
    R, T, d, V = 4, 1, 3, 5
    h = g.standard_normal((R, T, d)); w = g.standard_normal((V, d)); y = g.integers(0, V, (R, T)).astype(np.int32)
    cur = np.take_along_axis(log_softmax(h @ w.T, axis=-1), y[..., None].astype(np.int64), axis=-1)[..., 0]
    old = cur - np.log(np.array([[1.5], [0.5], [1.5], [1.0]]))       # rho = 1.5, 0.5, 1.5, 1.0
    adv = np.array([1.0, -1.0, -1.0, 0.0])
    out = po.grpo_token_loss(h, w, y, old, adv, None, 0.2)
    assert np.all(out["d_hidden"][0] == 0) and np.all(out["d_hidden"][1] == 0)
    assert np.any(out["d_hidden"][2] != 0)
    assert np.all(out["d_hidden"][3] == 0)                           # zero advantage
    # the mask of cut tokens: exactly the first two (a zero advantage is not "clipped")
    assert out["clipped"][:, 0].tolist() == [True, True, False, False]
    assert np.allclose(out["rho"][:, 0], [1.5, 0.5, 1.5, 1.0], rtol=1e-12)
    # loss value: clipped terms contribute (1+eps)*a, (1-eps)*a; third min(1.5*-1, 1.2*-1) = -1.5
    assert out["loss"] == pytest.approx(-(1.2 * 1.0 + 0.8 * -1.0 + 1.5 * -1.0 + 0.0) / 4, rel=1e-12)


def test_invariants_padding_and_vocab_permutation():
    h, w, y, old, adv, lens = _problem(6, R=4, T=6, d=5, V=9)
    out = po.grpo_token_loss(h, w, y, old, adv, lens, 0.2)
    assert np.allclose(out["d_w"].sum(axis=0), 0.0, atol=1e-14)      # each softmax-gradient row sums to 0
    for i in range(h.shape[0]):
        assert np.all(out["d_hidden"][i, lens[i]:] == 0) and np.all(out["logp"][i, lens[i]:] == 0)
    # garbage in the padded region changes nothing
    h2, y2, old2 = h.copy(), y.copy(), old.copy()
    for i in range(h.shape[0]):
        h2[i, lens[i]:] = 1e3; y2[i, lens[i]:] = 0; old2[i, lens[i]:] = -50.0
    out2 = po.grpo_token_loss(h2, w, y2, old2, adv, lens, 0.2)
    assert out2["loss"] == out["loss"] and np.array_equal(out2["d_w"], out["d_w"])
    # relabelling the vocabulary permutes d_w's rows and leaves loss and d_hidden alone
    perm = np.random.default_rng(0).permutation(w.shape[0])
    inv = np.argsort(perm)
    out3 = po.grpo_token_loss(h, w[perm], inv[y].astype(np.int32), old, adv, lens, 0.2)
    assert out3["loss"] == pytest.approx(out["loss"], rel=1e-13)
    assert np.allclose(out3["d_hidden"], out["d_hidden"], rtol=1e-11, atol=1e-14)
    assert np.allclose(out3["d_w"], out["d_w"][perm], rtol=1e-11, atol=1e-14)


def test_keep_all_equals_grpo_objective():
    """m = n: the PODS objective over S = {1..n} is the GRPO objective with the full-group
    advantages (same formula, 1/n in place of 1/m)."""
    h, w, y, old, _, lens = _problem(8, R=6)
    r = np.array([[0, 1, 1, 0, 1, 0.5]], dtype=np.float32)
    sel, k = po.select_batch(r, 6)
    assert sorted(sel[0]) == list(range(6)) and k[0] == 0
    a_sel = po.advantage(r, sel)[0]
    r64 = r[0].astype(np.float64)
    a_full = (r64 - r64.mean()) / r64.std()                          # numpy's population std
    lhs = po.grpo_token_loss(h[sel[0]], w, y[sel[0]], old[sel[0]], a_sel, lens[sel[0]], 0.2)
    rhs = po.grpo_token_loss(h, w, y, old, a_full, lens, 0.2)
    assert lhs["loss"] == pytest.approx(rhs["loss"], rel=1e-12)
    assert np.allclose(lhs["d_w"], rhs["d_w"], rtol=1e-10, atol=1e-14)


def test_fp32_gemm_variant_close_to_fp64():
    h, w, y, old, adv, lens = _problem(10, R=3, T=8, d=16, V=33)
    a = po.grpo_token_loss(h.astype(np.float32), w.astype(np.float32), y, old, adv, lens, 0.2)
    b = po.grpo_token_loss(h.astype(np.float32), w.astype(np.float32), y, old, adv, lens, 0.2,
                           gemm_dtype=np.float32, block=5)
    assert a["loss"] == pytest.approx(b["loss"], rel=1e-5)
    assert np.allclose(a["d_w"], b["d_w"], rtol=1e-4, atol=1e-6)


# ---- KL penalty (Table 2 lists a coefficient; the estimator is a reading, see the oracle) ----------

def _ref_logp(seed, old):
    return (old + np.random.default_rng(seed + 100).normal(0, 0.3, old.shape)).astype(np.float32)


def test_kl_definition_by_plain_loops_and_sign():
    h, w, y, old, adv, lens = _problem(5)
    ref = _ref_logp(5, old)
    R = h.shape[0]; eps = 0.2; beta = 0.04
    total, kl_total = 0.0, 0.0
    for i in range(R):
        acc = 0.0
        for t in range(lens[i]):
            lp = log_softmax(w @ h[i, t])[y[i, t]]
            rho = math.exp(lp - old[i, t])
            x = float(ref[i, t]) - lp
            kl = math.exp(x) - x - 1.0
            assert kl >= 0.0
            kl_total += kl
            acc += min(rho * adv[i], min(max(rho, 1 - eps), 1 + eps) * adv[i]) - beta * kl
        total += acc / lens[i]
    with_kl = po.grpo_token_loss(h, w, y, old, adv, lens, eps, ref_logp=ref, kl_coef=beta)["loss"]
    without = po.grpo_token_loss(h, w, y, old, adv, lens, eps)["loss"]
    assert with_kl == pytest.approx(-total / R, rel=1e-12)
    assert kl_total > 0 and with_kl > without                      # a penalty raises the loss


def test_kl_vanishes_at_the_reference_and_with_zero_coefficient():
    h, w, y, old, adv, lens = _problem(6)
    base = po.grpo_token_loss(h, w, y, old, adv, lens, 0.2)
    same = po.grpo_token_loss(h, w, y, old, adv, lens, 0.2, ref_logp=_ref_logp(6, old), kl_coef=0.0)
    for k in ("logp", "d_hidden", "d_w"):
        assert np.array_equal(base[k], same[k])
    # ref = the policy's own log-probs: KL and its gradient are zero (its minimum)
    at_ref = po.grpo_token_loss(h, w, y, old, adv, lens, 0.2, ref_logp=base["logp"].astype(np.float64), kl_coef=5.0)
    assert at_ref["loss"] == pytest.approx(base["loss"], rel=1e-12)
    assert np.allclose(at_ref["d_hidden"], base["d_hidden"], rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", [7, 8])
def test_kl_finite_differences(seed):
    h, w, y, old, adv, lens = _problem(seed, sigma=0.3)
    ref = _ref_logp(seed, old)
    eps, beta = 0.2, 0.7
    out = po.grpo_token_loss(h, w, y, old, adv, lens, eps, grad_scale=3.0, ref_logp=ref, kl_coef=beta)
    f = lambda hh, ww: po.grpo_token_loss(hh, ww, y, old, adv, lens, eps, want_dw=False, ref_logp=ref, kl_coef=beta)["loss"]
    step = 1e-6
    g = np.random.default_rng(seed)
    for _ in range(20):
        i, t, k = g.integers(0, h.shape[0]), g.integers(0, h.shape[1]), g.integers(0, h.shape[2])
        hp, hm = h.copy(), h.copy(); hp[i, t, k] += step; hm[i, t, k] -= step
        fd = 3.0 * (f(hp, w) - f(hm, w)) / (2 * step)
        assert out["d_hidden"][i, t, k] == pytest.approx(fd, rel=2e-6, abs=1e-8)
        v, k = g.integers(0, w.shape[0]), g.integers(0, w.shape[1])
        wp, wm = w.copy(), w.copy(); wp[v, k] += step; wm[v, k] -= step
        fd = 3.0 * (f(h, wp) - f(h, wm)) / (2 * step)
        assert out["d_w"][v, k] == pytest.approx(fd, rel=2e-6, abs=1e-8)


def test_kl_second_order_expansion():
    """Near the reference the estimator is x^2 / 2 to leading order (the KL of nearby distributions)."""
    for x in (1e-3, -2e-3, 5e-3):
        kl = math.exp(x) - x - 1.0
        assert kl == pytest.approx(x * x / 2, rel=abs(x))
