"""GPU parity: grpo_token_loss_fwd_bwd_kl (the objective with the KL penalty whose coefficient the
paper's Table 2 lists) through the C ABI against the CPU oracle."""
import numpy as np
import pytest

from oracle import pods_oracle as po
from tests import helpers as H

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _run(pods, case, ref, beta, grad_scale=1.0, **kw):
    dv = H.to_device(case, torch)
    out = pods.grpo_token_loss_fwd_bwd(dv["hidden"], dv["w"], dv["tokens"], dv["old_logp"], dv["adv"], dv["lengths"],
                                       case["clip_eps"], grad_scale=grad_scale,
                                       ref_logp=torch.from_numpy(ref).cuda(), kl_coef=beta, **kw)
    torch.cuda.synchronize()
    return dict(loss=float(out["loss"].cpu()[0]), logp=out["logp"].cpu().numpy().astype(np.float64),
                d_hidden=out["d_hidden"].cpu().numpy().astype(np.float64),
                d_w=out["d_w_lm"].cpu().numpy().astype(np.float64))


def _oracle(case, ref, beta, grad_scale=1.0):
    return po.grpo_token_loss(case["hidden"], case["w"], case["tokens"], case["old_logp"], case["adv"],
                              case["lengths"], case["clip_eps"], grad_scale=grad_scale, gemm_dtype=np.float32,
                              ref_logp=ref, kl_coef=beta)


@pytest.mark.parametrize("cfg,R,T,d,V,beta", [(0, 8, 32, 64, 500, 0.04), (1, 6, 120, 256, 1300, 0.04),
                                              (4, 5, 90, 512, 3000, 1.5)])
def test_kl_penalty_matches_oracle(pods, cfg, R, T, d, V, beta):
    case = H.loss_case(cfg, R, T, d, V, sigma=0.2)
    ref = (case["old_logp"] + np.random.default_rng(cfg).normal(0, 0.3, case["old_logp"].shape)).astype(np.float32)
    H.check_loss(_run(pods, case, ref, beta), _oracle(case, ref, beta))
    scale = float(R * case["lengths"].mean())
    H.check_loss(_run(pods, case, ref, beta, grad_scale=scale), _oracle(case, ref, beta, grad_scale=scale))


def test_kl_zero_coefficient_is_the_plain_objective(pods):
    case = H.loss_case(1, 4, 100, 256, 900, sigma=0.2)
    ref = (case["old_logp"] + 0.5).astype(np.float32)
    a = _run(pods, case, ref, 0.0)
    b = H.gpu_loss(pods, torch, case)
    for key in ("logp", "d_hidden", "d_w"):
        assert np.array_equal(a[key], b[key])
    assert a["loss"] == b["loss"]


def test_kl_moves_tokens_without_advantage(pods):
    """With a zero advantage the surrogate gives no gradient; the penalty still pulls towards the reference."""
    case = H.loss_case(1, 4, 100, 256, 900, sigma=0.2)
    case["adv"][:] = 0.0
    ref = (case["old_logp"] + 0.7).astype(np.float32)
    got = _run(pods, case, ref, 0.5)
    assert np.abs(got["d_hidden"]).max() > 0
    H.check_loss(got, _oracle(case, ref, 0.5))


def test_kl_argument_checks(pods):
    case = H.loss_case(0, 2, 8, 64, 50)
    dv = H.to_device(case, torch)
    with pytest.raises(pods.PodsError):
        pods.grpo_token_loss_fwd_bwd(dv["hidden"], dv["w"], dv["tokens"], dv["old_logp"], dv["adv"], dv["lengths"], 0.2,
                                     ref_logp=dv["old_logp"], kl_coef=-1.0)
