"""GPU parity: grpo_token_loss_fwd_bwd_ex with PODS_LOSS_SKIP_ZERO_ADVANTAGE (rollouts whose
advantage is zero, i.e. the kept rollouts of a prompt without reward variance, Sec. 3.2, are left out
of the backward pass) through the C ABI against the CPU oracle, which knows no skipping: the flag
must not change what is computed."""
import numpy as np
import pytest

from oracle import pods_oracle as po
from tests import helpers as H

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _run(pods, case, grad_scale=1.0, use_lengths=True, **kw):
    dv = H.to_device(case, torch)
    out = pods.grpo_token_loss_fwd_bwd(dv["hidden"], dv["w"], dv["tokens"], dv["old_logp"], dv["adv"],
                                       dv["lengths"] if use_lengths else None, case["clip_eps"],
                                       grad_scale=grad_scale, skip_zero_advantage=True, **kw)
    torch.cuda.synchronize()
    return dict(loss=float(out["loss"].cpu()[0]), logp=out["logp"].cpu().numpy().astype(np.float64),
                d_hidden=out["d_hidden"].cpu().numpy().astype(np.float64),
                d_w=out["d_w_lm"].cpu().numpy().astype(np.float64))


def _zero_some(case, every):
    """Zero advantages in a pattern that leaves live and skipped rollouts interleaved."""
    a = case["adv"]
    a[::every] = 0.0
    a[1] = -0.0                                   # a negative zero is a zero
    if not np.any(a != 0):
        a[-1] = 1.0
    return case


@pytest.mark.parametrize("cfg,R,T,d,V", [(0, 9, 40, 48, 333),          # fp32 path
                                         (1, 8, 300, 256, 1300),       # bf16: several token tiles, ragged
                                         (2, 7, 130, 512, 2100),
                                         (4, 12, 70, 320, 777)])
def test_skip_matches_oracle(pods, cfg, R, T, d, V):
    case = _zero_some(H.loss_case(cfg, R, T, d, V, sigma=0.2), 3)
    H.check_loss(_run(pods, case), H.oracle_loss(case))
    scale = float(R * case["lengths"].mean())
    H.check_loss(_run(pods, case, grad_scale=scale), H.oracle_loss(case, grad_scale=scale))


@pytest.mark.parametrize("cfg,R,T,d,V", [(0, 6, 24, 64, 300), (1, 6, 260, 256, 1300)])
def test_skip_changes_nothing_but_summation_order(pods, cfg, R, T, d, V):
    """Against the same call without the flag: log-probs and d_hidden bit for bit (a token's
    row does not depend on where it is packed); d_w_lm, summed over tokens in another order, to
    rounding."""
    case = _zero_some(H.loss_case(cfg, R, T, d, V, sigma=0.2), 2)
    a = _run(pods, case)
    b = H.gpu_loss(pods, torch, case)
    assert a["loss"] == pytest.approx(b["loss"], rel=1e-6)            # block partials in another order
    assert np.array_equal(a["logp"], b["logp"])
    assert np.array_equal(a["d_hidden"], b["d_hidden"])
    assert np.linalg.norm(a["d_w"] - b["d_w"]) <= 1e-5 * np.linalg.norm(b["d_w"])
    # skipped rollouts: exact zero rows; live rollouts: something flows
    dead = case["adv"] == 0
    assert np.all(a["d_hidden"][dead] == 0) and np.abs(a["d_hidden"][~dead]).max() > 0


def test_skip_without_lengths_and_with_nothing_live(pods):
    case = H.loss_case(1, 5, 64, 256, 900, sigma=0.2, ragged=False)
    case = _zero_some(case, 2)
    H.check_loss(_run(pods, case, use_lengths=False), H.oracle_loss(case))
    case["adv"][:] = 0.0                          # every prompt without reward variance
    got = _run(pods, case)
    assert got["loss"] == 0.0 and not got["d_hidden"].any() and not got["d_w"].any()
    assert np.allclose(got["logp"], H.oracle_loss(case)["logp"], rtol=H.RTOL, atol=H.ATOL)


def test_skip_with_accumulation_and_with_kl(pods):
    case = _zero_some(H.loss_case(1, 6, 100, 256, 900, sigma=0.2), 2)
    ref = H.oracle_loss(case)
    acc = torch.full((900, 256), 0.5, dtype=torch.float32, device="cuda")
    got = _run(pods, case, out={"d_w_lm": acc}, accumulate_d_w=True)
    H.assert_close_tensor("d_w", got["d_w"] - 0.5, ref["d_w"])
    # a KL penalty gives zero-advantage rollouts a gradient: the flag must then skip nothing
    rl = (case["old_logp"] + 0.4).astype(np.float32)
    got = _run(pods, case, ref_logp=torch.from_numpy(rl).cuda(), kl_coef=0.3)
    want = po.grpo_token_loss(case["hidden"], case["w"], case["tokens"], case["old_logp"], case["adv"],
                              case["lengths"], case["clip_eps"], gemm_dtype=np.float32, ref_logp=rl, kl_coef=0.3)
    H.check_loss(got, want)
    assert np.abs(got["d_hidden"][case["adv"] == 0]).max() > 0


def test_skip_flag_checks(pods):
    case = H.loss_case(0, 2, 8, 16, 40)
    dv = H.to_device(case, torch)
    lib = pods.load()
    out = [torch.empty(s, device="cuda") for s in ((1,), (2, 8), (2, 8, 16), (40, 16))]
    ws = torch.empty(pods.grpo_token_loss_workspace_bytes(2, 8, 16, 40, pods.PODS_F32), dtype=torch.uint8, device="cuda")
    import ctypes
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    args = lambda flags, kl: (vp(dv["hidden"]), vp(dv["w"]), vp(dv["tokens"]), vp(dv["old_logp"]), None, vp(dv["adv"]),
                              vp(dv["lengths"]), 2, 8, 16, 40, pods.PODS_F32, 0.2, kl, 1.0, flags, vp(out[0]), vp(out[1]),
                              vp(out[2]), vp(out[3]), vp(ws), ws.numel(), None)
    assert lib.grpo_token_loss_fwd_bwd_ex(*args(4, 0.0)) == 1           # unknown flag bit
    assert lib.grpo_token_loss_fwd_bwd_ex(*args(0, 0.1)) == 1           # KL coefficient without ref_logp
    assert lib.grpo_token_loss_fwd_bwd_ex(*args(3, 0.0)) == 0
    torch.cuda.synchronize()


def test_skip_at_full_size_matches_the_plain_call(pods):
    """Config 1 at the benchmark's size and launch configuration: with the flag, d_hidden and the
    log-probs are the plain call's bit for bit, d_w_lm agrees to summation order, and the rows of
    zero-advantage rollouts are exact zeros."""
    import bench
    from paper_2504_13818_amd import inputs
    cfg = 1
    c = inputs.CONFIGS[cfg]
    B, m, T, d, V = c["B"], c["m"], c["T"], c["d"], c["V"]
    R = B * m
    dev = torch.device("cuda:0")
    rewards = torch.from_numpy(inputs.rewards(cfg)).to(dev)
    lengths = torch.from_numpy(inputs.lengths(cfg)).to(dev)
    tokens = torch.from_numpy(inputs.tokens(cfg, R, T, V)).to(dev)
    hidden, w = inputs.dense_torch(cfg, dev)
    cur = bench.current_logp_torch(torch, hidden, w, tokens)
    g = torch.Generator(device=dev)
    g.manual_seed(inputs.seed_for(cfg, 5))
    old_logp = (cur + 0.05 * torch.randn(cur.shape, generator=g, device=dev)).contiguous()
    del cur
    sel, _ = pods.pods_select(rewards, m)
    adv = pods.pods_advantage(rewards, sel).view(-1)
    dead = adv == 0
    assert 0 < int(dead.sum()) < R                                    # the config has prompts without reward variance
    plain = pods.grpo_token_loss_fwd_bwd(hidden, w, tokens, old_logp, adv, lengths, c["clip_eps"])
    ws = plain.pop("workspace")
    skip = pods.grpo_token_loss_fwd_bwd(hidden, w, tokens, old_logp, adv, lengths, c["clip_eps"], workspace=ws,
                                        skip_zero_advantage=True)
    torch.cuda.synchronize()
    assert torch.equal(skip["logp"], plain["logp"])
    assert torch.equal(skip["d_hidden"], plain["d_hidden"])
    assert float(skip["d_hidden"][dead].abs().max()) == 0.0
    assert float(skip["loss"]) == pytest.approx(float(plain["loss"]), rel=1e-6, abs=1e-12)
    diff = float((skip["d_w_lm"].double() - plain["d_w_lm"].double()).norm())
    assert diff <= 1e-5 * float(plain["d_w_lm"].double().norm())
