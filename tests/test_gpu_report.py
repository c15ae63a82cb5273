"""The token loss's report (diagnostic counters and what the call found in its device-side arguments),
the range scales of its fp16 operands, and the optional reward check, through the C ABI."""
import numpy as np
import pytest

from paper_2504_13818_amd import inputs
from tests import helpers as H

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _run(pods, case, grad_scale=1.0, **kw):
    dv = H.to_device(case, torch)
    out = pods.grpo_token_loss_fwd_bwd(dv["hidden"], dv["w"], dv["tokens"], dv["old_logp"], dv["adv"], dv["lengths"],
                                       case["clip_eps"], grad_scale=grad_scale, **kw)
    rep = pods.grpo_token_loss_report(out["workspace"])
    return out, rep


@pytest.mark.parametrize("cfg,R,T,d,V,dtype", [(1, 12, 200, 256, 3000, "bf16"), (0, 8, 64, 96, 500, "f32")])
def test_clip_counter_matches_the_oracle(pods, cfg, R, T, d, V, dtype):
    """clipped_tokens = number of valid tokens whose clipped term is selected.  Both sides decide rho > 1+eps
    in their own precision, so tokens whose ratio lies within 1e-4 of a clip bound may fall either way."""
    case = H.loss_case(cfg, R, T, d, V, sigma=0.3, gemm_dtype=np.float64 if dtype == "f32" else np.float32)
    case["dtype"] = dtype
    ref = H.oracle_loss(case, gemm_dtype=np.float64 if dtype == "f32" else np.float32)
    out, rep = _run(pods, case)
    eps = case["clip_eps"]
    valid = np.arange(T)[None, :] < case["lengths"][:, None]
    a = case["adv"][:, None]
    near = valid & (a != 0) & ((np.abs(ref["rho"] - (1 + eps)) < 1e-4) | (np.abs(ref["rho"] - (1 - eps)) < 1e-4))
    want = int(ref["clipped"].sum())
    assert want > 50                                                  # the case really clips
    assert abs(rep["clipped_tokens"] - want) <= int(near.sum())
    assert rep["valid_tokens"] == int(case["lengths"].sum()) == rep["backward_tokens"]
    assert rep["bad_lengths"] == 0 and rep["bad_tokens"] == 0
    # the cut tokens are exactly those with a zero d_hidden row although the advantage is not zero
    dh = out["d_hidden"].cpu().numpy()
    zero_rows = (np.abs(dh).sum(axis=-1) == 0) & valid & (a != 0)
    assert int(zero_rows.sum()) == rep["clipped_tokens"]


def test_report_maxima_and_skipped_rollouts(pods):
    case = H.loss_case(1, 8, 96, 256, 1500, sigma=0.2)
    case["adv"][::3] = 0.0
    ref = H.oracle_loss(case, grad_scale=50.0)
    out, rep = _run(pods, case, grad_scale=50.0, skip_zero_advantage=True)
    lens = case["lengths"]
    assert rep["valid_tokens"] == int(lens.sum())
    assert rep["backward_tokens"] == int(lens[case["adv"] != 0].sum())
    valid = np.arange(96)[None, :] < lens[:, None]
    assert rep["max_abs_w"] == np.abs(case["w"]).max()
    assert rep["max_abs_hidden"] == np.abs(case["hidden"][valid]).max()
    # g = d loss / d logp = -c a rho grad_scale where active
    c = 1.0 / (8 * lens.astype(np.float64))[:, None]
    g = np.where(ref["clipped"] | ~valid, 0.0, c * case["adv"][:, None] * ref["rho"] * 50.0)
    assert rep["max_abs_g"] == pytest.approx(np.abs(g).max(), rel=1e-4)


def test_out_of_range_token_ids_and_lengths_are_clamped_and_counted(pods):
    """A token id outside [0, V) or a length outside [0, T] must not make any kernel index out of bounds:
    both are taken as clamped and counted, and the call equals the call on the clamped inputs."""
    R, T, d, V = 6, 70, 128, 900
    case = H.loss_case(4, R, T, d, V, sigma=0.2)
    lens = case["lengths"].copy()
    lens[1], lens[4] = T + 9, -3
    tok = case["tokens"].copy()
    tok[0, 0], tok[2, 5], tok[3, 1] = V, -7, V + 100000          # positions inside their rollouts' lengths
    assert lens[0] > 0 and lens[2] > 5 and lens[3] > 1
    bad = dict(case, lengths=lens, tokens=tok)
    good = dict(case, lengths=np.clip(lens, 0, T).astype(np.int32), tokens=np.clip(tok, 0, V - 1).astype(np.int32))
    out_b, rep_b = _run(pods, bad)
    out_g, rep_g = _run(pods, good)
    assert rep_b["bad_lengths"] == 2 and rep_b["bad_tokens"] == 3
    assert rep_g["bad_lengths"] == 0 and rep_g["bad_tokens"] == 0
    assert rep_b["valid_tokens"] == rep_g["valid_tokens"] == int(good["lengths"].sum())
    for key in ("loss", "logp", "d_hidden", "d_w_lm"):
        assert torch.equal(out_b[key], out_g[key]), key
    H.check_loss(dict(loss=float(out_g["loss"].cpu()[0]), logp=out_g["logp"].cpu().numpy().astype(np.float64),
                      d_hidden=out_g["d_hidden"].cpu().numpy().astype(np.float64),
                      d_w=out_g["d_w_lm"].cpu().numpy().astype(np.float64)), H.oracle_loss(good))


@pytest.mark.parametrize("w_big,h_gain", [(300.0, 1.0), (0.5, 4096.0), (2.0 ** -20, 2.0 ** -12)])
def test_bf16_operand_ranges_follow_the_inputs(pods, w_big, h_gain):
    """The fp16 working copies of W_lm and of the token-weighted hidden states are scaled from the inputs'
    own maxima: a weight of 300 (beyond fp16 under a fixed scale of 256), hidden states in the thousands,
    or tiny ones, give finite gradients within the parity bar."""
    R, T, d, V = 4, 80, 128, 700
    case = H.loss_case(1, R, T, d, V, sigma=0.1)
    w = case["w"].copy()
    w[5, 7] = w_big
    w[123, 64] = -w_big
    h = inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(case["hidden"] * np.float32(h_gain * 0.05)))
    w = inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(w))
    case = dict(case, w=w, hidden=h)
    # old_logp near the current log-prob of THIS problem, so that ratios stay near 1
    from oracle import pods_oracle as po
    cur = po.grpo_token_loss(h, w, case["tokens"], np.zeros((R, T), np.float32), case["adv"], case["lengths"], 0.2,
                             gemm_dtype=np.float32, want_dw=False)["logp"]
    case["old_logp"] = inputs.old_logp_from(cur, 1, 0.1)
    scale = float(R * case["lengths"].mean())
    ref = H.oracle_loss(case, grad_scale=scale)
    got = H.gpu_loss(pods, torch, case, grad_scale=scale)
    for key in ("logp", "d_hidden", "d_w"):
        assert np.isfinite(got[key]).all(), key
    assert abs(got["loss"] - ref["loss"]) <= H.RTOL * abs(ref["loss"]) + 1e-7
    H.assert_close_tensor("logp", got["logp"], ref["logp"])
    # the gradients' sizes follow the inputs' here (far above or below 1), where a fixed absolute floor
    # means nothing: the bar is taken against the size of each tensor, in max- and in Frobenius norm
    for key in ("d_hidden", "d_w"):
        diff = got[key] - ref[key]
        assert np.abs(ref[key]).max() > 0
        assert np.abs(diff).max() <= H.RTOL * np.abs(ref[key]).max(), key
        assert np.linalg.norm(diff) <= H.RTOL * np.linalg.norm(ref[key]), key


def test_check_rewards_counts_non_finite_values(pods):
    r = inputs.rewards(2).copy()
    rep = pods.pods_check_rewards(torch.from_numpy(r).cuda())
    torch.cuda.synchronize()
    assert rep.cpu().tolist() == [0, -1]
    r[3, 5] = np.nan
    r[1, 30] = np.inf
    r[9, 0] = -np.inf
    rep = pods.pods_check_rewards(torch.from_numpy(r).cuda())
    torch.cuda.synchronize()
    assert rep.cpu().tolist() == [3, 1 * r.shape[1] + 30]
    big = np.zeros((70000, 33), np.float32)
    big[69999, 32] = np.nan
    rep = pods.pods_check_rewards(torch.from_numpy(big).cuda())
    assert rep.cpu().tolist() == [1, 70000 * 33 - 1]
