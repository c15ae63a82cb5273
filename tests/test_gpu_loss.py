"""GPU parity: grpo_token_loss_fwd_bwd through the C ABI against the CPU oracle
(loss, log-probs, d_hidden, d_w_lm within 2e-3 relative / 1e-4 absolute, plus norm-wise checks)."""
import numpy as np
import pytest

from paper_2504_13818_amd import inputs
from tests import helpers as H

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_config0_fp32_full(pods):
    """B=4, m=4 -> R=16 rollouts, T=64, d=256, V=1024, fp32; oracle in fp64."""
    case = H.loss_case(0, 16, 64, 256, 1024, sigma=0.05, gemm_dtype=np.float64)
    H.check_loss(H.gpu_loss(pods, torch, case), H.oracle_loss(case, gemm_dtype=np.float64))


def test_config0_fp32_clipping_active_and_unit_scale(pods):
    case = H.loss_case(0, 16, 64, 256, 1024, sigma=0.3, gemm_dtype=np.float64)
    scale = 16 * 64.0
    got = H.gpu_loss(pods, torch, case, grad_scale=scale)
    ref = H.oracle_loss(case, grad_scale=scale, gemm_dtype=np.float64)
    H.check_loss(got, ref)
    assert (np.abs(ref["d_hidden"]).sum(axis=-1) == 0).any()      # some tokens really were clipped
    zero_rows = np.abs(ref["d_hidden"]).sum(axis=-1) == 0
    assert np.all(got["d_hidden"][zero_rows] == 0)


def test_fp32_ragged_odd_shapes(pods):
    case = H.loss_case(0, 5, 37, 100, 333, sigma=0.3, gemm_dtype=np.float64)
    case["lengths"][2] = 0                                        # an empty rollout still counts in R
    H.check_loss(H.gpu_loss(pods, torch, case), H.oracle_loss(case, gemm_dtype=np.float64))


@pytest.mark.parametrize("R,T,d,V", [(6, 96, 256, 1000), (3, 300, 512, 2500), (9, 64, 192, 777)])
def test_bf16_small_shapes(pods, R, T, d, V):
    """bf16 matrix-core path at sizes spanning several tiles with ragged tails in every dimension."""
    case = H.loss_case(1, R, T, d, V, sigma=0.2)
    H.check_loss(H.gpu_loss(pods, torch, case), H.oracle_loss(case))
    scale = float(R * case["lengths"].mean())
    H.check_loss(H.gpu_loss(pods, torch, case, grad_scale=scale), H.oracle_loss(case, grad_scale=scale))


def test_bf16_small_workspace_many_token_blocks(pods):
    case = H.loss_case(4, 4, 128, 256, 3000, sigma=0.2)
    ws = torch.empty((pods.grpo_token_loss_workspace_min_bytes(4, 128, 256, 3000, pods.PODS_BF16),),
                     dtype=torch.uint8, device="cuda")
    H.check_loss(H.gpu_loss(pods, torch, case, workspace=ws), H.oracle_loss(case))


def test_bf16_no_lengths_and_determinism(pods):
    case = H.loss_case(1, 4, 128, 256, 1500, sigma=0.2, ragged=False)
    a = H.gpu_loss(pods, torch, case, use_lengths=False)
    b = H.gpu_loss(pods, torch, case, use_lengths=True)
    H.check_loss(a, H.oracle_loss(case))
    for key in ("logp", "d_hidden", "d_w"):
        assert np.array_equal(a[key], b[key])
    assert a["loss"] == b["loss"]


@pytest.mark.parametrize("R,T,d,V", [(4, 320, 2048, 151936), (3, 700, 512, 20000), (9, 130, 768, 9000)])
def test_bf16_padded_batches_are_bitwise_repeatable(pods, R, T, d, V):
    """Ragged batches whose padded capacity spans more 256-token tiles than their valid tokens do, small
    enough that a launch has only a few blocks of tiles: every tile must be taken by exactly one
    workgroup (two would race on d_hidden), so four runs agree bit for bit and with the oracle."""
    case = H.loss_case(1, R, T, d, V, sigma=0.05)
    assert (int(case["lengths"].sum()) + 255) // 256 < (R * T + 255) // 256
    scale = float(R * case["lengths"].mean())
    runs = [H.gpu_loss(pods, torch, case, grad_scale=scale) for _ in range(4)]
    for other in runs[1:]:
        for key in ("logp", "d_hidden", "d_w"):
            assert np.array_equal(runs[0][key], other[key]), key
    H.check_loss(runs[0], H.oracle_loss(case, grad_scale=scale))


@pytest.mark.parametrize("cfg,R,T", [(1, 4, 320), (2, 2, 400), (4, 6, 160)])
def test_bf16_full_head_reduced_tokens(pods, cfg, R, T):
    """Full d and V of the config (lm_head shape), a few hundred valid tokens."""
    c = inputs.CONFIGS[cfg]
    case = H.loss_case(cfg, R, T, c["d"], c["V"], sigma=0.05)
    scale = float(R * case["lengths"].mean())
    H.check_loss(H.gpu_loss(pods, torch, case, grad_scale=scale), H.oracle_loss(case, grad_scale=scale))


def test_bf16_peaked_logits_beyond_the_first_forward_launch(pods):
    """A vocabulary of three forward launches (8192 columns each) where some tokens have one logit about 15 nats
    above the rest, sitting in the second or third launch.  For half of them it is the generated token's own
    logit (the exponent the token's tiles agree on after the first launch then already covers it); for the
    other half it is another row (that row's tile lies far above the agreed exponent, keeps its own, and every
    other tile of the token is brought down to it afterwards, most of its numerators into fp16's subnormal
    range or to zero).  Both must match the oracle like any other case."""
    from oracle import pods_oracle as po
    cfg, R, T, d, V = 1, 6, 100, 256, 20000
    c = inputs.CONFIGS[cfg]
    h, w = inputs.dense(cfg, R, T, d, V)
    tok = inputs.tokens(cfg, R, T, V)
    lens = inputs.lengths(cfg, R, T)
    rng = np.random.default_rng(77)
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    hot_rows = rng.choice(np.arange(8192, V), size=24, replace=False)
    w[hot_rows] += 0.5 * u                                       # z rises by 0.5 * beta at the hot rows
    peaked = rng.random((R, T)) < 0.4
    h[peaked] += 30.0 * u                                        # ... by about 15 nats for these tokens
    own = peaked & (rng.random((R, T)) < 0.5)
    tok[own] = rng.choice(hot_rows, size=int(own.sum())).astype(tok.dtype)
    h = inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(h))
    w = inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(w))
    adv = H.oracle_adv(cfg, R)
    cur = po.grpo_token_loss(h, w, tok, np.zeros((R, T), np.float32), adv, lens, c["clip_eps"],
                             want_dw=False)["logp"]
    valid = np.arange(T)[None, :] < lens[:, None]
    assert (cur[valid & own] > -6.0).mean() > 0.9 and (cur[valid & peaked & ~own] < -8.0).mean() > 0.9
    case = dict(cfg=cfg, hidden=h, w=w, tokens=tok, lengths=lens, adv=adv,
                old_logp=inputs.old_logp_from(cur, cfg, 0.2), clip_eps=c["clip_eps"], dtype="bf16")
    H.check_loss(H.gpu_loss(pods, torch, case), H.oracle_loss(case))
    # unit scale: the hot rows of d_w_lm are cancelling sums of terms of size 0.1 (probabilities of 1/24 times
    # hidden elements of size 2), so d_w_lm gets the rounding allowance of its fp16 operands, as in the large cases
    scale = float(R * lens.mean())
    got, ref = H.gpu_loss(pods, torch, case, grad_scale=scale), H.oracle_loss(case, grad_scale=scale)
    assert abs(got["loss"] - ref["loss"]) <= H.RTOL * abs(ref["loss"]) + 1e-7
    H.assert_close_tensor("logp", got["logp"], ref["logp"])
    H.assert_close_tensor("d_hidden", got["d_hidden"], ref["d_hidden"])
    H.assert_close_dw_unit_scale(got["d_w"], ref["d_w"], H.softmax_term_magnitudes(case, grad_scale=scale))
