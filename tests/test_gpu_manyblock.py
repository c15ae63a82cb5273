"""Elementwise oracle parity where the token-tiled matrix-core kernels take the tile mapping the
benchmark shapes run: a token-tile capacity of 512 (R = 128 rollouts x T = 1024, about 290 tiles of valid
tokens), so that the forward launches (32 and 15 vocabulary tiles) and the d_hidden launches
(8 d-tiles at d = 2048, as in the Qwen2.5-3B-shaped config) all have at least 64 blocks of tiles, and a
vocabulary of two forward launches with a ragged last tile.  Every element of logp, d_hidden and d_w_lm is
compared with the CPU oracle, at the natural scale of the loss (the plain 2e-3 / 1e-4 bar) and at unit
scale (d_w_lm there with the rounding allowance its fp16 operands call for)."""
import numpy as np
import pytest

import bench
from paper_2504_13818_amd import inputs
from tests import helpers as H

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


# (config, R, T, d, V, least token-tile capacity for 64 blocks of tiles in the d_hidden launch: blocks are
# 4 token tiles x up to 8 d-tiles, so 8 d-tiles need 253 token tiles, 14 or 16 d-tiles (two block columns) 125)
CASES = [(1, 128, 1024, 2048, 12000, 253), (2, 64, 1024, 3584, 12000, 125), (4, 96, 512, 4096, 10000, 125)]


@pytest.mark.parametrize("cfg,R,T,d,V,min_tiles", CASES)
def test_bf16_many_blocks_of_tiles_elementwise(pods, cfg, R, T, d, V, min_tiles):
    c = inputs.CONFIGS[cfg]
    print(f"many-block case cfg={cfg} R={R} T={T} d={d} V={V}", flush=True)
    h, w = inputs.dense(cfg, R, T, d, V)
    tok = inputs.tokens(cfg, R, T, V)
    lens = inputs.lengths(cfg, R, T)
    adv = H.oracle_adv(cfg, R)
    n_valid = int(lens.sum())
    assert (R * T) // 256 >= min_tiles            # the launch is sized (and its tiles mapped) by the capacity
    assert n_valid // 256 >= min_tiles // 2       # ... and valid tokens reach far into it
    dev = torch.device("cuda:0")
    hd, wd = torch.from_numpy(h).to(dev).bfloat16(), torch.from_numpy(w).to(dev).bfloat16()
    tokd, lend, advd = torch.from_numpy(tok).to(dev), torch.from_numpy(lens).to(dev), torch.from_numpy(adv).to(dev)
    # old_logp is an input: the current log-prob (plain torch ops, input synthesis) plus noise
    cur = bench.current_logp_torch(torch, hd, wd, tokd).cpu().numpy()
    old = inputs.old_logp_from(cur, cfg, 0.1)
    oldd = torch.from_numpy(old).to(dev)
    case = dict(cfg=cfg, hidden=h, w=w, tokens=tok, lengths=lens, adv=adv, old_logp=old, clip_eps=c["clip_eps"],
                dtype="bf16")
    scale = float(R * lens.mean())
    print("oracle ...", flush=True)
    ref = H.oracle_loss(case, grad_scale=scale)                       # one pass: about a minute of CPU time
    print("oracle done", flush=True)

    def run(gs):
        out = pods.grpo_token_loss_fwd_bwd(hd, wd, tokd, oldd, advd, lend, c["clip_eps"], grad_scale=gs)
        torch.cuda.synchronize()
        return dict(loss=float(out["loss"].cpu()[0]), logp=out["logp"].cpu().numpy().astype(np.float64),
                    d_hidden=out["d_hidden"].cpu().numpy().astype(np.float64),
                    d_w=out["d_w_lm"].cpu().numpy().astype(np.float64))

    got = run(scale)
    # unit scale: per-token weights are O(1), so an element of d_w_lm can be a cancelling sum of O(1) terms;
    # log-probs and d_hidden meet the plain elementwise bar, d_w_lm the bar plus the fp16 rounding of its terms
    assert abs(got["loss"] - ref["loss"]) <= H.RTOL * abs(ref["loss"]) + 1e-7
    H.assert_close_tensor("logp", got["logp"], ref["logp"])
    H.assert_close_tensor("d_hidden", got["d_hidden"], ref["d_hidden"])
    H.assert_close_dw_unit_scale(got["d_w"], ref["d_w"], H.softmax_term_magnitudes(case, grad_scale=scale))
    assert np.abs(ref["d_hidden"]).max() > 1e-2 and np.abs(ref["d_w"]).max() > 1e-2     # not vacuous at unit scale
    # natural scale: the oracle's gradients are linear in grad_scale (it multiplies g by it), so the
    # reference is the same pass divided by the scale
    del got
    got1 = run(1.0)
    ref1 = dict(loss=ref["loss"], logp=ref["logp"], d_hidden=ref["d_hidden"] / scale, d_w=ref["d_w"] / scale)
    H.check_loss(got1, ref1)
