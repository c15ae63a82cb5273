"""Shared pieces of the GPU parity tests: seeded cases, oracle references, tolerance checks."""
from __future__ import annotations

import numpy as np

from oracle import fast, pods_oracle as po
from paper_2504_13818_amd import inputs

# Tolerances from the build's stated bar: loss / gradients within 2e-3 relative, 1e-4 absolute.
RTOL, ATOL = 2e-3, 1e-4


def oracle_adv(cfg: int, R: int) -> np.ndarray:
    """adv[R] from the oracle's own select + advantage on the config's rewards.  The kept rollouts
    are taken in a fixed shuffled order, so that a short list still mixes prompt groups with and
    without reward variance (the latter have all-zero advantages) and both signs."""
    c = inputs.CONFIGS[cfg]
    r = inputs.rewards(cfg)
    sel, _, _ = fast.select(r, c["m"])
    a = fast.advantage(r, sel).reshape(-1)
    a = a[np.random.default_rng(cfg).permutation(a.size)]
    reps = -(-R // a.size)
    return np.tile(a, reps)[:R].astype(np.float32)


def loss_case(cfg: int, R: int, T: int, d: int, V: int, sigma: float = 0.05, ragged: bool = True,
              gemm_dtype=np.float32):
    """Inputs for one token-loss call in the config's value distributions, at the given sizes."""
    c = inputs.CONFIGS[cfg]
    h, w = inputs.dense(cfg, R, T, d, V)
    tok = inputs.tokens(cfg, R, T, V)
    lens = inputs.lengths(cfg, R, T) if ragged else np.full(R, T, np.int32)
    adv = oracle_adv(cfg, R)
    zeros = np.zeros((R, T), np.float32)
    cur = po.grpo_token_loss(h, w, tok, zeros, adv, lens, c["clip_eps"], gemm_dtype=gemm_dtype,
                             want_dw=False)["logp"]
    old = inputs.old_logp_from(cur, cfg, sigma)
    return dict(cfg=cfg, hidden=h, w=w, tokens=tok, lengths=lens, adv=adv, old_logp=old,
                clip_eps=c["clip_eps"], dtype=c["dtype"])


def to_device(case, torch, device="cuda"):
    dt = torch.bfloat16 if case["dtype"] == "bf16" else torch.float32
    t = lambda x, d=None: torch.from_numpy(np.ascontiguousarray(x)).to(device)
    return dict(hidden=t(case["hidden"]).to(dt), w=t(case["w"]).to(dt), tokens=t(case["tokens"]),
                lengths=t(case["lengths"]), adv=t(case["adv"]), old_logp=t(case["old_logp"]))


def gpu_loss(lib, torch, case, grad_scale=1.0, workspace=None, use_lengths=True):
    dv = to_device(case, torch)
    out = lib.grpo_token_loss_fwd_bwd(dv["hidden"], dv["w"], dv["tokens"], dv["old_logp"], dv["adv"],
                                      dv["lengths"] if use_lengths else None, case["clip_eps"],
                                      grad_scale=grad_scale, workspace=workspace)
    torch.cuda.synchronize()
    return dict(loss=float(out["loss"].cpu()[0]), logp=out["logp"].cpu().numpy().astype(np.float64),
                d_hidden=out["d_hidden"].cpu().numpy().astype(np.float64),
                d_w=out["d_w_lm"].cpu().numpy().astype(np.float64))


def oracle_loss(case, grad_scale=1.0, gemm_dtype=np.float32):
    return po.grpo_token_loss(case["hidden"], case["w"], case["tokens"], case["old_logp"], case["adv"],
                              case["lengths"], case["clip_eps"], grad_scale=grad_scale,
                              gemm_dtype=gemm_dtype)


def assert_close_tensor(name, got, ref, rtol=RTOL, atol=ATOL):
    """Elementwise rtol/atol plus the scale-aware checks (max and Frobenius norm)."""
    diff = np.abs(got - ref)
    bad = diff > rtol * np.abs(ref) + atol
    assert not bad.any(), f"{name}: {bad.sum()} elements outside rtol={rtol} atol={atol}; max diff {diff.max():.3e}"
    scale = np.abs(ref).max()
    assert diff.max() <= rtol * scale + 1e-30, f"{name}: max|diff| {diff.max():.3e} > {rtol} * max|ref| {scale:.3e}"
    fro = np.linalg.norm(ref)
    assert np.linalg.norm(got - ref) <= rtol * fro + 1e-30, \
        f"{name}: Frobenius diff {np.linalg.norm(got - ref):.3e} > {rtol} * {fro:.3e}"


def check_loss(got, ref):
    assert abs(got["loss"] - ref["loss"]) <= RTOL * abs(ref["loss"]) + 1e-7, (got["loss"], ref["loss"])
    assert_close_tensor("logp", got["logp"], ref["logp"])
    assert_close_tensor("d_hidden", got["d_hidden"], ref["d_hidden"])
    assert_close_tensor("d_w", got["d_w"], ref["d_w"])


def softmax_term_magnitudes(case, grad_scale=1.0, gemm_dtype=np.float32, block=256):
    """A[v, k] = sum over valid tokens t with y_t != v of |dz_tv| |h_tk|: the summed magnitudes of the terms
    of d_w_lm[v, k] that come from the softmax part of the logit gradient (everything but the generated
    token's own logit), from the oracle's per-token rows.  The matrix-core path rounds exactly these
    terms' two factors to fp16 (unit roundoff 2^-11 each), so 2^-10 A bounds what that rounding can move
    an element by, whatever cancellation its terms undergo."""
    h, w, tok, lens = case["hidden"], case["w"], case["tokens"], case["lengths"].astype(np.int64)
    R, T, d = h.shape
    ii = np.concatenate([np.full(int(lens[i]), i, dtype=np.int64) for i in range(R)])
    tt = np.concatenate([np.arange(int(lens[i]), dtype=np.int64) for i in range(R)])
    A = np.zeros((w.shape[0], d))
    for s in range(0, len(ii), block):
        bi, bt = ii[s:s + block], tt[s:s + block]
        hb = h[bi, bt]
        cb = 1.0 / (R * lens[bi].astype(np.float64))
        out = po.token_rows(hb, w, tok[bi, bt], case["old_logp"][bi, bt], case["adv"][bi], cb, case["clip_eps"],
                            grad_scale, gemm_dtype)
        mag = np.abs(out["dz"])
        mag[np.arange(len(bi)), tok[bi, bt]] = 0.0
        A += (mag.astype(gemm_dtype).T @ np.abs(hb).astype(gemm_dtype)).astype(np.float64)
    return A


def assert_close_dw_unit_scale(got, ref, A, rtol=RTOL, atol=ATOL):
    """d_w_lm at a gradient scale where its terms are O(1): elementwise rtol / atol plus the worst-case fp16
    rounding of the softmax terms (see softmax_term_magnitudes), and the norm-wise bars."""
    diff = np.abs(got - ref)
    bad = diff > rtol * np.abs(ref) + atol + 2.0 ** -10 * A
    assert not bad.any(), f"d_w: {bad.sum()} elements outside the bound; max diff {diff.max():.3e}"
    assert diff.max() <= rtol * np.abs(ref).max()
    assert np.linalg.norm(got - ref) <= rtol * np.linalg.norm(ref)
