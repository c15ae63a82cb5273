"""CPU oracle for the PODS hot path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the GPU library must compute.  It is imported
only by tests, by the smoke check and by the benchmark's cpu_baseline leg; the product path
never calls it, and it shares no code with the HIP kernels.

What each function follows:

* ``stable_argsort``           Alg. 2 step 1 ("argsort"), with the tie order fixed as
                               (reward, index) ascending.
* ``select_exact``             Alg. 2 as printed: start from the m lowest, try every split k,
                               replace only on a strictly larger variance.  Variance is the
                               population variance of Lemma 3.1's proof, evaluated in exact
                               rational arithmetic on the float32 inputs.
* ``max_variance_bruteforce``  the definition S = argmax_{|S|=m} Var (Sec. 3.3), all C(n,m)
                               subsets, exact rationals.
* ``select_prefix``            Theorem 1's O(n log n) evaluation: prefix sums of r and r^2,
                               Var = E[x^2] - E[x]^2, O(1) per k; float64.
* ``downsample_maxr`` / ``downsample_perc`` / ``downsample_rand``
                               the other rules of Sec. 3.2 (max-reward, percentile, random), each
                               written as its definition on the (reward, index) sorted order.
* ``advantage``                a_{S,i} = (r_i - mu_S) / sigma_S over the kept rollouts (Sec. 3.2).
* ``advantage_before``         the "Before" variant of App. "On Advantage Normalization": mean and
                               standard deviation from all n rollouts of the group.
* ``gather_kept``              the kept rollouts of every prompt, concatenated (Sec. 3.2).
* ``grpo_token_loss``          L_PODS (Sec. 3.2) with the policy's last layer written out
                               (logits = hidden . W_lm^T, softmax over the vocabulary), returned
                               as loss = -L_PODS with its analytic gradient w.r.t. hidden and W_lm.

Pins (tests/test_oracle_*.py): brute force for n <= 12, Lemma 3.1's structure, Theorem 2's closed
form for binary rewards, hand-worked small cases, Sigma a = 0 (App. "On Advantage Normalization"),
the rho == 1 reduction to a library log-softmax NLL gradient, finite differences, m = n (PODS
objective equals the GRPO objective), the clip branches, vocabulary-permutation equivariance.
"""
from __future__ import annotations

import itertools
from fractions import Fraction

import numpy as np


# --------------------------------------------------------------------------------------------
# Stage 1: max-variance down-sampling (Alg. 2, Lemma 3.1, Theorem 1)
# --------------------------------------------------------------------------------------------

def stable_argsort(r) -> list[int]:
    """Indices of r in ascending (reward, index) order.  -0.0 and +0.0 compare equal."""
    return sorted(range(len(r)), key=lambda i: (float(r[i]), i))


def _variance_exact(vals) -> Fraction:
    """Population variance (1/m) sum x^2 - mean^2 of float values, as an exact rational."""
    m = len(vals)
    xs = [Fraction(float(v)) for v in vals]
    mean = sum(xs, Fraction(0)) / m
    return sum((x * x for x in xs), Fraction(0)) / m - mean * mean


def select_exact(r, m: int):
    """Alg. 2 on one group.  Returns (indices, k): the m-k lowest then the k highest of the
    sorted order, for the smallest k that attains the maximal variance."""
    n = len(r)
    assert 0 < m <= n
    ind = stable_argsort(r)
    best_k = 0
    best_var = _variance_exact([r[i] for i in ind[:m]])
    for k in range(1, m + 1):
        cand = ind[: m - k] + ind[n - k:]
        v = _variance_exact([r[i] for i in cand])
        if v > best_var:
            best_var, best_k = v, k
    return ind[: m - best_k] + ind[n - best_k:], best_k


def max_variance_bruteforce(r, m: int) -> Fraction:
    """max over all subsets of size m of the exact population variance (Sec. 3.3 definition)."""
    return max(_variance_exact([r[i] for i in S]) for S in itertools.combinations(range(len(r)), m))


def select_prefix(r, m: int):
    """Theorem 1's evaluation on one group in float64.

    Sort, prefix-sum r and r^2 over the sorted order, then for each k the candidate's
    m * sum(x^2) - (sum x)^2 (m^2 times its variance, so the same arg-max) in O(1).
    Candidates whose multiset equals the previous candidate's (the value entering at the top
    equals the value leaving at the bottom) are passed over, so that a tie between identical
    multisets can never be decided by rounding; the first of each such run is the smallest k.
    """
    n = len(r)
    ind = stable_argsort(r)
    s = np.array([float(r[i]) for i in ind], dtype=np.float64)
    p1 = np.zeros(n + 1)
    p2 = np.zeros(n + 1)
    for j in range(n):
        p1[j + 1] = p1[j] + s[j]
        p2[j + 1] = p2[j] + s[j] * s[j]
    u1 = np.zeros(m + 1)   # sum of the k highest, accumulated from the top down
    u2 = np.zeros(m + 1)
    for k in range(1, m + 1):
        u1[k] = u1[k - 1] + s[n - k]
        u2[k] = u2[k - 1] + s[n - k] * s[n - k]
    best_k = 0
    best = m * p2[m] - p1[m] * p1[m]
    for k in range(1, m + 1):
        if s[n - k] == s[m - k]:
            continue
        S = p1[m - k] + u1[k]
        Q = p2[m - k] + u2[k]
        D = m * Q - S * S
        if D > best:
            best, best_k = D, k
    return ind[: m - best_k] + ind[n - best_k:], best_k


def select_batch(rewards: np.ndarray, m: int, exact: bool = False):
    """Apply the selector to every row of rewards[B, n] -> (sel_idx[B, m] int32, sel_k[B] int32)."""
    B = rewards.shape[0]
    idx = np.zeros((B, m), dtype=np.int32)
    ks = np.zeros(B, dtype=np.int32)
    f = select_exact if exact else select_prefix
    for b in range(B):
        i, k = f(rewards[b], m)
        idx[b], ks[b] = i, k
    return idx, ks


# --------------------------------------------------------------------------------------------
# Stage 1, other rules (Sec. 3.2: random, percentile and max-reward down-sampling)
# --------------------------------------------------------------------------------------------

def downsample_maxr(r, m: int) -> list[int]:
    """D_maxr: the m highest rewards.  Returned in ascending (reward, index) order, so among equal
    rewards at the cut the highest indices are the ones kept."""
    n = len(r)
    assert 0 < m <= n
    return stable_argsort(r)[n - m:]


def downsample_perc(r, m: int) -> list[int]:
    """D_perc: the (j - 0.5)/m quantiles of the group's rewards, j = 1..m.

    The paper does not say which order statistic realises a quantile q.  Reading taken: position
    floor(q n) of the ascending (reward, index) order (0-based), i.e. floor((2j - 1) n / (2m)),
    in integer arithmetic.  The m positions are distinct whenever m <= n."""
    n = len(r)
    assert 0 < m <= n
    ind = stable_argsort(r)
    return [ind[((2 * j - 1) * n) // (2 * m)] for j in range(1, m + 1)]


def downsample_rand(keys, m: int) -> list[int]:
    """D_rand: m indices uniformly without replacement.  The randomness is an input: one key per
    rollout (independent uniform 32-bit integers); the m smallest keys are kept, ties by index,
    returned in ascending (key, index) order.  With exchangeable keys every m-subset is equally
    likely.  The rewards play no part."""
    n = len(keys)
    assert 0 < m <= n
    return sorted(range(n), key=lambda i: (int(keys[i]), i))[:m]


def downsample_batch(rewards: np.ndarray, m: int, rule: str, keys: np.ndarray | None = None) -> np.ndarray:
    """Row-wise application of one of the rules above -> sel_idx[B, m] int32."""
    B = rewards.shape[0]
    out = np.zeros((B, m), dtype=np.int32)
    for b in range(B):
        if rule == "maxr":
            out[b] = downsample_maxr(rewards[b], m)
        elif rule == "perc":
            out[b] = downsample_perc(rewards[b], m)
        elif rule == "rand":
            out[b] = downsample_rand(keys[b], m)
        else:
            raise ValueError(rule)
    return out


# --------------------------------------------------------------------------------------------
# Stage 2: advantages over the kept rollouts (Sec. 3.2)
# --------------------------------------------------------------------------------------------

def advantage(rewards: np.ndarray, sel_idx: np.ndarray, std_eps: float = 0.0) -> np.ndarray:
    """adv[B, m] = (r_i - mu_S) / (sigma_S + std_eps), population sigma, float64.

    A group whose kept rewards are all equal has sigma_S = 0; its advantages are 0.
    """
    B, m = sel_idx.shape
    out = np.zeros((B, m), dtype=np.float64)
    for b in range(B):
        x = rewards[b, sel_idx[b]].astype(np.float64)
        if x.max() == x.min():
            continue
        mu = x.sum() / m
        sigma = np.sqrt(((x - mu) ** 2).sum() / m)
        out[b] = (x - mu) / (sigma + std_eps)
    return out


def gather_kept(per_rollout: np.ndarray, sel_idx: np.ndarray) -> np.ndarray:
    """Concatenation of the kept rollouts over a batch of prompts (Sec. 3.2; Alg. 1 steps 3-4):
    per_rollout[B, n, ...] (any per-rollout record: token ids, old log-probs, lengths, ...) and
    sel_idx[B, m] -> out[B*m, ...] with out[b*m + j] = per_rollout[b, sel_idx[b, j]]."""
    B, m = sel_idx.shape
    out = np.empty((B * m,) + per_rollout.shape[2:], dtype=per_rollout.dtype)
    for b in range(B):
        for j in range(m):
            out[b * m + j] = per_rollout[b, sel_idx[b, j]]
    return out


def advantage_before(rewards: np.ndarray, sel_idx: np.ndarray, std_eps: float = 0.0) -> np.ndarray:
    """ "Before" normalisation (App. "On Advantage Normalization"): the statistics come from all n
    rollouts of the group, a_i = (r_i - mu_all) / (sigma_all + std_eps) for the kept i; float64.
    A group whose n rewards are all equal gets 0."""
    B, m = sel_idx.shape
    n = rewards.shape[1]
    out = np.zeros((B, m), dtype=np.float64)
    for b in range(B):
        x = rewards[b].astype(np.float64)
        if x.max() == x.min():
            continue
        mu = x.sum() / n
        sigma = np.sqrt(((x - mu) ** 2).sum() / n)
        out[b] = (x[sel_idx[b]] - mu) / (sigma + std_eps)
    return out


# --------------------------------------------------------------------------------------------
# Stage 3: GRPO-PODS token loss through the lm_head (Sec. 3.1 / 3.2 objective)
# --------------------------------------------------------------------------------------------

def token_rows(h: np.ndarray, w: np.ndarray, y: np.ndarray, old_logp: np.ndarray,
               a: np.ndarray, c: np.ndarray, clip_eps: float, grad_scale: float = 1.0,
               gemm_dtype=np.float64, ref_logp: np.ndarray | None = None, kl_coef: float = 0.0):
    """The objective's inner term for K independent token positions.

    h[K, d] hidden rows, w[V, d], y[K] generated token, old_logp[K] = log pi_fixed(y),
    a[K] the rollout's advantage, c[K] = 1 / (R * |o_i|) the averaging weight.
    Returns dict with logp[K], obj[K] (the min[...] term, minus the KL penalty if any),
    g[K] = d loss / d logp, dz[K, V] = d loss / d logits, d_h[K, d]; all float64.

    KL penalty (Table 2 lists a KL coefficient, 0.04 in one setting and 0 in the others; the paper
    gives no formula).  Reading taken: the per-token estimator of the GRPO objective the paper
    builds on, with x = log pi_ref(y) - log pi_theta(y):  KL = exp(x) - x - 1  (>= 0, 0 iff the two
    agree), subtracted from the token's term with weight kl_coef.
    """
    K = h.shape[0]
    wg = w.astype(gemm_dtype, copy=False)
    z = (h.astype(gemm_dtype, copy=False) @ wg.T).astype(np.float64)      # logits
    zmax = z.max(axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=1))
    rows = np.arange(K)
    logp = z[rows, y] - lse                                                    # log pi_theta(y)
    rho = np.exp(logp - old_logp.astype(np.float64))                           # importance ratio
    a = a.astype(np.float64)
    unclipped = rho * a
    clipped = np.clip(rho, 1.0 - clip_eps, 1.0 + clip_eps) * a
    obj = np.minimum(unclipped, clipped)
    # d obj / d rho: a where the unclipped term is the one selected, else 0.
    inactive = ((a > 0) & (rho > 1.0 + clip_eps)) | ((a < 0) & (rho < 1.0 - clip_eps))
    dobj_dlogp = np.where(inactive, 0.0, a * rho)
    if ref_logp is not None and kl_coef != 0.0:
        x = ref_logp.astype(np.float64) - logp
        obj = obj - kl_coef * (np.exp(x) - x - 1.0)
        dobj_dlogp = dobj_dlogp - kl_coef * (1.0 - np.exp(x))                  # d(-KL)/d logp = exp(x) - 1
    g = -c.astype(np.float64) * dobj_dlogp * grad_scale                        # loss = -objective
    p = np.exp(z - lse[:, None])                                               # softmax
    dz = -g[:, None] * p
    dz[rows, y] += g
    d_h = (dz.astype(gemm_dtype, copy=False) @ wg).astype(np.float64)
    return dict(logp=logp, obj=obj, g=g, dz=dz, d_h=d_h, lse=lse, inactive=inactive, rho=rho)


def grpo_token_loss(hidden: np.ndarray, w: np.ndarray, tokens: np.ndarray, old_logp: np.ndarray,
                    adv: np.ndarray, lengths: np.ndarray | None, clip_eps: float,
                    grad_scale: float = 1.0, gemm_dtype=np.float64, block: int = 256,
                    want_dw: bool = True, ref_logp: np.ndarray | None = None, kl_coef: float = 0.0):
    """loss = -(1/R) sum_i (1/|o_i|) sum_{t<|o_i|} { min[rho a_i, clip(rho, 1-eps, 1+eps) a_i]
    - kl_coef KL_t } over R kept rollouts, and its gradient (KL_t: see token_rows; absent by default).

    hidden[R, T, d], w[V, d], tokens[R, T], old_logp[R, T], adv[R], lengths[R] (None: all T).
    Returns dict(loss, logp[R, T], d_hidden[R, T, d], d_w[V, d]); float64.  Positions at or past
    a rollout's length get logp = 0 and a zero d_hidden row.  The gradients are those of
    grad_scale * loss.  Also returned: clipped[R, T] (bool), the valid positions where the clipped
    term is the selected one so that no gradient flows, and rho[R, T], the importance ratios there.
    """
    R, T, d = hidden.shape
    V = w.shape[0]
    lens = np.full(R, T, dtype=np.int64) if lengths is None else lengths.astype(np.int64)
    ii, tt = [], []
    for i in range(R):
        ii.extend([i] * int(lens[i]))
        tt.extend(range(int(lens[i])))
    ii = np.array(ii, dtype=np.int64)
    tt = np.array(tt, dtype=np.int64)
    loss = 0.0
    logp = np.zeros((R, T))
    d_hidden = np.zeros((R, T, d))
    d_w = np.zeros((V, d)) if want_dw else None
    clipped = np.zeros((R, T), dtype=bool)
    rho = np.zeros((R, T))
    for s in range(0, len(ii), block):
        bi, bt = ii[s:s + block], tt[s:s + block]
        hb = hidden[bi, bt]
        cb = 1.0 / (R * lens[bi].astype(np.float64))
        out = token_rows(hb, w, tokens[bi, bt], old_logp[bi, bt], adv[bi], cb, clip_eps,
                         grad_scale, gemm_dtype, None if ref_logp is None else ref_logp[bi, bt], kl_coef)
        loss -= float((cb * out["obj"]).sum())
        logp[bi, bt] = out["logp"]
        d_hidden[bi, bt] = out["d_h"]
        clipped[bi, bt] = out["inactive"]
        rho[bi, bt] = out["rho"]
        if want_dw:
            d_w += (out["dz"].astype(gemm_dtype, copy=False).T @ hb.astype(gemm_dtype, copy=False)).astype(np.float64)
    return dict(loss=loss, logp=logp, d_hidden=d_hidden, d_w=d_w, clipped=clipped, rho=rho)
