"""Benchmark of the PODS hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: pods_select -> pods_advantage ->
grpo_token_loss_fwd_bwd, with every input already resident in HBM.  The default workload is the
Qwen2.5-3B-shaped head (B=32 prompt groups, n=64 -> m=16, T=1024 ragged, d=2048, V=151936, bf16).
Prints ONE JSON line: whole-step valid-token throughput (the timed steps carry nothing but the path's own
launches), the roofline of the dominant kernel (the same steps repeated with a HIP event pair around each
launch), the selector's bandwidth figures on the
selector-stress workload, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 / fp16 MFMA peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_counters.txt")
# Kernel names as rocprofv3 prints them, demangled or mangled, matched exactly (template arguments
# included: the selector-stress launch is select_quarter_kernel<64>, not the other group sizes' variants).
KERNEL_SYMBOLS = {"token loss forward": (r"::fwd_kernel\(", r"\d+fwd_kernelE"),
                  "token loss normalise": (r"::rescale_kernel\(", r"\d+rescale_kernelE"),
                  "token loss d_hidden": (r"::dh_kernel\(", r"\d+dh_kernelE"),
                  "token loss d_w_lm": (r"::dw_kernel\(", r"\d+dw_kernelE"),
                  "pods_select": (r"::select_quarter_kernel<64>\(", r"\d+select_quarter_kernelILi64EE")}
PROBE_BYTES = 1 << 30         # the calibration copy reads and writes this many bytes


LOSS_SOURCES = ("common.h", "loss.h", "loss.hip", "loss_mfma.hip")
SELECT_SOURCES = ("common.h", "select.hip")


def sources_of(kernel):
    return SELECT_SOURCES if kernel == "pods_select" else LOSS_SOURCES


def source_digest(names=LOSS_SOURCES):
    """sha256 over a kernel family's HIP sources (comments and whitespace aside): HBM-traffic counters
    are only quoted for the kernels they were taken on."""
    import hashlib
    import re
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2504_13818_amd", "csrc")
    for name in names:
        text = open(os.path.join(csrc, name), encoding="utf-8").read()
        text = re.sub(r"//[^\n]*", "", text)                      # comments and layout do not change a kernel
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()


def summarize_traffic(fetch_csv, write_csv, out_path=TRAFFIC_FILE):
    """Turn two `rocprofv3 --pmc` runs of `bench.py --traffic-probe` (FETCH_SIZE, then WRITE_SIZE; KiB per
    dispatch) into bytes per launch for each kernel, each counter scaled by what it reads for a plain
    copy kernel of known size."""
    import csv
    import collections
    import re

    def load(path, counter):
        per = collections.defaultdict(list)
        probe = []
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            name, val = r["Kernel_Name"], float(r["Counter_Value"])
            dur = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
            for label, patterns in KERNEL_SYMBOLS.items():
                if any(re.search(pat, name) for pat in patterns):
                    per[label].append(val)
            if "MulFunctor" in name and "vectorized_elementwise_kernel" in name:
                probe.append((dur, val))
        probe_kib = max(probe)[1]            # the 1 GiB probe is by far the longest such kernel
        factor = (PROBE_BYTES / 1024.0) / probe_kib
        return {k: 1024.0 * factor * sum(v) / len(v) for k, v in per.items()}, factor, probe_kib

    fetch, f_fac, f_probe = load(fetch_csv, "FETCH_SIZE")
    write, w_fac, w_probe = load(write_csv, "WRITE_SIZE")
    out = {"source_sha256": {"loss": source_digest(LOSS_SOURCES), "select": source_digest(SELECT_SOURCES)},
           "calibration": {"probe": "torch.mul(x, 1.0, out=y) on 2^28 fp32 elements: reads 1 GiB, writes 1 GiB",
                           "fetch_factor": f_fac, "fetch_probe_kib": f_probe,
                           "write_factor": w_fac, "write_probe_kib": w_probe},
           "kernels": {k: {"fetch_bytes_per_launch": fetch.get(k), "write_bytes_per_launch": write.get(k)}
                       for k in sorted(set(fetch) | set(write))}}
    with open(out_path, "w") as f:
        json.dump(out, f, indent=1)
    return out


def recorded_traffic(kernel):
    """HBM bytes per launch (fetch + write) from profiles/hbm_traffic_counters.txt, or None when absent or stale."""
    try:
        t = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None
    family = "select" if kernel == "pods_select" else "loss"
    digests = t.get("source_sha256")
    if not isinstance(digests, dict) or digests.get(family) != source_digest(sources_of(kernel)):
        return None
    k = t.get("kernels", {}).get(kernel)
    if not k or k.get("fetch_bytes_per_launch") is None or k.get("write_bytes_per_launch") is None:
        return None
    return k["fetch_bytes_per_launch"] + k["write_bytes_per_launch"]


def current_logp_torch(torch, hidden, w, tokens, chunk=4096):
    """log-softmax(hidden . w^T)[token] with plain torch ops, in token chunks (input synthesis only:
    old_logp is an input of the path, defined as the current log-prob plus noise)."""
    R, T, d = hidden.shape
    h2 = hidden.reshape(R * T, d)
    tok = tokens.reshape(R * T).long()
    out = torch.empty(R * T, dtype=torch.float32, device=hidden.device)
    for s in range(0, R * T, chunk):
        z = (h2[s:s + chunk] @ w.T).float()
        out[s:s + chunk] = z.gather(1, tok[s:s + chunk, None])[:, 0] - torch.logsumexp(z, dim=1)
    return out.reshape(R, T)


def sample_tokens_torch(torch, hidden, w, generator, chunk=4096):
    """Tokens drawn from softmax(hidden . w^T) (Gumbel-max) and their log-probs, with plain torch ops in token
    chunks (input synthesis only, for the context measurement on policy-sampled tokens)."""
    R, T, d = hidden.shape
    h2 = hidden.reshape(R * T, d)
    tok = torch.empty(R * T, dtype=torch.int64, device=hidden.device)
    logp = torch.empty(R * T, dtype=torch.float32, device=hidden.device)
    for s in range(0, R * T, chunk):
        z = (h2[s:s + chunk] @ w.T).float()
        u = torch.rand(z.shape, generator=generator, device=z.device).clamp_(1e-20, 1.0)
        t = (z - torch.log(-torch.log(u))).argmax(dim=1)
        tok[s:s + chunk] = t
        logp[s:s + chunk] = z.gather(1, t[:, None])[:, 0] - torch.logsumexp(z, dim=1)
        del z, u
    return tok.reshape(R, T).to(torch.int32), logp.reshape(R, T)


def time_selector(lib, torch, inputs, steps, large_launch=True):
    """pods_select on the selector-stress workload (B=65536, n=256, m=64), rotating over enough
    buffer sets that no input or output is served from the 256 MiB Infinity Cache."""
    import numpy as np
    c = inputs.CONFIGS[3]
    B, n, m = c["B"], c["n"], c["m"]
    r = torch.from_numpy(inputs.rewards(3)).cuda()
    sets = 6                                    # 6 x (64 + 16) MiB
    rs = [r.clone() for _ in range(sets)]
    idx = [torch.empty((B, m), dtype=torch.int32, device="cuda") for _ in range(sets)]
    ks = [torch.empty((B,), dtype=torch.int32, device="cuda") for _ in range(sets)]
    for i in range(sets):
        lib.pods_select(rs[i], m, idx[i], ks[i])
    torch.cuda.synchronize()
    lib.pods_profile_enable(True)
    reps = max(steps, 3) * sets
    for i in range(reps):
        lib.pods_select(rs[i % sets], m, idx[i % sets], ks[i % sets])
    prof = lib.pods_profile_read()
    lib.pods_profile_enable(False)
    ms = float(np.mean([t for _, t in prof]))
    bytes_per_group = 4 * n + 4 * m + 4
    gbs = bytes_per_group * B / (ms * 1e-3) / 1e9
    res = dict(workload="selector-stress B=65536 n=256 m=64 fp32", ms_per_launch=ms,
               groups_per_s=B / (ms * 1e-3), launches=len(prof),
               roofline=dict(bound="hbm", achieved=gbs, peak=PEAK_HBM_GBS, unit="GB/s",
                             frac=gbs / PEAK_HBM_GBS, traffic=recorded_traffic("pods_select"),
                             bytes_per_launch=bytes_per_group * B, bytes_per_group=bytes_per_group))
    if not large_launch:
        return res
    # Context (not the workload of the metric): the same kernel on eight times the groups, where the fixed cost of a
    # launch (start, first loads, end) weighs an eighth as much as on the workload's 84 MB.
    del rs, idx, ks
    big = 8
    rb = [torch.cat([r.roll(j + 3 * i, dims=0) for j in range(big)]) for i in range(2)]   # 2 x 512 MiB
    ib = [torch.empty((big * B, m), dtype=torch.int32, device="cuda") for _ in range(2)]
    kb = [torch.empty((big * B,), dtype=torch.int32, device="cuda") for _ in range(2)]
    for i in range(2):
        lib.pods_select(rb[i], m, ib[i], kb[i])
    torch.cuda.synchronize()
    lib.pods_profile_enable(True)
    for i in range(10):
        lib.pods_select(rb[i % 2], m, ib[i % 2], kb[i % 2])
    big_ms = float(np.mean([t for _, t in lib.pods_profile_read()]))
    lib.pods_profile_enable(False)
    big_gbs = bytes_per_group * big * B / (big_ms * 1e-3) / 1e9
    res["large_launch"] = dict(what="context: the same kernel on 524288 groups (8 x the workload) per launch",
                               ms_per_launch=big_ms, groups_per_s=big * B / (big_ms * 1e-3), achieved=big_gbs,
                               unit="GB/s", frac=big_gbs / PEAK_HBM_GBS)
    return res


def time_gather(lib, torch, steps):
    """pods_gather_rows on 4096 prompt groups of 64 rollouts, 16 kept, 4 KiB records (token ids at
    T = 1024): 1 GiB of source records, 256 MiB read and 256 MiB written per launch."""
    import numpy as np
    B, n, m, row = 4096, 64, 16, 1024
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    src = torch.randint(0, 150000, (B, n, row), generator=g, device="cuda", dtype=torch.int32)
    sel = torch.stack([torch.randperm(n, generator=g, device="cuda")[:m] for _ in range(64)]).to(torch.int32)
    sel = sel.repeat(B // 64, 1).contiguous()
    dst = torch.empty((B * m, row), dtype=torch.int32, device="cuda")
    lib.pods_gather_rows(src, sel, dst)
    torch.cuda.synchronize()
    lib.pods_profile_enable(True)
    for _ in range(max(steps, 5)):
        lib.pods_gather_rows(src, sel, dst)
    prof = lib.pods_profile_read()
    lib.pods_profile_enable(False)
    ms = float(np.mean([t for _, t in prof]))
    nbytes = 2 * B * m * row * 4 + B * m * 4
    gbs = nbytes / (ms * 1e-3) / 1e9
    return dict(workload="B=4096 n=64 m=16, 4 KiB records", ms_per_launch=ms, launches=len(prof),
                roofline=dict(bound="hbm", achieved=gbs, peak=PEAK_HBM_GBS, unit="GB/s", frac=gbs / PEAK_HBM_GBS,
                              traffic=None, bytes_per_launch=nbytes))


def cpu_selector(inputs):
    from oracle import fast
    r = inputs.rewards(3)
    fast.select(r[:1024], 64)
    t = time.perf_counter()
    _, _, used = fast.select(r, 64)
    dt = time.perf_counter() - t
    return dict(value=r.shape[0] / dt, unit="groups/s", cores=int(used), kind="oracle",
                sample="all 65536 groups of the selector-stress workload, C oracle, OpenMP")


def cpu_loss(inputs, cfg, tokens_sample=4096):
    """The numpy oracle (fp32 GEMM, fp64 reductions) forward + backward on a bounded sample."""
    import numpy as np
    from oracle import pods_oracle as po
    c = inputs.CONFIGS[cfg]
    R, T = 2, tokens_sample // 2
    h, w = inputs.dense(cfg, R, T, c["d"], c["V"])
    tok = inputs.tokens(cfg, R, T, c["V"])
    adv = np.array([1.0, -1.0], np.float32)
    old = np.full((R, T), -12.0, np.float32)
    t = time.perf_counter()
    po.grpo_token_loss(h, w, tok, old, adv, None, c["clip_eps"], gemm_dtype=np.float32)
    dt = time.perf_counter() - t
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    return dict(value=R * T / dt, unit="tokens/s", cores=int(cores), kind="oracle",
                sample=f"{R * T} valid tokens ({R} rollouts x {T}) at full d={c['d']}, V={c['V']}; "
                       f"fp32 GEMM, fp64 reductions; forward + backward, {dt:.1f} s; cost is linear in tokens")


def make_inputs(torch, inputs, cfg, dev):
    """Synthetic inputs of one config, resident on the device."""
    c = inputs.CONFIGS[cfg]
    B, n, m, T, d, V = c["B"], c["n"], c["m"], c["T"], c["d"], c["V"]
    R = B * m
    rewards = torch.from_numpy(inputs.rewards(cfg)).to(dev)
    lens_np = inputs.lengths(cfg)
    lengths = torch.from_numpy(lens_np).to(dev)
    tokens = torch.from_numpy(inputs.tokens(cfg, R, T, V)).to(dev)
    hidden, w = inputs.dense_torch(cfg, dev)
    cur = current_logp_torch(torch, hidden, w, tokens)
    g = torch.Generator(device=dev)
    g.manual_seed(inputs.seed_for(cfg, 5))
    old_logp = (cur + 0.05 * torch.randn(cur.shape, generator=g, device=dev)).contiguous()
    del cur
    return dict(c=c, B=B, n=n, m=m, T=T, d=d, V=V, R=R, rewards=rewards, lens_np=lens_np, lengths=lengths,
                tokens=tokens, hidden=hidden, w=w, old_logp=old_logp, n_valid=int(lens_np.sum()))


GEMM_NAMES = ["token loss forward", "token loss d_hidden", "token loss d_w_lm"]


def run_config(lib, torch, inputs, cfg, steps, warmup, dev, traffic_probe=False, with_skip=False,
               with_constant_operands=False):
    """Times `steps` whole steps (pods_select + pods_advantage + grpo_token_loss_fwd_bwd) of one config, with
    HIP events around every kernel launch."""
    import numpy as np
    x = make_inputs(torch, inputs, cfg, dev)
    c, B, m, T, d, V, R, n_valid = x["c"], x["B"], x["m"], x["T"], x["d"], x["V"], x["R"], x["n_valid"]
    dt = lib.PODS_BF16 if c["dtype"] == "bf16" else lib.PODS_F32
    ws = torch.empty((lib.grpo_token_loss_workspace_bytes(R, T, d, V, dt),), dtype=torch.uint8, device=dev)
    out = dict(loss=torch.empty(1, dtype=torch.float32, device=dev),
               logp=torch.empty((R, T), dtype=torch.float32, device=dev),
               d_hidden=torch.empty((R, T, d), dtype=torch.float32, device=dev),
               d_w_lm=torch.empty((V, d), dtype=torch.float32, device=dev))
    sel_idx = torch.empty((B, m), dtype=torch.int32, device=dev)
    sel_k = torch.empty((B,), dtype=torch.int32, device=dev)
    adv = torch.empty((B, m), dtype=torch.float32, device=dev)

    def step(skip=False):
        lib.pods_select(x["rewards"], m, sel_idx, sel_k)
        lib.pods_advantage(x["rewards"], sel_idx, 0.0, adv)
        lib.grpo_token_loss_fwd_bwd(x["hidden"], x["w"], x["tokens"], x["old_logp"], adv.view(-1), x["lengths"],
                                    c["clip_eps"], 1.0, workspace=ws, out=out, skip_zero_advantage=skip)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if traffic_probe:
        px = torch.ones(PROBE_BYTES // 4, dtype=torch.float32, device=dev)
        py = torch.empty_like(px)
        torch.mul(px, 1.0, out=py)
        torch.cuda.synchronize()
        del px, py
    # The timed region: `steps` steps between two synchronisations, nothing but the path's own launches on the
    # stream (one event per step boundary for the median and the minimum).
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]   # same stream as the launches
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    # The same steps once more with a HIP event pair around every launch, on the launch stream: the per-kernel
    # durations.  The 1460 event records of a step cost about 1 % of it, which is why the throughput above is
    # taken without them; the kernels themselves take the same time in both passes.
    lib.pods_profile_enable(True)
    t0 = time.perf_counter()
    for i in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_events = (time.perf_counter() - t0) * 1e3 / steps
    prof = lib.pods_profile_read()
    lib.pods_profile_enable(False)
    loss_val = float(out["loss"].cpu()[0])
    assert np.isfinite(loss_val)
    report = lib.grpo_token_loss_report(ws)
    assert report["valid_tokens"] == n_valid and report["bad_tokens"] == 0 and report["bad_lengths"] == 0

    per = {}
    for name, ms in prof:
        e = per.setdefault(name, [0, 0.0])
        e[0] += 1
        e[1] += ms
    kernels = {k: dict(launches_per_step=v[0] / steps, ms_per_step=v[1] / steps, avg_ms=v[1] / v[0])
               for k, v in per.items()}
    flops_family = 2.0 * n_valid * d * V        # each of the three contractions, per step
    for k in GEMM_NAMES:
        if k in kernels:
            kernels[k]["tflops"] = flops_family / (kernels[k]["ms_per_step"] * 1e-3) / 1e12
    dominant = max((k for k in GEMM_NAMES if k in kernels), key=lambda k: kernels[k]["ms_per_step"])
    dk = kernels[dominant]
    flops_per_launch = flops_family / dk["launches_per_step"]
    achieved = flops_per_launch / (dk["avg_ms"] * 1e-3) / 1e12
    gpu_ms = sum(v["ms_per_step"] for v in kernels.values())
    roofline = dict(bound="mfma", kernel=dominant, achieved=achieved, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=achieved / PEAK_BF16_TFLOPS, traffic=recorded_traffic(dominant) if cfg == 1 else None,
                    flops_per_launch=flops_per_launch, avg_launch_ms=dk["avg_ms"],
                    # the path executes the method's three contractions (logits, d_hidden, d_w_lm: 6 N d V) and no
                    # recomputation, so executed and algorithmic floating-point operations coincide
                    path_executed_tflops=3 * flops_family / (gpu_ms * 1e-3) / 1e12,
                    path_executed_frac=3 * flops_family / (gpu_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                    path_model_frac=3 * flops_family / (gpu_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS)
    res = dict(workload=f"configs[{cfg}] {c['name']}: B={B} n={x['n']} m={m} R={R} T={T} "
                        f"valid_tokens={n_valid} d={d} V={V} {c['dtype']} eps={c['clip_eps']}",
               value=n_valid / (ms_per_step * 1e-3), unit="tokens/s", steps=steps, warmup=warmup,
               ms_per_step=ms_per_step, ms_per_step_median=step_ms[len(step_ms) // 2], ms_per_step_min=step_ms[0],
               ms_per_step_with_launch_events=ms_per_step_events,
               roofline=roofline, kernels=kernels, loss=loss_val,
               clip_fraction=report["clipped_tokens"] / max(n_valid, 1), n_valid=n_valid)

    if with_skip:
        # Beside the headline (which back-propagates every valid token): the same step with the rollouts
        # of prompts without reward variance (advantage exactly 0) left out of the backward pass.
        skip_steps = max(3, steps // 4)
        step(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(skip_steps):
            step(True)
        torch.cuda.synchronize()
        skip_ms = (time.perf_counter() - t0) * 1e3 / skip_steps
        live = int(x["lens_np"][(adv.view(-1) != 0).cpu().numpy()].sum())
        res["skip_zero_advantage"] = dict(
            ms_per_step=skip_ms, steps=skip_steps, valid_tokens=n_valid, tokens_back_propagated=live,
            note="not the headline: value counts every valid token and is measured without skipping")
    if with_constant_operands:
        # Context (never a result): the same shapes with a softmax as peaked as a trained policy's and tokens that
        # were sampled from it, instead of the workload's flat softmax (logit standard deviation 0.9, entropy
        # 11.5 nats) and uniformly drawn tokens.  Hidden states times 5: logit standard deviation 4.5.
        gen = torch.Generator(device=dev)
        gen.manual_seed(inputs.seed_for(cfg, 6))
        x["hidden"].mul_(5.0)
        toks, cur = sample_tokens_torch(torch, x["hidden"], x["w"], gen)
        x["tokens"].copy_(toks)
        x["old_logp"].copy_(cur + 0.05 * torch.randn(cur.shape, generator=gen, device=dev))
        valid = torch.arange(T, device=dev)[None, :] < x["lengths"][:, None]
        mean_logp = float(cur[valid].mean().cpu())
        del toks, cur
        peak_steps = max(3, steps // 4)
        step()
        torch.cuda.synchronize()
        lib.pods_profile_enable(True)
        t0 = time.perf_counter()
        for _ in range(peak_steps):
            step()
        torch.cuda.synchronize()
        peak_ms = (time.perf_counter() - t0) * 1e3 / peak_steps
        pk = {}
        for name, ms in lib.pods_profile_read():
            pk[name] = pk.get(name, 0.0) + ms / peak_steps
        lib.pods_profile_enable(False)
        res["policy_sampled_peaked"] = dict(
            what="the headline shapes with hidden states times 5 (logit standard deviation 4.5) and tokens sampled from "
                 "the policy itself (Gumbel-max), old_logp = their log-prob + N(0, 0.05)",
            mean_logp_of_sampled_tokens=mean_logp, ms_per_step=peak_ms, steps=peak_steps,
            tokens_per_s=n_valid / (peak_ms * 1e-3),
            frac_of_peak=3 * flops_family / (peak_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            kernel_ms_per_step={k: pk[k] for k in GEMM_NAMES + ["token loss normalise"] if k in pk})
        # Context for the roofline fraction (never a result): the very same launches on hidden states that are all
        # zero, so that every logit is 0, all softmax numerators are equal and one operand of every matrix
        # instruction is constant.  The instruction streams, addresses and bytes moved are those of the headline
        # step; what changes is how many operand bits toggle, i.e. the power the matrix pipe draws.
        x["hidden"].zero_()
        const_steps = max(3, steps // 4)
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(const_steps):
            step()
        torch.cuda.synchronize()
        const_ms = (time.perf_counter() - t0) * 1e3 / const_steps
        res["constant_operands"] = dict(
            what="the headline step's launches on all-zero hidden states (equal softmax numerators, one constant "
                 "operand per matrix instruction): same instructions, addresses and traffic, fewer toggling bits",
            ms_per_step=const_ms, steps=const_steps,
            tflops=3 * flops_family / (const_ms * 1e-3) / 1e12,
            frac_of_peak=3 * flops_family / (const_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS)
    return res


def context_numbers(lib, torch, dev, n_tokens, d, vc=8192):
    """Numbers measured in this process beside the token loss's own, as context for its fraction of the
    published matrix-core peak (never the target): the vendor GEMM (torch.matmul, bf16) on the shape of
    d_w_lm's contraction for 8192 vocabulary columns, and a loop of matrix instructions with no memory traffic at all."""
    import numpy as np
    ctx = {}
    n_tok = (n_tokens // 256) * 256
    a = torch.randn((n_tok, vc), device=dev, dtype=torch.float32).to(torch.bfloat16)
    b = torch.randn((n_tok, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
    c = torch.empty((vc, d), device=dev, dtype=torch.bfloat16)
    at = a.t()
    for _ in range(2):
        torch.matmul(at, b, out=c)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    ev[0].record()
    for i in range(5):
        torch.matmul(at, b, out=c)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(5)]))
    tf = 2.0 * n_tok * vc * d / (ms * 1e-3) / 1e12
    ctx["vendor_gemm"] = dict(what=f"torch.matmul bf16, [{vc} x {n_tok}] . [{n_tok} x {d}] (d_w_lm's contraction for 8192 vocabulary columns), "
                                   "random normal operands, median of 5", ms=ms, tflops=tf, frac_of_peak=tf / PEAK_BF16_TFLOPS)
    del a, b, c, at
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    lib.pods_profile_mfma_only(256, 2000, sink)
    torch.cuda.synchronize()
    lib.pods_profile_enable(True)
    flops = [lib.pods_profile_mfma_only(2048, 20000, sink) for _ in range(3)]
    prof = lib.pods_profile_read()
    lib.pods_profile_enable(False)
    ms = float(np.median([t for _, t in prof]))
    tf = flops[0] / (ms * 1e-3) / 1e12
    ctx["mfma_only"] = dict(what="v_mfma_f32_32x32x16_bf16 on register operands, 2048 workgroups x 4 wavefronts x 640000 "
                                 "instructions, no loads; median of 3 launches", ms=ms, tflops=tf,
                            frac_of_peak=tf / PEAK_BF16_TFLOPS)
    return ctx


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1, choices=[1, 2, 4])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-headline", action="store_true",
                    help="skip the other loss configs, the context numbers and the gather figure")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run a 1 GiB copy kernel, the calibration for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--summarize-traffic", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: write profiles/hbm_traffic_counters.txt from two --pmc counter_collection.csv files")
    args = ap.parse_args()
    if args.summarize_traffic:
        print(json.dumps(summarize_traffic(*args.summarize_traffic), indent=1))
        return
    if args.gpus != 1:
        print("bench.py measures the single-GPU hot path only: run it with --gpus 1 "
              "(prompt groups and kept rollouts shard across GPUs without exchange; only d_w_lm is reduced).", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2504_13818_amd as lib
    from paper_2504_13818_amd import inputs

    lib.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = args.config
    head = run_config(lib, torch, inputs, cfg, args.steps, args.warmup, dev, traffic_probe=args.traffic_probe,
                      with_skip=True, with_constant_operands=not args.only_headline)
    torch.cuda.empty_cache()
    c = inputs.CONFIGS[cfg]

    selector = time_selector(lib, torch, inputs, args.steps, large_launch=not args.only_headline)
    result = {
        "metric": "GRPO token-loss fwd+bwd tokens/s (% MFMA peak); pods_select groups/s (% HBM)",
        "value": head["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "ms_per_step_median": head["ms_per_step_median"],
        "ms_per_step_min": head["ms_per_step_min"],
        "ms_per_step_with_launch_events": head["ms_per_step_with_launch_events"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": c["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"],
                   "step": "pods_select + pods_advantage + grpo_token_loss_fwd_bwd",
                   "arithmetic": "logits: bf16 MFMA (v_mfma_f32_32x32x16_bf16); gradients: fp16 MFMA on exact fp16 copies of "
                                 "the bf16 inputs and an fp16 softmax operand; fp32 accumulation; fp64 selector scores"},
        "roofline": head["roofline"],
        # context, not a target and not comparable: the paper times whole training runs, never this path
        "paper_context": "The paper reports no kernel- or stage-level timing.  Its figures are end-to-end wall-clock "
                         "ratios to reach 0.99 x GRPO's peak test accuracy, GRPO-PODS over GRPO (Table 3): 2.0x, 3.0x, "
                         "2.0x and 1.8x on one L40S (LoRA; Qwen2.5-3B / Llama3.2-3B on GSM8K, MATH, SciKnowEval chemistry) "
                         "and 1.7x on 8 H100 and on 8 A100 (full-parameter, ZeRO-2; Qwen2.5-3B and 7B on GSM8K); "
                         "precision not stated.",
        "kernels": head["kernels"],
        "selector": selector,
        "skip_zero_advantage": head["skip_zero_advantage"],
        "loss": head["loss"],
        "clip_fraction": head["clip_fraction"],
    }
    if not args.only_headline:
        # the other two loss workloads of the metric, a few steps each (not the headline value)
        others = {}
        for other in (1, 2, 4):
            if other == cfg:
                continue
            r = run_config(lib, torch, inputs, other, max(3, args.steps // 4), 1, dev)
            torch.cuda.empty_cache()
            rf = r["roofline"]
            others[str(other)] = dict(
                workload=r["workload"], tokens_per_s=r["value"], ms_per_step=r["ms_per_step"], steps=r["steps"],
                warmup=r["warmup"], dominant_kernel=rf["kernel"], dominant_kernel_frac=rf["frac"],
                path_executed_frac=rf["path_executed_frac"], path_model_frac=rf["path_model_frac"],
                gemm_tflops={k: r["kernels"][k]["tflops"] for k in GEMM_NAMES if k in r["kernels"]},
                loss=r["loss"], clip_fraction=r["clip_fraction"])
        result["configs"] = others
        result["gather"] = time_gather(lib, torch, args.steps)
        result["context"] = context_numbers(lib, torch, dev, head["n_valid"], c["d"])
        result["context"]["constant_operands"] = head["constant_operands"]
        result["context"]["policy_sampled_peaked"] = head["policy_sampled_peaked"]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_loss(inputs, cfg)
        result["selector"]["cpu_baseline"] = cpu_selector(inputs)
        if not args.only_headline:
            for other in result["configs"]:
                result["configs"][other]["cpu_baseline"] = cpu_loss(inputs, int(other), tokens_sample=2048)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
