"""ctypes binding for libpods_hip.so (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpods_hip.so")
_lib = None

PODS_F32, PODS_BF16 = 0, 1
PODS_RULE_MAXVAR, PODS_RULE_MAXR, PODS_RULE_PERC, PODS_RULE_RAND = 0, 1, 2, 3
PODS_LOSS_ACCUMULATE_D_W, PODS_LOSS_SKIP_ZERO_ADVANTAGE = 1, 2
EXPORTED_SYMBOLS = ("pods_select", "pods_downsample", "pods_advantage", "pods_advantage_before",
                    "pods_gather_rows", "pods_downsample_gather", "grpo_token_loss_fwd_bwd_accumulate", "grpo_token_loss_fwd_bwd_kl",
                    "grpo_token_loss_fwd_bwd_ex",
                    "grpo_token_loss_workspace_bytes",
                    "grpo_token_loss_workspace_min_bytes", "grpo_token_loss_workspace_used_bytes",
                    "grpo_token_loss_fwd_bwd", "grpo_token_loss_fwd_bwd_static",
                    "grpo_token_loss_static_workspace_bytes", "grpo_token_loss_report", "pods_check_rewards",
                    "pods_last_error", "pods_profile_enable", "pods_profile_count", "pods_profile_get", "pods_profile_mfma_only")

_vp, _i32, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t


class PodsRecord(ctypes.Structure):
    """pods_record of include/pods.h."""
    _fields_ = [("src", ctypes.c_void_p), ("dst", ctypes.c_void_p), ("row_bytes", ctypes.c_size_t)]


class PodsLossReport(ctypes.Structure):
    """pods_loss_report of include/pods.h."""
    _fields_ = [("valid_tokens", ctypes.c_int32), ("backward_tokens", ctypes.c_int32),
                ("clipped_tokens", ctypes.c_int32), ("bad_lengths", ctypes.c_int32), ("bad_tokens", ctypes.c_int32),
                ("max_abs_g", ctypes.c_float), ("max_abs_w", ctypes.c_float), ("max_abs_hidden", ctypes.c_float),
                ("reserved", ctypes.c_int32 * 8)]


class PodsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pods status {status}: {message}")
        self.status = status


def library_path() -> str:
    return _LIB_PATH


def load():
    """Load libpods_hip.so (built by paper_2504_13818_amd/build.py).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} not built: run `python -m paper_2504_13818_amd.build` "
                                "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.pods_last_error.restype = ctypes.c_char_p
    lib.pods_last_error.argtypes = []
    lib.pods_select.restype = ctypes.c_int
    lib.pods_select.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _vp]
    lib.pods_downsample.restype = ctypes.c_int
    lib.pods_downsample.argtypes = [_vp, _vp, _i32, _i32, _i32, ctypes.c_int, _vp, _vp, _vp]
    for name in ("pods_advantage", "pods_advantage_before"):
        f = getattr(lib, name)
        f.restype = ctypes.c_int
        f.argtypes = [_vp, _vp, _i32, _i32, _i32, _f32, _vp, _vp]
    for name in ("grpo_token_loss_workspace_bytes", "grpo_token_loss_workspace_min_bytes"):
        f = getattr(lib, name)
        f.restype = _sz
        f.argtypes = [_i32, _i32, _i32, _i32, ctypes.c_int]
    lib.grpo_token_loss_workspace_used_bytes.restype = _sz
    lib.grpo_token_loss_workspace_used_bytes.argtypes = [_i32, _i32, _i32, _i32, ctypes.c_int, _sz]
    for name in ("grpo_token_loss_fwd_bwd", "grpo_token_loss_fwd_bwd_accumulate"):
        f = getattr(lib, name)
        f.restype = ctypes.c_int
        f.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32,
                      ctypes.c_int, _f32, _f32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.grpo_token_loss_fwd_bwd_static.restype = ctypes.c_int
    lib.grpo_token_loss_fwd_bwd_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32,
                                                   ctypes.c_int, _f32, _f32, _vp, _vp, _vp, _vp, _vp]
    lib.grpo_token_loss_static_workspace_bytes.restype = _sz
    lib.grpo_token_loss_static_workspace_bytes.argtypes = []
    lib.grpo_token_loss_report.restype = ctypes.c_int
    lib.grpo_token_loss_report.argtypes = [_vp, ctypes.POINTER(PodsLossReport), _vp]
    lib.pods_check_rewards.restype = ctypes.c_int
    lib.pods_check_rewards.argtypes = [_vp, _i32, _i32, _vp, _vp]
    lib.grpo_token_loss_fwd_bwd_kl.restype = ctypes.c_int
    lib.grpo_token_loss_fwd_bwd_kl.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32,
                                               ctypes.c_int, _f32, _f32, _f32, _i32, _vp, _vp, _vp, _vp, _vp, _sz,
                                               _vp]
    lib.grpo_token_loss_fwd_bwd_ex.restype = ctypes.c_int
    lib.grpo_token_loss_fwd_bwd_ex.argtypes = list(lib.grpo_token_loss_fwd_bwd_kl.argtypes)
    lib.pods_gather_rows.restype = ctypes.c_int
    lib.pods_gather_rows.argtypes = [_vp, _vp, _i32, _i32, _i32, _sz, _vp, _vp]
    lib.pods_downsample_gather.restype = ctypes.c_int
    lib.pods_downsample_gather.argtypes = [_vp, _vp, _i32, _i32, _i32, ctypes.c_int, _f32, _i32,
                                           ctypes.POINTER(PodsRecord), _i32, _vp, _vp, _vp, _vp]
    lib.pods_profile_enable.restype = ctypes.c_int
    lib.pods_profile_enable.argtypes = [_i32]
    lib.pods_profile_count.restype = _i32
    lib.pods_profile_count.argtypes = []
    lib.pods_profile_get.restype = ctypes.c_int
    lib.pods_profile_get.argtypes = [_i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(_f32)]
    lib.pods_profile_mfma_only.restype = ctypes.c_int
    lib.pods_profile_mfma_only.argtypes = [_i32, _i32, _vp, ctypes.POINTER(ctypes.c_double), _vp]
    _lib = lib
    return lib


def pods_profile_enable(enable: bool = True):
    """Bracket every later kernel launch of this thread's library calls with HIP events."""
    _check(load().pods_profile_enable(1 if enable else 0))


def pods_profile_read():
    """[(kernel name, milliseconds)] for every launch recorded since pods_profile_enable(True).
    Waits for the recorded launches to finish."""
    lib = load()
    out = []
    name, ms = ctypes.c_char_p(), _f32()
    for i in range(lib.pods_profile_count()):
        _check(lib.pods_profile_get(i, ctypes.byref(name), ctypes.byref(ms)))
        out.append((name.value.decode(), float(ms.value)))
    return out


def pods_last_error() -> str:
    return load().pods_last_error().decode()


def _check(status: int):
    if status != 0:
        raise PodsError(status, pods_last_error())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _need(t, dtype, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of dtype {dtype}")


def pods_select(rewards, m: int, sel_idx=None, sel_k=None, stream=None):
    """rewards[B, n] float32 (device) -> (sel_idx[B, m] int32, sel_k[B] int32)."""
    import torch
    _need(rewards, torch.float32, "rewards")
    B, n = rewards.shape
    if sel_idx is None:
        sel_idx = torch.empty((B, max(m, 0)), dtype=torch.int32, device=rewards.device)
    if sel_k is None:
        sel_k = torch.empty((B,), dtype=torch.int32, device=rewards.device)
    _check(load().pods_select(_ptr(rewards), B, n, m, _ptr(sel_idx), _ptr(sel_k), _stream(stream)))
    return sel_idx, sel_k


def pods_downsample(rewards, m: int, rule: int, rand_keys=None, sel_idx=None, sel_k=None, stream=None):
    """rewards[B, n] float32 (device; may be None for the random rule) and, for the random rule,
    rand_keys[B, n] uint32 or int32 (read as unsigned) -> (sel_idx[B, m] int32, sel_k[B] int32)."""
    import torch
    if rewards is not None:
        _need(rewards, torch.float32, "rewards")
    if rand_keys is not None and not (isinstance(rand_keys, torch.Tensor) and rand_keys.is_cuda and
                                      rand_keys.is_contiguous() and
                                      rand_keys.dtype in (torch.int32, torch.uint32)):
        raise TypeError("rand_keys: expected a contiguous CUDA tensor of dtype int32 or uint32")
    shaped = rewards if rewards is not None else rand_keys
    if shaped is None:
        raise TypeError("pods_downsample: rewards or rand_keys is required")
    B, n = shaped.shape
    if sel_idx is None:
        sel_idx = torch.empty((B, max(m, 0)), dtype=torch.int32, device=shaped.device)
    if sel_k is None:
        sel_k = torch.empty((B,), dtype=torch.int32, device=shaped.device)
    _check(load().pods_downsample(_ptr(rewards), _ptr(rand_keys), B, n, m, int(rule), _ptr(sel_idx),
                                  _ptr(sel_k), _stream(stream)))
    return sel_idx, sel_k


def pods_advantage_before(rewards, sel_idx, std_eps: float = 0.0, adv=None, stream=None):
    """As pods_advantage, with the mean and standard deviation of all n rewards of each group."""
    return pods_advantage(rewards, sel_idx, std_eps, adv, stream, _entry="pods_advantage_before")


def pods_advantage(rewards, sel_idx, std_eps: float = 0.0, adv=None, stream=None, _entry="pods_advantage"):
    """rewards[B, n] float32, sel_idx[B, m] int32 (device) -> adv[B, m] float32."""
    import torch
    _need(rewards, torch.float32, "rewards")
    _need(sel_idx, torch.int32, "sel_idx")
    B, n = rewards.shape
    m = sel_idx.shape[1]
    if adv is None:
        adv = torch.empty((B, m), dtype=torch.float32, device=rewards.device)
    _check(getattr(load(), _entry)(_ptr(rewards), _ptr(sel_idx), B, n, m, float(std_eps), _ptr(adv),
                                   _stream(stream)))
    return adv


def _dt(t):
    import torch
    if t.dtype == torch.float32:
        return PODS_F32
    if t.dtype == torch.bfloat16:
        return PODS_BF16
    raise TypeError(f"hidden / w_lm must be float32 or bfloat16, got {t.dtype}")


def grpo_token_loss_workspace_bytes(R, T, d, V, dt) -> int:
    return int(load().grpo_token_loss_workspace_bytes(R, T, d, V, dt))


def grpo_token_loss_workspace_min_bytes(R, T, d, V, dt) -> int:
    return int(load().grpo_token_loss_workspace_min_bytes(R, T, d, V, dt))


def grpo_token_loss_workspace_used_bytes(R, T, d, V, dt, workspace_bytes) -> int:
    return int(load().grpo_token_loss_workspace_used_bytes(R, T, d, V, dt, workspace_bytes))


def pods_gather_rows(per_rollout, sel_idx, out=None, stream=None):
    """per_rollout[B, n, ...] (any dtype, device) and sel_idx[B, m] int32 -> out[B*m, ...]: the kept
    rollouts' records, concatenated over the prompts."""
    import torch
    _need(sel_idx, torch.int32, "sel_idx")
    if not (isinstance(per_rollout, torch.Tensor) and per_rollout.is_cuda and per_rollout.is_contiguous()
            and per_rollout.dim() >= 2):
        raise TypeError("per_rollout: expected a contiguous CUDA tensor [B, n, ...]")
    B, n = per_rollout.shape[:2]
    m = sel_idx.shape[1]
    row_bytes = per_rollout[0, 0].numel() * per_rollout.element_size() if per_rollout.dim() > 2 \
        else per_rollout.element_size()
    if out is None:
        out = torch.empty((B * m,) + tuple(per_rollout.shape[2:]), dtype=per_rollout.dtype,
                          device=per_rollout.device)
    _check(load().pods_gather_rows(_ptr(per_rollout), _ptr(sel_idx), B, n, m, row_bytes, _ptr(out),
                                   _stream(stream)))
    return out


def pods_downsample_gather(rewards, m: int, records=(), rule: int = PODS_RULE_MAXVAR, rand_keys=None,
                           std_eps: float = 0.0, stats_from_all: bool = False, outs=None, stream=None):
    """One launch for down-sampling, advantages and the kept rollouts' records.  rewards[B, n] float32;
    records: contiguous CUDA tensors [B, n, ...] of any dtype; outs: optional preallocated [B*m, ...]
    tensors, one per record.  Returns (sel_idx[B, m], sel_k[B], adv[B, m], [gathered records])."""
    import torch
    _need(rewards, torch.float32, "rewards")
    if rand_keys is not None and not (isinstance(rand_keys, torch.Tensor) and rand_keys.is_cuda and
                                      rand_keys.is_contiguous() and
                                      rand_keys.dtype in (torch.int32, torch.uint32)):
        raise TypeError("rand_keys: expected a contiguous CUDA tensor of dtype int32 or uint32")
    B, n = rewards.shape
    records = list(records)
    if outs is None:
        outs = [torch.empty((B * max(m, 0),) + tuple(t.shape[2:]), dtype=t.dtype, device=t.device)
                for t in records]
    if len(outs) != len(records):
        raise ValueError("outs: one tensor per record")
    descr = (PodsRecord * max(len(records), 1))()
    for q, (t, o) in enumerate(zip(records, outs)):
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dim() >= 2
                and tuple(t.shape[:2]) == (B, n)):
            raise TypeError(f"records[{q}]: expected a contiguous CUDA tensor [B, n, ...]")
        row_bytes = (t[0, 0].numel() if t.dim() > 2 else 1) * t.element_size()
        if not (isinstance(o, torch.Tensor) and o.is_cuda and o.is_contiguous() and o.dtype == t.dtype
                and o.numel() * o.element_size() == B * m * row_bytes):
            raise TypeError(f"outs[{q}]: expected a contiguous CUDA tensor [B*m, ...] of records[{q}]'s dtype")
        descr[q] = PodsRecord(t.data_ptr(), o.data_ptr(), row_bytes)
    sel_idx = torch.empty((B, max(m, 0)), dtype=torch.int32, device=rewards.device)
    sel_k = torch.empty((B,), dtype=torch.int32, device=rewards.device)
    adv = torch.empty((B, max(m, 0)), dtype=torch.float32, device=rewards.device)
    _check(load().pods_downsample_gather(_ptr(rewards), _ptr(rand_keys), B, n, m, int(rule), float(std_eps),
                                         1 if stats_from_all else 0, descr, len(records), _ptr(sel_idx),
                                         _ptr(sel_k), _ptr(adv), _stream(stream)))
    return sel_idx, sel_k, adv, outs


def grpo_token_loss_fwd_bwd(hidden, w_lm, tokens, old_logp, adv, lengths, clip_eps: float,
                            grad_scale: float = 1.0, workspace=None, want_logp: bool = True,
                            out=None, stream=None, accumulate_d_w: bool = False, ref_logp=None,
                            kl_coef: float = 0.0, skip_zero_advantage: bool = False):
    """Returns dict(loss[1], logp[R, T] or None, d_hidden[R, T, d], d_w_lm[V, d]), float32 on device.

    `workspace` is a uint8 CUDA tensor (allocated at the recommended size when None); `out` may
    carry preallocated loss / logp / d_hidden / d_w_lm tensors.  With accumulate_d_w the gradient is
    added to out["d_w_lm"] (grpo_token_loss_fwd_bwd_accumulate).  With ref_logp[R, T] float32 the KL
    penalty kl_coef * KL is subtracted from every token's term (grpo_token_loss_fwd_bwd_kl).  With
    skip_zero_advantage the backward pass leaves out rollouts whose advantage is zero
    (grpo_token_loss_fwd_bwd_ex).
    """
    import torch
    dt = _dt(hidden)
    _need(hidden, hidden.dtype, "hidden")
    _need(w_lm, hidden.dtype, "w_lm")
    _need(tokens, torch.int32, "tokens")
    _need(old_logp, torch.float32, "old_logp")
    _need(adv, torch.float32, "adv")
    if lengths is not None:
        _need(lengths, torch.int32, "lengths")
    R, T, d = hidden.shape
    V = w_lm.shape[0]
    dev = hidden.device
    if accumulate_d_w and "d_w_lm" not in (out or {}):
        raise ValueError("accumulate_d_w needs out['d_w_lm'] to accumulate into")
    out = dict(out or {})
    if "loss" not in out:
        out["loss"] = torch.empty((1,), dtype=torch.float32, device=dev)
    if "logp" not in out:
        out["logp"] = torch.empty((R, T), dtype=torch.float32, device=dev) if want_logp else None
    if "d_hidden" not in out:
        out["d_hidden"] = torch.empty((R, T, d), dtype=torch.float32, device=dev)
    if "d_w_lm" not in out:
        out["d_w_lm"] = torch.empty((V, d), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty((grpo_token_loss_workspace_bytes(R, T, d, V, dt),), dtype=torch.uint8,
                                device=dev)
    if ref_logp is not None:
        _need(ref_logp, torch.float32, "ref_logp")
    if skip_zero_advantage:
        _check(load().grpo_token_loss_fwd_bwd_ex(
            _ptr(hidden), _ptr(w_lm), _ptr(tokens), _ptr(old_logp), _ptr(ref_logp), _ptr(adv), _ptr(lengths), R, T,
            d, V, dt, float(clip_eps), float(kl_coef), float(grad_scale),
            PODS_LOSS_SKIP_ZERO_ADVANTAGE | (PODS_LOSS_ACCUMULATE_D_W if accumulate_d_w else 0),
            _ptr(out["loss"]), _ptr(out["logp"]), _ptr(out["d_hidden"]), _ptr(out["d_w_lm"]), _ptr(workspace),
            workspace.numel(), _stream(stream)))
        out["workspace"] = workspace
        return out
    if ref_logp is not None:
        _check(load().grpo_token_loss_fwd_bwd_kl(
            _ptr(hidden), _ptr(w_lm), _ptr(tokens), _ptr(old_logp), _ptr(ref_logp), _ptr(adv), _ptr(lengths), R, T,
            d, V, dt, float(clip_eps), float(kl_coef), float(grad_scale), 1 if accumulate_d_w else 0,
            _ptr(out["loss"]), _ptr(out["logp"]), _ptr(out["d_hidden"]), _ptr(out["d_w_lm"]), _ptr(workspace),
            workspace.numel(), _stream(stream)))
        out["workspace"] = workspace
        return out
    entry = load().grpo_token_loss_fwd_bwd_accumulate if accumulate_d_w else load().grpo_token_loss_fwd_bwd
    _check(entry(
        _ptr(hidden), _ptr(w_lm), _ptr(tokens), _ptr(old_logp), _ptr(adv), _ptr(lengths), R, T, d, V,
        dt, float(clip_eps), float(grad_scale), _ptr(out["loss"]), _ptr(out["logp"]),
        _ptr(out["d_hidden"]), _ptr(out["d_w_lm"]), _ptr(workspace), workspace.numel(),
        _stream(stream)))
    out["workspace"] = workspace
    return out


def grpo_token_loss_static_workspace_bytes() -> int:
    return int(load().grpo_token_loss_static_workspace_bytes())


def grpo_token_loss_fwd_bwd_static(hidden, w_lm, tokens, old_logp, adv, lengths, clip_eps: float,
                                   grad_scale: float = 1.0, out=None, stream=None):
    """grpo_token_loss_fwd_bwd on the library's built-in workspace: the call itself allocates nothing, so
    `out` must carry all four preallocated outputs (loss[1], logp[R, T] or None, d_hidden[R, T, d],
    d_w_lm[V, d], float32 on the device)."""
    import torch
    dt = _dt(hidden)
    _need(hidden, hidden.dtype, "hidden")
    _need(w_lm, hidden.dtype, "w_lm")
    _need(tokens, torch.int32, "tokens")
    _need(old_logp, torch.float32, "old_logp")
    _need(adv, torch.float32, "adv")
    if lengths is not None:
        _need(lengths, torch.int32, "lengths")
    if out is None or any(k not in out for k in ("loss", "logp", "d_hidden", "d_w_lm")):
        raise ValueError("grpo_token_loss_fwd_bwd_static: out must hold loss, logp (or None), d_hidden and d_w_lm")
    R, T, d = hidden.shape
    V = w_lm.shape[0]
    _check(load().grpo_token_loss_fwd_bwd_static(
        _ptr(hidden), _ptr(w_lm), _ptr(tokens), _ptr(old_logp), _ptr(adv), _ptr(lengths), R, T, d, V, dt,
        float(clip_eps), float(grad_scale), _ptr(out["loss"]), _ptr(out["logp"]), _ptr(out["d_hidden"]),
        _ptr(out["d_w_lm"]), _stream(stream)))
    return out


def grpo_token_loss_report(workspace=None, stream=None) -> dict:
    """The report of the last token-loss call on `workspace` (a uint8 CUDA tensor; None = the built-in
    workspace of grpo_token_loss_fwd_bwd_static) as a dict.  Waits for the stream."""
    rep = PodsLossReport()
    _check(load().grpo_token_loss_report(_ptr(workspace), ctypes.byref(rep), _stream(stream)))
    return {name: getattr(rep, name) for name, _ in PodsLossReport._fields_ if name != "reserved"}


def pods_check_rewards(rewards, report=None, stream=None):
    """rewards[B, n] float32 (device) -> report[2] int32 (device): number of non-finite rewards and the
    flat index of the first one (-1 if none)."""
    import torch
    _need(rewards, torch.float32, "rewards")
    B, n = rewards.shape
    if report is None:
        report = torch.empty((2,), dtype=torch.int32, device=rewards.device)
    _check(load().pods_check_rewards(_ptr(rewards), B, n, _ptr(report), _stream(stream)))
    return report


def pods_profile_mfma_only(workgroups: int, iters: int, sink, stream=None) -> float:
    """Launch the matrix-core-only loop of include/pods_profile.h; returns its floating-point operations."""
    flops = ctypes.c_double()
    _check(load().pods_profile_mfma_only(workgroups, iters, _ptr(sink), ctypes.byref(flops), _stream(stream)))
    return float(flops.value)
