"""grpo_token_loss_fwd_bwd_static (the entry point that allocates nothing: its working arrays live in a
device array built into the library) against grpo_token_loss_fwd_bwd, through the C ABI: two calls in a
row, the second on a smaller input, so that whatever the first call left in the shared array is there
when the second one runs."""
import ctypes

import numpy as np
import pytest

from tests import helpers as H

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _outputs(R, T, d, V):
    return dict(loss=torch.full((1,), 7.0, dtype=torch.float32, device="cuda"),
                logp=torch.full((R, T), 7.0, dtype=torch.float32, device="cuda"),
                d_hidden=torch.full((R, T, d), 7.0, dtype=torch.float32, device="cuda"),
                d_w_lm=torch.full((V, d), 7.0, dtype=torch.float32, device="cuda"))


def _host(out):
    torch.cuda.synchronize()
    return dict(loss=float(out["loss"].cpu()[0]), logp=out["logp"].cpu().numpy().astype(np.float64),
                d_hidden=out["d_hidden"].cpu().numpy().astype(np.float64),
                d_w=out["d_w_lm"].cpu().numpy().astype(np.float64))


def test_static_workspace_entry_matches_the_workspace_entry(pods):
    size = pods.grpo_token_loss_static_workspace_bytes()
    assert size == 64 << 20
    # the second case is smaller in every dimension; the third is the fp32 path on the same array
    shapes = [(1, 6, 200, 512, 5000, "bf16"), (1, 3, 70, 256, 1300, "bf16"), (0, 4, 33, 96, 500, "f32")]
    for cfg, R, T, d, V, dtype in shapes:
        print(f"static workspace case cfg={cfg} R={R} T={T} d={d} V={V} {dtype}", flush=True)
        case = H.loss_case(cfg, R, T, d, V, sigma=0.2, gemm_dtype=np.float64 if dtype == "f32" else np.float32)
        case["dtype"] = dtype
        dt = pods.PODS_BF16 if dtype == "bf16" else pods.PODS_F32
        assert pods.grpo_token_loss_workspace_min_bytes(R, T, d, V, dt) <= size
        scale = float(R * case["lengths"].mean())
        dv = H.to_device(case, torch)
        out = pods.grpo_token_loss_fwd_bwd_static(dv["hidden"], dv["w"], dv["tokens"], dv["old_logp"], dv["adv"],
                                                  dv["lengths"], case["clip_eps"], grad_scale=scale,
                                                  out=_outputs(R, T, d, V))
        got = _host(out)
        # the existing entry point on a caller's workspace of the same size takes the same plan: same bits
        ws = torch.empty((size,), dtype=torch.uint8, device="cuda")
        same = _host(pods.grpo_token_loss_fwd_bwd(dv["hidden"], dv["w"], dv["tokens"], dv["old_logp"], dv["adv"],
                                                  dv["lengths"], case["clip_eps"], grad_scale=scale, workspace=ws,
                                                  out=_outputs(R, T, d, V)))
        assert got["loss"] == same["loss"]
        for key in ("logp", "d_hidden", "d_w"):
            assert np.array_equal(got[key], same[key]), key
        # ... and on its recommended workspace, within the parity bar (another token block size, another
        # summation order), as is the oracle
        rec = H.gpu_loss(pods, torch, case, grad_scale=scale)
        H.check_loss(got, rec)
        H.check_loss(got, H.oracle_loss(case, grad_scale=scale,
                                        gemm_dtype=np.float64 if dtype == "f32" else np.float32))


def test_static_workspace_entry_rejects_sizes_beyond_its_array(pods):
    one = ctypes.c_void_p(256)   # never dereferenced: the sizes are rejected first
    l = pods.load()
    st = l.grpo_token_loss_fwd_bwd_static(one, one, one, one, one, None, 512, 1024, 2048, 151936, pods.PODS_BF16,
                                          0.2, 1.0, one, None, one, one, None)
    assert st == 2 and "built-in" in pods.pods_last_error()
