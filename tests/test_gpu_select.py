"""GPU parity: pods_select and pods_advantage through the C ABI against the CPU oracle.

Index arrays and k must match bit-exactly.  The batched reference is the C oracle (double
precision sums); wherever the GPU disagrees with it the exact-rational oracle referees."""
import numpy as np
import pytest

from oracle import fast, pods_oracle as po
from paper_2504_13818_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _gpu_select(lib, r, m):
    rt = torch.from_numpy(r).cuda()
    idx, k = lib.pods_select(rt, m)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), k.cpu().numpy()


def _assert_select_parity(lib, r, m, exact_sample=64):
    idx, k = _gpu_select(lib, r, m)
    ridx, rk, _ = fast.select(r, m)
    bad = np.nonzero((idx != ridx).any(axis=1) | (k != rk))[0]
    for b in bad:      # the paper's rule in exact arithmetic decides any disagreement
        eidx, ek = po.select_exact(r[b], m)
        assert list(idx[b]) == eidx and k[b] == ek, f"group {b}: gpu {idx[b]}, k={k[b]} vs exact {eidx}, k={ek}"
    assert len(bad) <= max(1, r.shape[0] // 10000), f"{len(bad)} groups differ from the double-precision oracle"
    rng = np.random.default_rng(0)
    for b in rng.choice(r.shape[0], min(exact_sample, r.shape[0]), replace=False) if exact_sample else []:
        eidx, ek = po.select_exact(r[b], m)
        assert list(idx[b]) == eidx and k[b] == ek
    return idx, k


@pytest.mark.parametrize("cfg", [0, 1, 2, 4])
def test_select_configs(pods, cfg):
    r = inputs.rewards(cfg)
    _assert_select_parity(pods, r, inputs.CONFIGS[cfg]["m"])


def test_select_stress_config_full_size(pods):
    """B=65536, n=256, m=64, the launch the benchmark times; about 10 % all-equal groups."""
    r = inputs.rewards(3)
    idx, k = _assert_select_parity(pods, r, 64, exact_sample=200)
    flat = r.max(axis=1) == r.min(axis=1)
    assert flat.sum() > 5000
    assert np.all(k[flat] == 0) and np.all(idx[flat] == np.arange(64, dtype=np.int32))


@pytest.mark.parametrize("n,m,B", [(1, 1, 3), (2, 1, 5), (7, 3, 9), (16, 16, 4), (63, 17, 11), (64, 64, 3),
                                   (65, 5, 7), (100, 33, 13), (129, 128, 5), (255, 64, 6), (300, 100, 9),
                                   (512, 128, 8), (1000, 333, 5), (2048, 64, 3), (4096, 1024, 2),
                                   (4095, 4095, 2), (64, 16, 37), (128, 32, 21), (256, 64, 19)])
def test_select_ragged_shapes(pods, n, m, B):
    rng = np.random.default_rng(n * 131 + m)
    for kind in range(4):
        if kind == 0:
            r = rng.standard_normal((B, n)).astype(np.float32)
        elif kind == 1:
            r = (rng.integers(0, 2, (B, n))).astype(np.float32)
        elif kind == 2:
            r = (rng.integers(-2, 3, (B, n)) * 0.25).astype(np.float32)
            r[r == 0] *= rng.choice([-1.0, 1.0], (r == 0).sum()).astype(np.float32)   # mix -0.0 / +0.0
        else:
            r = np.full((B, n), np.float32(0.1)) + (rng.random((B, n)) < 0.02).astype(np.float32)
        _assert_select_parity(pods, r, m, exact_sample=0 if m * m > 20000 else 8)


@pytest.mark.parametrize("n,m,B", [(16, 16, 19), (17, 5, 21), (32, 32, 18), (64, 32, 40), (64, 33, 40), (128, 32, 33),
                                   (128, 33, 33), (256, 64, 70), (256, 65, 70), (256, 255, 9), (257, 128, 9),
                                   (512, 128, 11), (512, 129, 11), (1024, 256, 5), (1024, 257, 5), (2048, 512, 3),
                                   (2048, 513, 3), (4096, 512, 2), (4096, 513, 2)])
def test_select_block_boundaries(pods, n, m, B):
    """Sizes on both sides of every switch inside the kernel: lanes per group, keys per lane, the
    register-resident candidate scan (at most 8 splits per lane) against the one through LDS, group
    counts that leave part of the last wavefront and workgroup idle."""
    rng = np.random.default_rng(n * 7 + m)
    r = (rng.integers(0, 4, (B, n)) * 0.25 + (rng.random((B, n)) < 0.3) * rng.standard_normal((B, n)) * 0.01).astype(np.float32)
    _assert_select_parity(pods, r, m, exact_sample=0 if m * n > 40000 else 4)


def test_select_unaligned_rewards_pointer(pods):
    """A rewards pointer that is only 4-byte aligned must take the scalar load path."""
    r = inputs.rewards(3, B=512)
    flat = torch.zeros(r.size + 1, dtype=torch.float32, device="cuda")
    flat[1:] = torch.from_numpy(r).cuda().reshape(-1)
    view = flat[1:].view(r.shape)
    assert view.data_ptr() % 16 == 4 and view.is_contiguous()
    idx, k = pods.pods_select(view, 64)
    torch.cuda.synchronize()
    ridx, rk, _ = fast.select(r, 64)
    assert np.array_equal(idx.cpu().numpy(), ridx) and np.array_equal(k.cpu().numpy(), rk)


def test_select_is_deterministic(pods):
    r = inputs.rewards(3, B=4096)
    a = _gpu_select(pods, r, 64)
    b = _gpu_select(pods, r, 64)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_select_without_k_output(pods):
    r = torch.from_numpy(inputs.rewards(1)).cuda()
    idx = torch.empty((32, 16), dtype=torch.int32, device="cuda")
    l = pods.load()
    import ctypes
    st = l.pods_select(ctypes.c_void_p(r.data_ptr()), 32, 64, 16, ctypes.c_void_p(idx.data_ptr()), None, None)
    torch.cuda.synchronize()
    assert st == 0
    ref, _, _ = fast.select(inputs.rewards(1), 16)
    assert np.array_equal(idx.cpu().numpy(), ref)


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_advantage_configs(pods, cfg):
    r = inputs.rewards(cfg)
    m = inputs.CONFIGS[cfg]["m"]
    sel, _, _ = fast.select(r, m)
    a = pods.pods_advantage(torch.from_numpy(r).cuda(), torch.from_numpy(sel).cuda())
    torch.cuda.synchronize()
    a = a.cpu().numpy().astype(np.float64)
    ref = fast.advantage(r, sel)
    assert np.allclose(a, ref, rtol=1e-5, atol=1e-6)
    kept = np.take_along_axis(r, sel, axis=1)
    flat = kept.max(axis=1) == kept.min(axis=1)
    assert np.all(a[flat] == 0.0)
    assert np.allclose(a.sum(axis=1), 0.0, atol=1e-4)


def test_advantage_std_eps_and_large_m(pods):
    rng = np.random.default_rng(3)
    r = rng.standard_normal((5, 3000)).astype(np.float32)
    sel, _, _ = fast.select(r, 1500)
    a = pods.pods_advantage(torch.from_numpy(r).cuda(), torch.from_numpy(sel).cuda(), std_eps=1e-3)
    torch.cuda.synchronize()
    assert np.allclose(a.cpu().numpy(), fast.advantage(r, sel, 1e-3), rtol=1e-5, atol=1e-6)
