"""The synthetic-input generator: shapes, determinism, subset regeneration, distributions."""
import numpy as np
import torch

import workloads as wl
from workloads.gen import _mix_py, random_bits, stream_key


def test_parameter_set_shapes():
    r = wl.resnet50_param_set()
    assert r.n_tensors == 161 and r.P == 25_557_032
    assert sum(1 for n in r.numel if n <= 2048) == 107 and max(r.numel) == 2_359_296
    b = wl.bert_large_param_set()
    assert b.n_tensors == 391 and b.P == 335_141_888
    assert wl.get_config("quadratic").P == 1 << 20
    for name, slots in (("quadratic", 2), ("resnet50_w8", 3), ("resnet50_w16", 1), ("bert_large_w4", 5)):
        assert wl.get_config(name).slots == slots


def test_bits_match_scalar_splitmix64():
    """The tensor generator equals the scalar splitmix64 definition in Python integers."""
    key = stream_key(7, 3, 11)
    idx = torch.tensor([0, 1, 2, 12345, (1 << 40) + 17], dtype=torch.int64)
    got = random_bits(key, idx).tolist()
    for i, g in zip(idx.tolist(), got):
        want = _mix_py(key + (i + 1) * 0x9E3779B97F4A7C15)
        assert (g & ((1 << 64) - 1)) == want


def test_subset_regeneration_is_bit_identical():
    cfg = wl.get_config("resnet50_w8").scaled(params=wl.shapes.custom_param_set([64, 1000, 4099, 7]))
    idx = torch.tensor([0, 63, 64, 1063, 1064, 5162, 5163, 5169])
    w0 = wl.init_weights(cfg)
    assert torch.equal(wl.init_weights(cfg, idx=idx), w0[idx])
    g = wl.gradient(cfg, 3, 1)
    assert torch.equal(wl.gradient(cfg, 3, 1, idx=idx), g[idx])
    assert not torch.equal(g, wl.gradient(cfg, 3, 2))
    assert not torch.equal(g, wl.gradient(cfg, 4, 1))
    assert torch.equal(g, wl.gradient(cfg, 3, 1))


def test_distributions():
    key = stream_key(0, 99)
    z = wl.normal_like_flat(key, 1 << 21)
    assert abs(float(z.mean())) < 3e-3 and abs(float(z.std()) - 1) < 3e-3
    assert abs(float((z ** 4).mean()) - 3) < 0.05 and float(z.abs().max()) < 5.0
    u = wl.uniform01(key, torch.arange(1 << 20))
    assert 0 < float(u.min()) and float(u.max()) < 1 and abs(float(u.mean()) - 0.5) < 2e-3


def test_relative_gradient_scale():
    """Gradient std of tensor t is 1e-3 * ||w0_t|| / sqrt(n_t) (norm at init)."""
    cfg = wl.get_config("resnet50_w8").scaled(params=wl.shapes.custom_param_set([4096, 65536]))
    w0 = wl.init_weights(cfg).double()
    g = wl.gradient(cfg, 0, 0).double()
    off = cfg.params.offsets
    for t in range(2):
        want = 1e-3 * float(w0[off[t]:off[t + 1]].norm()) / np.sqrt(cfg.params.numel[t])
        got = float(g[off[t]:off[t + 1]].std())
        assert abs(got / want - 1) < 0.02


def test_quadratic_problem():
    cfg = wl.get_config("quadratic").scaled(params=wl.flat_param_set(4096))
    q = wl.QuadraticProblem.build(cfg)
    assert q.h.shape == (4096,) and q.c.shape == (4, 4096)
    assert 0.1 <= float(q.h.min()) and float(q.h.max()) <= 1.0
    idx = torch.tensor([5, 77, 4095])
    qs = wl.QuadraticProblem.build(cfg, idx=idx)
    assert torch.equal(qs.h, q.h[idx]) and torch.equal(qs.c, q.c[:, idx])
    x = torch.randn(4096)
    assert torch.equal(qs.grad(x[idx], 2, 1, idx=idx), q.grad(x, 2, 1)[idx])
    g64 = q.grad(x.double(), 2, 1)
    assert g64.dtype == torch.float64 and torch.allclose(g64.float(), q.grad(x, 2, 1), atol=1e-6)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU program: asking for more must end with a message, not a run."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
