#!/usr/bin/env python3
"""Benchmark of the DaSGD per-step parameter pipeline on one MI355X.

A step is one pass of the whole hot path over all W replicas: local step, launch of the W-way mean
on the side stream, and the delayed merge (folded into the local-step kernel by default).  The default workload
is the ResNet-50-shaped set with W=8, tau=1, d=2 (every step launches an average and merges the one
launched two steps earlier).  Inputs (weights, momentum, gradients) are resident in HBM before the
timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50_w8|resnet50_w16|bert_large_w4|quadratic]
                    [--no-cpu-baseline] [--no-overlap-study] [--only-timed]
    python bench.py --sweep      # xi / d / tau study on the quadratic instead (its own JSON line)
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
ALU_STANDIN_ITERS = 18000      # loop trips of the ALU-bound stand-in (about the duration of the 8192^3 GEMM)
PROFILE_EVERY = 8              # per-kernel event timing samples one launch in 8 (an event pair costs ~5 us)


def algorithmic_bytes_per_rp(kernel: str, W: int) -> float:
    """Bytes the method itself must move per replica-parameter (fp32), by kernel."""
    return {"local_step": 20.0,                    # read x, v, g; write x, v
            "local_step_snapshot": 24.0,           # + write the snapshot
            "local_step_to_snapshot": 20.0,        # read x, v, g; write v and the snapshot (x is written by the merge)
            "step_merge": 20.0 + 4.0 / W,          # local step with the merge folded in: + read the average
            "step_snapshot_merge": 24.0 + 4.0 / W,  # ... + write the snapshot
            "step_mean": 20.0 + 4.0 / W,           # local step that also writes the mean
            "step_mean_merge": 20.0 + 8.0 / W,     # local step, mean and merge in one pass
            "mean": 4.0 + 4.0 / W,                 # read W rows, write one average
            "mean_reconstruct": 4.0 + 8.0 / W,     # ... and read the merged-in average to undo the merge
            "merge": 8.0 + 4.0 / W}[kernel]        # read x and the average (once), write x


class Bench:
    """Device state for one workload: W replicas of (x, v, g) in flat arenas plus a bound context."""

    fusion = None
    layout = "matrix"      # "matrix": W x P arenas, rows 128-byte aligned (arithmetic addressing);
                           # "separate": one allocation per tensor (chunk-table addressing)

    def __init__(self, cfg, schedule: int, gemm=False):
        """gemm: False = no forward/backward stand-in; True = one bf16 8192^3 torch.matmul per step;
        "alu" = the register-light ALU-bound stand-in kernel of bench_standin.hip."""
        import torch
        import workloads as wl
        import paper_2006_00441_amd as pkg
        self.torch, self.pkg, self.cfg = torch, pkg, cfg
        dev = torch.device("cuda:0")
        self.main = torch.cuda.Stream(dev)
        self.side = torch.cuda.Stream(dev)
        W, P = cfg.W, cfg.P
        off, n = cfg.params.offsets, cfg.params.n_tensors
        with torch.cuda.stream(self.main):
            w0 = wl.init_weights(cfg, dev)
            # W x ld matrices, rows 1 KiB aligned to each other: the layout of the arithmetic-addressed kernels
            self._full = [pkg.DaSGD.replica_matrix(W, cfg.params.numel, dev)[0] for _ in range(3)]
            self.x, self.v, self.g = (a[:, :P] for a in self._full)
            self.x.copy_(w0.unsqueeze(0).expand(W, P))
            if cfg.kind == "external":
                sigma = wl.grad_sigma_vector(cfg, dev)
                for j in range(W):
                    wl.gradient(cfg, 0, j, dev, sigma=sigma, out=self.g[j])
            else:
                q = wl.QuadraticProblem.build(cfg, dev)
                for j in range(W):
                    self.g[j].copy_(q.grad(self.x[j], 0, j))
            if gemm == "alu":
                self.alu = ctypes.CDLL(os.path.join(ROOT, "bench_standin.so"))
                self.alu.bench_alu_standin.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
                self.alu_blocks, self.alu_iters = 1024, ALU_STANDIN_ITERS
                self.alu_out = torch.empty(self.alu_blocks * 256, device=dev)
            elif gemm:   # forward/backward stand-in: bf16 GEMM 8192^3 from seeded N(0,1) data
                ii = torch.arange(8192 * 8192, device=dev, dtype=torch.int64)
                self.ga = wl.standard_normal(wl.stream_key(cfg.seed, 101), ii).view(8192, 8192).to(torch.bfloat16)
                self.gb = wl.standard_normal(wl.stream_key(cfg.seed, 102), ii).view(8192, 8192).to(torch.bfloat16)
                self.gc = torch.empty(8192, 8192, device=dev, dtype=torch.bfloat16)
                del ii
        self.gemm = gemm
        if Bench.layout == "separate":      # every tensor its own allocation: the multi-tensor (chunk table) path
            view = lambda a: [[a[j, off[t]:off[t + 1]].clone() for t in range(n)] for j in range(W)]
        else:
            view = lambda a: [[a[j, off[t]:off[t + 1]] for t in range(n)] for j in range(W)]
        self.opt = pkg.DaSGD(W, P, cfg.d, cfg.tau, cfg.lr, cfg.momentum, cfg.wd, xi=cfg.xi)
        with torch.cuda.stream(self.main):
            xs, vs, gs = view(self.x), view(self.v), view(self.g)
        self.main.synchronize()
        if Bench.layout == "separate":
            self.x = self.v = self.g = self._full = None
            torch.cuda.empty_cache()
        self._tensors = (xs, vs, gs)
        self.ws = self.opt.bind_tensors(xs, vs, self.main, self.side)
        self.opt.set_schedule(schedule)
        if Bench.fusion is not None:
            self.opt.set_fusion(Bench.fusion)
        self.g_ptrs = pkg.DaSGD.grad_pointers(gs)
        self.first = True
        self.steps_done = 0
        self.main.synchronize()

    def step(self):
        if self.gemm == "alu":
            rc = self.alu.bench_alu_standin(self.alu_out.data_ptr(), self.alu_blocks, self.alu_iters, self.main.cuda_stream)
            assert rc == 0, rc
        elif self.gemm:
            with self.torch.cuda.stream(self.main):
                self.torch.matmul(self.ga, self.gb, out=self.gc)
        self.opt.step(self.g_ptrs if self.first else None)
        self.first = False
        self.steps_done += 1

    def settle(self, limit: int = 512) -> int:
        """Untimed steps beyond the warm-up until the library has finished measuring its band lengths
        (a warm-up matter, like any autotuning): returns how many were needed."""
        extra = 0
        for _ in range(max(0, min(self.cfg.d + self.cfg.tau + 1, 64) - self.steps_done)):    # reach the first merge
            self.step()
            extra += 1
        self.torch.cuda.synchronize()
        prev = None
        while extra < limit:
            # (trial launches issued, settled) per kernel kind; a kind that is neither settled nor issuing
            # trials any more is simply not launched in this configuration: nothing to wait for
            now = {k: self.opt.band_state(k)[1:] for k in self.pkg.KERNEL_NAMES}
            busy = [k for k, (settled, trials) in now.items()
                    if trials > 0 and not settled and (prev is None or prev[k][1] != trials)]
            if not busy:
                break
            prev = now
            for _ in range(2 * self.cfg.tau):
                self.step()
            extra += 2 * self.cfg.tau
            self.torch.cuda.synchronize()
        return extra

    def run(self, steps: int, warmup: int):
        """Returns (wall seconds for `steps` steps, main-stream event milliseconds)."""
        torch = self.torch
        for _ in range(warmup):
            self.step()
        if warmup:
            self.settle()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(self.main)
        for _ in range(steps):
            self.step()
        e1.record(self.main)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return t1 - t0, e0.elapsed_time(e1)

    def close(self):
        self.opt.destroy()
        for a in ("x", "v", "g", "_full", "ws", "ga", "gb", "gc", "_tensors"):
            if hasattr(self, a):
                delattr(self, a)
        self.torch.cuda.empty_cache()


def copy_ceiling(cfg):
    """Bandwidth (read + write bytes over time) of a plain copy of W*P floats on this machine, with the
    harness's own copy kernel in the library's launch shape: what a pure stream reaches in practice,
    beside the vendor peak.  Both buffers are allocated afresh, like the arenas."""
    import torch
    lib = ctypes.CDLL(os.path.join(ROOT, "bench_standin.so"))
    lib.bench_copy_stream.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    n = (cfg.W * cfg.P + 3) // 4 * 4
    # weight-like values, not zeros: on MI355X a stream of zeros runs about 5 % faster than real data
    src = torch.empty(n, device="cuda:0").normal_(0.0, 0.05); dst = torch.empty_like(src)
    stream = torch.cuda.current_stream().cuda_stream

    def go():
        rc = lib.bench_copy_stream(dst.data_ptr(), src.data_ptr(), n, stream)
        if rc:
            raise RuntimeError(f"bench_copy_stream: {rc}")
    for _ in range(3):
        go()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(10):
        go()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 10
    del src, dst
    torch.cuda.empty_cache()
    return 2.0 * n * 4 / (ms * 1e-3) / 1e9


def timed_region(cfg, steps: int, warmup: int, gemm: bool = False):
    """The headline measurement: overlap schedule, per-kernel event timing live in the timed region."""
    import paper_2006_00441_amd as pkg
    b = Bench(cfg, pkg.SCHED_OVERLAP, gemm=gemm)
    for _ in range(warmup):
        b.step()
    tuning_steps = b.settle()
    b.opt.profile(PROFILE_EVERY, 4 * steps + 16)
    wall, ev_ms = b.run(steps, 0)
    kernels = {}
    for kid, name in pkg.KERNEL_NAMES.items():
        ms, n, launched = b.opt.profile_read(kid)
        if n:
            kernels[name] = {"launches": launched, "timed_launches": n, "avg_ms": ms / n}
    b.opt.profile(0)
    tuning = {"extra_untimed_steps": tuning_steps,
              "log2_band": {name: b.opt.band(k)[0] for k, name in pkg.KERNEL_NAMES.items() if b.opt.band_state(k)[2]}}
    b.close()
    return wall, ev_ms, kernels, tuning


def repeats(cfg, n: int = 5, steps: int = 50, warmup: int = 10, gemm=False):
    """Spread of the step time: n back-to-back timings of `steps` steps each (main-stream events)."""
    import paper_2006_00441_amd as pkg
    b = Bench(cfg, pkg.SCHED_OVERLAP, gemm=gemm)
    ms = []
    for r in range(n):
        _, ev = b.run(steps, warmup if r == 0 else 0)
        ms.append(ev / steps)
    b.close()
    ms.sort()
    return {"steps_each": steps, "ms_per_step": [round(m, 5) for m in ms], "median_ms_per_step": round(ms[n // 2], 5)}


def local_step_alone(cfg, steps: int, warmup: int):
    """Local step only (tau so large that no average is ever due): 20 B per replica-parameter."""
    import paper_2006_00441_amd as pkg
    b = Bench(cfg.scaled(tau=1 << 30), pkg.SCHED_OVERLAP)
    wall, _ = b.run(steps, warmup)
    b.close()
    rp = cfg.W * cfg.P
    gbs = 20.0 * rp * steps / wall / 1e9
    return {"ms_per_step": round(wall / steps * 1e3, 5), "value": rp * steps / wall, "unit": "replica-params/s",
            "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}


def fusion_all_region(cfg, steps: int, warmup: int):
    """The same workload with the mean folded into the local-step kernel as well (fusion level 3: one
    kernel per step, nothing on the side stream).  Reported beside the headline, never as it."""
    import paper_2006_00441_amd as pkg
    keep = Bench.fusion
    Bench.fusion = pkg.FUSE_ALL
    try:
        b = Bench(cfg, pkg.SCHED_OVERLAP)
        for _ in range(warmup):
            b.step()
        b.opt.profile(PROFILE_EVERY, 4 * steps + 16)
        wall, _ = b.run(steps, 0)
        ks = {}
        for kid, name in pkg.KERNEL_NAMES.items():
            ms, n, launched = b.opt.profile_read(kid)
            if n:
                bts = algorithmic_bytes_per_rp(name, cfg.W) * cfg.W * cfg.P
                ks[name] = {"avg_ms": round(ms / n, 5), "launches": launched,
                            "frac_of_hbm_peak": round(bts / (ms / n * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        b.close()
    finally:
        Bench.fusion = keep
    return {"ms_per_step": wall / steps * 1e3, "value": cfg.W * cfg.P * steps / wall, "kernels": ks}


def overlap_study(cfg, steps: int, warmup: int, gemm: bool):
    """Three schedules with identical kernels: S0 everything on one stream, S1 the mean on the side
    stream, F = S0 without snapshot and mean (timing floor).  hidden = (T(S0)-T(S1)) / (T(S0)-T(F))."""
    import paper_2006_00441_amd as pkg
    t = {}
    for name, sched in (("S0_serial", pkg.SCHED_SERIAL), ("S1_overlap", pkg.SCHED_OVERLAP),
                        ("S1_overlap_free", pkg.SCHED_OVERLAP_FREE), ("F_no_average", pkg.SCHED_NO_AVERAGE_TIMING_ONLY)):
        b = Bench(cfg, sched, gemm=gemm)
        best = min(b.run(steps, warmup if r == 0 else 2)[0] for r in range(3))
        t[name] = best / steps * 1e3
        b.close()
    t_avg = t["S0_serial"] - t["F_no_average"]
    hidden = (t["S0_serial"] - t["S1_overlap"]) / t_avg if t_avg > 0 else None
    hidden_free = (t["S0_serial"] - t["S1_overlap_free"]) / t_avg if t_avg > 0 else None
    return {"stand_in": {False: "none", True: "bf16 GEMM 8192^3 (torch.matmul)", "alu": "ALU-bound kernel, 4 waves/SIMD, 16 VGPRs"}[gemm],
            "ms_per_step": {k: round(v, 4) for k, v in t.items()},
            "averaging_ms": round(t_avg, 4), "hidden_frac": None if hidden is None else round(hidden, 4),
            "hidden_frac_overlap_free": None if hidden_free is None else round(hidden_free, 4),
            "speedup_S0_over_S1": round(t["S0_serial"] / t["S1_overlap"], 4)}


def compare_algorithms(cfg, steps: int, warmup: int):
    """The paper's three update schedules (Fig. 4; Eq. 4-6) timed on the same kernels, each local step
    preceded by the forward/backward stand-in (one bf16 8192^3 GEMM): synchronous Mini-batch SGD
    (blocking gradient mean every step, Eq. 1), Local SGD (tau = 4, blocking weight average, i.e.
    d = 0, xi = 0) and DaSGD (tau = 4, d = 2, xi = 0.25, the paper's parameter-study baseline), against a
    floor with local steps only.  share = (T - T_floor) / T, the on-device counterpart of the
    communication shares the paper simulates (Section 5.2)."""
    import torch
    import paper_2006_00441_amd as pkg
    variants = {
        "local_steps_only": dict(tau=10 ** 9, d=0, xi=1.0, mb=False),
        "minibatch_sgd": dict(tau=10 ** 9, d=0, xi=1.0, mb=True),
        "local_sgd_tau4": dict(tau=4, d=0, xi=0.0, mb=False),
        "dasgd_tau4_d2": dict(tau=4, d=2, xi=0.25, mb=False),
        "dasgd_tau1_d2": dict(tau=1, d=2, xi=0.25, mb=False),
    }
    out = {}
    for name, v in variants.items():
        c = cfg.scaled(tau=min(v["tau"], 2 ** 30), d=v["d"], xi=v["xi"])
        b = Bench(c, pkg.SCHED_OVERLAP, gemm=True)
        if v["mb"]:
            gbar = torch.zeros(c.P, device="cuda:0")
            off = c.params.offsets
            bcast = [gbar[off[t]:off[t + 1]].data_ptr() for _ in range(c.W) for t in range(c.params.n_tensors)]
            G = torch.zeros(c.W, c.P, device="cuda:0")      # gradient_average wants rows back to back
            G.copy_(b.g)
            Gp = G.data_ptr()

            def step(b=b, gbar=gbar, bcast=bcast, Gp=Gp):
                with torch.cuda.stream(b.main):
                    torch.matmul(b.ga, b.gb, out=b.gc)
                b.opt.gradient_average(Gp, gbar.data_ptr())
                b.opt.step(bcast if b.first else None)
                b.first = False
            b.step = step
        best = min(b.run(steps, warmup if r == 0 else 2)[0] for r in range(3))
        out[name] = best / steps * 1e3
        b.close()
    floor = out["local_steps_only"]
    return {"ms_per_step": {k: round(t, 4) for k, t in out.items()},
            "averaging_share": {k: round((t - floor) / t, 4) for k, t in out.items() if k != "local_steps_only"},
            "note": "each step = bf16 8192^3 GEMM stand-in + the schedule's parameter work, W=%d replicas" % cfg.W}


def quadratic_period_maps(a, lr: float, momentum: float, xi: float, d: int):
    """Linear maps of the replica-mean error on the noise-free quadratic (curvature + weight decay = a
    per coordinate; Eq. 2 with heavy-ball momentum).  State per coordinate: (e, vbar, ytilde_{k-1}, ...,
    ytilde_{k-d}) with e the distance of the replica mean from the fixed point.  Returns (plain step,
    merge step), each of shape [len(a), d+2, d+2], fp64."""
    import numpy as np
    a = np.asarray(a, dtype=np.float64)
    n = d + 2
    y = np.zeros((a.size, n)); y[:, 0] = 1.0 - lr * a; y[:, 1] = -lr * momentum   # ytilde from (e, vbar)
    plain = np.zeros((a.size, n, n))
    plain[:, 0] = y
    plain[:, 1, 0] = a; plain[:, 1, 1] = momentum
    if d:
        plain[:, 2] = y
        for i in range(3, n):
            plain[:, i, i - 1] = 1.0
    merge = plain.copy()
    if d:
        merge[:, 0] = xi * y
        merge[:, 0, n - 1] += 1.0 - xi
    return plain, merge


def sweep_quadratic(K0: int = 48, K1: int = 144):
    """Parameter study on the quadratic (xi, d and tau ranges of the paper's Fig. 6(d), 6(e) and its tau
    advice, Section 4): the HIP path runs the noise-free problem and the decay rate of the replica mean's
    distance to the fixed point between steps K0 and K1 is set beside the rate the linear recurrence
    predicts for the same window and beside its asymptote, the spectral radius of one period's map."""
    import numpy as np
    import torch
    import workloads as wl
    import paper_2006_00441_amd as pkg
    base = wl.get_config("quadratic")
    dev = torch.device("cuda:0")
    grid = [("xi", dict(xi=x, tau=4, d=2)) for x in (0.0, 0.1, 0.25, 0.5, 0.75, 0.9, 1.0)]
    grid += [("d", dict(xi=0.25, tau=8, d=d)) for d in range(8)]
    grid += [("tau", dict(xi=0.25, tau=t, d=1)) for t in (1, 2, 4, 8, 16, 48)]
    main, side = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
    rows = []
    for axis, kw in grid:
        cfg = base.scaled(**kw)
        W, P, tau, d, xi = cfg.W, cfg.P, cfg.tau, cfg.d, cfg.xi
        with torch.cuda.stream(main):
            q = wl.QuadraticProblem.build(cfg, dev, noise=False)
            x = torch.zeros(W, P, device=dev); v = torch.zeros_like(x); g = torch.empty_like(x)
            a32 = q.h.double() + float(np.float32(cfg.wd))
            wstar = q.h.double() * q.c.double().mean(0) / a32
        main.synchronize()
        opt = pkg.DaSGD(W, P, d, tau, cfg.lr, cfg.momentum, cfg.wd, xi=xi)
        ws = opt.bind_tensors([[x[j]] for j in range(W)], [[v[j]] for j in range(W)], main, side)
        gp = pkg.DaSGD.grad_pointers([[g[j]] for j in range(W)])
        sel = torch.arange(0, P, 64, device=dev)     # both sides look at every 64th coordinate
        err = {}
        for k in range(K1):
            with torch.cuda.stream(main):
                torch.mul(x - q.c, q.h, out=g)       # gradient at each replica's current iterate
            opt.step(gp if k == 0 else None)
            if k + 1 in (K0, K1):
                with torch.cuda.stream(main):
                    err[k + 1] = float((x[:, sel].double().mean(0) - wstar[sel]).norm())
        main.synchronize()
        opt.destroy()
        a = a32[sel].cpu().numpy()
        f = lambda z: float(np.float32(z))
        plain, merge = quadratic_period_maps(a, f(cfg.lr), f(cfg.momentum), f(xi), d)
        st = np.zeros((a.size, d + 2)); st[:, 0] = -wstar[sel].cpu().numpy()        # w0 = 0
        pred = {}
        for k in range(K1):
            is_merge = (k + 1 - d) % tau == 0 and k - d >= tau - 1
            st = np.einsum("pij,pj->pi", merge if is_merge else plain, st)
            if k + 1 in (K0, K1):
                pred[k + 1] = float(np.linalg.norm(st[:, 0]))
        period = np.broadcast_to(np.eye(d + 2), plain.shape).copy()
        for k in range(d, d + tau):                                       # one period in steady state
            period = np.einsum("pij,pjk->pik", merge if (k + 1 - d) % tau == 0 else plain, period)
        rho = float(np.abs(np.linalg.eigvals(period)).max() ** (1.0 / tau))
        rate = lambda e: (e[K1] / e[K0]) ** (1.0 / (K1 - K0))
        rows.append({"axis": axis, "xi": xi, "tau": tau, "d": d,
                     "error_at_K0": err[K0], "error_at_K1": err[K1],
                     "measured_rate_per_step": round(rate(err), 6), "recurrence_rate_per_step": round(rate(pred), 6),
                     "predicted_error_at_K1": pred[K1], "spectral_radius_per_step": round(rho, 6)})
        del ws
    return {"sweep": "noise-free quadratic, W=4, P=2^20, lr 0.1, momentum 0.9, wd 1e-4; error = L2 distance of the "
                     "replica mean from the fixed point over every 64th coordinate", "K0": K0, "K1": K1, "dtype": "f32", "rows": rows}


def cpu_baseline(cfg, budget_s: float = 12.0):
    """The CPU oracle (fp32 variant, as it stands) timed on this machine's host cores on a bounded number
    of steps of the same workload at full size."""
    import numpy as np
    import torch
    import oracle
    import workloads as wl
    cores = len(os.sched_getaffinity(0))
    threads = oracle.set_threads(cores)
    dev = torch.device("cuda:0")
    sigma = wl.grad_sigma_vector(cfg, dev) if cfg.kind == "external" else None
    g = np.empty((cfg.W, cfg.P), dtype=np.float32)
    for j in range(cfg.W):
        if sigma is not None:
            g[j] = wl.gradient(cfg, 0, j, dev, sigma=sigma).cpu().numpy()
        else:
            g[j] = 0.01
    w0 = wl.init_weights(cfg, dev).cpu().numpy()
    del sigma
    torch.cuda.empty_cache()
    o = oracle.Oracle(cfg.W, cfg.P, cfg.d, cfg.tau, cfg.lr, cfg.momentum, cfg.wd, w0, xi=cfg.xi, dtype="f32")
    for _ in range(cfg.d + 1):            # reach the steady state where every kind of step occurs
        o.step(g)
    t0 = time.perf_counter(); o.step(g); one = time.perf_counter() - t0
    n = int(max(3, min(200, budget_s / max(one, 1e-6))))
    n = max(cfg.tau, n // cfg.tau * cfg.tau)
    t0 = time.perf_counter()
    for _ in range(n):
        o.step(g)
    dt = time.perf_counter() - t0
    # the same oracle on one thread, a few steps (context: what one host core does)
    oracle.set_threads(1)
    n1 = max(cfg.tau, min(n, int(2.0 / max(one * threads / 4, 1e-6))) // cfg.tau * cfg.tau)
    t0 = time.perf_counter()
    for _ in range(n1):
        o.step(g)
    dt1 = time.perf_counter() - t0
    oracle.set_threads(threads)
    o.close()
    return {"value": cfg.W * cfg.P * n / dt, "unit": "replica-params/s", "cores": threads, "kind": "oracle",
            "single_thread_value": cfg.W * cfg.P * n1 / dt1, "single_thread_steps": n1,
            "sample": f"{n} steps of {cfg.name} at full size (W={cfg.W}, P={cfg.P}), fp32 oracle, "
                      f"{threads} OpenMP threads, {dt:.1f} s", "ms_per_step": dt / n * 1e3}


def pmc_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet50_w8")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap-study", action="store_true")
    ap.add_argument("--only-timed", action="store_true", help="just the timed region (for profilers)")
    ap.add_argument("--layout", default="matrix", choices=["matrix", "separate"],
                    help="matrix: x, v, g as W x P arenas (default); separate: one allocation per tensor")
    ap.add_argument("--fusion", type=int, default=None, help="fusion level 0..3 (default: the library's)")
    ap.add_argument("--stand-in", default=None, choices=["none", "gemm", "alu"],
                    help="forward/backward stand-in on the main stream before every step of the timed region: "
                         "bf16 8192^3 GEMM (default for --workload overlap), the register-light ALU kernel, or none")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark: xi / d / tau study on the quadratic, one JSON line")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="first run 5 plain torch copies of W*P floats (a kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the DaSGD pipeline on ONE GPU (W replicas share its HBM); "
              "--gpus above 1 is not supported", file=sys.stderr)
        return 2

    import torch
    import workloads as wl
    import paper_2006_00441_amd as pkg
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU implementation of this path", file=sys.stderr)
        return 2
    pkg.lib()
    if args.sweep:
        print(json.dumps(sweep_quadratic()))
        return 0
    Bench.layout = args.layout
    Bench.fusion = args.fusion
    cfg = wl.get_config(args.workload)
    rp = cfg.W * cfg.P

    if args.pmc_calibration:
        src = torch.zeros(cfg.W, cfg.P, device="cuda:0"); dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    stand_in = args.stand_in or ("gemm" if cfg.name == "overlap" else "none")
    wall, ev_ms, kernels, tuning = timed_region(cfg, args.steps, args.warmup,
                                                gemm={"none": False, "gemm": True, "alu": "alu"}[stand_in])
    ms_per_step = wall / args.steps * 1e3
    for name, k in kernels.items():
        b = algorithmic_bytes_per_rp(name, cfg.W) * rp
        k["algorithmic_bytes"] = b
        k["GBps"] = b / (k["avg_ms"] * 1e-3) / 1e9
        k["frac_of_hbm_peak"] = k["GBps"] / HBM_PEAK_GBS
    # the dominant kernel is the one that moves the most bytes over the run (a side-stream kernel that sits
    # behind a stand-in of the caller's looks long by the clock without being the one that does the work)
    dom = max(kernels, key=lambda k: kernels[k]["algorithmic_bytes"] * kernels[k]["launches"])
    d = kernels[dom]
    out = {
        "metric": "replica-params updated/s + achieved HBM GB/s; % averaging time hidden",
        "value": rp * args.steps / wall,
        "unit": "replica-params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_main_stream_events": ev_ms / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.params.name}-shaped, {cfg.params.n_tensors} fp32 tensors, "
                               f"P={cfg.P}, W={cfg.W}, tau={cfg.tau}, d={cfg.d}, xi={cfg.xi}",
                   "schedule": "overlap (mean on side stream)", "layout": args.layout, "replica_params": rp,
                   "stand_in": stand_in},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": d["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": d["frac_of_hbm_peak"], "avg_ms": d["avg_ms"], "launches": d["launches"], "timed_launches": d["timed_launches"],
                     "algorithmic_bytes_per_launch": d["algorithmic_bytes"],
                     "traffic": pmc_traffic(dom, cfg.name)},
        "kernels": {n: {"avg_ms": round(k["avg_ms"], 5), "launches": k["launches"], "timed_launches": k["timed_launches"],
                        "GBps": round(k["GBps"], 1),
                        "frac_of_hbm_peak": round(k["frac_of_hbm_peak"], 4)} for n, k in kernels.items()},
    }
    out["band_tuning"] = tuning
    step_bytes = sum(k["algorithmic_bytes"] * k["launches"] for k in kernels.values()) / args.steps
    out["whole_step"] = {"algorithmic_bytes": step_bytes, "GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
                         "frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS}
    if not args.only_timed and os.path.exists(os.path.join(ROOT, "bench_standin.so")):
        ceil_gbs = copy_ceiling(cfg)
        out["roofline"]["copy_ceiling_GBps"] = round(ceil_gbs, 1)
        out["roofline"]["frac_of_copy_ceiling"] = round(d["GBps"] / ceil_gbs, 4)
    if not args.only_timed and not args.no_overlap_study:
        k = max(20, min(args.steps, 100))
        out["overlap"] = {"hbm_bound_steps_only": overlap_study(cfg, k, 10, gemm=False),
                          "with_compute_stand_in": overlap_study(cfg, k, 10, gemm=True)}
        if os.path.exists(os.path.join(ROOT, "bench_standin.so")):
            out["overlap"]["with_register_light_stand_in"] = overlap_study(cfg, k, 10, gemm="alu")
        if cfg.kind == "external" and cfg.P % 4 == 0 and args.layout == "matrix":
            out["algorithms"] = compare_algorithms(cfg, 40, 8)
    if not args.only_timed:
        out["repeats"] = repeats(cfg, gemm={"none": False, "gemm": True, "alu": "alu"}[stand_in])
        out["local_step_alone"] = local_step_alone(cfg, args.steps, args.warmup)
    if not args.only_timed and args.layout == "matrix" and args.fusion is None:
        out["fusion_all"] = fusion_all_region(cfg, args.steps, args.warmup)
    if not args.only_timed and not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
