"""Checks that pin the CPU oracle to facts fixed by the paper and by mathematics.

Each check takes the loaded oracle library, so the mutation tests can run the same checks on
deliberately broken copies of the oracle and show that every planted mistake is caught.
None of these checks re-types the oracle's loop: they compare it with library routines
(torch.optim.SGD, torch.mean), with the paper's averaged-model recursion, with a closed-form
matrix power, with hand-worked exact numbers and with invariants of Eq. 2.
"""
from __future__ import annotations

import os

import numpy as np
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _torch_sgd_run(w0, grads, lr, momentum, wd, lr_schedule=None):
    """Plain momentum SGD by the library routine; grads: [K, P] (fp64). Returns [K+1, P]."""
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=oracle.f32(lr), momentum=oracle.f32(momentum),
                          weight_decay=oracle.f32(wd), dampening=0.0, nesterov=False)
    traj = [p.detach().clone().numpy()]
    for k in range(grads.shape[0]):
        if lr_schedule is not None:
            for grp in opt.param_groups:
                grp["lr"] = oracle.f32(lr_schedule[k])
        p.grad = torch.tensor(grads[k], dtype=torch.float64)
        opt.step()
        traj.append(p.detach().clone().numpy())
    return np.stack(traj)


# ----------------------------------------------------------------------------------------------
def check_hand_example(lib, dtype="f32"):
    """Hand-worked dyadic example of Eq. 2 (tests/golden/eq2_hand_example.txt): bit-exact."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq2_hand_example.txt"))
            if l.strip() and not l.startswith("#")]
    g = np.array([[1.0], [3.0]])
    for mom in (0.0, 0.5):
        o = oracle.Oracle(2, 1, 1, 2, 1.0, mom, 0.0, np.zeros(1), xi=0.25, dtype=dtype, lib=lib)
        want = {int(r[1]): (float(r[2]), float(r[3])) for r in rows if float(r[0]) == mom}
        for k in range(max(want)):
            o.step(g)
            assert tuple(o.x[:, 0]) == want[k + 1], (mom, k + 1, o.x[:, 0], want[k + 1])
        o.close()


def check_local_update_is_library_sgd(lib):
    """With no averaging in reach (tau > steps) every replica is plain momentum SGD with coupled
    weight decay: compare with torch.optim.SGD, including a learning-rate change mid-run (which
    separates 'lr outside the momentum buffer' from 'lr folded into it')."""
    r = _rng(1)
    W, P, K = 3, 17, 25
    w0 = r.standard_normal(P)
    g = r.standard_normal((K, W, P))
    lrs = [0.1 if k < 10 else 0.03 for k in range(K)]
    o = oracle.Oracle(W, P, 0, 1000, lrs[0], 0.9, 0.01, w0, dtype="f64", lib=lib)
    for k in range(K):
        o.set_lr(lrs[k])
        assert o.step(g[k]) == 0
    for j in range(W):
        ref = _torch_sgd_run(w0, g[:, j], lrs[0], 0.9, 0.01, lr_schedule=lrs)[-1]
        np.testing.assert_allclose(o.x[j], ref, rtol=1e-12, atol=1e-13)
    o.close()


def check_w1_d0_is_plain_sgd(lib):
    """One worker, no delay: the merge folds the worker's own value into itself, for any xi
    (Eq. 2 with M = 1, d = 0) -> plain momentum SGD."""
    r = _rng(2)
    P, K = 11, 30
    w0 = r.standard_normal(P)
    g = r.standard_normal((K, 1, P))
    for xi, tau in ((0.25, 1), (0.0, 3), (0.7, 2)):
        o = oracle.Oracle(1, P, 0, tau, 0.05, 0.9, 1e-3, w0, xi=xi, dtype="f64", lib=lib)
        for k in range(K):
            o.step(g[k])
        ref = _torch_sgd_run(w0, g[:, 0], 0.05, 0.9, 1e-3)[-1]
        np.testing.assert_allclose(o.x[0], ref, rtol=1e-11, atol=1e-12)
        o.close()


def check_xi1_is_plain_sgd(lib):
    """xi = 1 keeps the whole local value at a merge: every replica is plain SGD for any d."""
    r = _rng(3)
    W, P, K = 4, 9, 24
    w0 = r.standard_normal(P)
    g = r.standard_normal((K, W, P))
    o = oracle.Oracle(W, P, 2, 3, 0.05, 0.9, 1e-3, w0, xi=1.0, dtype="f64", lib=lib)
    merged = 0
    for k in range(K):
        merged += (o.step(g[k]) & 2) != 0
    assert merged >= 6
    for j in range(W):
        ref = _torch_sgd_run(w0, g[:, j], 0.05, 0.9, 1e-3)[-1]
        np.testing.assert_allclose(o.x[j], ref, rtol=1e-11, atol=1e-12)
    o.close()


def check_minibatch_sgd_special_case(lib):
    """d = 0, tau = 1, xi = 0 is synchronous model averaging: all replicas coincide after every
    step and follow one-worker SGD on the mean gradient (Section 2.1, per-worker form of Eq. 1).
    For any xi the replica MEAN follows that same trajectory (gradients are external)."""
    r = _rng(4)
    W, P, K = 4, 13, 20
    w0 = r.standard_normal(P)
    g = r.standard_normal((K, W, P))
    ref = _torch_sgd_run(w0, g.mean(axis=1), 0.1, 0.9, 1e-2)
    o = oracle.Oracle(W, P, 0, 1, 0.1, 0.9, 1e-2, w0, xi=0.0, dtype="f64", lib=lib)
    for k in range(K):
        assert o.step(g[k]) == 3
        for j in range(W):
            np.testing.assert_allclose(o.x[j], ref[k + 1], rtol=1e-11, atol=1e-12)
    o.close()
    o = oracle.Oracle(W, P, 0, 1, 0.1, 0.9, 1e-2, w0, xi=0.4, dtype="f64", lib=lib)
    for k in range(K):
        o.step(g[k])
        np.testing.assert_allclose(o.x.mean(axis=0), ref[k + 1], rtol=1e-11, atol=1e-12)
    assert np.abs(o.x[0] - o.x[1]).max() > 1e-3      # xi > 0 keeps replicas apart
    o.close()


def check_local_sgd_special_case(lib):
    """Delay 0 is Local SGD (Section 4.3, 'Delay'): tau independent local steps per worker, then
    every worker takes the plain average (xi = 0).  Reference: W torch.optim.SGD workers whose
    parameters are replaced by torch.mean every tau steps (momentum buffers stay local)."""
    r = _rng(5)
    W, P, K, tau = 3, 7, 18, 3
    w0 = r.standard_normal(P)
    g = r.standard_normal((K, W, P))
    ps = [torch.tensor(w0, dtype=torch.float64, requires_grad=True) for _ in range(W)]
    opts = [torch.optim.SGD([p], lr=oracle.f32(0.05), momentum=oracle.f32(0.9),
                            weight_decay=oracle.f32(1e-3)) for p in ps]
    o = oracle.Oracle(W, P, 0, tau, 0.05, 0.9, 1e-3, w0, xi=0.0, dtype="f64", lib=lib)
    for k in range(K):
        for j in range(W):
            ps[j].grad = torch.tensor(g[k, j]); opts[j].step()
        if (k + 1) % tau == 0:
            avg = torch.mean(torch.stack([p.detach() for p in ps]), dim=0)
            for p in ps:
                p.data.copy_(avg)
        what = o.step(g[k])
        assert what == (3 if (k + 1) % tau == 0 else 0)
        for j in range(W):
            np.testing.assert_allclose(o.x[j], ps[j].detach().numpy(), rtol=1e-11, atol=1e-12)
    o.close()


def check_averaged_model_identity(lib):
    """The paper's recursion for the averaged model (Section 3.3.1; derived in the appendix):
        mu_{tau(n+1)+d} = mu_{tau n+d} - eta [ xi sum_{i=tau-d}^{tau-1} gbar_{tau n+d+i}
                                               + sum_{i=0}^{tau-1-d} gbar_{tau n+d+i} ]
    for plain SGD local steps and d < tau; gbar_k is the replica-mean gradient at iteration k
    and mu_k the replica mean of x_k.  Gradients here depend on x (nonlinearly) plus noise."""
    for (tau, d, xi, W) in ((4, 2, 0.25, 16), (3, 1, 0.6, 5), (5, 4, 0.1, 2), (2, 0, 0.3, 3), (4, 3, 0.0, 4)):
        r = _rng(100 + 10 * tau + d)
        P, periods, eta = 6, 5, 0.07
        K = tau * periods + d
        w0 = r.standard_normal(P)
        o = oracle.Oracle(W, P, d, tau, eta, 0.0, 0.0, w0, xi=xi, dtype="f64", lib=lib)
        shift = r.standard_normal((W, P))
        mu = [o.x.mean(axis=0).copy()]
        gbar = []
        for k in range(K):
            g = np.sin(o.x + shift) + 0.3 * r.standard_normal((W, P))
            gbar.append(g.mean(axis=0))
            o.step(g)
            mu.append(o.x.mean(axis=0).copy())
        eta32 = oracle.f32(eta); xi32 = oracle.f32(xi)
        for n in range(periods):
            base = tau * n + d
            rhs = mu[base] - eta32 * (xi32 * sum((gbar[base + i] for i in range(tau - d, tau)), np.zeros(P))
                                      + sum((gbar[base + i] for i in range(0, tau - d)), np.zeros(P)))
            np.testing.assert_allclose(mu[tau * (n + 1) + d], rhs, rtol=1e-11, atol=1e-12,
                                       err_msg=f"tau={tau} d={d} period {n}")
        o.close()


def check_merge_steps(lib):
    """Merges happen exactly at iterations k with (k+1-d) mod tau == 0 (appendix form of the
    trigger) once an average launched at k-d exists; averages launch at (k+1) mod tau == 0."""
    for (tau, d) in ((1, 0), (1, 1), (1, 2), (1, 4), (4, 2), (3, 3), (2, 5), (4, 1)):
        o = oracle.Oracle(2, 3, d, tau, 0.1, 0.0, 0.0, np.zeros(3), dtype="f64", lib=lib)
        g = np.ones((2, 3))
        for k in range(6 * tau + d + 3):
            what = o.step(g)
            launch = (k + 1) % tau == 0
            merge = (k + 1 - d) % tau == 0 and (k - d) >= tau - 1
            assert what == (1 if launch else 0) + (2 if merge else 0), (tau, d, k, what)
            assert o.n_pending <= d // tau + 1
        o.close()


def check_identical_replicas(lib):
    """Identical init and identical gradients on every worker: the average equals each worker's
    own delayed value, so the W-replica run equals the one-replica run bit for bit (power-of-two
    W, tree-order mean), in both precisions."""
    r = _rng(6)
    P, K = 33, 40
    w0 = r.standard_normal(P).astype(np.float32)
    g1 = r.standard_normal((K, 1, P)).astype(np.float32)
    for dtype in ("f32", "f64"):
        for (W, tau, d) in ((8, 1, 2), (4, 4, 2), (16, 2, 1)):
            a = oracle.Oracle(1, P, d, tau, 0.1, 0.9, 1e-4, w0, dtype=dtype, lib=lib)
            b = oracle.Oracle(W, P, d, tau, 0.1, 0.9, 1e-4, w0, dtype=dtype, lib=lib)
            for k in range(K):
                a.step(g1[k]); b.step(np.repeat(g1[k], W, axis=0))
            for j in range(W):
                assert np.array_equal(b.x[j], a.x[0]), (dtype, W, tau, d, j)
            a.close(); b.close()


def check_delayed_self_merge(lib):
    """One worker with delay: Eq. 2 with M = 1 reads x_{k+1} = xi y_k + (1-xi) y_{k-d}, where
    y_k = x_k - lr v_{k+1}.  y is rebuilt here from the oracle's own x before and v after."""
    r = _rng(7)
    P, K, d, tau, xi, lr = 5, 20, 2, 1, 0.25, 0.1
    w0 = r.standard_normal(P)
    g = r.standard_normal((K, 1, P))
    o = oracle.Oracle(1, P, d, tau, lr, 0.9, 1e-3, w0, xi=xi, dtype="f64", lib=lib)
    ys = []
    for k in range(K):
        x_before = o.x[0].copy()
        what = o.step(g[k])
        ys.append(x_before - oracle.f32(lr) * o.v[0])
        if k >= d:
            assert what & 2
            want = oracle.f32(xi) * ys[k] + (1 - oracle.f32(xi)) * ys[k - d]
        else:
            assert not what & 2
            want = ys[k]
        np.testing.assert_allclose(o.x[0], want, rtol=1e-12, atol=1e-13)
    o.close()


def check_matrix_form(lib):
    """The appendix's matrix form for plain SGD local steps:
        X_{k+1} = xi (X_k - eta G_k) + (1 - xi) (X_{k-d} - eta G_{k-d}) J   when (k+1-d) mod tau == 0,
        X_{k+1} = X_k - eta G_k                                              otherwise,
    with J = 1 1^T / M applied as a matrix product (columns = workers).  Y_k = X_k - eta G_k is formed
    here from the oracle's X_k and the gradients it was fed."""
    r = _rng(12)
    for (tau, d, xi, M) in ((1, 2, 0.25, 8), (4, 2, 0.25, 4), (3, 3, 0.6, 5), (2, 1, 0.0, 3)):
        P, K, eta = 7, 6 * tau + d, 0.05
        J = np.full((M, M), 1.0 / M)
        o = oracle.Oracle(M, P, d, tau, eta, 0.0, 0.0, r.standard_normal(P), xi=xi, dtype="f64", lib=lib)
        Y = []
        for k in range(K):
            G = r.standard_normal((M, P))
            Y.append(o.x.T.copy() - oracle.f32(eta) * G.T)            # dim x M, as in the paper
            o.step(G)
            merge = (k + 1 - d) % tau == 0 and k - d >= tau - 1
            want = oracle.f32(xi) * Y[k] + (1 - oracle.f32(xi)) * (Y[k - d] @ J) if merge else Y[k]
            np.testing.assert_allclose(o.x.T, want, rtol=1e-12, atol=1e-13, err_msg=f"tau={tau} d={d} k={k}")
        o.close()


def check_xi_contraction(lib):
    """At a merge every replica moves toward a common point: the spread around the replica mean
    is multiplied by exactly xi, and the replica mean becomes xi ybar_k + (1-xi) A_{k-d}
    (Eq. 2, second branch; J(J - I) = 0 in the appendix's matrix form)."""
    r = _rng(8)
    W, P, K, d, tau, xi = 8, 12, 12, 2, 1, 0.25
    w0 = r.standard_normal(P)
    o = oracle.Oracle(W, P, d, tau, 0.1, 0.9, 1e-4, w0, xi=xi, dtype="f64", lib=lib)
    means_y = []
    for k in range(K):
        g = r.standard_normal((W, P))
        y = o.x.copy(); v = o.v.copy()
        oracle.local_update(y, v, g, 0.1, 0.9, 1e-4, lib=lib)
        means_y.append(y.mean(axis=0))
        what = o.step(g)
        if what & 2:
            np.testing.assert_allclose(o.x - o.x.mean(axis=0), oracle.f32(xi) * (y - y.mean(axis=0)),
                                       rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(o.x.mean(axis=0),
                                       oracle.f32(xi) * means_y[k] + (1 - oracle.f32(xi)) * means_y[k - d],
                                       rtol=1e-11, atol=1e-12)
        else:
            np.testing.assert_allclose(o.x, y, rtol=0, atol=0)
    o.close()


def quadratic_mean_closed_form(h, cbar, w0bar, K, tau, d, lr, momentum, wd, xi):
    """Replica-mean of the noise-free diagonal quadratic after K iterations, by matrix products.
    Per coordinate with a = h + wd, w* = h cbar / a, e = wbar - w*: the state
    s = (e, vbar, ytilde_{k-1}, ..., ytilde_{k-d}) evolves linearly:
        vbar' = momentum vbar + a e ;  ytilde = e - lr vbar'
        plain step:  e' = ytilde ;   merge step:  e' = xi ytilde + (1 - xi) ytilde_{k-d}
    fp64; independent of the time-stepping code (no replicas, no FIFO)."""
    lr, momentum, wd, xi = (oracle.f32(z) for z in (lr, momentum, wd, xi))
    a = h + wd
    wstar = h * cbar / a
    n = 2 + d
    P = h.shape[0]
    Tp = np.zeros((P, n, n)); Tm = np.zeros((P, n, n))
    for T, is_merge in ((Tp, False), (Tm, True)):
        yrow = np.zeros((P, n)); yrow[:, 0] = 1 - lr * a; yrow[:, 1] = -lr * momentum
        T[:, 1, 0] = a; T[:, 1, 1] = momentum
        if is_merge:
            T[:, 0, :] = xi * yrow
            T[:, 0, n - 1] += (1 - xi)           # old ytilde_{k-d}; for d = 0 this is ytilde itself
            if d == 0:
                T[:, 0, :] = yrow
        else:
            T[:, 0, :] = yrow
        if d >= 1:
            T[:, 2, :] = yrow
            for i in range(3, n):
                T[:, i, i - 1] = 1.0
    s = np.zeros((P, n)); s[:, 0] = w0bar - wstar
    for k in range(K):
        merge = (k + 1 - d) % tau == 0 and (k - d) >= tau - 1
        s = np.einsum("pij,pj->pi", Tm if merge else Tp, s)
    return wstar + s[:, 0], wstar


def check_quadratic_closed_form(lib):
    """Noise-free diagonal quadratic (worker j: 0.5 sum h (w - c_j)^2): the replica mean after K
    steps equals the closed-form matrix-power evolution; run long, it reaches the fixed point
    w* = h cbar / (h + wd)."""
    r = _rng(9)
    P = 24
    h = r.uniform(0.1, 1.0, P)
    c0 = r.standard_normal(P)
    for (W, tau, d, K) in ((4, 1, 1, 20), (8, 1, 2, 37), (4, 4, 2, 41), (2, 2, 5, 30), (4, 1, 0, 15), (3, 1, 1, 2500)):
        c = c0 + 0.1 * r.standard_normal((W, P))
        w0 = np.zeros(P)
        o = oracle.Oracle(W, P, d, tau, 0.1, 0.9, 1e-4, w0, xi=0.25, dtype="f64", lib=lib)
        o.run(K, lambda k, x: h * (x - c))
        want, wstar = quadratic_mean_closed_form(h, c.mean(axis=0), w0, K, tau, d, 0.1, 0.9, 1e-4, 0.25)
        np.testing.assert_allclose(o.x.mean(axis=0), want, rtol=1e-9, atol=1e-11,
                                   err_msg=f"W={W} tau={tau} d={d} K={K}")
        if K >= 2000:
            np.testing.assert_allclose(o.x.mean(axis=0), wstar, rtol=1e-9, atol=1e-10)
        o.close()


def check_mean(lib):
    """The mean agrees with numpy's fp64 mean; identical inputs at power-of-two W come back
    bit-exactly; W = 1 is the identity."""
    r = _rng(10)
    for W in (1, 2, 3, 4, 5, 8, 16, 17):
        y = r.standard_normal((W, 50))
        np.testing.assert_allclose(oracle.mean(y, lib=lib), y.mean(axis=0), rtol=1e-14, atol=1e-15)
        y32 = y.astype(np.float32)
        np.testing.assert_allclose(oracle.mean(y32, lib=lib), y.mean(axis=0), rtol=0, atol=W * 6e-8 * 4)
    row = r.standard_normal((1, 50)).astype(np.float32)
    for W in (1, 2, 4, 8, 16):
        assert np.array_equal(oracle.mean(np.repeat(row, W, axis=0), lib=lib), row[0])


def check_f32_tracks_f64(lib):
    """The fp32 run stays within 1e-5 of the parameter scale of the fp64 run (the tolerance the
    GPU path is held to) on a run shaped like the benchmark configs."""
    r = _rng(11)
    W, P, K = 8, 4096, 100
    w0 = (r.standard_normal(P) * 0.05).astype(np.float32)
    a = oracle.Oracle(W, P, 2, 1, 0.1, 0.9, 1e-4, w0, dtype="f32", lib=lib)
    b = oracle.Oracle(W, P, 2, 1, 0.1, 0.9, 1e-4, w0, dtype="f64", lib=lib)
    for k in range(K):
        g = (r.standard_normal((W, P)) * 5e-5).astype(np.float32)
        a.step(g); b.step(g.astype(np.float64))
    scale = max(np.sqrt((b.x ** 2).mean()), np.sqrt((w0.astype(np.float64) ** 2).mean()))
    assert np.abs(a.x - b.x).max() <= 1e-5 * scale
    a.close(); b.close()


ALL_CHECKS = [
    check_hand_example,
    check_local_update_is_library_sgd,
    check_w1_d0_is_plain_sgd,
    check_xi1_is_plain_sgd,
    check_minibatch_sgd_special_case,
    check_local_sgd_special_case,
    check_averaged_model_identity,
    check_merge_steps,
    check_identical_replicas,
    check_delayed_self_merge,
    check_matrix_form,
    check_xi_contraction,
    check_quadratic_closed_form,
    check_mean,
    check_f32_tracks_f64,
]
