"""The C ABI without a GPU: exported symbols, argument validation, and the host-side state machine
(step counter, pending-average ring, due / overdue rules) in dry-run mode."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

import paper_2006_00441_amd as pkg
from paper_2006_00441_amd import DaSGD, DasgdError

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_in(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dasgd_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    """Both headers: the method's calls (dasgd.h) and the diagnostics (dasgd_diag.h)."""
    method, diag = declared_in("dasgd.h"), declared_in("dasgd_diag.h")
    assert {"dasgd_create", "dasgd_bind", "dasgd_local_step", "dasgd_average_begin", "dasgd_merge", "dasgd_destroy",
            "dasgd_set_xi", "dasgd_set_lr", "dasgd_workspace_bytes", "dasgd_query", "dasgd_step"} <= set(method)
    assert len(method) <= 20, "diagnostics belong in dasgd_diag.h"
    assert not set(method) & set(diag)
    assert {"dasgd_profile", "dasgd_band", "dasgd_check_work_map", "dasgd_bind_dry_run"} <= set(diag)
    names = sorted(method + diag)
    assert sorted(pkg.EXPORTS) == names, "binding and header disagree"
    L = pkg.lib()
    for n in names:
        assert hasattr(L, n), n
    out = subprocess.run(["nm", "-D", "--defined-only", pkg.library_path()], capture_output=True, text=True).stdout
    exported = set(re.findall(r" T (dasgd_[a-z_]+)", out))
    assert exported == set(names)


def test_library_has_gfx950_code_object():
    data = open(pkg.library_path(), "rb").read()
    assert b"gfx950" in data


def test_create_validates_arguments():
    ok = dict(W=4, P=100, d=1, tau=1, lr=0.1, momentum=0.9, wd=1e-4)
    DaSGD(**ok).destroy()
    bad = [dict(W=0), dict(P=0), dict(d=-1), dict(tau=0), dict(lr=float("nan")), dict(lr=-1.0),
           dict(momentum=1.0), dict(momentum=-0.1), dict(wd=-1.0), dict(wd=float("inf"))]
    for b in bad:
        with pytest.raises(DasgdError):
            DaSGD(**{**ok, **b})
    o = DaSGD(**ok)
    for xi in (-0.1, 1.5, float("nan")):
        with pytest.raises(DasgdError):
            o.set_xi(xi)
    o.set_xi(0.0); o.set_xi(1.0)
    with pytest.raises(DasgdError):
        o.set_lr(float("inf"))
    with pytest.raises(DasgdError):
        o.set_schedule(7)
    o.set_schedule(pkg.SCHED_AUTO)
    assert o.schedule_in_use()[:2] == (pkg.SCHED_AUTO, False)
    o.set_schedule(pkg.SCHED_SERIAL)
    assert o.schedule_in_use()[:2] == (pkg.SCHED_SERIAL, True)
    for f in (-1, 5):
        with pytest.raises(DasgdError):
            o.set_fusion(f)
    for f in (pkg.FUSE_NONE, pkg.FUSE_SNAPSHOT, pkg.FUSE_STEP_MERGE, pkg.FUSE_ALL, pkg.FUSE_AUTO):
        o.set_fusion(f)
    for m in (-1, 3):
        with pytest.raises(DasgdError):
            o.set_snapshot(m)
    o.set_snapshot(pkg.SNAPSHOT_COPY); o.set_snapshot(pkg.SNAPSHOT_ZERO_COPY); o.set_snapshot(pkg.SNAPSHOT_AUTO)
    o.set_side_stream_threshold(0); o.set_side_stream_threshold(1 << 40)
    o.set_side_stream_head_start(0); o.set_side_stream_head_start(200)
    with pytest.raises(pkg.DasgdError):
        o.set_side_stream_head_start(201)
    for b in (-2, 12):
        with pytest.raises(DasgdError):
            o.set_band(b)
    for b in (-1, 0, 11):
        o.set_band(b)
    with pytest.raises(DasgdError) as e:
        o.band(pkg.K_STEP_MERGE)                 # nothing bound yet
    assert e.value.code == pkg.DASGD_ESTATE
    o.destroy()


def test_workspace_bytes_and_shapes():
    o = DaSGD(8, 64 + 1000 + 5000, 2, 1, 0.1, 0.9, 0.0)
    assert o.workspace_bytes([64, 1000, 5001]) == 0          # does not sum to P
    assert o.workspace_bytes([64, 0, 6000]) == 0
    n = o.workspace_bytes([64, 1000, 5000])
    ppad = 64 + 1024 + 5056 + 256        # tensors padded to 64 elements (a multiple of 256 in all), plus 256
    slots = 3
    assert n >= 4 * slots * (8 + 1) * ppad and n % 256 == 0
    with pytest.raises(DasgdError) as e:
        o.local_step(None)
    assert e.value.code == pkg.DASGD_ESTATE                  # not bound
    o.bind_dry_run([64, 1000, 5000])
    assert o.layout() == ([0, 64, 64 + 1024], ppad)
    with pytest.raises(DasgdError) as e:
        o.bind_dry_run([64, 1000, 5000])
    assert e.value.code == pkg.DASGD_ESTATE                  # already bound
    o.destroy()


@pytest.mark.parametrize("tau,d", [(1, 0), (1, 1), (1, 2), (1, 4), (4, 2), (3, 3), (2, 5), (4, 1), (5, 4)])
def test_state_machine_follows_the_oracle_schedule(tau, d):
    """The library's begin_due / merge_due sequence equals the oracle's launch / merge sequence."""
    import oracle
    o = DaSGD(2, 3, d, tau, 0.1, 0.0, 0.0)
    o.bind_dry_run([3])
    ref = oracle.Oracle(2, 3, d, tau, 0.1, 0.0, 0.0, np.zeros(3))
    g = np.zeros((2, 3))
    assert o.query() == (-1, 0, False, False)
    for k in range(7 * tau + d + 2):
        what = ref.step(g)
        o.local_step(None)
        kk, _, b, m0 = o.query()
        assert kk == k and b == bool(what & 1)
        if b:
            o.average_begin()
        _, npend, b2, m = o.query()
        assert not b2 and m == bool(what & 2)
        assert npend <= d // tau + 1
        if m:
            o.merge()
        assert o.query()[1] == ref.n_pending
    o.destroy(); ref.close()


def test_illegal_call_orders_are_rejected():
    E = pkg.DASGD_ESTATE
    o = DaSGD(2, 8, 1, 2, 0.1, 0.9, 0.0)           # tau=2, d=1
    o.bind_dry_run([8])

    def fails(f):
        with pytest.raises(DasgdError) as e:
            f()
        assert e.value.code == E

    fails(o.average_begin)                          # before any local step
    fails(o.merge)
    o.local_step(None)                              # k=0: nothing due
    fails(o.average_begin); fails(o.merge)
    o.local_step(None)                              # k=1: begin due
    fails(o.merge)                                  # nothing pending yet
    fails(lambda: o.local_step(None))               # begin not issued
    fails(lambda: o.set_schedule(pkg.SCHED_SERIAL))
    o.average_begin()
    fails(o.average_begin)                          # twice for the same step
    fails(o.merge)                                  # launched at k=1, due at k=2
    fails(lambda: o.set_schedule(pkg.SCHED_SERIAL)) # an average is pending
    o.local_step(None)                              # k=2: merge due
    fails(lambda: o.local_step(None))               # merge not issued
    o.merge()
    fails(o.merge)
    assert o.query() == (2, 0, False, False)
    o.set_schedule(pkg.SCHED_SERIAL)
    o.destroy()


def test_gpu_calls_fail_loudly_without_a_device():
    """No GPU here: binding real memory must fail with an error, never fall back to anything."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    o = DaSGD(1, 4, 0, 1, 0.1, 0.0, 0.0)
    with pytest.raises(RuntimeError):
        o.bind_tensors([[torch.zeros(4)]], [[torch.zeros(4)]], None, None)
    with pytest.raises(DasgdError):
        o.profile(1)
    o.destroy()


def test_choose_delay_reproduces_table_2():
    """The delay / period guideline (Section 3.4 Eq. 3, Section 6.4) gives the paper's own choices for
    all 14 cells of Table 2 (tests/golden/table2_delay.txt)."""
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "table2_delay.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 14
    for model, cluster, t_p, t_c, d, tau in rows:
        assert pkg.choose_delay(float(t_c), float(t_p)) == (int(d), int(tau)), (model, cluster)
    assert pkg.choose_delay(0.0, 1.0) == (1, 2)
    assert pkg.choose_delay(2.0, 1.0) == (3, 4)          # t_c < d t_p is strict
    for bad in ((-1.0, 1.0), (1.0, 0.0), (float("nan"), 1.0), (1.0, float("inf"))):
        with pytest.raises(DasgdError):
            pkg.choose_delay(*bad)


def test_step_is_the_canonical_loop():
    """dasgd_step == local_step + average_begin when due + merge when due (dry run: state only)."""
    for tau, d in ((1, 2), (4, 2), (3, 0)):
        a = DaSGD(2, 8, d, tau, 0.1, 0.9, 0.0); a.bind_dry_run([8])
        b = DaSGD(2, 8, d, tau, 0.1, 0.9, 0.0); b.bind_dry_run([8])
        for k in range(5 * tau + d + 2):
            began, merged = a.step(None)
            b.local_step(None)
            _, _, bd, _ = b.query()
            if bd:
                b.average_begin()
            _, _, _, md = b.query()
            if md:
                b.merge()
            assert (began, merged) == (bd, md)
            assert a.query() == b.query()
        a.destroy(); b.destroy()


def test_work_maps_cover_every_column_once():
    """The index arithmetic that decides which workgroup and lane touch which kilobyte, checked on the host
    with the functions the kernels themselves call: rows of any length and any offset from a kilobyte
    boundary over every band length, and the window order of the mean kernels.  A gap would leave elements
    un-updated; an overlap or an overrun would race or fault."""
    for row4 in (1, 2, 63, 64, 65, 100, 127, 128, 129, 640, 1000, 4099, 70001):
        for head in (0, 1, 17, 62, 63):
            for lb in (0, 1, 3, 5, 8, 11):
                assert pkg.check_work_map(pkg.MAP_ROWS, row4, head, lb) == 0, (row4, head, lb)
        for kind in (pkg.MAP_MEAN, pkg.MAP_MEAN_RUNS):
            assert pkg.check_work_map(kind, row4) == 0, (kind, row4)
    for row4, head, lb in ((6389258, 40, 9), (6389312, 0, 5), (83785472, 0, 9), (83785472, 63, 11), (2 ** 27, 1, 0)):
        assert pkg.check_work_map(pkg.MAP_ROWS, row4, head, lb) == 0, (row4, head, lb)
        assert pkg.check_work_map(pkg.MAP_MEAN_RUNS, row4) == 0
    for bad in ((pkg.MAP_ROWS, 0, 0, 0), (pkg.MAP_ROWS, 100, 64, 0), (pkg.MAP_ROWS, 100, -1, 0), (pkg.MAP_ROWS, 100, 0, 12),
                (pkg.MAP_ROWS, 2 ** 27 + 1, 0, 0), (7, 100, 0, 0), (pkg.MAP_MEAN, 2 ** 31, 0, 0)):
        with pytest.raises(DasgdError):
            pkg.check_work_map(*bad)


def test_replica_matrix_helper_lays_rows_out_as_documented():
    import torch
    m, views = DaSGD.replica_matrix(3, [5, 300, 7], device="cpu")
    assert m.shape == (3, 512) and m.dtype == torch.float32 and float(m.abs().sum()) == 0.0
    assert [v.numel() for v in views[2]] == [5, 300, 7]
    base = m.data_ptr()
    assert views[0][0].data_ptr() == base and views[0][1].data_ptr() == base + 4 * 5
    assert views[2][2].data_ptr() == base + 4 * (2 * 512 + 305)
    assert DaSGD.replica_matrix(2, [256], device="cpu")[0].shape == (2, 256)
    assert DaSGD.replica_matrix(2, [10], device="cpu", row_align=4)[0].shape == (2, 12)
    with pytest.raises(ValueError):
        DaSGD.replica_matrix(2, [10], device="cpu", row_align=8192)
