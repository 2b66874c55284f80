"""ctypes binding of include/dasgd.h and include/dasgd_diag.h: argument marshalling only.

`lib()` returns the loaded shared library with typed signatures; `DaSGD` wraps one context and
turns negative return codes into `DasgdError`.  Every method maps one-to-one onto the C call of
the same name (dasgd_local_step -> DaSGD.local_step, ...).  The only convenience is
`bind_tensors`, which takes torch tensors, collects their data pointers and allocates the
workspace with torch (PyTorch supplies device memory and streams; it computes nothing here).
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

from . import build as _build

DASGD_OK, DASGD_EINVAL, DASGD_ESTATE, DASGD_ENOMEM, DASGD_EHIP = 0, -1, -2, -3, -4
SCHED_OVERLAP, SCHED_SERIAL, SCHED_NO_AVERAGE_TIMING_ONLY, SCHED_OVERLAP_FREE, SCHED_AUTO = 0, 1, 2, 3, 4
K_LOCAL_STEP, K_LOCAL_STEP_SNAP, K_MEAN, K_MERGE, K_LOCAL_STEP_TO_SNAP, K_STEP_MERGE, K_STEP_SNAP_MERGE = 0, 1, 2, 3, 4, 5, 6
K_STEP_MEAN, K_STEP_MEAN_MERGE, K_MEAN_RECONSTRUCT = 7, 8, 9
SNAPSHOT_COPY, SNAPSHOT_ZERO_COPY, SNAPSHOT_AUTO = 0, 1, 2
ADDR_RECORDS, ADDR_ROWS, ADDR_ROWS_XV = 0, 1, 2
MAP_ROWS, MAP_MEAN, MAP_MEAN_RUNS = 0, 1, 2
FUSE_NONE, FUSE_SNAPSHOT, FUSE_STEP_MERGE, FUSE_ALL, FUSE_AUTO = 0, 1, 2, 3, 4
KERNEL_NAMES = {K_LOCAL_STEP: "local_step", K_LOCAL_STEP_SNAP: "local_step_snapshot",
                K_MEAN: "mean", K_MERGE: "merge", K_LOCAL_STEP_TO_SNAP: "local_step_to_snapshot",
                K_STEP_MERGE: "step_merge", K_STEP_SNAP_MERGE: "step_snapshot_merge",
                K_STEP_MEAN: "step_mean", K_STEP_MEAN_MERGE: "step_mean_merge",
                K_MEAN_RECONSTRUCT: "mean_reconstruct"}
_ERR = {DASGD_EINVAL: "DASGD_EINVAL (bad argument)", DASGD_ESTATE: "DASGD_ESTATE (call illegal in this state)",
        DASGD_ENOMEM: "DASGD_ENOMEM (workspace too small)", DASGD_EHIP: "DASGD_EHIP (HIP call failed)"}

_vp = ctypes.c_void_p
_i64 = ctypes.c_int64
_pp = ctypes.POINTER(ctypes.c_void_p)
_pi64 = ctypes.POINTER(ctypes.c_int64)
_pint = ctypes.POINTER(ctypes.c_int)

# name -> (restype, argtypes): every symbol include/dasgd.h and include/dasgd_diag.h declare
EXPORTS = {
    "dasgd_create": (_vp, [ctypes.c_int, _i64, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_float, ctypes.c_float]),
    "dasgd_set_xi": (ctypes.c_int, [_vp, ctypes.c_float]),
    "dasgd_set_lr": (ctypes.c_int, [_vp, ctypes.c_float]),
    "dasgd_set_schedule": (ctypes.c_int, [_vp, ctypes.c_int]),
    "dasgd_set_side_stream_threshold": (ctypes.c_int, [_vp, ctypes.c_size_t]),
    "dasgd_set_fusion": (ctypes.c_int, [_vp, ctypes.c_int]),
    "dasgd_set_snapshot": (ctypes.c_int, [_vp, ctypes.c_int]),
    "dasgd_workspace_bytes": (ctypes.c_size_t, [_vp, ctypes.c_int, _pi64]),
    "dasgd_bind": (ctypes.c_int, [_vp, ctypes.c_int, _pi64, _pp, _pp, _vp, ctypes.c_size_t, _vp, _vp]),
    "dasgd_bind_dry_run": (ctypes.c_int, [_vp, ctypes.c_int, _pi64]),
    "dasgd_local_step": (ctypes.c_int, [_vp, _pp]),
    "dasgd_average_begin": (ctypes.c_int, [_vp]),
    "dasgd_merge": (ctypes.c_int, [_vp]),
    "dasgd_step": (ctypes.c_int, [_vp, _pp, _pint, _pint]),
    "dasgd_gradient_average": (ctypes.c_int, [_vp, _vp, _vp]),
    "dasgd_average_now": (ctypes.c_int, [ctypes.c_int, _i64, _pp, ctypes.c_float, _vp, ctypes.c_size_t, _vp]),
    "dasgd_average_now_static": (ctypes.c_int, [ctypes.c_int, _i64, _pp, ctypes.c_float, _vp]),
    "dasgd_choose_delay": (ctypes.c_int, [ctypes.c_double, ctypes.c_double, _pint, _pint]),
    "dasgd_query": (ctypes.c_int, [_vp, _pi64, _pint, _pint, _pint]),
    "dasgd_layout": (ctypes.c_int, [_vp, _pi64, _pi64, _pint]),
    "dasgd_pending_average": (ctypes.c_int, [_vp, ctypes.c_int, _pi64, ctypes.POINTER(ctypes.c_size_t)]),
    "dasgd_profile": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int]),
    "dasgd_profile_read": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double), _pi64, _pi64]),
    "dasgd_set_band": (ctypes.c_int, [_vp, ctypes.c_int]),
    "dasgd_band": (ctypes.c_int, [_vp, ctypes.c_int, _pint, _pint, _pint]),
    "dasgd_device_extent": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_size_t)]),
    "dasgd_check_work_map": (ctypes.c_int, [ctypes.c_int, _i64, ctypes.c_int, ctypes.c_int]),
    "dasgd_schedule_in_use": (ctypes.c_int, [_vp, _pint, _pint, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]),
    "dasgd_set_side_stream_head_start": (ctypes.c_int, [_vp, ctypes.c_uint]),
    "dasgd_schedule_trial": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_float)]),
    "dasgd_last_hip_error": (ctypes.c_int, [_vp]),
    "dasgd_destroy": (None, [_vp]),
}

_LIB: Optional[ctypes.CDLL] = None


class DasgdError(RuntimeError):
    def __init__(self, call: str, code: int, hip: int = 0):
        self.call, self.code, self.hip = call, code, hip
        msg = f"{call} failed: {_ERR.get(code, code)}"
        if code == DASGD_EHIP:
            msg += f" [hipError {hip}]"
        super().__init__(msg)


def library_path() -> str:
    return _build.LIB


def lib() -> ctypes.CDLL:
    """Load libdasgd.so (what is built in-tree; built here if nothing is, rebuilt if a source is newer
    where a compiler is at hand -- a library older than its sources is never loaded silently)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if os.path.exists(path) and _build.stale():
        try:
            _build.hipcc()
        except RuntimeError:
            raise RuntimeError("libdasgd.so is older than its sources and there is no hipcc here to rebuild it; "
                               "run `python -c 'import __graft_entry__ as g; g.build()'` where there is one") from None
        _build.build()
    if not os.path.exists(path):
        try:
            _build.build()
        except Exception as e:  # no silent fallback: there is no other implementation
            raise RuntimeError(f"libdasgd.so is not built and could not be built here ({e}); "
                               "run `python -c 'import __graft_entry__ as g; g.build()'`") from e
    L = ctypes.CDLL(path)
    for name, (res, args) in EXPORTS.items():
        f = getattr(L, name)
        f.restype = res
        f.argtypes = args
    _LIB = L
    return L


def choose_delay(t_c: float, t_p: float) -> Tuple[int, int]:
    """(d, tau) by the paper's guideline (dasgd_choose_delay)."""
    d = ctypes.c_int(); tau = ctypes.c_int()
    rc = lib().dasgd_choose_delay(float(t_c), float(t_p), ctypes.byref(d), ctypes.byref(tau))
    if rc < 0:
        raise DasgdError("dasgd_choose_delay", rc)
    return int(d.value), int(tau.value)


def average_now(x_rows: Sequence[int], P: int, xi: float, workspace_ptr: int, workspace_bytes: int, stream: int) -> None:
    """x_j <- xi x_j + (1 - xi) mean_j x_j over the W rows of P floats at the device pointers x_rows
    (dasgd_average_now); the mean is left in the workspace."""
    rc = lib().dasgd_average_now(len(x_rows), int(P), _ptr_array(x_rows), float(xi), ctypes.c_void_p(int(workspace_ptr)),
                                 int(workspace_bytes), ctypes.c_void_p(int(stream)))
    if rc < 0:
        raise DasgdError("dasgd_average_now", rc, lib().dasgd_last_hip_error(None))


def average_now_static(x_rows: Sequence[int], P: int, xi: float, stream: int) -> None:
    """dasgd_average_now with the library's own static scratch array in place of a workspace
    (dasgd_average_now_static): allocates nothing."""
    rc = lib().dasgd_average_now_static(len(x_rows), int(P), _ptr_array(x_rows), float(xi), ctypes.c_void_p(int(stream)))
    if rc < 0:
        raise DasgdError("dasgd_average_now_static", rc, lib().dasgd_last_hip_error(None))


def device_extent(ptr: int) -> int:
    """Bytes from ptr to the end of the device allocation that holds it (dasgd_device_extent)."""
    n = ctypes.c_size_t()
    rc = lib().dasgd_device_extent(ctypes.c_void_p(int(ptr)), ctypes.byref(n))
    if rc < 0:
        raise DasgdError("dasgd_device_extent", rc)
    return int(n.value)


def check_work_map(kind: int, row4: int, head: int = 0, log_band: int = 0) -> int:
    """0 if the work map `kind` (MAP_*) covers a row of row4 128-bit columns exactly once
    (dasgd_check_work_map); 1..4 name the violated property; raises on arguments out of range."""
    rc = lib().dasgd_check_work_map(int(kind), int(row4), int(head), int(log_band))
    if rc < 0:
        raise DasgdError("dasgd_check_work_map", rc)
    return rc


def _ptr_array(ptrs: Sequence[int]):
    """Pointers as a C array of void*; an array made earlier (DaSGD.grad_pointers) is passed through."""
    if isinstance(ptrs, ctypes.Array):
        return ptrs
    return (ctypes.c_void_p * len(ptrs))(*[int(p) for p in ptrs])


class DaSGD:
    """One DaSGD context: W replicas of P fp32 parameters; see include/dasgd.h for semantics."""

    def __init__(self, W: int, P: int, d: int, tau: int, lr: float, momentum: float, wd: float,
                 xi: Optional[float] = None):
        self._lib = lib()
        self._h = self._lib.dasgd_create(int(W), int(P), int(d), int(tau), float(lr), float(momentum), float(wd))
        if not self._h:
            raise DasgdError("dasgd_create", DASGD_EINVAL)
        self.W, self.P, self.d, self.tau = int(W), int(P), int(d), int(tau)
        self.n_tensors = 0
        self._keep = []            # torch objects whose memory the library points into
        self._g_arr = None
        if xi is not None:
            self.set_xi(xi)

    # -- helpers -------------------------------------------------------------------------------
    def _check(self, call: str, rc: int) -> int:
        if rc < 0:
            raise DasgdError(call, rc, self._lib.dasgd_last_hip_error(self._h))
        return rc

    # -- one method per C call -------------------------------------------------------------------
    def set_xi(self, xi: float) -> None:
        self._check("dasgd_set_xi", self._lib.dasgd_set_xi(self._h, float(xi)))

    def set_lr(self, lr: float) -> None:
        self._check("dasgd_set_lr", self._lib.dasgd_set_lr(self._h, float(lr)))

    def set_schedule(self, schedule: int) -> None:
        self._check("dasgd_set_schedule", self._lib.dasgd_set_schedule(self._h, int(schedule)))

    def set_fusion(self, fusion: int) -> None:
        self._check("dasgd_set_fusion", self._lib.dasgd_set_fusion(self._h, int(fusion)))

    def set_snapshot(self, mode: int) -> None:
        self._check("dasgd_set_snapshot", self._lib.dasgd_set_snapshot(self._h, int(mode)))

    def workspace_bytes(self, numel: Sequence[int]) -> int:
        arr = (ctypes.c_int64 * len(numel))(*[int(n) for n in numel])
        return int(self._lib.dasgd_workspace_bytes(self._h, len(numel), arr))

    def bind(self, numel: Sequence[int], x_ptrs: Sequence[int], v_ptrs: Sequence[int],
             workspace_ptr: int, workspace_bytes: int, main_stream: int, side_stream: int) -> None:
        n = len(numel)
        arr = (ctypes.c_int64 * n)(*[int(z) for z in numel])
        if len(x_ptrs) != self.W * n or len(v_ptrs) != self.W * n:
            raise DasgdError("dasgd_bind", DASGD_EINVAL)
        self._check("dasgd_bind", self._lib.dasgd_bind(self._h, n, arr, _ptr_array(x_ptrs), _ptr_array(v_ptrs),
                                                       ctypes.c_void_p(int(workspace_ptr)), int(workspace_bytes),
                                                       ctypes.c_void_p(int(main_stream)), ctypes.c_void_p(int(side_stream))))
        self.n_tensors = n

    def bind_dry_run(self, numel: Sequence[int]) -> None:
        n = len(numel)
        arr = (ctypes.c_int64 * n)(*[int(z) for z in numel])
        self._check("dasgd_bind_dry_run", self._lib.dasgd_bind_dry_run(self._h, n, arr))
        self.n_tensors = n

    def local_step(self, g_ptrs: Optional[Sequence[int]] = None) -> None:
        """g_ptrs: W*n_tensors device pointers (replica-major) or None to re-use the last table."""
        if g_ptrs is None:
            arr = None
        else:
            if len(g_ptrs) != self.W * self.n_tensors:
                raise DasgdError("dasgd_local_step", DASGD_EINVAL)
            arr = _ptr_array(g_ptrs)
        self._check("dasgd_local_step", self._lib.dasgd_local_step(self._h, arr))

    def gradient_average(self, G_ptr: int, out_ptr: int) -> None:
        """out = mean over the W rows of the W x P gradient matrix at G_ptr (dasgd_gradient_average)."""
        self._check("dasgd_gradient_average",
                    self._lib.dasgd_gradient_average(self._h, ctypes.c_void_p(int(G_ptr)), ctypes.c_void_p(int(out_ptr))))

    def average_begin(self) -> None:
        self._check("dasgd_average_begin", self._lib.dasgd_average_begin(self._h))

    def merge(self) -> None:
        self._check("dasgd_merge", self._lib.dasgd_merge(self._h))

    def query(self) -> Tuple[int, int, bool, bool]:
        """(k, n_pending, begin_due, merge_due)"""
        k = ctypes.c_int64(); n = ctypes.c_int(); b = ctypes.c_int(); m = ctypes.c_int()
        self._check("dasgd_query", self._lib.dasgd_query(self._h, ctypes.byref(k), ctypes.byref(n),
                                                         ctypes.byref(b), ctypes.byref(m)))
        return int(k.value), int(n.value), bool(b.value), bool(m.value)

    def layout(self) -> Tuple[List[int], int]:
        """(flat offset of every tensor in a snapshot row / average, padded row length)"""
        off = (ctypes.c_int64 * max(self.n_tensors, 1))()
        pp = ctypes.c_int64()
        self._check("dasgd_layout", self._lib.dasgd_layout(self._h, off, ctypes.byref(pp), None))
        return [int(o) for o in off[: self.n_tensors]], int(pp.value)

    def addressing(self) -> int:
        """ADDR_RECORDS, ADDR_ROWS or ADDR_ROWS_XV (-1 for a dry run): how the kernels find the data."""
        a = ctypes.c_int()
        self._check("dasgd_layout", self._lib.dasgd_layout(self._h, None, None, ctypes.byref(a)))
        return int(a.value)

    def schedule_in_use(self) -> Tuple[int, bool, float, float]:
        """(schedule in force -- SCHED_AUTO while still measuring --, settled?, overlap ms, serial ms)"""
        sc = ctypes.c_int(); st = ctypes.c_int(); a = ctypes.c_double(); b = ctypes.c_double()
        self._check("dasgd_schedule_in_use", self._lib.dasgd_schedule_in_use(self._h, ctypes.byref(sc), ctypes.byref(st),
                                                                             ctypes.byref(a), ctypes.byref(b)))
        return int(sc.value), bool(st.value), float(a.value), float(b.value)

    def schedule_trial(self) -> Tuple[float, ...]:
        """ms of the six measured phases of SCHED_AUTO (overlap, serial, overlap, ...); zeros until settled"""
        ms = (ctypes.c_float * 6)()
        self._check("dasgd_schedule_trial", self._lib.dasgd_schedule_trial(self._h, ms))
        return tuple(float(v) for v in ms)

    def pending_average(self, which: int = 0) -> Tuple[int, int]:
        """(launch step, byte offset into the workspace) of pending average `which` (0 = oldest)"""
        ls = ctypes.c_int64(); bo = ctypes.c_size_t()
        self._check("dasgd_pending_average",
                    self._lib.dasgd_pending_average(self._h, int(which), ctypes.byref(ls), ctypes.byref(bo)))
        return int(ls.value), int(bo.value)

    def profile(self, every_n: int, max_records: int = 4096) -> None:
        """Time one launch in every_n of each kernel kind (0 = off)."""
        self._check("dasgd_profile", self._lib.dasgd_profile(self._h, int(every_n), int(max_records)))

    def profile_read(self, kernel: int) -> Tuple[float, int, int]:
        """(milliseconds summed over the timed launches, timed launches, all launches) of one kernel
        since profiling was enabled / last read; blocks until both streams have drained."""
        ms = ctypes.c_double(); n = ctypes.c_int64(); m = ctypes.c_int64()
        self._check("dasgd_profile_read", self._lib.dasgd_profile_read(self._h, int(kernel), ctypes.byref(ms),
                                                                       ctypes.byref(n), ctypes.byref(m)))
        return float(ms.value), int(n.value), int(m.value)

    def set_side_stream_threshold(self, nbytes: int) -> None:
        """Means smaller than this stay on the main stream even in the overlap schedules (0: none do)."""
        self._check("dasgd_set_side_stream_threshold", self._lib.dasgd_set_side_stream_threshold(self._h, int(nbytes)))

    def set_side_stream_head_start(self, microseconds: int) -> None:
        """Hold a side-stream mean back by this long so that the caller's next kernel is dispatched first (0: not)."""
        self._check("dasgd_set_side_stream_head_start",
                    self._lib.dasgd_set_side_stream_head_start(self._h, int(microseconds)))

    def set_band(self, log_band: int) -> None:
        """-1: measure the band length in place (default); 0..11: fix it."""
        self._check("dasgd_set_band", self._lib.dasgd_set_band(self._h, int(log_band)))

    def band(self, kernel: int) -> Tuple[int, bool]:
        """(log2 of the band length in use for `kernel`, -1 while still being measured; settled?)"""
        lb, st, _ = self.band_state(kernel)
        return lb, st

    def band_state(self, kernel: int) -> Tuple[int, bool, int]:
        """(log2 band length or -1, settled?, timed trial launches issued so far)"""
        lb = ctypes.c_int(); st = ctypes.c_int(); tr = ctypes.c_int()
        self._check("dasgd_band", self._lib.dasgd_band(self._h, int(kernel), ctypes.byref(lb), ctypes.byref(st),
                                                       ctypes.byref(tr)))
        return int(lb.value), bool(st.value), int(tr.value)

    def bands_in_flux(self) -> bool:
        """True while a band measurement has started and not finished (never blocks)."""
        return any(tr > 0 and not st for _, st, tr in (self.band_state(k) for k in KERNEL_NAMES))

    def destroy(self) -> None:
        if getattr(self, "_h", None):
            self._lib.dasgd_destroy(self._h)
            self._h = None
            self._keep = []

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def step(self, g_ptrs: Optional[Sequence[int]] = None) -> Tuple[bool, bool]:
        """One whole iteration (dasgd_step): local_step, then average_begin / merge when due.
        Returns (began, merged)."""
        if g_ptrs is None:
            arr = None
        else:
            if len(g_ptrs) != self.W * self.n_tensors:
                raise DasgdError("dasgd_step", DASGD_EINVAL)
            arr = _ptr_array(g_ptrs)
        b = ctypes.c_int(); m = ctypes.c_int()
        self._check("dasgd_step", self._lib.dasgd_step(self._h, arr, ctypes.byref(b), ctypes.byref(m)))
        return bool(b.value), bool(m.value)

    # -- torch marshalling -------------------------------------------------------------------------
    def bind_tensors(self, x: Sequence[Sequence["torch.Tensor"]], v: Sequence[Sequence["torch.Tensor"]],
                     main_stream: "torch.cuda.Stream", side_stream: "torch.cuda.Stream") -> "torch.Tensor":
        """x[j][t], v[j][t]: fp32 contiguous device tensors of replica j.  Allocates the workspace
        with torch and returns it (a uint8 tensor the caller may inspect but must not free)."""
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("dasgd: no GPU visible; there is no CPU implementation of this path")
        assert len(x) == self.W and len(v) == self.W
        numel = [int(t.numel()) for t in x[0]]
        for rows in (x, v):
            for rep in rows:
                assert [int(t.numel()) for t in rep] == numel
                for t in rep:
                    assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
        nbytes = self.workspace_bytes(numel)
        if nbytes == 0:
            raise DasgdError("dasgd_workspace_bytes", DASGD_EINVAL)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=x[0][0].device)
        self.bind(numel, [t.data_ptr() for rep in x for t in rep], [t.data_ptr() for rep in v for t in rep],
                  ws.data_ptr(), nbytes, main_stream.cuda_stream, side_stream.cuda_stream)
        self._keep = [x, v, ws, main_stream, side_stream]
        return ws

    @staticmethod
    def replica_matrix(W: int, numel: Sequence[int], device="cuda:0", row_align: int = 256):
        """Storage in the layout the row kernels take (see dasgd_local_step): one zero-filled W x ld
        fp32 matrix, ld = sum(numel) rounded up to row_align floats (256 floats = 1 KiB: rows that start
        on kilobyte boundaries are the fastest; any stride works), and the per-tensor views
        views[j][t] into row j.  Allocate one for the weights, one for the momentum buffers and one for
        the gradients; the views are what a model uses as its parameters / gradient buffers.
        Returns (matrix, views)."""
        import torch
        if row_align < 4 or row_align > 4096 or row_align % 4:
            raise ValueError("row_align must be a multiple of 4 floats, at most 4096")
        P = int(sum(int(n) for n in numel))
        ld = (P + row_align - 1) // row_align * row_align
        m = torch.zeros(int(W), ld, dtype=torch.float32, device=device)
        off = [0]
        for n in numel:
            off.append(off[-1] + int(n))
        views = [[m[j, off[t]:off[t + 1]] for t in range(len(numel))] for j in range(int(W))]
        return m, views

    @staticmethod
    def grad_pointers(g: Sequence[Sequence["torch.Tensor"]]):
        """The gradient table of local_step/step, marshalled once: W*n_tensors device pointers,
        replica-major, as a C array that can be passed at every step without being rebuilt."""
        return _ptr_array([t.data_ptr() for rep in g for t in rep])
