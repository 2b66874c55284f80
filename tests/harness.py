"""Drivers that run one configuration through the GPU library and through the CPU oracle on the
same seeded inputs, and the error measure both are compared with.

Nothing here does DaSGD arithmetic: the GPU driver only allocates memory, generates inputs and
calls the library; the oracle driver only generates the same inputs and calls the oracle.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np
import torch

import workloads as wl
from workloads.configs import Config

TOL = 1e-5      # bound on |x_gpu - x_oracle| / parameter scale, per tensor, whole run (fp32 path)


# ------------------------------------------------------------------------------------------------
# GPU side
class DeviceRun:
    """Device state of one configuration bound to a library context.

    layout "arena": x, v, g each one W x P allocation, rows back to back; tensors are views at the
    unpadded offsets (so odd-sized tensors make their successors 16-byte misaligned).
    layout "arena_padded": the same with the row stride rounded up to a multiple of 32 floats
    (plus 32 when it already is one, so that there is always padding), padding poisoned with NaN.
    layout "matrix": what the benchmark allocates: W x ld with ld a multiple of 256 floats (rows on kilobyte
    boundaries), zero padding.
    layout "separate": every tensor is its own allocation.
    layout "rows": one allocation per replica and quantity, the tensors back to back inside it; every
    row starts a different number of 16-byte units behind a kilobyte boundary (and x, v, g differently).
    layout "rows_g_separate": weights and momentum as in "rows", every gradient tensor its own allocation.
    """

    def __init__(self, cfg: Config, layout: str = "arena", schedule: Optional[int] = None,
                 device: str = "cuda:0", xi: Optional[float] = None, fusion: Optional[int] = None,
                 snapshot: Optional[int] = None, side_threshold: Optional[int] = 0):
        """side_threshold: bytes below which the library keeps the mean on the main stream; 0 (the
        default HERE, not the library's) sends every mean to the side stream so that small test
        problems exercise the two-stream path; None leaves the library's default."""
        import paper_2006_00441_amd as pkg
        self.pkg = pkg
        self.cfg = cfg
        self.dev = torch.device(device)
        self.main = torch.cuda.Stream(self.dev)
        self.side = torch.cuda.Stream(self.dev)
        W, P = cfg.W, cfg.P
        off = cfg.params.offsets
        n = cfg.params.n_tensors
        with torch.cuda.stream(self.main):
            w0 = wl.init_weights(cfg, self.dev)
            if layout in ("arena", "arena_padded", "matrix"):
                ld = P if layout == "arena" else (P + 31) // 32 * 32 + (28 if P % 32 == 0 else 0)
                if layout == "matrix":
                    ld = (P + 255) // 256 * 256
                full = [torch.full((W, ld), float("nan"), device=self.dev) for _ in range(3)]
                self.full = full                   # (the padding must come back untouched)
                self.x_flat, self.v_flat, self.g_flat = (a[:, :P] for a in full)
                self.x_flat.copy_(w0.unsqueeze(0).expand(W, P))
                self.v_flat.zero_()
                self.g_flat.zero_()
                view = lambda a: [[a[j, off[t]:off[t + 1]] for t in range(n)] for j in range(W)]
                self.x, self.v, self.g = view(self.x_flat), view(self.v_flat), view(self.g_flat)
            elif layout in ("rows", "rows_g_separate"):
                def rows(skew):                    # W separate buffers; row j starts 4*(skew + 3j) floats into its own
                    bufs = [torch.full((P + 4 * (skew + 3 * j) + 8,), float("nan"), device=self.dev) for j in range(W)]
                    return bufs, [b[4 * (skew + 3 * j): 4 * (skew + 3 * j) + P] for j, b in enumerate(bufs)]
                self.full, rx = rows(1)
                fv, rv = rows(5)
                fg, rg = rows(2)
                self.full = self.full + fv + fg
                for j in range(W):
                    rx[j].copy_(w0); rv[j].zero_(); rg[j].zero_()
                self.x_flat = self.v_flat = self.g_flat = None
                self.x_rows, self.v_rows, self.g_rows = rx, rv, rg
                view = lambda r: [[r[j][off[t]:off[t + 1]] for t in range(n)] for j in range(W)]
                self.x, self.v, self.g = view(rx), view(rv), view(rg)
                if layout == "rows_g_separate":
                    self.g_rows = None
                    self.g = [[torch.zeros(off[t + 1] - off[t], device=self.dev) for t in range(n)] for _ in range(W)]
            elif layout == "separate":
                self.x_flat = self.v_flat = self.g_flat = None
                self.x = [[w0[off[t]:off[t + 1]].clone() for t in range(n)] for _ in range(W)]
                self.v = [[torch.zeros(off[t + 1] - off[t], device=self.dev) for t in range(n)] for _ in range(W)]
                self.g = [[torch.zeros(off[t + 1] - off[t], device=self.dev) for t in range(n)] for _ in range(W)]
            else:
                raise ValueError(layout)
            self.sigma = wl.grad_sigma_vector(cfg, self.dev) if cfg.kind == "external" else None
            self.quad = wl.QuadraticProblem.build(cfg, self.dev) if cfg.kind == "quadratic" else None
        self.main.synchronize()
        self.opt = pkg.DaSGD(W, P, cfg.d, cfg.tau, cfg.lr, cfg.momentum, cfg.wd, xi=cfg.xi if xi is None else xi)
        self.ws = self.opt.bind_tensors(self.x, self.v, self.main, self.side)
        if side_threshold is not None:
            self.opt.set_side_stream_threshold(side_threshold)
        if schedule is not None:
            self.opt.set_schedule(schedule)
        if fusion is not None:
            self.opt.set_fusion(fusion)
        if snapshot is not None:
            self.opt.set_snapshot(snapshot)
        self.g_ptrs = pkg.DaSGD.grad_pointers(self.g)
        self.k = 0

    # inputs ------------------------------------------------------------------------------------
    def _flat(self, rows: Sequence[Sequence[torch.Tensor]], j: int) -> torch.Tensor:
        return torch.cat([t.reshape(-1) for t in rows[j]])

    def x_of(self, j: int) -> torch.Tensor:
        if self.x_flat is not None:
            return self.x_flat[j]
        if getattr(self, "x_rows", None) is not None:
            return self.x_rows[j]
        return self._flat(self.x, j)

    def padding_untouched(self) -> bool:
        """Everything the harness allocated around the rows (poisoned with NaN) is still NaN."""
        self.main.synchronize(); self.side.synchronize()
        P, W = self.cfg.P, self.cfg.W
        full = getattr(self, "full", None)
        if full is None:
            return True
        if full[0].dim() == 2:
            return all(bool(torch.isnan(a[:, P:]).all()) for a in full)
        ok = True
        for q, skew in enumerate((1, 5, 2)):
            for j in range(W):
                b, lo = full[q * W + j], 4 * (skew + 3 * j)
                ok = ok and bool(torch.isnan(b[:lo]).all()) and bool(torch.isnan(b[lo + P:]).all())
        return ok

    def fill_gradients(self, k: int) -> None:
        """Write the gradients of iteration k into the g buffers (on the main stream)."""
        cfg = self.cfg
        with torch.cuda.stream(self.main):
            for j in range(cfg.W):
                if cfg.kind == "quadratic":
                    gj = self.quad.grad(self.x_of(j), k, j)
                else:
                    gj = wl.gradient(cfg, k, j, self.dev, sigma=self.sigma,
                                     out=self.g_flat[j] if self.g_flat is not None else None)
                if self.g_flat is not None:
                    if gj.data_ptr() != self.g_flat[j].data_ptr():
                        self.g_flat[j].copy_(gj)
                elif getattr(self, "g_rows", None) is not None:
                    self.g_rows[j].copy_(gj)
                else:
                    off = cfg.params.offsets
                    for t, dst in enumerate(self.g[j]):
                        dst.copy_(gj[off[t]:off[t + 1]])

    # stepping ----------------------------------------------------------------------------------
    def step(self) -> None:
        self.fill_gradients(self.k)
        self.opt.step(self.g_ptrs)
        self.k += 1

    def weights(self, idx: Optional[torch.Tensor] = None) -> np.ndarray:
        """Current weights [W, P] (or [W, len(idx)]) on the host, after draining both streams."""
        self.main.synchronize(); self.side.synchronize()
        rows = [self.x_of(j) if idx is None else self.x_of(j)[idx.to(self.dev)] for j in range(self.cfg.W)]
        return torch.stack(rows).cpu().numpy()

    def momentum(self) -> np.ndarray:
        self.main.synchronize()
        rows = [self.v_flat[j] if self.v_flat is not None else self._flat(self.v, j) for j in range(self.cfg.W)]   # (views: cat copies)
        return torch.stack(rows).cpu().numpy()

    def pending_average(self, which: int = 0) -> np.ndarray:
        """Pending average `which` as an unpadded [P] host vector."""
        self.main.synchronize(); self.side.synchronize()
        _, byte_off = self.opt.pending_average(which)
        foff, ppad = self.opt.layout()
        row = self.ws[byte_off: byte_off + 4 * ppad].view(torch.float32)
        numel = self.cfg.params.numel
        return torch.cat([row[foff[t]: foff[t] + numel[t]] for t in range(len(numel))]).cpu().numpy()

    def close(self) -> None:
        self.opt.destroy()


def run_gpu(cfg: Config, steps: Optional[int] = None, layout: str = "arena", schedule: Optional[int] = None,
            observer: Optional[Callable[[int, DeviceRun], None]] = None, idx: Optional[torch.Tensor] = None,
            xi: Optional[float] = None, fusion: Optional[int] = None, snapshot: Optional[int] = None) -> np.ndarray:
    """Run cfg on the GPU through the C ABI; returns the final weights [W, P] (or at idx)."""
    run = DeviceRun(cfg, layout=layout, schedule=schedule, xi=xi, fusion=fusion, snapshot=snapshot)
    try:
        for k in range(cfg.steps if steps is None else steps):
            run.step()
            if observer is not None:
                observer(k, run)
        return run.weights(idx)
    finally:
        run.close()


# ------------------------------------------------------------------------------------------------
# oracle side
def run_oracle(cfg: Config, dtype: str = "f64", steps: Optional[int] = None, idx: Optional[torch.Tensor] = None,
               observer: Optional[Callable] = None, xi: Optional[float] = None, gen_device: Optional[str] = None) -> np.ndarray:
    """Run cfg through the CPU oracle (on all coordinates, or only on the coordinates idx: the
    method is elementwise across coordinates, so a subset evolves exactly as inside the full run).
    gen_device: evaluate the seeded input generator there (it gives the same bits on every device) and
    copy the inputs to the host; the oracle itself always runs on the host."""
    import oracle
    npdt = np.float32 if dtype == "f32" else np.float64
    w0 = wl.init_weights(cfg, "cpu", idx).numpy()
    P = w0.shape[0]
    o = oracle.Oracle(cfg.W, P, cfg.d, cfg.tau, cfg.lr, cfg.momentum, cfg.wd, w0,
                      xi=cfg.xi if xi is None else xi, dtype=dtype)
    sigma = wl.grad_sigma_vector(cfg, "cpu", idx) if cfg.kind == "external" else None
    quad = wl.QuadraticProblem.build(cfg, "cpu", idx) if cfg.kind == "quadratic" else None

    stage = None
    if gen_device is not None and quad is None:
        n = cfg.P if idx is None else idx.numel()
        idx_dev = None if idx is None else idx.to(gen_device)
        sigma_dev = wl.grad_sigma_vector(cfg, gen_device, idx_dev)
        stage = torch.empty((cfg.W, n), dtype=torch.float64 if dtype == "f64" else torch.float32,
                            pin_memory=torch.device(gen_device).type == "cuda")
        stage_dev = torch.empty((cfg.W, n), dtype=stage.dtype, device=gen_device)     # widened there, copied once

    def grads(k: int, x: np.ndarray) -> np.ndarray:
        if quad is not None:
            return np.stack([quad.grad(torch.from_numpy(x[j]), k, j, idx=idx).numpy() for j in range(cfg.W)])
        if stage is not None:
            for j in range(cfg.W):
                stage_dev[j].copy_(wl.gradient(cfg, k, j, gen_device, idx=idx_dev, sigma=sigma_dev))
            stage.copy_(stage_dev)
            return stage.numpy()
        return np.stack([wl.gradient(cfg, k, j, "cpu", idx=idx, sigma=sigma).numpy() for j in range(cfg.W)]).astype(npdt)

    out = o.run(cfg.steps if steps is None else steps, grads, observer).copy()
    o.close()
    return out


# ------------------------------------------------------------------------------------------------
def tensor_of_index(cfg: Config, idx: Optional[torch.Tensor]) -> np.ndarray:
    off = np.asarray(cfg.params.offsets[1:], dtype=np.int64)
    ii = np.arange(cfg.P, dtype=np.int64) if idx is None else idx.numpy().astype(np.int64)
    return np.searchsorted(off, ii, side="right")


def max_scaled_error(cfg: Config, x_test: np.ndarray, x_ref: np.ndarray, idx: Optional[torch.Tensor] = None) -> float:
    """max over tensors t of  max |x_test - x_ref| / scale_t  with scale_t = max(rms(x_ref_t),
    rms(w0_t), 1e-30), rms over all replicas (and over the sampled coordinates when idx is given)."""
    tens = tensor_of_index(cfg, idx)
    w0 = wl.init_weights(cfg, "cpu", idx).numpy().astype(np.float64)
    diff = np.abs(x_test.astype(np.float64) - x_ref.astype(np.float64)).max(axis=0)
    ref2 = (x_ref.astype(np.float64) ** 2).mean(axis=0)
    nt = cfg.params.n_tensors
    cnt = np.bincount(tens, minlength=nt).astype(np.float64)
    have = cnt > 0
    rms_ref = np.sqrt(np.bincount(tens, weights=ref2, minlength=nt)[have] / cnt[have])
    rms_w0 = np.sqrt(np.bincount(tens, weights=w0 ** 2, minlength=nt)[have] / cnt[have])
    scale = np.maximum(np.maximum(rms_ref, rms_w0), 1e-30)
    dmax = np.zeros(nt)
    np.maximum.at(dmax, tens, diff)
    return float((dmax[have] / scale).max())


def sample_indices(cfg: Config, per_tensor: int = 512, seed: int = 1234, chunk: int = 4096) -> torch.Tensor:
    """Coordinates for full-size checks: every element of tensors up to `chunk` elements; for larger
    tensors the first and last 8 elements, 4 elements on each side of a few chunk boundaries, and
    `per_tensor` random elements."""
    rng = np.random.default_rng(seed)
    off = cfg.params.offsets
    out: List[np.ndarray] = []
    for t, n in enumerate(cfg.params.numel):
        if n <= chunk:
            loc = np.arange(n)
        else:
            parts = [np.arange(8), np.arange(n - 8, n), rng.integers(0, n, per_tensor)]
            nb = (n - 1) // chunk
            for b in {1, nb, int(rng.integers(1, nb + 1))}:
                parts.append(np.arange(max(0, b * chunk - 4), min(n, b * chunk + 4)))
            loc = np.unique(np.concatenate(parts))
        out.append(loc + off[t])
    return torch.from_numpy(np.concatenate(out).astype(np.int64))
