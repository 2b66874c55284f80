"""Every coordinate of every replica at full size: the benchmark configurations run through the GPU
library in the layout the benchmark times, and through the fp64 CPU oracle over ALL coordinates.

The method is elementwise across coordinates (Eq. 2 couples replicas, never coordinates), so the oracle
is streamed over contiguous coordinate slices, one test case per slice; its inputs come from the seeded
generator (evaluated on the GPU and copied to the host: it gives the same bits on every device, which
test_generator_is_bit_identical_on_host_and_device checks), never from the library.
Bar: max |x_gpu - x_oracle| <= 1e-5 * parameter scale per tensor, every replica, at every checkpoint.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from harness import TOL, DeviceRun, max_scaled_error, run_oracle

pytestmark = pytest.mark.gpu

SLICE = {"resnet50_w8": 1 << 23, "resnet50_w16": 1 << 23, "bert_large_w4": 1 << 25}
# configuration -> {layout: checkpoints}; None: {1, tau + d, K/2, K}.  "separate" = one allocation per tensor (the
# record-table kernels; resnet50_w16 is the configuration whose many small tensors are there to stress them),
# "rows" = one allocation per replica at odd offsets; the layouts of a configuration are compared with the same
# oracle pass.
CHECKPOINTS = {"resnet50_w8": {"matrix": None, "rows": "final"}, "resnet50_w16": {"matrix": None, "separate": "final"},
               "bert_large_w4": {"matrix": "final", "separate": "final"}}


def cases():
    out = []
    for name, n in SLICE.items():
        P = wl.get_config(name).P
        out += [(name, lo) for lo in range(0, P, n)]
    return out


_gpu = {}       # name -> {layout: {step: weights [W, P] on the host}}; one configuration at a time


def gpu_checkpoints(name):
    if name not in _gpu:
        _gpu.clear()
        cfg = wl.get_config(name)
        _gpu[name] = {}
        for layout, which in CHECKPOINTS[name].items():
            cps = [cfg.steps] if which == "final" else sorted({1, cfg.tau + cfg.d, cfg.steps // 2, cfg.steps})
            run = DeviceRun(cfg, layout=layout, side_threshold=None)       # the library's defaults, as the benchmark runs it
            snaps = {}
            for k in range(cfg.steps):
                run.step()
                if k + 1 in cps:
                    snaps[k + 1] = run.weights()
            assert run.padding_untouched()
            run.close()
            del run
            torch.cuda.empty_cache()
            _gpu[name][layout] = snaps
    return _gpu[name]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,lo", cases())
def test_all_coordinates_at_full_size(name, lo):
    cfg = wl.get_config(name)
    by_layout = gpu_checkpoints(name)
    hi = min(cfg.P, lo + SLICE[name])
    idx = torch.arange(lo, hi, dtype=torch.int64)
    errs = {layout: {} for layout in by_layout}

    def obs(k, o, what):
        for layout, snaps in by_layout.items():
            if k + 1 in snaps:
                errs[layout][k + 1] = max_scaled_error(cfg, snaps[k + 1][:, lo:hi], o.x, idx)

    run_oracle(cfg, "f64", idx=idx, observer=obs, gen_device="cuda:0")
    for layout, e in errs.items():
        print(f"[{name}, {layout}] coordinates {lo}..{hi}: scaled error " + ", ".join(f"step {k}: {v:.2e}" for k, v in e.items()), flush=True)
        assert sorted(e) == sorted(by_layout[layout]) and max(e.values()) <= TOL
    if hi == cfg.P:
        _gpu.clear()
