"""The entry point that allocates nothing (dasgd_average_now_static) against dasgd_average_now: same
kernels, the average in the library's static scratch array instead of a caller's workspace.  Two calls
in a row, the second on a smaller input (the scratch array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def rows_of(W, P, seed, dev):
    bufs = [torch.full((P + 64,), float("nan"), device=dev) for _ in range(W)]
    rows = [b[4 * (j % 5): 4 * (j % 5) + P] for j, b in enumerate(bufs)]
    for j in range(W):
        rows[j].copy_(wl.normal_like_flat(wl.stream_key(seed, j), P, dev) * (1.0 + 0.02 * j))
    return bufs, rows


def test_static_scratch_entry_point_matches_the_workspace_one():
    import oracle
    import paper_2006_00441_amd as pkg
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream(dev)
    for W, P, xi, seed in ((8, 4096 * 17 + 360, 0.25, 5), (4, 1028, 0.5, 6)):        # several blocks and a ragged tail; then smaller
        keep_a, a = rows_of(W, P, seed, dev)
        keep_b, b = rows_of(W, P, seed, dev)
        x0 = torch.stack(a).cpu().numpy()
        ws = torch.empty(P, device=dev)
        torch.cuda.synchronize()
        pkg.average_now_static([r.data_ptr() for r in a], P, xi, stream.cuda_stream)
        pkg.average_now([r.data_ptr() for r in b], P, xi, ws.data_ptr(), 4 * P, stream.cuda_stream)
        stream.synchronize()
        got, ref = torch.stack(a).cpu().numpy(), torch.stack(b).cpu().numpy()
        assert np.array_equal(got, ref), (W, P)
        want = x0.astype(np.float64)
        oracle.merge(want, oracle.mean(np.ascontiguousarray(want)), xi)
        scale = np.sqrt((want ** 2).mean())
        assert np.abs(got - want).max() <= 2e-6 * scale
        for j, buf in enumerate(keep_a):                                  # nothing outside the rows was written
            lo = 4 * (j % 5)
            assert bool(torch.isnan(buf[:lo]).all()) and bool(torch.isnan(buf[lo + P:]).all())
    # larger than the scratch array: refused before anything is touched
    with pytest.raises(pkg.DasgdError) as e:
        pkg.average_now_static([r.data_ptr() for r in a], (32 << 20) + 4, 0.25, stream.cuda_stream)
    assert e.value.code == pkg.DASGD_ENOMEM
