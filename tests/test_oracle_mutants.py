"""Planted mistakes in copies of the CPU oracle must each be caught by at least one pin.

The oracle's C source is altered textually (one mistake per copy), compiled to a temporary
library and run through the same checks as the real oracle.  This shows the pins are strong
enough that a dropped term, a wrong sign, index or trigger, or a transposed operand fails.
Everything here runs on the host.
"""
import os
import re

import pytest

import oracle
from oracle import build as obuild
from oracle_pins import ALL_CHECKS

HERE = os.path.dirname(os.path.abspath(obuild.__file__))


def _swap_launch_and_merge(src: str) -> str:
    """Move the 'launch the average' block after the 'merge' block inside the step function."""
    a = src.index("    if ((k + 1) % o->tau == 0) {")
    b = src.index("    if (o->count > 0 && o->fifo[o->head].launch_step == k - o->d) {")
    c = src.index("    o->k = k + 1;")
    return src[:a] + src[b:c] + src[a:b] + src[c:]


MUTANTS = {
    "drop_weight_decay": ("REAL gp = g[e] + wd * x[e];", "REAL gp = g[e];"),
    "lr_inside_buffer": ("REAL vn = momentum * v[e] + gp;\n        v[e] = vn;\n        x[e] = x[e] - lr * vn;",
                         "REAL vn = momentum * v[e] + lr * gp;\n        v[e] = vn;\n        x[e] = x[e] - vn;"),
    "ascent_sign": ("x[e] = x[e] - lr * vn;", "x[e] = x[e] + lr * vn;"),
    "dampened_momentum": ("REAL vn = momentum * v[e] + gp;", "REAL vn = momentum * (v[e] + gp);"),
    "decay_on_buffer": ("REAL gp = g[e] + wd * x[e];", "REAL gp = g[e] + wd * v[e];"),
    "merge_weights_swapped": ("x[e] = xi * x[e] + om * A[i];", "x[e] = om * x[e] + xi * A[i];"),
    "merge_transposed_index": ("int64_t e = (int64_t)j * P + i;\n            x[e] = xi",
                               "int64_t e = (int64_t)i * W + j;\n            x[e] = xi"),
    "merge_one_step_early": ("launch_step == k - o->d) {", "launch_step == k - o->d + 1) {"),
    "launch_off_by_one": ("if ((k + 1) % o->tau == 0) {", "if (k % o->tau == 0) {"),
    "mean_not_divided": ("REAL inv = (REAL)1 / (REAL)W;", "REAL inv = (REAL)1;"),
    "mean_skips_last": ("A[i] = NAME(pairwise_sum)(y, P, i, 0, W) * inv;",
                        "A[i] = NAME(pairwise_sum)(y, P, i, 0, W > 1 ? W - 1 : W) * inv;"),
    "mean_transposed_index": ("if (hi - lo == 1) return y[(int64_t)lo * P + i];",
                              "if (hi - lo == 1) return y[(int64_t)lo + i * 0 + (i % P)];"),
    "merge_one_step_late": ("launch_step == k - o->d) {", "launch_step == k - o->d - 1) {"),
    "merge_newest_not_oldest": ("NAME(dasgd_oracle_merge)(o->W, o->P, o->xi, o->x, o->fifo[o->head].A);",
                                "NAME(dasgd_oracle_merge)(o->W, o->P, o->xi, o->x, "
                                "o->fifo[(o->head + o->count - 1) % o->cap].A);"),
    "merge_is_convex_in_xi_only": ("REAL om = (REAL)1 - xi;\n    #pragma omp parallel for schedule(static)\n"
                                   "    for (int64_t i = 0; i < P; ++i)\n        for (int j = 0; j < W; ++j) {",
                                   "REAL om = (REAL)1;\n    #pragma omp parallel for schedule(static)\n"
                                   "    for (int64_t i = 0; i < P; ++i)\n        for (int j = 0; j < W; ++j) {"),
    "mean_of_first_replica_only": ("A[i] = NAME(pairwise_sum)(y, P, i, 0, W) * inv;",
                                   "A[i] = y[i] + (NAME(pairwise_sum)(y, P, i, 0, W) * inv) * (REAL)0;"),
    "average_after_merge": _swap_launch_and_merge,
    "momentum_reset_at_merge": ("        o->head = (o->head + 1) % o->cap;",
                                "        memset(o->v, 0, sizeof(REAL) * (size_t)o->W * (size_t)o->P);\n"
                                "        o->head = (o->head + 1) % o->cap;"),
}


def _mutate(name: str, tmp_path) -> str:
    impl = open(os.path.join(HERE, "dasgd_oracle_impl.h")).read()
    m = MUTANTS[name]
    if callable(m):
        out = m(impl)
    else:
        old, new = m
        assert impl.count(old) == 1, f"mutation anchor for {name} not found exactly once"
        out = impl.replace(old, new)
    assert out != impl
    d = tmp_path / name
    d.mkdir()
    (d / "dasgd_oracle_impl.h").write_text(out)
    main = open(os.path.join(HERE, "dasgd_oracle.c")).read()
    (d / "dasgd_oracle.c").write_text(main)
    lib_path = str(d / "libmutant.so")
    import subprocess
    subprocess.run(["gcc", *obuild.FLAGS, "-I", str(d), "-o", lib_path, str(d / "dasgd_oracle.c")], check=True)
    return lib_path


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path):
    lib = oracle.load(_mutate(name, tmp_path))
    caught = []
    for check in ALL_CHECKS:
        try:
            check(lib)
        except (AssertionError, RuntimeError, ValueError):
            caught.append(check.__name__)
    assert caught, f"no pin noticed the planted mistake '{name}'"
    print(name, "caught by", caught)
