"""The five benchmark workloads as records.

Each record fixes the parameter set, the number of replicas W (the paper's M, Section 3.3.1),
the averaging period tau, the delay d, the optimiser constants and the step count.
xi (the local update proportion of Eq. 2) is 0.25 everywhere: the only value the paper prints
(Section 4.3, parameter-study baseline).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

from .shapes import ParamSet, bert_large_param_set, flat_param_set, resnet50_param_set


@dataclass(frozen=True)
class Config:
    name: str
    params: ParamSet
    W: int
    tau: int
    d: int
    lr: float
    momentum: float
    wd: float
    steps: int
    seed: int = 0
    xi: float = 0.25
    kind: str = "external"      # "external": gradients are pure inputs; "quadratic": g depends on x
    init: str = "kaiming"       # "zero" | "kaiming" | "normal"
    init_std: float = 0.0       # for init == "normal"
    grad_std: float = 0.0       # absolute gradient std; 0 => relative to the tensor's init norm
    grad_rel: float = 0.0       # s_t = grad_rel * ||w_t||_2 / sqrt(n_t), norm taken at init

    @property
    def P(self) -> int:
        return self.params.P

    @property
    def slots(self) -> int:
        """Averages that can be in flight at once: floor(d / tau) + 1."""
        return self.d // self.tau + 1

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


def _build() -> Dict[str, Config]:
    rn = resnet50_param_set()
    bl = bert_large_param_set()
    return {
        "quadratic": Config("quadratic", flat_param_set(1 << 20, "quadratic"), W=4, tau=1, d=1,
                            lr=0.1, momentum=0.9, wd=1e-4, steps=20, seed=0,
                            kind="quadratic", init="zero", grad_std=0.01),
        "resnet50_w8": Config("resnet50_w8", rn, W=8, tau=1, d=2, lr=0.1, momentum=0.9, wd=1e-4,
                              steps=100, seed=0, init="kaiming", grad_rel=1e-3),
        "resnet50_w16": Config("resnet50_w16", rn, W=16, tau=4, d=2, lr=0.1, momentum=0.9, wd=1e-4,
                               steps=200, seed=0, init="kaiming", grad_rel=1e-3),
        "bert_large_w4": Config("bert_large_w4", bl, W=4, tau=1, d=4, lr=1e-3, momentum=0.9, wd=0.01,
                                steps=50, seed=0, init="normal", init_std=0.02, grad_std=1e-4),
        # overlap stress: same numbers as resnet50_w8; the GEMM stand-in lives in the benchmark.
        "overlap": Config("overlap", rn, W=8, tau=1, d=2, lr=0.1, momentum=0.9, wd=1e-4,
                          steps=50, seed=0, init="kaiming", grad_rel=1e-3),
    }


CONFIGS: Dict[str, Config] = _build()


def get_config(name: str) -> Config:
    return CONFIGS[name]
