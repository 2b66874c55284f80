"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests.

This package holds parameter-set shapes, configuration records and a counter-based
random generator.  It contains none of the DaSGD arithmetic (no optimiser step, no
averaging, no merge): it only produces the numbers that both implementations are fed.
"""
from .shapes import ParamSet, resnet50_param_set, bert_large_param_set, flat_param_set
from .configs import Config, CONFIGS, get_config
from .gen import (stream_key, random_bits, uniform01, standard_normal, normal_like_flat,
                  QuadraticProblem, init_weights, grad_sigma_vector, gradient)

__all__ = [
    "ParamSet", "resnet50_param_set", "bert_large_param_set", "flat_param_set",
    "Config", "CONFIGS", "get_config",
    "stream_key", "random_bits", "uniform01", "standard_normal", "normal_like_flat",
    "QuadraticProblem", "init_weights", "grad_sigma_vector", "gradient",
]
