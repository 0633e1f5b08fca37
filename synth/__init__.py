"""Seeded synthetic inputs (features, predictor parameters, weight matrices).

Shared by the CPU checker's tests and the GPU library's tests and benchmark;
contains no part of either implementation.
"""
from . import rng
from .workloads import (CONFIGS, INFEASIBLE, RoundConfig, device_masked_matrix, fit_memory_scale, gpu_types, mixture_features,
                        permutation, planted_matrix, predictor_params, rank_one_matrix,
                        scheduling_round, threshold_matrix, typed_predictors, uniform_features, with_sm_input, with_slowdown_unit,
                        uniform_matrix)
