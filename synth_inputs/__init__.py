"""Seeded synthetic inputs (model shapes, weights, token prefixes) shared by the CPU oracle's
tests and the GPU path's tests / benchmark.

This package holds no arithmetic of the method: it only names the workload shapes, draws
random numbers from seeded numpy generators and rounds values to the storage type.
It imports neither the oracle nor the HIP binding.
"""
from .configs import MODEL_SHAPES, WORKLOADS, model_shape, workload          # noqa: F401
from .gen import (round_to_bf16, bf16_bits, make_weights, make_prefix,       # noqa: F401
                  make_probs, weight_names, correlated_draft_weights)
