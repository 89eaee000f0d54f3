"""Seeded synthetic workloads: parameter-shape lists and gradient generators.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds only shapes and random-number draws; none of the
arithmetic of bucketed gradient synchronization (no bucket assignment, no
summation, no averaging) lives here.

The shape lists stand in for the two models the paper evaluates (ResNet50 and
BERT, Section 5, with random synthetic inputs): only the *parameter-list
shapes* matter to gradient synchronization, so the gradients themselves are
seeded Gaussians.
"""
from .shapes import (tiny_shapes, resnet50_shapes, bert_large_shapes, uniform_shapes,
                     numel_of, WORKLOAD_SHAPES)
from .grads import (DT_FP32, DT_FP16, DT_BF16, ESIZE, NP_STORAGE,
                    gaussian_grad, gaussian_replica, tag_grad, integer_grad,
                    linear_regression_problem, unused_param_set,
                    f32_to_storage_trunc)

__all__ = [
    "tiny_shapes", "resnet50_shapes", "bert_large_shapes", "uniform_shapes", "numel_of",
    "WORKLOAD_SHAPES", "DT_FP32", "DT_FP16", "DT_BF16", "ESIZE", "NP_STORAGE",
    "gaussian_grad", "gaussian_replica", "tag_grad", "integer_grad",
    "linear_regression_problem", "unused_param_set", "f32_to_storage_trunc",
]
