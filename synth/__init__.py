"""Seeded synthetic inputs (model shapes, weights, clean/corrupt token batches).

This package is the only code shared by the CPU oracle and the HIP path. It
holds no arithmetic of the method itself: it draws random numbers and lays
them out in the array layouts that both sides accept.
"""
from .workloads import (CONFIGS, ModelShape, make_shape, make_weights,
                        make_tokens, make_answers, make_receiver_sample, make_workload)

__all__ = ["CONFIGS", "ModelShape", "make_shape", "make_weights",
           "make_tokens", "make_answers", "make_receiver_sample", "make_workload"]
