"""Seeded synthetic DiT-feature generators.

This package only *makes inputs*: random low-rank-plus-residual feature
matrices shaped like FLUX / HunyuanVideo hidden states.  It contains none of
the cache method's arithmetic (no projection, residual, EMA, forecast or basis
fit) and is the one piece of code that both the CPU oracle's tests and the
GPU tests / benchmark are allowed to share.
"""
from .features import Workload, WORKLOADS, FeatureStream, is_full_step, torch_dtype

__all__ = ["Workload", "WORKLOADS", "FeatureStream", "is_full_step", "torch_dtype"]
