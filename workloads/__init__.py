"""Seeded synthetic inputs and the five named workload descriptions.

This package is the only code shared by the CPU oracle's tests and the HIP path's
tests/bench.  It holds shapes, hyper-parameters and random *input data* only: none of
the method's arithmetic (no Philox, no PGPE, no policy forward, no task dynamics).
"""
from .configs import (CONFIGS, WorkloadConfig, mlp_param_count, convnet_param_count,  # noqa: F401
                      lstm_seq2seq_param_count)
from . import generators  # noqa: F401
