"""Seeded synthetic inputs for the attention hot path.

This package holds input generation and workload shapes only: none of the
method's arithmetic (no scores, softmax, merge) lives here.  Both the CPU
oracle's tests and the HIP path's tests draw their tensors from it so that the
two sides see bit-identical bf16 payloads.
"""
from .inputs import (gen_tensor, gen_qkv, gen_qkv_parallel, to_dev_bf16, bf16_bits_to_f32, f32_to_bf16_bits,  # noqa: F401
                     Q_ID, K_ID, V_ID)
from .configs import CONFIGS, Workload, get_config  # noqa: F401
