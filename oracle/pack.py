"""Oracle of the pre-attention pack.  TEST INFRASTRUCTURE ONLY.

The step before the attention call: the Q, K, V projections of a DiT block come
out token-major, [B, S, H, d] (one row of H*d features per token), while
Algorithm 1 takes head-major tensors (Q in R^{B x h x S x D}, sliced as
Q[:, j, :, :]).  The pack moves every d-vector to its head-major place and
rounds it to bf16; with unit_rms it first divides the vector by its own root
mean square (the per-head query/key normalisation of the synthetic workloads:
no mean subtraction, no gain, no epsilon).  A zero vector stays zero.

    y[b, h, s, :] = bf16( premul * x[b, s, h, :] / sqrt(mean_c x[b, s, h, c]^2) )

premul (default 1) lets the producer of Q fold the softmax scale, times log2(e), into Q before
the one rounding, so that the attention kernel can take the scores as exponents of 2.

Evaluated in fp64 and rounded ONCE to bf16 (nearest, ties to even).  The kernel
works in fp32, so a result that lies within fp32 rounding of a bf16 rounding
boundary may land on the neighbouring bf16 value; tests bound how often.

Pins (tests/test_oracle_pack.py): the rounding against an independent bit-level
fp32->bf16 routine on fp32 inputs; placement with self-describing tensors; unit
RMS of the result; exact invariance under power-of-two rescaling; zero vectors.
"""
from __future__ import annotations

import numpy as np


def round_to_bf16(y: np.ndarray) -> np.ndarray:
    """Nearest bf16 (8 significant bits, ties to even) of fp64 values of normal magnitude, as fp64."""
    m, e = np.frexp(np.asarray(y, dtype=np.float64))      # y = m * 2^e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)        # rint rounds half to even


def pack_heads(x: np.ndarray, unit_rms: bool, premul: float = 1.0) -> np.ndarray:
    """x [B,S,H,d] (any float dtype) -> bf16 values as fp64, [B,H,S,d]; premul multiplies before the rounding."""
    x = np.asarray(x, dtype=np.float64)
    if unit_rms:
        rms = np.sqrt(np.mean(x * x, axis=-1, keepdims=True))
        x = np.divide(x, rms, out=np.zeros_like(x), where=rms > 0)
    x = x * float(premul)
    return round_to_bf16(np.ascontiguousarray(x.transpose(0, 2, 1, 3)))
