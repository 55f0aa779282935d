"""Oracle of the GPU-partitioning and Attention Co-processing formulas.  TEST INFRASTRUCTURE ONLY.

Memory-Efficient Diffusion-VAE Decoupling, "Optimal GPU partitioning": with N
GPUs, T_denoise the time to denoise one prompt on one GPU and T_decode the time
to decode one latent on one GPU, the balance condition with the communication
term dropped gives

    N_decode = ceil( T_decode / (T_decode + T_denoise) * N ).

Attention Co-processing, "Performance Analysis" (Eq. 1-3): with t_L the time of
the linear projections and t_A of the attention kernel on the denoising GPUs,

    T_baseline = t_L + t_A
    T_coop     = t_L + t_A * N_denoise / (N_denoise + N_decode)
    S          = T_baseline / T_coop.

Head padding (same section, closing paragraph): if the head count H is not
divisible by N_denoise and only head-wise splitting is available, heads are
padded to the next multiple; the worked example there is H = 24 on 7 GPUs ->
28 heads, 4 per GPU, of which only 6 GPUs are needed.

Readings where the text is silent: the ceiling is evaluated in double precision
in the order written above; the result is clamped to [1, N-1] because both
groups need a GPU (the formula alone can return N when T_denoise is tiny); the
number of GPUs "effectively needed" is ceil(H / heads_per_gpu); a ragged split
(no padding) gives the first H mod n GPUs one head more than the others.

Pins (tests/test_oracle_planner.py): exact rational arithmetic away from ties,
T_decode = T_denoise -> ceil(N/2), monotonicity, S -> 1 for t_A -> 0 and
S -> N/N_denoise for t_L -> 0, the H = 24 / 7-GPU example of the paper
(tests/golden/head_padding_example.txt).
"""
from __future__ import annotations

import math


def n_decode(t_denoise: float, t_decode: float, N: int) -> int:
    assert N >= 2 and t_denoise > 0 and t_decode > 0
    raw = math.ceil(t_decode / (t_decode + t_denoise) * N)
    return min(max(raw, 1), N - 1)


def aco_times(t_L: float, t_A: float, n_denoise: int, n_decode_: int):
    """(T_baseline, T_coop, S) of Eq. 1-3."""
    assert n_denoise >= 1 and n_decode_ >= 0 and t_L >= 0 and t_A >= 0 and t_L + t_A > 0
    t_base = t_L + t_A
    t_coop = t_L + t_A * (n_denoise / (n_denoise + n_decode_))
    return t_base, t_coop, t_base / t_coop


def head_padding(H: int, n_denoise: int):
    """(padded head count, heads per GPU, GPUs effectively needed)."""
    assert H >= 1 and n_denoise >= 1
    per = -(-H // n_denoise)
    return per * n_denoise, per, -(-H // per)


def ragged_groups(H: int, n: int):
    """Head counts per GPU without padding: sizes differ by at most one, larger ones first."""
    assert H >= 0 and n >= 1
    base, extra = divmod(H, n)
    return [base + 1 if i < extra else base for i in range(n)]
