"""Oracle of PipeSP's hand-off layouts and post-processing.  TEST INFRASTRUCTURE ONLY.

Setting (Methodology, PipeSP; Algorithm 1; Supplement, consistency proof of
PipeSP).  n GPUs run Ulysses-style sequence parallelism over H = n*h heads.
GPU i owns the global heads i*h .. i*h+h-1 over the FULL sequence of S tokens
and, after attention, the sequence is re-distributed: GPU r ends up with the
tokens of its slice r (S/n of them) for ALL heads.

  * Original Ulysses: one All-to-All after all h local heads.  GPU r then holds
    hidden[t, i*h + j, :] = result of global head i*h+j at token t of slice r
    (head-contiguous order, k_orig(i,j) = i*h + j).
  * PipeSP: one All-to-All per local head j (Algorithm 1, steps 3-8).  The
    exchange of step j delivers to GPU r one piece per source GPU i, i.e. a
    chunk [rows, n, D] whose middle axis is the source GPU.  Concatenating the h
    chunks along that axis (step 10) gives the interleaved head order
    k_mod(i,j) = j*n + i, and steps 11-13 (view(-1,h,n,D), permute(0,2,1,3),
    view(-1,h*n,D)) restore the head-contiguous order.

Reading taken where the algorithm is terse: a chunk is [rows, n, D] with rows
the flattened (batch, local token) axes, and "dim=1" of the concat is the
gathered-head axis.  The proof in the Supplement drops the sequence axis in the
same way (its tensors are B x H x D).

Functions follow the algorithm's steps as printed, with numpy's reshape and
transpose as the view and permute.  Pins (tests/test_oracle_layout.py): the
index formulas k_orig / k_mod of the Supplement evaluated by explicit loops, a
simulated n-GPU exchange compared with the original Ulysses layout, n = 1 and
h = 1 (identity), and the inverse relation Psi_{n,h} o Psi_{h,n} = id.
"""
from __future__ import annotations

import numpy as np


def postprocess(chunks, h: int, n: int, D: int) -> np.ndarray:
    """Algorithm 1, steps 10-13: h chunks [rows, n, D] -> hidden [rows, h*n, D]."""
    assert len(chunks) == h
    hidden = np.concatenate(chunks, axis=1)           # step 10: [rows, h*n, D], head order j*n+i
    hidden = hidden.reshape(-1, h, n, D)              # step 11: view(-1, h, n, D)
    hidden = hidden.transpose(0, 2, 1, 3)             # step 12: permute(0, 2, 1, 3)
    return np.ascontiguousarray(hidden).reshape(-1, h * n, D)   # step 13: view(-1, h*n, D)


def psi(t_mod: np.ndarray, h: int, n: int) -> np.ndarray:
    """The composite map Psi of the Supplement on an already concatenated [rows, h*n, D] tensor."""
    rows, H, D = t_mod.shape
    assert H == h * n
    return postprocess([t_mod[:, j * n:(j + 1) * n, :] for j in range(h)], h, n, D)


def exchange_step(results, r: int) -> np.ndarray:
    """What GPU r receives from the All-to-All of one pipeline step (Algorithm 1, step 7).

    results[i] is GPU i's attention result of its current local head over the
    full sequence, [S, D].  GPU r gets tokens of slice r from every source:
    chunk[t, i, :] = results[i][r*S/n + t, :].
    """
    n = len(results)
    S = results[0].shape[0]
    assert S % n == 0
    sl = S // n
    return np.stack([results[i][r * sl:(r + 1) * sl] for i in range(n)], axis=1)


def ulysses_hidden(out_heads: np.ndarray, n: int, r: int) -> np.ndarray:
    """Original Ulysses layout on GPU r: out_heads [H, S, D] (global head order) -> [S/n, H, D]."""
    H, S, D = out_heads.shape
    assert S % n == 0
    sl = S // n
    return np.ascontiguousarray(out_heads[:, r * sl:(r + 1) * sl, :].transpose(1, 0, 2))
