"""fp64 oracle: per-head scaled dot-product attention and the exact merge of partials.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is computed.  The paper treats attention as a black box applied to one
head at a time over the whole sequence (Algorithm 1, step 3:
attention(Q[:,j], K[:,j], V[:,j], mask[:,j]); Attention Co-processing:
Attn(Q,K,V)) and states that heads are independent.  The box is taken to be
standard scaled-dot-product softmax attention, with the mask reduced to a
key-padding tail: keys at index >= kv_valid_len are hidden from every query.
For a query row i of one head, with n_v = kv_valid_len:

    s_j   = scale * sum_c q[i,c] * k[j,c]             j = 0 .. n_v-1
    m     = max_j s_j
    Z     = sum_j exp(s_j - m)
    lse_i = m + ln Z                                   (natural log)
    out_i = sum_j exp(s_j - m) * v[j,:] / Z

n_v = 0 gives out = 0 and lse = -inf (an empty share of the keys, which must
drop out of a merge with weight zero).

The definition is written out as is: the whole score row is formed, then a
two-pass softmax.  Rows are independent, so they are processed in blocks
purely to bound memory; no row's arithmetic depends on the blocking.  The
matrix products are numpy's (a library matmul serves as a step).

Exact merge of partial attentions over disjoint key sets (what recombines
Ring-Attention style key shares, and query shares padded with empty rows):

    L    = ln sum_p exp(lse_p)        (evaluated as M + ln sum_p exp(lse_p - M), M = max_p lse_p)
    out  = sum_p exp(lse_p - L) * out_p

with the convention that partials whose lse is -inf carry weight 0, and that
if every partial is empty then out = 0 and L = -inf.

Pins (tests/test_oracle_pins.py): brute force with exact rational/fsum
arithmetic on tiny inputs, scipy's softmax/logsumexp on the unmasked case,
closed forms (single key, zero keys, scale 0, identical V rows), permutation
and shift identities, truncation == masking, split+merge == unsplit.  The
paper prints no numeric worked example of attention, so beyond those pins the
values are fixed by the definition alone.
"""
from __future__ import annotations

import numpy as np


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 payloads (uint16) -> fp64, exactly (bf16 is a subset of fp64)."""
    b = np.ascontiguousarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("expected uint16 bf16 payloads")
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def _as_f64(x: np.ndarray) -> np.ndarray:
    return widen_bf16(x) if x.dtype == np.uint16 else np.asarray(x, dtype=np.float64)


def attention_head(q, k, v, scale, kv_valid_len=None, rows=None, row_block=1024):
    """One head.  q [Sq,d], k [Skv,d], v [Skv,d] (uint16 bf16 payloads or floats).

    rows: optional 1-D index array of query rows to evaluate (each against all
    valid keys).  Returns (out [n,d] fp64, lse [n] fp64).
    """
    k64, v64 = _as_f64(k), _as_f64(v)
    Skv, d = k64.shape
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    if not (0 <= n_v <= Skv):
        raise ValueError("kv_valid_len out of range")
    q_sel = q if rows is None else np.asarray(q)[np.asarray(rows, dtype=np.int64)]
    q64 = _as_f64(q_sel)
    n = q64.shape[0]
    out = np.zeros((n, d), dtype=np.float64)
    lse = np.full((n,), -np.inf, dtype=np.float64)
    if n_v == 0 or n == 0:
        return out, lse
    kk, vv = k64[:n_v], v64[:n_v]
    for r0 in range(0, n, row_block):
        r1 = min(r0 + row_block, n)
        s = (q64[r0:r1] @ kk.T) * float(scale)            # [rows, n_v] full score rows
        m = s.max(axis=1)
        e = np.exp(s - m[:, None])
        Z = e.sum(axis=1)
        lse[r0:r1] = m + np.log(Z)
        out[r0:r1] = (e @ vv) / Z[:, None]
    return out, lse


def attention(q, k, v, scale, kv_valid_len=None):
    """q [B,H,Sq,d], k/v [B,H,Skv,d] -> (out [B,H,Sq,d], lse [B,H,Sq]), heads independent."""
    B, H, Sq, d = q.shape
    out = np.empty((B, H, Sq, d), dtype=np.float64)
    lse = np.empty((B, H, Sq), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h], lse[b, h] = attention_head(q[b, h], k[b, h], v[b, h], scale, kv_valid_len)
    return out, lse


def merge_partials(outs, lses):
    """outs: sequence of [R,d]; lses: sequence of [R].  Returns (out [R,d], lse [R]) in fp64."""
    O = np.stack([np.asarray(o, dtype=np.float64) for o in outs])       # [n,R,d]
    L = np.stack([np.asarray(l, dtype=np.float64) for l in lses])       # [n,R]
    M = L.max(axis=0)
    Msafe = np.where(np.isneginf(M), 0.0, M)
    w = np.exp(L - Msafe[None, :])                                      # exp(-inf)=0 for empty partials
    tot = w.sum(axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = np.where(tot > 0, Msafe + np.log(tot), -np.inf)
        wn = np.where(tot[None, :] > 0, w / tot[None, :], 0.0)          # = exp(lse_p - L)
    Oz = np.where(wn[:, :, None] > 0, O, 0.0)                           # weight-0 partials contribute nothing
    out = (wn[:, :, None] * Oz).sum(axis=0)
    return out, lse
