"""Pins for the fp64 oracle: things fixed by the mathematics, not by the oracle itself.

Attention is a black box in the paper (Algorithm 1 step 3; Attn(Q,K,V) in the
Attention Co-processing section) and no numeric worked example is printed, so
the pins are: an independent brute-force evaluation with exactly-rounded sums
on tiny inputs, scipy's softmax/logsumexp on the unmasked case, closed forms,
and identities.  Each would fail for a dropped term, a wrong sign or index, or
a transposed operand in the oracle.
"""
import math

import numpy as np
import pytest
import scipy.special

from oracle import attention, attention_head, merge_partials, widen_bf16


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def brute_force_row(q_row, k, v, scale, n_v):
    """Pure-Python evaluation of one query row, sums by math.fsum."""
    d = len(q_row)
    s = [scale * math.fsum(q_row[c] * k[j][c] for c in range(d)) for j in range(n_v)]
    m = max(s)
    e = [math.exp(x - m) for x in s]
    Z = math.fsum(e)
    out = [math.fsum(e[j] * v[j][c] for j in range(n_v)) / Z for c in range(len(v[0]))]
    return out, m + math.log(Z)


@pytest.mark.parametrize("Sq,Skv,d,n_v,scale", [(5, 7, 3, 7, 0.7), (4, 13, 5, 9, 1.3), (3, 32, 8, 31, 0.35), (1, 1, 2, 1, 2.0)])
def test_brute_force_tiny(Sq, Skv, d, n_v, scale):
    rng = np.random.default_rng(100 + Skv)
    q, k, v = _rand(rng, Sq, d), _rand(rng, Skv, d) * 2.0, _rand(rng, Skv, d)
    out, lse = attention_head(q, k, v, scale, n_v)
    for i in range(Sq):
        o_ref, l_ref = brute_force_row(q[i].tolist(), k.tolist(), v.tolist(), scale, n_v)
        assert np.allclose(out[i], o_ref, rtol=0, atol=1e-12)
        assert abs(lse[i] - l_ref) < 1e-12


def test_non_square_value_dim_and_operand_order():
    # distinct Sq, Skv, d so any transposed operand changes shapes or values
    rng = np.random.default_rng(7)
    q, k, v = _rand(rng, 6, 4), _rand(rng, 11, 4), _rand(rng, 11, 4)
    out, lse = attention_head(q, k, v, 0.5)
    p = scipy.special.softmax(0.5 * (q @ k.T), axis=1)
    assert np.allclose(out, p @ v, atol=1e-13)
    assert np.allclose(lse, scipy.special.logsumexp(0.5 * (q @ k.T), axis=1), atol=1e-13)
    assert out.shape == (6, 4) and lse.shape == (6,)


def test_single_key():
    rng = np.random.default_rng(1)
    q, k, v = _rand(rng, 9, 6), _rand(rng, 1, 6), _rand(rng, 1, 6)
    out, lse = attention_head(q, k, v, 0.3)
    assert np.allclose(out, np.repeat(v, 9, axis=0), atol=1e-15)
    assert np.allclose(lse, 0.3 * (q @ k[0]), atol=1e-14)


def test_two_keys_closed_form():
    rng = np.random.default_rng(2)
    q, k, v = _rand(rng, 5, 3), _rand(rng, 2, 3), _rand(rng, 2, 3)
    scale = 1.7
    out, lse = attention_head(q, k, v, scale)
    for i in range(5):
        s1, s2 = (scale * float(q[i] @ k[j]) for j in range(2))
        w1 = 1.0 / (1.0 + math.exp(s2 - s1))
        assert np.allclose(out[i], w1 * v[0] + (1 - w1) * v[1], atol=1e-14)
        assert abs(lse[i] - (max(s1, s2) + math.log1p(math.exp(-abs(s1 - s2))))) < 1e-14


@pytest.mark.parametrize("n_v", [1, 5, 12])
def test_zero_keys_give_mean_of_valid_values(n_v):
    rng = np.random.default_rng(3)
    q, v = _rand(rng, 4, 8), _rand(rng, 12, 8)
    k = np.zeros((12, 8))
    out, lse = attention_head(q, k, v, 0.9, n_v)
    assert np.allclose(out, np.tile(v[:n_v].mean(axis=0), (4, 1)), atol=1e-14)
    assert np.allclose(lse, math.log(n_v), atol=1e-14)


def test_scale_zero_gives_mean():
    rng = np.random.default_rng(4)
    q, k, v = _rand(rng, 4, 8), _rand(rng, 10, 8), _rand(rng, 10, 8)
    out, lse = attention_head(q, k, v, 0.0)
    assert np.allclose(out, np.tile(v.mean(axis=0), (4, 1)), atol=1e-14)
    assert np.allclose(lse, math.log(10), atol=1e-14)


def test_identical_value_rows():
    rng = np.random.default_rng(5)
    q, k = _rand(rng, 6, 8) * 3, _rand(rng, 20, 8) * 3
    row = _rand(rng, 8)
    out, _ = attention_head(q, k, np.tile(row, (20, 1)), 0.8, 17)
    assert np.allclose(out, np.tile(row, (6, 1)), atol=1e-14)


def test_key_permutation_invariance_and_query_equivariance():
    rng = np.random.default_rng(6)
    q, k, v = _rand(rng, 7, 4), _rand(rng, 15, 4), _rand(rng, 15, 4)
    out, lse = attention_head(q, k, v, 0.6)
    pk = rng.permutation(15)
    out2, lse2 = attention_head(q, k[pk], v[pk], 0.6)
    assert np.allclose(out, out2, atol=1e-14) and np.allclose(lse, lse2, atol=1e-14)
    pq = rng.permutation(7)
    out3, lse3 = attention_head(q[pq], k, v, 0.6)
    assert np.allclose(out[pq], out3, atol=1e-15) and np.allclose(lse[pq], lse3, atol=1e-15)


def test_key_shift_identity():
    rng = np.random.default_rng(8)
    q, k, v = _rand(rng, 5, 6), _rand(rng, 9, 6), _rand(rng, 9, 6)
    c = _rand(rng, 6)
    out, lse = attention_head(q, k, v, 0.4)
    out2, lse2 = attention_head(q, k + c, v, 0.4)
    assert np.allclose(out, out2, atol=1e-13)
    assert np.allclose(lse2 - lse, 0.4 * (q @ c), atol=1e-13)


def test_mask_equals_truncation_and_hidden_keys_never_read():
    rng = np.random.default_rng(9)
    q, k, v = _rand(rng, 5, 6), _rand(rng, 14, 6), _rand(rng, 14, 6)
    k[10:], v[10:] = np.nan, np.inf          # poison the hidden tail
    out, lse = attention_head(q, k, v, 0.4, 10)
    out2, lse2 = attention_head(q, k[:10], v[:10], 0.4)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)
    assert np.isfinite(out).all()


def test_duplicated_key_counts_as_weight():
    rng = np.random.default_rng(10)
    q, k, v = _rand(rng, 3, 4), _rand(rng, 2, 4), _rand(rng, 2, 4)
    r = 5
    kd = np.vstack([np.tile(k[0], (r, 1)), k[1:2]])
    vd = np.vstack([np.tile(v[0], (r, 1)), v[1:2]])
    out, lse = attention_head(q, kd, vd, 1.0)
    for i in range(3):
        s1, s2 = float(q[i] @ k[0]), float(q[i] @ k[1])
        Z = r * math.exp(s1) + math.exp(s2)
        assert np.allclose(out[i], (r * math.exp(s1) * v[0] + math.exp(s2) * v[1]) / Z, atol=1e-13)
        assert abs(lse[i] - math.log(Z)) < 1e-13


def test_output_in_convex_hull_and_probabilities_sum_to_one():
    rng = np.random.default_rng(11)
    q, k, v = _rand(rng, 8, 4) * 4, _rand(rng, 30, 4), _rand(rng, 30, 4)
    out, lse = attention_head(q, k, v, 1.0)
    assert (out <= v.max(axis=0) + 1e-12).all() and (out >= v.min(axis=0) - 1e-12).all()
    s = q @ k.T
    assert np.allclose(np.exp(s - lse[:, None]).sum(axis=1), 1.0, atol=1e-13)


def test_empty_share():
    rng = np.random.default_rng(12)
    q, k, v = _rand(rng, 3, 4), _rand(rng, 5, 4), _rand(rng, 5, 4)
    out, lse = attention_head(q, k, v, 1.0, 0)
    assert (out == 0).all() and np.isneginf(lse).all()


def test_rows_argument_selects_rows():
    rng = np.random.default_rng(13)
    q, k, v = _rand(rng, 40, 4), _rand(rng, 50, 4), _rand(rng, 50, 4)
    out, lse = attention_head(q, k, v, 0.5, 45, row_block=7)
    rows = np.array([39, 0, 17, 17])
    o2, l2 = attention_head(q, k, v, 0.5, 45, rows=rows, row_block=3)
    assert np.allclose(out[rows], o2, atol=1e-15) and np.allclose(lse[rows], l2, atol=1e-15)


def test_widen_bf16_known_payloads():
    bits = np.array([0x3F80, 0xC000, 0x3DCC, 0x0000, 0x8000, 0x7F7F, 0x0080], dtype=np.uint16)
    want = [1.0, -2.0, 0.099609375, 0.0, -0.0, (2 - 2 ** -7) * 2.0 ** 127, 2.0 ** -126]
    got = widen_bf16(bits)
    assert got.dtype == np.float64 and got.tolist() == want


def test_multihead_wrapper_matches_per_head_and_heads_are_independent():
    rng = np.random.default_rng(14)
    q, k, v = _rand(rng, 2, 3, 6, 4), _rand(rng, 2, 3, 9, 4), _rand(rng, 2, 3, 9, 4)
    out, lse = attention(q, k, v, 0.5, 8)
    k2 = k.copy(); k2[1, 2] += 10.0          # perturb one head: the others must not move
    out2, _ = attention(q, k2, v, 0.5, 8)
    for b in range(2):
        for h in range(3):
            o, l = attention_head(q[b, h], k[b, h], v[b, h], 0.5, 8)
            assert np.array_equal(out[b, h], o) and np.array_equal(lse[b, h], l)
            if (b, h) != (1, 2):
                assert np.array_equal(out[b, h], out2[b, h])


# ---------------------------------------------------------------- merge

def test_key_split_merge_equals_unsplit():
    rng = np.random.default_rng(20)
    q, k, v = _rand(rng, 9, 6) * 2, _rand(rng, 41, 6), _rand(rng, 41, 6)
    full, lfull = attention_head(q, k, v, 0.7, 37)
    cuts = [0, 10, 11, 30, 41]
    parts = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        nv = max(0, min(37, b) - a)
        parts.append(attention_head(q, k[a:b], v[a:b], 0.7, nv))
    out, lse = merge_partials([p[0] for p in parts], [p[1] for p in parts])
    assert np.allclose(out, full, atol=1e-13) and np.allclose(lse, lfull, atol=1e-13)


def test_query_split_merge_equals_concatenation():
    rng = np.random.default_rng(21)
    q, k, v = _rand(rng, 10, 4), _rand(rng, 12, 4), _rand(rng, 12, 4)
    full, lfull = attention_head(q, k, v, 0.7)
    outs, lses = [], []
    for a, b in [(0, 4), (4, 7), (7, 10)]:
        o = np.full((10, 4), np.nan); l = np.full(10, -np.inf)   # rows outside the range are empty
        o[a:b], l[a:b] = attention_head(q[a:b], k, v, 0.7)
        outs.append(o); lses.append(l)
    out, lse = merge_partials(outs, lses)
    assert np.array_equal(out, full) and np.array_equal(lse, lfull)


def test_merge_two_partials_closed_form():
    o1, o2 = np.array([[1.0, 2.0]]), np.array([[3.0, -4.0]])
    l1, l2 = np.array([0.3]), np.array([-1.1])
    out, lse = merge_partials([o1, o2], [l1, l2])
    w1 = 1.0 / (1.0 + math.exp(l2[0] - l1[0]))
    assert np.allclose(out, w1 * o1 + (1 - w1) * o2, atol=1e-15)
    assert abs(lse[0] - math.log(math.exp(0.3) + math.exp(-1.1))) < 1e-15


def test_merge_brute_force():
    rng = np.random.default_rng(22)
    n, R, d = 5, 6, 3
    O, L = _rand(rng, n, R, d), _rand(rng, n, R) * 5
    out, lse = merge_partials(list(O), list(L))
    for r in range(R):
        Z = math.fsum(math.exp(L[p, r]) for p in range(n))
        assert abs(lse[r] - math.log(Z)) < 1e-12
        for c in range(d):
            assert abs(out[r, c] - math.fsum(math.exp(L[p, r]) * O[p, r, c] for p in range(n)) / Z) < 1e-12


def test_merge_all_empty_and_single_and_order():
    rng = np.random.default_rng(23)
    O, L = _rand(rng, 3, 4, 2), _rand(rng, 3, 4)
    L[:, 1] = -np.inf                         # row 1 empty everywhere
    L[0, 2] = -np.inf                         # row 2: first partial empty
    out, lse = merge_partials(list(O), list(L))
    assert (out[1] == 0).all() and np.isneginf(lse[1])
    o2, l2 = merge_partials([O[1], O[2]], [L[1], L[2]])
    assert np.allclose(out[2], o2[2], atol=1e-15) and abs(lse[2] - l2[2]) < 1e-15
    o3, l3 = merge_partials([O[2], O[0], O[1]], [L[2], L[0], L[1]])
    assert np.allclose(out, o3, atol=1e-14) and np.allclose(lse[np.isfinite(lse)], l3[np.isfinite(l3)], atol=1e-14)
    o1, l1 = merge_partials([O[0]], [L[0]])
    fin = np.isfinite(L[0])
    assert np.array_equal(o1[fin], O[0][fin]) and np.array_equal(l1[fin], L[0][fin])


def test_merge_associative():
    rng = np.random.default_rng(24)
    O, L = _rand(rng, 4, 5, 3), _rand(rng, 4, 5) * 3
    a, la = merge_partials(list(O), list(L))
    b01, l01 = merge_partials([O[0], O[1]], [L[0], L[1]])
    b23, l23 = merge_partials([O[2], O[3]], [L[2], L[3]])
    b, lb = merge_partials([b01, b23], [l01, l23])
    assert np.allclose(a, b, atol=1e-14) and np.allclose(la, lb, atol=1e-14)


def test_large_scores_do_not_overflow():
    q = np.array([[300.0, 0.0]]); k = np.array([[3.0, 0.0], [-3.0, 0.0], [2.9, 1.0]]); v = np.eye(3)[:, :2]
    out, lse = attention_head(q, k, v, 1.0)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert abs(lse[0] - (900.0 + math.log1p(math.exp(-30.0) + math.exp(-1800.0)))) < 1e-9
