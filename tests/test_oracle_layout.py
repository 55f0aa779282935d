"""Pins of the PipeSP layout oracle (Algorithm 1 steps 10-13; Supplement, consistency proof)."""
import numpy as np
import pytest

from oracle import pipesp_layout as L


def _tagged(rows, H, D):
    """Tensor whose every element encodes its own (row, head, column)."""
    r, k, c = np.meshgrid(np.arange(rows), np.arange(H), np.arange(D), indexing="ij")
    return (r * 10000 + k * 100 + c).astype(np.float64)


@pytest.mark.parametrize("h,n", [(3, 8), (4, 2), (1, 5), (6, 1), (2, 3), (5, 4)])
def test_psi_moves_k_mod_to_k_orig(h, n):
    # Supplement: the head that sits at k_mod(i,j) = j*n+i must end at k_orig(i,j) = i*h+j.
    rows, D = 3, 4
    t_mod = _tagged(rows, h * n, D)
    t = L.psi(t_mod, h, n)
    for i in range(n):
        for j in range(h):
            for r in range(rows):
                for c in range(D):
                    assert t[r, i * h + j, c] == t_mod[r, j * n + i, c]


@pytest.mark.parametrize("h,n", [(3, 8), (2, 2), (4, 3)])
def test_pipelined_exchange_plus_postprocess_equals_ulysses(h, n):
    # n simulated GPUs; GPU i owns global heads i*h..i*h+h-1 over the full sequence.
    rng = np.random.default_rng(7 + h * 10 + n)
    S, D = 4 * n, 5
    out_heads = rng.standard_normal((n * h, S, D))
    for r in range(n):
        chunks = []
        for j in range(h):                                  # Algorithm 1 steps 2-9
            results = [out_heads[i * h + j] for i in range(n)]
            chunks.append(L.exchange_step(results, r))
        got = L.postprocess(chunks, h, n, D)                # steps 10-13
        want = L.ulysses_hidden(out_heads, n, r)            # one All-to-All after all heads
        assert got.shape == want.shape
        assert np.array_equal(got, want)


def test_without_postprocess_the_order_is_wrong():
    # the mis-order the post-processing exists for: a plain concat differs from Ulysses when h,n > 1
    h, n, S, D = 3, 2, 4, 2
    out_heads = np.random.default_rng(0).standard_normal((n * h, S, D))
    chunks = [L.exchange_step([out_heads[i * h + j] for i in range(n)], 0) for j in range(h)]
    assert not np.array_equal(np.concatenate(chunks, axis=1), L.ulysses_hidden(out_heads, n, 0))


@pytest.mark.parametrize("h,n", [(1, 7), (7, 1)])
def test_identity_cases(h, n):
    t = _tagged(5, h * n, 3)
    assert np.array_equal(L.psi(t, h, n), t)


@pytest.mark.parametrize("h,n", [(3, 8), (5, 2)])
def test_inverse_is_psi_with_roles_swapped(h, n):
    t = _tagged(4, h * n, 3)
    assert np.array_equal(L.psi(L.psi(t, h, n), n, h), t)


def test_is_a_permutation_of_heads_only():
    h, n = 4, 3
    t = _tagged(6, h * n, 8)
    u = L.psi(t, h, n)
    heads = (u[0, :, 0] // 100 % 100).astype(int)
    assert sorted(heads.tolist()) == list(range(h * n))
    # rows and columns stay in place
    assert np.array_equal(u // 10000, t // 10000) and np.array_equal(u % 100, t % 100)
