"""Shared helpers of the GPU parity tests: upload of bf16 payloads, tolerances, row sampling."""
from __future__ import annotations

import numpy as np

from synth import gen_qkv_parallel, to_dev_bf16  # noqa: F401  (re-exported for the tests)

# Tolerances of the GPU path against the fp64 oracle on bf16 inputs with fp32 accumulation.
MAX_ABS, MEAN_ABS, LSE_REL = 2e-2, 2e-3, 1e-3
# Self-imposed on top: at long sequences outputs are O(sqrt(e/S)), so the absolute gates alone
# would pass an all-zero result.  Relative L2 error over the compared rows.
REL_L2 = 1e-2


def sample_rows(Sq: int, n: int, seed: int, tile: int = 256, extra=()):
    """Seeded row sample that always holds the first/last rows and both sides of tile boundaries
    near the start and the end, plus the given extra rows."""
    rng = np.random.default_rng(seed)
    forced = {0, 1, Sq - 1, Sq - 2}
    for t in (tile, 2 * tile, (Sq // tile) * tile, (Sq // tile - 1) * tile, 32, 64, 128):
        forced.update({t - 1, t, t + 1})
    forced.update(extra)
    forced = {r for r in forced if 0 <= r < Sq}
    rest = rng.choice(Sq, size=max(0, min(n, Sq) - len(forced)), replace=False)
    return np.array(sorted(forced.union(rest.tolist())), dtype=np.int64)


def errors(out_gpu: np.ndarray, lse_gpu: np.ndarray, out_ref: np.ndarray, lse_ref: np.ndarray):
    diff = out_gpu.astype(np.float64) - out_ref
    e = {
        "max_abs": float(np.abs(diff).max()) if diff.size else 0.0,
        "mean_abs": float(np.abs(diff).mean()) if diff.size else 0.0,
        "rel_l2": float(np.sqrt((diff ** 2).sum() / max((out_ref ** 2).sum(), 1e-300))) if diff.size else 0.0,
        "lse_rel": float((np.abs(lse_gpu.astype(np.float64) - lse_ref) / np.maximum(np.abs(lse_ref), 1.0)).max())
        if lse_ref.size else 0.0,
    }
    return e


def assert_close(out_gpu, lse_gpu, out_ref, lse_ref, what=""):
    assert np.isfinite(out_gpu).all() and np.isfinite(lse_gpu).all(), f"{what}: non-finite GPU result"
    e = errors(out_gpu, lse_gpu, out_ref, lse_ref)
    msg = f"{what}: {e}"
    assert e["max_abs"] <= MAX_ABS, msg
    assert e["mean_abs"] <= MEAN_ABS, msg
    assert e["rel_l2"] <= REL_L2, msg
    assert e["lse_rel"] <= LSE_REL, msg
    return e


def tail_plan(BH: int, Sq: int, n_v: int, d: int, n_cu: int):
    """Which query tiles an attention launch (d = 64 or 128) computes as merged key-range partials, and
    over which key ranges: the rule of pda_attn_tail_plan written out independently.  Tiles of 256
    rows; the rem = n_tiles mod n_cu tiles that do not fill a round of whole tiles are cut into s =
    round(3*n_cu/rem) key ranges, at least 2 and at most min(16, L, n_v // 512, 1 + (9*n_cu//4) //
    rem) with nt the key tiles (of 64) of a whole sweep and L = max(nt // 100, min(nt // 50, 4)),
    lowered until the last range is not empty; uncut if that leaves less than 2.  A launch of fewer
    tiles than compute units, or one with nt < 200 whose left-over tiles fill at most half the
    machine, is cut so that one round of parts fills the machine instead: s = n_cu // rem under the
    same caps except L.  Ranges are equal, ceil(n_v / s) keys rounded up to a multiple of 64, except
    (a) decreasing ranges and (b) a long first range, both described where they are computed."""
    plan = {"n_tiles": 0, "n_cut": 0, "split": 1, "part_offsets": [], "workspace_slots": 0}
    if d not in (64, 128) or n_v <= 0 or BH * Sq <= 0:
        return plan
    tiles = -(-Sq // 256) * BH
    plan["n_tiles"] = tiles
    rem = tiles % n_cu
    if rem == 0:
        return plan
    nt = -(-n_v // 64)

    def keys(s):
        return -(-(-(-n_v // s)) // 64) * 64

    one_round = tiles < n_cu or (nt < 200 and 2 * rem <= n_cu)   # short parts that start together
    if one_round:
        s_max = min(16, n_v // 512, 1 + (9 * n_cu // 4) // rem)
        s = min(n_cu // rem, s_max)
    else:
        by_len = max(nt // 100, min(nt // 50, 4))
        s_max = min(16, by_len, n_v // 512, 1 + (9 * n_cu // 4) // rem)
        s = min(max((6 * n_cu + rem) // (2 * rem), 2), s_max)
    while s >= 2 and (s - 1) * keys(s) >= n_v:
        s -= 1
    if s >= 2:
        offs = [j * keys(s) for j in range(s)] + [n_v]
        # (a) After four or more rounds of whole tiles (and at most 6 ranges): decreasing ranges, each 5/8
        # of the one before, boundaries rounded down to multiples of 64; kept equal if the last range
        # would hold fewer than 3200 keys or a range would be empty.
        if not one_round and tiles >= 4 * n_cu and s <= 6:
            w = [8 ** (s - 1 - j) * 5 ** j for j in range(s)]
            dec = [0] + [n_v * sum(w[:j]) // sum(w) // 64 * 64 for j in range(1, s)] + [n_v]
            if n_v - dec[s - 1] >= 3200 and all(b > a for a, b in zip(dec, dec[1:])):
                offs = dec
        plan.update(n_cut=rem, split=s, part_offsets=offs, workspace_slots=rem * (s - 1))
    # (b) Where the left-over tiles fill more than half the machine after one to three rounds of whole
    # tiles: a long first range (a fraction k / (k + s - 1) of the keys plus 1 %, up to the next
    # multiple of 64) and s - 1 short ones of at least 1024 keys, k = ceil(rem (s-1) / (n_cu - rem));
    # s = 4 after one round of whole tiles, else 3, within the workspace cap, lowered until it fits.
    if 2 * rem > n_cu and n_cu < tiles < 4 * n_cu:
        s = min(4 if tiles < 2 * n_cu else 3, 1 + (9 * n_cu // 4) // rem)
        while s >= 2:
            k = -(-rem * (s - 1) // (n_cu - rem))
            first = ((n_v * k // (k + s - 1) + n_v // 100) // 64 + 1) * 64
            part = -(-(-(-(n_v - first) // (s - 1))) // 64) * 64 if first < n_v else 0
            if first < n_v and part >= 1024 and first + (s - 2) * part < n_v:
                plan.update(n_cut=rem, split=s, part_offsets=[0] + [first + j * part for j in range(s - 1)] + [n_v],
                            workspace_slots=rem * (s - 1))
                break
            s -= 1
    return plan


def cut_row_mask(B: int, H: int, Sq: int, n_v: int, d: int, n_cu: int):
    """Boolean [B, H, Sq]: rows lying in a query tile that a launch over all B*H heads cuts."""
    plan = tail_plan(B * H, Sq, n_v, d, n_cu)
    mask = np.zeros((B * H, Sq), dtype=bool)
    tph = -(-Sq // 256)
    for t in range(plan["n_tiles"] - plan["n_cut"], plan["n_tiles"]):
        bh, qt = divmod(t, tph)
        mask[bh, qt * 256:(qt + 1) * 256] = True
    return mask.reshape(B, H, Sq)
