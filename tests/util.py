"""Shared helpers of the GPU parity tests: upload of bf16 payloads, tolerances, row sampling."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

from synth import K_ID, Q_ID, V_ID, gen_tensor

# Tolerances of the GPU path against the fp64 oracle on bf16 inputs with fp32 accumulation.
MAX_ABS, MEAN_ABS, LSE_REL = 2e-2, 2e-3, 1e-3
# Self-imposed on top: at long sequences outputs are O(sqrt(e/S)), so the absolute gates alone
# would pass an all-zero result.  Relative L2 error over the compared rows.
REL_L2 = 1e-2


def to_dev_bf16(bits: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def gen_qkv_parallel(w, heads=None, workers=8):
    """q, k, v payloads of workload w (optionally a head range), generated head by head in threads."""
    h0, h1 = heads if heads is not None else (0, w.H)
    jobs = []
    for tid, S in ((Q_ID, w.Sq), (K_ID, w.Skv), (V_ID, w.Skv)):
        for h in range(h0, h1):
            jobs.append((tid, S, h))

    def run(job):
        tid, S, h = job
        return gen_tensor(w.seed, tid, (w.B, w.H, S, w.d), unit_rms=w.unit_rms, heads=(h, h + 1))

    with ThreadPoolExecutor(max_workers=workers) as ex:
        parts = list(ex.map(run, jobs))
    n = h1 - h0
    q = np.concatenate(parts[0:n], axis=1)
    k = np.concatenate(parts[n:2 * n], axis=1)
    v = np.concatenate(parts[2 * n:3 * n], axis=1)
    return q, k, v


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
