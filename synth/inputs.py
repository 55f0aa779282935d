"""Counter-based Gaussian tensors, rounded to bf16 (stored as uint16 payloads).

Every element is a pure function of (seed, tensor id, flat element index), so
any head or row range of a large tensor can be produced on its own and always
carries the same bits.  Recipe:

  key      = mix64(seed * 0x9E3779B97F4A7C15 + tensor_id)
  z        = mix64(key + pair_index * 0xD1B54A32D192ED03)        (pair = 2 elements)
  u1, u2   = ((z >> 32) + 0.5) / 2^32 , ((z & 0xffffffff) + 0.5) / 2^32
  n0, n1   = sqrt(-2 ln u1) * (cos, sin)(2 pi u2)                (Box-Muller, fp64)
  x        = float32(n)
  optional: every d-vector divided by its own RMS (fp32)          ("unit-RMS rows")
  payload  = round-to-nearest-even of x to bf16

mix64 is the splitmix64 finaliser.
"""
from __future__ import annotations

import numpy as np

Q_ID, K_ID, V_ID = 1, 2, 3

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_STEP = np.uint64(0xD1B54A32D192ED03)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns the uint16 payloads."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 payloads exactly to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normals(seed: int, tensor_id: int, first_elem: int, count: int) -> np.ndarray:
    """fp32 N(0,1) values for flat element indices [first_elem, first_elem+count); both even."""
    assert first_elem % 2 == 0 and count % 2 == 0
    with np.errstate(over="ignore"):
        key = _mix64(np.array([np.uint64(seed) * _GOLD + np.uint64(tensor_id)], dtype=np.uint64))[0]
        pairs = np.arange(first_elem // 2, (first_elem + count) // 2, dtype=np.uint64)
        z = _mix64(key + pairs * _STEP)
    u1 = ((z >> np.uint64(32)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    u2 = ((z & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    r = np.sqrt(-2.0 * np.log(u1))
    ang = (2.0 * np.pi) * u2
    out = np.empty(count, dtype=np.float32)
    out[0::2] = r * np.cos(ang)
    out[1::2] = r * np.sin(ang)
    return out


def gen_tensor(seed: int, tensor_id: int, shape, *, unit_rms: bool, heads=None,
               rows=None, chunk_rows: int = 1 << 16) -> np.ndarray:
    """bf16 payloads (uint16) of a [B,H,S,d] tensor, or of a slice of it.

    heads: optional (h0, h1) range of the H axis; rows: optional (r0, r1) range
    of the S axis.  The slice carries exactly the bits the full tensor would.
    """
    B, H, S, d = (int(x) for x in shape)
    assert d % 2 == 0
    h0, h1 = heads if heads is not None else (0, H)
    r0, r1 = rows if rows is not None else (0, S)
    out = np.empty((B, h1 - h0, r1 - r0, d), dtype=np.uint16)
    for b in range(B):
        for h in range(h0, h1):
            for c0 in range(r0, r1, chunk_rows):
                c1 = min(c0 + chunk_rows, r1)
                first = ((b * H + h) * S + c0) * d
                x = _normals(seed, tensor_id, first, (c1 - c0) * d).reshape(c1 - c0, d)
                if unit_rms:
                    rms = np.sqrt(np.mean(x * x, axis=1, dtype=np.float32), dtype=np.float32)
                    x = x / rms[:, None]
                out[b, h - h0, c0 - r0:c1 - r0] = f32_to_bf16_bits(x)
    return out


def gen_qkv(seed: int, B: int, H: int, Sq: int, Skv: int, d: int, *, unit_rms: bool, heads=None):
    """(q, k, v) bf16 payloads with shapes [B,H',Sq,d], [B,H',Skv,d], [B,H',Skv,d]."""
    q = gen_tensor(seed, Q_ID, (B, H, Sq, d), unit_rms=unit_rms, heads=heads)
    k = gen_tensor(seed, K_ID, (B, H, Skv, d), unit_rms=unit_rms, heads=heads)
    v = gen_tensor(seed, V_ID, (B, H, Skv, d), unit_rms=unit_rms, heads=heads)
    return q, k, v


def gen_qkv_parallel(w, heads=None, workers: int = 8):
    """q, k, v payloads of workload w (optionally a head range), generated head by head in threads."""
    from concurrent.futures import ThreadPoolExecutor
    h0, h1 = heads if heads is not None else (0, w.H)
    jobs = [(tid, S, h) for tid, S in ((Q_ID, w.Sq), (K_ID, w.Skv), (V_ID, w.Skv)) for h in range(h0, h1)]

    def run(job):
        tid, S, h = job
        return gen_tensor(w.seed, tid, (w.B, w.H, S, w.d), unit_rms=w.unit_rms, heads=(h, h + 1))

    with ThreadPoolExecutor(max_workers=workers) as ex:
        parts = list(ex.map(run, jobs))
    n = h1 - h0
    return (np.concatenate(parts[0:n], axis=1), np.concatenate(parts[n:2 * n], axis=1),
            np.concatenate(parts[2 * n:3 * n], axis=1))


def to_dev_bf16(bits: np.ndarray):
    """Upload uint16 bf16 payloads as a torch.bfloat16 tensor on the current GPU (same bits)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()
