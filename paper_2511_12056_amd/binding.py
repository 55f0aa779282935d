"""ctypes binding of libpipedit_attn: same names as the C entry points, argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and
streams); the binding passes raw device pointers and sizes across the C ABI.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpipedit_attn.so")

PDA_OK, PDA_ERR_INVALID_ARG, PDA_ERR_UNSUPPORTED, PDA_ERR_HIP = 0, 1, 2, 3
PDA_MAX_PARTIALS = 16


class PdaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libpipedit_attn error {code}: {message}")
        self.code = code


def lib_path() -> str:
    return _LIB_PATH


def _load() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
            "or python paper_2511_12056_amd/build.py). There is no fallback path.")
    lib = C.CDLL(_LIB_PATH)
    vp, fp, i32, i64, f32 = C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_float
    lib.pda_attn_fwd.argtypes = [vp, vp, vp, fp, fp, i32, i32, i64, i64, i32, f32, i64, i64, vp]
    lib.pda_attn_fwd.restype = i32
    lib.pda_attn_merge.argtypes = [C.POINTER(vp), C.POINTER(vp), i32, fp, fp, i64, i32, vp]
    lib.pda_attn_merge.restype = i32
    lib.pda_headchunk_run.argtypes = [vp, vp, vp, fp, fp, i32, i32, i64, i64, i32, f32, i64, i32, vp, vp, fp,
                                      C.POINTER(f32), C.POINTER(f32)]
    lib.pda_headchunk_run.restype = i32
    lib.pda_last_error.argtypes = []
    lib.pda_last_error.restype = C.c_char_p
    lib.pda_version.argtypes = []
    lib.pda_version.restype = i32
    return lib


lib = _load()


def last_error() -> str:
    return lib.pda_last_error().decode()


def version() -> int:
    return lib.pda_version()


def _check(rc: int) -> None:
    if rc != PDA_OK:
        raise PdaError(rc, last_error())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream
    return h if h else None


def _expect(t, dtype, shape, name):
    import torch
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{name}: expected contiguous cuda {dtype} of shape {tuple(shape)}, "
                         f"got {t.dtype} {tuple(t.shape)} contiguous={t.is_contiguous()} cuda={t.is_cuda}")


def attn_fwd(q, k, v, out, lse, scale: float, kv_valid_len: Optional[int] = None, q_offset: int = 0, stream=None):
    """pda_attn_fwd: q [B,H,Sq,d] bf16, k/v [B,H,Skv,d] bf16 -> out [B,H,Sq,d] fp32, lse [B,H,Sq] fp32."""
    import torch
    B, H, Sq, d = q.shape
    Skv = k.shape[2]
    _expect(q, torch.bfloat16, (B, H, Sq, d), "q")
    _expect(k, torch.bfloat16, (B, H, Skv, d), "k")
    _expect(v, torch.bfloat16, (B, H, Skv, d), "v")
    _expect(out, torch.float32, (B, H, Sq, d), "out")
    _expect(lse, torch.float32, (B, H, Sq), "lse")
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    _check(lib.pda_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, Sq, Skv, d, float(scale),
                            n_v, int(q_offset), _stream_handle(stream)))
    return out, lse


def attn_merge(partials: Sequence, lses: Sequence, out, lse_out=None, stream=None):
    """pda_attn_merge: partials n x [rows,d] fp32, lses n x [rows] fp32 -> out [rows,d] (+ lse_out [rows])."""
    import torch
    n = len(partials)
    if len(lses) != n:
        raise ValueError("partials and lses differ in length")
    d = out.shape[-1]
    rows = out.numel() // d if d else 0
    for i, (pt, lt) in enumerate(zip(partials, lses)):
        if pt.dtype != torch.float32 or lt.dtype != torch.float32 or not pt.is_contiguous() or not lt.is_contiguous():
            raise ValueError(f"partial {i}: expected contiguous fp32")
        if pt.numel() != rows * d or lt.numel() != rows:
            raise ValueError(f"partial {i}: size mismatch")
    if lse_out is not None and (lse_out.dtype != torch.float32 or lse_out.numel() != rows):
        raise ValueError("lse_out: expected fp32 with one entry per row")
    arr_p = (C.c_void_p * max(n, 1))(*[pt.data_ptr() for pt in partials])
    arr_l = (C.c_void_p * max(n, 1))(*[lt.data_ptr() for lt in lses])
    _check(lib.pda_attn_merge(arr_p, arr_l, n, _ptr(out), _ptr(lse_out), rows, d, _stream_handle(stream)))
    return out, lse_out


def headchunk_run(q, k, v, out, lse, scale: float, heads_per_group: int, compute_stream, drain_stream,
                  kv_valid_len: Optional[int] = None, sink=None, timed: bool = False):
    """pda_headchunk_run.  Returns (group_ms list, total_ms) when timed, else None (caller syncs both streams)."""
    import torch
    B, H, Sq, d = q.shape
    Skv = k.shape[2]
    _expect(q, torch.bfloat16, (B, H, Sq, d), "q")
    _expect(k, torch.bfloat16, (B, H, Skv, d), "k")
    _expect(v, torch.bfloat16, (B, H, Skv, d), "v")
    _expect(out, torch.float32, (B, H, Sq, d), "out")
    _expect(lse, torch.float32, (B, H, Sq), "lse")
    if sink is not None:
        _expect(sink, torch.float32, (B, H, Sq, d), "sink")
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    n_groups = (H + heads_per_group - 1) // heads_per_group if heads_per_group > 0 and H > 0 else 0
    gms = (C.c_float * max(n_groups, 1))() if timed else None
    tms = C.c_float(0.0) if timed else None
    _check(lib.pda_headchunk_run(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, Sq, Skv, d, float(scale),
                                 n_v, int(heads_per_group), _stream_handle(compute_stream),
                                 _stream_handle(drain_stream), _ptr(sink),
                                 gms if timed else None, C.byref(tms) if timed else None))
    if timed:
        return [gms[i] for i in range(n_groups)], tms.value
    return None
