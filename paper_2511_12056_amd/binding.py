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

PDA_OK, PDA_ERR_INVALID_ARG, PDA_ERR_UNSUPPORTED, PDA_ERR_HIP, PDA_ERR_NOMEM = 0, 1, 2, 3, 4
PDA_MAX_PARTIALS = 16
PDA_NOALLOC_MAX_SLOTS = 576
PDA_MAX_KEY_RANGES = 16
PDA_MAX_LOCAL_HEADS = 64
PDA_SINK_HEAD_MAJOR, PDA_SINK_TOKEN_ARRIVAL, PDA_SINK_TOKEN_FINAL = 0, 1, 2


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
    lib.pda_attn_fwd_strided.argtypes = [vp, vp, vp, fp, fp, i32, i32, i64, i64, i32] + [i64] * 8 + [f32, i64, i64, vp]
    lib.pda_attn_fwd_strided.restype = i32
    lib.pda_attn_fwd_noalloc.argtypes = [vp, vp, vp, fp, fp, i32, i32, i64, i64, i32, f32, i64, i64, vp]
    lib.pda_attn_fwd_noalloc.restype = i32
    lib.pda_attn_fwd_variant.argtypes = [vp, vp, vp, fp, fp, i32, i32, i64, i64, i32, f32, i64, i32, vp]
    lib.pda_attn_fwd_variant.restype = i32
    lib.pda_attn_tail_plan.argtypes = [i32, i32, i64, i64, i32, i32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32),
                                       C.POINTER(i64), C.POINTER(i64)]
    lib.pda_attn_tail_plan.restype = i32
    lib.pda_attn_merge.argtypes = [C.POINTER(vp), C.POINTER(vp), i32, fp, fp, i64, i32, vp]
    lib.pda_attn_merge.restype = i32
    lib.pda_headchunk_run.argtypes = [vp, vp, vp, fp, fp, i32, i32, i64, i64, i32, f32, i64, i32, vp, vp, fp,
                                      C.POINTER(f32), C.POINTER(f32)]
    lib.pda_headchunk_run.restype = i32
    lib.pda_headchunk_run_ex.argtypes = [vp, vp, vp, fp, fp, i32, i32, i64, i64, i32, f32, i64, C.POINTER(i32), i32,
                                         i32, i32, vp, vp, fp, C.POINTER(f32), C.POINTER(f32)]
    lib.pda_headchunk_run_ex.restype = i32
    lib.pda_pipesp_postprocess.argtypes = [C.POINTER(vp), i32, i32, i64, fp, i64, i32, vp]
    lib.pda_pipesp_postprocess.restype = i32
    lib.pda_pack_heads.argtypes = [fp, vp, i32, i64, i32, i32, i32, f32, vp]
    lib.pda_attn_fwd_bf16out.argtypes = [vp, vp, vp, vp, fp, i32, i32, i64, i64, i32, f32, i64, vp]
    lib.pda_attn_fwd_bf16out.restype = i32
    lib.pda_attn_fwd_base2.argtypes = [vp, vp, vp, fp, fp, i32, i32, i64, i64, i32, i64, vp]
    lib.pda_attn_fwd_base2.restype = i32
    lib.pda_pack_heads.restype = i32
    f64 = C.c_double
    lib.pda_plan_n_decode.argtypes = [f64, f64, i32, C.POINTER(i32)]
    lib.pda_plan_n_decode.restype = i32
    lib.pda_plan_aco.argtypes = [f64, f64, i32, i32, C.POINTER(f64), C.POINTER(f64), C.POINTER(f64)]
    lib.pda_plan_aco.restype = i32
    lib.pda_plan_head_padding.argtypes = [i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    lib.pda_plan_head_padding.restype = i32
    lib.pda_plan_ragged_groups.argtypes = [i32, i32, C.POINTER(i32)]
    lib.pda_plan_ragged_groups.restype = i32
    lib.pda_probe_mfma_rate.argtypes = [vp, i64, i64, C.POINTER(f32), C.POINTER(f32), vp]
    lib.pda_probe_mfma_rate.restype = i32
    lib.pda_probe_loop_rate.argtypes = [vp, i64, i64, i32, C.POINTER(f32), C.POINTER(f32), vp]
    lib.pda_probe_loop_rate.restype = i32
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


def attn_fwd_noalloc(q, k, v, out, lse, scale: float, kv_valid_len: Optional[int] = None, q_offset: int = 0, stream=None):
    """pda_attn_fwd_noalloc: attn_fwd with the partials of cut tiles in the library's static device buffer."""
    import torch
    B, H, Sq, d = q.shape
    Skv = k.shape[2]
    _expect(q, torch.bfloat16, (B, H, Sq, d), "q")
    _expect(k, torch.bfloat16, (B, H, Skv, d), "k")
    _expect(v, torch.bfloat16, (B, H, Skv, d), "v")
    _expect(out, torch.float32, (B, H, Sq, d), "out")
    _expect(lse, torch.float32, (B, H, Sq), "lse")
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    _check(lib.pda_attn_fwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, Sq, Skv, d, float(scale),
                                    n_v, int(q_offset), _stream_handle(stream)))
    return out, lse


def attn_fwd_variant(q, k, v, out, lse, scale: float, variant: int, kv_valid_len: Optional[int] = None, stream=None):
    """pda_attn_fwd_variant: attn_fwd with an explicit kernel choice (testing aid)."""
    import torch
    B, H, Sq, d = q.shape
    Skv = k.shape[2]
    _expect(q, torch.bfloat16, (B, H, Sq, d), "q")
    _expect(k, torch.bfloat16, (B, H, Skv, d), "k")
    _expect(v, torch.bfloat16, (B, H, Skv, d), "v")
    _expect(out, torch.float32, (B, H, Sq, d), "out")
    _expect(lse, torch.float32, (B, H, Sq), "lse")
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    _check(lib.pda_attn_fwd_variant(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, Sq, Skv, d, float(scale),
                                    n_v, int(variant), _stream_handle(stream)))
    return out, lse


def attn_tail_plan(B: int, H: int, Sq: int, kv_valid_len: int, d: int, n_cu: int = 0):
    """pda_attn_tail_plan: dict(n_tiles, n_cut, split, part_offsets, workspace_slots); part_offsets lists the
    split + 1 boundaries of the key ranges of a cut tile ([] if nothing is cut); n_cu = 0 asks the current device."""
    a, b, c, f = C.c_int64(0), C.c_int64(0), C.c_int(0), C.c_int64(0)
    offs = (C.c_int64 * (PDA_MAX_KEY_RANGES + 1))()
    _check(lib.pda_attn_tail_plan(int(B), int(H), int(Sq), int(kv_valid_len), int(d), int(n_cu),
                                  C.byref(a), C.byref(b), C.byref(c), offs, C.byref(f)))
    return {"n_tiles": a.value, "n_cut": b.value, "split": c.value,
            "part_offsets": [offs[j] for j in range(c.value + 1)] if c.value > 1 else [], "workspace_slots": f.value}


def attn_fwd_bf16out(q, k, v, out, lse, scale: float, kv_valid_len: Optional[int] = None, stream=None):
    """pda_attn_fwd_bf16out: as attn_fwd with out [B,H,Sq,d] in bf16."""
    import torch
    B, H, Sq, d = q.shape
    Skv = k.shape[2]
    _expect(q, torch.bfloat16, (B, H, Sq, d), "q")
    _expect(k, torch.bfloat16, (B, H, Skv, d), "k")
    _expect(v, torch.bfloat16, (B, H, Skv, d), "v")
    _expect(out, torch.bfloat16, (B, H, Sq, d), "out")
    _expect(lse, torch.float32, (B, H, Sq), "lse")
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    _check(lib.pda_attn_fwd_bf16out(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, Sq, Skv, d, float(scale),
                                    n_v, _stream_handle(stream)))
    return out, lse


def attn_fwd_base2(q, k, v, out, lse, kv_valid_len: Optional[int] = None, stream=None):
    """pda_attn_fwd_base2: as attn_fwd with the scores q.k already in log2 units (weights 2^(q.k))."""
    import torch
    B, H, Sq, d = q.shape
    Skv = k.shape[2]
    _expect(q, torch.bfloat16, (B, H, Sq, d), "q")
    _expect(k, torch.bfloat16, (B, H, Skv, d), "k")
    _expect(v, torch.bfloat16, (B, H, Skv, d), "v")
    _expect(out, torch.float32, (B, H, Sq, d), "out")
    _expect(lse, torch.float32, (B, H, Sq), "lse")
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    _check(lib.pda_attn_fwd_base2(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, Sq, Skv, d, n_v,
                                  _stream_handle(stream)))
    return out, lse


def _view_strides(t, inner, name):
    """(batch stride, head stride) of a [B,H,S,...] view whose rows are compact."""
    if not t.is_cuda:
        raise ValueError(f"{name}: expected a cuda tensor")
    st = t.stride()
    if inner == 2 and (st[3] != 1 or st[2] != t.shape[3]):
        raise ValueError(f"{name}: rows must be compact (stride {st})")
    if inner == 1 and st[2] != 1:
        raise ValueError(f"{name}: rows must be compact (stride {st})")
    return int(st[0]), int(st[1])


def attn_fwd_strided(q, k, v, out, lse, scale: float, kv_valid_len: Optional[int] = None, q_offset: int = 0, stream=None):
    """pda_attn_fwd_strided: as attn_fwd, on [B,H,S,d] VIEWS (e.g. x[:, :, a:b]) with compact rows; no copies."""
    import torch
    B, H, Sq, d = q.shape
    Skv = k.shape[2]
    if q.dtype != torch.bfloat16 or k.dtype != torch.bfloat16 or v.dtype != torch.bfloat16:
        raise ValueError("q/k/v: expected bf16")
    if out.dtype != torch.float32 or lse.dtype != torch.float32:
        raise ValueError("out/lse: expected fp32")
    if tuple(k.shape) != (B, H, Skv, d) or tuple(v.shape) != (B, H, Skv, d) or tuple(out.shape) != (B, H, Sq, d) \
            or tuple(lse.shape) != (B, H, Sq):
        raise ValueError("shape mismatch")
    qs, ks, vs, os_, ls = (_view_strides(q, 2, "q"), _view_strides(k, 2, "k"), _view_strides(v, 2, "v"),
                           _view_strides(out, 2, "out"), _view_strides(lse, 1, "lse"))
    if ks != vs:
        raise ValueError("k and v must share their strides")
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    _check(lib.pda_attn_fwd_strided(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, Sq, Skv, d,
                                    qs[0], qs[1], ks[0], ks[1], os_[0], os_[1], ls[0], ls[1],
                                    float(scale), n_v, int(q_offset), _stream_handle(stream)))
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


def headchunk_run_ex(q, k, v, out, lse, scale: float, group_sizes: Sequence[int], compute_stream, drain_stream,
                     kv_valid_len: Optional[int] = None, sink=None, sp_ranks: int = 1,
                     sink_layout: int = PDA_SINK_HEAD_MAJOR, timed: bool = False):
    """pda_headchunk_run_ex.  sink is [B,H,Sq,d] (head-major layout) or [B,Sq,H,d] (token-major layouts)."""
    import torch
    B, H, Sq, d = q.shape
    Skv = k.shape[2]
    _expect(q, torch.bfloat16, (B, H, Sq, d), "q")
    _expect(k, torch.bfloat16, (B, H, Skv, d), "k")
    _expect(v, torch.bfloat16, (B, H, Skv, d), "v")
    _expect(out, torch.float32, (B, H, Sq, d), "out")
    _expect(lse, torch.float32, (B, H, Sq), "lse")
    if sink is not None:
        _expect(sink, torch.float32, (B, H, Sq, d) if sink_layout == PDA_SINK_HEAD_MAJOR else (B, Sq, H, d), "sink")
    n_v = Skv if kv_valid_len is None else int(kv_valid_len)
    n_groups = len(group_sizes)
    sizes = (C.c_int * max(n_groups, 1))(*[int(x) for x in group_sizes])
    gms = (C.c_float * max(n_groups, 1))() if timed else None
    tms = C.c_float(0.0) if timed else None
    _check(lib.pda_headchunk_run_ex(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, Sq, Skv, d, float(scale),
                                    n_v, sizes, n_groups, int(sp_ranks), int(sink_layout),
                                    _stream_handle(compute_stream), _stream_handle(drain_stream), _ptr(sink),
                                    gms if timed else None, C.byref(tms) if timed else None))
    if timed:
        return [gms[i] for i in range(n_groups)], tms.value
    return None


def pipesp_postprocess(chunks: Sequence, h: int, n: int, hidden, chunk_row_stride: Optional[int] = None, stream=None):
    """pda_pipesp_postprocess: h chunks [rows,n,D] fp32 -> hidden [rows,n*h,D] fp32.

    chunks may also be ONE concatenated tensor [rows,h*n,D]; its h slices are then passed with the
    concatenated tensor's row stride.
    """
    import torch
    rows, HH, D = hidden.shape
    if HH != h * n:
        raise ValueError("hidden: middle axis must be n*h")
    _expect(hidden, torch.float32, (rows, h * n, D), "hidden")
    if hasattr(chunks, "data_ptr"):
        _expect(chunks, torch.float32, (rows, h * n, D), "t_mod")
        ptrs = [chunks.data_ptr() + j * n * D * 4 for j in range(h)]
        stride = h * n * D if chunk_row_stride is None else int(chunk_row_stride)
    else:
        if len(chunks) != h:
            raise ValueError("need h chunks")
        for j, c in enumerate(chunks):
            _expect(c, torch.float32, (rows, n, D), f"chunk {j}")
        ptrs = [c.data_ptr() for c in chunks]
        stride = n * D if chunk_row_stride is None else int(chunk_row_stride)
    arr = (C.c_void_p * max(h, 1))(*ptrs)
    _check(lib.pda_pipesp_postprocess(arr, int(h), int(n), stride, _ptr(hidden), rows, D, _stream_handle(stream)))
    return hidden


def pack_heads(x, y, unit_rms: bool, premul: float = 1.0, stream=None):
    """pda_pack_heads: x [B,S,H,d] fp32 -> y [B,H,S,d] bf16 (every element times premul before rounding)."""
    import torch
    B, S, H, d = x.shape
    _expect(x, torch.float32, (B, S, H, d), "x")
    _expect(y, torch.bfloat16, (B, H, S, d), "y")
    _check(lib.pda_pack_heads(_ptr(x), _ptr(y), B, S, H, d, 1 if unit_rms else 0, float(premul), _stream_handle(stream)))
    return y


def plan_n_decode(t_denoise: float, t_decode: float, N: int) -> int:
    out = C.c_int(0)
    _check(lib.pda_plan_n_decode(float(t_denoise), float(t_decode), int(N), C.byref(out)))
    return out.value


def plan_aco(t_L: float, t_A: float, n_denoise: int, n_decode: int):
    """(T_baseline, T_coop, speed-up S)."""
    a, b, c = C.c_double(0), C.c_double(0), C.c_double(0)
    _check(lib.pda_plan_aco(float(t_L), float(t_A), int(n_denoise), int(n_decode), C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def plan_head_padding(H: int, n_denoise: int):
    """(padded heads, heads per GPU, GPUs effectively needed)."""
    a, b, c = C.c_int(0), C.c_int(0), C.c_int(0)
    _check(lib.pda_plan_head_padding(int(H), int(n_denoise), C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def plan_ragged_groups(H: int, n: int):
    arr = (C.c_int * max(int(n), 1))()
    _check(lib.pda_plan_ragged_groups(int(H), int(n), arr))
    return [arr[i] for i in range(int(n))]


def probe_mfma_rate(operands, mfma_per_wave: int = 1 << 20, stream=None):
    """pda_probe_mfma_rate on a bf16 tensor: (TFLOP/s, ms) of an MFMA-only loop fed with its values."""
    import torch
    if operands.dtype != torch.bfloat16 or not operands.is_contiguous() or not operands.is_cuda:
        raise ValueError("operands: expected a contiguous cuda bf16 tensor")
    tf, ms = C.c_float(0.0), C.c_float(0.0)
    _check(lib.pda_probe_mfma_rate(_ptr(operands), operands.numel(), int(mfma_per_wave), C.byref(tf), C.byref(ms),
                                   _stream_handle(stream)))
    return tf.value, ms.value


def probe_loop_rate(operands, mix: int, mfma_per_wave: int = 1 << 20, stream=None):
    """pda_probe_loop_rate: (TFLOP/s, ms) of the MFMA loop with the attention loop's other instruction classes (mix 0..3)."""
    import torch
    if operands.dtype != torch.bfloat16 or not operands.is_contiguous() or not operands.is_cuda:
        raise ValueError("operands: expected a contiguous cuda bf16 tensor")
    tf, ms = C.c_float(0.0), C.c_float(0.0)
    _check(lib.pda_probe_loop_rate(_ptr(operands), operands.numel(), int(mfma_per_wave), int(mix), C.byref(tf), C.byref(ms),
                                   _stream_handle(stream)))
    return tf.value, ms.value
