"""Host-side checks of the C ABI: the library loads, exports every declared symbol, and rejects
bad arguments before touching the device (so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pda():
    import paper_2511_12056_amd as pda
    return pda


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "pipedit_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pda_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(pda):
    names = _declared_symbols()
    assert names == ["pda_attn_fwd", "pda_attn_fwd_base2", "pda_attn_fwd_bf16out", "pda_attn_fwd_noalloc", "pda_attn_fwd_strided",
                     "pda_attn_fwd_variant", "pda_attn_merge", "pda_attn_tail_plan",
                     "pda_headchunk_run", "pda_headchunk_run_ex", "pda_last_error",
                     "pda_pack_heads", "pda_pipesp_postprocess", "pda_plan_aco", "pda_plan_head_padding",
                     "pda_plan_n_decode", "pda_plan_ragged_groups", "pda_probe_loop_rate", "pda_probe_mfma_rate", "pda_version"]
    lib = C.CDLL(pda.lib_path())
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_last_error_are_callable(pda):
    assert pda.version() >= 100
    assert isinstance(pda.last_error(), str)


def _fwd(pda, q=8, k=8, v=8, out=8, lse=8, B=1, H=1, Sq=8, Skv=8, d=64, scale=1.0, n_v=8, qoff=0):
    # small integers stand in for (16-byte aligned multiples are needed: use 16*x) device addresses;
    # every call below must fail validation before any of them is dereferenced
    return pda.lib.pda_attn_fwd(q * 16 or None, k * 16 or None, v * 16 or None, out * 16 or None, lse * 16 or None,
                                B, H, Sq, Skv, d, scale, n_v, qoff, None)


def test_attn_fwd_rejects_bad_arguments(pda):
    assert _fwd(pda, d=32) == 2 and "head dim" in pda.last_error()
    assert _fwd(pda, n_v=9) == 1 and "kv_valid_len" in pda.last_error()
    assert _fwd(pda, n_v=-1) == 1
    assert _fwd(pda, Sq=-1) == 1
    assert _fwd(pda, scale=-0.5) == 1
    assert _fwd(pda, scale=float("nan")) == 1
    assert _fwd(pda, q=0) == 1 and "null" in pda.last_error()
    assert _fwd(pda, qoff=-3) == 1 and "q_offset" in pda.last_error()
    assert _fwd(pda, B=70000, H=1) == 2
    assert pda.lib.pda_attn_fwd(8, 16, 16, 16, 16, 1, 1, 8, 8, 64, 1.0, 8, 0, None) == 2      # misaligned q
    # empty problems succeed without touching anything
    assert _fwd(pda, q=0, k=0, v=0, out=0, lse=0, Sq=0) == 0
    assert _fwd(pda, q=0, k=0, v=0, out=0, lse=0, B=0) == 0


def test_merge_rejects_bad_arguments(pda):
    arr = (C.c_void_p * 2)(64, 128)
    f = pda.lib.pda_attn_merge
    assert f(arr, arr, 0, 64, None, 4, 128, None) == 1
    assert f(arr, arr, 17, 64, None, 4, 128, None) == 2
    assert f(arr, arr, 2, 64, None, -1, 128, None) == 1
    assert f(arr, arr, 2, 64, None, 4, 130, None) == 2
    assert f(arr, arr, 2, None, None, 4, 128, None) == 1
    assert f(None, arr, 2, 64, None, 4, 128, None) == 1
    bad = (C.c_void_p * 2)(64, None)
    assert f(bad, arr, 2, 64, None, 4, 128, None) == 1
    assert f(arr, arr, 2, 64, 128, 4, 128, None) == 1 and "alias" in pda.last_error()     # lse_out == lses[1]
    assert f(arr, arr, 2, 64, None, 0, 128, None) == 0


def test_headchunk_rejects_bad_arguments(pda):
    f = pda.lib.pda_headchunk_run
    args = [16, 16, 16, 16, 16, 1, 4, 8, 8, 64, 1.0, 8]
    assert f(*args, 0, 16, 32, None, None, None) == 1 and "heads_per_group" in pda.last_error()
    assert f(*args, 2, 16, 16, None, None, None) == 1 and "streams" in pda.last_error()
    assert f(*args, 2, 16, 32, 16, None, None) == 1 and "overlap" in pda.last_error()    # sink == out
    assert f(*args, 2, 16, 32, 16 + 1024, None, None) == 1 and "overlap" in pda.last_error()   # sink inside out (8 KB)
    assert f(*(args[:7] + [0] + args[8:]), 2, 16, 32, 16 + 8192, None, None) == 0              # Sq = 0: nothing to overlap
    assert f(*args[:9], 48, 1.0, 8, 2, 16, 32, None, None, None) == 2
    # an empty problem reports zero times
    gms = (C.c_float * 2)(1.0, 1.0)
    tot = C.c_float(1.0)
    assert f(None, None, None, None, None, 1, 4, 0, 8, 64, 1.0, 8, 2, 16, 32, None, gms, C.byref(tot)) == 0
    assert list(gms) == [0.0, 0.0] and tot.value == 0.0


def test_headchunk_ex_rejects_bad_arguments(pda):
    f = pda.lib.pda_headchunk_run_ex
    args = [16, 16, 16, 16, 16, 1, 4, 8, 8, 64, 1.0, 8]
    g22 = (C.c_int * 2)(2, 2)
    g21 = (C.c_int * 2)(2, 1)
    g40 = (C.c_int * 2)(4, 0)
    assert f(*args, g21, 2, 1, 0, 16, 32, None, None, None) == 1 and "sum" in pda.last_error()
    assert f(*args, g40, 2, 1, 0, 16, 32, None, None, None) == 1 and "group_sizes[1]" in pda.last_error()
    assert f(*args, None, 2, 1, 0, 16, 32, None, None, None) == 1
    assert f(*args, g22, 2, 1, 7, 16, 32, None, None, None) == 1 and "sink_layout" in pda.last_error()
    assert f(*args, g22, 2, 0, 0, 16, 32, None, None, None) == 1 and "sp_ranks" in pda.last_error()
    assert f(*args, g22, 2, 2, 1, 16, 32, None, None, None) == 1 and "needs a sink" in pda.last_error()
    assert f(*args, g22, 2, 3, 2, 16, 32, 64, None, None) == 1 and "multiple" in pda.last_error()
    assert f(*args, g22, 2, 2, 2, 16, 16, 64, None, None) == 1 and "streams" in pda.last_error()


def test_postprocess_rejects_bad_arguments(pda):
    f = pda.lib.pda_pipesp_postprocess
    arr = (C.c_void_p * 3)(1 << 20, 2 << 20, 3 << 20)
    hid = 16 << 20
    assert f(arr, 0, 2, 256, hid, 4, 128, None) == 1
    assert f(arr, 3, 0, 256, hid, 4, 128, None) == 1
    assert f(arr, 65, 2, 256, hid, 4, 128, None) == 2 and "PDA_MAX_LOCAL_HEADS" in pda.last_error()
    assert f(arr, 3, 2, 256, hid, -1, 128, None) == 1
    assert f(arr, 3, 2, 256, hid, 4, 126, None) == 2
    assert f(arr, 3, 2, 255, hid, 4, 128, None) == 1 and "chunk_row_stride" in pda.last_error()
    assert f(arr, 3, 2, 254, hid, 4, 128, None) == 1
    assert f(None, 3, 2, 256, hid, 4, 128, None) == 1
    assert f(arr, 3, 2, 256, None, 4, 128, None) == 1
    assert f(arr, 3, 2, 256, hid + 4, 4, 128, None) == 2
    bad = (C.c_void_p * 3)(1 << 20, None, 3 << 20)
    assert f(bad, 3, 2, 256, hid, 4, 128, None) == 1
    assert f(arr, 3, 2, 256, (2 << 20) + 1024, 4, 128, None) == 1 and "overlaps" in pda.last_error()
    assert f(arr, 3, 2, 256, hid, 0, 128, None) == 0


def test_pack_rejects_bad_arguments(pda):
    f = pda.lib.pda_pack_heads
    assert f(64, 128, 1, 8, 2, 32, 1, 1.0, None) == 2 and "head dim" in pda.last_error()
    assert f(64, 128, -1, 8, 2, 64, 1, 1.0, None) == 1
    assert f(None, 128, 1, 8, 2, 64, 1, 1.0, None) == 1
    assert f(64, 72, 1, 8, 2, 64, 1, 1.0, None) == 2
    assert f(64, 64, 1, 8, 2, 64, 1, 1.0, None) == 1 and "alias" in pda.last_error()
    assert f(64, 128, 1, 8, 2, 64, 1, float("inf"), None) == 1 and "premul" in pda.last_error()
    assert f(None, None, 1, 0, 2, 64, 1, 1.0, None) == 0
    g = pda.lib.pda_attn_fwd_base2
    assert g(128, 128, 128, 128, 128, 1, 1, 8, 8, 32, 8, None) == 2
    assert g(128, 128, 128, 128, 128, 1, 1, 8, 8, 64, 9, None) == 1
    assert g(None, 128, 128, 128, 128, 1, 1, 8, 8, 64, 8, None) == 1
    assert g(None, None, None, None, None, 1, 1, 0, 8, 64, 8, None) == 0


def test_planner_rejects_bad_arguments(pda):
    out = C.c_int(0)
    assert pda.lib.pda_plan_n_decode(1.0, 1.0, 1, C.byref(out)) == 1
    assert pda.lib.pda_plan_n_decode(0.0, 1.0, 8, C.byref(out)) == 1
    assert pda.lib.pda_plan_n_decode(1.0, float("inf"), 8, C.byref(out)) == 1
    assert pda.lib.pda_plan_n_decode(1.0, 1.0, 8, None) == 1
    assert pda.lib.pda_plan_aco(0.0, 0.0, 4, 4, None, None, None) == 1
    assert pda.lib.pda_plan_aco(1.0, 1.0, 0, 4, None, None, None) == 1
    assert pda.lib.pda_plan_aco(1.0, -1.0, 4, 4, None, None, None) == 1
    assert pda.lib.pda_plan_aco(1.0, 1.0, 4, 4, None, None, None) == 0
    assert pda.lib.pda_plan_head_padding(0, 4, None, None, None) == 1
    assert pda.lib.pda_plan_ragged_groups(4, 0, C.byref(out)) == 1
    assert pda.lib.pda_plan_ragged_groups(4, 2, None) == 1


def test_probe_rejects_bad_arguments(pda):
    f = pda.lib.pda_probe_mfma_rate
    out = C.c_float(0)
    assert f(None, 8192, 1000, C.byref(out), None, None) == 1
    assert f(64, 100, 1000, C.byref(out), None, None) == 1
    assert f(64, 8192, 0, C.byref(out), None, None) == 1
    assert f(64, 8192, 1000, None, None, None) == 1
    assert f(72, 8192, 1000, C.byref(out), None, None) == 2
    g = pda.lib.pda_probe_loop_rate
    assert g(64, 8192, 1000, 4, C.byref(out), None, None) == 1 and "mix" in pda.last_error()
    assert g(64, 8192, 1000, -1, C.byref(out), None, None) == 1
    assert g(None, 8192, 1000, 1, C.byref(out), None, None) == 1


def test_attn_fwd_strided_rejects_bad_arguments(pda):
    f = pda.lib.pda_attn_fwd_strided
    base = [128, 128, 128, 128, 128, 2, 2, 8, 8, 64]
    good = [2048, 1024, 2048, 1024, 2048, 1024, 32, 16]

    def call(strides, scale=1.0, n_v=8, qoff=0, shape=None):
        return f(*(shape or base), *strides, scale, n_v, qoff, None)

    assert call(good, n_v=9) == 1
    assert call(good, qoff=-1) == 1
    assert call([2048, 1020] + good[2:]) == 2 and "multiples of 8" in pda.last_error()
    assert call(good[:4] + [2048, 1022] + good[6:]) == 2 and "multiples of 4" in pda.last_error()
    assert call(good[:5] + [256] + good[6:]) == 1 and "head stride" in pda.last_error()
    assert call(good[:7] + [4]) == 1
    assert call(good[:4] + [1024, 1024] + good[6:]) == 1 and "batch stride" in pda.last_error()
    assert call([-8] + good[1:]) == 1
    assert call(good, shape=[128, 128, 128, 128, 128, 2, 2, 0, 8, 64]) == 0      # empty: no-op


def test_header_is_plain_c(tmp_path):
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "hdr.c"
    src.write_text('#include "pipedit_attn.h"\nint main(void) { return PDA_MAX_PARTIALS == 16 ? 0 : 1; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)


def test_bf16out_rejects_bad_arguments(pda):
    f = pda.lib.pda_attn_fwd_bf16out
    assert f(128, 128, 128, 128, 128, 1, 1, 8, 8, 96, 1.0, 8, None) == 2 and "head dim" in pda.last_error()
    assert f(128, 128, 128, 128, 128, 1, 1, 8, 8, 128, 1.0, 9, None) == 1
    assert f(128, 128, 128, None, 128, 1, 1, 8, 8, 128, 1.0, 8, None) == 1
    assert f(None, None, None, None, None, 0, 1, 8, 8, 128, 1.0, 8, None) == 0


def test_variant_entry_rejects_bad_arguments(pda):
    f = pda.lib.pda_attn_fwd_variant
    assert f(128, 128, 128, 128, 128, 1, 1, 8, 8, 128, 1.0, 8, 4, None) == 1 and "variant" in pda.last_error()
    assert f(128, 128, 128, 128, 128, 1, 1, 8, 8, 128, 1.0, 8, -1, None) == 1
    assert f(128, 128, 128, 128, 128, 1, 1, 8, 8, 32, 1.0, 8, 1, None) == 2
    assert f(None, None, None, None, None, 1, 1, 0, 8, 128, 1.0, 8, 2, None) == 0


def test_tail_plan_matches_the_rule_restated_in_python(pda):
    """pda_attn_tail_plan is host arithmetic: compare it with the rule written out independently
    (tests/util.py: tail_plan) over a sweep of launch sizes and CU counts, and pin the plans of the
    workloads (256 compute units)."""
    from tests.util import tail_plan
    import numpy as np
    rng = np.random.default_rng(5)
    for _ in range(3000):
        n_cu = int(rng.choice([256, 304, 64, 1, 7]))
        BH = int(rng.integers(1, 40))
        Sq = int(rng.integers(1, 200000)) if rng.random() < 0.3 else int(rng.integers(1, 5000))
        n_v = int(rng.choice([0, 1, 511, 512, 1023, 1024, 1535, 1536, 2047, 2048, int(rng.integers(1, 200000))]))
        d = int(rng.choice([64, 128]))
        got = pda.attn_tail_plan(1, BH, Sq, n_v, d, n_cu)
        want = tail_plan(BH, Sq, n_v, d, n_cu)
        assert got == want, (n_cu, BH, Sq, n_v, d, got, want)
    # the workloads: one 3-head group at 720p is 1 398 tiles = 5 x 256 + 118; round(768/118) = 7 ranges, 5 fit the
    # workspace; after five rounds of whole tiles the ranges decrease by 5/8 each (41 / 26 / 16 / 10 / 6 % of the keys)
    assert pda.attn_tail_plan(1, 3, 119056, 119056, 128, 256) == {
        "n_tiles": 1398, "n_cut": 118, "split": 5, "part_offsets": [0, 49344, 80192, 99456, 111488, 119056], "workspace_slots": 472}
    # six heads at 720p: 2 796 tiles = 10 x 256 + 236, three ranges of 50 / 31 / 19 %
    assert pda.attn_tail_plan(1, 6, 119056, 119056, 128, 256) == {
        "n_tiles": 2796, "n_cut": 236, "split": 3, "part_offsets": [0, 59008, 95936, 119056], "workspace_slots": 472}
    # 24 heads x 9 600: 912 tiles = 3 x 256 + 144 (more than half a round): a long first range for 144 CUs,
    # two short ones that the other 112 work off three each: A = 3/5 of the keys plus 1 %
    assert pda.attn_tail_plan(1, 24, 9600, 9600, 128, 256) == {
        "n_tiles": 912, "n_cut": 144, "split": 3, "part_offsets": [0, 5888, 7744, 9600], "workspace_slots": 288}
    # one head at 720p: 466 tiles = 256 + 210: k = ceil(420 / 46) = 10, A = 10/12
    assert pda.attn_tail_plan(1, 1, 119056, 119056, 128, 256) == {
        "n_tiles": 466, "n_cut": 210, "split": 3, "part_offsets": [0, 100416, 109760, 119056], "workspace_slots": 420}
    # 10 heads x 9 600: 380 tiles = 256 + 124 short ones: one round of 248 equal parts
    assert pda.attn_tail_plan(1, 10, 9600, 9600, 128, 256) == {
        "n_tiles": 380, "n_cut": 124, "split": 2, "part_offsets": [0, 4800, 9600], "workspace_slots": 124}
    # 30 heads x 9 600: four rounds of whole tiles, but short sweeps: one round of equal parts, not decreasing ones
    assert pda.attn_tail_plan(1, 30, 9600, 9600, 128, 256)["part_offsets"] == [0, 4800, 9600]
    # 24 heads x 4 800: 456 tiles = 256 + 200 of 75 key tiles: left uncut
    assert pda.attn_tail_plan(1, 24, 4800, 4800, 128, 256) == {
        "n_tiles": 456, "n_cut": 0, "split": 1, "part_offsets": [], "workspace_slots": 0}
    # one head group of the 544 x 960 clip: 792 tiles = 3 x 256 + 24, 1 055 key tiles: 10 equal ranges
    assert pda.attn_tail_plan(1, 3, 67576, 67476, 128, 256) == {
        "n_tiles": 792, "n_cut": 24, "split": 10, "part_offsets": [6784 * j for j in range(10)] + [67476], "workspace_slots": 216}
    # no plan needs more than 9/4 slots per compute unit for the parts beyond the first; the ranges of every plan
    # start at 0, end at n_v, are not empty and begin at multiples of 64
    for t in range(1, 1400):
        for n_v in (1 << 20, 12800, 8200, 8193, 51200 + t, 3300 + 7 * t):
            pl = pda.attn_tail_plan(1, 1, 256 * t, n_v, 128, 256)
            assert pl["workspace_slots"] <= 576
            if pl["split"] > 1:
                o = pl["part_offsets"]
                assert len(o) == pl["split"] + 1 and o[0] == 0 and o[-1] == n_v, (t, n_v, pl)
                assert all(b > a for a, b in zip(o, o[1:])) and all(a % 64 == 0 for a in o[:-1]), (t, n_v, pl)
    # a launch of fewer tiles than compute units: one head of the 9 600-token clip is 38 tiles, 256 // 38 = 6 ranges each
    assert pda.attn_tail_plan(1, 1, 9600, 9600, 128, 256) == {
        "n_tiles": 38, "n_cut": 38, "split": 6, "part_offsets": [1600 * j for j in range(7)], "workspace_slots": 190}
    # the tiny workload (d = 64): 8 tiles, 1 024 keys allow two ranges of 512
    assert pda.attn_tail_plan(1, 2, 1024, 1024, 64, 256) == {
        "n_tiles": 8, "n_cut": 8, "split": 2, "part_offsets": [0, 512, 1024], "workspace_slots": 8}
    # an empty key set is never cut
    assert pda.attn_tail_plan(1, 3, 5000, 0, 128, 256)["n_cut"] == 0
    assert pda.lib.pda_attn_tail_plan(1, 1, 8, 8, 32, 256, None, None, None, None, None) == 2
    assert pda.lib.pda_attn_tail_plan(1, 1, -1, 8, 128, 256, None, None, None, None, None) == 1
