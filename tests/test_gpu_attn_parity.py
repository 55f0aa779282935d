"""GPU parity of pda_attn_fwd against the fp64 oracle (element by element, through the C ABI)."""
import numpy as np
import pytest

from synth import CONFIGS, K_ID, Q_ID, V_ID, bf16_bits_to_f32, f32_to_bf16_bits, gen_qkv, gen_tensor
from tests.util import assert_close, gen_qkv_parallel, sample_rows, to_dev_bf16

pytestmark = pytest.mark.gpu


def _run(q, k, v, scale, n_v=None, q_offset=0):
    import torch
    import paper_2511_12056_amd as pda
    B, H, Sq, d = q.shape
    out = torch.full((B, H, Sq, d), float("nan"), device="cuda", dtype=torch.float32)
    lse = torch.full((B, H, Sq), float("nan"), device="cuda", dtype=torch.float32)
    pda.attn_fwd(to_dev_bf16(q), to_dev_bf16(k), to_dev_bf16(v), out, lse, scale, n_v, q_offset)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def _oracle(q, k, v, scale, n_v=None):
    from oracle import attention
    return attention(q, k, v, scale, n_v)


def test_c1_tiny_full():
    w = CONFIGS[1]
    q, k, v = gen_qkv(w.seed, w.B, w.H, w.Sq, w.Skv, w.d, unit_rms=w.unit_rms)
    o, l = _run(q, k, v, w.scale)
    ro, rl = _oracle(q, k, v, w.scale)
    e = assert_close(o, l, ro, rl, "C1")
    print("C1", e)


@pytest.mark.parametrize("B,H,Sq,Skv,d,n_v", [
    (1, 1, 32, 64, 128, None),        # exactly one tile
    (1, 1, 1, 1, 128, None),          # single query, single key
    (1, 2, 700, 901, 128, 845),       # several tiles, ragged rows and keys, masked tail inside the last tile
    (2, 3, 333, 517, 64, 500),        # batch > 1, d = 64
    (1, 1, 257, 129, 128, 65),        # mask hides whole trailing tiles
    (1, 2, 130, 4099, 128, 4097),     # long key axis, short query axis
    (1, 1, 513, 64, 64, 1),           # one valid key
    (1, 2, 700, 901, 64, 845),        # d = 64: several tiles, masked tail inside the last tile
    (1, 1, 257, 129, 64, 65),         # d = 64: mask hides whole trailing tiles
    (1, 1, 1, 1, 64, None),           # d = 64: single query, single key
    (1, 2, 130, 4099, 64, 4097),      # d = 64: long key axis, short query axis
])
def test_ragged_shapes_and_masks(B, H, Sq, Skv, d, n_v):
    q, k, v = gen_qkv(900 + Sq, B, H, Sq, Skv, d, unit_rms=False)
    scale = d ** -0.5
    o, l = _run(q, k, v, scale, n_v)
    ro, rl = _oracle(q, k, v, scale, n_v)
    assert_close(o, l, ro, rl, f"{(B, H, Sq, Skv, d, n_v)}")


@pytest.mark.parametrize("gain,d", [(4.0, 128), (8.0, 128), (8.0, 64)])
def test_peaked_scores(gain, d):
    # scores with standard deviation 4-8: outputs are O(1), the running max keeps moving
    B, H, Sq, Skv = 1, 2, 640, 2100
    q, k, v = gen_qkv(77, B, H, Sq, Skv, d, unit_rms=True)
    q = f32_to_bf16_bits(bf16_bits_to_f32(q) * np.float32(gain))
    scale = d ** -0.5
    o, l = _run(q, k, v, scale, 2050)
    ro, rl = _oracle(q, k, v, scale, 2050)
    assert_close(o, l, ro, rl, f"peaked x{gain}")


def test_scale_zero_and_empty_share():
    q, k, v = gen_qkv(5, 1, 1, 100, 200, 128, unit_rms=False)
    o, l = _run(q, k, v, 0.0, 150)
    ro, rl = _oracle(q, k, v, 0.0, 150)
    assert_close(o, l, ro, rl, "scale 0")
    o, l = _run(q, k, v, 0.1, 0)
    assert (o == 0).all() and np.isneginf(l).all()


def test_hidden_keys_are_never_read():
    B, H, Sq, Skv, d, n_v = 1, 2, 300, 777, 128, 650
    q, k, v = gen_qkv(11, B, H, Sq, Skv, d, unit_rms=True)
    o, l = _run(q, k, v, 0.09, n_v)
    kp, vp = k.copy(), v.copy()
    kp[:, :, n_v:] = 0x7FC0          # NaN payload
    vp[:, :, n_v:] = 0x7F80          # +inf payload
    o2, l2 = _run(q, kp, vp, 0.09, n_v)
    assert np.array_equal(o, o2) and np.array_equal(l, l2)


def test_q_offset_has_no_effect_and_runs_are_bitwise_reproducible():
    q, k, v = gen_qkv(12, 1, 2, 400, 900, 128, unit_rms=True)
    o, l = _run(q, k, v, 0.09)
    o2, l2 = _run(q, k, v, 0.09, None, 12345)
    assert np.array_equal(o, o2) and np.array_equal(l, l2)


def test_query_range_call_equals_rows_of_full_call():
    # a query range is a separate call on a row slice of q: same rows, same bits
    q, k, v = gen_qkv(13, 1, 1, 1000, 1500, 128, unit_rms=True)
    o, l = _run(q, k, v, 0.09)
    a, b = 391, 777
    o2, l2 = _run(np.ascontiguousarray(q[:, :, a:b]), k, v, 0.09, None, a)
    assert np.array_equal(o[:, :, a:b], o2) and np.array_equal(l[:, :, a:b], l2)


def test_invariants_on_gpu():
    # identical V rows -> that row; zero K -> mean of V and lse = ln n
    B, H, Sq, Skv, d = 1, 1, 200, 300, 128
    q, k, v = gen_qkv(14, B, H, Sq, Skv, d, unit_rms=False)
    vrow = np.tile(v[:, :, :1], (1, 1, Skv, 1))
    o, _ = _run(q, k, vrow, 0.09)
    # not exact on the GPU: probabilities are rounded to bf16 for the PV product while the
    # normaliser sums them unrounded, so the weights sum to 1 only to about 2^-9 / sqrt(keys)
    assert np.abs(o - bf16_bits_to_f32(vrow[:, :, :1])).max() < 4e-3
    o, l = _run(q, np.zeros_like(k), v, 0.09)
    vm = bf16_bits_to_f32(v).astype(np.float64).mean(axis=2, keepdims=True)
    assert np.abs(o - vm).max() < 2e-3 and np.abs(l - np.log(Skv)).max() < 1e-5


def test_c2_lowres_clip():
    w = CONFIGS[2]
    q, k, v = gen_qkv_parallel(w)
    o, l = _run(q, k, v, w.scale)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    from oracle import attention_head
    for h in (0, 11, 23):                                   # three heads in full
        ro, rl = attention_head(q[0, h], k[0, h], v[0, h], w.scale)
        e = assert_close(o[0, h], l[0, h], ro, rl, f"C2 head {h}")
        print("C2 head", h, e)
    for h in range(w.H):                                    # every head on sampled rows
        rows = sample_rows(w.Sq, 128, w.seed + h)
        ro, rl = attention_head(q[0, h], k[0, h], v[0, h], w.scale, rows=rows)
        assert_close(o[0, h][rows], l[0, h][rows], ro, rl, f"C2 head {h} sampled")


def test_c3_masked_group_sampled_rows():
    w = CONFIGS[3]
    q, k, v = gen_qkv_parallel(w)
    k[:, :, w.kv_valid_len:] = 0x7FC0                        # poison the hidden text tokens
    v[:, :, w.kv_valid_len:] = 0x7FC0
    o, l = _run(q, k, v, w.scale, w.kv_valid_len)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    from oracle import attention_head
    for h in range(w.H):
        rows = sample_rows(w.Sq, 512, w.seed + h)
        ro, rl = attention_head(q[0, h], k[0, h], v[0, h], w.scale, w.kv_valid_len, rows=rows)
        e = assert_close(o[0, h][rows], l[0, h][rows], ro, rl, f"C3 head {h}")
        print("C3 head", h, e)


def test_seeded_shape_sweep():
    """Random small and medium shapes (ragged tiles, masks inside and across tiles, several batches,
    launches whose tiles are cut into 2 to 6 key ranges) against the oracle, every element."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    rng = np.random.default_rng(20251112)
    for case in range(24):
        d = 128 if case % 3 else 64
        B = int(rng.integers(1, 3))
        H = int(rng.integers(1, 6))
        Sq = int(rng.integers(1, 900))
        Skv = int(rng.choice([rng.integers(1, 700), rng.integers(1500, 4200)]))
        if case % 3 == 2:
            Skv = int(rng.integers(12800, 40000))            # long enough for the launch's tiles to be cut into key ranges
        n_v = int(rng.choice([Skv, rng.integers(0, Skv + 1), max(0, Skv - int(rng.integers(0, 70)))]))
        scale = float(rng.choice([d ** -0.5, 0.02, 0.3]))
        qb, kb, vb = gen_qkv(1000 + case, B, H, Sq, Skv, d, unit_rms=bool(case % 2))
        q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
        out = torch.full((B, H, Sq, d), float("nan"), device="cuda")
        lse = torch.full((B, H, Sq), float("nan"), device="cuda")
        print("sweep case", case, dict(B=B, H=H, Sq=Sq, Skv=Skv, n_v=n_v, d=d, scale=scale), flush=True)
        pda.attn_fwd(q, k, v, out, lse, scale, n_v)
        torch.cuda.synchronize()
        ro, rl = attention(qb, kb, vb, scale, n_v)
        o, l = out.cpu().numpy(), lse.cpu().numpy()
        if n_v == 0:
            assert (o == 0).all() and np.isneginf(l).all()
        else:
            assert_close(o, l, ro, rl, f"sweep case {case}")


@pytest.mark.parametrize("d", [128, 64])
def test_scores_far_above_the_first_tile_take_the_running_max_path(d):
    """The kernel's first attempt keeps the max of a row's first key tile as its only reference; rows
    whose later scores exceed it by more than ~2^64 (in powers of two) would overflow and must be
    recomputed with the running max.  Keys beyond the first tile score hundreds to thousands above
    it here, for some rows only, in some heads only, and once in the middle of a tile sweep."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    rng = np.random.default_rng(77)
    B, H, Sq, Skv = 1, 3, 600, 1500
    q = rng.standard_normal((B, H, Sq, d)).astype(np.float32)
    k = (rng.standard_normal((B, H, Skv, d)) * 0.01).astype(np.float32)
    v = rng.standard_normal((B, H, Skv, d)).astype(np.float32)
    k[:, 0, 300:] *= 3000.0                      # head 0: every key after the 4th tile is huge for every row
    k[0, 1, 1111] = q[0, 1, 5] * 40.0            # head 1: one outlier key aligned with query row 5
    # head 2: ordinary
    qb, kb, vb = f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)
    for n_v in (Skv, 1200):
        out = torch.full((B, H, Sq, d), float("nan"), device="cuda")
        lse = torch.full((B, H, Sq), float("nan"), device="cuda")
        pda.attn_fwd(to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb), out, lse, 1.0, n_v)
        torch.cuda.synchronize()
        ro, rl = attention(qb, kb, vb, 1.0, n_v)
        assert np.abs(rl).max() > 500                                   # the inputs do what they are meant to
        assert_close(out.cpu().numpy(), lse.cpu().numpy(), ro, rl, f"overflow redo n_v={n_v}")


def test_reference_tilings_and_forced_second_sweep_agree_with_the_oracle():
    """pda_attn_fwd_variant selects the reference tilings (1, 2) or forces the default kernel's
    running-max sweep on every item (3); all of them against the oracle."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    shapes = [(1, 2, 515, 1100, 1050, 0.09, 128), (2, 1, 300, 4200, 4200, 0.3, 128), (1, 3, 777, 64, 40, 0.0883883, 128),
              (1, 24, 700, 12900, 12850, 0.0883883, 128),           # every tile cut in three
              (1, 2, 515, 1100, 1050, 0.125, 64), (1, 24, 700, 12900, 12850, 0.125, 64), (2, 1, 300, 4200, 4200, 0.3, 64)]
    for i, (B, H, Sq, Skv, n_v, scale, d) in enumerate(shapes):
        qb, kb, vb = gen_qkv(500 + i, B, H, Sq, Skv, d, unit_rms=bool(i % 2))
        ro, rl = attention(qb, kb, vb, scale, n_v)
        q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
        for variant in (0, 1, 2, 3):
            out = torch.full((B, H, Sq, d), float("nan"), device="cuda"); lse = torch.full((B, H, Sq), float("nan"), device="cuda")
            print("variant", variant, "shape", i, flush=True)
            pda.attn_fwd_variant(q, k, v, out, lse, scale, variant, n_v)
            torch.cuda.synchronize()
            assert_close(out.cpu().numpy(), lse.cpu().numpy(), ro, rl, f"variant {variant} shape {i}")


@pytest.mark.parametrize("d", [128, 64])
def test_large_finite_values_take_the_running_max_path(d):
    """With the fixed reference of the first sweep the weights may reach 2^64; times finite V entries
    of magnitude up to 2^100 that overflows the output accumulators although every row sum stays in
    range.  Such items must be redone with the running max (weights <= 2^8), where the result is
    finite like the oracle's.  Scores rise by tens of log2 units after the first key tile."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    rng = np.random.default_rng(99)
    B, H, Sq, Skv = 1, 3, 520, 1300
    q = rng.standard_normal((B, H, Sq, d)).astype(np.float32)
    k = (rng.standard_normal((B, H, Skv, d)) * 0.05).astype(np.float32)
    v = rng.standard_normal((B, H, Skv, d)).astype(np.float32)
    k[:, 0, 64:] *= np.float32(12.0 * (128 / d) ** 0.5)    # head 0: scores grow ~40 log2 units after the first tile
    k[0, 1, 700] = q[0, 1, 9] * np.float32(0.45 * 128 / d) # head 1: one key ~50 above everything for query row 9
    v[:, 0] *= np.float32(2.0 ** 100)                      # head 0: huge values everywhere
    v[:, 1] *= np.float32(2.0 ** 90)
    v[0, 2, 5::7] *= np.float32(2.0 ** 100)                # head 2: ordinary scores, some huge values (no overflow: weights <= ~2^10)
    qb, kb, vb = f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)
    out = torch.full((B, H, Sq, d), float("nan"), device="cuda")
    lse = torch.full((B, H, Sq), float("nan"), device="cuda")
    pda.attn_fwd(to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb), out, lse, 1.0)
    torch.cuda.synchronize()
    ro, rl = attention(qb, kb, vb, 1.0)
    o, l = out.cpu().numpy().astype(np.float64), lse.cpu().numpy()
    assert np.isfinite(ro).all() and np.isfinite(o).all() and np.isfinite(l).all()
    s = bf16_bits_to_f32(kb[0, 0]).astype(np.float64) @ bf16_bits_to_f32(qb[0, 0]).astype(np.float64).T
    assert (s[64:].max(axis=0) - s[:64].max(axis=0)).max() > 30    # the inputs do what they are meant to (natural-log units)
    for h in range(H):                                      # relative gates: the values span 2^100
        ref = ro[0, h]
        assert np.sqrt(((o[0, h] - ref) ** 2).sum() / (ref ** 2).sum()) <= 1e-2, h
        assert np.abs(o[0, h] - ref).max() <= 2e-2 * np.abs(ref).max(), h
    assert (np.abs(l - rl) / np.maximum(np.abs(rl), 1.0)).max() <= 1e-3


def _assert_close_bf16(o16, l, ro, rl, what):
    """The gates of the fp32 result with the rounding of the result itself added: half a bf16 step,
    2^-9 relative per element (2^-9 / sqrt(3) in the L2 norm)."""
    o = o16.astype(np.float64)
    assert np.isfinite(o).all() and np.isfinite(l).all(), what
    diff = np.abs(o - ro)
    half_ulp = np.abs(ro) * 2.0 ** -9
    assert (diff <= 2e-2 + half_ulp).all(), what
    assert diff.mean() <= 2e-3 + half_ulp.mean(), what
    assert np.sqrt((diff ** 2).sum() / (ro ** 2).sum()) <= 1e-2 + 2.0 ** -9 / np.sqrt(3.0), what
    assert (np.abs(l.astype(np.float64) - rl) / np.maximum(np.abs(rl), 1.0)).max() <= 1e-3, what


@pytest.mark.parametrize("d", [128, 64])
def test_many_key_ranges_per_cut_tile(d):
    """A launch of few tiles over a long key axis cuts every tile into the largest number of key
    ranges (16); fp32 result against the oracle, masked tail inside the last range."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    B, H, Sq, Skv, n_v = 1, 3, 600, 102500, 102440
    plan = pda.attn_tail_plan(B, H, Sq, n_v, d)
    if torch.cuda.get_device_properties(0).multi_processor_count == 256:
        assert plan["split"] == 16 and plan["n_cut"] == 9, plan
    qb, kb, vb = gen_qkv(4711, B, H, Sq, Skv, d, unit_rms=True)
    o, l = _run(qb, kb, vb, d ** -0.5, n_v)
    ro, rl = _oracle(qb, kb, vb, d ** -0.5, n_v)
    assert_close(o, l, ro, rl, f"16 key ranges, d = {d}")


@pytest.mark.parametrize("d", [128, 64])
def test_unequal_key_ranges(d):
    """A launch of one round of whole tiles plus many left-over tiles (420 tiles on 256 CUs: 164 left
    over) cuts those into a long first key range and short others; sampled rows of whole and of cut
    tiles, with the masked tail inside the last short range, against the oracle."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention_head
    B, H, Sq, Skv, n_v = 1, 20, 5200, 13100, 13050
    plan = pda.attn_tail_plan(B, H, Sq, n_v, d)
    if torch.cuda.get_device_properties(0).multi_processor_count == 256:
        o = plan["part_offsets"]
        assert plan["n_cut"] == 164 and plan["split"] == 4 and o[1] - o[0] > 2 * (o[2] - o[1]), plan
    qb, kb, vb = gen_qkv(4242, B, H, Sq, Skv, d, unit_rms=True)
    o, l = _run(qb, kb, vb, d ** -0.5, n_v)
    rng = np.random.default_rng(3)
    for h in (0, 7, 12, 13, 19):            # heads 0-11 are whole tiles, head 12 both, heads 13-19 cut (256 CUs)
        rows = np.unique(np.concatenate([[0, 255, 256, Sq - 1], rng.choice(Sq, size=120, replace=False)]))
        ro, rl = attention_head(qb[0, h], kb[0, h], vb[0, h], d ** -0.5, n_v, rows=rows)
        assert_close(o[0, h][rows], l[0, h][rows], ro, rl, f"unequal ranges, d = {d}, head {h}")


def test_decreasing_key_ranges():
    """A launch of four rounds of whole tiles plus 16 left-over tiles cuts those into key ranges of
    decreasing size (each 5/8 of the one before); sampled rows of whole and of cut tiles of the
    last head, masked tail inside the last range, against the oracle.  (The 26 heads repeat four
    generated ones.)"""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention_head
    B, H, Sq, Skv, n_v, d = 1, 26, 10100, 31100, 31000, 128
    plan = pda.attn_tail_plan(B, H, Sq, n_v, d)
    if torch.cuda.get_device_properties(0).multi_processor_count == 256:
        o = plan["part_offsets"]
        assert plan["n_tiles"] == 1040 and plan["n_cut"] == 16 and plan["split"] == 4, plan
        assert o[1] - o[0] > o[2] - o[1] > o[3] - o[2] > o[4] - o[3] >= 3200, plan
    q4, k4, v4 = gen_qkv(808, B, 4, Sq, Skv, d, unit_rms=True)
    idx = np.arange(H) % 4
    qb, kb, vb = q4[:, idx], k4[:, idx], v4[:, idx]
    o, l = _run(qb, kb, vb, d ** -0.5, n_v)
    rng = np.random.default_rng(5)
    for h in (0, 25):                       # head 25: tiles 0-23 whole, tiles 24-39 (rows 6144..) cut (256 CUs)
        rows = np.unique(np.concatenate([[0, 6143, 6144, 6400, Sq - 1], rng.choice(Sq, size=150, replace=False)]))
        ro, rl = attention_head(qb[0, h], kb[0, h], vb[0, h], d ** -0.5, n_v, rows=rows)
        assert_close(o[0, h][rows], l[0, h][rows], ro, rl, f"decreasing ranges, head {h}")
    # the same rows of equal heads agree bit for bit where both lie in whole tiles
    assert np.array_equal(o[0, 1, :6144], o[0, 25, :6144]) and np.array_equal(l[0, 1, :6144], l[0, 25, :6144])


@pytest.mark.parametrize("B,H,Sq,Skv,n_v,all_cut,d", [(1, 24, 700, 12900, 12850, True, 128),  # 72 tiles, every one cut in three
                                                       (1, 3, 600, 102500, 102440, True, 128), # 9 tiles, every one cut in sixteen
                                                       (1, 4, 16384, 600, 570, False, 128),   # 256 tiles: one full round, none cut
                                                       (2, 5, 300, 2500, 2500, None, 128),
                                                       (1, 24, 700, 12900, 12850, True, 64),
                                                       (1, 4, 16384, 600, 570, False, 64),
                                                       (2, 5, 300, 2500, 2500, None, 64)])
def test_bf16_output_against_the_oracle(B, H, Sq, Skv, n_v, all_cut, d):
    """pda_attn_fwd_bf16out element by element against the fp64 oracle (its cut tiles take their own
    path: all parts go through the workspace and the merge pass writes bf16)."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    if all_cut is not None:
        plan = pda.attn_tail_plan(B, H, Sq, n_v, d)
        if plan["n_tiles"] % torch.cuda.get_device_properties(0).multi_processor_count == 0:
            assert plan["n_cut"] == 0 and not all_cut
        else:
            assert (plan["n_cut"] == plan["n_tiles"]) == all_cut
    qb, kb, vb = gen_qkv(700 + H, B, H, Sq, Skv, d, unit_rms=True)
    o16 = torch.full((B, H, Sq, d), float("nan"), device="cuda", dtype=torch.bfloat16)
    l16 = torch.full((B, H, Sq), float("nan"), device="cuda")
    pda.attn_fwd_bf16out(to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb), o16, l16, d ** -0.5, n_v)
    torch.cuda.synchronize()
    ro, rl = attention(qb, kb, vb, d ** -0.5, n_v)
    _assert_close_bf16(o16.float().cpu().numpy(), l16.cpu().numpy(), ro, rl, f"bf16 out {(B, H, Sq, Skv, n_v)}")


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("B,H,Sq,Skv,n_v", [(1, 2, 515, 1100, 1050), (2, 5, 300, 2500, 2500), (1, 3, 5000, 5000, 4990),
                                            (1, 1, 77, 64, 0), (1, 24, 700, 12900, 12850), (2, 3, 300, 40000, 39990)])
def test_bf16_output_is_the_rounded_fp32_output(B, H, Sq, Skv, n_v, d):
    """Same kernels, same arithmetic; only the last store differs (tiles cut into key ranges are
    merged from fp32 partials in both cases).  Hence bit equality with the rounded fp32 result, and
    through it parity with the oracle."""
    import torch
    import paper_2511_12056_amd as pda
    qb, kb, vb = gen_qkv(300 + H, B, H, Sq, Skv, d, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    o32 = torch.full((B, H, Sq, d), float("nan"), device="cuda"); l32 = torch.full((B, H, Sq), float("nan"), device="cuda")
    o16 = torch.full((B, H, Sq, d), float("nan"), device="cuda", dtype=torch.bfloat16); l16 = torch.full_like(l32, float("nan"))
    pda.attn_fwd(q, k, v, o32, l32, d ** -0.5, n_v)
    pda.attn_fwd_bf16out(q, k, v, o16, l16, d ** -0.5, n_v)
    torch.cuda.synchronize()
    assert torch.equal(o16, o32.to(torch.bfloat16))
    assert torch.equal(l16, l32)


def test_key_axis_beyond_2_gib():
    """One head whose K (and V) tensor is larger than 2^31 bytes (8.4 M keys x 256 B): every key
    address needs 64-bit arithmetic.  Four query rows; the launch's single tile is cut into 16 key
    ranges.  Oracle: the pinned per-chunk oracle on chunks of 1 M keys, combined with the pinned
    oracle merge (bounds host memory)."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention_head, merge_partials
    Sq, Skv, d = 4, 8_400_000, 128
    n_v = Skv - 37
    rng = np.random.default_rng(2511)
    qb = f32_to_bf16_bits(rng.standard_normal((1, 1, Sq, d), dtype=np.float32))
    kb = np.empty((1, 1, Skv, d), dtype=np.uint16)
    vb = np.empty((1, 1, Skv, d), dtype=np.uint16)
    step = 1 << 20
    for a in range(0, Skv, step):
        b = min(Skv, a + step)
        kb[0, 0, a:b] = f32_to_bf16_bits(rng.standard_normal((b - a, d), dtype=np.float32))
        vb[0, 0, a:b] = f32_to_bf16_bits(rng.standard_normal((b - a, d), dtype=np.float32))
    # make the last keys matter: the query rows point at keys near the end of the tensor
    kb[0, 0, n_v - 3] = f32_to_bf16_bits(bf16_bits_to_f32(qb[0, 0, 1]) * np.float32(2.5))
    kb[0, 0, n_v - 1] = f32_to_bf16_bits(bf16_bits_to_f32(qb[0, 0, 2]) * np.float32(2.0))
    scale = d ** -0.5
    o, l = _run(qb, kb, vb, scale, n_v)
    parts = []
    for a in range(0, n_v, step):
        b = min(n_v, a + step)
        parts.append(attention_head(qb[0, 0], kb[0, 0, a:b], vb[0, 0, a:b], scale))
    ro, rl = merge_partials([p[0] for p in parts], [p[1] for p in parts])
    assert rl[1] > rl[0] + 1 and rl[2] > rl[0] + 1            # the planted keys near the end carry weight
    assert_close(o[0, 0], l[0, 0], ro, rl, "K larger than 2 GiB")
