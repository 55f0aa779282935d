"""GPU parity of pda_attn_merge and pda_headchunk_run (C4 and C5 shapes included)."""
import numpy as np
import pytest

from synth import CONFIGS, gen_qkv
from tests.util import assert_close, cut_row_mask, gen_qkv_parallel, sample_rows, to_dev_bf16

pytestmark = pytest.mark.gpu


def test_merge_matches_oracle_random_partials():
    import torch
    import paper_2511_12056_amd as pda
    from oracle import merge_partials
    rng = np.random.default_rng(3)
    for n, rows, d in [(1, 100, 128), (2, 1000, 128), (4, 5003, 128), (3, 777, 64), (7, 300, 128), (16, 64, 128)]:
        O = rng.standard_normal((n, rows, d)).astype(np.float32)
        L = (rng.standard_normal((n, rows)) * 4).astype(np.float32)
        L[rng.random((n, rows)) < 0.1] = -np.inf
        L[:, 5] = -np.inf                                   # a row that is empty everywhere
        O[np.isneginf(L)] = np.nan                          # values of empty partials must never be used
        po = [torch.from_numpy(O[i]).cuda() for i in range(n)]
        pl = [torch.from_numpy(L[i]).cuda() for i in range(n)]
        out = torch.empty(rows, d, device="cuda")
        lse = torch.empty(rows, device="cuda")
        pda.attn_merge(po, pl, out, lse)
        torch.cuda.synchronize()
        ro, rl = merge_partials(list(O), list(L))
        o, l = out.cpu().numpy(), lse.cpu().numpy()
        fin = np.isfinite(rl)
        assert np.array_equal(np.isneginf(l), ~fin)
        assert np.abs(o - ro).max() < 2e-5, (n, rows, d)
        assert (np.abs(l[fin] - rl[fin]) / np.maximum(np.abs(rl[fin]), 1)).max() < 1e-5
        assert (o[5] == 0).all()
        # in place on the first partial, no lse_out
        pda.attn_merge(po, pl, po[0], None)
        torch.cuda.synchronize()
        assert np.array_equal(po[0].cpu().numpy(), o)


def _n_cu():
    import torch
    return torch.cuda.get_device_properties(0).multi_processor_count


def _assert_same_except_cut_rows(out, lse, ref_out, ref_lse, cut):
    """The paper's claim that chunked execution gives identical results (Experiments; Supplement,
    visual comparison), made exact: two launches that cover the same rows with different grids
    agree BIT FOR BIT on every row outside the query tiles that either launch computes as merged
    key-range partials (`cut`: boolean [B,H,Sq], from the launch plans), and to the rounding of the
    probabilities on those."""
    import torch
    cut = torch.from_numpy(cut).cuda()
    assert 0 < int(cut.sum()) < cut.numel()                       # both kinds of rows are present
    same = (out == ref_out).all(dim=-1) & (lse == ref_lse)
    assert bool(same[~cut].all()), f"{int((~same[~cut]).sum())} uncut rows differ"
    d_out, r_out = (out - ref_out)[cut], ref_out[cut]
    assert (d_out.norm() / r_out.norm()).item() < 5e-3
    assert ((lse - ref_lse).abs() / ref_lse.abs().clamp(min=1))[cut].max().item() < 1e-5


def _fwd(q, k, v, scale, n_v=None, q_offset=0):
    import torch
    import paper_2511_12056_amd as pda
    B, H, Sq, d = q.shape
    out = torch.empty(B, H, Sq, d, device="cuda")
    lse = torch.empty(B, H, Sq, device="cuda")
    pda.attn_fwd(q, k, v, out, lse, scale, n_v, q_offset)
    return out, lse


def test_key_split_and_query_split_merge_small():
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    B, H, Sq, Skv, d = 1, 2, 500, 1203, 128
    qb, kb, vb = gen_qkv(21, B, H, Sq, Skv, d, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    n_v = 1100
    full, lfull = _fwd(q, k, v, 0.09, n_v)
    cuts = [0, 300, 301, 900, 1150, 1203]                  # the last chunk lies wholly in the padding
    po, pl = [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        o, l = _fwd(q, k[:, :, a:b].contiguous(), v[:, :, a:b].contiguous(), 0.09, max(0, min(n_v, b) - a))
        po.append(o); pl.append(l)
    out = torch.empty_like(full); lse = torch.empty_like(lfull)
    pda.attn_merge(po, pl, out, lse)
    torch.cuda.synchronize()
    ro, rl = attention(qb, kb, vb, 0.09, n_v)
    assert_close(out.cpu().numpy(), lse.cpu().numpy(), ro, rl, "key split + merge")
    # against the unsplit GPU run: each chunk rounds its probabilities to bf16 relative to its own
    # running max, so the two differ at the level of that rounding (both sit within it of the oracle)
    assert ((out - full).norm() / full.norm()).item() < 5e-3
    # query ranges embedded in full-length partials with empty rows elsewhere
    po, pl = [], []
    for a, b in [(0, 200), (200, 375), (375, 500)]:
        o = torch.full_like(full, float("nan")); l = torch.full_like(lfull, float("-inf"))
        oo, ll = _fwd(q[:, :, a:b].contiguous(), k, v, 0.09, n_v, a)
        o[:, :, a:b] = oo; l[:, :, a:b] = ll
        po.append(o); pl.append(l)
    pda.attn_merge(po, pl, out, lse)
    torch.cuda.synchronize()
    assert torch.equal(out, full) and torch.equal(lse, lfull)


def test_headchunk_small_bitwise_and_sink_and_ragged_groups():
    import torch
    import paper_2511_12056_amd as pda
    B, H, Sq, Skv, d = 2, 7, 300, 400, 128
    qb, kb, vb = gen_qkv(31, B, H, Sq, Skv, d, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    full, lfull = _fwd(q, k, v, 0.09, 390)
    cs, ds = torch.cuda.Stream(), torch.cuda.Stream()
    for hpg in (1, 3, 7, 10):
        out = torch.full_like(full, float("nan")); lse = torch.full_like(lfull, float("nan"))
        sink = torch.full_like(full, float("nan"))
        torch.cuda.synchronize()
        gms, tms = pda.headchunk_run(q, k, v, out, lse, 0.09, hpg, cs, ds, kv_valid_len=390, sink=sink, timed=True)
        assert len(gms) == (H + hpg - 1) // hpg and all(g > 0 for g in gms) and tms > 0
        assert torch.equal(out, full) and torch.equal(lse, lfull)
        assert torch.equal(sink, out)                       # every hand-off waited for its group
        # untimed form: caller waits on both streams
        out.fill_(float("nan")); sink.fill_(float("nan"))
        torch.cuda.synchronize()
        assert pda.headchunk_run(q, k, v, out, lse, 0.09, hpg, cs, ds, kv_valid_len=390, sink=sink) is None
        cs.synchronize(); ds.synchronize()
        assert torch.equal(out, full) and torch.equal(sink, full)


def test_c4_headchunk_720p():
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention_head
    w = CONFIGS[4]
    qb, kb, vb = gen_qkv_parallel(w)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    out = torch.full((w.B, w.H, w.Sq, w.d), float("nan"), device="cuda")
    lse = torch.full((w.B, w.H, w.Sq), float("nan"), device="cuda")
    sink = torch.full_like(out, float("nan"))
    cs, ds = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    gms, tms = pda.headchunk_run(q, k, v, out, lse, w.scale, w.heads_per_group, cs, ds, sink=sink, timed=True)
    print("C4 group ms", [round(g, 2) for g in gms], "total", round(tms, 2),
          "TFLOP/s", round(w.flops / (tms * 1e-3) * 1e-12, 1))
    assert len(gms) == 8
    assert torch.equal(sink, out)
    assert sum(gms) <= tms * 1.01 + 0.2                     # groups run back to back inside the total
    full, lfull = _fwd(q, k, v, w.scale)                     # one launch over all 24 heads
    torch.cuda.synchronize()
    # rows cut by one of the eight 3-head launches or by the 24-head launch
    n_cu = _n_cu()
    cut = cut_row_mask(1, w.H, w.Sq, w.Skv, w.d, n_cu)[0]
    for g in range(w.H // w.heads_per_group):
        h0 = g * w.heads_per_group
        cut[h0:h0 + w.heads_per_group] |= cut_row_mask(1, w.heads_per_group, w.Sq, w.Skv, w.d, n_cu)[0]
    _assert_same_except_cut_rows(out, lse, full, lfull, cut[None])
    del full, lfull, sink
    for h in (0, 7, 13, 23):
        rows = sample_rows(w.Sq, 512, w.seed + h)
        ro, rl = attention_head(qb[0, h], kb[0, h], vb[0, h], w.scale, rows=rows)
        idx = torch.from_numpy(rows).cuda()
        e = assert_close(out[0, h][idx].cpu().numpy(), lse[0, h][idx].cpu().numpy(), ro, rl, f"C4 head {h}")
        print("C4 head", h, e)


def test_c5_split_merge_720p():
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention_head
    w = CONFIGS[5]
    qb, kb, vb = gen_qkv_parallel(w)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    full, lfull = _fwd(q, k, v, w.scale)
    # three query ranges written straight into their rows (concatenation) ...
    out_q = torch.full_like(full, float("nan")); lse_q = torch.full_like(lfull, float("nan"))
    po, pl = [], []
    for off, n in w.query_ranges:
        o, l = _fwd(q[:, :, off:off + n].contiguous(), k, v, w.scale, None, off)
        out_q[:, :, off:off + n] = o; lse_q[:, :, off:off + n] = l
        # ... and embedded in full-length partials for the merge call
        fo = torch.zeros_like(full); fl = torch.full_like(lfull, float("-inf"))
        fo[:, :, off:off + n] = o; fl[:, :, off:off + n] = l
        po.append(fo); pl.append(fl)
    n_cu = _n_cu()
    cut = cut_row_mask(1, w.H, w.Sq, w.Skv, w.d, n_cu)
    for off, n in w.query_ranges:
        cut[:, :, off:off + n] |= cut_row_mask(1, w.H, n, w.Skv, w.d, n_cu)
    _assert_same_except_cut_rows(out_q, lse_q, full, lfull, cut)
    # the same three ranges as bench.py issues them: views of the full tensors, written in place
    out_s = torch.full_like(full, float("nan")); lse_s = torch.full_like(lfull, float("nan"))
    for off, n in w.query_ranges:
        pda.attn_fwd_strided(q[:, :, off:off + n], k, v, out_s[:, :, off:off + n], lse_s[:, :, off:off + n],
                             w.scale, None, off)
    torch.cuda.synchronize()
    assert torch.equal(out_s, out_q) and torch.equal(lse_s, lse_q)
    del out_s, lse_s
    out_m = torch.empty_like(full); lse_m = torch.empty_like(lfull)
    pda.attn_merge(po, pl, out_m, lse_m)
    torch.cuda.synchronize()
    assert torch.equal(out_m, out_q) and torch.equal(lse_m, lse_q)     # the merge call reproduces concatenation exactly
    del po, pl, out_q, lse_q
    # four key chunks merged
    po, pl = [], []
    for off, n in w.key_chunks:
        o, l = _fwd(q, k[:, :, off:off + n].contiguous(), v[:, :, off:off + n].contiguous(), w.scale)
        po.append(o); pl.append(l)
    # bench.py's form of the first chunk: key views, no copy
    o_s = torch.empty_like(full); l_s = torch.empty_like(lfull)
    off, n = w.key_chunks[1]
    pda.attn_fwd_strided(q, k[:, :, off:off + n], v[:, :, off:off + n], o_s, l_s, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(o_s, po[1]) and torch.equal(l_s, pl[1])
    del o_s, l_s
    pda.attn_merge(po, pl, out_m, lse_m)
    torch.cuda.synchronize()
    rel = ((out_m - full).norm() / full.norm()).item()
    assert rel < 5e-3, rel                                   # bf16 rounding of P differs per chunk
    assert ((lse_m - lfull).abs() / lfull.abs().clamp(min=1)).max().item() < 1e-5
    bounds = [off for off, _ in w.query_ranges] + [off + n - 1 for off, n in w.query_ranges]
    for h in (0, 5):
        rows = sample_rows(w.Sq, 512, w.seed + h, extra=bounds + [b + 1 for b in bounds] + [b - 1 for b in bounds])
        ro, rl = attention_head(qb[0, h], kb[0, h], vb[0, h], w.scale, rows=rows)
        idx = torch.from_numpy(rows).cuda()
        for name, (oo, ll) in {"unsplit": (full, lfull), "key-merged": (out_m, lse_m)}.items():
            e = assert_close(oo[0, h][idx].cpu().numpy(), ll[0, h][idx].cpu().numpy(), ro, rl, f"C5 {name} head {h}")
            print("C5", name, h, e)


def test_strided_views_equal_compact_copies():
    """Query ranges and key chunks passed as views of the full tensors (no copies) give bit for bit
    what the compact-copy calls give, and write only their own rows of the full out/lse."""
    import torch
    import paper_2511_12056_amd as pda
    B, H, S, d = 2, 3, 700, 128
    qb, kb, vb = gen_qkv(31, B, H, S, S, d, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    scale = d ** -0.5
    ref, rlse = _fwd(q, k, v, scale)
    # query ranges written in place into one full result
    out = torch.full((B, H, S, d), float("nan"), device="cuda")
    lse = torch.full((B, H, S), float("nan"), device="cuda")
    for a, b in ((0, 280), (280, 525), (525, 700)):
        pda.attn_fwd_strided(q[:, :, a:b], k, v, out[:, :, a:b], lse[:, :, a:b], scale, None, a)
        co, cl = _fwd(q[:, :, a:b].contiguous(), k, v, scale, None, a)
        torch.cuda.synchronize()
        assert torch.equal(out[:, :, a:b], co) and torch.equal(lse[:, :, a:b], cl)
    assert torch.equal(out, ref) and torch.equal(lse, rlse)
    # key chunks as views, masked tail inside the last chunk, merged
    n_v = 650
    full, lfull = _fwd(q, k, v, scale, n_v)
    po, pl = [], []
    for a, b in ((0, 256), (256, 448), (448, 700)):
        o = torch.empty(B, H, S, d, device="cuda"); l = torch.empty(B, H, S, device="cuda")
        pda.attn_fwd_strided(q, k[:, :, a:b], v[:, :, a:b], o, l, scale, max(0, min(n_v, b) - a))
        co, cl = _fwd(q, k[:, :, a:b].contiguous(), v[:, :, a:b].contiguous(), scale, max(0, min(n_v, b) - a))
        torch.cuda.synchronize()
        assert torch.equal(o, co) and torch.equal(l, cl)
        po.append(o); pl.append(l)
    mo = torch.empty_like(full); ml = torch.empty_like(lfull)
    pda.attn_merge(po, pl, mo, ml)
    torch.cuda.synchronize()
    assert ((mo - full).norm() / full.norm()).item() < 5e-3
    # the normaliser is an fp32 sum of unrounded weights in both groupings
    assert ((ml - lfull).abs() / lfull.abs().clamp(min=1)).max().item() < 1e-5
    # a head subset of a larger tensor (what a co-processing helper receives) with d = 64
    qb, kb, vb = gen_qkv(32, 1, 4, 300, 300, 64, unit_rms=False)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    ref, rlse = _fwd(q, k, v, 0.125)
    out = torch.zeros_like(ref); lse = torch.zeros_like(rlse)
    pda.attn_fwd_strided(q[:, 1:3], k[:, 1:3], v[:, 1:3], out[:, 1:3], lse[:, 1:3], 0.125)
    torch.cuda.synchronize()
    assert torch.equal(out[:, 1:3], ref[:, 1:3]) and torch.equal(lse[:, 1:3], rlse[:, 1:3])
    assert (out[:, 0] == 0).all() and (out[:, 3] == 0).all()


def test_launches_on_two_streams_do_not_share_a_workspace():
    """Two attention launches whose tiles are cut into key ranges, enqueued on two streams without
    any ordering between them: each stream has its own partial slots and work counters, so both
    give bit for bit what they give alone."""
    import torch
    import paper_2511_12056_amd as pda
    shapes = [(1, 24, 700, 12900, 12850), (1, 5, 300, 19300, 19300)]
    data = []
    for i, (B, H, Sq, Skv, n_v) in enumerate(shapes):
        qb, kb, vb = gen_qkv(60 + i, B, H, Sq, Skv, 128, unit_rms=True)
        q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
        ref, rlse = _fwd(q, k, v, 0.09, n_v)
        data.append((q, k, v, n_v, ref, rlse, torch.full_like(ref, float("nan")), torch.full_like(rlse, float("nan"))))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):
        for st, (q, k, v, n_v, _, _, out, lse) in zip(streams, data):
            pda.attn_fwd(q, k, v, out, lse, 0.09, n_v, stream=st)
    torch.cuda.synchronize()
    for (_, _, _, _, ref, rlse, out, lse) in data:
        assert torch.equal(out, ref) and torch.equal(lse, rlse)


def test_headchunk_pipeline_captured_into_a_graph():
    """The head-by-head pipeline (two streams, one event per group) captured into a HIP graph after
    one eager call (which allocates the compute stream's workspace); the drain stream is joined
    back inside the capture.  Every replay, with eager pipelines and synchronisations in between,
    reproduces the eager result bit for bit in out, lse and the hand-off buffer."""
    import torch
    import paper_2511_12056_amd as pda
    B, H, S = 1, 6, 2100
    scale = 128 ** -0.5
    qb, kb, vb = gen_qkv(55, B, H, S, S, 128, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    ref = torch.empty(B, H, S, 128, device="cuda"); rlse = torch.empty(B, H, S, device="cuda"); rsink = torch.empty_like(ref)
    out = torch.empty_like(ref); lse = torch.empty_like(rlse); sink = torch.empty_like(ref)
    cs, ds = torch.cuda.Stream(), torch.cuda.Stream()
    pda.headchunk_run(q, k, v, ref, rlse, scale, 1, cs, ds, sink=rsink)
    cs.synchronize(); ds.synchronize()
    assert torch.equal(ref, rsink)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=cs):
        pda.headchunk_run(q, k, v, out, lse, scale, 1, cs, ds, sink=sink)
        cs.wait_stream(ds)
    for rep in range(3):
        out.fill_(float("nan")); sink.fill_(float("nan")); lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref) and torch.equal(sink, rsink) and torch.equal(lse, rlse), rep
        pda.headchunk_run(q, k, v, out, lse, scale, 2, cs, ds, sink=sink)      # eager work between the replays, other grouping
        cs.synchronize(); ds.synchronize()
