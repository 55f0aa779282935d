"""GPU parity of the steps next to the attention call: PipeSP post-processing, the token-major
hand-off layouts and unequal head groups of pda_headchunk_run_ex, and the pre-attention pack.
Pure data movement is compared bit for bit."""
import numpy as np
import pytest

from synth import gen_qkv
from synth.inputs import bf16_bits_to_f32, f32_to_bf16_bits
from tests.util import assert_close, to_dev_bf16

pytestmark = pytest.mark.gpu


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


@pytest.mark.parametrize("rows,h,n,D", [(37, 3, 8, 128), (1000, 24, 1, 128), (513, 1, 7, 64), (2051, 4, 2, 128),
                                        (5, 64, 3, 4), (14882, 3, 8, 128)])
def test_postprocess_separate_chunks_bit_exact(rows, h, n, D):
    import torch
    import paper_2511_12056_amd as pda
    from oracle.pipesp_layout import postprocess
    chunks = [_rand((rows, n, D), 100 + j) for j in range(h)]
    want = postprocess(chunks, h, n, D)
    dev = [torch.from_numpy(c).cuda() for c in chunks]
    hidden = torch.full((rows, h * n, D), float("nan"), device="cuda")
    pda.pipesp_postprocess(dev, h, n, hidden)
    torch.cuda.synchronize()
    assert np.array_equal(hidden.cpu().numpy(), want)


@pytest.mark.parametrize("rows,h,n,D", [(301, 3, 8, 128), (64, 6, 4, 64), (1, 2, 2, 8)])
def test_postprocess_concatenated_tensor_bit_exact(rows, h, n, D):
    import torch
    import paper_2511_12056_amd as pda
    from oracle.pipesp_layout import psi
    t_mod = _rand((rows, h * n, D), 7)
    hidden = torch.full((rows, h * n, D), float("nan"), device="cuda")
    pda.pipesp_postprocess(torch.from_numpy(t_mod).cuda(), h, n, hidden)
    torch.cuda.synchronize()
    assert np.array_equal(hidden.cpu().numpy(), psi(t_mod, h, n))


def test_postprocess_empty_is_a_noop():
    import torch
    import paper_2511_12056_amd as pda
    hidden = torch.empty(0, 6, 128, device="cuda")
    pda.pipesp_postprocess([torch.empty(0, 2, 128, device="cuda") for _ in range(3)], 3, 2, hidden)
    torch.cuda.synchronize()


def _run_ex(q, k, v, scale, groups, sp_ranks, layout, n_v=None, timed=False):
    import torch
    import paper_2511_12056_amd as pda
    B, H, Sq, d = q.shape
    out = torch.full((B, H, Sq, d), float("nan"), device="cuda")
    lse = torch.full((B, H, Sq), float("nan"), device="cuda")
    shape = (B, H, Sq, d) if layout == pda.PDA_SINK_HEAD_MAJOR else (B, Sq, H, d)
    sink = torch.full(shape, float("nan"), device="cuda")
    cs, ds = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    t = pda.headchunk_run_ex(q, k, v, out, lse, scale, groups, cs, ds, kv_valid_len=n_v, sink=sink,
                             sp_ranks=sp_ranks, sink_layout=layout, timed=timed)
    cs.synchronize(); ds.synchronize()
    return out, lse, sink, t


def test_token_major_handoff_and_postprocess_reproduce_ulysses():
    """n = 4 simulated GPUs with h = 3 local heads, pipelined one head per step (Algorithm 1): the
    arrival-order buffer, post-processed, equals the buffer written in final order, and rank r's
    rows of it equal what the original single All-to-All would have left there."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    from oracle.pipesp_layout import exchange_step, postprocess, ulysses_hidden
    B, n, h, S, d = 1, 4, 3, 520, 128
    H = n * h
    qb, kb, vb = gen_qkv(99, B, H, S, S, d, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    scale = d ** -0.5
    out, lse, arrival, _ = _run_ex(q, k, v, scale, [1] * H, n, pda.PDA_SINK_TOKEN_ARRIVAL)
    out2, lse2, final, _ = _run_ex(q, k, v, scale, [1] * H, n, pda.PDA_SINK_TOKEN_FINAL)
    assert torch.equal(out, out2) and torch.equal(lse, lse2)
    o = out.cpu().numpy()
    # attention itself against the oracle
    ro, rl = attention(qb, kb, vb, scale, S)
    assert_close(o, lse.cpu().numpy(), ro, rl, "headchunk_run_ex")
    # final order == transposition of out (head k at slot k)
    assert np.array_equal(final.cpu().numpy(), o.transpose(0, 2, 1, 3))
    # arrival order == what the per-step exchanges deliver, built on the CPU from the GPU's out
    a = arrival.cpu().numpy()[0]
    sl = S // n
    for r in range(n):
        chunks = [exchange_step([o[0, i * h + j] for i in range(n)], r) for j in range(h)]
        assert np.array_equal(a[r * sl:(r + 1) * sl], np.concatenate(chunks, axis=1))
        assert np.array_equal(postprocess(chunks, h, n, d), ulysses_hidden(o[0], n, r))
    # library post-processing of the arrival buffer == final buffer, bit for bit
    fixed = torch.full((B * S, H, d), float("nan"), device="cuda")
    pda.pipesp_postprocess(arrival.view(B * S, H, d), h, n, fixed)
    torch.cuda.synchronize()
    assert torch.equal(fixed.view(B, S, H, d), final)


def test_unequal_groups_and_batches():
    """H = 7 heads as groups 3,2,2 (what a 3-GPU ragged split gives), two batches, masked tail."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    B, H, S, d, n_v = 2, 7, 300, 128, 280
    qb, kb, vb = gen_qkv(5, B, H, S, S, d, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    groups = pda.plan_ragged_groups(H, 3)
    assert groups == [3, 2, 2]
    out, lse, sink, t = _run_ex(q, k, v, 0.1, groups, 1, pda.PDA_SINK_HEAD_MAJOR, n_v=n_v, timed=True)
    gms, total = t
    assert len(gms) == 3 and all(g > 0 for g in gms) and total >= max(gms)
    assert torch.equal(sink, out)
    ro, rl = attention(qb, kb, vb, 0.1, n_v)
    assert_close(out.cpu().numpy(), lse.cpu().numpy(), ro, rl, "ragged groups")
    # same result as one call over all heads (small shapes: no tile is cut, so bit for bit)
    ref = torch.empty_like(out); rlse = torch.empty_like(lse)
    pda.attn_fwd(q, k, v, ref, rlse, 0.1, n_v)
    torch.cuda.synchronize()
    assert torch.equal(out, ref) and torch.equal(lse, rlse)
    # token-major, 7 = 7 x 1: both orders coincide with the transposition
    _, _, tok, _ = _run_ex(q, k, v, 0.1, groups, 7, pda.PDA_SINK_TOKEN_ARRIVAL, n_v=n_v)
    assert torch.equal(tok, out.permute(0, 2, 1, 3).contiguous())


@pytest.mark.parametrize("B,S,H,d", [(1, 300, 3, 128), (2, 77, 5, 64), (1, 4099, 24, 128), (1, 1, 1, 64)])
def test_pack_plain_is_bit_exact(B, S, H, d):
    import torch
    import paper_2511_12056_amd as pda
    from oracle.pack import pack_heads
    x = _rand((B, S, H, d), 11) * np.float32(3.0)
    y = torch.zeros(B, H, S, d, dtype=torch.bfloat16, device="cuda")
    pda.pack_heads(torch.from_numpy(x).cuda(), y, unit_rms=False)
    torch.cuda.synchronize()
    got = bf16_bits_to_f32(y.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    assert np.array_equal(got, pack_heads(x, unit_rms=False))


@pytest.mark.parametrize("B,S,H,d", [(1, 300, 3, 128), (2, 77, 5, 64), (1, 4099, 24, 128)])
def test_pack_unit_rms_matches_oracle(B, S, H, d):
    """The kernel normalises in fp32, the oracle in fp64 with one rounding: a value within fp32
    rounding (~2^-23 relative, a few operations) of a bf16 rounding boundary (spacing 2^-8 relative)
    may land on the neighbouring bf16 value, so about 1e-4 of the elements may differ by one bf16
    step; none may differ by more."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle.pack import pack_heads
    rng = np.random.default_rng(13)
    x = _rand((B, S, H, d), 12) * rng.uniform(0.01, 100.0, (B, S, H, 1)).astype(np.float32)
    x[0, 0, 0] = 0.0                                                   # a zero vector stays zero
    y = torch.zeros(B, H, S, d, dtype=torch.bfloat16, device="cuda")
    pda.pack_heads(torch.from_numpy(x).cuda(), y, unit_rms=True)
    torch.cuda.synchronize()
    bits = y.view(torch.int16).cpu().numpy().view(np.uint16)
    got = bf16_bits_to_f32(bits).astype(np.float64)
    want = pack_heads(x, unit_rms=True)
    assert np.isfinite(got).all() and (got[0, 0, 0] == 0).all()
    wbits = f32_to_bf16_bits(want.astype(np.float32))                  # want holds bf16 values: exact
    step = np.abs(bits.astype(np.int32) - wbits.astype(np.int32))      # same sign: payload distance = bf16 steps
    assert np.array_equal(np.signbit(got), np.signbit(want))
    assert step.max() <= 1
    assert (step != 0).mean() < 1e-3


def test_pack_feeds_attention():
    """pack(unit-RMS) of token-major fp32 inputs, then attention, against the oracle run on the
    oracle's own pack of the same inputs."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention_head
    from oracle.pack import pack_heads
    B, S, H, d = 1, 700, 2, 128
    xs = [_rand((B, S, H, d), 20 + i) for i in range(3)]
    dev = []
    for x in xs:
        y = torch.empty(B, H, S, d, dtype=torch.bfloat16, device="cuda")
        pda.pack_heads(torch.from_numpy(x).cuda(), y, unit_rms=True)
        dev.append(y)
    out = torch.empty(B, H, S, d, device="cuda"); lse = torch.empty(B, H, S, device="cuda")
    pda.attn_fwd(dev[0], dev[1], dev[2], out, lse, d ** -0.5)
    torch.cuda.synchronize()
    qo, ko, vo = (pack_heads(x, True) for x in xs)
    for hh in range(H):
        ro, rl = attention_head(qo[0, hh], ko[0, hh], vo[0, hh], d ** -0.5, S)
        assert_close(out[0, hh].cpu().numpy(), lse[0, hh].cpu().numpy(), ro, rl, f"pack+attention head {hh}")


def test_mfma_rate_probe_runs():
    import torch
    import paper_2511_12056_amd as pda
    x = torch.randn(1 << 16, device="cuda").to(torch.bfloat16)
    tf, ms = pda.probe_mfma_rate(x, 1 << 14)
    assert ms > 0 and 100.0 < tf < 2600.0, (tf, ms)          # between a tenth of and the nominal bf16 peak
    tz, _ = pda.probe_mfma_rate(torch.zeros_like(x), 1 << 14)
    assert 100.0 < tz < 2600.0


@pytest.mark.parametrize("B,H,S,Skv,d,n_v", [(1, 2, 515, 1100, 128, 1050), (2, 3, 300, 4200, 128, 4200), (1, 2, 200, 333, 64, 300),
                                             (1, 5, 300, 2500, 128, 2500)])
def test_base2_attention_matches_oracle(B, H, S, Skv, d, n_v):
    """Scores taken as exponents of 2 == the oracle with scale = ln 2."""
    import math
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    qb, kb, vb = gen_qkv(700 + H, B, H, S, Skv, d, unit_rms=True)
    # bring the scores into a sensible range for exponents of 2: Q times scale*log2(e), rounded to bf16
    c = d ** -0.5 * math.log2(math.e)
    qb = f32_to_bf16_bits(bf16_bits_to_f32(qb) * np.float32(c))
    out = torch.full((B, H, S, d), float("nan"), device="cuda"); lse = torch.full((B, H, S), float("nan"), device="cuda")
    pda.attn_fwd_base2(to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb), out, lse, n_v)
    torch.cuda.synchronize()
    ro, rl = attention(qb, kb, vb, math.log(2.0), n_v)
    assert_close(out.cpu().numpy(), lse.cpu().numpy(), ro, rl, "base2")
    # the general entry point with scale = ln 2 computes the same function
    out2 = torch.empty_like(out); lse2 = torch.empty_like(lse)
    pda.attn_fwd(to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb), out2, lse2, math.log(2.0), n_v)
    torch.cuda.synchronize()
    assert ((out - out2).norm() / out2.norm()).item() < 5e-3
    assert ((lse - lse2).abs() / lse2.abs().clamp(min=1)).max().item() < 1e-5


def test_base2_overflow_redo():
    import math
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    rng = np.random.default_rng(78)
    B, H, Sq, Skv, d = 1, 2, 300, 900, 128
    q = rng.standard_normal((B, H, Sq, d)).astype(np.float32)
    k = (rng.standard_normal((B, H, Skv, d)) * 0.01).astype(np.float32)
    v = rng.standard_normal((B, H, Skv, d)).astype(np.float32)
    k[:, 0, 200:] *= 2000.0
    qb, kb, vb = f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)
    out = torch.full((B, H, Sq, d), float("nan"), device="cuda"); lse = torch.full((B, H, Sq), float("nan"), device="cuda")
    pda.attn_fwd_base2(to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb), out, lse)
    torch.cuda.synchronize()
    ro, rl = attention(qb, kb, vb, math.log(2.0), Skv)
    assert np.abs(rl).max() > 200
    assert_close(out.cpu().numpy(), lse.cpu().numpy(), ro, rl, "base2 overflow redo")


def test_pack_with_folded_scale_feeds_base2_attention():
    """Q packed with premul = scale*log2(e) + base-2 attention against the oracle on the oracle's
    own pack (same premul, one rounding) with scale ln 2."""
    import math
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention_head
    from oracle.pack import pack_heads
    B, S, H, d = 1, 700, 2, 128
    c = d ** -0.5 * math.log2(math.e)
    xs = [_rand((B, S, H, d), 40 + i) for i in range(3)]
    dev = []
    for i, x in enumerate(xs):
        y = torch.empty(B, H, S, d, dtype=torch.bfloat16, device="cuda")
        pda.pack_heads(torch.from_numpy(x).cuda(), y, unit_rms=True, premul=c if i == 0 else 1.0)
        dev.append(y)
    out = torch.empty(B, H, S, d, device="cuda"); lse = torch.empty(B, H, S, device="cuda")
    pda.attn_fwd_base2(dev[0], dev[1], dev[2], out, lse)
    torch.cuda.synchronize()
    qo = pack_heads(xs[0], True, premul=c)
    ko, vo = pack_heads(xs[1], True), pack_heads(xs[2], True)
    for hh in range(H):
        ro, rl = attention_head(qo[0, hh], ko[0, hh], vo[0, hh], math.log(2.0), S)
        assert_close(out[0, hh].cpu().numpy(), lse[0, hh].cpu().numpy(), ro, rl, f"folded scale head {hh}")


def test_streaming_kernels_beyond_2_to_31_elements():
    """Post-processing, pack and merge on tensors of more than 2^31 elements (64-bit offsets, grids
    that use all three dimensions), generated on the device; sampled rows against the oracles."""
    import torch
    import paper_2511_12056_amd as pda
    from oracle import merge_partials
    from oracle.pack import pack_heads
    from oracle.pipesp_layout import psi
    rows, h, n, D = 700_001, 3, 8, 128                      # 2.15e9 floats
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    rng = np.random.default_rng(5)
    pick = np.unique(np.concatenate([[0, 1, rows - 2, rows - 1, 65534, 65535, 65536, 524287, 524288],
                                     rng.choice(rows, size=1500, replace=False)]))
    idx = torch.from_numpy(pick).cuda()
    x = torch.randn(rows, h * n, D, device="cuda", generator=g)
    # Algorithm 1 steps 10-13 on one concatenated tensor
    hidden = torch.empty_like(x)
    pda.pipesp_postprocess(x, h, n, hidden)
    torch.cuda.synchronize()
    assert np.array_equal(hidden[idx].cpu().numpy(), psi(x[idx].cpu().numpy(), h, n))
    del hidden
    # pack: x as [1, S, H, d] token-major
    y = torch.empty(1, h * n, rows, D, dtype=torch.bfloat16, device="cuda")
    pda.pack_heads(x.view(1, rows, h * n, D), y, unit_rms=False)
    torch.cuda.synchronize()
    got = y[0][:, idx].float().cpu().numpy().astype(np.float64)                       # [H, picked, d]
    want = pack_heads(x[idx].cpu().numpy()[None], unit_rms=False)[0]                # [H, picked, d]
    assert np.array_equal(got, want)
    del y
    # merge of two partials of rows*24 rows x 128 values... the same buffer viewed as [rows*24, 128]
    R = rows * h * n
    lse = [torch.randn(R, device="cuda", generator=g) * 3 for _ in range(2)]
    p1 = torch.randn(R, D, device="cuda", generator=g)
    out = torch.empty(R, D, device="cuda")
    lo = torch.empty(R, device="cuda")
    pda.attn_merge([x.view(R, D), p1], lse, out, lo)
    torch.cuda.synchronize()
    rpick = np.unique(np.concatenate([[0, R - 1, (1 << 24) - 1, 1 << 24], rng.choice(R, size=2000, replace=False)]))
    ridx = torch.from_numpy(rpick).cuda()
    ro, rl = merge_partials([x.view(R, D)[ridx].cpu().numpy(), p1[ridx].cpu().numpy()], [l[ridx].cpu().numpy() for l in lse])
    assert np.abs(out[ridx].cpu().numpy() - ro).max() < 2e-5
    assert np.abs(lo[ridx].cpu().numpy() - rl).max() < 1e-5
