"""pda_attn_fwd_noalloc (partials of cut tiles in the library's static device buffer) against
pda_attn_fwd, through the C ABI, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from synth import gen_qkv, to_dev_bf16

pytestmark = pytest.mark.gpu


def _pair(pda, torch, seed, B, H, Sq, Skv, n_v, scale):
    qb, kb, vb = gen_qkv(seed, B, H, Sq, Skv, 128, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    ref = torch.full((B, H, Sq, 128), float("nan"), device="cuda"); rlse = torch.full((B, H, Sq), float("nan"), device="cuda")
    out = torch.full_like(ref, float("nan")); lse = torch.full_like(rlse, float("nan"))
    pda.attn_fwd(q, k, v, ref, rlse, scale, n_v)
    return (qb, kb, vb), (q, k, v), (ref, rlse), (out, lse)


def test_noalloc_entry_matches_the_allocating_one_on_two_calls_in_a_row():
    import torch
    import paper_2511_12056_amd as pda
    from oracle import attention
    from tests.util import assert_close
    scale = 128 ** -0.5
    # first call: 24 heads x 700 rows = 72 tiles, every one cut in three (144 scratch slots);
    # second call, smaller: 5 heads x 300 rows = 10 tiles, each cut in sixteen (150 slots, over the first call's leftovers)
    cases = [(11, 1, 24, 700, 12900, 12850), (12, 1, 5, 300, 19300, 19300)]
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    data = []
    for seed, B, H, Sq, Skv, n_v in cases:
        plan = pda.attn_tail_plan(B, H, Sq, n_v, 128)
        if n_cu == 256:
            assert plan["n_cut"] == plan["n_tiles"] and plan["split"] >= 2, plan
        data.append(_pair(pda, torch, seed, B, H, Sq, Skv, n_v, scale))
    # set-up: the first call on a device looks up the address of the static buffer (the runtime
    # materialises the array then: 76 MB); nothing may change after that
    pda.attn_fwd_noalloc(data[1][1][0], data[1][1][1], data[1][1][2], data[1][3][0], data[1][3][1], scale, cases[1][5])
    torch.cuda.synchronize()
    data[1][3][0].fill_(float("nan")); data[1][3][1].fill_(float("nan"))
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    for (seed, B, H, Sq, Skv, n_v), (_, (q, k, v), _, (out, lse)) in zip(cases, data):
        pda.attn_fwd_noalloc(q, k, v, out, lse, scale, n_v)            # back to back on one stream, no sync in between
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before - (1 << 20)    # nothing was allocated on the device (a workspace is 101 MB)
    for (seed, B, H, Sq, Skv, n_v), ((qb, kb, vb), _, (ref, rlse), (out, lse)) in zip(cases, data):
        # same kernels, same plan, same arithmetic: bit equality with the allocating entry point ...
        assert torch.equal(out, ref) and torch.equal(lse, rlse)
        # ... and therefore parity with the oracle at the usual gates
        ro, rl = attention(qb, kb, vb, scale, n_v)
        assert_close(out.cpu().numpy(), lse.cpu().numpy(), ro, rl, f"noalloc {(B, H, Sq, Skv, n_v)}")
    # the second call again, alone, over the scratch the larger call left behind
    (_, (q, k, v), (ref, rlse), (out, lse)) = data[1]
    out.fill_(float("nan")); lse.fill_(float("nan"))
    pda.attn_fwd_noalloc(q, k, v, out, lse, scale, cases[1][5])
    torch.cuda.synchronize()
    assert torch.equal(out, ref) and torch.equal(lse, rlse)


def test_noalloc_entry_covers_uncut_launches_and_d64_and_rejects_bad_arguments():
    import torch
    import paper_2511_12056_amd as pda
    for d, (B, H, Sq, Skv, n_v) in ((64, (1, 2, 333, 517, 500)), (128, (1, 1, 40, 90, 0))):
        qb, kb, vb = gen_qkv(13 + d, B, H, Sq, Skv, d, unit_rms=False)
        q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
        ref = torch.empty(B, H, Sq, d, device="cuda"); rlse = torch.empty(B, H, Sq, device="cuda")
        out = torch.empty_like(ref); lse = torch.empty_like(rlse)
        pda.attn_fwd(q, k, v, ref, rlse, 0.1, n_v)
        pda.attn_fwd_noalloc(q, k, v, out, lse, 0.1, n_v)
        torch.cuda.synchronize()
        assert torch.equal(out, ref) and torch.equal(lse, rlse)
    f = pda.lib.pda_attn_fwd_noalloc
    assert f(128, 128, 128, 128, 128, 1, 1, 8, 8, 32, 1.0, 8, 0, None) == 2
    assert f(128, 128, 128, 128, 128, 1, 1, 8, 8, 128, 1.0, 9, 0, None) == 1
    assert f(128, 128, 128, 128, 128, 1, 1, 8, 8, 128, 1.0, 8, -1, None) == 1
    assert f(None, None, None, None, None, 1, 1, 0, 8, 128, 1.0, 8, 0, None) == 0


def test_noalloc_entry_under_graph_capture():
    """What the entry point is for: captured into a HIP graph (after one call outside the capture,
    which looks up the static buffer) and replayed several times, with eager work and
    synchronisations between the replays; every replay must reproduce the eager result."""
    import torch
    import paper_2511_12056_amd as pda
    B, H, Sq, Skv, n_v = 1, 24, 700, 12900, 12850
    scale = 128 ** -0.5
    qb, kb, vb = gen_qkv(21, B, H, Sq, Skv, 128, unit_rms=True)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    ref = torch.empty(B, H, Sq, 128, device="cuda"); rlse = torch.empty(B, H, Sq, device="cuda")
    out = torch.empty_like(ref); lse = torch.empty_like(rlse)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        pda.attn_fwd_noalloc(q, k, v, ref, rlse, scale, n_v, stream=side)          # eager; also the set-up call
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pda.attn_fwd_noalloc(q, k, v, out, lse, scale, n_v, stream=side)
    for rep in range(3):
        out.fill_(float("nan")); lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref) and torch.equal(lse, rlse), rep
        # eager work between the replays, through the same static buffer
        pda.attn_fwd_noalloc(q, k, v, out, lse, scale, n_v)
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
