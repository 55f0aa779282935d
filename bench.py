"""Benchmark of the attention hot path at the 720p x 129-frame shape on one MI355X.

One step = one pass of the whole path over one batch of synthetic Q/K/V resident in HBM:
  1. pda_headchunk_run: 24 heads x 119 056 tokens x d=128 as 8 groups of 3 heads, two streams,
     hand-off copy of every group's result (the PipeSP loop on one GPU's heads);
  2. the Aco-style work split on the first 6 heads: three query ranges (40/35/25 %) as separate
     pda_attn_fwd_strided calls on views, then four key chunks as separate calls merged by
     pda_attn_merge.
Prints ONE JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_720p.json")


def measured_traffic(kernel):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE runs,
    calibrated on the hand-off copy kernel); None if no summary is there.  bench.py cannot run the
    profiler around itself, so this is the last profiled value, with its source named."""
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get(kernel)
    except (OSError, ValueError):
        return None


def cpu_baseline(w, qb, kb, vb, target_s=15.0):
    """The fp64 oracle, as it stands, on a bounded row sample of head 0 against all keys."""
    import numpy as np
    from oracle import attention_head
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    rows = np.arange(0, 256, dtype=np.int64)
    t0 = time.perf_counter()
    attention_head(qb[0, 0], kb[0, 0], vb[0, 0], w.scale, rows=rows)          # calibration
    per_row = (time.perf_counter() - t0) / len(rows)
    n = int(min(w.Sq, max(512, target_s / max(per_row, 1e-9))))
    n = min(n, 65536)
    rows = np.linspace(0, w.Sq - 1, n).astype(np.int64)
    t0 = time.perf_counter()
    attention_head(qb[0, 0], kb[0, 0], vb[0, 0], w.scale, rows=rows)
    dt = time.perf_counter() - t0
    flops = 4.0 * n * w.Skv * w.d
    return {"value": flops / dt * 1e-12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n} query rows of head 0 against all {w.Skv} keys, fp64 numpy, {dt:.1f} s",
            "full_problem_extrapolated_s": w.flops / (flops / dt)}


class ClockSampler:
    """Best effort: samples the shader clock the driver reports (sysfs pp_dpm_sclk, the starred
    level) from a host thread while a region runs; empty if the file is not readable."""

    def __init__(self, period_s=0.02):
        import glob
        import threading
        files = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.path = files[0] if files else None
        self.period = period_s
        self.samples = []
        self._stop = threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _read(self):
        try:
            with open(self.path) as f:
                for line in f:
                    if "*" in line:
                        return int("".join(ch for ch in line.split(":")[1] if ch.isdigit()))
        except (OSError, ValueError, IndexError, TypeError):
            return None
        return None

    def _run(self):
        while not self._stop.is_set():
            v = self._read()
            if v is not None:
                self.samples.append(v)
            self._stop.wait(self.period)

    def __enter__(self):
        if self.path:
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self.path:
            self._thread.join(timeout=1.0)

    def summary(self):
        if not self.samples:
            return None
        x = sorted(self.samples)
        return {"min": x[0], "median": x[len(x) // 2], "max": x[-1], "samples": len(x),
                "source": "sysfs pp_dpm_sclk sampled from the host during the timed steps"}


def _event_ms(torch, stream, fn, iters=5):
    """Mean duration of fn() (which enqueues on `stream`) over `iters` calls, by events on that stream."""
    fn()
    stream.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(iters):
        fn()
    b.record(stream)
    stream.synchronize()
    return a.elapsed_time(b) / iters


def _errors(out_gpu, lse_gpu, out_ref, lse_ref):
    """The error measures of the parity gates, against fp64 oracle rows."""
    import numpy as np
    diff = out_gpu.astype(np.float64) - out_ref
    return {"max_abs": float(np.abs(diff).max()), "mean_abs": float(np.abs(diff).mean()),
            "rel_l2": float(np.sqrt((diff ** 2).sum() / max((out_ref ** 2).sum(), 1e-300))),
            "lse_rel": float((np.abs(lse_gpu.astype(np.float64) - lse_ref) / np.maximum(np.abs(lse_ref), 1.0)).max())}


def _timed_launches(torch, stream, fn, iters):
    """Durations (ms) of `iters` single calls of fn() on `stream`, one event pair per call."""
    fn(); fn(); fn()
    stream.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in ev:
        a.record(stream)
        fn()
        b.record(stream)
    stream.synchronize()
    return sorted(a.elapsed_time(b) for a, b in ev)


def measure_config(pda, torch, idx, cs, tensors=None, oracle_rows=192):
    """One workload of the benchmark spec through pda_attn_fwd: median / min launch time over its own
    iteration count, TFLOP/s with the nominal key count, fraction of the bf16 peak, and the parity
    errors of that launch against the fp64 oracle (C1: every row; others: a seeded row sample of the
    first and last head against all keys).  C4 is one 3-head group of its pipeline, C5 its unsplit
    6-head pass (the split passes are part of the timed step and of the GPU tests)."""
    import numpy as np
    from oracle import attention_head
    from synth import CONFIGS, gen_qkv_parallel, to_dev_bf16
    w = CONFIGS[idx]
    H = w.heads_per_group if idx == 4 else w.H
    if tensors is None:
        qb, kb, vb = gen_qkv_parallel(w, heads=(0, H), workers=min(16, os.cpu_count() or 8))
        q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    else:
        (qb, kb, vb), (q, k, v) = tensors
        qb, kb, vb = qb[:, :H], kb[:, :H], vb[:, :H]
        q, k, v = q[:, :H].contiguous(), k[:, :H].contiguous(), v[:, :H].contiguous()
    out = torch.empty(w.B, H, w.Sq, w.d, device="cuda")
    lse = torch.empty(w.B, H, w.Sq, device="cuda")
    n_v = w.kv_valid_len
    iters = {1: 200, 2: 50, 3: 10, 4: 8, 5: 5}[idx]
    with torch.cuda.stream(cs):
        ms = _timed_launches(torch, cs, lambda: pda.attn_fwd(q, k, v, out, lse, w.scale, n_v, stream=cs), iters)
    med, mn = ms[len(ms) // 2], ms[0]
    flops = 4.0 * w.Sq * w.Skv * w.d * H * w.B
    res = {"workload": w.name, "launch": f"pda_attn_fwd B={w.B} H={H} Sq={w.Sq} Skv={w.Skv} d={w.d} kv_valid_len={n_v}",
           "iters": iters, "median_ms": med, "min_ms": mn, "tflops": flops / (med * 1e-3) * 1e-12,
           "frac_of_bf16_peak": flops / (med * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS,
           "plan": pda.attn_tail_plan(w.B, H, w.Sq, n_v, w.d)}
    if idx == 1:
        res["note"] = "cache resident and launch bound: 0.54 GFLOP per launch"
    o, l = out.cpu().numpy(), lse.cpu().numpy()
    errs = {}
    for h in sorted({0, H - 1}):
        rng = np.random.default_rng(w.seed + h)
        rows = np.arange(w.Sq) if idx == 1 else np.unique(np.concatenate(
            [[0, w.Sq - 1, 255, 256], rng.choice(w.Sq, size=oracle_rows, replace=False)]))
        ro, rl = attention_head(qb[0, h], kb[0, h], vb[0, h], w.scale, n_v, rows=rows)
        errs[f"head{h}"] = _errors(o[0, h][rows], l[0, h][rows], ro, rl)
    res["parity_vs_oracle"] = {key: max(e[key] for e in errs.values()) for key in ("max_abs", "mean_abs", "rel_l2", "lse_rel")}
    res["parity_rows_per_head"] = int(len(rows))
    return res



def next_rows(pda, torch, w, q, k, v, out, lse, sink, cs, ds, t_linear_ms):
    """The steps next to the attention call at the same 720p shape, outside the timed step:
    post-processing, token-major hand-off, pack, unequal vs padded head groups, planner."""
    S, H, d, hg = w.Sq, w.H, w.d, w.heads_per_group
    n = H // hg                                              # 8 simulated GPUs with 3 local heads each
    res = {}

    def bw(name, ms, nbytes, extra=None, traffic_key=None):
        gbs = nbytes / (ms * 1e-3) * 1e-9
        res[name] = {"bound": "hbm", "launch_ms": ms, "bytes_per_launch": nbytes, "achieved": gbs, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "traffic": measured_traffic(traffic_key)}
        if extra:
            res[name].update(extra)

    # Algorithm 1 steps 10-13 over every receiver's rows at once: [S, 24, 128] fp32 in and out
    t_mod, hidden = sink.view(S, H, d), out.view(S, H, d)
    ms = _event_ms(torch, cs, lambda: pda.pipesp_postprocess(t_mod, hg, n, hidden, stream=cs))
    bw("pipesp_postprocess", ms, 2.0 * S * H * d * 4, {"kernel": "postprocess_kernel", "rows": S, "h": hg, "n": n},
       "postprocess_kernel")

    # pack: token-major fp32 [1,S,24,128] -> head-major bf16, unit-RMS vectors
    x = out.view(1, S, H, d)
    y = torch.empty(1, H, S, d, dtype=torch.bfloat16, device="cuda")
    ms = _event_ms(torch, cs, lambda: pda.pack_heads(x, y, True, stream=cs))
    bw("pack_heads_unit_rms", ms, S * H * d * 6.0, {"kernel": "pack_heads_kernel<32>"}, "pack_heads_kernel_32")
    del y

    # the softmax scale folded into Q where Q is packed (one rounding there), attention on exponents of 2:
    # one 3-head group, same K and V
    import math
    xq = q[:, :hg].float().permute(0, 2, 1, 3).contiguous()          # stands in for the fp32 Q projections [1,S,3,d]
    q2 = torch.empty(1, hg, S, d, dtype=torch.bfloat16, device="cuda")
    pda.pack_heads(xq, q2, True, premul=w.scale * math.log2(math.e), stream=cs)
    o2 = out[:, :hg]
    l2 = lse[:, :hg]
    ms = _event_ms(torch, cs, lambda: pda.attn_fwd_base2(q2, k[:, :hg], v[:, :hg], o2, l2, stream=cs))
    fl = 4.0 * S * S * d * hg
    res["attn_base2_scale_folded_into_q_pack"] = {"bound": "mfma", "launch_ms": ms, "flops_per_launch": fl,
                                                  "achieved": fl / (ms * 1e-3) * 1e-12, "peak": PEAK_BF16_TFLOPS,
                                                  "unit": "TFLOP/s", "frac": fl / (ms * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS,
                                                  "kernel": "attn_fwd_sp_kernel<128, 1, true> (one 3-head group)"}
    del xq, q2

    # the d = 64 instance of the attention kernel on a long sequence (the workloads have d = 64 only in
    # the tiny one): the 544 x 960 token count, 6 heads, inputs = the halves of the workload's vectors
    S64, h64 = 67576, 6
    q64, k64, v64 = (t.view(1, H, 2 * S, 64)[:, :h64, :S64].contiguous() for t in (q, k, v))
    o64 = torch.empty(1, h64, S64, 64, device="cuda")
    l64 = torch.empty(1, h64, S64, device="cuda")
    ms = _event_ms(torch, cs, lambda: pda.attn_fwd(q64, k64, v64, o64, l64, 0.125, stream=cs))
    fl = 4.0 * S64 * S64 * 64 * h64
    res["attn_d64_6_heads_x_67576"] = {"bound": "alu", "launch_ms": ms, "flops_per_launch": fl,
                                       "achieved": fl / (ms * 1e-3) * 1e-12, "unit": "TFLOP/s",
                                       "frac_of_bf16_mfma_peak": fl / (ms * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS,
                                       "kernel": "attn_fwd_sp_kernel<64, 1, false>",
                                       "note": "half the MFMA work per score: bound by the issue of the softmax arithmetic"}
    del q64, k64, v64, o64, l64

    # head-chunk pipeline with the post-processing folded into the hand-off (token-major, final order)
    tok = sink.view(1, S, H, d)
    pda.headchunk_run_ex(q, k, v, out, lse, w.scale, [hg] * n, cs, ds, sink=tok, sp_ranks=n,
                         sink_layout=pda.PDA_SINK_TOKEN_FINAL, timed=True)
    gms, tms = pda.headchunk_run_ex(q, k, v, out, lse, w.scale, [hg] * n, cs, ds, sink=tok, sp_ranks=n,
                                    sink_layout=pda.PDA_SINK_TOKEN_FINAL, timed=True)
    res["headchunk_token_major_final"] = {"total_ms": tms, "sum_group_ms": sum(gms)}

    # 24 heads on 7 GPUs played one after the other: padded to 28 heads (7 groups of 4) against the
    # unequal split 4,4,4,3,3,3,3.  The padding heads repeat real heads so that they cost the same.
    n7 = 7
    padded, per, needed = pda.plan_head_padding(H, n7)
    pad = padded - H
    qp, kp, vp = (torch.cat([t, t[:, :pad]], dim=1) for t in (q, k, v))
    outp = torch.empty(1, padded, S, d, device="cuda")
    lsep = torch.empty(1, padded, S, device="cuda")
    gp, tp = pda.headchunk_run_ex(qp, kp, vp, outp, lsep, w.scale, [per] * n7, cs, ds, timed=True)
    del qp, kp, vp, outp, lsep
    groups = pda.plan_ragged_groups(H, n7)
    gr, tr = pda.headchunk_run_ex(q, k, v, out, lse, w.scale, groups, cs, ds, timed=True)
    res["heads_24_on_7_gpus"] = {"padded_heads": padded, "heads_per_gpu": per, "gpus_needed": needed,
                                 "padded_group_ms": gp, "padded_total_ms": tp, "ragged_groups": groups,
                                 "ragged_group_ms": gr, "ragged_total_ms": tr,
                                 "gpu_time_wasted_by_padding": 1.0 - tr / tp,
                                 "critical_path_ms": {"padded": max(gp), "ragged": max(gr)}}

    # planner fed with the measured attention time of one GPU's share (t_A) and a supplied t_L
    t_A = sum(gms) / n
    t_L = t_linear_ms if t_linear_ms is not None else 0.25 * t_A
    res["planner"] = {"t_A_ms": t_A, "t_L_ms": t_L, "t_L_source": "argument" if t_linear_ms is not None else "assumed 0.25 * t_A",
                      "aco": {f"{a}+{b}": pda.plan_aco(t_L, t_A, a, b)[2] for a, b in ((7, 1), (6, 2), (4, 4))}}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true", help="skip the measurements of the steps next to the attention call")
    ap.add_argument("--t-linear-ms", type=float, default=None, help="time of the linear projections for the planner example")
    ap.add_argument("--config", type=int, default=0, choices=[0, 1, 2, 3, 4, 5],
                    help="measure only workload N of BASELINE.json through pda_attn_fwd and print its JSON line "
                         "(0, the default: the headline step, with every workload in the all_configs block)")
    ap.add_argument("--no-all-configs", action="store_true", help="skip the per-workload block of the default run")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    import paper_2511_12056_amd as pda
    from synth import CONFIGS, gen_qkv_parallel, to_dev_bf16

    if args.config:
        cs = torch.cuda.Stream()
        r = measure_config(pda, torch, args.config, cs)
        print(json.dumps({"metric": "attention TFLOP/s and % of bf16 MFMA peak (1 GPU), one workload", "value": r["tflops"],
                          "unit": "TFLOP/s", "n_gpus": 1, "steps": r["iters"], "warmup": 3, "ms_per_step": r["median_ms"],
                          "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
                          "data": "synthetic", "config": {"workload": r["workload"]},
                          "roofline": {"bound": "mfma", "achieved": r["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                       "frac": r["frac_of_bf16_peak"], "traffic": None}, "detail": r}))
        return

    w, w5 = CONFIGS[4], CONFIGS[5]
    workers = min(16, os.cpu_count() or 8)
    qb, kb, vb = gen_qkv_parallel(w, workers=workers)
    q, k, v = to_dev_bf16(qb), to_dev_bf16(kb), to_dev_bf16(vb)
    out = torch.empty(w.B, w.H, w.Sq, w.d, device="cuda")
    lse = torch.empty(w.B, w.H, w.Sq, device="cuda")
    sink = torch.empty_like(out)
    cs, ds = torch.cuda.Stream(), torch.cuda.Stream()

    # Aco-style split on the first 6 heads: query ranges and key chunks are VIEWS of the same
    # tensors (pda_attn_fwd_strided, no copies); query ranges write their rows of one full result
    H5 = w5.H
    q5, k5, v5 = q[:, :H5], k[:, :H5], v[:, :H5]
    out5 = torch.empty(1, H5, w.Sq, w.d, device="cuda")
    lse5 = torch.empty(1, H5, w.Sq, device="cuda")
    outq = torch.empty(1, H5, w.Sq, w.d, device="cuda")
    lseq = torch.empty(1, H5, w.Sq, device="cuda")
    qr = [(q5[:, :, o:o + n], o, outq[:, :, o:o + n], lseq[:, :, o:o + n]) for o, n in w5.query_ranges]
    kc = [(k5[:, :, o:o + n], v5[:, :, o:o + n]) for o, n in w5.key_chunks]
    kc_out = [(torch.empty_like(out5), torch.empty_like(lse5)) for _ in kc]
    merge_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    split_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]

    group_ms_all, total_ms_all = [], []

    def step(i, timed):
        gms, tms = pda.headchunk_run(q, k, v, out, lse, w.scale, w.heads_per_group, cs, ds, sink=sink, timed=True)
        if timed:
            group_ms_all.extend(gms); total_ms_all.append(tms)
        with torch.cuda.stream(cs):
            if timed: split_ev[i][0].record(cs)
            for qq, off, oo, ll in qr:
                pda.attn_fwd_strided(qq, k5, v5, oo, ll, w.scale, None, off, stream=cs)
            for (kk, vv), (oo, ll) in zip(kc, kc_out):
                pda.attn_fwd_strided(q5, kk, vv, oo, ll, w.scale, None, 0, stream=cs)
            if timed: split_ev[i][1].record(cs); merge_ev[i][0].record(cs)
            pda.attn_merge([o for o, _ in kc_out], [l for _, l in kc_out], out5, lse5, stream=cs)
            if timed: merge_ev[i][1].record(cs)

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    with ClockSampler() as clocks:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0

    flops_chunked = float(w.flops)
    flops_split = 2.0 * 4.0 * w.Sq * w.Skv * w.d * H5          # query-range pass + key-chunk pass
    flops_step = flops_chunked + flops_split
    ms_per_step = dt / args.steps * 1e3
    value = flops_step / (dt / args.steps) * 1e-12

    # dominant kernel: the attention forward; one launch = one 3-head group of the pipeline
    launch_ms = sum(group_ms_all) / len(group_ms_all)
    flops_launch = 4.0 * w.Sq * w.Skv * w.d * w.heads_per_group
    achieved = flops_launch / (launch_ms * 1e-3) * 1e-12
    merge_ms = sum(a.elapsed_time(b) for a, b in merge_ev) / args.steps
    split_ms = sum(a.elapsed_time(b) for a, b in split_ev) / args.steps
    n_p = len(kc)
    merge_bytes = (n_p + 1) * (w.d + 1) * 4.0 * H5 * w.Sq
    res = {
        "metric": "attention TFLOP/s and % of bf16 MFMA peak at 720p x 129f latent (1 GPU)",
        "value": value, "unit": "TFLOP/s", "pct_of_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c4_720p_headchunk (24 heads as 8 groups of 3, S=119056, d=128) + "
                               "c5_720p_split_merge (6 heads: 3 query ranges, 4 key chunks + merge)",
                   "B": w.B, "H": w.H, "d": w.d, "S": w.Sq, "heads_per_group": w.heads_per_group,
                   "seed": w.seed, "flops_per_step": flops_step},
        "roofline": {"kernel": "attn_fwd_sp_kernel<128, 1, false> (one 3-head group)", "bound": "mfma", "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "launch_ms": launch_ms, "flops_per_launch": flops_launch,
                     "traffic": measured_traffic("attn_fwd_sp_kernel_3head_group")},
        "roofline_merge": {"kernel": "merge_kernel<4>", "bound": "hbm", "achieved": merge_bytes / (merge_ms * 1e-3) * 1e-9,
                           "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": merge_bytes / (merge_ms * 1e-3) * 1e-9 / PEAK_HBM_GBS,
                           "launch_ms": merge_ms, "bytes_per_launch": merge_bytes,
                           "traffic": measured_traffic("merge_kernel_4")},
        "pipeline": {"group_ms_mean": launch_ms, "group_ms_median": sorted(group_ms_all)[len(group_ms_all) // 2],
                     "group_ms_min": min(group_ms_all), "total_ms_mean": sum(total_ms_all) / len(total_ms_all),
                     "sum_group_ms_mean": sum(group_ms_all) / args.steps, "split_pass_ms": split_ms,
                     "chunked_tflops": flops_chunked / (sum(total_ms_all) / len(total_ms_all) * 1e-3) * 1e-12},
    }
    res["roofline"]["sclk_mhz"] = clocks.summary()
    # context for the clock the chip sustains on this data: an MFMA-only loop fed with Q's values
    probe_tf, probe_ms = pda.probe_mfma_rate(q, 1 << 20, stream=cs)
    res["roofline"]["mfma_only_same_data"] = {"achieved": probe_tf, "unit": "TFLOP/s", "ms": probe_ms,
                                              "what": "loop of bf16 32x32x16 MFMAs only, operands = values of Q, 2 wavefronts per SIMD"}
    res["roofline"]["frac_of_mfma_only"] = achieved / probe_tf
    # what the other instruction classes of the kernel's loop cost on this data under the power limit:
    # the same MFMA loop with them added one after the other at the kernel's density (no DMA, no barriers)
    ladder = {}
    for mix, name in ((1, "plus_softmax_arithmetic"), (2, "plus_operand_reads_from_lds"), (3, "with_half_the_operand_reads")):
        tf, _ = pda.probe_loop_rate(q, mix, 1 << 19, stream=cs)
        ladder[name] = tf
    res["roofline"]["loop_budget"] = {"unit": "TFLOP/s", "mfma_only": probe_tf, **ladder, "attention_launch": achieved,
                                      "frac_of_loop_with_reads": achieved / ladder["plus_operand_reads_from_lds"],
                                      "what": "MFMA-only loop on Q's values, then with the softmax arithmetic and the LDS operand "
                                              "reads of the attention loop added at the kernel's density (pda_probe_loop_rate)"}
    # the pipeline against ONE launch over all 24 heads (no groups, no hand-off): what the granularity costs
    with torch.cuda.stream(cs):
        ms_one = _event_ms(torch, cs, lambda: pda.attn_fwd(q, k, v, out, lse, w.scale, stream=cs), iters=2)
    res["pipeline"]["single_launch_all_heads_ms"] = ms_one
    res["pipeline"]["pipeline_over_single_launch"] = res["pipeline"]["total_ms_mean"] / ms_one
    # same-run reference for the HBM-bound kernels: torch's device-to-device copy of the full output tensor
    with torch.cuda.stream(cs):
        ms_t = _event_ms(torch, cs, lambda: sink.copy_(out))
    copy_bytes = 2.0 * out.numel() * 4
    res["roofline_merge"]["same_run_copy"] = {"torch_copy_GBs": copy_bytes / (ms_t * 1e-3) * 1e-9, "bytes": copy_bytes,
                                              "what": "torch fp32 copy_ of the [24, 119056, 128] output on the compute stream"}
    if not args.no_next_rows:
        del qr, kc, kc_out, outq, lseq
        res["next_rows"] = next_rows(pda, torch, w, q, k, v, out, lse, sink, cs, ds, args.t_linear_ms)
    if not args.no_all_configs:
        # every workload of the benchmark spec through pda_attn_fwd, after the timed steps (not part of `value`)
        # (C4 and C5 reuse the step's tensors: the first 3 and 6 heads of the C4 workload)
        res["all_configs"] = {f"c{i}": measure_config(pda, torch, i, cs, tensors=((qb, kb, vb), (q, k, v)) if i >= 4 else None)
                              for i in (1, 2, 3, 4, 5)}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, qb, kb, vb)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
