#!/usr/bin/env python3
"""Benchmark of the Round Attention hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch with every input resident in
HBM: round scores at the watershed layer and round selection (one call) -> round-sparse attention of a
post-watershed layer (decode, or question prefill for the prefill workload).  Prints ONE JSON line.

The headline is the largest single-GPU decode configuration, cfg5 (70B-shaped slice, batch 64, 32K-token
contexts in 16-token pages), at the default selection rule (lambda = 1): whole-step throughput, the
roofline figure of the decode-attention kernel measured live with events on its launch, the same kernel at
three kept-token fractions (about 6 %, 14 % and 60 %), the fp64 CPU oracle timed on a sample of the same
batch (which also gives the parity figures of the timed inputs), and compact results of the other
configurations: cfg2 (launch-bound small batch), cfg3 (question prefill on the matrix cores) and cfg4
(long context, selected rounds staged from pinned host memory while the 24 layers decode).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg1|cfg2|cfg3|cfg4] [--no-extras]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
CACHE_DEFEAT_BYTES = 512 << 20  # bytes touched between two uses of the same buffer (Infinity Cache: 256 MB)
MIN_TIMED_SECONDS = 0.2         # the timed region is repeated until it is at least this long
METRIC = "round-sparse decode attn tokens/s + achieved HBM GB/s (% of peak), 1 GPU"

WORKLOADS = {
    "cfg1": "tiny fp32: B=1, 4/2 heads, d=64, 8 rounds x 64 tokens, decode",
    "cfg2": "Llama-3-8B-shaped layer, bf16, B=8 decode, 32/8 heads, d=128, 20 rounds of U[200,1000] tokens",
    "cfg3": "question prefill, bf16, B=4, q_len=128, 32/8 heads, d=128, 60 lognormal rounds totalling 32K tokens",
    "cfg4": "long context, bf16, B=16 decode, 32/8 heads, d=128, 200 lognormal rounds totalling 128K tokens, "
            "24 post-watershed layers staged from pinned host memory",
    "cfg5": "70B-shaped layer slice, bf16, B=64 decode, 64/8 heads, d=128, 50 rounds of U[300,1000] tokens, "
            "16-token paged blocks",
}
# HBM bytes per launch of the attention kernel (read + written) from hardware-counter runs (rocprofv3 --pmc
# FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for a 1 GiB copy: 2 KiB and 1 KiB per
# count).  RECORDED figures for the workload's own inputs at lambda = 1, copied from the files named below; they are
# not measurements of the current run, and other lambda / alpha report null.
RECORDED_TRAFFIC = {
    ("cfg5", "ra_round_sparse_attn_decode"): 1195384732 + 6290224,
    ("cfg2", "ra_round_sparse_attn_decode"): 49712314 + 1630784,
}
TRAFFIC_SOURCES = {
    "cfg5": "profiles/attn_mfma_kernel_cfg5_paged_decode.md",
    "cfg2": "profiles/attn_mfma_kernel_cfg2_small_batch_decode.md",
}
MFMA_BUSY_SOURCE = "profiles/attn_prefill_mfma_kernel_cfg3_question_prefill.md (rocprofv3 --pmc; recorded, not measured in this run)"
RECORDED_MFMA_BUSY = {"scores_prefill_mfma_kernel": 0.381, "attn_prefill_mfma_kernel": 0.476}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg5", choices=sorted(WORKLOADS))
    ap.add_argument("--lam", type=float, default=1.0, help="multiplier of the adaptive selection rule")
    ap.add_argument("--alpha", type=float, default=None, help="override the key bias strength of the workload")
    ap.add_argument("--replicas", type=int, default=0, help="input replicas rotated through (0 = enough to defeat the Infinity Cache)")
    ap.add_argument("--prefill-p", default="bf16x2", choices=["bf16x2", "f16"],
                    help="how the many-row prefill kernel feeds P to the matrix cores (ra_set_prefill_precision); "
                         "f16 is the named lower-precision mode and is reported as such in config")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the workload itself: no kept-fraction points, no cfg2 / cfg3 / cfg4 summaries")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three device-to-device copies of 1 GiB, so that a hardware-counter run of this "
                         "command contains a copy kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--sweep", action="store_true",
                    help="cfg5 only: measure the key bias alpha in {0.5, 1, 2, 4} x lambda in {0, 0.5, 1} (kept fraction "
                         "from about 5 to 60 %%) and print one JSON line with a `sweep` table instead of the usual line")
    ap.add_argument("--no-dense-comparison", action="store_true",
                    help="skip the attention-over-all-rounds timing (keeps a kernel trace of the step clean)")
    ap.add_argument("--monitor", action="store_true",
                    help="time the statistics beside the hot path (answer re-scoring, selection coverage, watershed curve) "
                         "on cfg2 and cfg5; prints one JSON line with a `monitor` list")
    ap.add_argument("--watershed", action="store_true",
                    help="measure the watershed layer (decode: cfg2, cfg5; question prefill: cfg3): score pass + dense attention as two calls "
                         "against the fused call; prints one JSON line with a `watershed_layer` list")
    ap.add_argument("--cpu-baseline-seqs", type=int, default=0, help="sequences the oracle is timed on (0 = auto)")
    ap.add_argument("--stage-order", default="grouped", choices=["round", "layer", "grouped"],
                    help="cfg4: order of the host-to-device copies")
    return ap.parse_args()


def cpu_baseline(w, lam: float, seqs, gpu=None):
    """Time the fp64 oracle (as it stands) on the host cores for the same step on a bounded sample of
    the batch.  Input generation is excluded: only the oracle's arithmetic is timed.  With the GPU's outputs of
    the same inputs (`gpu` = S, sel_idx, n_sel, out as host arrays) the sample also gives the parity figures."""
    from oracle import round_attention as ora
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    seqs = list(seqs)
    data = []
    for b in seqs:
        R = w.n_rounds(b)
        data.append(dict(q0=w.q(0)[b], q1=w.q(1)[b], k0=[w.k_round(b, 0, r) for r in range(R)],
                         k1=[w.k_round(b, 1, r) for r in range(R)], v1=[w.v_round(b, 1, r) for r in range(R)],
                         ck0=None if w.cur_len == 0 else w.cur_k(0)[b], ck1=None if w.cur_len == 0 else w.cur_k(1)[b],
                         cv1=None if w.cur_len == 0 else w.cur_v(1)[b]))
    # the sample is repeated until about ten seconds of oracle work have been timed (a single pass over a small
    # workload takes a fraction of a second, too little to time well), at most 100 passes
    passes, dt, first = 0, 0.0, []
    t0 = time.perf_counter()
    while passes < 100 and (passes == 0 or dt < 10.0):
        for d in data:
            _, S = ora.round_scores(d["q0"], d["k0"], w.scale, d["ck0"])
            sel, info = ora.select_rounds(S, lam=lam)
            O, _ = ora.sparse_attention(d["q1"], d["k1"], d["v1"], sel, w.scale, d["ck1"], d["cv1"])
            if passes == 0:
                first.append((S, sel, info, O))
        passes += 1
        dt = time.perf_counter() - t0
    res = {"value": passes * len(seqs) * w.q_len / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": f"sequences {seqs} of the {w.B} of the same workload and inputs, one post-watershed layer, whole "
                     f"step (scores, selection, sparse attention) in fp64 numpy, {passes} pass(es) in {dt:.2f} s"}
    parity = None
    if gpu is not None:
        S_g, sel_g, n_g, out_g = gpu
        row, big, margin, score, exact = 0.0, 0.0, float("inf"), 0.0, True
        for b, (S, sel, info, O) in zip(seqs, first):
            R = w.n_rounds(b)
            score = max(score, float(np.abs(S_g[b, :R] - S).max()))
            exact = exact and sel_g[b, :n_g[b]].tolist() == sel
            if info["margin"] is not None:
                margin = min(margin, float(info["margin"]))
            ref = O if out_g[b].ndim == 3 else O[0]
            row = max(row, ora.row_error(out_g[b], ref))
            big = max(big, ora.large_entry_error(out_g[b], ref))
        parity = {"sequences_checked": seqs, "selection_bit_exact": bool(exact), "min_margin": margin,
                  "max_score_error": score, "max_row_error": row, "max_large_entry_error": big,
                  "note": "GPU outputs of the timed inputs against the fp64 oracle; row error = max|out - ref| / "
                          "max|ref| per (token, head) row, bar 2e-3; large-entry error = elementwise relative error "
                          "on entries of at least 5 % of their row's largest magnitude"}
    return res, parity


def cpu_baseline_once(w, lam, b, gpu):
    """One oracle pass over sequence b (untimed use): the parity figures of the GPU outputs `gpu`."""
    from oracle import round_attention as ora
    R = w.n_rounds(b)
    ck0 = None if w.cur_len == 0 else w.cur_k(0)[b]
    _, S = ora.round_scores(w.q(0)[b], [w.k_round(b, 0, r) for r in range(R)], w.scale, ck0)
    sel, info = ora.select_rounds(S, lam=lam)
    O, _ = ora.sparse_attention(w.q(1)[b], [w.k_round(b, 1, r) for r in range(R)], [w.v_round(b, 1, r) for r in range(R)],
                                sel, w.scale, None if w.cur_len == 0 else w.cur_k(1)[b],
                                None if w.cur_len == 0 else w.cur_v(1)[b])
    S_g, sel_g, n_g, out_g = gpu
    ref = O if out_g[b].ndim == 3 else O[0]
    return O, {"selection_bit_exact": sel_g[b, :n_g[b]].tolist() == sel, "margin": info["margin"],
               "max_score_error": float(np.abs(S_g[b, :R] - S).max()), "max_row_error": ora.row_error(out_g[b], ref),
               "max_large_entry_error": ora.large_entry_error(out_g[b], ref)}


def bench_step(name, plan, alpha, replicas, dense=True, keep_outputs=False, p_mode=0):
    """scores + selection -> sparse attention on one post-watershed layer, everything resident in HBM.
    `plan` is a list of (lambda, steps, warmup, min_seconds); returns one result per entry."""
    import torch
    import paper_2502_15294_amd as ra
    from synth import make_workload
    from synth.device import Engine, device_view, to_device

    over = {} if alpha is None else {"alpha": alpha}
    w = make_workload(name, **over)
    prefill = w.q_len > 1
    eb = 2 if w.dtype == "bf16" else 4
    eng = Engine(w)
    ra.ra_set_prefill_precision(eng.ctx, p_mode)
    t_gen = time.perf_counter()
    view0 = device_view(w, 0, with_v=False, threads=16)
    view1 = device_view(w, 1, threads=16)
    q0 = to_device(w.q(0), w.dtype)
    q1 = to_device(w.q(1) if prefill else w.q(1)[:, 0], w.dtype)
    ck0 = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    ck1 = to_device(w.cur_k(1), w.dtype) if w.cur_len else None
    cv1 = to_device(w.cur_v(1), w.dtype) if w.cur_len else None
    cl1 = torch.full((w.B,), w.cur_len, dtype=torch.int32, device="cuda") if w.cur_len else None
    t_gen = time.perf_counter() - t_gen
    hist_tokens = sum(w.total_tokens(b) for b in range(w.B))
    k_bytes_tok = w.Hkv * w.d * eb

    def measure(lam, steps, warmup, min_seconds):
        params = ra.make_select_params(lam=lam)
        P = torch.empty((w.B, w.Hq, view0.R_max), dtype=torch.float32, device="cuda")
        S = torch.empty((w.B, view0.R_max), dtype=torch.float32, device="cuda")
        sel_idx = torch.empty((w.B, view0.R_max), dtype=torch.int32, device="cuda")
        n_sel = torch.empty((w.B,), dtype=torch.int32, device="cuda")
        out = torch.empty((w.B, w.q_len, w.Hq, w.d) if prefill else (w.B, w.Hq, w.d), dtype=torch.float32, device="cuda")
        lse = torch.empty((w.B, w.q_len, w.Hq) if prefill else (w.B, w.Hq), dtype=torch.float32, device="cuda")

        def attend(v1, sel=True):
            si, ns = (sel_idx, n_sel) if sel else (None, None)
            if prefill:
                ra.ra_round_sparse_attn_prefill(eng.ctx, q1, v1, si, ns, ck1, cv1, scale=w.scale, out=out, lse=lse)
            else:
                ra.ra_round_sparse_attn_decode(eng.ctx, q1, v1, si, ns, ck1, cv1, cl1, scale=w.scale, out=out, lse=lse)

        def step(v0, v1, ev=None):
            if ev: ev[0].record()
            ra.ra_round_scores_select(eng.ctx, q0, v0, params, ck0, scale=w.scale, scores_head=P, scores=S,
                                      sel_idx=sel_idx, n_sel=n_sel)
            if ev: ev[1].record()
            attend(v1)
            if ev: ev[2].record()

        step(view0, view1)
        torch.cuda.synchronize()
        n_sel_h, sel_h = n_sel.cpu().numpy(), sel_idx.cpu().numpy()
        kept = (S.cpu().numpy(), sel_h.copy(), n_sel_h.copy(), out.cpu().numpy()) if keep_outputs else None
        sel_tokens = int(sum(int(w.lens[b][sel_h[b, :n_sel_h[b]]].sum()) for b in range(w.B)))
        step_bytes = hist_tokens * k_bytes_tok + sel_tokens * 2 * k_bytes_tok
        n_rep = replicas or int(max(1, min(8, -(-CACHE_DEFEAT_BYTES // max(step_bytes, 1)))))

        def clone_view(v):
            k, vv, seg_off, seg_len, n_rounds, bt, seg_off_v = v.tensors
            return ra.KVView(k.clone(), None if vv is None else vv.clone(), seg_off, seg_len, n_rounds, v.Hkv, v.d,
                             v.c.max_tokens, block_table=bt, block_size=v.c.block_size, seg_off_v=seg_off_v)

        reps = [(view0, view1)] + [(clone_view(view0), clone_view(view1)) for _ in range(n_rep - 1)]
        for i in range(warmup):
            step(*reps[i % n_rep])
        # EXACTLY `steps` steps per pass, the pass repeated until the timed region is long enough to time well
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        passes = 0
        while True:
            for i in range(steps):
                step(*reps[i % n_rep])
            torch.cuda.synchronize()
            passes += 1
            total = time.perf_counter() - t0
            if total >= min_seconds or passes >= 10000:
                break
        iters = passes * steps

        # Per-call durations: a second pass with events between the calls (recording them costs about 3 us each,
        # so they stay out of the timed region above).
        n_ev = min(max(steps, 20), 100)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_ev)]
        for i in range(n_ev):
            step(*reps[i % n_rep], evs[i])
        torch.cuda.synchronize()
        ms = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(2)] for e in evs])
        avg_ms, med_ms = ms.mean(axis=0), np.median(ms, axis=0)

        # Duration of the streaming kernel inside the two calls (the library attaches two events to its launch on
        # request, which then carry the kernel's own start and end time stamps); separate pass.
        ra.ra_profile_kernels(eng.ctx, True)
        kern_ms = [[], []]
        for i in range(min(max(steps, 20), 50)):
            v0, v1 = reps[i % n_rep]
            ra.ra_round_scores_select(eng.ctx, q0, v0, params, ck0, scale=w.scale, scores_head=P, scores=S,
                                      sel_idx=sel_idx, n_sel=n_sel)
            kern_ms[0].append(ra.ra_profile_last_ms(eng.ctx))
            attend(v1)
            kern_ms[1].append(ra.ra_profile_last_ms(eng.ctx))
        ra.ra_profile_kernels(eng.ctx, False)

        # The paper's comparison (Sec. 4.3, Fig. 3: Round Attention against dense attention), at the level of one
        # post-watershed layer's attention call: all rounds against the selected ones, same kernel, same inputs.
        def wall(fn):
            n = min(steps, 50)
            for i in range(min(warmup, 5)):
                fn(reps[i % n_rep][1])
            torch.cuda.synchronize()
            t = time.perf_counter()
            for i in range(n):
                fn(reps[i % n_rep][1])
            torch.cuda.synchronize()
            return (time.perf_counter() - t) / n * 1e3

        dense_ms, sparse_ms = (wall(lambda v: attend(v, sel=False)), wall(attend)) if dense else (None, None)
        many_rows = w.q_len * (w.Hq // w.Hkv) > 16
        mfma = w.dtype == "bf16" and w.d == 128
        scores_kernel = ("scores_prefill_mfma_kernel" if many_rows else "scores_mfma_kernel") if mfma else "scores_stream_kernel"
        attn_kernel = (("attn_prefill_mfma_kernel" if w.q_len * (w.Hq // w.Hkv) > 32 else "attn_mfma_kernel") if mfma
                       else "decode_generic_kernel")

        q_rows = w.B * w.q_len * w.Hq
        attn_name = "ra_round_sparse_attn_prefill" if prefill else "ra_round_sparse_attn_decode"
        groups = {
            "ra_round_scores_select": {"ms": float(avg_ms[0]), "median_ms": float(med_ms[0]),
                                       "bytes": int(hist_tokens * k_bytes_tok + q_rows * w.d * eb),
                                       "kernel": scores_kernel, "kernel_ms": float(np.mean(kern_ms[0]))},
            attn_name: {"ms": float(avg_ms[1]), "median_ms": float(med_ms[1]),
                        "bytes": int((sel_tokens + w.B * w.cur_len) * 2 * k_bytes_tok + q_rows * w.d * (eb + 4)),
                        "kernel": attn_kernel, "kernel_ms": float(np.mean(kern_ms[1]))},
        }
        for g in groups.values():
            g["GB/s"] = g["bytes"] / (g["ms"] * 1e-3) / 1e9 if g["ms"] > 0 else None
            g["kernel_GB/s"] = g["bytes"] / (g["kernel_ms"] * 1e-3) / 1e9 if g["kernel_ms"] > 0 else None
        if prefill:  # contractions: QK^T for the score pass, QK^T + PV for attention (causal part of the question half)
            for key, mult, toks in (("ra_round_scores_select", 2, hist_tokens), (attn_name, 4, sel_tokens)):
                fl = mult * q_rows * w.d * (toks / w.B + w.cur_len / 2)
                groups[key]["flop"] = fl
                groups[key]["kernel_TFLOP/s"] = fl / (groups[key]["kernel_ms"] * 1e-3) / 1e12
        g_attn = groups[attn_name]
        if prefill:
            roof = {"bound": "mfma", "kernel": attn_kernel, "achieved": g_attn["kernel_TFLOP/s"],
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": g_attn["kernel_TFLOP/s"] / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": None, "whole_call_achieved": g_attn["flop"] / (g_attn["ms"] * 1e-3) / 1e12}
        else:
            roof = {"bound": "hbm", "kernel": attn_kernel, "achieved": g_attn["kernel_GB/s"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": g_attn["kernel_GB/s"] / HBM_PEAK_GBS,
                    "traffic": RECORDED_TRAFFIC.get((w.name, attn_name)) if (lam == 1.0 and alpha is None) else None,
                    "traffic_source": (TRAFFIC_SOURCES.get(w.name, "none recorded for this workload")
                                       + " (rocprofv3 --pmc runs of this command; recorded, not measured in this run)"),
                    "whole_call_achieved": g_attn["GB/s"],
                    "algorithmic_bytes_per_launch": g_attn["bytes"], "kernel_us": g_attn["kernel_ms"] * 1e3,
                    "score_pass": {"kernel": scores_kernel, "achieved": groups["ra_round_scores_select"]["kernel_GB/s"],
                                   "frac": groups["ra_round_scores_select"]["kernel_GB/s"] / HBM_PEAK_GBS}}
        res = {
            "value": w.B * w.q_len * iters / total,
            "ms_per_step": total / iters * 1e3,
            "timed_region_s": total, "timed_iterations": iters,
            "dtype": w.dtype,
            "config": {"workload": f"{name}: {WORKLOADS[name]}", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "d": w.d,
                       "q_len": w.q_len, "history_tokens": hist_tokens, "selected_tokens": sel_tokens,
                       "kept_token_fraction": sel_tokens / max(hist_tokens, 1),
                       "selected_rounds": [int(x) for x in n_sel_h], "lambda": lam, "alpha": w.alpha,
                       "replicas_rotated": n_rep,
                       "step": f"ra_round_scores_select -> {attn_name}"},
            "roofline": roof,
            "kernel_groups": groups,
            "dense_comparison": None if not dense else {
                                 "dense_attention_ms": dense_ms, "round_sparse_attention_ms": sparse_ms,
                                 "attention_speedup": dense_ms / sparse_ms,
                                 "note": "one post-watershed layer: attention over all rounds against attention over the "
                                         "selected rounds (the score pass and the selection run once per question, "
                                         "not per layer or per decoded token)"},
            "input_generation_s": t_gen,
            "_gpu_outputs": kept,
        }
        return res

    results = [measure(*p) for p in plan]
    eng.close()
    return results, w


def bench_watershed(name, steps, warmup):
    """Decode (or question prefill) at the watershed layer: round scores + dense attention as two calls (K read twice)
    against the fused call that takes the scores from the attention pass itself."""
    import torch
    import paper_2502_15294_amd as ra
    from synth import make_workload
    from synth.device import Engine, device_view, to_device

    w = make_workload(name)
    prefill = w.q_len > 1
    eng = Engine(w)
    view = device_view(w, 0, threads=16)          # the watershed layer, keys and values
    q4 = to_device(w.q(0), w.dtype)
    q = q4 if prefill else to_device(w.q(0)[:, 0], w.dtype)
    ck = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    cv = to_device(w.cur_v(0), w.dtype) if w.cur_len else None
    hist_tokens = sum(w.total_tokens(b) for b in range(w.B))
    kv_bytes = hist_tokens * 2 * w.Hkv * w.d * 2
    P = torch.empty((w.B, w.Hq, view.R_max), dtype=torch.float32, device="cuda")
    S = torch.empty((w.B, view.R_max), dtype=torch.float32, device="cuda")
    out = torch.empty((w.B, w.q_len, w.Hq, w.d) if prefill else (w.B, w.Hq, w.d), dtype=torch.float32, device="cuda")
    lse = torch.empty((w.B, w.q_len, w.Hq) if prefill else (w.B, w.Hq), dtype=torch.float32, device="cuda")

    def clone_view(v):
        k, vv, seg_off, seg_len, n_rounds, bt, seg_off_v = v.tensors
        return ra.KVView(k.clone(), vv.clone(), seg_off, seg_len, n_rounds, v.Hkv, v.d, v.c.max_tokens, block_table=bt,
                         block_size=v.c.block_size, seg_off_v=seg_off_v)

    n_rep = int(max(1, min(4, -(-CACHE_DEFEAT_BYTES // kv_bytes))))
    reps = [view] + [clone_view(view) for _ in range(n_rep - 1)]

    def separate(v):
        if prefill:
            ra.ra_round_scores(eng.ctx, q4, v, ck, scale=w.scale, scores_head=P, scores=S)
            ra.ra_round_sparse_attn_prefill(eng.ctx, q, v, None, None, ck, cv, scale=w.scale, out=out, lse=lse)
        else:
            ra.ra_round_scores(eng.ctx, q4, v, scale=w.scale, scores_head=P, scores=S)
            ra.ra_round_sparse_attn_decode(eng.ctx, q, v, scale=w.scale, out=out, lse=lse)

    def fused(v):
        if prefill:
            ra.ra_watershed_attn_prefill(eng.ctx, q, v, ck, cv, scale=w.scale, out=out, lse=lse, scores_head=P, scores=S)
        else:
            ra.ra_watershed_attn_decode(eng.ctx, q, v, scale=w.scale, out=out, lse=lse, scores_head=P, scores=S)

    res = {}
    for label, fn in (("two_calls", separate), ("fused", fused)):
        for i in range(warmup):
            fn(reps[i % n_rep])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(reps[i % n_rep])
        torch.cuda.synchronize()
        res[label + "_ms"] = (time.perf_counter() - t0) / steps * 1e3
    ra.ra_profile_kernels(eng.ctx, True)
    km = []
    for i in range(min(steps, 20)):
        fused(reps[i % n_rep])
        km.append(ra.ra_profile_last_ms(eng.ctx))
    ra.ra_profile_kernels(eng.ctx, False)
    kms = float(np.mean(km))
    res.update({"workload": f"{name}: {WORKLOADS[name]}", "history_tokens": hist_tokens, "replicas_rotated": n_rep,
                "fused_kernel": "attn_prefill_mfma_kernel" if prefill else "attn_mfma_kernel", "fused_kernel_ms": kms,
                "speedup": res["two_calls_ms"] / res["fused_ms"]})
    if prefill:
        flops = 4 * w.B * w.q_len * w.Hq * w.d * (hist_tokens / w.B + w.cur_len / 2)
        res["fused_kernel_TFLOP/s"] = flops / kms / 1e9
    else:
        res["kv_bytes"] = kv_bytes
        res["fused_kernel_GB/s"] = kv_bytes / kms / 1e6
    eng.close()
    return res


def bench_long_context(steps, warmup, lam, order_name, pinned_budget=24 << 30, distinct_layers=6):
    """Config 4: scores on the watershed layer, selection, staging of the selected rounds of 24
    post-watershed layers from pinned host memory on a side stream, decode over the staged views."""
    import torch
    import paper_2502_15294_amd as ra
    from concurrent.futures import ThreadPoolExecutor
    from synth import make_workload, pack_round_host, round_host_elems
    from synth.device import Engine, device_view, to_device

    w = make_workload("cfg4")
    L_all = w.n_post_layers
    eng = Engine(w)
    t_gen = time.perf_counter()
    view0 = device_view(w, 0, with_v=False, threads=16)
    q0 = to_device(w.q(0), w.dtype)
    params = ra.make_select_params(lam=lam)
    P, S, sel_idx, n_sel = ra.ra_round_scores_select(eng.ctx, q0, view0, params, scale=w.scale)
    sel_h, n_h = sel_idx.cpu(), n_sel.cpu()                       # the path's one host synchronisation
    sel_tokens = int(sum(int(w.lens[b][sel_h[b, :n_h[b]].numpy()].sum()) for b in range(w.B)))
    hist_tokens = sum(w.total_tokens(b) for b in range(w.B))
    k_bytes_tok = w.Hkv * w.d * 2

    # Host store: the selected rounds are materialised in pinned memory with as many of their post-watershed layers
    # as `pinned_budget` allows (the boxes used refuse to pin much more than that; the 24 decode launches cycle
    # through the layers that are there); every other round is registered with one shared pinned buffer of the largest
    # size (it is never copied), because the full host store would take ~206 GB.  To bound the time spent drawing
    # random numbers, only `distinct_layers` layers are generated; the further layer slots of a round's tensor hold
    # copies of them (same bytes to move, same shapes to attend over).
    L = int(max(1, min(L_all, pinned_budget // max(1, sel_tokens * 2 * k_bytes_tok))))
    Lg = min(L, distinct_layers)
    gen_layers = list(range(1, Lg + 1))
    jobs = [(b, int(r)) for b in range(w.B) for r in sel_h[b, :n_h[b]].tolist()]
    sel_set = set(jobs)
    host = {}
    for (b, r) in jobs:
        host[(b, r)] = torch.empty(round_host_elems(w, int(w.lens[b][r]), L), dtype=torch.int16, pin_memory=True)

    def fill(job):
        b, r = job
        buf = host[job].numpy().view(np.uint16)
        per = buf.size // L
        pack_round_host(w, b, r, gen_layers, out=buf[:per * Lg])
        for l in range(Lg, L):
            buf[l * per:(l + 1) * per] = buf[(l % Lg) * per:(l % Lg + 1) * per]
    with ThreadPoolExecutor(max_workers=16) as ex:
        list(ex.map(fill, jobs))
    max_unsel = max([int(w.lens[b][r]) for b in range(w.B) for r in range(w.n_rounds(b)) if (b, r) not in sel_set] + [1])
    dummy = torch.zeros(round_host_elems(w, max_unsel, L), dtype=torch.int16, pin_memory=True)
    pool_bytes = sum(t.numel() * 2 for t in host.values()) + (1 << 20)
    store = ra.ra_kv_store_create(0, L, w.B, w.R_max, w.Hkv, w.d, ra.RA_BF16, pool_bytes)
    for b in range(w.B):
        for r in range(w.n_rounds(b)):
            ra.ra_kv_store_register_round(store, b, r, host.get((b, r), dummy), int(w.lens[b][r]))
    qs = [to_device(w.q(1 + li % Lg)[:, 0], w.dtype) for li in range(L_all)]
    t_gen = time.perf_counter() - t_gen
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda")
    lse = torch.empty((w.B, w.Hq), dtype=torch.float32, device="cuda")
    order = {"round": ra.RA_STAGE_ROUND_MAJOR, "layer": ra.RA_STAGE_LAYER_MAJOR, "grouped": ra.RA_STAGE_GROUPED}[order_name]
    side = torch.cuda.Stream()

    # ---- staging alone, then staging overlapped with the 24 layers of decode -------------------------------
    def stage_and_decode(run_layers):
        ev0 = torch.cuda.Event(enable_timing=True)
        ev_first = torch.cuda.Event(enable_timing=True)
        ev_all = torch.cuda.Event(enable_timing=True)
        ev_done = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t_host = time.perf_counter()
        ev0.record(side)
        ra.ra_kv_store_stage(store, sel_h, n_h, order, side)
        ev_all.record(side)
        t_host = time.perf_counter() - t_host
        if run_layers:
            # the 24 layers' attention calls follow the transfer as they would with 24 layers in the store: call li
            # waits for the slot that holds the same share of the bytes (li * L / 24)
            for li in range(L_all):
                slot = li * L // L_all
                ra.ra_kv_store_wait_layer(store, slot)
                if li == 0:
                    ev_first.record()
                ra.ra_round_sparse_attn_decode(eng.ctx, qs[li], ra.ra_kv_store_layer_view(store, slot),
                                               scale=w.scale, out=out, lse=lse)
            ev_done.record()
        torch.cuda.synchronize()
        r = {"host_issue_ms": t_host * 1e3, "all_layers_ready_ms": ev0.elapsed_time(ev_all)}
        if run_layers:
            r["first_layer_started_ms"] = ev0.elapsed_time(ev_first)
            r["last_layer_done_ms"] = ev0.elapsed_time(ev_done)
        return r

    stage_only = stage_and_decode(False)
    staged, registered, n_copies = ra.ra_kv_store_stats(store)
    ra.ra_kv_store_release(store)
    overlapped = stage_and_decode(True)
    views = [ra.ra_kv_store_layer_view(store, li) for li in range(L)]

    # ---- steady state: everything resident (watershed K in HBM, selected rounds staged) -----------------------
    def step(ev=None):
        if ev: ev[0].record()
        ra.ra_round_scores_select(eng.ctx, q0, view0, params, scale=w.scale, scores_head=P, scores=S, sel_idx=sel_idx,
                                  n_sel=n_sel)
        if ev: ev[1].record()
        for li in range(L_all):
            ra.ra_round_sparse_attn_decode(eng.ctx, qs[li], views[li % L], scale=w.scale, out=out, lse=lse)
        if ev: ev[2].record()

    steps = max(1, min(steps, 20))
    warmup = min(warmup, 3)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    passes = 0
    while True:
        for i in range(steps):
            step()
        torch.cuda.synchronize()
        passes += 1
        total = time.perf_counter() - t0
        if total >= MIN_TIMED_SECONDS:
            break
    iters = passes * steps
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]  # per-call times: second pass
    for i in range(steps):
        step(evs[i])
    torch.cuda.synchronize()
    ms = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(2)] for e in evs])
    avg_ms, med_ms = ms.mean(axis=0), np.median(ms, axis=0)
    # duration of the streaming kernels themselves (events attached to their launches by the library)
    ra.ra_profile_kernels(eng.ctx, True)
    kern_ms = [[], []]
    for i in range(min(steps, 5)):
        ra.ra_round_scores_select(eng.ctx, q0, view0, params, scale=w.scale, scores_head=P, scores=S, sel_idx=sel_idx,
                                  n_sel=n_sel)
        kern_ms[0].append(ra.ra_profile_last_ms(eng.ctx))
        for li in range(L_all):
            ra.ra_round_sparse_attn_decode(eng.ctx, qs[li], views[li % L], scale=w.scale, out=out, lse=lse)
            kern_ms[1].append(ra.ra_profile_last_ms(eng.ctx))
    ra.ra_profile_kernels(eng.ctx, False)
    q_rows = w.B * w.Hq
    groups = {
        "ra_round_scores_select": {"ms": float(avg_ms[0]), "median_ms": float(med_ms[0]),
                                   "bytes": int(hist_tokens * k_bytes_tok + q_rows * w.d * 2),
                                   "kernel": "scores_mfma_kernel", "kernel_ms": float(np.mean(kern_ms[0]))},
        "ra_round_sparse_attn_decode": {"ms": float(avg_ms[1]) / L_all, "median_ms": float(med_ms[1]) / L_all,
                                        "bytes": int(sel_tokens * 2 * k_bytes_tok + q_rows * w.d * 6),
                                        "launches_per_step": L_all,
                                        "kernel": "attn_mfma_kernel", "kernel_ms": float(np.mean(kern_ms[1]))},
    }
    for g in groups.values():
        g["GB/s"] = g["bytes"] / (g["ms"] * 1e-3) / 1e9
        g["kernel_GB/s"] = g["bytes"] / (g["kernel_ms"] * 1e-3) / 1e9
    g_dec = groups["ra_round_sparse_attn_decode"]
    decode_all_ms = float(avg_ms[1])
    exposed_ms = max(0.0, overlapped["last_layer_done_ms"] - overlapped["all_layers_ready_ms"])
    res = {
        "value": w.B * iters / total,
        "ms_per_step": total / iters * 1e3,
        "timed_region_s": total, "timed_iterations": iters,
        "dtype": "bf16",
        "config": {"workload": f"cfg4: {WORKLOADS['cfg4']}", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "d": w.d, "q_len": 1,
                   "post_watershed_layers": L_all, "layers_in_host_store": L, "distinct_layers_generated": Lg,
                   "history_tokens": hist_tokens, "selected_tokens": sel_tokens,
                   "kept_token_fraction": sel_tokens / hist_tokens, "selected_rounds": [int(x) for x in n_h],
                   "lambda": lam, "alpha": w.alpha,
                   "step": f"ra_round_scores_select -> {L_all} x ra_round_sparse_attn_decode on staged views"},
        "roofline": {"bound": "hbm", "kernel": "attn_mfma_kernel", "achieved": g_dec["kernel_GB/s"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": g_dec["kernel_GB/s"] / HBM_PEAK_GBS, "traffic": None,
                     "whole_call_achieved": g_dec["GB/s"]},
        "kernel_groups": groups,
        "staging": {"order": order_name, "bytes": staged, "copies": n_copies, "registered_bytes_logical": registered,
                    "alone": stage_only, "overlapped_with_decode": overlapped,
                    "h2d_GB/s": staged / (stage_only["all_layers_ready_ms"] * 1e-3) / 1e9,
                    "first_layer_start_over_all_ready": overlapped["first_layer_started_ms"] / overlapped["all_layers_ready_ms"],
                    "decode_of_all_layers_alone_ms": decode_all_ms,
                    "decode_exposed_after_last_copy_ms": exposed_ms,
                    "decode_hidden_fraction": 1.0 - min(1.0, exposed_ms / decode_all_ms),
                    "end_to_end_over_transfer_alone": overlapped["last_layer_done_ms"] / stage_only["all_layers_ready_ms"],
                    "layers_staged": L,
                    "note": "the selected rounds are materialised in pinned host memory with `layers_in_host_store` layer "
                            "slots each (`distinct_layers_generated` layers of random data, repeated); unselected rounds "
                            "share one buffer; staging is never part of `value`"},
        "input_generation_s": t_gen,
    }
    # ---- end of the turn: the new round of every sequence goes back to pinned host memory -------------------
    new_len, Lw = 512, min(L, 9)
    wb_store = ra.ra_kv_store_create(0, Lw, w.B, 1, w.Hkv, w.d, ra.RA_BF16,
                                     w.B * Lw * 2 * new_len * k_bytes_tok + (1 << 20))
    g = torch.Generator(device="cuda").manual_seed(4)
    cur_k = [torch.randn((w.B, new_len, w.Hkv, w.d), generator=g, device="cuda").bfloat16() for _ in range(Lw)]
    cur_v = [torch.randn((w.B, new_len, w.Hkv, w.d), generator=g, device="cuda").bfloat16() for _ in range(Lw)]
    wb_host = [torch.empty(ra.ra_kv_store_round_bytes(wb_store, new_len) // 2, dtype=torch.int16, pin_memory=True)
               for _ in range(w.B)]
    wb_round = torch.zeros(w.B, dtype=torch.int32)
    wb_len = torch.full((w.B,), new_len, dtype=torch.int32)
    wb = []
    for i in range(4):
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        torch.cuda.synchronize()
        e0.record()
        ra.ra_kv_store_save_round(wb_store, wb_round, wb_len, cur_k, cur_v, wb_host, None, side)
        e1.record()
        e2.record(side)
        saved = ra.ra_kv_store_save_wait(wb_store)
        torch.cuda.synchronize()
        wb.append((e0.elapsed_time(e1), e0.elapsed_time(e2)))
    pack_ms, total_ms = (float(np.mean([x[j] for x in wb[1:]])) for j in range(2))
    res["write_back"] = {"new_round_tokens": new_len, "sequences": w.B, "layers": Lw, "bytes": saved,
                         "gather_kernels_ms": pack_ms, "gather_GB/s": 2 * saved / (pack_ms * 1e-3) / 1e9,
                         "until_in_host_memory_ms": total_ms,
                         "d2h_GB/s": saved / ((total_ms - pack_ms) * 1e-3) / 1e9,
                         "all_24_layers_extrapolated_ms": total_ms * L_all / Lw}
    ra.ra_kv_store_destroy(wb_store)
    ra.ra_kv_store_release(store)
    ra.ra_kv_store_destroy(store)
    eng.close()
    return res, w


def bench_monitor(name, steps, warmup, n_layers):
    """The statistics beside the hot path: re-scoring of each decode token into the answer's running round
    distribution (against the plain score pass), the coverage of the selection, and the watershed curve over
    `n_layers` layers' score vectors."""
    import torch
    import paper_2502_15294_amd as ra
    from synth import make_workload
    from synth.device import Engine, device_view, to_device

    w = make_workload(name, cur_len=64)
    eng = Engine(w)
    view = device_view(w, 0, with_v=False, threads=16)
    q = to_device(w.q(0), w.dtype)
    ck = to_device(w.cur_k(0), w.dtype)
    P = torch.empty((w.B, w.Hq, view.R_max), dtype=torch.float32, device="cuda")
    S = torch.empty((w.B, view.R_max), dtype=torch.float32, device="cuda")
    acc = torch.zeros((w.B, w.Hq, view.R_max), dtype=torch.float32, device="cuda")
    sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, ra.ra_round_scores(eng.ctx, q, view, scale=w.scale)[1], view.n_rounds,
                                         ra.make_select_params(lam=0.0))
    layers = torch.rand((n_layers, w.B, view.R_max), device="cuda") + 0.01
    layers /= layers.sum(dim=2, keepdim=True)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    res = {"workload": f"{name}: {WORKLOADS[name]}, 64 tokens in the current round",
           "round_scores_ms": timed(lambda: ra.ra_round_scores(eng.ctx, q, view, scale=w.scale, scores_head=P, scores=S)),
           "round_scores_accumulate_ms": timed(lambda: ra.ra_round_scores_accumulate(eng.ctx, q, view, acc, cur_k=ck, scale=w.scale,
                                                                                     scores_head=P, scores=S)),
           "selection_coverage_ms": timed(lambda: ra.ra_selection_coverage(eng.ctx, S, sel_idx, n_sel)),
           "layer_divergence_layers": n_layers,
           "layer_divergence_ms": timed(lambda: ra.ra_layer_divergence(eng.ctx, layers, view.n_rounds))}
    eng.close()
    return res


def _compact(r):
    """A result of bench_step reduced to what a sub-entry of the line needs."""
    groups = {k: {kk: v[kk] for kk in ("ms", "kernel", "kernel_ms", "bytes", "GB/s", "kernel_GB/s", "kernel_TFLOP/s") if kk in v}
              for k, v in r["kernel_groups"].items()}
    return {"workload": r["config"]["workload"], "lambda": r["config"]["lambda"],
            "kept_token_fraction": r["config"]["kept_token_fraction"], "tokens/s": r["value"],
            "ms_per_step": r["ms_per_step"], "timed_iterations": r["timed_iterations"], "kernel_groups": groups,
            "roofline": {k: r["roofline"][k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac")}}


def _sweep_point(r):
    g = r["kernel_groups"]["ra_round_sparse_attn_decode"]
    return {"alpha": r["config"]["alpha"], "lambda": r["config"]["lambda"],
            "kept_token_fraction": r["config"]["kept_token_fraction"], "decode_kernel_us": g["kernel_ms"] * 1e3,
            "decode_kernel_GB/s": g["kernel_GB/s"], "frac_of_hbm_peak": g["kernel_GB/s"] / HBM_PEAK_GBS,
            "decode_call_us": g["ms"] * 1e3, "ms_per_step": r["ms_per_step"], "tokens/s": r["value"]}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 (nothing here uses a second GPU)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2502_15294_amd as ra
    ra.lib()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.pmc_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    head = {"metric": METRIC, "unit": "tokens/s", "n_gpus": 1, "data": "synthetic", "dtype": "bf16"}

    if args.watershed:
        rows = [bench_watershed("cfg2", 200, 20), bench_watershed("cfg5", 20, 3), bench_watershed("cfg3", 20, 3)]
        print(json.dumps({**head, "watershed_layer": rows}))
        return
    if args.monitor:
        rows = [bench_monitor("cfg2", 200, 20, 36), bench_monitor("cfg5", 20, 3, 28)]
        print(json.dumps({**head, "monitor": rows}))
        return
    if args.sweep:
        table = []
        for alpha in (0.5, 1.0, 2.0, 4.0):
            many, _ = bench_step("cfg5", [(l, 10, 2, 0.0) for l in (0.0, 0.5, 1.0)], alpha, 0, dense=False)
            table += [_sweep_point(r) for r in many]
        print(json.dumps({**head, "config": {"workload": f"cfg5: {WORKLOADS['cfg5']}", "steps": 10, "warmup": 2},
                          "sweep": table}))
        return

    dense = not args.no_dense_comparison
    extras = {}
    if args.workload == "cfg4":
        res, w = bench_long_context(args.steps, args.warmup, args.lam, args.stage_order)
        sample = [0, w.B // 2]
        gpu = None
    else:
        plan = [(args.lam, args.steps, args.warmup, MIN_TIMED_SECONDS)]
        sweep_here = args.workload == "cfg5" and not args.no_extras and args.alpha is None
        if sweep_here:
            plan.append((0.0, 20, 3, 0.0))  # same inputs, the "greater than the average" rule of Sec. 4.4: about 60 % kept
        many, w = bench_step(args.workload, plan, args.alpha, args.replicas, dense=dense, keep_outputs=True,
                             p_mode=ra.RA_PREFILL_P_F16 if args.prefill_p == "f16" else ra.RA_PREFILL_P_BF16X2)
        res = many[0]
        gpu = res.pop("_gpu_outputs")
        for r in many[1:]:
            r.pop("_gpu_outputs")
        if sweep_here:
            low, _ = bench_step("cfg5", [(1.0, 20, 3, 0.0)], 4.0, args.replicas, dense=False)  # stronger bias: about 6 % kept
            low[0].pop("_gpu_outputs")
            extras["kept_fraction_sweep"] = [_sweep_point(low[0]), _sweep_point(res), _sweep_point(many[1])]
        n = args.cpu_baseline_seqs or {"cfg1": w.B, "cfg2": w.B, "cfg3": 1, "cfg5": 8}.get(args.workload, 2)
        sample = sorted({int(round(i * (w.B - 1) / max(n - 1, 1))) for i in range(n)})
    result = {**head, "value": res.pop("value"), "steps": args.steps, "warmup": args.warmup,
              "ms_per_step": res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": res.pop("dtype")}
    res.pop("_gpu_outputs", None)
    result.update(res)
    result.update(extras)
    if args.workload != "cfg4" and result["config"].get("q_len", 1) > 1:
        result["config"]["prefill_p"] = args.prefill_p

    if not args.no_extras and args.workload == "cfg5":
        # the other configurations, compact (each also runs on its own with --workload)
        def guarded(label, fn):
            try:
                result[label] = fn()
            except Exception as e:  # a sub-entry must not take the headline down
                result[label] = {"error": f"{type(e).__name__}: {e}"}

        def run_cfg2():
            r, _ = bench_step("cfg2", [(1.0, 200, 20, MIN_TIMED_SECONDS)], None, 0, dense=False)
            r[0].pop("_gpu_outputs")
            return _compact(r[0])

        def run_cfg3():
            r, w3 = bench_step("cfg3", [(1.0, 50, 5, MIN_TIMED_SECONDS)], None, 0, dense=False, keep_outputs=True)
            gpu3 = r[0].pop("_gpu_outputs")
            c = _compact(r[0])
            c["mfma_busy"] = RECORDED_MFMA_BUSY
            c["mfma_busy_source"] = MFMA_BUSY_SOURCE
            c["frac_of_bf16_mfma_peak"] = {k: v["kernel_TFLOP/s"] / MFMA_BF16_PEAK_TFLOPS for k, v in c["kernel_groups"].items()}
            # the same step with the named fp16-P mode of the attention kernel (one pass over V instead of two)
            h, _ = bench_step("cfg3", [(1.0, 50, 5, MIN_TIMED_SECONDS)], None, 0, dense=False, keep_outputs=True,
                              p_mode=ra.RA_PREFILL_P_F16)
            gpu3h = h[0].pop("_gpu_outputs")
            g = h[0]["kernel_groups"]["ra_round_sparse_attn_prefill"]
            c["attention_with_p_f16"] = {"mode": "RA_PREFILL_P_F16 (ra_set_prefill_precision; not the default)",
                                         "kernel_ms": g["kernel_ms"], "kernel_TFLOP/s": g["kernel_TFLOP/s"],
                                         "frac_of_bf16_mfma_peak": g["kernel_TFLOP/s"] / MFMA_BF16_PEAK_TFLOPS,
                                         "ms_per_step": h[0]["ms_per_step"], "tokens/s": h[0]["value"]}
            if not args.no_cpu_baseline:  # one sequence of the batch against the oracle, both modes
                _, par = cpu_baseline_once(w3, 1.0, 0, gpu3)
                _, parh = cpu_baseline_once(w3, 1.0, 0, gpu3h)
                c["parity"] = {"sequence": 0, "p_bf16x2": par, "p_f16": parh}
            return c

        def run_cfg4():
            r, _ = bench_long_context(10, 2, 1.0, args.stage_order)
            st = r["staging"]
            return {"workload": r["config"]["workload"], "kept_token_fraction": r["config"]["kept_token_fraction"],
                    "steady_state": {"tokens/s": r["value"], "ms_per_step": r["ms_per_step"],
                                     "decode_kernel_GB/s": r["roofline"]["achieved"], "frac_of_hbm_peak": r["roofline"]["frac"],
                                     "decode_call_GB/s": r["roofline"]["whole_call_achieved"],
                                     "scores_kernel_GB/s": r["kernel_groups"]["ra_round_scores_select"]["kernel_GB/s"]},
                    "staging": {k: st[k] for k in ("order", "bytes", "copies", "h2d_GB/s", "first_layer_start_over_all_ready",
                                                   "decode_of_all_layers_alone_ms", "decode_exposed_after_last_copy_ms",
                                                   "decode_hidden_fraction", "end_to_end_over_transfer_alone",
                                                   "layers_staged")},
                    "staging_ms": {"alone_all_ready": st["alone"]["all_layers_ready_ms"],
                                   "overlapped_first_layer_started": st["overlapped_with_decode"]["first_layer_started_ms"],
                                   "overlapped_all_ready": st["overlapped_with_decode"]["all_layers_ready_ms"],
                                   "overlapped_last_layer_done": st["overlapped_with_decode"]["last_layer_done_ms"],
                                   "host_issue": st["alone"]["host_issue_ms"]},
                    "write_back": r["write_back"]}

        guarded("cfg2", run_cfg2)
        guarded("cfg3", run_cfg3)
        guarded("cfg4", run_cfg4)

    # the practical ceiling beside the published peak: what a plain read kernel reaches on this GPU right now
    ctx = ra.ra_create(0)
    ws = torch.empty(1 << 18, dtype=torch.uint8, device="cuda")
    ra.ra_set_workspace(ctx, ws)
    probe = torch.empty(1 << 30, dtype=torch.float32, device="cuda")  # 4 GiB, never initialised: only read
    result["roofline"]["stream_read_GB/s"] = ra.ra_measure_read_bandwidth(ctx, probe, iters=5)
    del probe
    ra.ra_destroy(ctx)
    if not args.no_cpu_baseline:
        result["cpu_baseline"], parity = cpu_baseline(w, args.lam, sample, gpu)
        if parity is not None:
            result["parity"] = parity
    print(json.dumps(result))


if __name__ == "__main__":
    main()
