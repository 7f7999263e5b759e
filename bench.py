#!/usr/bin/env python3
"""Benchmark of the Round Attention hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch, all inputs resident in HBM:
round scores at the watershed layer -> round selection -> round-sparse decode attention of one
post-watershed layer (for the prefill workload: the prefill attention instead of decode).  Prints ONE
JSON line with the whole-job throughput, the roofline figure of the dominant kernel group measured
live with events on the launch stream, and the fp64 CPU oracle timed on the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg1|cfg5|cfg3] [--no-cpu-baseline]
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
CACHE_DEFEAT_BYTES = 512 << 20  # bytes touched between two uses of the same buffer (Infinity Cache is 256 MB)

WORKLOADS = {
    "cfg1": ("cfg1", {}, "tiny fp32: B=1, 4/2 heads, d=64, 8 rounds x 64 tokens, decode"),
    "cfg2": ("cfg2", {}, "Llama-3-8B-shaped layer, bf16, B=8 decode, 32/8 heads, d=128, 20 rounds of U[200,1000] tokens"),
    "cfg5": ("cfg5", {}, "70B-shaped layer slice, bf16, B=64 decode, 64/8 heads, d=128, 50 rounds of U[300,1000] tokens, 16-token paged blocks"),
    "cfg3": ("cfg3", {}, "question prefill, bf16, B=4, q_len=128, 32/8 heads, d=128, 60 lognormal rounds totalling 32K tokens"),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=sorted(WORKLOADS))
    ap.add_argument("--lam", type=float, default=1.0, help="multiplier of the adaptive selection rule")
    ap.add_argument("--alpha", type=float, default=None, help="override the key bias strength of the workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--replicas", type=int, default=0, help="input replicas rotated through (0 = enough to defeat the Infinity Cache)")
    ap.add_argument("--cpu-baseline-seqs", type=int, default=0, help="sequences the oracle is timed on (0 = auto)")
    return ap.parse_args()


def cpu_baseline(w, lam: float, n_seqs: int):
    """Time the fp64 oracle (as it stands) on the host cores for the same step on a bounded sample of
    the batch.  Input generation is excluded: only the oracle's arithmetic is timed."""
    from oracle import round_attention as ora
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    n_seqs = max(1, min(n_seqs, w.B))
    data = []
    for b in range(n_seqs):
        R = w.n_rounds(b)
        data.append(dict(q0=w.q(0)[b], q1=w.q(1)[b], k0=[w.k_round(b, 0, r) for r in range(R)],
                         k1=[w.k_round(b, 1, r) for r in range(R)], v1=[w.v_round(b, 1, r) for r in range(R)],
                         ck0=None if w.cur_len == 0 else w.cur_k(0)[b], ck1=None if w.cur_len == 0 else w.cur_k(1)[b],
                         cv1=None if w.cur_len == 0 else w.cur_v(1)[b]))
    t0 = time.perf_counter()
    for d in data:
        _, S = ora.round_scores(d["q0"], d["k0"], w.scale, d["ck0"])
        sel, _ = ora.select_rounds(S, lam=lam)
        ora.sparse_attention(d["q1"], d["k1"], d["v1"], sel, w.scale, d["ck1"], d["cv1"])
    dt = time.perf_counter() - t0
    tokens = n_seqs * w.q_len
    return {"value": tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n_seqs} of {w.B} sequences of the same workload, whole step (scores, selection, sparse "
                      f"attention) in fp64 numpy, {dt:.2f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 (nothing here uses a second GPU)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2502_15294_amd as ra
    from synth import make_workload
    from synth.device import Engine, device_view, to_device

    ra.lib()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    cfg, over, desc = WORKLOADS[args.workload]
    over = dict(over)
    if args.alpha is not None:
        over["alpha"] = args.alpha
    w = make_workload(cfg, **over)
    prefill = w.q_len > 1
    eb = 2 if w.dtype == "bf16" else 4

    # ---- inputs resident in HBM, in enough replicas that a buffer is cold again when it is reused --------
    eng = Engine(w)
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

    params = ra.make_select_params(lam=args.lam)
    P = torch.empty((w.B, w.Hq, view0.R_max), dtype=torch.float32, device="cuda")
    S = torch.empty((w.B, view0.R_max), dtype=torch.float32, device="cuda")
    sel_idx = torch.empty((w.B, view0.R_max), dtype=torch.int32, device="cuda")
    n_sel = torch.empty((w.B,), dtype=torch.int32, device="cuda")
    out = torch.empty((w.B, w.q_len, w.Hq, w.d) if prefill else (w.B, w.Hq, w.d), dtype=torch.float32, device="cuda")
    lse = torch.empty((w.B, w.q_len, w.Hq) if prefill else (w.B, w.Hq), dtype=torch.float32, device="cuda")

    def step(v0, v1):
        ra.ra_round_scores(eng.ctx, q0, v0, ck0, scale=w.scale, scores_head=P, scores=S)
        ra.ra_select_rounds(eng.ctx, S, v0.n_rounds, params, sel_idx=sel_idx, n_sel=n_sel)
        if prefill:
            ra.ra_round_sparse_attn_prefill(eng.ctx, q1, v1, sel_idx, n_sel, ck1, cv1, scale=w.scale, out=out, lse=lse)
        else:
            ra.ra_round_sparse_attn_decode(eng.ctx, q1, v1, sel_idx, n_sel, ck1, cv1, cl1, scale=w.scale, out=out,
                                           lse=lse)

    step(view0, view1)
    torch.cuda.synchronize()
    n_sel_h = n_sel.cpu().numpy()
    sel_h = sel_idx.cpu().numpy()
    sel_tokens = int(sum(int(w.lens[b][sel_h[b, :n_sel_h[b]]].sum()) for b in range(w.B)))
    step_bytes = hist_tokens * k_bytes_tok + sel_tokens * 2 * k_bytes_tok
    n_rep = args.replicas or int(max(1, min(8, -(-CACHE_DEFEAT_BYTES // max(step_bytes, 1)))))

    def clone_view(v):
        k, vv, seg_off, seg_len, n_rounds, bt, seg_off_v = v.tensors
        return ra.KVView(k.clone(), None if vv is None else vv.clone(), seg_off, seg_len, n_rounds, v.Hkv, v.d,
                         v.c.max_tokens, block_table=bt, block_size=v.c.block_size, seg_off_v=seg_off_v)

    reps = [(view0, view1)] + [(clone_view(view0), clone_view(view1)) for _ in range(n_rep - 1)]

    # ---- timed region -----------------------------------------------------------------------------------
    for i in range(args.warmup):
        step(*reps[i % n_rep])
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        v0, v1 = reps[i % n_rep]
        e = ev[i]
        e[0].record()
        ra.ra_round_scores(eng.ctx, q0, v0, ck0, scale=w.scale, scores_head=P, scores=S)
        e[1].record()
        ra.ra_select_rounds(eng.ctx, S, v0.n_rounds, params, sel_idx=sel_idx, n_sel=n_sel)
        e[2].record()
        if prefill:
            ra.ra_round_sparse_attn_prefill(eng.ctx, q1, v1, sel_idx, n_sel, ck1, cv1, scale=w.scale, out=out, lse=lse)
        else:
            ra.ra_round_sparse_attn_decode(eng.ctx, q1, v1, sel_idx, n_sel, ck1, cv1, cl1, scale=w.scale, out=out,
                                           lse=lse)
        e[3].record()
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    ms = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in ev])  # [steps, 3] milliseconds
    avg_ms = ms.mean(axis=0)
    med_ms = np.median(ms, axis=0)

    # ---- algorithmic work of each kernel group per launch ----------------------------------------------------
    q_rows = w.B * w.q_len * w.Hq
    scores_bytes = hist_tokens * k_bytes_tok + q_rows * w.d * eb
    attn_bytes = (sel_tokens + w.B * w.cur_len) * 2 * k_bytes_tok + q_rows * w.d * (eb + 4)
    groups = {
        "ra_round_scores": {"ms": float(avg_ms[0]), "median_ms": float(med_ms[0]), "bytes": int(scores_bytes)},
        "ra_select_rounds": {"ms": float(avg_ms[1]), "median_ms": float(med_ms[1]), "bytes": int(w.B * view0.R_max * 8)},
        ("ra_round_sparse_attn_prefill" if prefill else "ra_round_sparse_attn_decode"):
            {"ms": float(avg_ms[2]), "median_ms": float(med_ms[2]), "bytes": int(attn_bytes)},
    }
    for g in groups.values():
        g["GB/s"] = g["bytes"] / (g["ms"] * 1e-3) / 1e9 if g["ms"] > 0 else None
    dom = max(groups, key=lambda k: groups[k]["ms"])
    if prefill and dom != "ra_select_rounds":
        # prefill contractions: QK^T for the scores pass, QK^T + PV for attention
        flops = (2 if dom == "ra_round_scores" else 4) * q_rows * w.d * \
                ((hist_tokens if dom == "ra_round_scores" else sel_tokens) / w.B + w.cur_len / 2)
        ach = flops / (groups[dom]["ms"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
    else:
        ach = groups[dom]["GB/s"]
        roofline = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ach / HBM_PEAK_GBS, "traffic": None}

    result = {
        "metric": "round-sparse decode attn tokens/s + achieved HBM GB/s (% of peak), 1 GPU",
        "value": w.B * w.q_len * args.steps / total,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": total / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "d": w.d,
                   "q_len": w.q_len, "history_tokens": hist_tokens, "selected_tokens": sel_tokens,
                   "kept_token_fraction": sel_tokens / max(hist_tokens, 1),
                   "selected_rounds": [int(x) for x in n_sel_h], "lambda": args.lam, "alpha": w.alpha,
                   "replicas_rotated": n_rep, "step": "ra_round_scores -> ra_select_rounds -> " +
                   ("ra_round_sparse_attn_prefill" if prefill else "ra_round_sparse_attn_decode")},
        "roofline": roofline,
        "kernel_groups": groups,
        "input_generation_s": t_gen,
    }
    if not args.no_cpu_baseline:
        n = args.cpu_baseline_seqs or (w.B if args.workload in ("cfg1", "cfg2") else 2)
        result["cpu_baseline"] = cpu_baseline(w, args.lam, n)
    eng.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
