"""Run every kernel family on small fixed workloads and print one JSON object of output hashes.

Helper of test_gpu_schedule_independence.py, run as a script in a process of its own so that the library named by
RA_LIBRARY is the one loaded.  Every entry is the hash of a call that follows unrelated kernels, of the call right
after it and of one more after unrelated kernels again; the three must agree (an entry that does not is reported
as a list), and the test compares the entries across builds."""
import hashlib
import json
import os
import sys

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import paper_2502_15294_amd as ra  # noqa: E402
from synth import make_workload  # noqa: E402
from synth.device import Engine, device_view, to_device  # noqa: E402

DECODE = [("cfg1", {}), ("cfg2", {}), ("cfg5", dict(B=4)),
          ("cfg4", dict(B=2, n_post_layers=1, length=("lognormal", 400.0, 0.8, 16384)))]
PREFILL = {
    "q40_cur64": dict(B=2, R=6, q_len=40, cur_len=64, length=("uniform", 20, 600)),
    "q128_paged": dict(B=2, R=5, q_len=128, cur_len=128, block_size=16, length=("uniform", 100, 900)),
    "q17_ragged": dict(B=3, R=7, q_len=17, cur_len=33, length=("uniform", 1, 70)),
}
WATERSHED_DECODE = [("cfg2", dict(B=3, R=7, cur_len=37, length=("uniform", 1, 260))),
                    ("cfg5", dict(B=2, R=6, length=("uniform", 1, 1000)))]


def other_kernels():
    x = torch.zeros(1 << 16, device="cuda")
    for _ in range(100):
        x = x * 1.5 + 1.0
    y = torch.randn(1 << 24, device="cuda")
    float((y * 2).sum().item())


def digest(tensors):
    torch.cuda.synchronize()
    h = hashlib.sha1()
    for t in tensors:
        h.update(np.ascontiguousarray(t.cpu().numpy()).tobytes())
    return h.hexdigest()[:16]


def main():
    res = {}

    def record(tag, fn):
        other_kernels()
        a = digest(fn())
        b = digest(fn())
        other_kernels()
        c = digest(fn())
        res[tag] = a if a == b == c else [a, b, c]

    for cfg, over in DECODE:
        w = make_workload(cfg, **over)
        eng = Engine(w)
        v0, v1 = device_view(w, 0, with_v=False), device_view(w, 1)
        q0, q1 = to_device(w.q(0), w.dtype), to_device(w.q(1)[:, 0], w.dtype)
        ck0 = to_device(w.cur_k(0), w.dtype) if w.cur_len else None

        def step():
            P, S = ra.ra_round_scores(eng.ctx, q0, v0, ck0, scale=w.scale)
            sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, S, v0.n_rounds)
            out, lse = ra.ra_round_sparse_attn_decode(eng.ctx, q1, v1, sel_idx, n_sel, scale=w.scale)
            return P, S, sel_idx, n_sel, out, lse

        record("decode step " + cfg, step)
        eng.close()
    for name, kw in PREFILL.items():
        w = make_workload("cfg3", **kw)
        eng = Engine(w)
        view = device_view(w, 0)
        q = to_device(w.q(0), w.dtype)
        ck, cv = to_device(w.cur_k(0), w.dtype), to_device(w.cur_v(0), w.dtype)
        for mode, tag in ((ra.RA_PREFILL_P_BF16X2, "bf16x2"), (ra.RA_PREFILL_P_F16, "f16")):
            ra.ra_set_prefill_precision(eng.ctx, mode)

            def calls():
                o1, l1, P, S = ra.ra_watershed_attn_prefill(eng.ctx, q, view, ck, cv, scale=w.scale)
                o2, l2 = ra.ra_round_sparse_attn_prefill(eng.ctx, q, view, None, None, ck, cv, scale=w.scale)
                P2, S2 = ra.ra_round_scores(eng.ctx, q, view, ck, scale=w.scale)
                return o1, l1, P, S, o2, l2, P2, S2

            record(f"prefill {name} {tag}", calls)
        eng.close()
    for cfg, over in WATERSHED_DECODE:
        w = make_workload(cfg, **over)
        eng = Engine(w)
        view = device_view(w, 0)
        q = to_device(w.q(0)[:, 0], w.dtype)
        ck = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
        cv = to_device(w.cur_v(0), w.dtype) if w.cur_len else None
        cl = torch.full((w.B,), w.cur_len, dtype=torch.int32, device="cuda") if w.cur_len else None
        record("watershed decode " + cfg, lambda: ra.ra_watershed_attn_decode(eng.ctx, q, view, ck, cv, cl, scale=w.scale))
        eng.close()
    print("HASHES " + json.dumps(res))


if __name__ == "__main__":
    main()
