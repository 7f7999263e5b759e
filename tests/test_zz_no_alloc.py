"""The decode entry point that allocates nothing (its scratch is an array inside the library's device code)
against the ordinary entry point, through the C ABI: same kernels, so the outputs must be bitwise equal.  Two calls
in a row on the shared array, the second with a smaller batch (the array keeps the first call's contents), then a
call that needs more scratch than the array has."""
import pytest
import torch

import paper_2502_15294_amd as ra
from synth import make_workload
from synth.device import Engine, device_view, sel_to_device, to_device

pytestmark = pytest.mark.gpu


def _both(w, sels, with_cur):
    eng = Engine(w)
    view = device_view(w, 1)
    q = to_device(w.q(1)[:, 0], w.dtype)
    sel_idx, n_sel = sel_to_device(sels, w.R_max)
    ck = to_device(w.cur_k(1), w.dtype) if with_cur else None
    cv = to_device(w.cur_v(1), w.dtype) if with_cur else None
    cl = torch.full((w.B,), w.cur_len, dtype=torch.int32, device="cuda") if with_cur else None
    out_ws, lse_ws = ra.ra_round_sparse_attn_decode(eng.ctx, q, view, sel_idx, n_sel, ck, cv, cl, scale=w.scale)
    ra.ra_set_workspace(eng.ctx, None)                     # the new call must not need the workspace
    out = torch.full_like(out_ws, float("nan"))
    lse = torch.full_like(lse_ws, float("nan"))
    ra.ra_round_sparse_attn_decode_noalloc(eng.ctx, q, view, out, lse, sel_idx, n_sel, ck, cv, cl, scale=w.scale)
    torch.cuda.synchronize()
    assert torch.equal(out, out_ws) and torch.equal(lse, lse_ws)
    assert torch.isfinite(out).all()
    eng.close()


def test_no_alloc_decode_equals_the_workspace_call_twice_in_a_row_second_call_smaller():
    # first call: the Llama-3-8B-shaped decode batch (every sequence is cut into several ranges: records are used)
    w = make_workload("cfg2")
    sels = [sorted({(3 * b + j * 5) % w.n_rounds(b) for j in range(4)}) for b in range(w.B)]
    _both(w, sels, with_cur=False)
    # second call, smaller: two sequences, five short rounds, a current round of 20 tokens
    w2 = make_workload("cfg2", B=2, R=5, cur_len=20, length=("uniform", 10, 150))
    _both(w2, [[0, 3], [1, 2, 4]], with_cur=True)
    # and the fp32 / head_dim 64 path (generic kernel, per-split pieces in the same array)
    w3 = make_workload("cfg1")
    _both(w3, [[1, 4, 6]], with_cur=False)


def test_no_alloc_decode_rejects_a_call_that_needs_more_than_the_built_in_scratch():
    # 1024 sequences x 8 KV heads leave more partial results than 32 MiB hold; nothing is launched
    B = 1024
    k = torch.zeros((B * 16 * 8 * 128,), dtype=torch.bfloat16, device="cuda")
    view = ra.KVView(k, k, torch.arange(B, dtype=torch.int64, device="cuda").reshape(B, 1) * 16,
                     torch.full((B, 1), 16, dtype=torch.int32, device="cuda"),
                     torch.ones((B,), dtype=torch.int32, device="cuda"), 8, 128, 16)
    ctx = ra.ra_create(0)
    q = torch.zeros((B, 32, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.full((B, 32, 128), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(ra.RaError) as e:
        ra.ra_round_sparse_attn_decode_noalloc(ctx, q, view, out, None, scale=0.1)
    assert e.value.code == ra.RA_ERR_WORKSPACE and "built-in scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (out == 7.0).all()
    ra.ra_destroy(ctx)
