"""Seeded random shapes through the whole path on the GPU against the oracle: head grouping, round counts and
lengths around the tile sizes (empty rounds included), several query tokens, current round, paged or
contiguous storage, random selections.  Every case is small enough for the oracle to run in full."""
import numpy as np
import pytest
import torch

import paper_2502_15294_amd as ra
from oracle import pipeline
from oracle import round_attention as ora
from synth import make_workload
from synth.device import Engine, device_view, sel_to_device, to_device

pytestmark = pytest.mark.gpu
OUT_TOL, STREAM_TOL, SCORE_TOL = 2e-3, 5e-5, 1e-5
EDGE_LENS = [0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 255, 256, 257]


def _draw_case(seed, max_rounds=12):
    rng = np.random.default_rng(7000 + seed)
    f32 = seed % 5 == 4                       # every fifth case on the generic fp32 / d = 64 kernels
    B = int(rng.integers(1, 5))
    if f32:
        Hkv, G, d, dtype, base = int(rng.choice([1, 2])), int(rng.choice([1, 2, 4, 8])), 64, "f32", "cfg1"
    else:
        Hkv, G, d, dtype, base = int(rng.choice([1, 2, 8])), int(rng.choice([1, 2, 3, 4, 8, 16])), 128, "bf16", "cfg2"
    prefill = (not f32) and seed % 3 == 0
    q_len = int(rng.choice([2, 3, 5, 9, 17, 40])) if prefill else 1
    cur_len = q_len + int(rng.integers(0, 30)) if (prefill or rng.random() < 0.5) else 0
    lens = []
    for _ in range(B):
        R = int(rng.integers(0, max_rounds + 1))
        lens.append([int(rng.choice(EDGE_LENS)) if rng.random() < 0.5 else int(rng.integers(1, 400)) for _ in range(R)])
    if max(len(l) for l in lens) == 0:
        lens[0] = [33]
    over = dict(B=B, Hq=Hkv * G, Hkv=Hkv, d=d, dtype=dtype, q_len=q_len, cur_len=cur_len, lens=lens,
                block_size=int(rng.choice([0, 16])) if not f32 else 0, n_relevant=2)
    sels = [sorted(rng.choice(len(l), size=int(rng.integers(0, len(l) + 1)), replace=False).tolist()) if l else []
            for l in lens]
    return base, over, sels, prefill


@pytest.mark.parametrize("seed", range(30))
def test_random_shape_whole_path(seed):
    base, over, sels, prefill = _draw_case(seed)
    w = make_workload(base, **over)
    print(f"random case {seed}: {over} sels={sels}", flush=True)
    eng = Engine(w)
    v0 = device_view(w, 0)                     # watershed layer (keys and values: also used fused)
    v1 = device_view(w, 1)
    q0 = to_device(w.q(0), w.dtype)
    ck0 = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    cv0 = to_device(w.cur_v(0), w.dtype) if w.cur_len else None
    ck1 = to_device(w.cur_k(1), w.dtype) if w.cur_len else None
    cv1 = to_device(w.cur_v(1), w.dtype) if w.cur_len else None
    cl = torch.full((w.B,), w.cur_len, dtype=torch.int32, device="cuda") if w.cur_len else None

    # ---- S1 scores, S2 selection --------------------------------------------------------------------------
    P, S = ra.ra_round_scores(eng.ctx, q0, v0, ck0, scale=w.scale)
    sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, S, v0.n_rounds, ra.make_select_params(lam=0.5))
    torch.cuda.synchronize()
    P, S, sel_idx, n_sel = P.cpu().numpy(), S.cpu().numpy(), sel_idx.cpu().numpy(), n_sel.cpu().numpy()
    for b in range(w.B):
        R = w.n_rounds(b)
        rP, rS = pipeline.scores_for_sequence(w, b)
        if R:
            assert np.abs(P[b, :, :R] - rP).max() < SCORE_TOL and np.abs(S[b, :R] - rS).max() < SCORE_TOL, b
        # the oracle's rule on the GPU's own scores: bit-exact
        assert sel_idx[b, :n_sel[b]].tolist() == ora.select_rounds([float(x) for x in S[b, :R]], lam=0.5)[0], b

    # ---- S4 / S5 attention over a random selection -----------------------------------------------------
    si, ns = sel_to_device(sels, v1.R_max)
    if prefill:
        out, lse = ra.ra_round_sparse_attn_prefill(eng.ctx, to_device(w.q(1), w.dtype), v1, si, ns, ck1, cv1,
                                                   scale=w.scale)
    else:
        out, lse = ra.ra_round_sparse_attn_decode(eng.ctx, to_device(w.q(1)[:, 0], w.dtype), v1, si, ns, ck1, cv1, cl,
                                                  scale=w.scale)
    torch.cuda.synchronize()
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for b in range(w.B):
        go, gl = (out[b], lse[b]) if prefill else (out[b][None], lse[b][None])
        n_keys = sum(int(w.lens[b][r]) for r in sels[b]) + w.cur_len
        if n_keys == 0:                       # nothing to attend over: the oracle leaves this undefined
            assert np.all(go == 0) and np.all(np.isneginf(gl)), b
            continue
        ro, rl = pipeline.attention_for_sequence(w, b, 1, sels[b])
        err = ora.row_error(go, ro)
        assert err < OUT_TOL and err < STREAM_TOL, (b, err)
        assert np.allclose(gl, rl, rtol=0, atol=2e-5 * max(1.0, np.abs(rl).max())), b

    # ---- watershed layer with the scores from the attention pass (matrix-core shapes only) -----------------------
    if w.dtype == "bf16":
        if prefill:
            o2, _, P2, S2 = ra.ra_watershed_attn_prefill(eng.ctx, q0, v0, ck0, cv0, scale=w.scale)
        else:
            o2, _, P2, S2 = ra.ra_watershed_attn_decode(eng.ctx, q0[:, 0].contiguous(), v0, ck0, cv0, cl, scale=w.scale)
        torch.cuda.synchronize()
        o2, S2 = o2.cpu().numpy(), S2.cpu().numpy()
        for b in range(w.B):
            R = w.n_rounds(b)
            if R and w.total_tokens(b):
                assert np.abs(S2[b, :R] - S[b, :R]).max() < SCORE_TOL, b
            if w.total_tokens(b) + w.cur_len:
                ro, _ = pipeline.attention_for_sequence(w, b, 0, list(range(R)))
                assert ora.row_error(o2[b] if prefill else o2[b][None], ro) < STREAM_TOL, b
    eng.close()


@pytest.mark.parametrize("seed", range(100, 130))
def test_random_shape_random_softmax_scale_and_bias(seed):
    """The same walk with a softmax scale drawn log-uniformly from [0.02, 0.4], a stronger or absent relevance
    bias on the keys and up to 40 rounds: nothing in the kernels may depend on the scale being 1/sqrt(d)."""
    base, over, sels, prefill = _draw_case(seed, max_rounds=40)
    rng = np.random.default_rng(seed)
    scale = float(np.exp(rng.uniform(np.log(0.02), np.log(0.4))))
    over["alpha"] = float(rng.choice([0.0, 2.0, 6.0]))
    w = make_workload(base, **over)
    print(f"random case {seed}: scale={scale:.4f} {over} sels={sels}", flush=True)
    eng = Engine(w)
    v0, v1 = device_view(w, 0), device_view(w, 1)
    dev = lambda x: to_device(x, w.dtype) if x is not None else None
    ck0, cv0, ck1, cv1 = dev(w.cur_k(0)), dev(w.cur_v(0)), dev(w.cur_k(1)), dev(w.cur_v(1))
    cl = torch.full((w.B,), w.cur_len, dtype=torch.int32, device="cuda") if w.cur_len else None
    P, S = ra.ra_round_scores(eng.ctx, dev(w.q(0)), v0, ck0, scale=scale)
    si, ns = sel_to_device(sels, v1.R_max)
    if prefill:
        out, lse = ra.ra_round_sparse_attn_prefill(eng.ctx, dev(w.q(1)), v1, si, ns, ck1, cv1, scale=scale)
        o2, _, _, S2 = ra.ra_watershed_attn_prefill(eng.ctx, dev(w.q(0)), v0, ck0, cv0, scale=scale)
    else:
        out, lse = ra.ra_round_sparse_attn_decode(eng.ctx, dev(w.q(1)[:, 0]), v1, si, ns, ck1, cv1, cl, scale=scale)
        o2, S2 = None, None
        if w.dtype == "bf16":
            o2, _, _, S2 = ra.ra_watershed_attn_decode(eng.ctx, dev(w.q(0)[:, 0]), v0, ck0, cv0, cl, scale=scale)
    torch.cuda.synchronize()
    P, S, out, lse = P.cpu().numpy(), S.cpu().numpy(), out.cpu().numpy(), lse.cpu().numpy()
    for b in range(w.B):
        R = w.n_rounds(b)
        cur = lambda layer, f: None if w.cur_len == 0 else f(layer)[b]
        k0 = [w.k_round(b, 0, r) for r in range(R)]
        if R:
            rP, rS = ora.round_scores(w.q(0)[b], k0, scale, cur(0, w.cur_k))
            assert np.abs(P[b, :, :R] - rP).max() < SCORE_TOL and np.abs(S[b, :R] - rS).max() < SCORE_TOL, b
            if S2 is not None and w.total_tokens(b):
                assert np.abs(S2[b, :R].cpu().numpy() - rS).max() < SCORE_TOL, b
        go, gl = (out[b], lse[b]) if prefill else (out[b][None], lse[b][None])
        if sum(int(w.lens[b][r]) for r in sels[b]) + w.cur_len == 0:
            assert np.all(go == 0) and np.all(np.isneginf(gl)), b
        else:
            kr = [w.k_round(b, 1, r) if r in sels[b] else None for r in range(R)]
            vr = [w.v_round(b, 1, r) if r in sels[b] else None for r in range(R)]
            ro, rl = ora.sparse_attention(w.q(1)[b], kr, vr, sels[b], scale, cur(1, w.cur_k), cur(1, w.cur_v))
            err = ora.row_error(go, ro)
            assert err < OUT_TOL and err < STREAM_TOL, (b, err)
            assert np.allclose(gl, rl, rtol=0, atol=2e-5 * max(1.0, np.abs(rl).max())), b
        if o2 is not None and w.total_tokens(b) + w.cur_len:
            v0r = [w.v_round(b, 0, r) for r in range(R)]
            ro, _ = ora.sparse_attention(w.q(0)[b], k0, v0r, list(range(R)), scale, cur(0, w.cur_k), cur(0, w.cur_v))
            g2 = o2[b].cpu().numpy()
            assert ora.row_error(g2 if prefill else g2[None], ro) < STREAM_TOL, b
    eng.close()


@pytest.mark.parametrize("seed", range(200, 208))
def test_random_many_sequences_decode(seed):
    """Batches past the size up to which the decode kernel plans a batch by itself (B * R_max > 1024): the planning
    kernel's tables, uneven round counts, short ragged rounds, random selections, per-sequence current lengths."""
    rng = np.random.default_rng(seed)
    _many_sequences_case(rng, seed, B=int(rng.integers(20, 33)), max_R=60, max_len=90)


@pytest.mark.parametrize("B", [65, 257, 1024])
def test_batches_beyond_one_wavefront_of_sequences_decode(B):
    """More sequences than a wavefront has lanes, up to the largest batch the library takes: the decode kernel then
    finds a range's first sequence by bisection of the batch's tile prefix, and most ranges hold several sequences."""
    rng = np.random.default_rng(9000 + B)
    _many_sequences_case(rng, 9000 + B, B=B, max_R={65: 17, 257: 17, 1024: 6}[B], max_len=70)


def _many_sequences_case(rng, seed, B, max_R, max_len, G=None):
    G = int(rng.choice([1, 4, 8])) if G is None else G
    lens = [[int(rng.choice(EDGE_LENS[:11])) if rng.random() < 0.4 else int(rng.integers(1, max_len))
             for _ in range(int(rng.integers(0, max_R + 1)))] for _ in range(B)]
    lens[0] = [int(rng.integers(1, max_len)) for _ in range(max_R)]          # R_max = max_R for certain
    cur_cap = int(rng.choice([0, 24]))
    w = make_workload("cfg2", B=B, Hq=8 * G, Hkv=8, q_len=1, cur_len=cur_cap, lens=lens,
                      block_size=int(rng.choice([0, 16])), n_relevant=2)
    assert w.B * w.R_max > 1024 or w.B > 64
    sels = [sorted(rng.choice(len(l), size=int(rng.integers(0, len(l) + 1)), replace=False).tolist()) if l else []
            for l in lens]
    cur_lens = [int(rng.integers(0, cur_cap + 1)) for _ in range(B)] if cur_cap else [0] * B
    print(f"many-sequence case {seed}: B={B} G={G} cur_cap={cur_cap} block={w.block_size}", flush=True)
    eng = Engine(w)
    v0, v1 = device_view(w, 0, with_v=False), device_view(w, 1)
    P, S = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), v0, scale=w.scale)
    si, ns = sel_to_device(sels, v1.R_max)
    ck = to_device(w.cur_k(1), w.dtype) if cur_cap else None
    cv = to_device(w.cur_v(1), w.dtype) if cur_cap else None
    cl = torch.tensor(cur_lens, dtype=torch.int32, device="cuda") if cur_cap else None
    out, lse = ra.ra_round_sparse_attn_decode(eng.ctx, to_device(w.q(1)[:, 0], w.dtype), v1, si, ns, ck, cv, cl,
                                              scale=w.scale)
    torch.cuda.synchronize()
    S, out, lse = S.cpu().numpy(), out.cpu().numpy(), lse.cpu().numpy()
    # (the generators make a whole batch per call: once, outside the loop over sequences)
    q0_h, q1_h = w.q(0), w.q(1)
    ck_h, cv_h = (w.cur_k(1), w.cur_v(1)) if cur_cap else (None, None)
    for b in range(B):
        R = w.n_rounds(b)
        if R:
            _, rS = ora.round_scores(q0_h[b], [w.k_round(b, 0, r) for r in range(R)], w.scale)
            assert np.abs(S[b, :R] - rS).max() < SCORE_TOL, b
        n_cur = cur_lens[b]
        if sum(int(w.lens[b][r]) for r in sels[b]) + n_cur == 0:
            assert np.all(out[b] == 0) and np.all(np.isneginf(lse[b])), b
            continue
        kr = [w.k_round(b, 1, r) if r in sels[b] else None for r in range(R)]
        vr = [w.v_round(b, 1, r) if r in sels[b] else None for r in range(R)]
        ro, rl = ora.sparse_attention(q1_h[b], kr, vr, sels[b], w.scale,
                                      ck_h[b, :n_cur] if n_cur else None, cv_h[b, :n_cur] if n_cur else None)
        err = ora.row_error(out[b][None], ro)
        assert err < OUT_TOL and err < STREAM_TOL, (b, err)
        assert np.allclose(lse[b][None], rl, rtol=0, atol=2e-5 * max(1.0, np.abs(rl).max())), b
    eng.close()
