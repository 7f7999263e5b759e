"""GPU parity: the HIP library, called through its C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Bars: selected indices bit-exact; attention outputs within 2e-3 (max over rows of
max|err| / max|ref|), and, for the fp32-accumulating streaming kernels, within the much tighter
bound their arithmetic implies; round scores within 1e-5 absolute."""
import numpy as np
import pytest
import torch

import paper_2502_15294_amd as ra
from oracle import pipeline
from oracle import round_attention as ora
from synth import make_workload
from select_edge_cases import select_edge_cases
from synth.device import Engine, device_view, sel_to_device, to_device

pytestmark = pytest.mark.gpu

OUT_TOL = 2e-3        # the contract
STREAM_TOL = 5e-5     # fp32 accumulation of exact bf16 products over <= 2^17 terms, exp2 to ~2 ulp
SCORE_TOL = 1e-5


def _say(msg):
    print(msg, flush=True)


def _oracle_attention(w, layer, sels):
    outs, lses = [], []
    for b in range(w.B):
        o, l = pipeline.attention_for_sequence(w, b, layer, sels[b])
        outs.append(o)
        lses.append(l)
    return np.stack(outs), np.stack(lses)


def _gpu_decode(eng, w, layer, sels, view=None, cur_len_dev=None, use_sel=True):
    view = view or device_view(w, layer)
    q = to_device(w.q(layer)[:, 0], w.dtype)
    sel_idx, n_sel = sel_to_device(sels, view.R_max) if use_sel else (None, None)
    ck = cv = cl = None
    if w.cur_len:
        ck, cv = to_device(w.cur_k(layer), w.dtype), to_device(w.cur_v(layer), w.dtype)
        cl = cur_len_dev if cur_len_dev is not None else torch.full((w.B,), w.cur_len, dtype=torch.int32, device="cuda")
    out, lse = ra.ra_round_sparse_attn_decode(eng.ctx, q, view, sel_idx, n_sel, ck, cv, cl, scale=w.scale)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


DECODE_CASES = {
    # name: (config, overrides, selections or None for "all rounds")
    "f32_d64_g2_tiny": ("cfg1", dict(), [[1, 3]]),
    "f32_d64_g2_all": ("cfg1", dict(), None),
    "bf16_g4_ragged": ("cfg2", dict(B=3, R=7, lens=[[5, 16, 17, 0, 33, 1, 250], [64, 3, 0, 0, 15, 48, 31],
                                                   [700, 1, 1, 1, 1, 1, 1]]),
                       [[0, 2, 4, 6], [1, 4], [0, 3, 6]]),
    "bf16_g4_cur": ("cfg2", dict(B=2, R=4, cur_len=37, lens=[[40, 9, 130, 77], [3, 300, 20, 5]]), [[2], [0, 1, 3]]),
    "bf16_g4_cur_only": ("cfg2", dict(B=2, R=3, cur_len=21, lens=[[40, 9, 13], [3, 30, 20]]), [[], []]),
    "bf16_g8_paged": ("cfg5", dict(B=3, R=6, lens=[[300, 17, 16, 1, 999, 50], [31, 32, 33, 0, 64, 5],
                                                  [450, 450, 450, 450, 450, 450]]),
                      [[0, 1, 4], [0, 1, 2, 3, 4, 5], [1, 5]]),
    "bf16_g8_contig": ("cfg5", dict(B=2, R=5, block_size=0, length=("uniform", 30, 400)), [[0, 4], [1, 2, 3]]),
    "bf16_g1_mha": ("cfg2", dict(B=2, R=5, Hq=8, Hkv=8, length=("uniform", 10, 200)), [[0, 1, 4], [2]]),
    "bf16_g2": ("cfg2", dict(B=2, R=5, Hq=16, Hkv=8, length=("uniform", 10, 200)), [[3], [0, 2, 4]]),
    "bf16_g3": ("cfg2", dict(B=2, R=5, Hq=24, Hkv=8, length=("uniform", 10, 200)), [[0, 3], [1, 2, 4]]),
    "bf16_g16_cur": ("cfg2", dict(B=2, R=4, Hq=32, Hkv=2, cur_len=19, length=("uniform", 10, 200)), [[0, 3], [1]]),
    "bf16_d64": ("cfg2", dict(B=2, R=5, d=64, length=("uniform", 10, 200)), [[0, 3], [1, 2, 4]]),
    "f32_d128_g4": ("cfg2", dict(B=2, R=4, dtype="f32", length=("uniform", 10, 120)), [[0, 3], [1, 2]]),
    "bf16_g4_many_rounds": ("cfg4", dict(B=2, R=200, length=("lognormal", 40.0, 0.8, 9000), n_post_layers=1),
                            [list(range(0, 200, 7)), list(range(3, 200, 11))]),
}


@pytest.mark.parametrize("name", list(DECODE_CASES))
def test_decode_matches_oracle(name):
    cfg, over, sels = DECODE_CASES[name]
    w = make_workload(cfg, **over)
    if sels is None:
        sels = [list(range(w.n_rounds(b))) for b in range(w.B)]
    _say(f"decode case {name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} d={w.d} dtype={w.dtype} block={w.block_size}")
    eng = Engine(w)
    ref_o, ref_l = _oracle_attention(w, 1, sels)
    out, lse = _gpu_decode(eng, w, 1, sels)
    err = ora.row_error(out, ref_o[:, 0])
    _say(f"  row error {err:.3e}, lse error {np.abs(lse - ref_l[:, 0]).max():.3e}")
    assert err < OUT_TOL and err < STREAM_TOL
    assert np.allclose(lse, ref_l[:, 0], rtol=0, atol=2e-5 * max(1.0, np.abs(ref_l).max()))
    eng.close()


def test_decode_identity_selection_equals_explicit_all_and_is_deterministic():
    w = make_workload("cfg2", B=2, R=6, length=("uniform", 20, 300))
    eng = Engine(w)
    view = device_view(w, 1)
    all_sel = [list(range(6)), list(range(6))]
    a, la = _gpu_decode(eng, w, 1, all_sel, view=view)
    b, lb = _gpu_decode(eng, w, 1, all_sel, view=view, use_sel=False)
    c, lc = _gpu_decode(eng, w, 1, all_sel, view=view)
    assert np.array_equal(a, b) and np.array_equal(la, lb)
    assert np.array_equal(a, c) and np.array_equal(la, lc)
    # order of the selected list does not matter for the result beyond rounding
    d, _ = _gpu_decode(eng, w, 1, [[5, 3, 4, 0, 2, 1], [1, 0, 3, 2, 5, 4]], view=view)
    assert ora.row_error(d, a) < STREAM_TOL
    eng.close()


def test_decode_per_sequence_cur_len_and_empty_key_set():
    w = make_workload("cfg2", B=3, R=3, cur_len=40, lens=[[20, 30, 40]] * 3)
    eng = Engine(w)
    cur_len = torch.tensor([40, 7, 0], dtype=torch.int32, device="cuda")
    sels = [[1], [0, 2], []]
    out, lse = _gpu_decode(eng, w, 1, sels, cur_len_dev=cur_len)
    for b, n_cur in enumerate([40, 7, 0]):
        if b == 2:
            assert np.all(out[b] == 0) and np.all(np.isneginf(lse[b]))      # empty key set: zeros, lse = -inf
            continue
        q = w.q(1)[b]
        ks = [w.k_round(b, 1, r) for r in range(3)]
        vs = [w.v_round(b, 1, r) for r in range(3)]
        ro, rl = ora.sparse_attention(q, ks, vs, sels[b], w.scale, w.cur_k(1)[b, :n_cur], w.cur_v(1)[b, :n_cur])
        assert ora.row_error(out[b], ro[0]) < STREAM_TOL
    eng.close()


SCORE_CASES = {
    "f32_cfg1": ("cfg1", dict()),
    "bf16_g4_ragged": ("cfg2", dict(B=3, R=7, lens=[[5, 16, 17, 0, 33, 1, 250], [64, 3, 0, 0, 15, 48, 31],
                                                   [700, 1, 1, 1, 1, 1, 1]])),
    "bf16_g8_paged": ("cfg5", dict(B=2, R=6, lens=[[300, 17, 16, 1, 999, 50], [31, 32, 33, 0, 64, 5]])),
    "bf16_uneven_round_counts": ("cfg2", dict(B=3, lens=[[30, 40], [10, 20, 30, 40, 50], []])),
    "bf16_qlen3_cur": ("cfg2", dict(B=2, R=5, q_len=3, cur_len=9, length=("uniform", 10, 150))),
    "bf16_qlen4_nocur": ("cfg2", dict(B=2, R=5, q_len=4, cur_len=0, length=("uniform", 10, 150))),
    "bf16_qlen1_cur_cancels": ("cfg2", dict(B=2, R=5, q_len=1, cur_len=6, length=("uniform", 10, 150))),
    # one query token, 64 heads x more than 256 partial values each: finished head by head, then averaged
    "bf16_g8_many_chunks": ("cfg5", dict(B=2, R=300, block_size=0, length=("uniform", 1, 40))),
    "bf16_g8_many_chunks_paged": ("cfg5", dict(B=3, R=270, length=("uniform", 1, 40))),
    # on either side of the number of rounds up to which a workgroup finds its round from scalar loads alone
    "bf16_32_rounds_cur": ("cfg2", dict(B=2, R=32, q_len=2, cur_len=300, length=("uniform", 0, 600))),
    "bf16_33_rounds_cur": ("cfg2", dict(B=2, R=33, q_len=2, cur_len=300, length=("uniform", 0, 600))),
    "bf16_32_rounds_paged": ("cfg5", dict(B=2, R=32, length=("uniform", 0, 600))),
    "bf16_1_round": ("cfg2", dict(B=2, R=1, length=("uniform", 500, 600))),
}


@pytest.mark.parametrize("name", list(SCORE_CASES))
def test_round_scores_match_oracle(name):
    cfg, over = SCORE_CASES[name]
    w = make_workload(cfg, **over)
    _say(f"scores case {name}: B={w.B} R_max={w.R_max} q_len={w.q_len} cur_len={w.cur_len}")
    eng = Engine(w)
    view = device_view(w, 0, with_v=False)
    q = to_device(w.q(0), w.dtype)
    ck = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    P, S = ra.ra_round_scores(eng.ctx, q, view, ck, scale=w.scale)
    torch.cuda.synchronize()
    P, S = P.cpu().numpy(), S.cpu().numpy()
    for b in range(w.B):
        rP, rS = pipeline.scores_for_sequence(w, b)
        R = w.n_rounds(b)
        if R:
            assert np.abs(P[b, :, :R] - rP).max() < SCORE_TOL and np.abs(S[b, :R] - rS).max() < SCORE_TOL
        assert np.all(P[b, :, R:] == 0) and np.all(S[b, R:] == 0)
        if R and w.total_tokens(b):
            assert np.abs(P[b].sum(axis=1) - 1).max() < SCORE_TOL       # per-head scores sum to one
    eng.close()


def _oracle_select_on(S_row, R, params):
    return ora.select_rounds([float(x) for x in S_row[:R]], **params)[0]


@pytest.mark.parametrize("cfg,over", [("cfg2", dict(B=1)), ("cfg5", dict(B=1, block_size=0)),
                                      ("cfg1", dict(B=1, Hq=4, Hkv=2)), ("cfg1", dict(B=1, Hq=8, Hkv=1))])
@pytest.mark.parametrize("scale", [0.03, 0.05, 0.0884, 0.1, 0.125, 0.2, 0.31])
def test_round_scores_with_lanes_that_see_no_token_at_any_scale(cfg, over, scale):
    """Rounds of 1, 2, 17 or 33 tokens leave lane groups of the streaming kernels without a single token in the
    first tile they process; their running maximum then stays at its finite stand-in and the rescaling factor must
    come out as exactly one whatever the softmax scale is (a fused multiply-add of the stand-in once left its
    rounding residue in the exponent, for some scales only)."""
    w = make_workload(cfg, lens=[[1, 64, 2, 17, 33, 3, 16, 145]], **over)
    eng = Engine(w)
    view = device_view(w, 0, with_v=False)
    P, S = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), view, scale=scale)
    torch.cuda.synchronize()
    ks = [w.k_round(0, 0, r) for r in range(w.n_rounds(0))]
    rP, rS = ora.round_scores(w.q(0)[0], ks, scale)
    assert np.abs(P[0].cpu().numpy() - rP).max() < SCORE_TOL and np.abs(S[0].cpu().numpy() - rS).max() < SCORE_TOL
    eng.close()


SELECT_PARAMS = [
    dict(strategy=ora.ADAPTIVE),
    dict(strategy=ora.ADAPTIVE, lam=0.0),
    dict(strategy=ora.ADAPTIVE, lam=0.5, ddof=1),
    dict(strategy=ora.ADAPTIVE, lam=3.0, min_rounds=2),
    dict(strategy=ora.ADAPTIVE, lam=-1.0, max_rounds=5),
    dict(strategy=ora.TOP_FRACTION),
    dict(strategy=ora.TOP_FRACTION, fraction=0.33),
    dict(strategy=ora.THRESHOLD),
    dict(strategy=ora.THRESHOLD, threshold=0.02, min_rounds=0),
    dict(strategy=ora.ADAPTIVE, keep_first=1, keep_last=2),
    dict(strategy=ora.ADAPTIVE, lam=2.0, max_rounds=3, keep_last=70),
    dict(strategy=ora.TOP_FRACTION, fraction=0.05, keep_first=300),
]


@pytest.mark.parametrize("pi", range(len(SELECT_PARAMS)))
def test_select_function_parity_is_bit_exact(pi):
    params = SELECT_PARAMS[pi]
    rng = np.random.default_rng(100 + pi)
    B, R_max = 12, 300
    n_rounds = np.array([300, 1, 2, 0, 64, 65, 256, 257, 10, 20, 200, 299], dtype=np.int32)
    S = np.zeros((B, R_max), dtype=np.float32)
    for b in range(B):
        R = n_rounds[b]
        if R == 0:
            continue
        x = rng.random(R) ** (1 + b)
        if b % 3 == 0:
            x = np.round(x, 2)              # exact ties
        if b == 4:
            x[:] = 1.0                      # uniform
        S[b, :R] = (x / max(x.sum(), 1e-30)).astype(np.float32)
    w = make_workload("cfg1")
    eng = Engine(w)
    p = ra.make_select_params(strategy=params["strategy"], lam=params.get("lam", 1.0),
                              fraction=params.get("fraction", 0.10), threshold=params.get("threshold", 0.10),
                              ddof=params.get("ddof", 0), min_rounds=params.get("min_rounds", 1),
                              max_rounds=params.get("max_rounds", 0), keep_first=params.get("keep_first", 0),
                              keep_last=params.get("keep_last", 0))
    sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, torch.from_numpy(S).cuda(), torch.from_numpy(n_rounds).cuda(), p)
    torch.cuda.synchronize()
    sel_idx, n_sel = sel_idx.cpu().numpy(), n_sel.cpu().numpy()
    for b in range(B):
        expect = _oracle_select_on(S[b], n_rounds[b], params)
        got = sel_idx[b, :n_sel[b]].tolist()
        assert got == expect, (b, params)
        assert np.all(sel_idx[b, n_sel[b]:] == -1)
    eng.close()


def test_select_scores_at_and_one_ulp_around_the_cut():
    """Scores placed exactly on the THRESHOLD and ADAPTIVE cuts, and one fp32 ulp above and below them: the
    inequality is strict, the cut is formed in double from the fp32 scores, and the kernel must take every one of
    these decisions as the oracle does (hand-derived expectations for the cases that have one)."""
    cases = select_edge_cases()
    R_max = 16
    ctx = ra.ra_create(0)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    ra.ra_set_workspace(ctx, ws)
    for scores, params, expected in cases:
        S = np.zeros((1, R_max), dtype=np.float32)
        S[0, :len(scores)] = np.asarray(scores, dtype=np.float32)
        n_rounds = np.array([len(scores)], dtype=np.int32)
        p = ra.make_select_params(strategy=params["strategy"], lam=params.get("lam", 1.0),
                                  threshold=params.get("threshold", 0.10), min_rounds=params.get("min_rounds", 1))
        sel_idx, n_sel = ra.ra_select_rounds(ctx, torch.from_numpy(S).cuda(), torch.from_numpy(n_rounds).cuda(), p)
        torch.cuda.synchronize()
        got = sel_idx.cpu().numpy()[0, :int(n_sel.cpu()[0])].tolist()
        want = _oracle_select_on(S[0], len(scores), params)
        assert got == want, (scores, params, got, want)
        if expected is not None:
            assert want == expected, ("the oracle itself disagrees with the hand-derived selection", scores, params, want)
    ra.ra_destroy(ctx)


SCORES_SELECT_CASES = {
    "fp32_generic": ("cfg1", {}),
    "bf16_decode": ("cfg2", {}),
    "bf16_decode_64_heads_paged": ("cfg5", dict(B=3)),
    "question_8_tokens": ("cfg3", dict(B=2, R=9, q_len=8, cur_len=8, length=("uniform", 20, 300))),
    "rounds_above_256": ("cfg2", dict(B=2, R=300, length=("uniform", 1, 40))),
}


@pytest.mark.parametrize("name", list(SCORES_SELECT_CASES))
def test_scores_and_selection_in_one_call_equal_the_two_calls_bitwise(name):
    cfg, over = SCORES_SELECT_CASES[name]
    w = make_workload(cfg, **over)
    eng = Engine(w)
    view = device_view(w, 0, with_v=False)
    q0 = to_device(w.q(0), w.dtype)
    ck0 = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    for params in SELECT_PARAMS[:9]:
        p = ra.make_select_params(strategy=params["strategy"], lam=params.get("lam", 1.0),
                                  fraction=params.get("fraction", 0.10), threshold=params.get("threshold", 0.10),
                                  ddof=params.get("ddof", 0), min_rounds=params.get("min_rounds", 1),
                                  max_rounds=params.get("max_rounds", 0))
        P1, S1 = ra.ra_round_scores(eng.ctx, q0, view, ck0, scale=w.scale)
        sel1, n1 = ra.ra_select_rounds(eng.ctx, S1, view.n_rounds, p)
        P2, S2, sel2, n2 = ra.ra_round_scores_select(eng.ctx, q0, view, p, ck0, scale=w.scale)
        torch.cuda.synchronize()
        assert torch.equal(P1, P2) and torch.equal(S1, S2) and torch.equal(sel1, sel2) and torch.equal(n1, n2), params
        S, sel, n = S2.cpu().numpy(), sel2.cpu().numpy(), n2.cpu().numpy()
        for b in range(w.B):   # and the oracle's rule on these scores
            assert sel[b, :n[b]].tolist() == _oracle_select_on(S[b], w.n_rounds(b), params), (b, params)
    eng.close()


def _run_gpu_pipeline(eng, w, select_params=None, block_size=None):
    wview = device_view(w, 0, with_v=False, block_size=block_size)
    q0 = to_device(w.q(0), w.dtype)
    ck0 = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    P, S = ra.ra_round_scores(eng.ctx, q0, wview, ck0, scale=w.scale)
    sp = select_params or {}
    p = ra.make_select_params(strategy=sp.get("strategy", 0), lam=sp.get("lam", 1.0))
    sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, S, wview.n_rounds, p)
    lview = device_view(w, 1, block_size=block_size)
    q1 = to_device(w.q(1)[:, 0], w.dtype)
    out, lse = ra.ra_round_sparse_attn_decode(eng.ctx, q1, lview, sel_idx, n_sel, scale=w.scale)
    torch.cuda.synchronize()
    return P.cpu().numpy(), S.cpu().numpy(), sel_idx.cpu().numpy(), n_sel.cpu().numpy(), out.cpu().numpy()


@pytest.mark.parametrize("cfg,over", [("cfg1", {}), ("cfg2", {}), ("cfg5", dict(B=4)), ("cfg4", dict(B=2, n_post_layers=1, length=("lognormal", 400.0, 0.8, 16384)))])
def test_decode_pipeline_end_to_end(cfg, over):
    """scores -> selection -> sparse decode on the GPU against the oracle's own pipeline."""
    w = make_workload(cfg, **over)
    _say(f"pipeline {cfg} {over}")
    eng = Engine(w)
    P, S, sel_idx, n_sel, out = _run_gpu_pipeline(eng, w)
    ref = pipeline.run(w)
    for b, r in enumerate(ref):
        R = w.n_rounds(b)
        assert np.abs(S[b, :R] - r.S).max() < SCORE_TOL
        assert r.info["margin"] > 1e-4, "ill-conditioned seed: a score sits on the cut"
        assert sel_idx[b, :n_sel[b]].tolist() == r.sel                       # bit-exact indices
        # function parity: the oracle's rule applied to the GPU's own fp32 scores
        assert sel_idx[b, :n_sel[b]].tolist() == ora.select_rounds([float(x) for x in S[b, :R]])[0]
        err = ora.row_error(out[b], r.out[1][0])
        assert err < OUT_TOL and err < STREAM_TOL
    eng.close()


def test_workspace_and_argument_errors():
    w = make_workload("cfg2", B=2, R=3, length=("uniform", 10, 50))
    eng = Engine(w)
    view = device_view(w, 1)
    q = to_device(w.q(1)[:, 0], w.dtype)
    ra.ra_set_workspace(eng.ctx, eng.workspace[:32768])
    with pytest.raises(ra.RaError) as e:
        ra.ra_round_sparse_attn_decode(eng.ctx, q, view, scale=w.scale)
    assert e.value.code == ra.RA_ERR_WORKSPACE
    ra.ra_set_workspace(eng.ctx, eng.workspace)
    with pytest.raises(ra.RaError) as e:                                       # Hq not a multiple of Hkv
        ra.ra_round_sparse_attn_decode(eng.ctx, q[:, :30].contiguous(), view, scale=w.scale)
    assert e.value.code == ra.RA_ERR_INVALID_ARG
    w64 = make_workload("cfg2", B=2, R=3, d=64, Hq=24, length=("uniform", 10, 50))
    with pytest.raises(ra.RaError) as e:                # group size 3 is not built for the head_dim 64 path
        ra.ra_round_sparse_attn_decode(eng.ctx, to_device(w64.q(1)[:, 0], "bf16"), device_view(w64, 1), scale=0.125)
    assert e.value.code == ra.RA_ERR_UNSUPPORTED
    sel_idx, n_sel = sel_to_device([[0], [1]], 3)
    with pytest.raises(ra.RaError) as e:                                       # sel_idx without n_sel
        ra.ra_round_sparse_attn_decode(eng.ctx, q, view, sel_idx, None, scale=w.scale)
    assert e.value.code == ra.RA_ERR_INVALID_ARG
    eng.close()


def test_shapes_beyond_the_limits_are_rejected_before_anything_is_launched():
    """A batch above 1024 and more than 16 query heads per KV head are refused by the matrix-core paths with
    RA_ERR_UNSUPPORTED, by the argument checks (the outputs, filled with a marker, stay untouched)."""
    ctx = ra.ra_create(0)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    ra.ra_set_workspace(ctx, ws)

    def tiny_view(B, Hkv):
        k = torch.zeros((B * 16 * Hkv * 128,), dtype=torch.bfloat16, device="cuda")
        seg_off = torch.arange(B, dtype=torch.int64, device="cuda").reshape(B, 1) * 16
        seg_len = torch.full((B, 1), 16, dtype=torch.int32, device="cuda")
        n_rounds = torch.ones((B,), dtype=torch.int32, device="cuda")
        return ra.KVView(k, k.clone(), seg_off, seg_len, n_rounds, Hkv, 128, 16)

    marker = 12345.0
    # batch of 1025
    v = tiny_view(1025, 1)
    q = torch.zeros((1025, 1, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.full((1025, 1, 128), marker, dtype=torch.float32, device="cuda")
    with pytest.raises(ra.RaError) as e:
        ra.ra_round_sparse_attn_decode(ctx, q, v, scale=0.1, out=out)
    assert e.value.code == ra.RA_ERR_UNSUPPORTED
    with pytest.raises(ra.RaError) as e:
        ra.ra_round_sparse_attn_prefill(ctx, q.reshape(1025, 1, 1, 128), v, scale=0.1, out=out.reshape(1025, 1, 1, 128))
    assert e.value.code == ra.RA_ERR_UNSUPPORTED
    # 32 query heads on one KV head
    v = tiny_view(2, 1)
    q = torch.zeros((2, 32, 128), dtype=torch.bfloat16, device="cuda")
    out2 = torch.full((2, 32, 128), marker, dtype=torch.float32, device="cuda")
    S = torch.full((2, 1), marker, dtype=torch.float32, device="cuda")
    with pytest.raises(ra.RaError) as e:
        ra.ra_round_sparse_attn_decode(ctx, q, v, scale=0.1, out=out2)
    assert e.value.code == ra.RA_ERR_UNSUPPORTED
    for q_len in (1, 4):                                   # both score kernels
        with pytest.raises(ra.RaError) as e:
            ra.ra_round_scores(ctx, torch.zeros((2, q_len, 32, 128), dtype=torch.bfloat16, device="cuda"), v, scale=0.1, scores=S)
        assert e.value.code == ra.RA_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert (out == marker).all() and (out2 == marker).all() and (S == marker).all()
    ra.ra_destroy(ctx)


# --------------------------------------------------------------------------- question prefill (matrix cores)
PREFILL_CASES = {
    # name: (overrides on cfg3, selections)
    "q8_cur8": (dict(B=2, R=5, q_len=8, cur_len=8, length=("uniform", 10, 150)), [[0, 3], [1, 2, 4]]),
    "q5_cur12": (dict(B=2, R=4, q_len=5, cur_len=12, length=("uniform", 10, 150)), [[1], [0, 2, 3]]),
    "q6_history_only": (dict(B=2, R=4, q_len=6, cur_len=0, length=("uniform", 10, 150)), [[1, 2], [3]]),
    "q40_two_rowblocks": (dict(B=2, R=6, q_len=40, cur_len=45, length=("uniform", 20, 300)), [[0, 5], [1, 2, 3, 4]]),
    "q16_cur_only": (dict(B=1, R=3, q_len=16, cur_len=16, length=("uniform", 10, 50)), [[]]),
    "q33_paged_g8": (dict(B=2, R=5, q_len=33, cur_len=40, Hq=64, block_size=16, length=("uniform", 5, 200)),
                     [[0, 1, 4], [2]]),
    "q128_long": (dict(B=1, R=12, q_len=128, cur_len=128, length=("lognormal", 400.0, 0.8, 6000)), [[1, 4, 7, 8, 11]]),
    # ragged rounds around the 16 / 32-token tile sizes, empty rounds (selected too), uneven round counts
    "q20_ragged_rounds": (dict(B=3, q_len=20, cur_len=23, lens=[[5, 16, 17, 0, 33, 1, 250], [64, 3, 0, 0, 15, 48, 31], [96]]),
                          [[0, 1, 2, 3, 4, 5, 6], [2, 3, 5], [0]]),
    "q20_ragged_rounds_paged_g8": (dict(B=2, q_len=20, cur_len=20, Hq=64, block_size=16,
                                        lens=[[300, 17, 16, 1, 999, 50], [31, 32, 33, 0, 64, 5]]), [[0, 3, 4], [0, 1, 2, 3, 5]]),
    "q24_many_short_rounds": (dict(B=2, R=300, q_len=24, cur_len=24, length=("uniform", 1, 40)),
                              [list(range(0, 300, 3)), list(range(5, 300, 7))]),
    # paged cache, eight heads per KV head, four row blocks, several pieces per sequence
    "q64_paged_g8_long_rounds": (dict(B=2, R=12, q_len=64, cur_len=70, Hq=64, block_size=16, length=("uniform", 300, 1000)),
                                 [[0, 2, 3, 5, 7, 8, 10, 11], [1, 4, 6, 9]]),
}


# Bar of the named fp16-P mode of the many-row prefill kernel.  Each weight is rounded to fp16 (relative error
# <= 2^-12, the same rounded values in numerator and denominator), so an output moves by at most
# 2^-11 * sum_i p_i |v_i| / sum_i p_i; row_error divides by the row's largest OUTPUT, which for averaged values is
# smaller than the mean |v|, hence a bar of 2^-10: half the 2e-3 contract, 20 times the default mode's bar.
HALF_TOL = 2.0 ** -10


@pytest.mark.parametrize("p_mode", [ra.RA_PREFILL_P_BF16X2, ra.RA_PREFILL_P_F16], ids=["p_bf16x2", "p_f16"])
@pytest.mark.parametrize("name", list(PREFILL_CASES))
def test_prefill_matches_oracle(name, p_mode):
    over, sels = PREFILL_CASES[name]
    w = make_workload("cfg3", **over)
    _say(f"prefill case {name}: B={w.B} q_len={w.q_len} cur_len={w.cur_len} Hq={w.Hq} block={w.block_size}")
    eng = Engine(w)
    ra.ra_set_prefill_precision(eng.ctx, p_mode)
    STREAM_TOL = HALF_TOL if p_mode == ra.RA_PREFILL_P_F16 else globals()["STREAM_TOL"]
    view = device_view(w, 1)
    q = to_device(w.q(1), w.dtype)
    ck = to_device(w.cur_k(1), w.dtype) if w.cur_len else None
    cv = to_device(w.cur_v(1), w.dtype) if w.cur_len else None
    sel_idx, n_sel = sel_to_device(sels, view.R_max)
    out, lse = ra.ra_round_sparse_attn_prefill(eng.ctx, q, view, sel_idx, n_sel, ck, cv, scale=w.scale)
    torch.cuda.synchronize()
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    ref_o, ref_l = _oracle_attention(w, 1, sels)
    err = ora.row_error(out, ref_o)
    _say(f"  row error {err:.3e}, lse error {np.abs(lse - ref_l).max():.3e}")
    assert err < OUT_TOL and err < STREAM_TOL
    lse_tol = 2e-5 if p_mode == ra.RA_PREFILL_P_BF16X2 else HALF_TOL   # ln of a sum of weights each rounded to fp16
    assert np.allclose(lse, ref_l, rtol=0, atol=lse_tol * max(1.0, np.abs(ref_l).max()))
    eng.close()


def test_prefill_with_one_query_token_equals_decode():
    w = make_workload("cfg2", B=2, R=5, cur_len=9, length=("uniform", 10, 200))
    eng = Engine(w)
    view = device_view(w, 1)
    sels = [[0, 2], [1, 3, 4]]
    d_out, d_lse = _gpu_decode(eng, w, 1, sels, view=view)
    sel_idx, n_sel = sel_to_device(sels, view.R_max)
    p_out, p_lse = ra.ra_round_sparse_attn_prefill(eng.ctx, to_device(w.q(1), w.dtype), view, sel_idx, n_sel,
                                                   to_device(w.cur_k(1), w.dtype), to_device(w.cur_v(1), w.dtype),
                                                   scale=w.scale)
    torch.cuda.synchronize()
    assert np.array_equal(p_out.cpu().numpy()[:, 0], d_out) and np.array_equal(p_lse.cpu().numpy()[:, 0], d_lse)
    eng.close()


SCORE_PREFILL_CASES = {
    "q3_cur7_one_row_tile": dict(B=2, R=4, q_len=3, cur_len=7, length=("uniform", 10, 300)),
    "q8_cur8": dict(B=2, R=5, q_len=8, cur_len=8, length=("uniform", 10, 150)),
    "q40_cur64": dict(B=2, R=6, q_len=40, cur_len=64, length=("uniform", 20, 600)),
    "q100_two_rowblocks": dict(B=1, R=7, q_len=100, cur_len=100, length=("uniform", 20, 400)),
    "q24_history_only_paged_g8": dict(B=2, R=5, q_len=24, cur_len=0, Hq=64, block_size=16, length=("uniform", 5, 300)),
    "q300_long_question": dict(B=1, R=4, q_len=300, cur_len=300, length=("uniform", 100, 700)),
    "q20_ragged_rounds": dict(B=3, q_len=20, cur_len=23, lens=[[5, 16, 17, 0, 33, 1, 250], [64, 3, 0, 0, 15, 48, 31], [96]]),
    "q20_ragged_rounds_paged_g8": dict(B=2, q_len=20, cur_len=0, Hq=64, block_size=16,
                                       lens=[[300, 17, 16, 1, 999, 50], [31, 32, 33, 0, 64, 5]]),
    "q24_many_short_rounds": dict(B=2, R=300, q_len=24, cur_len=24, length=("uniform", 1, 40)),
    "q20_chunk_boundaries": dict(B=1, q_len=20, cur_len=300, lens=[[256, 257, 255, 512, 1, 513, 32, 31]]),
}


@pytest.mark.parametrize("name", list(SCORE_PREFILL_CASES))
def test_round_scores_prefill_shape_match_oracle(name):
    w = make_workload("cfg3", **SCORE_PREFILL_CASES[name])
    _say(f"scores (prefill shape) case {name}: B={w.B} q_len={w.q_len} cur_len={w.cur_len} Hq={w.Hq}")
    eng = Engine(w)
    view = device_view(w, 0, with_v=False)
    ck = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    P, S = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), view, ck, scale=w.scale)
    torch.cuda.synchronize()
    P, S = P.cpu().numpy(), S.cpu().numpy()
    for b in range(w.B):
        rP, rS = pipeline.scores_for_sequence(w, b)
        R = w.n_rounds(b)
        assert np.abs(P[b, :, :R] - rP).max() < SCORE_TOL and np.abs(S[b, :R] - rS).max() < SCORE_TOL
        assert np.all(P[b, :, R:] == 0) and np.all(S[b, R:] == 0)
        assert np.abs(P[b].sum(axis=1) - 1).max() < SCORE_TOL
    eng.close()


@pytest.mark.parametrize("p_mode", [ra.RA_PREFILL_P_BF16X2, ra.RA_PREFILL_P_F16], ids=["p_bf16x2", "p_f16"])
def test_prefill_pipeline_end_to_end_reduced_config3(p_mode):
    """scores (q_len 128, causal current round) -> selection -> prefill attention, config 3 at reduced batch / context."""
    w = make_workload("cfg3", B=2, length=("lognormal", 400.0, 0.8, 8192))
    eng = Engine(w)
    ra.ra_set_prefill_precision(eng.ctx, p_mode)
    STREAM_TOL = HALF_TOL if p_mode == ra.RA_PREFILL_P_F16 else globals()["STREAM_TOL"]
    v0, v1 = device_view(w, 0, with_v=False), device_view(w, 1)
    P, S = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), v0, to_device(w.cur_k(0), w.dtype), scale=w.scale)
    sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, S, v0.n_rounds)
    out, _ = ra.ra_round_sparse_attn_prefill(eng.ctx, to_device(w.q(1), w.dtype), v1, sel_idx, n_sel,
                                             to_device(w.cur_k(1), w.dtype), to_device(w.cur_v(1), w.dtype),
                                             scale=w.scale)
    torch.cuda.synchronize()
    S, sel_idx, n_sel, out = S.cpu().numpy(), sel_idx.cpu().numpy(), n_sel.cpu().numpy(), out.cpu().numpy()
    for b, r in enumerate(pipeline.run(w)):
        assert np.abs(S[b] - r.S).max() < SCORE_TOL
        assert r.info["margin"] > 1e-4
        assert sel_idx[b, :n_sel[b]].tolist() == r.sel
        err = ora.row_error(out[b], r.out[1])
        _say(f"  seq {b}: {len(r.sel)} rounds selected, row error {err:.3e}")
        assert err < OUT_TOL and err < STREAM_TOL
    eng.close()


# --------------------------------------------------------------------------- degenerate cases and determinism
def test_first_turn_without_history_attends_over_the_current_round_only():
    """R = 0 history rounds (first turn of a dialogue): nothing to score or select; decode and prefill
    attend over the current round alone."""
    w = make_workload("cfg2", B=2, R=0, cur_len=23, q_len=1)
    assert w.R_max == 0
    eng = Engine(w)
    view = device_view(w, 1)
    out, lse = _gpu_decode(eng, w, 1, [[], []], view=view, use_sel=False)
    ref_o, ref_l = _oracle_attention(w, 1, [[], []])
    assert ora.row_error(out, ref_o[:, 0]) < STREAM_TOL
    wp = make_workload("cfg3", B=2, R=0, cur_len=40, q_len=40)
    engp = Engine(wp)
    o, _ = ra.ra_round_sparse_attn_prefill(engp.ctx, to_device(wp.q(1), wp.dtype), device_view(wp, 1), None, None,
                                           to_device(wp.cur_k(1), wp.dtype), to_device(wp.cur_v(1), wp.dtype),
                                           scale=wp.scale)
    torch.cuda.synchronize()
    ref_o, _ = _oracle_attention(wp, 1, [[], []])
    assert ora.row_error(o.cpu().numpy(), ref_o) < STREAM_TOL
    # no history and no current round: the key set is empty, which only the device can see -> zeros, lse = -inf
    o, l = ra.ra_round_sparse_attn_decode(eng.ctx, to_device(w.q(1)[:, 0], w.dtype), view, scale=w.scale)
    torch.cuda.synchronize()
    assert (o.cpu().numpy() == 0).all() and np.isneginf(l.cpu().numpy()).all()
    eng.close()
    engp.close()


def test_whole_path_is_bitwise_deterministic():
    w = make_workload("cfg2", B=4)
    eng = Engine(w)
    runs = []
    for it in range(3):
        if it != 1:  # a stale register read shows on the call that follows other kernels
            _other_kernels_leave_their_registers_behind()
        runs.append(_run_gpu_pipeline(eng, w))
    for other in runs[1:]:
        for x, y in zip(runs[0], other):
            assert np.array_equal(x, y)
    wp = make_workload("cfg3", B=1, R=6, q_len=48, cur_len=48, length=("uniform", 50, 400))
    engp = Engine(wp)
    v0, v1 = device_view(wp, 0, with_v=False), device_view(wp, 1)
    outs = []
    for _ in range(2):
        _other_kernels_leave_their_registers_behind()
        P, S = ra.ra_round_scores(engp.ctx, to_device(wp.q(0), wp.dtype), v0, to_device(wp.cur_k(0), wp.dtype), scale=wp.scale)
        sel_idx, n_sel = ra.ra_select_rounds(engp.ctx, S, v0.n_rounds)
        o, l = ra.ra_round_sparse_attn_prefill(engp.ctx, to_device(wp.q(1), wp.dtype), v1, sel_idx, n_sel,
                                               to_device(wp.cur_k(1), wp.dtype), to_device(wp.cur_v(1), wp.dtype), scale=wp.scale)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy() for t in (P, S, sel_idx, n_sel, o, l)])
    for x, y in zip(*outs):
        assert np.array_equal(x, y)
    eng.close()
    engp.close()


def test_understated_max_tokens_is_reported_as_nan_scores():
    """max_tokens sizes the score pass; a value below the true history length must not go unnoticed."""
    w = make_workload("cfg2", B=1, R=6, length=("fixed", 600))
    eng = Engine(w)
    view = device_view(w, 0, with_v=False)
    k, v, seg_off, seg_len, n_rounds, bt, seg_off_v = view.tensors
    small = ra.KVView(k, v, seg_off, seg_len, n_rounds, view.Hkv, view.d, 256)      # truth: 3600 tokens
    _, S = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), small, scale=w.scale)
    torch.cuda.synchronize()
    assert np.isnan(S.cpu().numpy()).all()
    # the kernel for many query rows walks the true lengths: it must drop the chunks that have no room, not write them
    wq = make_workload("cfg3", B=1, R=6, q_len=24, cur_len=24, length=("fixed", 600))
    engq = Engine(wq)
    vq = device_view(wq, 0, with_v=False)
    k, v, seg_off, seg_len, n_rounds, bt, seg_off_v = vq.tensors
    smallq = ra.KVView(k, v, seg_off, seg_len, n_rounds, vq.Hkv, vq.d, 256)
    _, Sq = ra.ra_round_scores(engq.ctx, to_device(wq.q(0), wq.dtype), smallq, to_device(wq.cur_k(0), wq.dtype),
                               scale=wq.scale)
    torch.cuda.synchronize()
    assert np.isnan(Sq.cpu().numpy()).all()
    engq.close()
    eng.close()


def test_kernel_timing_hooks():
    """The measurement aid brackets the streaming kernel of a call: its time is positive and below the whole call's."""
    w = make_workload("cfg2", B=2, R=6, length=("uniform", 200, 600))
    eng = Engine(w)
    view = device_view(w, 0, with_v=False)
    q = to_device(w.q(0), w.dtype)
    with pytest.raises(ra.RaError):
        ra.ra_profile_last_ms(eng.ctx)            # not enabled
    ra.ra_profile_kernels(eng.ctx, True)
    with pytest.raises(ra.RaError):
        ra.ra_profile_last_ms(eng.ctx)            # no call yet
    ra.ra_round_scores(eng.ctx, q, view, scale=w.scale)          # warm-up
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    _, S1 = ra.ra_round_scores(eng.ctx, q, view, scale=w.scale)
    e1.record()
    k_ms = ra.ra_profile_last_ms(eng.ctx)
    torch.cuda.synchronize()
    assert 0.0 < k_ms <= e0.elapsed_time(e1)
    ra.ra_profile_kernels(eng.ctx, False)
    _, S2 = ra.ra_round_scores(eng.ctx, q, view, scale=w.scale)
    torch.cuda.synchronize()
    assert np.array_equal(S1.cpu().numpy(), S2.cpu().numpy())
    eng.close()


@pytest.mark.parametrize("B", [2, 1])
def test_largest_round_count_decode_and_prefill(B):
    """R_max = 1024 rounds (the largest the entry points accept): the segment tables are at their biggest.  (With one
    sequence the batch is small enough for the decode kernel to plan it by itself, were it not for the table sizes.)"""
    w = make_workload("cfg2", B=B, R=1024, length=("uniform", 1, 6))
    eng = Engine(w)
    v0, v1 = device_view(w, 0, with_v=False), device_view(w, 1)
    P, S = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), v0, scale=w.scale)
    sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, S, v0.n_rounds, ra.make_select_params(lam=0.0))
    out, _ = ra.ra_round_sparse_attn_decode(eng.ctx, to_device(w.q(1)[:, 0], w.dtype), v1, sel_idx, n_sel, scale=w.scale)
    torch.cuda.synchronize()
    S, sel_idx, n_sel, out = S.cpu().numpy(), sel_idx.cpu().numpy(), n_sel.cpu().numpy(), out.cpu().numpy()
    for b in range(w.B):
        _, rS = pipeline.scores_for_sequence(w, b)
        assert np.abs(S[b] - rS).max() < SCORE_TOL
        sel = sel_idx[b, :n_sel[b]].tolist()
        assert sel == _oracle_select_on(S[b], 1024, dict(strategy=ora.ADAPTIVE, lam=0.0))
        ref_o, _ = pipeline.attention_for_sequence(w, b, 1, sel)
        assert ora.row_error(out[b], ref_o[0]) < STREAM_TOL
    eng.close()

    w = make_workload("cfg3", B=1, R=1024, q_len=40, cur_len=40, length=("uniform", 1, 6))
    eng = Engine(w)
    v0, v1 = device_view(w, 0, with_v=False), device_view(w, 1)
    P, S = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), v0, to_device(w.cur_k(0), w.dtype), scale=w.scale)
    sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, S, v0.n_rounds, ra.make_select_params(lam=0.0))
    out, _ = ra.ra_round_sparse_attn_prefill(eng.ctx, to_device(w.q(1), w.dtype), v1, sel_idx, n_sel,
                                             to_device(w.cur_k(1), w.dtype), to_device(w.cur_v(1), w.dtype), scale=w.scale)
    torch.cuda.synchronize()
    S, sel_idx, n_sel, out = S.cpu().numpy(), sel_idx.cpu().numpy(), n_sel.cpu().numpy(), out.cpu().numpy()
    _, rS = pipeline.scores_for_sequence(w, 0)
    assert np.abs(S[0] - rS).max() < SCORE_TOL
    sel = sel_idx[0, :n_sel[0]].tolist()
    ref_o, _ = pipeline.attention_for_sequence(w, 0, 1, sel)
    assert ora.row_error(out[0], ref_o) < STREAM_TOL
    # the same question at the watershed layer, scores from the attention pass (chunk prefix table at its biggest)
    o2, _, _, S2 = ra.ra_watershed_attn_prefill(eng.ctx, to_device(w.q(0), w.dtype), device_view(w, 0),
                                                to_device(w.cur_k(0), w.dtype), to_device(w.cur_v(0), w.dtype), scale=w.scale)
    torch.cuda.synchronize()
    assert np.abs(S2[0].cpu().numpy() - rS).max() < SCORE_TOL
    ref_o, _ = pipeline.attention_for_sequence(w, 0, 0, list(range(1024)))
    assert ora.row_error(o2[0].cpu().numpy(), ref_o) < STREAM_TOL
    eng.close()


WATERSHED_CASES = {
    "bf16_g4_ragged_cur": ("cfg2", dict(B=3, R=7, cur_len=37, lens=[[5, 16, 17, 0, 33, 1, 250], [64, 3, 0, 0, 15, 48, 31],
                                                                    [7, 9, 200, 31, 32, 33, 1]])),
    "bf16_g8_paged": ("cfg5", dict(B=2, R=6, lens=[[300, 17, 16, 1, 999, 50], [31, 32, 33, 0, 64, 5]])),
    "bf16_uneven_round_counts": ("cfg2", dict(B=3, lens=[[30, 40], [10, 20, 30, 40, 50], [700]])),
    "bf16_many_rounds": ("cfg2", dict(B=2, R=300, length=("uniform", 1, 40))),
    "bf16_cfg2_full": ("cfg2", dict()),
    "bf16_g8_many_tiles": ("cfg5", dict(B=2, R=300, block_size=0, length=("uniform", 1, 40))),
}


@pytest.mark.parametrize("staged", [False, True], ids=["direct", "staged"])
@pytest.mark.parametrize("name", list(WATERSHED_CASES))
def test_watershed_decode_attention_and_scores_match_oracle(name, staged):
    """Dense decode attention at the watershed layer with the round scores from the same pass: both against the
    oracle, the scores also against the stand-alone score pass, the output bitwise against the plain decode call."""
    cfg, over = WATERSHED_CASES[name]
    w = make_workload(cfg, **over)
    _say(f"watershed decode case {name}: B={w.B} R_max={w.R_max} cur_len={w.cur_len} block={w.block_size}")
    # A generous bound on the history length makes the library expect long pieces and write the per-tile
    # values out in staged blocks; with the true bound it stores them one by one.
    extra = (1 << 20) if staged else 0
    eng = Engine(w, extra_tokens=extra)
    view = device_view(w, 0)                      # watershed layer with values
    if staged:
        k, v, seg_off, seg_len, n_rounds, bt, seg_off_v = view.tensors
        view = ra.KVView(k, v, seg_off, seg_len, n_rounds, view.Hkv, view.d, view.c.max_tokens + extra,
                         block_table=bt, block_size=view.c.block_size, seg_off_v=seg_off_v)
    q = to_device(w.q(0)[:, 0], w.dtype)
    ck = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    cv = to_device(w.cur_v(0), w.dtype) if w.cur_len else None
    cl = torch.full((w.B,), w.cur_len, dtype=torch.int32, device="cuda") if w.cur_len else None
    out, lse, P, S = ra.ra_watershed_attn_decode(eng.ctx, q, view, ck, cv, cl, scale=w.scale)
    out2, lse2 = ra.ra_round_sparse_attn_decode(eng.ctx, q, view, None, None, ck, cv, cl, scale=w.scale)
    P2, S2 = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), view, scale=w.scale)
    torch.cuda.synchronize()
    assert torch.equal(out, out2) and torch.equal(lse, lse2)
    out, P, S, P2, S2 = out.cpu().numpy(), P.cpu().numpy(), S.cpu().numpy(), P2.cpu().numpy(), S2.cpu().numpy()
    assert np.abs(P - P2).max() < SCORE_TOL and np.abs(S - S2).max() < SCORE_TOL
    for b in (range(w.B) if w.B <= 4 else (0, w.B - 1)):
        R = w.n_rounds(b)
        rP, rS = pipeline.scores_for_sequence(w, b)
        assert np.abs(P[b, :, :R] - rP).max() < SCORE_TOL and np.abs(S[b, :R] - rS).max() < SCORE_TOL
        assert np.all(P[b, :, R:] == 0) and np.all(S[b, R:] == 0)
        ref_o, _ = pipeline.attention_for_sequence(w, b, 0, list(range(R)))
        assert ora.row_error(out[b], ref_o[0]) < STREAM_TOL
    eng.close()


# (workload, overrides, extra tokens of declared capacity, workgroups at which the launch changes its prologue)
CAPACITY_CASES = {
    # more than 32 rounds: the table in LDS, or per-chunk descriptors from 2048 workgroups on
    "many_rounds_contiguous": ("cfg5", dict(B=2, R=40, length=("uniform", 20, 90), block_size=0), 40000, 2048),
    "many_rounds_paged": ("cfg5", dict(B=2, R=40, length=("uniform", 20, 90)), 40000, 2048),
    "many_rounds_current_round": ("cfg5", dict(B=3, R=40, length=("uniform", 20, 90), cur_len=40), 40000, 2048),
    # up to 32 rounds: their lengths by scalar loads, or descriptors from 32768 workgroups on
    "few_rounds_contiguous": ("cfg2", dict(B=2), 530000, 32768),
    "few_rounds_paged": ("cfg2", dict(B=2, block_size=16), 530000, 32768),
    "few_rounds_current_round": ("cfg2", dict(B=3, cur_len=40), 360000, 32768),
}


@pytest.mark.gpu
@pytest.mark.parametrize("case", list(CAPACITY_CASES))
def test_score_pass_does_not_depend_on_the_declared_capacity(case):
    """A store that declares room for a longer history gets a larger launch, and from some size on the score
    kernel's workgroups read per-chunk descriptors instead of working out their round themselves (from a table in
    LDS, or for sequences of few rounds from scalar loads).  Same chunks, same arithmetic: the scores, the per-head
    scores and the selection must not change.  (Bit for bit where both sizes finish in the same kernel; the much
    larger launch of the few-round cases finishes by rows, another order of the same sums.)"""
    name, over, extra, switch = CAPACITY_CASES[case]
    w = make_workload(name, **over)
    _say(f"score capacity case {case}: B={w.B} R_max={w.R_max} cur_len={w.cur_len} block={w.block_size}")
    eng = Engine(w, extra_tokens=extra)
    view = device_view(w, 0)
    k, v, seg_off, seg_len, n_rounds, bt, seg_off_v = view.tensors
    roomy = ra.KVView(k, v, seg_off, seg_len, n_rounds, view.Hkv, view.d, view.c.max_tokens + extra,
                      block_table=bt, block_size=view.c.block_size, seg_off_v=seg_off_v)
    assert (view.c.max_tokens // 256 + w.R_max + 1) * view.Hkv * w.B < switch <= (extra // 256) * view.Hkv * w.B
    assert (w.R_max <= 32) == (switch == 32768)
    q = to_device(w.q(0), w.dtype)
    ck = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    params = ra.make_select_params(lam=1.0)
    got = []
    for vw in (view, roomy):
        if ck is None:
            got.append(ra.ra_round_scores_select(eng.ctx, q, vw, params, scale=w.scale))
        else:  # several query tokens' worth of masses: the current round's keys are read as well
            acc = torch.zeros(w.B, w.Hq, w.R_max, dtype=torch.float32, device="cuda")
            P, S = ra.ra_round_scores_accumulate(eng.ctx, q, vw, acc, cur_k=ck, scale=w.scale)
            got.append((P, S, acc))
    torch.cuda.synchronize()
    same_finish = (w.Hq * (view.c.max_tokens // 256 + w.R_max + 1) >= 16384) == (w.Hq * (extra // 256) >= 16384)
    for x, y in zip(*got):
        if same_finish or not x.dtype.is_floating_point:
            assert torch.equal(x, y)
        else:
            assert (x - y).abs().max().item() < 1e-6
    if ck is None:
        rP, rS = pipeline.scores_for_sequence(w, 0)
        R = w.n_rounds(0)
        assert np.abs(got[1][0][0, :, :R].cpu().numpy() - rP).max() < SCORE_TOL
    eng.close()


def test_watershed_decode_rejects_what_it_cannot_do():
    w = make_workload("cfg1")                     # fp32, d = 64
    eng = Engine(w)
    view = device_view(w, 0)
    with pytest.raises(ra.RaError) as e:
        ra.ra_watershed_attn_decode(eng.ctx, to_device(w.q(0)[:, 0], w.dtype), view, scale=w.scale)
    assert e.value.code == ra.RA_ERR_UNSUPPORTED
    eng.close()
    w = make_workload("cfg2", B=1, R=6, length=("fixed", 600))
    eng = Engine(w)
    view = device_view(w, 0)
    k, v, seg_off, seg_len, n_rounds, bt, seg_off_v = view.tensors
    small = ra.KVView(k, v, seg_off, seg_len, n_rounds, view.Hkv, view.d, 256, seg_off_v=seg_off_v)   # truth: 3600 tokens
    _, _, _, S = ra.ra_watershed_attn_decode(eng.ctx, to_device(w.q(0)[:, 0], w.dtype), small, scale=w.scale)
    torch.cuda.synchronize()
    assert np.isnan(S.cpu().numpy()).all()
    eng.close()


WATERSHED_PREFILL_CASES = {
    "q8_cur8_few_rows": dict(B=2, R=5, q_len=8, cur_len=8, length=("uniform", 10, 150)),
    "q40_cur64": dict(B=2, R=6, q_len=40, cur_len=64, length=("uniform", 20, 600)),
    "q20_ragged_rounds": dict(B=3, q_len=20, cur_len=23, lens=[[5, 16, 17, 0, 33, 1, 250], [64, 3, 0, 0, 15, 48, 31], [96]]),
    "q24_history_only_paged_g8": dict(B=2, R=5, q_len=24, cur_len=0, Hq=64, block_size=16, length=("uniform", 5, 300)),
    "q1_cur9": dict(B=2, R=5, q_len=1, cur_len=9, length=("uniform", 10, 200)),
    "q128_long": dict(B=1, R=12, q_len=128, cur_len=128, length=("lognormal", 400.0, 0.8, 6000)),
}


@pytest.mark.parametrize("name", list(WATERSHED_PREFILL_CASES))
def test_watershed_prefill_attention_and_scores_match_oracle(name):
    w = make_workload("cfg3", **WATERSHED_PREFILL_CASES[name])
    _say(f"watershed prefill case {name}: B={w.B} q_len={w.q_len} cur_len={w.cur_len} Hq={w.Hq} block={w.block_size}")
    eng = Engine(w)
    view = device_view(w, 0)
    q = to_device(w.q(0), w.dtype)
    ck = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    cv = to_device(w.cur_v(0), w.dtype) if w.cur_len else None
    out, lse, P, S = ra.ra_watershed_attn_prefill(eng.ctx, q, view, ck, cv, scale=w.scale)
    out2, lse2 = ra.ra_round_sparse_attn_prefill(eng.ctx, q, view, None, None, ck, cv, scale=w.scale)
    P2, S2 = ra.ra_round_scores(eng.ctx, q, view, ck, scale=w.scale)
    torch.cuda.synchronize()
    if w.q_len * w.G <= 32:
        assert torch.equal(out, out2) and torch.equal(lse, lse2)          # same kernel, same pieces
    else:
        # the pieces of the fused pass end on 256-token chunk boundaries: other pieces, other softmax references,
        # so the two results differ by the arithmetic's own error (both are held to the oracle below)
        assert ora.row_error(out.cpu().numpy(), out2.cpu().numpy()) < STREAM_TOL
        assert (lse - lse2).abs().max().item() < 2e-5
    # the fp16-P mode is for the post-watershed layers: the watershed call, whose scores decide the selection, ignores it
    ra.ra_set_prefill_precision(eng.ctx, ra.RA_PREFILL_P_F16)
    out3, lse3, P3, S3 = ra.ra_watershed_attn_prefill(eng.ctx, q, view, ck, cv, scale=w.scale)
    ra.ra_set_prefill_precision(eng.ctx, ra.RA_PREFILL_P_BF16X2)
    torch.cuda.synchronize()
    assert torch.equal(out, out3) and torch.equal(lse, lse3) and torch.equal(P, P3) and torch.equal(S, S3)
    out, P, S, P2, S2 = out.cpu().numpy(), P.cpu().numpy(), S.cpu().numpy(), P2.cpu().numpy(), S2.cpu().numpy()
    assert np.abs(P - P2).max() < SCORE_TOL and np.abs(S - S2).max() < SCORE_TOL
    for b in range(w.B):
        R = w.n_rounds(b)
        rP, rS = pipeline.scores_for_sequence(w, b)
        assert np.abs(P[b, :, :R] - rP).max() < SCORE_TOL and np.abs(S[b, :R] - rS).max() < SCORE_TOL
        assert np.all(P[b, :, R:] == 0) and np.all(S[b, R:] == 0)
        ref_o, _ = pipeline.attention_for_sequence(w, b, 0, list(range(R)))
        assert ora.row_error(out[b], ref_o) < STREAM_TOL
    eng.close()


def test_one_very_long_round_next_to_a_tiny_one():
    """A single round of 100 000 tokens (thousands of tiles and hundreds of score chunks in one segment) beside
    rounds of 7 and 1 tokens: scores, selection-free decode and a short question prefill."""
    w = make_workload("cfg2", B=1, R=3, q_len=3, cur_len=5, lens=[[100000, 7, 1]])
    _say(f"long-round case: tokens={w.total_tokens(0)}")
    eng = Engine(w)
    v0, v1 = device_view(w, 0, with_v=False, threads=8), device_view(w, 1, threads=8)
    ck0, ck1, cv1 = (to_device(x, w.dtype) for x in (w.cur_k(0), w.cur_k(1), w.cur_v(1)))
    P, S = ra.ra_round_scores(eng.ctx, to_device(w.q(0), w.dtype), v0, ck0, scale=w.scale)
    po, pl = ra.ra_round_sparse_attn_prefill(eng.ctx, to_device(w.q(1), w.dtype), v1, None, None, ck1, cv1, scale=w.scale)
    cl = torch.full((1,), w.cur_len, dtype=torch.int32, device="cuda")
    do, dl = ra.ra_round_sparse_attn_decode(eng.ctx, to_device(w.q(1)[:, -1], w.dtype), v1, None, None, ck1, cv1, cl,
                                            scale=w.scale)
    torch.cuda.synchronize()
    rP, rS = pipeline.scores_for_sequence(w, 0)
    assert np.abs(P[0].cpu().numpy() - rP).max() < SCORE_TOL and np.abs(S[0].cpu().numpy() - rS).max() < SCORE_TOL
    ro, rl = pipeline.attention_for_sequence(w, 0, 1, [0, 1, 2])
    assert ora.row_error(po[0].cpu().numpy(), ro) < STREAM_TOL
    assert np.allclose(pl[0].cpu().numpy(), rl, rtol=0, atol=2e-5 * np.abs(rl).max())
    # the last question token sees the whole current round: the decode call must give the prefill's last row
    assert ora.row_error(do[0].cpu().numpy()[None], ro[-1:]) < STREAM_TOL
    eng.close()


def test_calls_on_a_side_stream_are_ordered_on_that_stream():
    """Every compute call only enqueues on the caller's stream: a whole step issued on a non-default stream, with
    the inputs produced on that stream just before, matches the oracle."""
    w = make_workload("cfg2", B=2, R=6, length=("uniform", 20, 300))
    eng = Engine(w)
    v0, v1 = device_view(w, 0, with_v=False), device_view(w, 1)
    q0_host, q1_host = to_device(w.q(0), w.dtype).cpu().pin_memory(), to_device(w.q(1)[:, 0], w.dtype).cpu().pin_memory()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        q0 = q0_host.to("cuda", non_blocking=True)        # the copies are ordered before the kernels on `side` only
        q1 = q1_host.to("cuda", non_blocking=True)
        P, S = ra.ra_round_scores(eng.ctx, q0, v0, scale=w.scale, stream=side)
        sel_idx, n_sel = ra.ra_select_rounds(eng.ctx, S, v0.n_rounds, ra.make_select_params(lam=0.5), stream=side)
        out, lse = ra.ra_round_sparse_attn_decode(eng.ctx, q1, v1, sel_idx, n_sel, scale=w.scale, stream=side)
    side.synchronize()
    ref = pipeline.run(w, select_params=dict(lam=0.5))
    for b, r in enumerate(ref):
        assert sel_idx[b, :n_sel[b]].tolist() == r.sel
        assert ora.row_error(out[b].cpu().numpy()[None], r.out[1]) < STREAM_TOL
    eng.close()


def test_read_bandwidth_probe_returns_a_plausible_figure():
    eng = Engine(make_workload("cfg1"))
    buf = torch.zeros(1 << 27, dtype=torch.float32, device="cuda")       # 512 MiB
    gbs = ra.ra_measure_read_bandwidth(eng.ctx, buf, iters=3)
    _say(f"plain read kernel: {gbs:.0f} GB/s")
    assert 500.0 < gbs < 8000.0                                          # below the published peak, above PCIe-class rates
    with pytest.raises(ra.RaError) as e:
        ra.ra_measure_read_bandwidth(eng.ctx, buf[1:5], iters=1)         # not 16-byte aligned
    assert e.value.code == ra.RA_ERR_INVALID_ARG
    eng.close()


def test_one_sequence_with_600_rounds_is_planned_inside_the_decode_kernel():
    """The largest single-sequence batch whose segment lists the decode kernel still keeps in LDS by itself."""
    w = make_workload("cfg2", B=1, R=600, cur_len=9, length=("uniform", 1, 40))
    eng = Engine(w)
    sels = [sorted(np.random.default_rng(1).choice(600, size=211, replace=False).tolist())]
    out, lse = _gpu_decode(eng, w, 1, sels)
    ref_o, ref_l = _oracle_attention(w, 1, sels)
    assert ora.row_error(out, ref_o[:, 0]) < STREAM_TOL
    assert np.allclose(lse, ref_l[:, 0], rtol=0, atol=2e-5 * np.abs(ref_l).max())
    eng.close()


def _other_kernels_leave_their_registers_behind():
    """Unrelated kernels on every compute unit: what they leave in the register files is what a stale read finds."""
    x = torch.zeros(1 << 16, device="cuda")
    for _ in range(100):
        x = x * 1.5 + 1.0
    y = torch.randn(1 << 24, device="cuda")
    float((y * 2).sum().item())


@pytest.mark.parametrize("name", list(WATERSHED_PREFILL_CASES))
@pytest.mark.parametrize("p_mode", [ra.RA_PREFILL_P_BF16X2, ra.RA_PREFILL_P_F16], ids=["p_bf16x2", "p_f16"])
def test_prefill_calls_are_bitwise_reproducible_after_other_kernels(name, p_mode):
    """Outputs, log-sum-exps and scores are identical to the bit from call to call, also for the call that follows
    unrelated kernels.  An instruction that reads a register too early (a matrix-core result still in flight, say)
    gets the previous tile's value, and on a wave's first tile whatever the last kernel on that compute unit left
    there: the results then differ in their last bits exactly on such a call, which is what this test provokes."""
    w = make_workload("cfg3", **WATERSHED_PREFILL_CASES[name])
    eng = Engine(w)
    ra.ra_set_prefill_precision(eng.ctx, p_mode)
    view = device_view(w, 0)
    q = to_device(w.q(0), w.dtype)
    ck = to_device(w.cur_k(0), w.dtype) if w.cur_len else None
    cv = to_device(w.cur_v(0), w.dtype) if w.cur_len else None
    first = None
    for it in range(5):
        if it in (0, 2, 3):
            _other_kernels_leave_their_registers_behind()
        o1, l1, P, S = ra.ra_watershed_attn_prefill(eng.ctx, q, view, ck, cv, scale=w.scale)
        o2, l2 = ra.ra_round_sparse_attn_prefill(eng.ctx, q, view, None, None, ck, cv, scale=w.scale)
        P2, S2 = ra.ra_round_scores(eng.ctx, q, view, ck, scale=w.scale)
        torch.cuda.synchronize()
        cur = [t.cpu().numpy().copy() for t in (o1, l1, P, S, o2, l2, P2, S2)]
        if first is None:
            first = cur
        else:
            for x, y in zip(first, cur):
                assert np.array_equal(x, y, equal_nan=True), (name, it)
    eng.close()
