"""GPU tests of the statistics beside the hot path: the answer tokens' running round distribution
(Eq. 1, right-hand form), the watershed curve (Sec. 3.1, Observation 2, Fig. 2b) and the coverage of
a selection."""
import math

import numpy as np
import pytest
import torch

import paper_2502_15294_amd as ra
from oracle import round_attention as ora
from synth import make_workload
from synth.device import Engine, device_view, sel_to_device, to_device

pytestmark = pytest.mark.gpu
SCORE_TOL = 1e-5


ACC_CASES = [
    # (name, workload overrides, question tokens already in the current round, query tokens per call)
    ("bf16_decode_steps", ("cfg2", dict(B=3, R=6, q_len=5, cur_len=12, length=("uniform", 20, 300))), 7, [1] * 5),
    ("bf16_no_question_tokens", ("cfg2", dict(B=2, R=5, q_len=4, cur_len=4, length=("uniform", 20, 300))), 0, [1] * 4),
    ("f32_decode_steps", ("cfg1", dict(B=2, q_len=4, cur_len=9)), 5, [1] * 4),
    ("bf16_small_groups", ("cfg2", dict(B=2, R=6, q_len=5, cur_len=9, length=("uniform", 20, 300))), 4, [3, 2]),
    ("bf16_many_rows", ("cfg3", dict(B=2, R=5, q_len=48, cur_len=50, length=("uniform", 40, 400))), 2, [24, 24]),
    ("bf16_many_rounds", ("cfg5", dict(B=2, R=150, q_len=3, cur_len=3, length=("uniform", 1, 40), block_size=0)), 0,
     [1, 1, 1]),
    ("bf16_finish_head_by_head", ("cfg5", dict(B=2, R=300, q_len=2, cur_len=5, length=("uniform", 1, 40), block_size=0)), 3,
     [1, 1]),
]


@pytest.mark.parametrize("case", ACC_CASES, ids=[c[0] for c in ACC_CASES])
def test_answer_scores_accumulate_to_eq1_right(case):
    name, (cfg, kw), c0, groups = case
    w = make_workload(cfg, **kw)
    print(f"accumulate case {name}: B={w.B} R={w.R_max} groups={groups}", flush=True)
    assert sum(groups) == w.q_len and c0 + w.q_len == w.cur_len
    eng = Engine(w)
    view = device_view(w, 0, with_v=False)
    q_all, cur_all = w.q(0), w.cur_k(0)
    acc = torch.zeros((w.B, w.Hq, view.R_max), dtype=torch.float32, device="cuda")
    done = 0
    for n in groups:
        q = to_device(np.ascontiguousarray(q_all[:, done:done + n]), w.dtype)
        cur = to_device(np.ascontiguousarray(cur_all[:, :c0 + done + n]), w.dtype)
        P, S = ra.ra_round_scores_accumulate(eng.ctx, q, view, acc, cur_k=cur, scale=w.scale)
        done += n
        # after every call the outputs are Eq. 1 over the answer tokens so far
        for b in range(w.B):
            k_rounds = [w.k_round(b, 0, r) for r in range(w.n_rounds(b))]
            Pr, Sr = ora.round_scores(q_all[b, :done], k_rounds, w.scale, cur_all[b, :c0 + done])
            R = w.n_rounds(b)
            assert np.abs(P[b, :, :R].cpu().numpy() - Pr).max() < SCORE_TOL, (name, b, done)
            assert np.abs(S[b, :R].cpu().numpy() - Sr).max() < SCORE_TOL, (name, b, done)
            assert np.all(S[b, R:].cpu().numpy() == 0)
    # one call over all the tokens gives the same distribution
    P1, S1 = ra.ra_round_scores(eng.ctx, to_device(q_all, w.dtype), view, cur_k=to_device(cur_all, w.dtype),
                                scale=w.scale)
    assert (S1 - S).abs().max().item() < SCORE_TOL
    # the totals themselves: their sum over the rounds is at most one per token and head
    tot = acc.sum(dim=2)
    assert (tot <= w.q_len * (1 + 1e-5)).all() and (tot > 0).all()
    eng.close()


def test_accumulate_from_zero_equals_plain_scores_for_several_tokens():
    w = make_workload("cfg2", B=2, R=6, q_len=3, cur_len=7, length=("uniform", 20, 300))
    eng = Engine(w)
    view = device_view(w, 0, with_v=False)
    q, cur = to_device(w.q(0), w.dtype), to_device(w.cur_k(0), w.dtype)
    acc = torch.zeros((w.B, w.Hq, view.R_max), dtype=torch.float32, device="cuda")
    Pa, Sa = ra.ra_round_scores_accumulate(eng.ctx, q, view, acc, cur_k=cur, scale=w.scale)
    P, S = ra.ra_round_scores(eng.ctx, q, view, cur_k=cur, scale=w.scale)
    assert torch.equal(Pa, P) and torch.equal(Sa, S)
    rc = ra.lib().ra_round_scores_accumulate(eng.ctx, None, q.data_ptr(), 3, w.Hq, view.c, cur.data_ptr(), 7, 1.0, None,
                                             None, S.data_ptr())
    assert rc == ra.RA_ERR_INVALID_ARG and b"acc" in ra.lib().ra_last_error()
    eng.close()


def _random_layers(rng, L, B, R_max, n_rounds):
    P = np.zeros((L, B, R_max), dtype=np.float32)
    for l in range(L):
        for b in range(B):
            R = n_rounds[b]
            if R == 0:
                continue
            # early layers differ a lot, later layers little: the shape of the paper's curve
            base = np.random.default_rng(1000 + b).random(R) ** 3
            x = base + rng.random(R) * (2.0 if l < L // 3 else 0.05)
            P[l, b, :R] = (x / x.sum()).astype(np.float32)
    return P


@pytest.mark.parametrize("L,B,R_max,n_rounds", [(6, 3, 20, [20, 7, 1]), (28, 2, 300, [300, 257]),
                                                (2, 4, 1024, [1024, 1000, 3, 0]), (36, 1, 64, [64])])
def test_layer_divergence_matches_the_oracle(L, B, R_max, n_rounds):
    rng = np.random.default_rng(L * 100 + R_max)
    P = _random_layers(rng, L, B, R_max, n_rounds)
    if R_max == 20:
        P[2, 0, 5] = 0.0          # a zero in the layer itself: its term vanishes (+inf for layers 0 and 1)
        P[4, 1, 3] = 0.0          # a zero in a later layer under a positive mass: +inf for layers 0..3
    eng = Engine(make_workload("cfg1"))
    kl, kl_mean = ra.ra_layer_divergence(eng.ctx, torch.from_numpy(P).cuda(),
                                         torch.tensor(n_rounds, dtype=torch.int32, device="cuda"))
    kl, kl_mean = kl.cpu().numpy(), kl_mean.cpu().numpy()
    for b in range(B):
        want = ora.mean_kl_to_later_layers(P[:, b, :n_rounds[b]])
        fin = np.isfinite(want)
        assert np.array_equal(np.isposinf(kl[b]), np.isposinf(want)), b
        assert np.allclose(kl[b][fin], want[fin], rtol=1e-11, atol=1e-15), (b, np.abs(kl[b][fin] - want[fin]).max())
    if R_max == 20:
        assert np.isposinf(kl[1, :4]).all() and np.isfinite(kl[1, 4:]).all()
        assert np.isposinf(kl[0, :2]).all() and np.isfinite(kl[0, 2:]).all()
    with np.errstate(invalid="ignore"):
        assert np.allclose(kl_mean, kl.sum(axis=0) / B, rtol=1e-14, equal_nan=True)
    if L >= 6 and R_max >= 64:    # the synthetic curve drops where the layers start to agree
        assert kl_mean[: L // 3].min() > 10 * kl_mean[L // 3:].max()
    eng.close()


def test_selection_coverage_matches_the_oracle():
    rng = np.random.default_rng(77)
    B, R_max = 5, 200
    n_rounds = [200, 130, 64, 1, 0]
    S = np.zeros((B, R_max), dtype=np.float32)
    sels = []
    for b, R in enumerate(n_rounds):
        if R:
            x = rng.random(R) ** 4
            S[b, :R] = (x / x.sum()).astype(np.float32)
        sels.append(sorted(rng.choice(R, size=min(R, [90, 10, 64, 1, 0][b]), replace=False).tolist()) if R else [])
    eng = Engine(make_workload("cfg1"))
    sel_idx, n_sel = sel_to_device(sels, R_max)
    cov = ra.ra_selection_coverage(eng.ctx, torch.from_numpy(S).cuda(), sel_idx, n_sel).cpu().numpy()
    for b in range(B):
        assert abs(cov[b] - ora.selection_coverage(S[b], sels[b])) < 1e-6, b
    assert cov[2] == pytest.approx(1.0, abs=1e-6) and cov[4] == 0.0
    eng.close()
