"""Pins for the CPU oracle: every check compares it with something it did not compute itself
(a closed form, a library routine, scalar brute force, or numbers the paper prints)."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import round_attention as ra
from oracle import memory_model
from oracle.dense_reference import dense_attention

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_case(seed, q_len=1, Hq=4, Hkv=2, d=16, lens=(5, 9, 1, 7), cur_len=0):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((q_len, Hq, d))
    ks = [rng.standard_normal((n, Hkv, d)) for n in lens]
    vs = [rng.standard_normal((n, Hkv, d)) for n in lens]
    ck = rng.standard_normal((cur_len, Hkv, d)) if cur_len else None
    cv = rng.standard_normal((cur_len, Hkv, d)) if cur_len else None
    return q, ks, vs, ck, cv


# --------------------------------------------------------------------------- S1: round scores
def test_scores_sum_to_one_per_head():
    # Sec. 3.1: P is qAtt normalised over rounds.
    for cur_len, q_len in ((0, 1), (0, 3), (6, 3), (4, 4)):
        q, ks, _, ck, _ = _rand_case(1, q_len=q_len, cur_len=cur_len)
        P, S = ra.round_scores(q, ks, 0.25, ck)
        assert np.allclose(P.sum(axis=1), 1.0, atol=1e-12)
        assert abs(S.sum() - 1.0) < 1e-12
        assert (P >= 0).all()


def test_scores_decode_closed_form_logsumexp():
    # One query token, no current round: P[h, :] = softmax over rounds of the per-round
    # log-sum-exp of the scaled logits.  Independent path through scipy.
    q, ks, _, _, _ = _rand_case(2, q_len=1, Hq=6, Hkv=2, d=8, lens=(3, 11, 4, 8, 2))
    scale = 1.0 / math.sqrt(8)
    P, _ = ra.round_scores(q, ks, scale)
    for h in range(6):
        g = h // 3
        lse = np.array([scipy.special.logsumexp(scale * (k[:, g, :] @ q[0, h])) for k in ks])
        assert np.allclose(P[h], scipy.special.softmax(lse), rtol=1e-12, atol=1e-15)


def test_scores_identical_keys_give_length_fractions():
    # All keys equal => every token has the same probability => P[h, r] = len_r / T exactly.
    rng = np.random.default_rng(3)
    lens = (4, 10, 1, 5)
    key = rng.standard_normal((1, 2, 16))
    ks = [np.repeat(key, n, axis=0) for n in lens]
    for q_len in (1, 3):
        q = rng.standard_normal((q_len, 4, 16))
        P, S = ra.round_scores(q, ks, 0.25)
        expect = np.array(lens) / sum(lens)
        assert np.allclose(P, expect[None, :], atol=1e-14)
        assert np.allclose(S, expect, atol=1e-14)
    # zero queries: same thing with arbitrary keys
    q, ks2, _, _, _ = _rand_case(4, lens=lens)
    P, _ = ra.round_scores(np.zeros_like(q), ks2, 0.25)
    assert np.allclose(P, expect[None, :], atol=1e-14)


def test_scores_concentrate_on_strongly_biased_round():
    q, ks, _, _, _ = _rand_case(5, Hq=2, Hkv=2, d=16, lens=(6, 6, 6, 6))
    for g in range(2):
        ks[2][:, g, :] += 40.0 * q[0, g] / np.linalg.norm(q[0, g])
    P, S = ra.round_scores(q, ks, 0.25)
    assert np.allclose(P[:, 2], 1.0, atol=1e-9) and np.argmax(S) == 2


def test_scores_brute_force_scalar_loops():
    # Eq. 1 written as scalar loops with math.exp, including GQA head mapping, several query
    # tokens and the causal current round.
    q_len, Hq, Hkv, d, lens, cur_len = 3, 4, 2, 5, (2, 4, 3), 4
    q, ks, _, ck, _ = _rand_case(6, q_len=q_len, Hq=Hq, Hkv=Hkv, d=d, lens=lens, cur_len=cur_len)
    scale = 0.3
    P, S = ra.round_scores(q, ks, scale, ck)
    G = Hq // Hkv
    Pb = [[0.0] * len(lens) for _ in range(Hq)]
    for h in range(Hq):
        g = h // G
        qatt = [0.0] * len(lens)
        for i in range(q_len):
            w_hist = [[math.exp(scale * sum(q[i, h, c] * ks[r][j, g, c] for c in range(d)))
                       for j in range(lens[r])] for r in range(len(lens))]
            w_cur = [math.exp(scale * sum(q[i, h, c] * ck[j, g, c] for c in range(d)))
                     for j in range(cur_len) if j <= cur_len - q_len + i]
            z = sum(sum(row) for row in w_hist) + sum(w_cur)
            for r in range(len(lens)):
                qatt[r] += sum(w_hist[r]) / z
        tot = sum(qatt)
        Pb[h] = [x / tot for x in qatt]
    assert np.allclose(P, np.array(Pb), rtol=1e-11)
    assert np.allclose(S, np.array(Pb).mean(axis=0), rtol=1e-11)


def test_scores_current_round_changes_multi_query_but_not_single_query():
    # With one query token the current round's share of the softmax cancels in the
    # normalisation over history rounds; with several query tokens it does not.
    q, ks, _, ck, _ = _rand_case(7, q_len=1, cur_len=5)
    P0, _ = ra.round_scores(q, ks, 0.25)
    P1, _ = ra.round_scores(q, ks, 0.25, ck)
    assert np.allclose(P0, P1, rtol=1e-12)
    q, ks, _, ck, _ = _rand_case(8, q_len=4, cur_len=6)
    P0, _ = ra.round_scores(q, ks, 0.25)
    P1, _ = ra.round_scores(q, ks, 0.25, ck)
    assert not np.allclose(P0, P1, rtol=1e-6)


def test_scores_empty_history_and_zero_length_round():
    q, ks, _, _, _ = _rand_case(9, lens=(4, 0, 3))
    P, S = ra.round_scores(q, ks, 0.25)
    assert P.shape == (4, 3) and np.all(P[:, 1] == 0.0) and abs(S.sum() - 1) < 1e-12
    P, S = ra.round_scores(q, [], 0.25)
    assert P.shape == (4, 0) and S.shape == (0,)


# --------------------------------------------------------------------------- S2: selection
def _constants():
    out = {}
    with open(os.path.join(GOLDEN, "selection_constants.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def test_select_paper_constants_are_the_defaults():
    c = _constants()
    import inspect
    sig = inspect.signature(ra.select_rounds)
    assert sig.parameters["threshold"].default == c["threshold_v"]
    assert sig.parameters["fraction"].default == c["top_fraction"]


def test_select_hand_worked_example():
    # S = [.5,.2,.1,.1,.1]: mean .2, population variance (.09+0+3*.01)/5 = .024, std .15492
    S = [0.5, 0.2, 0.1, 0.1, 0.1]
    sel, info = ra.select_rounds(S, ra.ADAPTIVE, lam=1.0)
    assert sel == [0] and abs(info["cut"] - (0.2 + math.sqrt(0.024))) < 1e-15
    # Sec. 4.4 rule (greater than the average), strict inequality.  Dyadic scores so that the mean
    # is exact: [.5,.25,.125,.125] has mean .25 and .25 > .25 is false.
    D = [0.5, 0.25, 0.125, 0.125]
    sel0, info0 = ra.select_rounds(D, ra.ADAPTIVE, lam=_constants()["mean_rule_lambda"])
    assert sel0 == [0] and info0["cut"] == 0.25
    # population variance (.0625 + 0 + 2 * .015625) / 4 = .0234375
    assert ra.select_rounds(D, ra.ADAPTIVE, lam=1.0)[1]["cut"] == 0.25 + math.sqrt(0.0234375)
    assert ra.select_rounds([0.5, 0.21, 0.09, 0.1, 0.1], ra.ADAPTIVE, lam=0.0)[0] == [0, 1]
    # strategy 1 with v = 0.1: .1 > .1 is false
    assert ra.select_rounds(S, ra.THRESHOLD)[0] == [0, 1]
    # strategy 2: top 10 % of 5 rounds -> ceil(.5) = 1 round; of 25 rounds -> 3
    assert ra.select_rounds(S, ra.TOP_FRACTION)[0] == [0]
    S25 = [(i * 7 % 25) / 300.0 for i in range(25)]
    top3 = sorted(sorted(range(25), key=lambda r: -S25[r])[:3])
    assert ra.select_rounds(S25, ra.TOP_FRACTION)[0] == top3
    # sample standard deviation: variance .03, std .17320
    _, info1 = ra.select_rounds(S, ra.ADAPTIVE, lam=1.0, ddof=1)
    assert abs(info1["cut"] - (0.2 + math.sqrt(0.03))) < 1e-15


def test_select_mean_is_one_over_R_for_a_distribution():
    rng = np.random.default_rng(10)
    S = rng.random(37)
    S /= S.sum()
    _, info = ra.select_rounds(S, ra.ADAPTIVE, lam=0.0)
    assert abs(info["cut"] - 1.0 / 37) < 1e-15
    lam = 1.3
    _, info = ra.select_rounds(S, ra.ADAPTIVE, lam=lam)
    assert abs(info["cut"] - (1.0 / 37 + lam * np.std(S))) < 1e-14
    sel = ra.select_rounds(S, ra.ADAPTIVE, lam=lam)[0]
    assert sel == [int(r) for r in np.nonzero(S > np.mean(S) + lam * np.std(S))[0]]


def test_select_degenerate_vectors():
    assert ra.select_rounds([0.25] * 4, ra.ADAPTIVE)[0] == [0]          # uniform: nothing passes, argmax fallback
    assert ra.select_rounds([0.25] * 4, ra.ADAPTIVE, min_rounds=0)[0] == []
    assert ra.select_rounds([0, 0, 1.0, 0], ra.ADAPTIVE)[0] == [2]      # one-hot
    assert ra.select_rounds([1.0], ra.ADAPTIVE)[0] == [0]
    assert ra.select_rounds([1.0], ra.ADAPTIVE, ddof=1)[0] == [0]
    assert ra.select_rounds([], ra.ADAPTIVE)[0] == []
    assert ra.select_rounds([0.0] * 5, ra.THRESHOLD)[0] == [0]          # all-zero: forced minimum picks round 0


def test_select_scale_invariance_and_caps():
    rng = np.random.default_rng(11)
    S = rng.random(50) ** 4
    S /= S.sum()
    for strat in (ra.ADAPTIVE, ra.TOP_FRACTION):
        assert ra.select_rounds(S, strat)[0] == ra.select_rounds(8.0 * S, strat)[0]
    full = ra.select_rounds(S, ra.ADAPTIVE, lam=0.0)[0]
    capped = ra.select_rounds(S, ra.ADAPTIVE, lam=0.0, max_rounds=3)[0]
    assert len(full) > 3 and len(capped) == 3
    assert capped == sorted(sorted(full, key=lambda r: -S[r])[:3])
    forced = ra.select_rounds(S, ra.THRESHOLD, threshold=2.0, min_rounds=4)[0]
    assert forced == sorted(np.argsort(-S, kind="stable")[:4].tolist())


def test_select_top_fraction_matches_stable_argsort_and_ties():
    rng = np.random.default_rng(12)
    for R in (1, 7, 10, 11, 64, 200):
        S = np.round(rng.random(R), 1)          # many exact ties
        k = max(1, math.ceil(0.10 * R))
        expect = sorted(np.argsort(-S, kind="stable")[:k].tolist())
        assert ra.select_rounds(S, ra.TOP_FRACTION)[0] == expect


def test_select_output_is_ascending_and_unique():
    rng = np.random.default_rng(13)
    S = rng.random(40)
    sel = ra.select_rounds(S, ra.ADAPTIVE, lam=-0.5)[0]
    assert sel == sorted(set(sel)) and len(sel) > 1


# --------------------------------------------------------------------------- S4 / S5: sparse attention
def test_select_all_reproduces_dense_attention_library():
    # Sec. 3.5: with K = T the method is the original inference.
    for q_len, cur_len in ((1, 0), (1, 3), (4, 4), (3, 7)):
        q, ks, vs, ck, cv = _rand_case(20, q_len=q_len, Hq=6, Hkv=2, d=16, lens=(5, 9, 1, 7), cur_len=cur_len)
        O, _ = ra.sparse_attention(q, ks, vs, [0, 1, 2, 3], 0.25, ck, cv)
        K = np.concatenate(ks + ([ck] if cur_len else []))
        V = np.concatenate(vs + ([cv] if cur_len else []))
        if cur_len == 0:
            ref = dense_attention(q, K, V, 0.25)
        else:
            # history fully visible + causal tail == lower-right aligned causal mask over the
            # concatenation, because the queries are the last q_len tokens of the current round
            ref = dense_attention(q, K, V, 0.25, causal_tail=True)
        assert np.allclose(O, ref, rtol=1e-12, atol=1e-13)


def test_sparse_equals_dense_on_gathered_rounds_and_permutation_invariance():
    q, ks, vs, _, _ = _rand_case(21, q_len=2, Hq=4, Hkv=4, d=8, lens=(5, 9, 3, 7, 2))
    sel = [1, 3, 4]
    O, lse = ra.sparse_attention(q, ks, vs, sel, 0.35)
    ref = dense_attention(q, np.concatenate([ks[r] for r in sel]), np.concatenate([vs[r] for r in sel]), 0.35)
    assert np.allclose(O, ref, rtol=1e-12, atol=1e-13)
    O2, lse2 = ra.sparse_attention(q, ks, vs, [4, 1, 3], 0.35)
    assert np.allclose(O, O2, rtol=1e-13) and np.allclose(lse, lse2, rtol=1e-13)


def test_current_round_only_is_causal_self_attention():
    rng = np.random.default_rng(22)
    n, Hq, Hkv, d = 9, 4, 2, 8
    q = rng.standard_normal((n, Hq, d))
    ck = rng.standard_normal((n, Hkv, d))
    cv = rng.standard_normal((n, Hkv, d))
    O, _ = ra.sparse_attention(q, [], [], [], 0.3, ck, cv)
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]
    kt = torch.from_numpy(ck).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    vt = torch.from_numpy(cv).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True, scale=0.3)
    assert np.allclose(O, ref[0].permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-13)


def test_sparse_attention_brute_force_scalar_loops():
    q_len, Hq, Hkv, d, lens, cur_len = 2, 4, 2, 3, (2, 3, 2), 3
    q, ks, vs, ck, cv = _rand_case(23, q_len=q_len, Hq=Hq, Hkv=Hkv, d=d, lens=lens, cur_len=cur_len)
    sel, scale = [0, 2], 0.4
    O, lse = ra.sparse_attention(q, ks, vs, sel, scale, ck, cv)
    for i in range(q_len):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            toks = [(ks[r][j, g], vs[r][j, g]) for r in sel for j in range(lens[r])]
            toks += [(ck[j, g], cv[j, g]) for j in range(cur_len) if j <= cur_len - q_len + i]
            wts = [math.exp(scale * sum(q[i, h, c] * k[c] for c in range(d))) for k, _ in toks]
            z = sum(wts)
            for c in range(d):
                assert abs(O[i, h, c] - sum(w * v[c] for w, (_, v) in zip(wts, toks)) / z) < 1e-12
            assert abs(lse[i, h] - math.log(z)) < 1e-12


def test_scores_and_sparse_attention_are_consistent():
    # O over a selected set = sum over its rounds of (round weight) x (attention inside that round
    # alone), the weights being the round scores renormalised over the set (same layer, one query).
    q, ks, vs, _, _ = _rand_case(24, q_len=1, Hq=4, Hkv=2, d=8, lens=(4, 6, 3, 5, 2))
    sel = [0, 2, 3]
    P, _ = ra.round_scores(q, ks, 0.3)
    O, _ = ra.sparse_attention(q, ks, vs, sel, 0.3)
    mix = np.zeros_like(O)
    for r in sel:
        Or, _ = ra.sparse_attention(q, ks, vs, [r], 0.3)
        mix += (P[:, r] / P[:, sel].sum(axis=1))[None, :, None] * Or
    assert np.allclose(O, mix, rtol=1e-12, atol=1e-14)


def test_empty_key_set_is_an_error():
    q, ks, vs, _, _ = _rand_case(25)
    with pytest.raises(ValueError):
        ra.sparse_attention(q, ks, vs, [], 0.3)


# --------------------------------------------------------------------------- memory model (Sec. 3.5)
def _table5():
    rows = []
    with open(os.path.join(GOLDEN, "table5_watershed_layers.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, L, Lw, pct = line.split()
                rows.append((name, int(L), int(Lw), int(pct)))
    return rows


def test_memory_ratio_matches_eq2_and_table5():
    T, n_tok, bpt = 40, 37, 4096
    lens = [n_tok] * T
    for name, L, Lw, pct in _table5():
        for K in (0, 6, 8, T):
            sel = list(range(0, K))
            ratio = memory_model.resident_kv_bytes(lens, sel, L, Lw, bpt) / memory_model.full_kv_bytes(lens, L, bpt)
            assert abs(ratio - (Lw / L + (K / T) * (1 - Lw / L))) < 1e-12, name
        saving = 1.0 - memory_model.resident_kv_bytes(lens, [], L, Lw, bpt) / memory_model.full_kv_bytes(lens, L, bpt)
        assert int(math.floor(100 * saving + 0.5)) == pct, name


# ---- watershed curve, forced rounds, coverage -----------------------------------------------------
def test_mean_kl_closed_forms_and_direction():
    P = np.array([[0.5, 0.5], [0.25, 0.75], [0.5, 0.5]])
    out = ra.mean_kl_to_later_layers(P)
    kl01 = 0.5 * math.log(4.0 / 3.0)                       # KL([1/2,1/2] || [1/4,3/4])
    kl12 = 0.25 * math.log(0.5) + 0.75 * math.log(1.5)     # KL([1/4,3/4] || [1/2,1/2]): the other direction
    assert abs(kl01 - 0.14384103622589045) < 1e-15 and abs(kl12 - 0.13081203594113694) < 1e-15
    assert np.allclose(out, [(kl01 + 0.0) / 2, kl12], rtol=1e-14, atol=0)
    # identical layers: zero; uniform target: ln R minus the entropy
    assert np.all(ra.mean_kl_to_later_layers(np.tile([0.2, 0.3, 0.5], (4, 1))) == 0.0)
    p = np.array([0.1, 0.2, 0.3, 0.4])
    H = -(p * np.log(p)).sum()
    assert abs(ra.mean_kl_to_later_layers(np.stack([p, np.full(4, 0.25)]))[0] - (math.log(4) - H)) < 1e-15
    # conventions at zero
    assert ra.mean_kl_to_later_layers(np.array([[0.0, 1.0], [0.5, 0.5]]))[0] == math.log(2.0)
    assert ra.mean_kl_to_later_layers(np.array([[0.5, 0.5], [0.0, 1.0]]))[0] == math.inf


def test_mean_kl_against_library_relative_entropy():
    from scipy.special import rel_entr
    rng = np.random.default_rng(11)
    P = rng.random((6, 37))
    P /= P.sum(axis=1, keepdims=True)
    want = [np.mean([rel_entr(P[l], P[m]).sum() for m in range(l + 1, 6)]) for l in range(5)]
    assert np.allclose(ra.mean_kl_to_later_layers(P), want, rtol=1e-12, atol=0)


def test_forced_rounds_join_the_rule_selection():
    S = [0.05, 0.30, 0.05, 0.05, 0.40, 0.05, 0.05, 0.05]
    base, info = ra.select_rounds(S, lam=1.0)
    assert base == [1, 4]
    sel, info2 = ra.select_rounds(S, lam=1.0, keep_first=1, keep_last=2)
    assert sel == [0, 1, 4, 6, 7] and info2["cut"] == info["cut"]      # the rule itself is unchanged
    assert ra.select_rounds(S, lam=1.0, keep_first=2)[0] == [0, 1, 4]  # a forced round that the rule kept anyway
    assert ra.select_rounds(S, lam=1.0, max_rounds=1, keep_last=1)[0] == [4, 7]   # the cap binds the rule only
    assert ra.select_rounds(S, lam=1.0, keep_first=5, keep_last=5)[0] == list(range(8))
    assert abs(ra.selection_coverage(S, [1, 4]) - 0.70) < 1e-15
    assert ra.selection_coverage(S, []) == 0.0


def test_answer_tokens_one_at_a_time_sum_to_eq1_right():
    """Eq. 1, right-hand form: the answer tokens' masses add up token by token.  Token t of the answer
    sees the history and the first c0 + t + 1 tokens of the current round; brute-force softmax per token."""
    rng = np.random.default_rng(5)
    Hq, Hkv, d, c0, T = 4, 2, 8, 3, 5
    lens = [4, 1, 6]
    k_rounds = [rng.standard_normal((n, Hkv, d)) for n in lens]
    cur = rng.standard_normal((c0 + T, Hkv, d))
    qa = rng.standard_normal((T, Hq, d))
    scale = 0.3
    P, S = ra.round_scores(qa, k_rounds, scale, cur)
    acc = np.zeros((Hq, len(lens)))
    for t in range(T):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            e_rounds = [sum(math.exp(scale * float(qa[t, h] @ k[j, g])) for j in range(k.shape[0])) for k in k_rounds]
            e_cur = sum(math.exp(scale * float(qa[t, h] @ cur[j, g])) for j in range(c0 + t + 1))
            z = sum(e_rounds) + e_cur
            acc[h] += np.array(e_rounds) / z
    assert np.allclose(P, acc / acc.sum(axis=1, keepdims=True), rtol=1e-12, atol=0)
    assert np.allclose(S, (acc / acc.sum(axis=1, keepdims=True)).mean(axis=0), rtol=1e-12, atol=0)


def test_select_scores_on_the_cut_and_one_ulp_beside_it_hand_values():
    """Strict inequality at the cut (Sec. 3.3 writes ">"), decided in double on fp32 scores: hand-derived selections
    for vectors whose mean / standard deviation are exact binary fractions."""
    from select_edge_cases import select_edge_cases
    n_hand = 0
    for scores, params, expected in select_edge_cases():
        got, _ = ra.select_rounds([float(np.float32(x)) for x in scores], **params)
        if expected is not None:
            assert got == expected, (scores, params)
            n_hand += 1
    assert n_hand >= 10


def test_row_error_hand_values():
    """row_error = max over rows of (largest absolute error of the row) / (largest magnitude of the row's reference):
    hand-worked, with the largest error of a row away from its largest entry, rows of different scale, a leading
    batch axis, and the uniform relative perturbation that must come back as itself."""
    ref = np.array([[1.0, -4.0, 2.0, 0.5], [0.1, 0.2, -0.05, 0.0]])
    out = ref.copy()
    out[0, 3] += 0.02       # row 0: 0.02 / 4 = 0.005, the error sits on the entry 0.5
    out[1, 0] -= 0.003      # row 1: 0.003 / 0.2 = 0.015
    assert ra.row_error(out, ref) == pytest.approx(0.015, rel=1e-12)
    out[1, 0] = ref[1, 0]
    assert ra.row_error(out, ref) == pytest.approx(0.005, rel=1e-12)
    # a wrong axis or a per-element denominator would give 0.02 / 0.5 or 0.003 / 0.1 instead
    assert ra.row_error(ref * (1 + 1e-3), ref) == pytest.approx(1e-3, rel=1e-9)
    # rows are the last axis, whatever lies in front: [token][head][channel]
    ref3 = np.stack([ref, 10 * ref])
    out3 = ref3.copy()
    out3[1, 0, 0] += 0.4    # 0.4 / 40
    out3[0, 1, 2] += 0.001  # 0.001 / 0.2
    assert ra.row_error(out3, ref3) == pytest.approx(0.01, rel=1e-12)
    assert ra.row_error(ref3, ref3) == 0.0


def test_large_entry_error_hand_values():
    """Elementwise relative error over the entries of at least 5 % of their row's largest magnitude."""
    ref = np.array([[1.0, -4.0, 2.0, 0.1], [0.1, 0.2, -0.05, 0.0]])
    out = ref.copy()
    out[0, 3] += 0.05       # 0.1 < 0.05 * 4: below the floor, ignored although its relative error is 50 %
    out[0, 2] += 0.004      # 0.004 / 2 = 0.002
    out[1, 2] += 0.001      # 0.05 >= 0.05 * 0.2: counted, 0.001 / 0.05 = 0.02
    assert ra.large_entry_error(out, ref) == pytest.approx(0.02, rel=1e-12)
    out[1, 2] = ref[1, 2]
    assert ra.large_entry_error(out, ref) == pytest.approx(0.002, rel=1e-12)
    assert ra.large_entry_error(out, ref, floor=0.01) == pytest.approx(0.5, rel=1e-12)
    assert ra.large_entry_error(np.ones((2, 3)), np.zeros((2, 3))) == 0.0
