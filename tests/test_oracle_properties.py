"""Property tests of the oracle over drawn inputs (hypothesis): structural facts of Eq. 1, of the selection rule and
of the divergence curve that hold for any input, beside the fixed pins."""
import math

import numpy as np
from hypothesis import given, settings
from hypothesis import strategies as st

from oracle import round_attention as ra
from oracle import store_lifecycle as sl

SETTINGS = dict(max_examples=60, deadline=None)


def _rounds(rng, lens, Hkv, d):
    return [rng.standard_normal((n, Hkv, d)) for n in lens]


@settings(**SETTINGS)
@given(seed=st.integers(0, 10_000), lens=st.lists(st.integers(1, 9), min_size=2, max_size=6),
       q_len=st.integers(1, 3), cut=st.integers(0, 4))
def test_round_mass_is_additive_under_merging_two_adjacent_rounds(seed, lens, q_len, cut):
    """Eq. 1 sums attention over the tokens of a round, so joining rounds r and r+1 into one round gives it the sum
    of their two scores and leaves every other round's score alone."""
    rng = np.random.default_rng(seed)
    Hq, Hkv, d = 4, 2, 8
    r = cut % (len(lens) - 1)
    ks = _rounds(rng, lens, Hkv, d)
    q = rng.standard_normal((q_len, Hq, d))
    cur = rng.standard_normal((q_len + 2, Hkv, d))
    P, S = ra.round_scores(q, ks, 0.3, cur)
    merged = ks[:r] + [np.concatenate([ks[r], ks[r + 1]])] + ks[r + 2:]
    Pm, Sm = ra.round_scores(q, merged, 0.3, cur)
    want = np.concatenate([P[:, :r], P[:, r:r + 1] + P[:, r + 1:r + 2], P[:, r + 2:]], axis=1)
    assert np.allclose(Pm, want, rtol=1e-11, atol=1e-14)
    assert np.allclose(P.sum(axis=1), 1.0, rtol=1e-12) and abs(S.sum() - 1.0) < 1e-12


@settings(**SETTINGS)
@given(scores=st.lists(st.floats(0.0, 1.0, allow_nan=False), min_size=1, max_size=40),
       lam=st.floats(-1.0, 3.0), min_rounds=st.integers(0, 3), max_rounds=st.integers(0, 5),
       keep_first=st.integers(0, 2), keep_last=st.integers(0, 2))
def test_adaptive_selection_is_what_the_rule_says(scores, lam, min_rounds, max_rounds, keep_first, keep_last):
    R = len(scores)
    sel, info = ra.select_rounds(scores, lam=lam, min_rounds=min_rounds, max_rounds=max_rounds,
                                 keep_first=keep_first, keep_last=keep_last)
    assert sel == sorted(set(sel)) and all(0 <= r < R for r in sel)
    forced = {r for r in range(R) if r < keep_first or r >= R - keep_last}
    assert forced <= set(sel)
    ruled = [r for r in sel if r not in forced]
    above = [r for r in range(R) if scores[r] > info["cut"]]
    n_rule = min(max(len(above), min_rounds), R)
    if max_rounds:
        n_rule = min(n_rule, max_rounds)
    # what the rule kept (before the forced rounds were added) are the n_rule best: no unkept round beats a kept one
    kept_by_rule = sorted(range(R), key=lambda r: (-scores[r], r))[:n_rule]
    assert set(sel) == set(kept_by_rule) | forced
    assert all(r in kept_by_rule for r in ruled)
    if not max_rounds and min_rounds <= len(above):
        assert set(above) <= set(sel)


@settings(**SETTINGS)
@given(scores=st.lists(st.floats(1e-6, 1.0), min_size=2, max_size=30), lam=st.floats(0.0, 2.0),
       factor=st.sampled_from([0.25, 0.5, 2.0, 8.0]))
def test_adaptive_and_top_fraction_do_not_depend_on_the_scale_of_the_scores(scores, lam, factor):
    """mean + lambda * std scales with the scores (powers of two keep the arithmetic exact), so the kept set cannot
    change; the fixed threshold of strategy 1 is the one rule that does depend on the scale."""
    scaled = [x * factor for x in scores]
    assert ra.select_rounds(scores, lam=lam)[0] == ra.select_rounds(scaled, lam=lam)[0]
    top = lambda x: ra.select_rounds(x, strategy=ra.TOP_FRACTION, fraction=0.3)[0]
    assert top(scores) == top(scaled)


@settings(**SETTINGS)
@given(seed=st.integers(0, 10_000), L=st.integers(2, 6), R=st.integers(1, 12))
def test_divergence_curve_is_nonnegative_and_zero_only_for_equal_layers(seed, L, R):
    rng = np.random.default_rng(seed)
    P = rng.random((L, R)) + 1e-3
    P /= P.sum(axis=1, keepdims=True)
    out = ra.mean_kl_to_later_layers(P)
    assert out.shape == (L - 1,) and (out >= -1e-15).all()                 # Gibbs' inequality
    same = np.tile(P[0], (L, 1))
    assert np.all(ra.mean_kl_to_later_layers(same) == 0.0)
    if R > 1:
        assert out[-1] > 0.0 or np.allclose(P[-2], P[-1])


@settings(**SETTINGS)
@given(seed=st.integers(0, 10_000), n_rounds=st.integers(1, 8), n_turns=st.integers(1, 6))
def test_ledger_counts(seed, n_rounds, n_turns):
    rng = np.random.default_rng(seed)
    led = sl.ActivityLedger()
    for r in range(n_rounds):
        led.add_round(r)
    chosen_ever = set()
    for _ in range(n_turns):
        pick = [r for r in range(n_rounds) if rng.random() < 0.4]
        led.record_selection(pick)
        chosen_ever |= set(pick)
    assert all(led.turns[r] == n_turns and 0 <= led.hits[r] <= n_turns for r in range(n_rounds))
    assert led.inactive(n_turns) == sorted(set(range(n_rounds)) - chosen_ever)
    assert led.inactive(n_turns + 1) == []


def test_select_all_weights_reassemble_attention_from_round_outputs():
    """O over a set of rounds = sum over the rounds of (round's share of the softmax mass) x (attention over that round
    alone): ties the score definition (Eq. 1) to the attention the later layers compute, for a drawn case."""
    rng = np.random.default_rng(3)
    Hq, Hkv, d, lens = 4, 2, 8, [5, 1, 7, 3]
    ks, vs = _rounds(rng, lens, Hkv, d), _rounds(rng, lens, Hkv, d)
    q = rng.standard_normal((1, Hq, d))
    P, _ = ra.round_scores(q, ks, 0.25)
    O, _ = ra.sparse_attention(q, ks, vs, [0, 1, 2, 3], 0.25)
    parts = [ra.sparse_attention(q, ks, vs, [r], 0.25)[0] for r in range(4)]
    want = sum(P[:, r][None, :, None] * parts[r] for r in range(4))
    assert np.allclose(O, want, rtol=1e-11, atol=1e-14)
    assert math.isclose(float(P.sum()), Hq, rel_tol=1e-12)
