"""CPU oracle for the Round Attention hot path.  TEST INFRASTRUCTURE, not product code.

Plain, slow, float64 numpy written from the paper's definitions.  It shares no code with the
HIP library and must never be imported by the product path: only tests, the smoke check and
the benchmark's `cpu_baseline` leg call it.

What follows the paper and what is a reading of it:

* attention probabilities  Att(Q, K) = softmax(Q K^T / sqrt(d_k))        -- Sec. 3.1
* round mass  qAtt_k = sum over query tokens i and tokens j of round k of Att(Q_i, K_j)
                                                                          -- Sec. 3.1, Eq. 1
* P = qAtt normalised to a distribution over the history rounds           -- Sec. 3.1 (text after Eq. 1)
* three selection rules: score > v (v = 0.1); top 10 % of rounds; score > mean + lambda * std
                                                                          -- Sec. 3.3, strategies 1-3
* layers after the watershed attend only over the selected rounds         -- Sec. 3.2 steps 3-5, Sec. 3.5

Readings where the paper is silent (each is listed in the design notes too):
  - grouped-query attention: query head h reads KV head h // (Hq / Hkv);
  - Eq. 1 carries no head index: every query head is normalised on its own and the
    per-sequence score is the arithmetic mean over query heads;
  - the softmax of Eq. 1 runs over history tokens plus, when given, the current round's own
    keys under a causal mask aligned to the end of the current round; the current round is
    never a candidate;
  - std is the population one by default (ddof = 0), the inequality is strict, the multiplier
    of strategy 3 (not given in the paper) defaults to 1, top-10 % means ceil(p * R) rounds,
    ties go to the lower round index, the index list is ascending, and at least `min_rounds`
    rounds are kept.

Parity unpinned (no value in the paper fixes them): the default lambda = 1 and ddof = 0.
The two error measures at the end of the file (row_error, large_entry_error) are pinned by hand values.

Shapes, per sequence: q [q_len, Hq, d]; a round's keys/values [len_r, Hkv, d];
cur_k / cur_v [cur_len, Hkv, d].
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

ADAPTIVE, TOP_FRACTION, THRESHOLD = 0, 1, 2


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def _cur_visible(q_len: int, cur_len: int) -> np.ndarray:
    """Causal mask inside the current round, aligned to its end: query i (0-based, the last
    q_len tokens of the current round) sees current-round token j iff j <= cur_len - q_len + i.
    Returns bool [q_len, cur_len]."""
    i = np.arange(q_len)[:, None]
    j = np.arange(cur_len)[None, :]
    return j <= (cur_len - q_len + i)


def logits(q: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """scale * Q K^T per query head (Sec. 3.1).  q [q_len, Hq, d], k [n, Hkv, d] -> [Hq, q_len, n]."""
    q, k = _f64(q), _f64(k)
    q_len, Hq, d = q.shape
    n, Hkv, _ = k.shape
    G = Hq // Hkv
    out = np.empty((Hq, q_len, n), dtype=np.float64)
    for h in range(Hq):
        out[h] = scale * (q[:, h, :] @ k[:, h // G, :].T)
    return out


def attention_probabilities(q, k_rounds: Sequence[np.ndarray], scale: float,
                            cur_k: Optional[np.ndarray] = None) -> Tuple[np.ndarray, List[Tuple[int, int]]]:
    """Softmax rows over all history tokens (rounds concatenated in order) followed by the
    visible current-round tokens.  Returns p [Hq, q_len, T + cur_len] and the (start, end)
    column span of every history round."""
    q = _f64(q)
    q_len, Hq, d = q.shape
    parts = [_f64(k) for k in k_rounds]
    spans, pos = [], 0
    for k in parts:
        spans.append((pos, pos + k.shape[0]))
        pos += k.shape[0]
    cur_len = 0 if cur_k is None else cur_k.shape[0]
    if cur_len:
        parts.append(_f64(cur_k))
    if not parts or sum(p.shape[0] for p in parts) == 0:
        raise ValueError("softmax over an empty key set is undefined")
    K = np.concatenate(parts, axis=0)
    s = logits(q, K, scale)
    if cur_len:
        vis = _cur_visible(q_len, cur_len)
        s[:, :, pos:] = np.where(vis[None, :, :], s[:, :, pos:], -np.inf)
    m = s.max(axis=2, keepdims=True)
    e = np.exp(s - m)
    p = e / e.sum(axis=2, keepdims=True)
    return p, spans


def round_scores(q, k_rounds: Sequence[np.ndarray], scale: float,
                 cur_k: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Per-head round distribution P [Hq, R] (Eq. 1 then normalisation) and its head mean S [R]."""
    R = len(k_rounds)
    q = _f64(q)
    Hq = q.shape[1]
    if R == 0:
        return np.zeros((Hq, 0)), np.zeros(0)
    if sum(k.shape[0] for k in k_rounds) == 0:
        return np.zeros((Hq, R)), np.zeros(R)
    p, spans = attention_probabilities(q, k_rounds, scale, cur_k)
    qatt = np.zeros((Hq, R), dtype=np.float64)
    for r, (lo, hi) in enumerate(spans):
        qatt[:, r] = p[:, :, lo:hi].sum(axis=(1, 2))        # sum over query tokens i and tokens j of round r
    P = qatt / qatt.sum(axis=1, keepdims=True)
    S = P.sum(axis=0) / Hq
    return P, S


def select_rounds(S: Sequence[float], strategy: int = ADAPTIVE, lam: float = 1.0, fraction: float = 0.10,
                  threshold: float = 0.10, ddof: int = 0, min_rounds: int = 1, max_rounds: int = 0,
                  keep_first: int = 0, keep_last: int = 0) -> Tuple[List[int], dict]:
    """Round selection (Sec. 3.3).  Plain Python floats (IEEE double), sums taken sequentially in
    round order, two passes for the variance.  Returns the ascending index list and a dict with
    the cut value and the relative distance of the closest score to it.

    keep_first / keep_last are not in the paper: an optional policy that always keeps the first
    and the most recent rounds.  The rule (statistics, min_rounds, max_rounds) is applied to all
    rounds exactly as without them; the forced rounds are then added to what the rule kept."""
    S = [float(x) for x in S]
    R = len(S)
    if R == 0:
        return [], {"cut": None, "margin": None, "n_pass": 0}
    # order of preference: higher score first, then lower round index
    order = sorted(range(R), key=lambda r: (-S[r], r))
    cut = None
    if strategy == ADAPTIVE:
        total = 0.0
        for x in S:
            total += x
        mean = total / R
        ss = 0.0
        for x in S:
            dev = x - mean
            ss += dev * dev
        den = R - ddof
        std = math.sqrt(ss / den) if den > 0 else 0.0
        cut = mean + lam * std
        n_keep = sum(1 for x in S if x > cut)
    elif strategy == THRESHOLD:
        cut = float(threshold)
        n_keep = sum(1 for x in S if x > cut)
    elif strategy == TOP_FRACTION:
        n_keep = max(1, math.ceil(fraction * R))
    else:
        raise ValueError("unknown strategy")
    n_pass = n_keep
    n_keep = max(n_keep, min_rounds)
    if max_rounds > 0:
        n_keep = min(n_keep, max_rounds)
    n_keep = min(n_keep, R)
    forced = [r for r in range(R) if r < keep_first or r >= R - keep_last]
    sel = sorted(set(order[:n_keep]) | set(forced))
    margin = None
    if cut is not None and cut != 0.0:
        margin = min(abs(x - cut) for x in S) / abs(cut)
    elif strategy == TOP_FRACTION and 0 < n_keep < R:
        a, b = S[order[n_keep - 1]], S[order[n_keep]]
        margin = (a - b) / a if a != 0.0 else 0.0
    return sel, {"cut": cut, "margin": margin, "n_pass": n_pass}


def mean_kl_to_later_layers(P) -> np.ndarray:
    """Curve that locates the watershed layer (Sec. 3.1, Observation 2; Fig. 2b).  P [L][R] holds one
    round distribution per layer; entry l of the result (l = 0 .. L-2) is the mean over the later
    layers l' > l of KL(P^l || P^l') = sum_r P^l_r ln(P^l_r / P^l'_r), natural logarithm, with the
    usual conventions: a term with P^l_r = 0 is 0, a term with P^l_r > 0 = P^l'_r is +inf."""
    P = _f64(P)
    L, R = P.shape
    out = np.zeros(max(L - 1, 0))
    for l in range(L - 1):
        total = 0.0
        for l2 in range(l + 1, L):
            kl = 0.0
            for r in range(R):
                p, q = float(P[l, r]), float(P[l2, r])
                if p > 0.0:
                    kl += math.inf if q <= 0.0 else p * math.log(p / q)
            total += kl
        out[l] = total / (L - 1 - l)
    return out


def selection_coverage(S: Sequence[float], sel: Sequence[int]) -> float:
    """Share of a round distribution that falls on the selected rounds (drift monitor for a long
    answer: S is the distribution of the answer tokens so far, Eq. 1 right-hand form)."""
    total = 0.0
    for r in sorted(int(x) for x in sel):
        total += float(S[r])
    return total


def sparse_attention(q, k_rounds: Sequence[np.ndarray], v_rounds: Sequence[np.ndarray], sel: Sequence[int],
                     scale: float, cur_k: Optional[np.ndarray] = None, cur_v: Optional[np.ndarray] = None
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """Attention of the queries over the tokens of the selected rounds plus the visible tokens of
    the current round (Sec. 3.2 steps 4-5).  Returns O [q_len, Hq, d] and the natural-log
    normaliser lse [q_len, Hq] of the scaled logits."""
    q = _f64(q)
    q_len, Hq, d = q.shape
    ks = [_f64(k_rounds[r]) for r in sel]
    vs = [_f64(v_rounds[r]) for r in sel]
    n_hist = sum(k.shape[0] for k in ks)
    cur_len = 0 if cur_k is None else cur_k.shape[0]
    if cur_len:
        ks.append(_f64(cur_k))
        vs.append(_f64(cur_v))
    if n_hist + cur_len == 0:
        raise ValueError("attention over an empty key set is undefined")
    K = np.concatenate(ks, axis=0)
    V = np.concatenate(vs, axis=0)
    Hkv = K.shape[1]
    G = Hq // Hkv
    s = logits(q, K, scale)
    if cur_len:
        vis = _cur_visible(q_len, cur_len)
        s[:, :, n_hist:] = np.where(vis[None, :, :], s[:, :, n_hist:], -np.inf)
    m = s.max(axis=2, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=2, keepdims=True)
    p = e / z
    O = np.empty((q_len, Hq, d), dtype=np.float64)
    for h in range(Hq):
        O[:, h, :] = p[h] @ V[:, h // G, :]
    lse = (m[:, :, 0] + np.log(z[:, :, 0])).T
    return O, lse


def row_error(out, ref) -> float:
    """Error measure used for attention outputs: max over rows (one row = the d outputs of one
    (token, head)) of max|out - ref| / max|ref|."""
    out, ref = _f64(out), _f64(ref)
    num = np.abs(out - ref).max(axis=-1)
    den = np.abs(ref).max(axis=-1)
    return float((num / den).max())


def large_entry_error(out, ref, floor: float = 0.05) -> float:
    """Second error measure: the largest elementwise relative error |out - ref| / |ref| over the entries whose
    reference value is at least `floor` times the largest magnitude of their row (entries near zero, where a
    relative error says nothing, are left out).  0.0 if no entry qualifies."""
    out, ref = _f64(out), _f64(ref)
    big = np.abs(ref) >= floor * np.abs(ref).max(axis=-1, keepdims=True)
    big &= ref != 0.0
    if not big.any():
        return 0.0
    return float((np.abs(out - ref)[big] / np.abs(ref)[big]).max())
