"""Whole-path driver of the oracle over a synthetic workload (TEST INFRASTRUCTURE).

Runs, per sequence, the paper's order of steps (Sec. 3.2, steps 3-5): round scores at the
watershed layer -> round selection -> attention over the selected rounds at every
post-watershed layer.  The workload object only supplies arrays (queries, one round's keys
or values at a time); all arithmetic is in `oracle.round_attention`.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import round_attention as ra


@dataclasses.dataclass
class SeqResult:
    P: np.ndarray                 # [Hq, R] per-head round distribution
    S: np.ndarray                 # [R] head mean
    sel: List[int]                # ascending selected rounds
    info: dict                    # cut value and margin of the selection
    out: Dict[int, np.ndarray]    # layer -> O [q_len, Hq, d]
    lse: Dict[int, np.ndarray]    # layer -> lse [q_len, Hq]


def scores_for_sequence(w, b: int, use_cur: bool = True):
    q0 = w.q(0)[b]
    k_rounds = [w.k_round(b, 0, r) for r in range(w.n_rounds(b))]
    cur_k = w.cur_k(0)
    cur = cur_k[b] if (use_cur and cur_k is not None) else None
    return ra.round_scores(q0, k_rounds, w.scale, cur)


def attention_for_sequence(w, b: int, layer: int, sel: Sequence[int], heads: Optional[Sequence[int]] = None):
    """Sparse attention of one post-watershed layer; only the selected rounds are generated."""
    q = w.q(layer)[b]
    R = w.n_rounds(b)
    k_rounds: List[Optional[np.ndarray]] = [None] * R
    v_rounds: List[Optional[np.ndarray]] = [None] * R
    for r in sel:
        k_rounds[r] = w.k_round(b, layer, r)
        v_rounds[r] = w.v_round(b, layer, r)
    ck, cv = w.cur_k(layer), w.cur_v(layer)
    return ra.sparse_attention(q, k_rounds, v_rounds, sel, w.scale,
                               None if ck is None else ck[b], None if cv is None else cv[b])


def run_sequence(w, b: int, select_params: Optional[dict] = None, layers: Optional[Sequence[int]] = None
                 ) -> SeqResult:
    params = dict(select_params or {})
    P, S = scores_for_sequence(w, b)
    sel, info = ra.select_rounds(S, **params)
    out, lse = {}, {}
    for layer in (layers if layers is not None else range(1, w.n_post_layers + 1)):
        out[layer], lse[layer] = attention_for_sequence(w, b, layer, sel)
    return SeqResult(P=P, S=S, sel=sel, info=info, out=out, lse=lse)


def run(w, select_params: Optional[dict] = None, layers: Optional[Sequence[int]] = None,
        seqs: Optional[Sequence[int]] = None) -> List[SeqResult]:
    return [run_sequence(w, b, select_params, layers) for b in (seqs if seqs is not None else range(w.B))]
