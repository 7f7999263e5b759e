"""Seeded synthetic dialogue-shaped workloads (round-segmented KV caches and queries).

The inputs stand in for the multi-round dialogues the paper evaluates on (tens to hundreds
of rounds of a few hundred tokens each, Sec. 4.1-4.2 and Table 1): the datasets themselves
are not used.  Everything is drawn on the host with numpy from a PCG64 stream seeded by the
integer list ``[2502, 15294, cfg_id, b, stream, layer, round]`` so that any (sequence, layer,
round) slice can be produced on its own, lazily, with identical bits for every consumer.

Streams: 0 round lengths, 1 choice of the "relevant" rounds, 2 queries, 3 history keys,
4 history values, 5 current-round keys, 6 current-round values, 7 paged block permutation.

No arithmetic of the method is in this module: values are drawn, a bias vector is added to
the keys of the seeded relevant rounds, and the result is rounded to the storage type.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import numpy as np

_SEED_PREFIX = (2502, 15294)

S_LEN, S_REL, S_Q, S_K, S_V, S_CURK, S_CURV, S_BLOCKS = range(8)


def _rng(cfg_id: int, b: int, stream: int, layer: int = 0, rnd: int = 0) -> np.random.Generator:
    return np.random.default_rng([*_SEED_PREFIX, cfg_id, b, stream, layer, rnd])


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) in integer arithmetic; returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bits to the float32 holding exactly the same value."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store_round(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round to the storage type and return the float32 array holding exactly the stored values."""
    if dtype == "bf16":
        return bf16_bits_to_f32(to_bf16_bits(x))
    return np.ascontiguousarray(x, dtype=np.float32)


def _draw_lengths(rng: np.random.Generator, R: int, spec: Tuple) -> np.ndarray:
    kind = spec[0]
    if R == 0:
        return np.zeros(0, dtype=np.int64)
    if kind == "fixed":
        return np.full(R, int(spec[1]), dtype=np.int64)
    if kind == "uniform":
        lo, hi = int(spec[1]), int(spec[2])
        return rng.integers(lo, hi + 1, size=R).astype(np.int64)
    if kind == "lognormal":
        median, sigma, total = float(spec[1]), float(spec[2]), int(spec[3])
        raw = np.exp(rng.normal(math.log(median), sigma, size=R))
        lens = np.maximum(1, np.rint(raw * (total / raw.sum()))).astype(np.int64)
        # put the rounding residual on the largest round so the total is exact
        lens[int(np.argmax(lens))] += total - int(lens.sum())
        assert lens.min() >= 1 and int(lens.sum()) == total
        return lens
    if kind == "list":
        return np.asarray(spec[1], dtype=np.int64)
    raise ValueError(f"unknown length spec {spec!r}")


# The five benchmark configurations.  `length` is the round-length recipe, `n_relevant` the
# number of seeded rounds whose keys are shifted towards the query by `alpha`.
CONFIGS: Dict[str, dict] = {
    "cfg1": dict(cfg_id=1, dtype="f32", B=1, Hq=4, Hkv=2, d=64, q_len=1, cur_len=0, R=8,
                 length=("fixed", 64), n_relevant=2, alpha=2.0, n_post_layers=1, block_size=0),
    "cfg2": dict(cfg_id=2, dtype="bf16", B=8, Hq=32, Hkv=8, d=128, q_len=1, cur_len=0, R=20,
                 length=("uniform", 200, 1000), n_relevant=3, alpha=2.0, n_post_layers=1, block_size=0),
    "cfg3": dict(cfg_id=3, dtype="bf16", B=4, Hq=32, Hkv=8, d=128, q_len=128, cur_len=128, R=60,
                 length=("lognormal", 400.0, 0.8, 32768), n_relevant=4, alpha=2.0, n_post_layers=1,
                 block_size=0),
    "cfg4": dict(cfg_id=4, dtype="bf16", B=16, Hq=32, Hkv=8, d=128, q_len=1, cur_len=0, R=200,
                 length=("lognormal", 400.0, 0.8, 131072), n_relevant=8, alpha=2.0, n_post_layers=24,
                 block_size=0),
    "cfg5": dict(cfg_id=5, dtype="bf16", B=64, Hq=64, Hkv=8, d=128, q_len=1, cur_len=0, R=50,
                 length=("uniform", 300, 1000), n_relevant=3, alpha=2.0, n_post_layers=1, block_size=16),
}


@dataclasses.dataclass
class Workload:
    """One synthetic batch.  Layer 0 is the watershed layer (only its keys are ever read);
    layers 1..n_post_layers are the post-watershed layers that run round-sparse attention."""

    name: str
    cfg_id: int
    dtype: str            # "f32" or "bf16": storage type of Q, K, V
    B: int
    Hq: int
    Hkv: int
    d: int
    q_len: int
    cur_len: int
    n_post_layers: int
    alpha: float
    block_size: int       # 0 = contiguous round segments, 16 = paged blocks
    lens: List[np.ndarray]        # per sequence: int64 [R_b]
    relevant: List[np.ndarray]    # per sequence: sorted round indices that carry the bias

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def R_max(self) -> int:
        return max([len(l) for l in self.lens] + [0])

    def n_rounds(self, b: int) -> int:
        return len(self.lens[b])

    def total_tokens(self, b: int) -> int:
        return int(self.lens[b].sum())

    # ---- queries -------------------------------------------------------------------
    def q(self, layer: int = 0) -> np.ndarray:
        """Queries of one layer, float32 [B, q_len, Hq, d], already rounded to the storage type."""
        out = np.empty((self.B, self.q_len, self.Hq, self.d), dtype=np.float32)
        for b in range(self.B):
            rng = _rng(self.cfg_id, b, S_Q, layer)
            out[b] = rng.standard_normal((self.q_len, self.Hq, self.d), dtype=np.float32)
        return _store_round(out, self.dtype)

    def _bias_dirs(self, b: int, layer: int) -> np.ndarray:
        """Per KV head: unit vector along the sum of that head group's queries, float32 [Hkv, d]."""
        rng = _rng(self.cfg_id, b, S_Q, layer)
        qb = _store_round(rng.standard_normal((self.q_len, self.Hq, self.d), dtype=np.float32), self.dtype)
        s = qb.reshape(self.q_len, self.Hkv, self.G, self.d).sum(axis=(0, 2), dtype=np.float32)
        n = np.sqrt((s.astype(np.float64) ** 2).sum(axis=1, keepdims=True)).astype(np.float32)
        return s / np.maximum(n, np.float32(1e-20))

    # ---- history K / V, one round at a time ------------------------------------------
    def k_round(self, b: int, layer: int, r: int) -> np.ndarray:
        """Keys of round r, float32 [len_r, Hkv, d] holding exactly the stored values."""
        n = int(self.lens[b][r])
        rng = _rng(self.cfg_id, b, S_K, layer, r)
        k = rng.standard_normal((n, self.Hkv, self.d), dtype=np.float32)
        if self.alpha != 0.0 and r in set(self.relevant[b].tolist()):
            k += np.float32(self.alpha) * self._bias_dirs(b, layer)[None, :, :]
        return _store_round(k, self.dtype)

    def v_round(self, b: int, layer: int, r: int) -> np.ndarray:
        n = int(self.lens[b][r])
        rng = _rng(self.cfg_id, b, S_V, layer, r)
        return _store_round(rng.standard_normal((n, self.Hkv, self.d), dtype=np.float32), self.dtype)

    # ---- current round (the question so far / the tokens generated so far) -----------
    def cur_k(self, layer: int) -> Optional[np.ndarray]:
        """float32 [B, cur_len, Hkv, d] or None when cur_len == 0."""
        return self._cur(layer, S_CURK)

    def cur_v(self, layer: int) -> Optional[np.ndarray]:
        return self._cur(layer, S_CURV)

    def _cur(self, layer: int, stream: int) -> Optional[np.ndarray]:
        if self.cur_len == 0:
            return None
        out = np.empty((self.B, self.cur_len, self.Hkv, self.d), dtype=np.float32)
        for b in range(self.B):
            rng = _rng(self.cfg_id, b, stream, layer)
            out[b] = rng.standard_normal((self.cur_len, self.Hkv, self.d), dtype=np.float32)
        return _store_round(out, self.dtype)

    def block_rng(self, layer: int) -> np.random.Generator:
        return _rng(self.cfg_id, 0, S_BLOCKS, layer)


def make_workload(name: str, **overrides) -> Workload:
    """Build a workload from a named configuration; keyword overrides replace its fields
    (e.g. ``B=2`` or ``length=("uniform", 20, 90)`` for a reduced-size variant, or
    ``lens=[...]`` to fix the round lengths of every sequence by hand)."""
    spec = dict(CONFIGS[name])
    lens_override = overrides.pop("lens", None)
    relevant_override = overrides.pop("relevant", None)
    spec.update(overrides)
    cfg_id, B, R = spec["cfg_id"], spec["B"], spec["R"]
    assert spec["Hq"] % spec["Hkv"] == 0
    lens, relevant = [], []
    for b in range(B):
        if lens_override is not None:
            lb = np.asarray(lens_override[b], dtype=np.int64)
        else:
            lb = _draw_lengths(_rng(cfg_id, b, S_LEN), R, spec["length"])
        lens.append(lb)
        if relevant_override is not None:
            rel = np.asarray(relevant_override[b], dtype=np.int64)
        else:
            n_rel = min(spec["n_relevant"], len(lb))
            rel = np.sort(_rng(cfg_id, b, S_REL).choice(len(lb), size=n_rel, replace=False)) if n_rel else \
                np.zeros(0, dtype=np.int64)
        relevant.append(rel.astype(np.int64))
    return Workload(name=name, cfg_id=cfg_id, dtype=spec["dtype"], B=B, Hq=spec["Hq"], Hkv=spec["Hkv"],
                    d=spec["d"], q_len=spec["q_len"], cur_len=spec["cur_len"],
                    n_post_layers=spec["n_post_layers"], alpha=float(spec["alpha"]),
                    block_size=spec["block_size"], lens=lens, relevant=relevant)
