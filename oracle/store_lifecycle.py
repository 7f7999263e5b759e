"""Life cycle of the per-round host tensors across dialogue turns (TEST INFRASTRUCTURE).

Plain models of the two bookkeeping steps the paper places around the hot path:

* End of a turn (Sec. 3.2, last step of the pipeline; Alg. 1, last line): the keys and values the
  post-watershed layers produced for the new round leave the GPU as ONE tensor per sequence and
  join the rounds kept in host memory.  `read_round_tensor` is the definition of that tensor's
  element order, written as the address of one element; the tests read a tensor written by the
  device library back through it, element by element.
* KV-cache dropping (Sec. 3.4): a round that was never among the selected ones is deleted instead
  of being kept.  `ActivityLedger` counts, per round, the turns it has been a candidate and the
  turns it was selected, and names the rounds with no selection so far.

Where the paper is silent: how many turns a round must have been a candidate before "never
active" is decided.  Reading taken: a threshold `min_turns` given by the caller; a round that has
been a candidate in at least `min_turns` selections and was chosen in none of them is inactive.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Sequence, Tuple

import numpy as np


def round_tensor_elems(n_layers: int, Hkv: int, d: int, n: int) -> int:
    """Elements of one round's host tensor: per layer n key rows and the value rows padded to a
    whole number of 16-token tiles."""
    return n_layers * (n + 16 * ((n + 15) // 16)) * Hkv * d


def key_address(layer: int, g: int, t: int, c: int, Hkv: int, d: int, n: int) -> int:
    """Index of K[layer][token t][kv head g][channel c] in the round tensor."""
    per_layer = (n + 16 * ((n + 15) // 16)) * Hkv * d
    return layer * per_layer + (g * n + t) * d + c


def value_address(layer: int, g: int, t: int, c: int, Hkv: int, d: int, n: int) -> int:
    """Index of V[layer][token t][kv head g][channel c]: after the layer's keys, head-major,
    tiles of 16 tokens, inside a tile channel-major with the 16 tokens of a channel adjacent."""
    tiles = (n + 15) // 16
    per_layer = (n + 16 * tiles) * Hkv * d
    return layer * per_layer + n * Hkv * d + ((g * tiles + t // 16) * d + c) * 16 + t % 16


def read_round_tensor(buf: np.ndarray, n_layers: int, Hkv: int, d: int, n: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Token-major K and V, each [n_layers][n][Hkv][d], read one element at a time, and the
    padding elements of the value tiles (which must be zero)."""
    assert buf.size == round_tensor_elems(n_layers, Hkv, d, n)
    K = np.empty((n_layers, n, Hkv, d), dtype=buf.dtype)
    V = np.empty((n_layers, n, Hkv, d), dtype=buf.dtype)
    pad: List = []
    tiles = (n + 15) // 16
    for layer in range(n_layers):
        for g in range(Hkv):
            for t in range(n):
                for c in range(d):
                    K[layer, t, g, c] = buf[key_address(layer, g, t, c, Hkv, d, n)]
                    V[layer, t, g, c] = buf[value_address(layer, g, t, c, Hkv, d, n)]
            for t in range(n, 16 * tiles):
                for c in range(d):
                    pad.append(buf[value_address(layer, g, t, c, Hkv, d, n)])
    return K, V, np.asarray(pad, dtype=buf.dtype)


class ActivityLedger:
    """Selection history of one sequence's rounds."""

    def __init__(self) -> None:
        self.turns: Dict[int, int] = {}   # round -> selections in which it was a candidate
        self.hits: Dict[int, int] = {}    # round -> selections in which it was chosen

    def add_round(self, r: int) -> None:
        self.turns[r] = 0
        self.hits[r] = 0

    def record_selection(self, selected: Iterable[int]) -> None:
        chosen = set(int(r) for r in selected)
        assert chosen <= set(self.turns), "selected a round that is not kept"
        for r in self.turns:
            self.turns[r] += 1
            if r in chosen:
                self.hits[r] += 1

    def inactive(self, min_turns: int) -> List[int]:
        return sorted(r for r in self.turns if self.turns[r] >= min_turns and self.hits[r] == 0)

    def drop(self, rounds: Sequence[int]) -> None:
        for r in rounds:
            del self.turns[r]
            del self.hits[r]
