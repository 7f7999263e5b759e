"""KV-cache residency accounting (TEST INFRASTRUCTURE), written out from Sec. 3.5.

Layers 1..L_w keep every round's KV on the GPU; layers L_w+1..L keep only the selected rounds.
Counting bytes round by round and layer by layer must reproduce Eq. 2,
M_round / M_orig = L_w/L + (K/T)(1 - L_w/L), when all T rounds have the same length.
"""
from __future__ import annotations

from typing import Sequence


def full_kv_bytes(lens: Sequence[int], L: int, bytes_per_token_layer: int) -> int:
    return sum(int(n) for n in lens) * L * bytes_per_token_layer


def resident_kv_bytes(lens: Sequence[int], sel: Sequence[int], L: int, L_w: int, bytes_per_token_layer: int) -> int:
    keep = set(int(r) for r in sel)
    total = 0
    for layer in range(1, L + 1):
        for r, n in enumerate(lens):
            if layer <= L_w or r in keep:
                total += int(n) * bytes_per_token_layer
    return total
