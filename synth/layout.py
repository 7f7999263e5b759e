"""Packing of round segments into the flat buffers the device library reads.

Two layouts, both round-indexed:

Keys are stored token-major (one row of d channels per token); values are stored transposed in
tiles of 16 tokens, ``[d][16]`` per tile, the last tile of a round zero-padded, so that a lane of
the matrix-core kernels reads several consecutive tokens of one channel with a single load.

contiguous (block_size == 0)
    Keys of round r of sequence b: one block of ``Hkv * len * d`` elements, ``[Hkv][len][d]``;
    ``seg_off[b, r]`` is its start in units of tokens:
    K(g, t, c) = ``(seg_off * Hkv + g * len + t) * d + c``.
    Values: one block of ``Hkv * L16 * d`` elements, ``[Hkv][L16 / 16][d][16]`` with
    ``L16 = 16 * ceil(len / 16)``; ``seg_off_v[b, r]`` is its start in units of (padded) tokens:
    V(g, t, c) = ``(seg_off_v * Hkv + g * L16 + (t // 16) * 16) * d + c * 16 + t % 16``.

paged (block_size == 16)
    Storage is an array of physical blocks, ``[n_blocks][Hkv][16][d]`` for keys and
    ``[n_blocks][Hkv][d][16]`` for values.  A round starts on a block boundary and owns
    ``ceil(len / 16)`` consecutive slots of its sequence's row of the block table.
    ``seg_off[b, r]`` is the round's first slot; with ``blk = block_table[b, seg_off + t // 16]``:
    K(g, t, c) = ``((blk * Hkv + g) * 16 + t % 16) * d + c``,
    V(g, t, c) = ``((blk * Hkv + g) * d + c) * 16 + t % 16``.

Pure data movement: nothing here computes anything of the method.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Optional

import numpy as np

from .workloads import Workload, to_bf16_bits


@dataclasses.dataclass
class PackedLayer:
    k: np.ndarray                       # flat; uint16 (bf16 bits) or float32
    v: Optional[np.ndarray]             # same shape as k, or None when only keys were packed
    seg_off: np.ndarray                 # int64 [B, R_max]
    seg_off_v: Optional[np.ndarray]     # int64 [B, R_max] for the values (contiguous layout) or None
    seg_len: np.ndarray                 # int32 [B, R_max]
    n_rounds: np.ndarray                # int32 [B]
    block_table: Optional[np.ndarray]   # int32 [B, max_blocks] (paged) or None
    block_size: int
    max_tokens: int                     # max over sequences of the total history tokens


def _encode(x: np.ndarray, dtype: str) -> np.ndarray:
    return to_bf16_bits(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def _packed(**kw) -> "PackedLayer":
    return PackedLayer(**kw)


def round_host_elems(w: Workload, n: int, n_layers: int) -> int:
    """Elements of one round's host tensor: per layer, keys [Hkv][len][d] then values
    [Hkv][ceil(len/16)][d][16]."""
    return n_layers * (n + 16 * (-(-n // 16))) * w.Hkv * w.d


def pack_round_host(w: Workload, b: int, r: int, layers, out: Optional[np.ndarray] = None) -> np.ndarray:
    """One round's post-watershed KV as the monolithic host tensor the KV store registers:
    for each layer in `layers`, keys head-major then values in transposed, zero-padded 16-token tiles."""
    n = int(w.lens[b][r])
    nb = -(-n // 16)
    Hkv, d = w.Hkv, w.d
    el = np.uint16 if w.dtype == "bf16" else np.float32
    per_layer = (n + nb * 16) * Hkv * d
    buf = out if out is not None else np.zeros(len(layers) * per_layer, dtype=el)
    assert buf.size == len(layers) * per_layer
    for i, layer in enumerate(layers):
        base = i * per_layer
        buf[base:base + n * Hkv * d] = _encode(w.k_round(b, layer, r).transpose(1, 0, 2), w.dtype).reshape(-1)
        pad = np.zeros((nb * 16, Hkv, d), dtype=el)
        pad[:n] = _encode(w.v_round(b, layer, r), w.dtype)
        buf[base + n * Hkv * d:base + per_layer] = pad.reshape(nb, 16, Hkv, d).transpose(2, 0, 3, 1).reshape(-1)
    return buf


def pack_layer(w: Workload, layer: int, with_v: bool = True, block_size: Optional[int] = None,
               threads: int = 8, seq_range: Optional[range] = None) -> PackedLayer:
    """Generate one layer's history K (and V) for every sequence and pack it for the device."""
    bs = w.block_size if block_size is None else block_size
    assert bs in (0, 16)
    B, R_max, Hkv, d = w.B, w.R_max, w.Hkv, w.d
    R_alloc = max(R_max, 1)
    seg_off = np.zeros((B, R_alloc), dtype=np.int64)
    seg_off_v = np.zeros((B, R_alloc), dtype=np.int64)
    seg_len = np.zeros((B, R_alloc), dtype=np.int32)
    n_rounds = np.array([w.n_rounds(b) for b in range(B)], dtype=np.int32)
    el = np.uint16 if w.dtype == "bf16" else np.float32
    seqs = range(B) if seq_range is None else seq_range

    jobs = []
    if bs == 0:
        tok = tok_v = 0
        for b in range(B):
            for r in range(w.n_rounds(b)):
                n = int(w.lens[b][r])
                seg_off[b, r], seg_off_v[b, r], seg_len[b, r] = tok, tok_v, n
                if b in seqs:
                    jobs.append((b, r, tok, tok_v, n))
                tok += n
                tok_v += 16 * (-(-n // 16))
        k = np.zeros(tok * Hkv * d, dtype=el)
        v = np.zeros(tok_v * Hkv * d, dtype=el) if with_v else None
        block_table = None

        def fill(job):
            b, r, off, off_v, n = job
            if n == 0:
                return
            lo, hi = off * Hkv * d, (off + n) * Hkv * d
            k[lo:hi] = _encode(w.k_round(b, layer, r).transpose(1, 0, 2), w.dtype).reshape(-1)
            if with_v:
                nb = -(-n // 16)
                pad = np.zeros((nb * 16, Hkv, d), dtype=el)
                pad[:n] = _encode(w.v_round(b, layer, r), w.dtype)
                # [nb, 16, Hkv, d] -> [Hkv, nb, d, 16]
                lo, hi = off_v * Hkv * d, (off_v + nb * 16) * Hkv * d
                v[lo:hi] = pad.reshape(nb, 16, Hkv, d).transpose(2, 0, 3, 1).reshape(-1)
    else:
        slots = [int(sum(-(-int(n) // bs) for n in w.lens[b])) for b in range(B)]
        max_blocks = max(slots + [1])
        n_blocks = int(sum(slots))
        perm = w.block_rng(layer).permutation(max(n_blocks, 1)).astype(np.int32)
        block_table = np.full((B, max_blocks), -1, dtype=np.int32)
        nxt = 0
        for b in range(B):
            slot = 0
            for r in range(w.n_rounds(b)):
                n = int(w.lens[b][r])
                nb = -(-n // bs)
                seg_off[b, r], seg_len[b, r] = slot, n
                block_table[b, slot:slot + nb] = perm[nxt:nxt + nb]
                if b in seqs:
                    jobs.append((b, r, slot, n))
                slot += nb
                nxt += nb
        k = np.zeros(max(n_blocks, 1) * Hkv * bs * d, dtype=el)
        v = np.zeros(max(n_blocks, 1) * Hkv * bs * d, dtype=el) if with_v else None
        k4 = k.reshape(-1, Hkv, bs, d)
        v4 = v.reshape(-1, Hkv, d, bs) if with_v else None

        def fill(job):
            b, r, slot, n = job
            if n == 0:
                return
            nb = -(-n // bs)
            blocks = block_table[b, slot:slot + nb]

            def scatter(dst, src, perm):  # src [len, Hkv, d] -> padded [nb, bs, Hkv, d] -> permuted blocks
                pad = np.zeros((nb * bs, Hkv, d), dtype=el)
                pad[:n] = _encode(src, w.dtype)
                dst[blocks] = pad.reshape(nb, bs, Hkv, d).transpose(*perm)

            scatter(k4, w.k_round(b, layer, r), (0, 2, 1, 3))      # [nb, Hkv, 16, d]
            if with_v:
                scatter(v4, w.v_round(b, layer, r), (0, 2, 3, 1))  # [nb, Hkv, d, 16]

    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    max_tokens = max([w.total_tokens(b) for b in range(B)] + [0])
    return _packed(k=k, v=v, seg_off=seg_off, seg_off_v=seg_off_v if bs == 0 else None, seg_len=seg_len,
                       n_rounds=n_rounds,
                       block_table=block_table, block_size=bs, max_tokens=max_tokens)
