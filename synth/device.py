"""Glue used by the GPU tests, the smoke check and the benchmark: moves a synthetic workload's
packed buffers to the device and wraps them in the binding's view objects.  No arithmetic.

Not imported by `synth/__init__`: the generators themselves stay independent of the HIP binding."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

import paper_2502_15294_amd as ra
from .layout import PackedLayer, pack_layer
from .workloads import Workload, to_bf16_bits


def to_device(x: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """float32 values (already exactly representable in `dtype`) -> device tensor of that dtype."""
    if dtype == "bf16":
        bits = to_bf16_bits(x).reshape(x.shape)
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)


def raw_to_device(buf: np.ndarray, device="cuda") -> torch.Tensor:
    if buf.size == 0:  # an empty cache still needs a valid (never dereferenced) device pointer
        buf = np.zeros(256, dtype=buf.dtype)
    if buf.dtype == np.uint16:
        return torch.from_numpy(buf.view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(buf).to(device)


def view_from_packed(p: PackedLayer, Hkv: int, d: int, device="cuda") -> ra.KVView:
    k = raw_to_device(p.k, device)
    v = raw_to_device(p.v, device) if p.v is not None else None
    bt = torch.from_numpy(p.block_table).to(device) if p.block_table is not None else None
    return ra.KVView(k, v, torch.from_numpy(p.seg_off).to(device), torch.from_numpy(p.seg_len).to(device),
                     torch.from_numpy(p.n_rounds).to(device), Hkv, d, p.max_tokens, block_table=bt,
                     block_size=p.block_size,
                     seg_off_v=None if p.seg_off_v is None else torch.from_numpy(p.seg_off_v).to(device))


def device_view(w: Workload, layer: int, with_v: bool = True, block_size: Optional[int] = None, threads: int = 8,
                device="cuda") -> ra.KVView:
    return view_from_packed(pack_layer(w, layer, with_v=with_v, block_size=block_size, threads=threads), w.Hkv, w.d,
                            device)


class Engine:
    """A context plus a workspace tensor sized for one workload."""

    def __init__(self, w: Workload, device: int = 0, extra_tokens: int = 0):
        self.ctx = ra.ra_create(device)
        max_tokens = max([w.total_tokens(b) for b in range(w.B)] + [0]) + w.cur_len + extra_tokens
        nbytes = ra.ra_workspace_bytes(w.B, max(w.R_max, 1), w.Hq, w.Hkv, w.d, max(w.q_len, 1),
                                       ra.RA_BF16 if w.dtype == "bf16" else ra.RA_F32, max_tokens)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=f"cuda:{device}")
        ra.ra_set_workspace(self.ctx, self.workspace)

    def close(self):
        if self.ctx is not None:
            ra.ra_destroy(self.ctx)
            self.ctx = None


def sel_to_device(sels, R_max: int, device="cuda"):
    """List of per-sequence index lists -> (sel_idx [B, R_max] padded with -1, n_sel [B])."""
    B = len(sels)
    idx = np.full((B, max(R_max, 1)), -1, dtype=np.int32)
    n = np.zeros(B, dtype=np.int32)
    for b, s in enumerate(sels):
        idx[b, :len(s)] = s
        n[b] = len(s)
    return torch.from_numpy(idx).to(device), torch.from_numpy(n).to(device)
