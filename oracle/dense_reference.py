"""Independent dense attention used to pin the oracle (TEST INFRASTRUCTURE).

Textbook softmax(Q K^T / sqrt(d)) V over one concatenated cache, taken from a library routine
(`torch.nn.functional.scaled_dot_product_attention`, CPU, float64) rather than from the oracle's
own code, so that "selecting every round reproduces the original inference" (Sec. 3.5, the
K = T remark after Eq. 2) can be checked against something the oracle did not compute.
"""
from __future__ import annotations

import numpy as np
import torch


def dense_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float, causal_tail: bool = False
                    ) -> np.ndarray:
    """q [q_len, Hq, d], K/V [n, Hkv, d] -> O [q_len, Hq, d] (float64).

    With `causal_tail` the queries are the last q_len positions of the n keys and each sees only
    keys at or before its own position (lower-right aligned causal mask)."""
    qt = torch.from_numpy(np.asarray(q, dtype=np.float64)).permute(1, 0, 2)[None]      # [1, Hq, q_len, d]
    Hq = qt.shape[1]
    Hkv = K.shape[1]
    rep = Hq // Hkv
    kt = torch.from_numpy(np.asarray(K, dtype=np.float64)).permute(1, 0, 2).repeat_interleave(rep, dim=0)[None]
    vt = torch.from_numpy(np.asarray(V, dtype=np.float64)).permute(1, 0, 2).repeat_interleave(rep, dim=0)[None]
    mask = None
    if causal_tail:
        q_len, n = qt.shape[2], kt.shape[2]
        i = torch.arange(q_len)[:, None]
        j = torch.arange(n)[None, :]
        mask = j <= (n - q_len + i)
    out = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=scale)
    return out[0].permute(1, 0, 2).contiguous().numpy()
