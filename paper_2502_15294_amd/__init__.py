"""Python binding of libround_attention (HIP, gfx950): argument marshalling only.

Every function below has the name of the C entry point it forwards to (see
include/round_attention.h) and does nothing but turn torch tensors into device pointers,
fill the C structs and check the returned status.  PyTorch supplies device memory and
streams; all computation happens in the library's kernels.  There is no fallback: if the
shared library has not been built, importing `lib()` users fail with an ImportError.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# RA_LIBRARY overrides the path (e.g. to load an instrumented build of the same sources)
LIB_PATH = os.environ.get("RA_LIBRARY") or os.path.join(_HERE, "libround_attention.so")

RA_F32, RA_BF16 = 0, 1
RA_SEL_ADAPTIVE, RA_SEL_TOP_FRACTION, RA_SEL_THRESHOLD = 0, 1, 2
RA_STAGE_ROUND_MAJOR, RA_STAGE_LAYER_MAJOR, RA_STAGE_GROUPED = 0, 1, 2
RA_PREFILL_P_BF16X2, RA_PREFILL_P_F16 = 0, 1
RA_OK, RA_ERR_INVALID_ARG, RA_ERR_UNSUPPORTED, RA_ERR_WORKSPACE, RA_ERR_STATE, RA_ERR_OOM, RA_ERR_HIP = \
    0, -1, -2, -3, -4, -5, -6

EXPORTS = [
    "ra_last_error", "ra_create", "ra_destroy", "ra_workspace_bytes", "ra_set_workspace",
    "ra_profile_kernels", "ra_profile_last_ms", "ra_set_prefill_precision",
    "ra_round_scores", "ra_round_scores_select", "ra_select_rounds", "ra_round_sparse_attn_decode", "ra_round_sparse_attn_decode_noalloc",
    "ra_watershed_attn_decode",
    "ra_round_sparse_attn_prefill", "ra_watershed_attn_prefill",
    "ra_kv_store_create", "ra_kv_store_destroy", "ra_kv_store_register_round", "ra_kv_store_round_bytes",
    "ra_kv_store_stage", "ra_kv_store_wait_layer", "ra_kv_store_layer_view", "ra_kv_store_stats",
    "ra_kv_store_release", "ra_kv_store_save_round", "ra_kv_store_save_wait", "ra_kv_store_round_activity",
    "ra_kv_store_drop_round", "ra_kv_store_drop_inactive",
    "ra_round_scores_accumulate", "ra_layer_divergence", "ra_selection_coverage", "ra_measure_read_bandwidth",
]


class RaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"round_attention error {code}: {msg}")
        self.code = code


class ra_select_params(C.Structure):
    _fields_ = [("strategy", C.c_int32), ("ddof", C.c_int32), ("min_rounds", C.c_int32), ("max_rounds", C.c_int32),
                ("lambda_", C.c_double), ("fraction", C.c_double), ("threshold", C.c_double),
                ("keep_first", C.c_int32), ("keep_last", C.c_int32)]


class ra_kv_view(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("seg_off", C.c_void_p), ("seg_off_v", C.c_void_p),
                ("seg_len", C.c_void_p), ("n_rounds", C.c_void_p), ("block_table", C.c_void_p),
                ("block_size", C.c_int32), ("max_blocks", C.c_int32),
                ("B", C.c_int32), ("R_max", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
                ("dtype", C.c_int32), ("reserved", C.c_int32), ("max_tokens", C.c_int64)]


class ra_problem(C.Structure):
    _fields_ = [("B", C.c_int32), ("R_max", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
                ("q_len_max", C.c_int32), ("dtype", C.c_int32), ("reserved", C.c_int32), ("max_tokens", C.c_int64)]


class ra_store_cfg(C.Structure):
    _fields_ = [("device", C.c_int32), ("n_layers", C.c_int32), ("B", C.c_int32), ("R_max", C.c_int32),
                ("Hkv", C.c_int32), ("d", C.c_int32), ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("device_pool_bytes", C.c_size_t)]


_lib = None


def lib() -> C.CDLL:
    """The loaded shared library.  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2502_15294_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.ra_last_error.restype = C.c_char_p
        L.ra_kv_store_round_bytes.restype = C.c_size_t
        L.ra_kv_store_round_bytes.argtypes = [C.c_void_p, C.c_int]
        L.ra_create.argtypes = [C.POINTER(C.c_void_p), C.c_int]
        L.ra_destroy.argtypes = [C.c_void_p]
        L.ra_workspace_bytes.argtypes = [C.POINTER(ra_problem), C.POINTER(C.c_size_t)]
        L.ra_set_workspace.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.ra_profile_kernels.argtypes = [C.c_void_p, C.c_int]
        L.ra_set_prefill_precision.argtypes = [C.c_void_p, C.c_int]
        L.ra_profile_last_ms.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        L.ra_round_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(ra_kv_view),
                                      C.c_void_p, C.c_int, C.c_float, C.c_void_p, C.c_void_p]
        L.ra_round_scores_select.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(ra_kv_view),
                                             C.c_void_p, C.c_int, C.c_float, C.POINTER(ra_select_params), C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
        L.ra_measure_read_bandwidth.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int,
                                                C.POINTER(C.c_float)]
        L.ra_round_scores_accumulate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                                 C.POINTER(ra_kv_view), C.c_void_p, C.c_int, C.c_float, C.c_void_p,
                                                 C.c_void_p, C.c_void_p]
        L.ra_layer_divergence.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                          C.c_void_p, C.c_void_p]
        L.ra_selection_coverage.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                            C.c_int, C.c_void_p]
        L.ra_select_rounds.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                       C.POINTER(ra_select_params), C.c_void_p, C.c_void_p]
        L.ra_round_sparse_attn_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.POINTER(ra_kv_view),
                                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                                  C.c_float, C.c_void_p, C.c_void_p]
        L.ra_round_sparse_attn_decode_noalloc.argtypes = L.ra_round_sparse_attn_decode.argtypes
        L.ra_watershed_attn_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.POINTER(ra_kv_view),
                                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_void_p,
                                               C.c_void_p, C.c_void_p, C.c_void_p]
        L.ra_round_sparse_attn_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                                   C.POINTER(ra_kv_view), C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.c_void_p, C.c_int, C.c_float, C.c_void_p, C.c_void_p]
        L.ra_watershed_attn_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(ra_kv_view),
                                                C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_void_p]
        L.ra_kv_store_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(ra_store_cfg)]
        L.ra_kv_store_destroy.argtypes = [C.c_void_p]
        L.ra_kv_store_register_round.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int]
        L.ra_kv_store_stage.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.ra_kv_store_wait_layer.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        L.ra_kv_store_layer_view.argtypes = [C.c_void_p, C.c_int, C.POINTER(ra_kv_view)]
        L.ra_kv_store_stats.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                                        C.POINTER(C.c_uint64)]
        L.ra_kv_store_release.argtypes = [C.c_void_p]
        L.ra_kv_store_save_round.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p),
                                             C.POINTER(C.c_void_p), C.c_int, C.POINTER(C.c_void_p), C.c_void_p,
                                             C.c_void_p]
        L.ra_kv_store_save_wait.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
        L.ra_kv_store_round_activity.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_uint32),
                                                 C.POINTER(C.c_uint32)]
        L.ra_kv_store_drop_round.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.ra_kv_store_drop_inactive.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise RaError(rc, lib().ra_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return RA_BF16
    if t.dtype == torch.float32:
        return RA_F32
    raise TypeError(f"unsupported KV dtype {t.dtype}")


class KVView:
    """Holds the device tensors of one layer's round-indexed KV cache and the C struct that
    points at them (the tensors are kept alive as long as the view is)."""

    def __init__(self, k: torch.Tensor, v: Optional[torch.Tensor], seg_off: torch.Tensor, seg_len: torch.Tensor,
                 n_rounds: torch.Tensor, Hkv: int, d: int, max_tokens: int,
                 block_table: Optional[torch.Tensor] = None, block_size: int = 0,
                 seg_off_v: Optional[torch.Tensor] = None):
        assert seg_off.dtype == torch.int64 and seg_len.dtype == torch.int32 and n_rounds.dtype == torch.int32
        B, R_max = seg_len.shape
        self.tensors = (k, v, seg_off, seg_len, n_rounds, block_table, seg_off_v)
        self.B, self.R_max, self.Hkv, self.d = B, R_max, Hkv, d
        self.n_rounds, self.seg_len = n_rounds, seg_len
        self.c = ra_kv_view(k=_ptr(k), v=_ptr(v), seg_off=_ptr(seg_off), seg_off_v=_ptr(seg_off_v),
                            seg_len=_ptr(seg_len), n_rounds=_ptr(n_rounds), block_table=_ptr(block_table),
                            block_size=block_size, max_blocks=0 if block_table is None else block_table.shape[1],
                            B=B, R_max=R_max, Hkv=Hkv, d=d, dtype=_dtype_code(k), reserved=0,
                            max_tokens=int(max_tokens))

    @classmethod
    def from_struct(cls, c_view: ra_kv_view, owner) -> "KVView":
        self = cls.__new__(cls)
        self.tensors = (owner,)
        self.c = c_view
        self.B, self.R_max, self.Hkv, self.d = c_view.B, c_view.R_max, c_view.Hkv, c_view.d
        self.n_rounds = self.seg_len = None
        return self


# ---- context -----------------------------------------------------------------------------------
def ra_create(device: int = 0) -> C.c_void_p:
    ctx = C.c_void_p()
    _check(lib().ra_create(C.byref(ctx), device))
    return ctx


def ra_destroy(ctx) -> None:
    _check(lib().ra_destroy(ctx))


def ra_workspace_bytes(B: int, R_max: int, Hq: int, Hkv: int, d: int, q_len_max: int, dtype: int,
                       max_tokens: int) -> int:
    p = ra_problem(B=B, R_max=R_max, Hq=Hq, Hkv=Hkv, d=d, q_len_max=q_len_max, dtype=dtype, reserved=0,
                   max_tokens=max_tokens)
    out = C.c_size_t()
    _check(lib().ra_workspace_bytes(C.byref(p), C.byref(out)))
    return out.value


def ra_set_workspace(ctx, workspace: Optional[torch.Tensor]) -> None:
    if workspace is None:
        _check(lib().ra_set_workspace(ctx, None, 0))
    else:
        _check(lib().ra_set_workspace(ctx, workspace.data_ptr(), workspace.numel() * workspace.element_size()))


def ra_set_prefill_precision(ctx, mode: int) -> None:
    _check(lib().ra_set_prefill_precision(ctx, mode))


def ra_profile_kernels(ctx, enable: bool) -> None:
    _check(lib().ra_profile_kernels(ctx, 1 if enable else 0))


def ra_profile_last_ms(ctx) -> float:
    ms = C.c_float(0.0)
    _check(lib().ra_profile_last_ms(ctx, C.byref(ms)))
    return ms.value


# ---- compute -----------------------------------------------------------------------------------
def ra_round_scores(ctx, q: torch.Tensor, view: KVView, cur_k: Optional[torch.Tensor] = None,
                    scale: Optional[float] = None, scores_head: Optional[torch.Tensor] = None,
                    scores: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    B, q_len, Hq, d = q.shape
    if scale is None:
        scale = d ** -0.5
    if scores_head is None:
        scores_head = torch.empty((B, Hq, view.R_max), dtype=torch.float32, device=q.device)
    if scores is None:
        scores = torch.empty((B, view.R_max), dtype=torch.float32, device=q.device)
    cur_len = 0 if cur_k is None else cur_k.shape[1]
    _check(lib().ra_round_scores(ctx, _stream(stream), _ptr(q), q_len, Hq, C.byref(view.c), _ptr(cur_k), cur_len,
                                 scale, _ptr(scores_head), _ptr(scores)))
    return scores_head, scores


def ra_round_scores_select(ctx, q: torch.Tensor, view: KVView, params: Optional["ra_select_params"] = None,
                           cur_k: Optional[torch.Tensor] = None, scale: Optional[float] = None,
                           scores_head: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                           sel_idx: Optional[torch.Tensor] = None, n_sel: Optional[torch.Tensor] = None, stream=None
                           ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """Returns (scores_head, scores, sel_idx, n_sel)."""
    B, q_len, Hq, d = q.shape
    if scale is None:
        scale = d ** -0.5
    if params is None:
        params = make_select_params()
    if scores_head is None:
        scores_head = torch.empty((B, Hq, view.R_max), dtype=torch.float32, device=q.device)
    if scores is None:
        scores = torch.empty((B, view.R_max), dtype=torch.float32, device=q.device)
    if sel_idx is None:
        sel_idx = torch.empty((B, view.R_max), dtype=torch.int32, device=q.device)
    if n_sel is None:
        n_sel = torch.empty((B,), dtype=torch.int32, device=q.device)
    cur_len = 0 if cur_k is None else cur_k.shape[1]
    _check(lib().ra_round_scores_select(ctx, _stream(stream), _ptr(q), q_len, Hq, C.byref(view.c), _ptr(cur_k), cur_len,
                                        scale, C.byref(params), _ptr(scores_head), _ptr(scores), _ptr(sel_idx),
                                        _ptr(n_sel)))
    return scores_head, scores, sel_idx, n_sel


def ra_round_scores_accumulate(ctx, q: torch.Tensor, view: KVView, acc: torch.Tensor,
                               cur_k: Optional[torch.Tensor] = None, scale: Optional[float] = None,
                               scores_head: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                               stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """acc: float32 [B, Hq, R_max], updated in place; returns the normalised running totals."""
    B, q_len, Hq, d = q.shape
    assert acc.dtype == torch.float32 and tuple(acc.shape) == (B, Hq, view.R_max)
    if scale is None:
        scale = d ** -0.5
    if scores_head is None:
        scores_head = torch.empty((B, Hq, view.R_max), dtype=torch.float32, device=q.device)
    if scores is None:
        scores = torch.empty((B, view.R_max), dtype=torch.float32, device=q.device)
    cur_len = 0 if cur_k is None else cur_k.shape[1]
    _check(lib().ra_round_scores_accumulate(ctx, _stream(stream), _ptr(q), q_len, Hq, C.byref(view.c), _ptr(cur_k),
                                            cur_len, scale, _ptr(acc), _ptr(scores_head), _ptr(scores)))
    return scores_head, scores


def ra_layer_divergence(ctx, p: torch.Tensor, n_rounds: torch.Tensor, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """p: float32 [L, B, R_max] -> (kl float64 [B, L-1], its mean over the sequences [L-1])."""
    L, B, R_max = p.shape
    assert p.dtype == torch.float32
    kl = torch.empty((B, L - 1), dtype=torch.float64, device=p.device)
    kl_mean = torch.empty((L - 1,), dtype=torch.float64, device=p.device)
    _check(lib().ra_layer_divergence(ctx, _stream(stream), _ptr(p), _ptr(n_rounds), L, B, R_max, _ptr(kl),
                                     _ptr(kl_mean)))
    return kl, kl_mean


def ra_selection_coverage(ctx, scores: torch.Tensor, sel_idx: torch.Tensor, n_sel: torch.Tensor, stream=None
                          ) -> torch.Tensor:
    B, R_max = scores.shape
    cov = torch.empty((B,), dtype=torch.float32, device=scores.device)
    _check(lib().ra_selection_coverage(ctx, _stream(stream), _ptr(scores), _ptr(sel_idx), _ptr(n_sel), B, R_max,
                                       _ptr(cov)))
    return cov


def make_select_params(strategy: int = RA_SEL_ADAPTIVE, lam: float = 1.0, fraction: float = 0.10,
                       threshold: float = 0.10, ddof: int = 0, min_rounds: int = 1, max_rounds: int = 0,
                       keep_first: int = 0, keep_last: int = 0) -> ra_select_params:
    return ra_select_params(strategy=strategy, ddof=ddof, min_rounds=min_rounds, max_rounds=max_rounds,
                            lambda_=lam, fraction=fraction, threshold=threshold, keep_first=keep_first,
                            keep_last=keep_last)


def ra_select_rounds(ctx, scores: torch.Tensor, n_rounds: torch.Tensor, params: Optional[ra_select_params] = None,
                     sel_idx: Optional[torch.Tensor] = None, n_sel: Optional[torch.Tensor] = None, stream=None
                     ) -> Tuple[torch.Tensor, torch.Tensor]:
    B, R_max = scores.shape
    if params is None:
        params = make_select_params()
    if sel_idx is None:
        sel_idx = torch.empty((B, R_max), dtype=torch.int32, device=scores.device)
    if n_sel is None:
        n_sel = torch.empty((B,), dtype=torch.int32, device=scores.device)
    _check(lib().ra_select_rounds(ctx, _stream(stream), _ptr(scores), _ptr(n_rounds), B, R_max, C.byref(params),
                                  _ptr(sel_idx), _ptr(n_sel)))
    return sel_idx, n_sel


def ra_round_sparse_attn_decode(ctx, q: torch.Tensor, view: KVView, sel_idx: Optional[torch.Tensor] = None,
                                n_sel: Optional[torch.Tensor] = None, cur_k: Optional[torch.Tensor] = None,
                                cur_v: Optional[torch.Tensor] = None, cur_len: Optional[torch.Tensor] = None,
                                scale: Optional[float] = None, out: Optional[torch.Tensor] = None,
                                lse: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    B, Hq, d = q.shape
    if scale is None:
        scale = d ** -0.5
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    cur_cap = 0 if cur_k is None else cur_k.shape[1]
    _check(lib().ra_round_sparse_attn_decode(ctx, _stream(stream), _ptr(q), Hq, C.byref(view.c), _ptr(sel_idx),
                                             _ptr(n_sel), _ptr(cur_k), _ptr(cur_v), _ptr(cur_len), cur_cap, scale,
                                             _ptr(out), _ptr(lse)))
    return out, lse


def ra_round_sparse_attn_decode_noalloc(ctx, q: torch.Tensor, view: KVView, out: torch.Tensor, lse: Optional[torch.Tensor],
                                        sel_idx: Optional[torch.Tensor] = None, n_sel: Optional[torch.Tensor] = None,
                                        cur_k: Optional[torch.Tensor] = None, cur_v: Optional[torch.Tensor] = None,
                                        cur_len: Optional[torch.Tensor] = None, scale: Optional[float] = None,
                                        stream=None) -> None:
    """The decode call on the library's built-in scratch: the caller passes every output, nothing is allocated."""
    B, Hq, d = q.shape
    if scale is None:
        scale = d ** -0.5
    cur_cap = 0 if cur_k is None else cur_k.shape[1]
    _check(lib().ra_round_sparse_attn_decode_noalloc(ctx, _stream(stream), _ptr(q), Hq, C.byref(view.c), _ptr(sel_idx),
                                                     _ptr(n_sel), _ptr(cur_k), _ptr(cur_v), _ptr(cur_len), cur_cap,
                                                     scale, _ptr(out), _ptr(lse)))


def ra_watershed_attn_decode(ctx, q: torch.Tensor, view: KVView, cur_k: Optional[torch.Tensor] = None,
                             cur_v: Optional[torch.Tensor] = None, cur_len: Optional[torch.Tensor] = None,
                             scale: Optional[float] = None, out: Optional[torch.Tensor] = None,
                             lse: Optional[torch.Tensor] = None, scores_head: Optional[torch.Tensor] = None,
                             scores: Optional[torch.Tensor] = None, stream=None
                             ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """Returns (out, lse, scores_head, scores)."""
    B, Hq, d = q.shape
    if scale is None:
        scale = d ** -0.5
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    if scores_head is None:
        scores_head = torch.empty((B, Hq, view.R_max), dtype=torch.float32, device=q.device)
    if scores is None:
        scores = torch.empty((B, view.R_max), dtype=torch.float32, device=q.device)
    cur_cap = 0 if cur_k is None else cur_k.shape[1]
    _check(lib().ra_watershed_attn_decode(ctx, _stream(stream), _ptr(q), Hq, C.byref(view.c), _ptr(cur_k), _ptr(cur_v),
                                          _ptr(cur_len), cur_cap, scale, _ptr(out), _ptr(lse), _ptr(scores_head),
                                          _ptr(scores)))
    return out, lse, scores_head, scores


def ra_round_sparse_attn_prefill(ctx, q: torch.Tensor, view: KVView, sel_idx: Optional[torch.Tensor] = None,
                                 n_sel: Optional[torch.Tensor] = None, cur_k: Optional[torch.Tensor] = None,
                                 cur_v: Optional[torch.Tensor] = None, scale: Optional[float] = None,
                                 out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None, stream=None
                                 ) -> Tuple[torch.Tensor, torch.Tensor]:
    B, q_len, Hq, d = q.shape
    if scale is None:
        scale = d ** -0.5
    if out is None:
        out = torch.empty((B, q_len, Hq, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((B, q_len, Hq), dtype=torch.float32, device=q.device)
    cur_len = 0 if cur_k is None else cur_k.shape[1]
    _check(lib().ra_round_sparse_attn_prefill(ctx, _stream(stream), _ptr(q), q_len, Hq, C.byref(view.c),
                                              _ptr(sel_idx), _ptr(n_sel), _ptr(cur_k), _ptr(cur_v), cur_len, scale,
                                              _ptr(out), _ptr(lse)))
    return out, lse


def ra_watershed_attn_prefill(ctx, q: torch.Tensor, view: KVView, cur_k: Optional[torch.Tensor] = None,
                              cur_v: Optional[torch.Tensor] = None, scale: Optional[float] = None,
                              out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                              scores_head: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                              stream=None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """Returns (out, lse, scores_head, scores)."""
    B, q_len, Hq, d = q.shape
    if scale is None:
        scale = d ** -0.5
    if out is None:
        out = torch.empty((B, q_len, Hq, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((B, q_len, Hq), dtype=torch.float32, device=q.device)
    if scores_head is None:
        scores_head = torch.empty((B, Hq, view.R_max), dtype=torch.float32, device=q.device)
    if scores is None:
        scores = torch.empty((B, view.R_max), dtype=torch.float32, device=q.device)
    cur_len = 0 if cur_k is None else cur_k.shape[1]
    _check(lib().ra_watershed_attn_prefill(ctx, _stream(stream), _ptr(q), q_len, Hq, C.byref(view.c), _ptr(cur_k),
                                           _ptr(cur_v), cur_len, scale, _ptr(out), _ptr(lse), _ptr(scores_head),
                                           _ptr(scores)))
    return out, lse, scores_head, scores


# ---- round-indexed KV store ----------------------------------------------------------------------
def ra_kv_store_create(device: int, n_layers: int, B: int, R_max: int, Hkv: int, d: int, dtype: int,
                       device_pool_bytes: int) -> C.c_void_p:
    cfg = ra_store_cfg(device=device, n_layers=n_layers, B=B, R_max=R_max, Hkv=Hkv, d=d, dtype=dtype, reserved=0,
                       device_pool_bytes=device_pool_bytes)
    store = C.c_void_p()
    _check(lib().ra_kv_store_create(C.byref(store), C.byref(cfg)))
    return store


def ra_kv_store_destroy(store) -> None:
    _check(lib().ra_kv_store_destroy(store))


def ra_kv_store_round_bytes(store, length: int) -> int:
    return lib().ra_kv_store_round_bytes(store, length)


def ra_kv_store_register_round(store, seq: int, rnd: int, host_kv: Optional[torch.Tensor], length: int) -> None:
    """host_kv: pinned CPU tensor holding [n_layers][2][Hkv][len][d]; the caller keeps it alive."""
    _check(lib().ra_kv_store_register_round(store, seq, rnd, None if host_kv is None else host_kv.data_ptr(), length))


def ra_kv_store_stage(store, sel_idx_host: torch.Tensor, n_sel_host: torch.Tensor,
                      order: int = RA_STAGE_ROUND_MAJOR, side_stream=None) -> None:
    assert sel_idx_host.device.type == "cpu" and n_sel_host.device.type == "cpu"
    assert sel_idx_host.dtype == torch.int32 and n_sel_host.dtype == torch.int32
    _check(lib().ra_kv_store_stage(store, _ptr(sel_idx_host), _ptr(n_sel_host), order, _stream(side_stream)))


def ra_kv_store_wait_layer(store, layer: int, compute_stream=None) -> None:
    _check(lib().ra_kv_store_wait_layer(store, layer, _stream(compute_stream)))


def ra_kv_store_layer_view(store, layer: int) -> KVView:
    v = ra_kv_view()
    _check(lib().ra_kv_store_layer_view(store, layer, C.byref(v)))
    return KVView.from_struct(v, store)


def ra_kv_store_stats(store) -> Tuple[int, int, int]:
    a, b, c = C.c_uint64(), C.c_uint64(), C.c_uint64()
    _check(lib().ra_kv_store_stats(store, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def ra_kv_store_release(store) -> None:
    _check(lib().ra_kv_store_release(store))


def ra_kv_store_save_round(store, round_host: torch.Tensor, len_host: torch.Tensor, cur_k_layers, cur_v_layers,
                           host_kv, compute_stream=None, side_stream=None) -> None:
    """cur_k_layers / cur_v_layers: one device tensor [B][cur_cap][Hkv][d] per post-watershed layer;
    host_kv: one pinned CPU tensor (or None) per sequence; the caller keeps all of them alive."""
    assert round_host.device.type == "cpu" and len_host.device.type == "cpu"
    assert round_host.dtype == torch.int32 and len_host.dtype == torch.int32
    n_layers, B = len(cur_k_layers), len(host_kv)
    ks = (C.c_void_p * n_layers)(*[_ptr(t) for t in cur_k_layers])
    vs = (C.c_void_p * n_layers)(*[_ptr(t) for t in cur_v_layers])
    hs = (C.c_void_p * B)(*[None if t is None else t.data_ptr() for t in host_kv])
    cur_cap = cur_k_layers[0].shape[1]
    _check(lib().ra_kv_store_save_round(store, _ptr(round_host), _ptr(len_host), ks, vs, cur_cap, hs,
                                        _stream(compute_stream), _stream(side_stream)))


def ra_kv_store_save_wait(store) -> int:
    n = C.c_uint64()
    _check(lib().ra_kv_store_save_wait(store, C.byref(n)))
    return n.value


def ra_kv_store_round_activity(store, seq: int, rnd: int) -> Tuple[int, int]:
    turns, hits = C.c_uint32(), C.c_uint32()
    _check(lib().ra_kv_store_round_activity(store, seq, rnd, C.byref(turns), C.byref(hits)))
    return turns.value, hits.value


def ra_kv_store_drop_round(store, seq: int, rnd: int) -> None:
    _check(lib().ra_kv_store_drop_round(store, seq, rnd))


def ra_kv_store_drop_inactive(store, min_turns: int, B: int, R_max: int) -> Tuple[torch.Tensor, torch.Tensor]:
    idx = torch.empty((B, R_max), dtype=torch.int32)
    n = torch.empty((B,), dtype=torch.int32)
    _check(lib().ra_kv_store_drop_inactive(store, min_turns, _ptr(idx), _ptr(n)))
    return idx, n


def ra_measure_read_bandwidth(ctx, buf: torch.Tensor, iters: int = 5, stream=None) -> float:
    """GB/s of a plain read kernel over `buf` (waits for the GPU)."""
    out = C.c_float()
    _check(lib().ra_measure_read_bandwidth(ctx, _stream(stream), _ptr(buf), buf.numel() * buf.element_size(), iters,
                                           C.byref(out)))
    return out.value
