"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments with the documented status before touching the GPU."""
import ctypes as C
import os
import re

import pytest

import paper_2502_15294_amd as ra

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "round_attention.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ra_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ra.lib()
    declared = _declared_symbols()
    assert len(declared) >= 18
    for name in declared:
        assert hasattr(L, name), f"{name} is declared in the header but not exported"
    assert sorted(ra.EXPORTS) == declared


def test_struct_sizes_match_the_header_layout():
    assert C.sizeof(ra.ra_select_params) == 48
    assert C.sizeof(ra.ra_kv_view) == 7 * 8 + 8 * 4 + 8
    assert C.sizeof(ra.ra_problem) == 8 * 4 + 8
    assert C.sizeof(ra.ra_store_cfg) == 8 * 4 + 8


def test_workspace_bytes_is_pure_host_arithmetic():
    n = ra.ra_workspace_bytes(B=8, R_max=20, Hq=32, Hkv=8, d=128, q_len_max=1, dtype=ra.RA_BF16, max_tokens=20000)
    assert n >= 8 * 32 * 64 * 130 * 4
    with pytest.raises(ra.RaError) as e:
        ra.ra_workspace_bytes(B=8, R_max=20, Hq=30, Hkv=8, d=128, q_len_max=1, dtype=ra.RA_BF16, max_tokens=1)
    assert e.value.code == ra.RA_ERR_INVALID_ARG


def test_null_arguments_are_rejected_before_any_launch():
    L = ra.lib()
    view = ra.ra_kv_view()
    p = ra.make_select_params()
    assert L.ra_round_scores(None, None, None, 1, 4, C.byref(view), None, 0, 1.0, None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_select_rounds(None, None, None, None, 1, 8, C.byref(p), None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_round_scores_select(None, None, None, 1, 4, C.byref(view), None, 0, 1.0, C.byref(p), None, None, None,
                                    None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_round_sparse_attn_decode(None, None, None, 4, C.byref(view), None, None, None, None, None, 0, 1.0,
                                         None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_watershed_attn_decode(None, None, None, 4, C.byref(view), None, None, None, 0, 1.0, None, None, None,
                                      None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_watershed_attn_prefill(None, None, None, 1, 4, C.byref(view), None, None, 0, 1.0, None, None, None,
                                       None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_round_sparse_attn_prefill(None, None, None, 1, 4, C.byref(view), None, None, None, None, 0, 1.0,
                                          None, None) != ra.RA_OK
    assert L.ra_round_scores_accumulate(None, None, None, 1, 4, C.byref(view), None, 0, 1.0, None, None,
                                        None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_layer_divergence(None, None, None, None, 2, 1, 8, None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_selection_coverage(None, None, None, None, None, 1, 8, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_set_workspace(None, None, 0) == ra.RA_ERR_INVALID_ARG
    assert L.ra_profile_kernels(None, 1) == ra.RA_ERR_INVALID_ARG
    assert L.ra_profile_last_ms(None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_measure_read_bandwidth(None, None, None, 0, 1, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_kv_store_create(None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_kv_store_register_round(None, 0, 0, None, 0) == ra.RA_ERR_INVALID_ARG
    assert L.ra_kv_store_stage(None, None, None, 0, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_kv_store_save_round(None, None, None, None, None, 16, None, None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_kv_store_save_wait(None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_kv_store_round_activity(None, 0, 0, None, None) == ra.RA_ERR_INVALID_ARG
    assert L.ra_kv_store_drop_round(None, 0, 0) == ra.RA_ERR_INVALID_ARG
    assert L.ra_kv_store_drop_inactive(None, 1, None, None) == ra.RA_ERR_INVALID_ARG
    assert b"NULL" in L.ra_last_error()


def test_header_is_plain_c():
    """round_attention.h declares a C boundary: a C11 compiler must accept it on its own, with all warnings on."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no host C compiler")
    hdr = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "round_attention.h")
    r = subprocess.run([gcc, "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x", "c", hdr],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
