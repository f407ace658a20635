"""CPU-only checks of the C-ABI library: it loads, exports what include/wind.h declares, and
rejects bad arguments before touching a GPU.  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2505_13765_amd import build, binding

    if build.stale():
        build.build(True)
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "wind.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wind_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    from paper_2505_13765_amd import binding

    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_argument_errors_without_gpu(lib):
    from paper_2505_13765_amd import binding

    out = C.c_void_p()
    assert lib.wind_load_weights(None, None, C.byref(out)) == binding.WIND_ERR_ARG
    assert b"null" in lib.wind_last_error()
    w = binding._Weights()
    w.D = w.E = w.Hp = w.Hj = w.V = 64
    w.L = 9
    assert lib.wind_load_weights(C.byref(w), None, C.byref(out)) == binding.WIND_ERR_ARG
    w.L = 1
    assert lib.wind_load_weights(C.byref(w), None, C.byref(out)) == binding.WIND_ERR_ARG   # null weight pointers
    assert lib.wind_greedy_decode(None, None, None, 1, 1, 1, 1, None, None, None, 1, None) == binding.WIND_ERR_ARG
    assert lib.wind_sequential_decode(None, None, None, 1, 1, 1, None, None, None, 1, None) == binding.WIND_ERR_ARG
    assert lib.wind_greedy_decode_async(None, None, None, 1, 1, 1, 1, None, None, None, 1, None, 0, 1, None) == binding.WIND_ERR_ARG
    assert lib.wind_get_stats(None, None) == binding.WIND_ERR_ARG
    assert lib.wind_set_option(None, b"graph", 1) == binding.WIND_ERR_ARG
    n = C.c_size_t(0)
    assert lib.wind_workspace_bytes(None, 1, 1, 1, C.byref(n)) == binding.WIND_ERR_ARG
    assert lib.wind_beam_decode(None, None, 0, 4, 4, 2, 1, None, None, 0, None, None, None, None, None, None) == binding.WIND_ERR_ARG
    assert lib.wind_beam_window_scores(None, None, 1, None, 1, 1, None, None, None, None) == binding.WIND_ERR_ARG
    k = C.c_int32(0)
    assert lib.wind_debug_enc_proj(None, None, None, 1, 1, None, None) == binding.WIND_ERR_ARG
    assert lib.wind_debug_joint_keys(None, None, None, 1, 1, 1, None, C.byref(k), C.byref(k), None) == binding.WIND_ERR_ARG
    assert lib.wind_get_joint_launches(None, None, None, 0, None) == binding.WIND_ERR_ARG
    assert lib.wind_get_call_times(None, None, None) == binding.WIND_ERR_ARG
    assert lib.wind_get_loop_info(None, None, None) == binding.WIND_ERR_ARG
    assert lib.wind_free(None) == binding.WIND_OK


def test_binding_struct_layout_matches_header():
    """The ctypes mirror of wind_weights / wind_stats must have the header's field order."""
    from paper_2505_13765_amd import binding

    text = open(os.path.join(ROOT, "include", "wind.h")).read()
    body = text[text.index("typedef struct {\n  int32_t D, E"): text.index("} wind_weights;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    order = re.findall(r"\b(D|E|Hp|L|Hj|V|dtype|emb|w_ih|w_hh|b_ih|b_hh|w_enc|b_enc|w_pred|b_pred|w_out|b_out)\b", body)
    assert order == [f[0] for f in binding._Weights._fields_]
    assert C.sizeof(binding.WindStats) == 8 * (7 + 65)
