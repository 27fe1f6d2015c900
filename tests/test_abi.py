"""CPU checks of the boundary: the library loads without a GPU, exports every function that
include/q8nmt.h declares, and its pure-host helpers behave."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "q8nmt.h")


@pytest.fixture(scope="module")
def lib():
    import paper_1804_05038_amd as q
    if not os.path.exists(q.LIB_PATH):
        from paper_1804_05038_amd import build
        build.build()
    return q.load_library()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    names = re.findall(r"^\s*(?:q8_status|size_t|const char \*)\s*\*?\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_declares_the_north_star_entry_points():
    names = declared_functions()
    for f in ("q8_quantize_matrix", "q8_gemv", "q8_gemm_narrow", "gru_step_q8", "cgru_decoder_step_q8",
              "output_logits_q8", "q8_encode", "q8_beam_update", "q8_translate", "q8_create", "q8_destroy"):
        assert f in names


def test_library_exports_every_declared_function(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_host_side_helpers(lib):
    import paper_1804_05038_amd as q
    small, big = q.q8_workspace_bytes(1, 1, 16, 16), q.q8_workspace_bytes(8, 64, 65536, 2048)
    assert 4096 < small < big < 1 << 30
    assert q.q8_beam_state_bytes(100) > q.q8_beam_state_bytes(10) > 0
    # a NULL context or output is an error code, not a crash, and nothing is launched
    out = ctypes.c_void_p()
    assert lib.q8_create(None, None, None, 0) == 1
    assert lib.q8_create(ctypes.byref(out), None, None, 0) == 1 and out.value is None
    assert lib.q8_create(ctypes.byref(out), None, ctypes.c_void_p(4096 + 8), 1 << 20) == 3      # misaligned workspace
    assert lib.q8_create(ctypes.byref(out), None, ctypes.c_void_p(4096), 16) == 4               # too small
    assert lib.q8_destroy(None) == 1
    assert lib.q8_gemv(None, None, None, None, None, None) == 1
    assert lib.q8_last_error(None) == b"NULL context"


def test_source_token_ids_are_range_checked_on_the_host():
    """Ids that arrive on the host are rejected before anything reaches the GPU (the embedding
    lookup indexes a device table with them)."""
    import numpy as np
    import torch
    import paper_1804_05038_amd as q
    ok = q.source_ids([0, 5, 9], 10)
    assert ok.dtype == torch.int32 and ok.tolist() == [0, 5, 9]
    assert q.source_ids(np.array([3], np.int64), 4).tolist() == [3]
    for bad in ([10], [-1], [2, 11, 3], np.array([2 ** 31 + 5], np.int64)):
        with pytest.raises(ValueError):
            q.source_ids(bad, 10)
    for bad in ([], [[1, 2]], [1.5]):
        with pytest.raises(ValueError):
            q.source_ids(bad, 10)
    with pytest.raises(ValueError):
        q.source_ids(torch.tensor([1, 20]), 10)


def test_loop_forms_without_a_context_return_the_null_code_and_drop_the_codes(lib):
    """The forms that hand codes from step to step mark every code set they were given as not
    valid before anything else, so a call that fails leaves nothing that a later call could
    mistake for this step's codes."""
    from paper_1804_05038_amd.binding import _Codes
    import ctypes as C

    def given(v):
        c = _Codes(None, None, 0, v)
        return c, C.byref(c)

    def nulls(fn, n_tail):              # NULL or 0 for every argument before the code sets
        head = fn.argtypes[:len(fn.argtypes) - n_tail]
        return [None if t is C.c_void_p or hasattr(t, "contents") else 0 for t in head]

    assert lib.q8_attention_options(None, 1, 0) == 1
    y, py = given(2); cx, pcx = given(1); sp, psp = given(2)
    args = nulls(lib.cgru_decoder_step_loop_q8, 3)
    assert lib.cgru_decoder_step_loop_q8(*args, py, pcx, psp) == 1
    assert (y.valid, cx.valid, sp.valid) == (0, 0, 0)

    y, py = given(1); cx, pcx = given(1); sn, psn = given(2)
    args = nulls(lib.output_logits_beam_loop_q8, 4)
    assert lib.output_logits_beam_loop_q8(*args, py, pcx, psn, None) == 1
    assert (y.valid, sn.valid) == (0, 0) and cx.valid == 1      # the context's codes are an input only

    y, py = given(2); cx, pcx = given(1); s, ps = given(1); sp, psp = given(2)
    args = nulls(lib.cgru_decoder_step_batch_loop_q8, 4)
    assert lib.cgru_decoder_step_batch_loop_q8(*args, py, pcx, ps, psp) == 1
    assert (y.valid, cx.valid, s.valid, sp.valid) == (0, 0, 0, 0)

    s, ps = given(1); yn, pyn = given(2); sn, psn = given(2)
    args = nulls(lib.q8_beam_update_batch_loop, 4)
    assert lib.q8_beam_update_batch_loop(*args, None, ps, pyn, psn) == 1
    assert (yn.valid, sn.valid) == (0, 0) and s.valid == 1

    # the loop with GRU r ahead of the decision, and the panel output layer with the search steps in its launch
    cx, pcx = given(1)
    args = nulls(lib.cgru_decoder_step_ahead_q8, 1)
    assert lib.cgru_decoder_step_ahead_q8(*args, pcx) == 1
    assert cx.valid == 0

    y, py = given(2); cx, pcx = given(1)
    args = nulls(lib.output_logits_beam_ahead_q8, 6)
    assert lib.output_logits_beam_ahead_q8(*args, py, pcx, None, None, None, None) == 1
    assert y.valid == 0 and cx.valid == 1

    s, ps = given(1); y, py = given(1); cx, pcx = given(1); sn, psn = given(2)
    args = nulls(lib.output_logits_beam_batch_q8, 5)
    assert lib.output_logits_beam_batch_q8(*args, ps, py, pcx, psn, None) == 1
    assert (y.valid, sn.valid) == (0, 0) and (s.valid, cx.valid) == (1, 1)
