"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header declares, and
rejects bad arguments with the documented status codes before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2505_14742_amd import binding as q

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "quaff.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(quaff_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = q.lib()
    names = _declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), "missing export " + n
    assert set(q.SIGNATURES) == set(names), "binding and header disagree: %s" % (set(q.SIGNATURES) ^ set(names))


def test_status_strings_and_sizes():
    lib = q.lib()
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert lib.quaff_status_string(code)
    assert q.padded_outliers(0) == 0 and q.padded_outliers(1) == 64 and q.padded_outliers(64) == 64
    assert q.padded_outliers(65) == 128
    assert 3072 * 9216 <= q.packed_weight_bytes(3072, 9216) < 3072 * 9216 + 4096      # one byte per weight
    assert q.packed_weight_bytes(80, 18) >= 128 * 18                                   # c_in rounded up to 64
    assert q.packed_weight_bytes(0, 16) == 0
    w0 = q.workspace_bytes(2048, 3072, 9216, 31, 16)
    assert w0 >= 2048 * 9216 + 2048 * 4 + 2 * 2048 * 16 * 2          # backward: codes of dY, steps, T hi/lo
    assert q.workspace_bytes(4096, 3072, 9216, 31, 16) > w0
    assert q.workspace_bytes(0, 3072, 9216, 31, 16) == 0


A16 = 0x1000    # a non-null, 16-byte aligned fake device address: argument checks come before any device access


def test_packed_weight_layout_is_a_bijection_with_whole_lines():
    """Every code has its own byte inside the packed weight, and a 128-byte line holds 64 consecutive input channels
    of two neighbouring output channels (what both products' direct loads rely on)."""
    for c_in, c_out in ((128, 64), (208, 18), (64, 2)):
        size = q.packed_weight_bytes(c_in, c_out)
        seen = {}
        for j in range(c_out):
            for k in range(c_in):
                off = q.packed_weight_offset(c_in, c_out, k, j)
                assert 0 <= off < size and off not in seen
                seen[off] = (j, k)
        for off, (j, k) in seen.items():
            line = off // 128
            assert line == q.packed_weight_offset(c_in, c_out, k - k % 64, j - j % 2) // 128
            if k % 16 < 15:                                   # 16-byte chunks are contraction-contiguous
                assert q.packed_weight_offset(c_in, c_out, k + 1, j) == off + 1
        assert q.packed_weight_offset(c_in, c_out, c_in, 0) == -1 and q.packed_weight_offset(c_in, c_out, 0, -1) == -1


def test_argument_errors_are_reported_without_touching_the_device():
    lib = q.lib()
    # NULL pointers
    assert lib.quaff_quant_act(None, 8, 64, 64, None, None, 0, A16, A16, None, None) == q.ERR_NULL
    assert lib.quaff_linear_fwd_acc(None, None, 8, A16, 64, 64, None, 0, A16, None, None) == q.ERR_NULL
    # shapes: t = 0, c not a multiple of 16, ldx < c, n_outlier > c
    assert lib.quaff_quant_act(A16, 0, 64, 64, None, None, 0, A16, A16, None, None) == q.ERR_SHAPE
    assert lib.quaff_quant_act(A16, 8, 72, 72, None, None, 0, A16, A16, None, None) == q.ERR_SHAPE
    assert lib.quaff_quant_act(A16, 8, 64, 32, None, None, 0, A16, A16, None, None) == q.ERR_SHAPE
    assert lib.quaff_quant_act(A16, 8, 64, 64, None, A16, 65, A16, A16, A16, None) == q.ERR_SHAPE
    # alignment: pointer not 16-byte aligned, leading dimension not a multiple of 8
    assert lib.quaff_quant_act(A16 + 2, 8, 64, 64, None, None, 0, A16, A16, None, None) == q.ERR_ALIGN
    assert lib.quaff_quant_act(A16, 8, 64, 68, None, None, 0, A16, A16, None, None) == q.ERR_ALIGN
    # workspace too small / missing
    need = q.workspace_bytes(8, 64, 64, 4, 16)
    args = [A16, 8, 64, A16, A16, 64, 64, A16, A16, 16, C.c_float(1.0), A16, 64]
    assert lib.quaff_linear_bwd_dx(*args, A16, need // 4, None) == q.ERR_WORKSPACE
    assert lib.quaff_linear_bwd_dx(*args, None, 0, None) == q.ERR_WORKSPACE
    # LoRA rank must be 0 or a multiple of 16 up to 64
    bad_rank = list(args)
    bad_rank[9] = 24
    assert lib.quaff_linear_bwd_dx(*bad_rank, A16, need, None) == q.ERR_SHAPE
    # leading dimension of dX beyond what the store addressing covers (2^27 elements)
    huge_ld = list(args)
    huge_ld[12] = 1 << 27
    assert lib.quaff_linear_bwd_dx(*huge_ld, A16, need, None) == q.ERR_SHAPE
    # gamma outside [0, 1]
    assert lib.quaff_scale_update(A16, 8, 64, 64, A16, 4, A16, A16, 64, C.c_float(1.5), A16, A16, A16, A16, None,
                                  A16, 1 << 20, None) == q.ERR_SHAPE
    # scale update with an empty outlier set is a legal no-op
    assert lib.quaff_scale_update(None, 8, 64, 64, None, 0, None, None, 64, C.c_float(0.2), None, None, None, None,
                                  None, None, 0, None) == q.OK
    # outlier check: the result pointer is required, a negative count and a misaligned list are rejected
    assert lib.quaff_check_outliers(A16, 4, 64, None, None) == q.ERR_NULL
    assert lib.quaff_check_outliers(None, 4, 64, A16, None) == q.ERR_NULL
    assert lib.quaff_check_outliers(A16, -1, 64, A16, None) == q.ERR_SHAPE
    assert lib.quaff_check_outliers(A16 + 2, 4, 64, A16, None) == q.ERR_ALIGN
    # static-scratch scale update: same checks as quaff_scale_update, plus its maximum outlier count
    assert lib.quaff_scale_update_static(A16, 8, 2048, 2048, A16, 1025, A16, A16, 64, C.c_float(0.2), A16, A16, A16,
                                         A16, None, None) == q.ERR_SHAPE
    assert lib.quaff_scale_update_static(None, 8, 64, 64, A16, 4, A16, A16, 64, C.c_float(0.2), A16, A16, A16, A16,
                                         None, None) == q.ERR_NULL
    assert lib.quaff_scale_update_static(None, 8, 64, 64, None, 0, None, None, 64, C.c_float(0.2), None, None, None,
                                         None, None, None) == q.OK
    # one-call backward: argument checks come before any use of the optional second stream and its events
    assert lib.quaff_linear_bwd_step(A16, 8, 64, None, 64, A16, A16, 64, 64, A16, A16, 16, C.c_float(1.0), A16, 64,
                                     A16, A16, A16, 1 << 30, None, None, None, None) == q.ERR_NULL
    assert lib.quaff_linear_bwd_step(A16, 8, 64, A16, 64, A16, A16, 64, 64, A16, A16, 16, C.c_float(1.0), A16, 64,
                                     A16, A16, A16, 16, None, A16, A16, A16) == q.ERR_WORKSPACE
    # prepare: workspace check
    assert lib.quaff_prepare_weight(A16, 64, 64, 64, None, 0, A16, A16, None, None, None, A16, 16, None) \
        == q.ERR_WORKSPACE


def test_grid_wait_bound_is_a_host_side_setting():
    prev = q.debug_grid_wait_ticks(-1)
    assert prev > 0
    assert q.debug_grid_wait_ticks(123) == prev and q.debug_grid_wait_ticks(-1) == 123
    assert q.debug_grid_wait_ticks(prev) == 123 and q.debug_grid_wait_ticks(-1) == prev


def test_binding_raises_with_status_text():
    with pytest.raises(q.QuaffError) as e:
        q._check(q.ERR_ALIGN)
    assert "ALIGN" in str(e.value)
