"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, sizes are right, and every argument check fires before any
launch (so none of this needs a GPU)."""
import ctypes
import os
import re

import pytest

import paper_2407_02891_amd as bcq
from paper_2407_02891_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "bcq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bcq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = bcq.lib()
    syms = header_symbols()
    assert set(syms) == set(B.EXPORTS)
    for s in syms:
        assert hasattr(L, s), s


def test_status_strings():
    assert bcq.status_string(0) == "ok"
    for s in range(1, 5):
        assert bcq.status_string(s) not in ("ok", "unknown status")
    assert bcq.status_string(99) == "unknown status"


def test_packed_bytes_equals_algorithmic_bytes_on_unpadded_shapes():
    for (M, N, q, z) in [(7168, 28672, 3, 0), (28672, 7168, 3, 0), (7168, 7168, 2, 1), (9216, 36864, 3, 0), (8192, 8192, 2, 0)]:
        d = bcq.Desc(M, N, q, 128, z, 0)
        G = N // 128
        want = q * M * N // 8 + q * M * G * 2 + z * M * G * 2
        assert bcq.packed_bytes(d) == want


def test_packed_bytes_pads_ragged_shapes():
    d = bcq.Desc(768, 768, 3, 128, 0, 0)              # N padded to 1024
    assert bcq.packed_bytes(d) == 2 * 24 * (2 * 3 * 1024 + 64 * 2 * 3 * 2)
    assert bcq.workspace_bytes(d, 1) == 768 * 8
    d1 = bcq.Desc(100, 512, 3, 128, 0, 0)             # single column slice: no split-K workspace
    assert bcq.workspace_bytes(d1, 1) == 0


@pytest.mark.parametrize("fields,status", [
    ((0, 128, 3, 128, 0), B.BCQ_ERR_INVALID_ARG),
    ((16, 100, 3, 100, 0), B.BCQ_ERR_INVALID_ARG),      # N not a multiple of 32
    ((16, 256, 0, 128, 0), B.BCQ_ERR_INVALID_ARG),
    ((16, 256, 3, 96, 0), B.BCQ_ERR_INVALID_ARG),       # group does not divide N
    ((16, 256, 3, 128, 2), B.BCQ_ERR_INVALID_ARG),
    ((16, 256, 5, 128, 0), B.BCQ_ERR_UNSUPPORTED),      # q > 4
    ((16, 384, 3, 96, 0), B.BCQ_ERR_UNSUPPORTED),       # group not 32, 64, k*128 or N
    ((16, 640, 3, 160, 0), B.BCQ_ERR_UNSUPPORTED),
])
def test_bad_descriptors_are_refused_before_launch(fields, status):
    d = bcq.Desc(*fields, 0)
    assert bcq.packed_bytes(d) == 0
    assert bcq.workspace_bytes(d, 1) == 0
    L = bcq.lib()
    # non-NULL dummy pointers: validation must fail before they are ever used
    rc = L.bcq_pack(ctypes.byref(d), 256, 256, None, 256, None)
    assert rc == status


def test_small_groups_are_sized_with_one_scale_set_per_group():
    for group, sub in ((32, 4), (64, 2), (128, 1)):
        d = bcq.Desc(32, 512, 3, group, 1, 0)
        assert bcq.packed_bytes(d) == 2 * 3 * 1024 + 64 * 2 * sub * 4 * 2


def test_row_wise_scales_are_stored_once_per_row():
    d = bcq.Desc(32, 1024, 3, 1024, 1, 0)        # group = N: 16 scale records per half tile instead of 64
    assert bcq.packed_bytes(d) == 2 * (2 * 3 * 1024 + 16 * 2 * 4 * 2)
    d = bcq.Desc(32, 1024, 3, 512, 1, 0)         # two groups per row: one record per lane
    assert bcq.packed_bytes(d) == 2 * (2 * 3 * 1024 + 64 * 2 * 4 * 2)


def test_pack_rows_argument_checks():
    L = bcq.lib()
    d = bcq.Desc(64, 1024, 3, 128, 0, 0)
    ok = (256, 256, None, 256, None)  # codes, alpha, offset, packed, stream
    assert L.bcq_pack_rows(ctypes.byref(d), -1, 8, *ok) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_pack_rows(ctypes.byref(d), 0, 0, *ok) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_pack_rows(ctypes.byref(d), 60, 5, *ok) == B.BCQ_ERR_INVALID_ARG      # past the last row
    assert L.bcq_pack_rows(ctypes.byref(d), 0, 8, None, 256, None, 256, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_pack_rows(ctypes.byref(d), 0, 8, 256, 256, 256, 256, None) == B.BCQ_ERR_INVALID_ARG  # offset w/o flag
    assert L.bcq_pack_rows(ctypes.byref(d), 0, 8, 256, 256, None, 255, None) == B.BCQ_ERR_INVALID_ARG  # misaligned
    assert d.layout_version == 0
    assert L.bcq_pack_rows(None, 0, 8, *ok) == B.BCQ_ERR_INVALID_ARG


def test_gemv_argument_checks():
    L = bcq.lib()
    d = bcq.Desc(64, 1024, 3, 128, 0, 0)
    ok = 0x1000
    assert L.bcq_gemv(ctypes.byref(d), ok, ok, ok, ok, None) == B.BCQ_ERR_INVALID_ARG   # not packed yet
    d.layout_version = B.BCQ_LAYOUT_VERSION
    assert L.bcq_gemv(None, ok, ok, ok, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_gemv(ctypes.byref(d), None, ok, ok, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_gemv(ctypes.byref(d), ok, None, ok, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_gemv(ctypes.byref(d), ok, ok, None, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_gemv(ctypes.byref(d), ok + 16, ok, ok, ok, None) == B.BCQ_ERR_INVALID_ARG  # blob not 256-aligned
    assert L.bcq_gemv(ctypes.byref(d), ok, ok + 2, ok, ok, None) == B.BCQ_ERR_INVALID_ARG   # x not 16-aligned
    assert L.bcq_gemv(ctypes.byref(d), ok, ok, ok + 1, ok, None) == B.BCQ_ERR_INVALID_ARG   # y not 2-aligned
    assert L.bcq_gemv(ctypes.byref(d), ok, ok, ok, None, None) == B.BCQ_ERR_WORKSPACE
    assert L.bcq_gemv(ctypes.byref(d), ok, ok, ok, ok + 4, None) == B.BCQ_ERR_WORKSPACE


def test_skinny_argument_checks():
    L = bcq.lib()
    d = bcq.Desc(64, 1024, 3, 128, 0, B.BCQ_LAYOUT_VERSION)
    ok = 0x1000
    f = lambda ldx, ldy, b: L.bcq_gemm_skinny(ctypes.byref(d), ok, ok, ldx, ok, ldy, b, ok, None)
    assert f(1024, 64, 0) == B.BCQ_ERR_INVALID_ARG
    assert f(1024, 64, B.BCQ_MAX_BATCH + 1) == B.BCQ_ERR_INVALID_ARG
    assert f(1016, 64, 2) == B.BCQ_ERR_INVALID_ARG     # ldx < N
    assert f(1028, 64, 2) == B.BCQ_ERR_INVALID_ARG     # ldx not a multiple of 8
    assert f(1024, 63, 2) == B.BCQ_ERR_INVALID_ARG     # ldy < M


def test_pack_pointer_checks():
    L = bcq.lib()
    d = bcq.Desc(64, 1024, 3, 128, 1, 0)
    ok = 0x1000
    assert L.bcq_pack(ctypes.byref(d), ok, ok, None, ok, None) == B.BCQ_ERR_INVALID_ARG   # offset missing
    d0 = bcq.Desc(64, 1024, 3, 128, 0, 0)
    assert L.bcq_pack(ctypes.byref(d0), ok, ok, ok, ok, None) == B.BCQ_ERR_INVALID_ARG    # offset unexpected
    assert L.bcq_pack(ctypes.byref(d0), None, ok, None, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_pack(ctypes.byref(d0), ok, ok, None, ok + 128, None) == B.BCQ_ERR_INVALID_ARG
    assert d0.layout_version == 0


def test_from_linear_argument_checks():
    L = bcq.lib()
    ok = 0x1000
    labels = lambda *v: (ctypes.c_int32 * len(v))(*v)
    f = lambda M, N, g, n, q, lab, *ptrs: L.bcq_from_linear(M, N, g, n, q, lab, *(ptrs or (ok,) * 6), None)
    good = labels(0, 1, 1)
    assert f(0, 256, 128, 3, 2, good) == B.BCQ_ERR_INVALID_ARG
    assert f(16, 256, 96, 3, 2, good) == B.BCQ_ERR_INVALID_ARG          # group does not divide N
    assert f(16, 256, 128, 9, 2, good) == B.BCQ_ERR_INVALID_ARG         # more than 8 linear bits
    assert f(16, 256, 128, 3, 4, labels(0, 1, 2)) == B.BCQ_ERR_INVALID_ARG   # more classes than planes
    assert f(16, 256, 128, 3, 2, labels(0, 0, 0)) == B.BCQ_ERR_INVALID_ARG   # class 1 empty
    assert f(16, 256, 128, 3, 2, labels(0, 2, 1)) == B.BCQ_ERR_INVALID_ARG   # label out of range
    assert f(16, 256, 128, 3, 2, None) == B.BCQ_ERR_INVALID_ARG
    assert f(16, 256, 128, 6, 5, labels(0, 1, 2, 3, 4, 4)) == B.BCQ_ERR_UNSUPPORTED  # q > 4
    for k in range(6):
        ptrs = [ok] * 6
        ptrs[k] = None
        assert f(16, 256, 128, 3, 2, good, *ptrs) == B.BCQ_ERR_INVALID_ARG
    assert f(16, 256, 128, 3, 2, good, ok, ok + 2, ok, ok, ok, ok) == B.BCQ_ERR_INVALID_ARG  # S misaligned


def test_quantizer_argument_checks():
    L = bcq.lib()
    ok = 0x1000
    assert L.bcq_quant_workspace_bytes(0, 64) == 0
    need = L.bcq_quant_workspace_bytes(70, 160)
    assert need >= 4 * (2 * 160 * 72 + 2 * 72 + 3 * 72 + 128 * 72) and need % 256 == 0   # row pitch 72
    assert L.bcq_quant_hessian(64, 0, ok, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_quant_hessian(66, 8, ok, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_quant_hessian(64, 8, None, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_quant_hessian(64, 8, ok, ok + 4, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_quant_hessian(1 << 16, 8, ok, ok, None) == B.BCQ_ERR_UNSUPPORTED
    assert L.bcq_quant_factor_workspace_bytes(66) == 0
    assert L.bcq_quant_factor_workspace_bytes(64) >= 4 * 3 * 64 * 64
    assert L.bcq_quant_factor(0, 0.01, ok, ok, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_quant_factor(64, -1.0, ok, ok, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_quant_factor(64, 0.01, None, ok, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_quant_factor(64, 0.01, ok, ok + 4, ok, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_quant_factor(64, 0.01, ok, ok, None, None) == B.BCQ_ERR_WORKSPACE
    assert L.bcq_quant_factor(1 << 16, 0.01, ok, ok, ok, None) == B.BCQ_ERR_UNSUPPORTED
    search = lambda M, N, n, q, grid, *p: L.bcq_quant_search(M, N, n, q, grid, *(p or (ok,) * 7), None)
    assert search(0, 64, 3, 2, 4) == B.BCQ_ERR_INVALID_ARG
    assert search(8, 64, 1, 1, 4) == B.BCQ_ERR_INVALID_ARG              # Eq. 7 needs n >= 2
    assert search(8, 64, 9, 2, 4) == B.BCQ_ERR_INVALID_ARG
    assert search(8, 64, 3, 4, 4) == B.BCQ_ERR_INVALID_ARG              # more classes than planes
    assert search(8, 64, 6, 5, 4) == B.BCQ_ERR_UNSUPPORTED
    assert search(8, 1 << 17, 3, 2, 4) == B.BCQ_ERR_UNSUPPORTED
    assert search(8, 66, 3, 2, 4) == B.BCQ_ERR_INVALID_ARG              # N not a multiple of 4
    assert search(8, 64, 3, 2, 0) == B.BCQ_ERR_INVALID_ARG
    for k in range(5):                                                  # W, H, S, qbias, labels
        p = [ok] * 7
        p[k] = None
        assert search(8, 64, 3, 2, 4, *p) == B.BCQ_ERR_INVALID_ARG
    assert search(8, 64, 3, 2, 4, ok, ok, ok, ok, ok, ok, None) == B.BCQ_ERR_WORKSPACE
    assert search(8, 64, 3, 2, 4, ok, ok, ok, ok, ok, ok, ok + 4) == B.BCQ_ERR_WORKSPACE
    assert search(8, 64, 3, 2, 4, ok + 2, ok, ok, ok, ok, ok, ok) == B.BCQ_ERR_INVALID_ARG
    assert search(8, 64, 3, 2, 4, ok, ok + 8, ok, ok, ok, ok, ok) == B.BCQ_ERR_INVALID_ARG   # H: 16 bytes
    gptq = lambda M, N, n, q, *p: L.bcq_quant_gptq(M, N, n, q, *(p or (ok,) * 7), None)
    assert gptq(8, 0, 3, 2) == B.BCQ_ERR_INVALID_ARG
    for k in range(6):
        p = [ok] * 7
        p[k] = None
        assert gptq(8, 64, 3, 2, *p) == B.BCQ_ERR_INVALID_ARG
    assert gptq(8, 64, 3, 2, ok, ok, ok, ok, ok, ok, None) == B.BCQ_ERR_WORKSPACE
    rows = lambda M, N, n, q, *p: L.bcq_from_linear_rows(M, N, n, q, *(p or (ok,) * 7), None)
    assert rows(8, 64, 3, 0) == B.BCQ_ERR_INVALID_ARG
    for k in range(7):
        p = [ok] * 7
        p[k] = None
        assert rows(8, 64, 3, 2, *p) == B.BCQ_ERR_INVALID_ARG
    assert rows(8, 64, 3, 2, ok, ok, ok, ok, ok, ok + 1, ok) == B.BCQ_ERR_INVALID_ARG   # alpha misaligned


def test_misc_argument_checks():
    L = bcq.lib()
    assert L.bcq_workspace_init(None, 64, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_workspace_init(None, 0, None) == B.BCQ_OK
    assert L.bcq_workspace_init(0x1008, 64, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_read_probe(None, 64, 0x1000, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_read_probe(0x1000, 24, 0x1000, None) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_set_option(b"no_such_option", 1) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_set_option(b"workgroups", -1) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_set_option(b"workgroups", 0) == B.BCQ_OK
    assert L.bcq_set_option(b"skinny_version", 7) == B.BCQ_ERR_INVALID_ARG
    assert L.bcq_set_option(b"skinny_lds_steps", 2) == B.BCQ_ERR_INVALID_ARG
    for name, ok_value in ((b"skinny_version", 1), (b"skinny_lds_steps", 3), (b"waves", 8), (b"skinny_parts", 5)):
        assert L.bcq_set_option(name, ok_value) == B.BCQ_OK
        assert L.bcq_set_option(name, 0) == B.BCQ_OK
    assert B.read_probe_sink_bytes() >= 4
