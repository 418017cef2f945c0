"""C-ABI checks that need no GPU: the library loads, exports every symbol the header declares,
sizes the state, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2410_01623_amd import fira

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return fira.load_library()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "fira.h")).read()
    declared = re.findall(r"FIRA_API\s+[\w\s\*]+?\b(fira_\w+)\s*\(", hdr)
    assert len(declared) >= 13 and len(set(declared)) == len(declared)
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in fira.h but not exported"
    assert set(declared) == set(fira.EXPORTS)


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        fira.load_library(str(tmp_path / "libfira.so"))


def test_method_state_count_matches_the_paper(lib):
    # Table "Comparison of different methods": Fira keeps m r + 2 n r + 1 numbers (m <= n)
    d = fira.fira_matrix_desc(2048, 5461, 5461, 512, fira.FIRA_BF16)
    assert fira.fira_method_state_numel(d) == 2048 * 512 + 2 * 5461 * 512 + 1
    d = fira.fira_matrix_desc(5461, 2048, 2048, 512, fira.FIRA_BF16)     # transposed count for m > n
    assert fira.fira_method_state_numel(d) == 2048 * 512 + 2 * 5461 * 512 + 1
    d = fira.fira_matrix_desc(16, 16, 16, 17, fira.FIRA_BF16)
    assert fira.fira_method_state_numel(d) == 0


def test_state_bytes(lib):
    descs = fira.make_descs([(256, 688)], 64, fira.FIRA_F32)
    b1 = fira.fira_state_bytes(descs)
    assert b1 >= 2 * 4 * 688 * 64 and b1 % 256 == 0
    two = fira.make_descs([(256, 688), (256, 688)], 64, fira.FIRA_F32)
    assert fira.fira_state_bytes(two) > 1.9 * b1 - 65536
    # M and V dominate the persistent part: 2 * 4 bytes * r * max(m, n)
    big = fira.make_descs([(2048, 5461)], 512, fira.FIRA_BF16)
    assert fira.fira_state_bytes(big) < 8 * 4 * 5461 * 512
    for bad in ([(0, 5)], [(5, 0)]):
        assert fira.fira_state_bytes(fira.make_descs(bad, 1, fira.FIRA_BF16)) == 0
    assert fira.fira_state_bytes(fira.make_descs([(8, 8)], 9, fira.FIRA_BF16)) == 0       # r > min(m, n)
    assert fira.fira_state_bytes(fira.make_descs([(8, 8)], 0, fira.FIRA_BF16)) == 0
    assert fira.fira_state_bytes(fira.make_descs([(8, 8)], 4, fira.FIRA_BF16, lds=[7])) == 0  # ld < n
    assert fira.fira_state_bytes(fira.make_descs([(8, 8)], 4, 7)) == 0                     # bad dtype


def test_host_side_argument_errors(lib):
    ctx = ctypes.c_void_p()
    hp = fira.make_hparams()
    descs = fira.make_descs([(8, 12)], 4, fira.FIRA_BF16)
    nb = fira.fira_state_bytes(descs)
    init = lib.fira_init_state
    assert init(None, descs, 1, ctypes.byref(hp), None, nb, None) == fira.FIRA_ERR_INVALID_ARG
    assert init(ctypes.byref(ctx), descs, 1, None, None, nb, None) == fira.FIRA_ERR_INVALID_ARG
    assert init(ctypes.byref(ctx), None, 1, ctypes.byref(hp), None, nb, None) == fira.FIRA_ERR_INVALID_ARG
    assert init(ctypes.byref(ctx), descs, 1, ctypes.byref(hp), None, nb, None) == fira.FIRA_ERR_INVALID_ARG
    assert b"dev_state" in lib.fira_last_error(None)
    bad = fira.make_descs([(8, 12)], 9, fira.FIRA_BF16)
    assert init(ctypes.byref(ctx), bad, 1, ctypes.byref(hp), ctypes.c_void_p(256), nb, None) == fira.FIRA_ERR_SHAPE
    bad = fira.make_descs([(8, 12)], 4, 3)
    assert init(ctypes.byref(ctx), bad, 1, ctypes.byref(hp), ctypes.c_void_p(256), nb, None) == fira.FIRA_ERR_DTYPE
    # misaligned or short slab
    assert init(ctypes.byref(ctx), descs, 1, ctypes.byref(hp), ctypes.c_void_p(260), nb, None) == fira.FIRA_ERR_WORKSPACE
    assert init(ctypes.byref(ctx), descs, 1, ctypes.byref(hp), ctypes.c_void_p(256), nb - 1, None) == fira.FIRA_ERR_WORKSPACE
    badhp = fira.make_hparams(beta1=1.0)
    assert init(ctypes.byref(ctx), descs, 1, ctypes.byref(badhp), ctypes.c_void_p(256), nb, None) == fira.FIRA_ERR_INVALID_ARG
    assert not ctx.value
    # null context
    assert lib.fira_step(None, 0, None, None, None) == fira.FIRA_ERR_INVALID_ARG
    assert lib.fira_set_projector(None, 0, None, 0) == fira.FIRA_ERR_INVALID_ARG
    assert lib.fira_set_projectors(None, 0, None, None, 0) == fira.FIRA_ERR_INVALID_ARG
    assert lib.fira_set_hparams(None, ctypes.byref(hp)) == fira.FIRA_ERR_INVALID_ARG
    assert lib.fira_get_diag(None, 0, None, None, None) == fira.FIRA_ERR_INVALID_ARG
    lib.fira_destroy(None)   # no-op
