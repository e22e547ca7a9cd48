"""The C-ABI library loads and exports every symbol include/sparseloco.h declares;
host-side argument validation works without a GPU (no compute call is made)."""
import ctypes
import os
import re

import pytest

from paper_2601_02360_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sparseloco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sparseloco_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_symbols()
    assert "sparseloco_compress" in names and "sparseloco_aggregate" in names and "sparseloco_outer_update" in names
    assert sorted(B.EXPORTS) == names
    L = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    L = B.lib()
    seen = set()
    for code in (B.SPLC_OK, B.SPLC_EINVAL, B.SPLC_EALIGN, B.SPLC_ENOMEM, B.SPLC_EHIP, B.SPLC_EPLAN, B.SPLC_ETOOBIG):
        s = L.sparseloco_strerror(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert L.sparseloco_strerror(-99).decode() == "unknown status"


@pytest.mark.parametrize("numels,chunk,kappa,quant", [([], 4096, 32, 1), ([4096], 4096, 0, 1), ([4096], 4096, 4097, 1),
                                                       ([-1], 4096, 32, 1), ([4096], 4096, 32, 7), ([4096], 2048, 32, 1)])
def test_plan_create_rejects_bad_arguments_on_the_host(numels, chunk, kappa, quant):
    h = ctypes.c_void_p()
    arr = (ctypes.c_int64 * max(len(numels), 1))(*numels)
    rc = B.lib().sparseloco_plan_create(ctypes.byref(h), len(numels), arr, chunk, kappa, quant, None)
    assert rc == B.SPLC_EINVAL and not h.value
    rc = B.lib().sparseloco_plan_create_2d(ctypes.byref(h), len(numels), arr, arr, chunk, kappa, quant, None)
    assert rc == B.SPLC_EINVAL and not h.value


def test_null_handles_are_rejected():
    L = B.lib()
    h = ctypes.c_void_p()
    assert L.sparseloco_compress(None, 0, None, None, None, 0, 0.95, None, None, None) == B.SPLC_EINVAL
    assert L.sparseloco_compress_batch(None, 1, None, None, None, 0.95, None, None) == B.SPLC_EINVAL
    assert L.sparseloco_aggregate(None, None, None, None) == B.SPLC_EINVAL
    assert L.sparseloco_aggregate_update(None, None, None, 1.0, None, None, None) == B.SPLC_EINVAL
    assert L.sparseloco_outer_update(None, None, None, 1.0, None) == B.SPLC_EINVAL
    assert L.sparseloco_plan_set_select(None, 0) == B.SPLC_EINVAL
    assert L.sparseloco_tensors_bind(ctypes.byref(h), None, 1, None, B.SPLC_F32, None) == B.SPLC_EINVAL and not h.value
    assert L.sparseloco_messages_bind(ctypes.byref(h), None, 1, None, None, None) == B.SPLC_EINVAL and not h.value
    L.sparseloco_plan_destroy(None)
    L.sparseloco_tensors_release(None)
    L.sparseloco_messages_release(None)


def test_matrix_calls_validate_on_the_host():
    """Bad shapes, a bad matmul mode and a too-large problem for the call that allocates nothing are refused
    before anything touches a GPU."""
    L = B.lib()
    p = ctypes.c_void_p(4096)            # never dereferenced: every call below is refused during validation
    assert L.sparseloco_reproject_embedding(p, p, p, p, 8, 8, 9, B.SPLC_MATMUL_FP32, None) == B.SPLC_EINVAL
    assert L.sparseloco_reproject_embedding(p, p, p, p, 8, 8, 4, 2, None) == B.SPLC_EINVAL
    assert L.sparseloco_reproject_embedding(p, ctypes.c_void_p(4098), p, p, 8, 8, 4, 0, None) == B.SPLC_EALIGN
    too_many_rows = B.SPLC_NOALLOC_MAX_COEFF // 8 + 1
    assert L.sparseloco_reproject_embedding_noalloc(p, p, p, too_many_rows, 8, 8, 0, None) == B.SPLC_ETOOBIG
    assert L.sparseloco_subspace_project(p, p, None, 5, None, 0, p, p, 4, 8, 2, 0, None) == B.SPLC_EINVAL   # no token ids
    assert L.sparseloco_subspace_reconstruct(p, None, None, 0, None, 0, p, p, 4, 8, 2, -1, None) == B.SPLC_EINVAL


def test_kernel_choice_follows_the_documented_rule():
    """Host logic of the matrix calls' launcher: narrow kernel up to 32 columns (16 with both tables), 64-column
    tiles for an odd number of 64-column blocks, 128 rows only with two workgroups per compute unit."""
    c = B.subspace_kernel_choice
    assert c(B.SPLC_OP_PROJECT, 16384, 2048, 16, 2) == (16, 16)
    assert c(B.SPLC_OP_PROJECT, 16384, 2048, 32, 2) == (64, 64)
    assert c(B.SPLC_OP_PROJECT, 16384, 2048, 32, 1) == (16, 32)
    assert c(B.SPLC_OP_PROJECT, 16384, 2050, 16, 0) == (64, 64)              # d not a multiple of 32
    assert c(B.SPLC_OP_PROJECT, 16384, 2048, 256, 2) == (64, 128)
    assert c(B.SPLC_OP_PROJECT, 32768, 2048, 256, 2) == (128, 128)
    assert c(B.SPLC_OP_REPROJECT_PASS1, 32000, 2048, 192) == (128, 64)
    assert c(B.SPLC_OP_REPROJECT_PASS2, 32000, 2048, 256) == (128, 128)
    assert c(B.SPLC_OP_REPROJECT_PASS2, 32000, 2048, 192) == (64, 64)
    assert c(B.SPLC_OP_RECONSTRUCT, 16384, 2048, 256, 2) == (64, 128)
    assert c(B.SPLC_OP_REPROJECT_PASS2, 32000, 2048, 256, 0, B.SPLC_MATMUL_BF16X3) == (128, 128)
    with pytest.raises(B.SparseLoCoError):
        c(9, 100, 64, 8)
    with pytest.raises(B.SparseLoCoError):
        c(B.SPLC_OP_PROJECT, 100, 64, 65)
