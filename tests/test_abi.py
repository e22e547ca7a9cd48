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
    for code in (B.SPLC_OK, B.SPLC_EINVAL, B.SPLC_EALIGN, B.SPLC_ENOMEM, B.SPLC_EHIP, B.SPLC_EPLAN):
        s = L.sparseloco_strerror(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert L.sparseloco_strerror(-99).decode() == "unknown status"


@pytest.mark.parametrize("numels,kappa,quant", [([], 32, True), ([4096], 0, True), ([4096], 4097, True),
                                                 ([-1], 32, True), ([4096], 32, 7)])
def test_plan_create_rejects_bad_arguments_on_the_host(numels, kappa, quant):
    h = ctypes.c_void_p()
    arr = (ctypes.c_int64 * max(len(numels), 1))(*numels)
    q = quant if isinstance(quant, int) and not isinstance(quant, bool) else B.SPLC_QUANT_2BIT
    rc = B.lib().sparseloco_plan_create(ctypes.byref(h), len(numels), arr, kappa, q)
    assert rc == B.SPLC_EINVAL and not h.value


def test_null_plan_is_rejected():
    L = B.lib()
    assert L.sparseloco_compress(None, 0, 0, None, None, None, 0.95, None, None, None) == B.SPLC_EINVAL
    assert L.sparseloco_aggregate(None, 1, None, None, None, None) == B.SPLC_EINVAL
    assert L.sparseloco_outer_update(None, None, None, 1.0, None) == B.SPLC_EINVAL
    assert L.sparseloco_plan_set_select(None, 0) == B.SPLC_EINVAL
    L.sparseloco_plan_destroy(None)


def test_matmul_mode_switch_needs_no_gpu():
    """The process-wide matmul mode: fp32 by default, accepted values stick, anything else is refused."""
    L = B.lib()
    assert L.sparseloco_get_matmul_mode() == B.SPLC_MATMUL_FP32
    try:
        assert L.sparseloco_set_matmul_mode(B.SPLC_MATMUL_BF16X3) == B.SPLC_OK
        assert L.sparseloco_get_matmul_mode() == B.SPLC_MATMUL_BF16X3
        assert L.sparseloco_set_matmul_mode(2) == B.SPLC_EINVAL
        assert L.sparseloco_set_matmul_mode(-1) == B.SPLC_EINVAL
        assert L.sparseloco_get_matmul_mode() == B.SPLC_MATMUL_BF16X3
    finally:
        assert L.sparseloco_set_matmul_mode(B.SPLC_MATMUL_FP32) == B.SPLC_OK
