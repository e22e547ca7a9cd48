"""The entry point that allocates nothing (sparseloco_reproject_embedding_noalloc) against the entry point it is
a variant of (sparseloco_reproject_embedding with a caller workspace): same kernels, so T_S and T_perp must agree
bit for bit.  Two calls in a row on the same GPU array, the second with a smaller problem."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2601_02360_amd import binding as B

pytestmark = pytest.mark.gpu


def _inputs(vocab, d, k, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    t_s = torch.randn(vocab, d, generator=g, device="cuda") * 0.02
    t_perp = torch.randn(vocab, d, generator=g, device="cuda") * 0.02
    q, _ = torch.linalg.qr(torch.randn(d, k, generator=g, device="cuda", dtype=torch.float64))
    return t_s, t_perp, q.to(torch.float32).contiguous()


def _both_ways(vocab, d, k, seed, mode):
    t_s, t_perp, u = _inputs(vocab, d, k, seed)
    ref_s, ref_p = t_s.clone(), t_perp.clone()
    ws = torch.empty(vocab * k, device="cuda")
    B.sparseloco_reproject_embedding(ref_s, ref_p, u, ws, matmul=mode)
    L = B.lib()
    rc = L.sparseloco_reproject_embedding_noalloc(t_s.data_ptr(), t_perp.data_ptr(), u.data_ptr(), vocab, d, k, mode,
                                                  torch.cuda.current_stream().cuda_stream or None)
    assert rc == B.SPLC_OK, L.sparseloco_strerror(rc).decode()
    torch.cuda.synchronize()
    assert not torch.equal(ref_s, _inputs(vocab, d, k, seed)[0]), "the reference call changed nothing"
    assert torch.equal(t_s, ref_s), "T_S differs (vocab %d d %d k %d)" % (vocab, d, k)
    assert torch.equal(t_perp, ref_p), "T_perp differs (vocab %d d %d k %d)" % (vocab, d, k)


@pytest.mark.parametrize("mode", [B.SPLC_MATMUL_FP32, B.SPLC_MATMUL_BF16X3], ids=["fp32", "bf16x3"])
def test_noalloc_reprojection_equals_the_workspace_call_twice_in_a_row(mode):
    _both_ways(4100, 1024, 128, 1, mode)       # several tiles and a ragged last row block
    _both_ways(517, 384, 20, 2, mode)          # smaller: the array still holds the first call's coefficients
    _both_ways(32000, 2048, 256, 3, mode)      # the 1B shape, 8 192 000 of the 8 388 608 floats


def test_noalloc_rejects_what_does_not_fit():
    t = torch.zeros(8, 8, device="cuda")
    L = B.lib()
    too_many_rows = B.SPLC_NOALLOC_MAX_COEFF // 8 + 1
    rc = L.sparseloco_reproject_embedding_noalloc(t.data_ptr(), t.data_ptr(), t.data_ptr(), too_many_rows, 8, 8, 0, None)
    assert rc == B.SPLC_ETOOBIG
    assert L.sparseloco_reproject_embedding_noalloc(None, t.data_ptr(), t.data_ptr(), 8, 8, 8, 0, None) == B.SPLC_EINVAL
    assert L.sparseloco_reproject_embedding_noalloc(t.data_ptr(), t.data_ptr(), t.data_ptr(), 0, 8, 8, 0, None) == B.SPLC_OK
