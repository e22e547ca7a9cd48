"""Pins for the oracle's 2-D tile geometry (paper section 3 / appendix table:
"chunk size 64 x 64"): a tiled run over a matrix must equal the already pinned
flat oracle applied to each block cut out with numpy slicing, with the block's
local index lr * T + lc; 1-D tensors stay flat; block numbering is row-major.
"""
import numpy as np
import pytest

import oracle


def blocks(rows, cols, T):
    for bi in range((rows + T - 1) // T):
        for bj in range((cols + T - 1) // T):
            yield bi, bj


@pytest.mark.parametrize("rows,cols,T,kappa", [(8, 8, 4, 3), (9, 10, 4, 5), (4, 13, 4, 16), (7, 3, 4, 2),
                                               (130, 70, 64, 32), (64, 64, 64, 32), (65, 1, 64, 3)])
@pytest.mark.parametrize("quant", [True, False])
def test_tiled_equals_flat_oracle_on_numpy_blocks(rows, cols, T, kappa, quant):
    rng = np.random.default_rng(rows * 1000 + cols)
    few = np.array([0.0, 0.5, -0.5, 1.0, -1.0, 2.0, -3.0, 0.25], np.float32)
    delta = few[rng.integers(0, len(few), (rows, cols))] if rows < 20 else \
        (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    e0 = (rng.integers(-4, 5, (rows, cols)) / 8.0).astype(np.float32)
    e = e0.copy()
    pairs, aux = oracle.compress([e], kappa, 0.95, delta=[delta], tile=T, quant=quant)
    n_blocks = len(list(blocks(rows, cols, T)))
    assert oracle.num_chunks([(rows, cols)], tile=T) == n_blocks and pairs.size == n_blocks * kappa
    for c, (bi, bj) in enumerate(blocks(rows, cols, T)):
        sl = (slice(bi * T, min((bi + 1) * T, rows)), slice(bj * T, min((bj + 1) * T, cols)))
        h, w = delta[sl].shape
        eb = np.ascontiguousarray(e0[sl]).reshape(-1)
        db = np.ascontiguousarray(delta[sl]).reshape(-1)
        pb, ab = oracle.compress([eb], kappa, 0.95, delta=[db], chunk=T * T, quant=quant)
        idx_b, code_b, valid_b = oracle.unpack(pb)
        # flattened position inside the block -> local index of the tile
        local = (idx_b // w) * T + idx_b % w
        got = pairs[c * kappa:(c + 1) * kappa]
        idx_g, code_g, valid_g = oracle.unpack(got)
        assert np.array_equal(valid_g, valid_b)
        assert np.array_equal(idx_g[valid_g], local[valid_b]) and np.array_equal(code_g[valid_g], code_b[valid_b])
        if quant:
            assert np.array_equal(aux[2 * c:2 * c + 2].view(np.uint32), ab.view(np.uint32))
        else:
            assert np.array_equal(aux[c * kappa:(c + 1) * kappa].view(np.uint32), ab.view(np.uint32))
        assert np.array_equal(e[sl].reshape(-1).view(np.uint32), eb.view(np.uint32))


def test_one_dimensional_tensors_stay_flat_under_tiling():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(100) * 1e-3).astype(np.float32)
    ea, eb = np.zeros(100, np.float32), np.zeros(100, np.float32)
    pa, aa = oracle.compress([ea], 3, 0.95, delta=[x], tile=4)
    pb, ab = oracle.compress([eb], 3, 0.95, delta=[x], chunk=16)
    assert np.array_equal(pa, pb) and np.array_equal(aa, ab) and np.array_equal(ea, eb)


@pytest.mark.parametrize("quant", [True, False])
def test_tiled_aggregate_is_the_dense_mean_of_tiled_decodes(quant):
    rng = np.random.default_rng(4)
    shapes = [(9, 10), (1, 7), (70, 5)]
    T, kappa, R = 4, 3, 3
    pairs, aux, dense = [], [], []
    for r in range(R):
        e = [np.zeros(s, np.float32) for s in shapes]
        d = [(rng.standard_normal(s) * 1e-3).astype(np.float32) for s in shapes]
        p, a = oracle.compress(e, kappa, 1.0, delta=d, tile=T, quant=quant)
        dec = oracle.decode(shapes, p, a, kappa, tile=T, quant=quant)
        if not quant:
            # Q = identity: what was sent plus what stayed is the folded buffer, element by element
            for t in range(len(shapes)):
                assert np.array_equal(dec[t] + e[t].reshape(-1), d[t].reshape(-1))
        pairs.append(p), aux.append(a), dense.append(dec)
    got = oracle.aggregate(shapes, pairs, aux, kappa, tile=T, quant=quant)
    for t in range(len(shapes)):
        mean64 = sum(dense[r][t].astype(np.float64) for r in range(R)) / R
        assert np.allclose(got[t], mean64, rtol=1e-6, atol=1e-9)       # addends ~1e-3 may cancel
    assert sum(np.count_nonzero(x) for x in dense[0]) > 0
