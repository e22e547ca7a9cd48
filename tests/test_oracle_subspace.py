"""Pins for the oracle of the embedding re-projection (paper section 2.4):
closed forms that do not go through the oracle's own matmuls (a coordinate
subspace, a hand-computed rotation), and the identities the section states --
T_S + T_perp unchanged, T_S in the subspace afterwards, idempotence."""
import numpy as np

from oracle import subspace


def test_coordinate_subspace_closed_form():
    rng = np.random.default_rng(0)
    v, d, k = 7, 6, 2
    u = np.zeros((d, k))
    u[4, 0] = 1.0                      # S = span(e_4, e_1)
    u[1, 1] = 1.0
    ts, tp = rng.standard_normal((v, d)), rng.standard_normal((v, d))
    new_ts, new_tp = subspace.reproject(ts, tp, u)
    keep = np.zeros(d, bool)
    keep[[1, 4]] = True
    assert np.array_equal(new_ts[:, keep], ts[:, keep]) and not new_ts[:, ~keep].any()
    assert np.array_equal(new_tp[:, keep], tp[:, keep])
    assert np.array_equal(new_tp[:, ~keep], tp[:, ~keep] + ts[:, ~keep])


def test_hand_computed_line_in_the_plane():
    # S = span((3, 4) / 5): the projection of (5, 0) is (9/5, 12/5), the residual (16/5, -12/5)
    u = np.array([[0.6], [0.8]])
    new_ts, new_tp = subspace.reproject(np.array([[5.0, 0.0]]), np.array([[1.0, 1.0]]), u)
    assert np.allclose(new_ts, [[1.8, 2.4]], rtol=0, atol=1e-15)
    assert np.allclose(new_tp, [[4.2, -1.4]], rtol=0, atol=1e-15)


def test_identities_of_section_2_4():
    rng = np.random.default_rng(1)
    v, d, k = 50, 64, 8
    u = subspace.orthonormal_basis(d, k, seed=3)
    assert np.allclose(u.T @ u, np.eye(k), atol=1e-13)
    ts, tp = rng.standard_normal((v, d)), rng.standard_normal((v, d))
    new_ts, new_tp = subspace.reproject(ts, tp, u)
    assert np.allclose(new_ts + new_tp, ts + tp, atol=1e-13)           # TE is the same after the step
    assert np.allclose((ts - new_ts) @ u, 0, atol=1e-13)               # what was removed is orthogonal to S
    again_ts, again_tp = subspace.reproject(new_ts, new_tp, u)         # T_S is in S: a second step changes nothing
    assert np.allclose(again_ts, new_ts, atol=1e-13) and np.allclose(again_tp, new_tp, atol=1e-13)
    # initialisation before training: T_perp = 0
    init_ts, init_tp = subspace.reproject(ts, np.zeros_like(ts), u)
    assert np.allclose(init_ts, ts @ u @ u.T, atol=1e-13) and np.allclose(init_tp, ts - init_ts, atol=1e-13)
    # k = d: the subspace is everything
    full = subspace.orthonormal_basis(d, d, seed=4)
    f_ts, f_tp = subspace.reproject(ts, tp, full)
    assert np.allclose(f_ts, ts, atol=1e-12) and np.allclose(f_tp, tp, atol=1e-12)


def test_projection_of_activations_closed_forms():
    """Section 2.2: activations whose low-rank part lies in Col(U) survive project -> reconstruct unchanged;
    with a coordinate subspace the transmitted values are the selected columns of x minus the high-rank part."""
    rng = np.random.default_rng(2)
    rows, d, k, vocab, seq = 12, 10, 3, 7, 4
    tp, pos = rng.standard_normal((vocab, d)), rng.standard_normal((seq, d))
    tok = rng.integers(0, vocab, rows)
    u = np.zeros((d, k))
    cols = [7, 2, 5]
    u[cols, np.arange(k)] = 1.0
    x = rng.standard_normal((rows, d))
    xt = subspace.project(x, u, tp, tok, pos)
    high = tp[tok] + pos[np.arange(rows) % seq]
    assert np.allclose(xt, (x - high)[:, cols], rtol=0, atol=1e-15)
    xh = subspace.reconstruct(xt, u, tp, tok, pos)
    assert np.allclose(xh[:, cols], x[:, cols], atol=1e-14)
    rest = np.setdiff1d(np.arange(d), cols)
    assert np.allclose(xh[:, rest], high[:, rest], atol=1e-15)
    # lossless when the residual activations live in the subspace
    q = subspace.orthonormal_basis(d, k, seed=9)
    x_in = rng.standard_normal((rows, k)) @ q.T + high
    assert np.allclose(subspace.reconstruct(subspace.project(x_in, q, tp, tok, pos), q, tp, tok, pos), x_in, atol=1e-13)
    # backward: plain product
    g = rng.standard_normal((rows, d))
    assert np.allclose(subspace.project(g, u), g[:, cols], rtol=0, atol=0)


def test_heterogeneous_aggregation_bias_identity():
    """Section 2.4, "Analysis of heterogeneous aggregation": with a fraction alpha of replicas sending
    the unbiased pseudo-gradient D* and the rest its projection Pi_S(D*), the aggregate is
    D* - (1 - alpha) B with B = D* - Pi_S(D*).  Checked through the outer-step oracle with everything
    sent (kappa = chunk, Q = identity), where the mean is the plain mean of the messages."""
    import oracle
    rng = np.random.default_rng(8)
    rows, d, k, M, n_full = 16, 16, 4, 8, 2                 # alpha = 2 / 8
    u = subspace.orthonormal_basis(d, k, seed=1)
    d_star = rng.standard_normal((rows, d))
    d_proj, _ = subspace.reproject(d_star, np.zeros_like(d_star), u)        # Pi_S(D*)
    bias = d_star - d_proj
    pairs, values = [], []
    for m in range(M):
        delta = (d_star if m < n_full else d_proj).astype(np.float32).reshape(-1)
        e = np.zeros(rows * d, np.float32)
        p, v = oracle.compress([e], rows * d, 0.95, delta=[delta], chunk=rows * d, quant=False)
        assert not e.any()
        pairs.append(p), values.append(v)
    mean = oracle.aggregate([rows * d], pairs, values, rows * d, chunk=rows * d, quant=False)[0].reshape(rows, d)
    alpha = n_full / M
    assert np.allclose(mean, d_star - (1 - alpha) * bias, atol=1e-6)
    assert np.allclose(mean, alpha * d_star + (1 - alpha) * d_proj, atol=1e-6)
