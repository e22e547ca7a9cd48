"""Pins for the oracle's chunk-wise Top-kappa (paper section 2.1: "retains only
the kappa largest-magnitude elements per chunk"), independent of the oracle's
own sort: brute force by a stable numpy argsort, a library top-k on tie-free
data, the definition's invariants, and the special cases kappa = 1 and
kappa >= n_c.  The unquantised mode is used so that the sent values are the
selected entries of the folded buffer themselves.
"""
import numpy as np
import pytest
import torch

import oracle


def fold_np(e, delta, beta):
    return (np.float32(beta) * e + delta).astype(np.float32)


def brute_force_select(eprime, chunk, kappa):
    """Indices kept per chunk: stable sort of -|x| keeps the lower index first among equals."""
    out = []
    for base in range(0, eprime.size, chunk):
        x = eprime[base:base + chunk]
        key = (x.view(np.uint32) & 0x7FFFFFFF).astype(np.int64)
        order = np.argsort(-key, kind="stable")
        out.append(np.sort(order[:min(kappa, x.size)]))
    return out


def run_unquantised(e0, delta, kappa, beta, chunk):
    e = e0.copy()
    pairs, values = oracle.compress([e], kappa, beta, delta=[delta], chunk=chunk, quant=False)
    return e, pairs, values


@pytest.mark.parametrize("chunk,kappa,n", [(8, 3, 8), (8, 3, 29), (16, 5, 16 * 7 + 3), (64, 32, 64 * 5 + 1),
                                           (8, 1, 40), (8, 8, 21), (8, 12, 21), (64, 7, 6)])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_matches_brute_force_with_ties(chunk, kappa, n, seed):
    rng = np.random.default_rng(1000 * seed + chunk + kappa)
    # few distinct magnitudes, both signs, exact zeros of both signs: ties everywhere
    vals = np.array([0.0, -0.0, 0.5, -0.5, 1.0, -1.0, 2.0, 3.0, -3.0], np.float32)
    delta = vals[rng.integers(0, len(vals), n)]
    e0 = np.zeros(n, np.float32)
    e, pairs, values = run_unquantised(e0, delta, kappa, 0.95, chunk)
    eprime = fold_np(e0, delta, 0.95)
    want = brute_force_select(eprime, chunk, kappa)
    idx, code, valid = oracle.unpack(pairs)
    for c, w in enumerate(want):
        got = idx[c * kappa:(c + 1) * kappa][valid[c * kappa:(c + 1) * kappa]]
        assert np.array_equal(got, w), (c, got, w)
        assert valid[c * kappa:c * kappa + len(w)].all() and not valid[c * kappa + len(w):(c + 1) * kappa].any()
        sent = values[c * kappa:c * kappa + len(w)]
        assert np.array_equal(sent.view(np.uint32), eprime[c * chunk + w].view(np.uint32))


@pytest.mark.parametrize("kappa", [1, 32, 64, 128])
def test_matches_library_topk_on_tie_free_data(kappa):
    chunk, n_chunks = 4096, 6
    g = torch.Generator().manual_seed(7)
    x = torch.randn(n_chunks * chunk, generator=g, dtype=torch.float32)
    mag = x.abs().view(n_chunks, chunk)
    top = torch.sort(mag, dim=1, descending=True).values
    assert torch.all(top[:, kappa - 1] > top[:, kappa])               # no tie at the cut, so the set is unique
    lib = torch.topk(mag, kappa, dim=1).indices.sort(dim=1).values.numpy()
    e0 = np.zeros(x.numel(), np.float32)
    e, pairs, values = run_unquantised(e0, x.numpy(), kappa, 0.0, chunk)
    idx, _, valid = oracle.unpack(pairs)
    assert valid.all()
    assert np.array_equal(idx.reshape(n_chunks, kappa), lib)


def test_kappa_one_is_first_argmax_and_full_kappa_is_identity():
    chunk = 16
    x = np.array([1, -7, 3, 7, 0, -7, 2, 2, 5, 5, 5, 5, 5, 5, 5, 5, 9, -9], np.float32)
    e, pairs, values = run_unquantised(np.zeros_like(x), x, 1, 1.0, chunk)
    idx, _, valid = oracle.unpack(pairs)
    assert idx.tolist() == [1, 0] and valid.all()          # |-7| at index 1 beats the equal 7 at 3; 9 at 0 beats -9
    assert values.tolist() == [-7.0, 9.0]
    e, pairs, values = run_unquantised(np.zeros_like(x), x, 16, 1.0, chunk)
    idx, _, valid = oracle.unpack(pairs)
    assert idx[:16].tolist() == list(range(16)) and valid[:16].all()
    assert idx[16:18].tolist() == [0, 1] and valid[16:18].all() and not valid[18:].any()
    assert np.all(pairs[18:] == 0xFFFF)
    assert np.array_equal(values[:16], x[:16]) and np.array_equal(values[16:18], x[16:])
    assert not e.any()                                      # everything was sent exactly


def test_definition_invariants_on_config0_like_tensor():
    """Exactly kappa distinct ascending in-range indices per chunk; no unselected
    entry beats a selected one; among equals the selected have the lower indices;
    the paper's density figure 32/4096 = 0.78 %."""
    chunk, kappa, n = 4096, 32, 4096 * 64
    g = torch.Generator().manual_seed(0)
    theta_o = (0.02 * torch.randn(n, generator=g)).numpy()
    theta_l = (torch.from_numpy(theta_o) - 1e-3 * torch.randn(n, generator=g)).numpy()
    e0 = (1e-4 * torch.randn(n, generator=g)).numpy()
    # plant ties and zeros
    theta_l[5:4096:97] = theta_o[5:4096:97]
    e0[5:4096:97] = 0
    e = e0.copy()
    pairs, values = oracle.compress([e], kappa, 0.95, theta_outer=[theta_o], theta_local=[theta_l],
                                    chunk=chunk, quant=False)
    idx, code, valid = oracle.unpack(pairs)
    assert valid.all() and not code.any()
    assert abs(valid.sum() / n - 0.0078125) < 1e-12 and round(100 * kappa / chunk, 2) == 0.78
    eprime = fold_np(e0, (theta_o - theta_l).astype(np.float32), 0.95)
    key = eprime.view(np.uint32) & 0x7FFFFFFF
    for c in range(n // chunk):
        sel = idx[c * kappa:(c + 1) * kappa].astype(np.int64)
        assert np.all(np.diff(sel) > 0) and sel[0] >= 0 and sel[-1] < chunk
        k = key[c * chunk:(c + 1) * chunk]
        mask = np.zeros(chunk, bool)
        mask[sel] = True
        thr = k[mask].min()
        assert thr >= k[~mask].max()
        eq_sel = np.nonzero(mask & (k == thr))[0]
        eq_uns = np.nonzero(~mask & (k == thr))[0]
        if len(eq_uns):
            assert eq_sel.max() < eq_uns.min()
        # unselected entries of the buffer are the folded values, bit for bit; sent ones are zero
        assert np.array_equal(e[c * chunk:(c + 1) * chunk][~mask].view(np.uint32),
                              eprime[c * chunk:(c + 1) * chunk][~mask].view(np.uint32))
        assert not e[c * chunk:(c + 1) * chunk][mask].any()


def test_zeros_are_selected_lowest_index_first_when_nonzeros_run_out():
    chunk, kappa = 32, 6
    x = np.zeros(32, np.float32)
    x[20] = -1.5
    x[9] = 0.25
    x[3] = -0.0
    e, pairs, values = run_unquantised(np.zeros_like(x), x, kappa, 1.0, chunk)
    idx, _, valid = oracle.unpack(pairs)
    assert idx.tolist() == [0, 1, 2, 3, 9, 20] and valid.all()
