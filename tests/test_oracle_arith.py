"""Pins for the oracle's floating-point steps (paper section 2.1 update
equations): pseudo-gradient, error-feedback fold, residual, mean over replicas
and the outer SGD update.  Expected values come from exact rational arithmetic
with an explicit model of binary32 rounding (tests/exact32.py), from values that
are exactly representable, and from conservation laws -- not from re-running the
same float formula.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from exact32 import F, bits, f32, rn

BETA = np.float32(0.95)


def send_everything(e0, beta, **src):
    """kappa = n_c and Q = identity: the message is the folded buffer itself."""
    n = e0.size
    e = e0.copy()
    pairs, values = oracle.compress([e], n, beta, chunk=n, quant=False, **src)
    idx, _, valid = oracle.unpack(pairs)
    assert valid.all() and idx.tolist() == list(range(n))
    return values, e


def test_fold_is_two_roundings_not_a_fused_multiply_add():
    rng = np.random.default_rng(3)
    n = 512
    e0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    theta_o = (rng.standard_normal(n) * 0.02).astype(np.float32)
    theta_l = (theta_o - (rng.standard_normal(n) * 1e-3).astype(np.float32)).astype(np.float32)
    values, e_after = send_everything(e0, float(BETA), theta_outer=[theta_o], theta_local=[theta_l])
    n_fma_differs = 0
    for i in range(n):
        delta = rn(F(theta_o[i]) - F(theta_l[i]))                      # pseudo-gradient: outer minus local
        want = rn(rn(F(BETA) * F(e0[i])) + delta)
        fused = rn(F(BETA) * F(e0[i]) + delta)
        n_fma_differs += want != fused
        assert Fraction(float(values[i])) == want, i
    assert n_fma_differs > 10            # the inputs do tell the two evaluation orders apart
    assert not e_after.any()             # e' - e' = 0 at every sent position


def test_pseudo_gradient_sign_is_outer_minus_local():
    theta_o = np.array([1.0, 2.0, -3.0, 0.5], np.float32)
    theta_l = np.array([0.75, 2.5, -3.0, 0.5], np.float32)
    values, _ = send_everything(np.zeros(4, np.float32), 0.0, theta_outer=[theta_o], theta_local=[theta_l])
    assert values.tolist() == [0.25, -0.5, 0.0, 0.0]


def test_fold_exact_cases_and_momentum_factor():
    e0 = np.array([1.0, -2.0, 4.0, 0.0], np.float32)
    delta = np.array([0.25, 0.5, -1.0, 8.0], np.float32)
    values, _ = send_everything(e0, 0.5, delta=[delta])
    assert values.tolist() == [0.75, -0.5, 1.0, 8.0]
    values, _ = send_everything(e0, 0.0, delta=[delta])
    assert values.tolist() == delta.tolist()
    values, _ = send_everything(e0, 1.0, delta=[np.zeros(4, np.float32)])
    assert values.tolist() == e0.tolist()


def test_bf16_delta_is_widened_exactly():
    raw = np.array([0x3F80, 0xBF80, 0x3A83, 0x0000, 0x8000, 0x0001, 0x7F7F], np.uint16)   # 1, -1, ~1e-3, +0, -0, tiny, max
    values, _ = send_everything(np.zeros(raw.size, np.float32), 0.0, delta=[raw])
    # beta*e = +0; +0 + (-0) = +0 in round-to-nearest
    want = (raw.astype(np.uint32) << 16)
    want[4] = 0
    assert np.array_equal(values.view(np.uint32), want)


def test_denormals_are_kept():
    tiny = np.array([1, 2, 0x7FFFFF], np.uint32).view(np.float32)       # subnormals
    values, _ = send_everything(tiny.copy(), 1.0, delta=[np.zeros(3, np.float32)])
    assert np.array_equal(values.view(np.uint32), tiny.view(np.uint32))
    # and they take part in the ranking: the larger subnormal wins a kappa = 1 selection
    e = tiny.copy()
    pairs, _ = oracle.compress([e], 1, 1.0, delta=[np.zeros(3, np.float32)], chunk=3, quant=False)
    assert oracle.unpack(pairs)[0].tolist() == [2]


@pytest.mark.parametrize("quant", [False, True])
def test_error_feedback_conserves_what_was_not_sent(quant):
    """beta = 1: sum_t decoded_t + e_T = e_0 + sum_t delta_t (paper section 2.1:
    the accumulator preserves discarded pseudo-gradient information).  Exactly
    representable dyadic inputs keep every sum exact, so equality is bit-exact."""
    rng = np.random.default_rng(11)
    chunk, kappa, n, T = 64, 4, 64 * 3 + 17, 6
    e = (rng.integers(-64, 65, n) / 64.0).astype(np.float32)
    total_in = e.astype(np.float64).copy()
    total_sent = np.zeros(n, np.float64)
    for t in range(T):
        delta = (rng.integers(-64, 65, n) / 64.0).astype(np.float32)
        total_in += delta
        pairs, aux = oracle.compress([e], kappa, 1.0, delta=[delta], chunk=chunk, quant=quant)
        total_sent += oracle.decode([n], pairs, aux, kappa, chunk=chunk, quant=quant)[0]
    assert np.array_equal(total_sent + e, total_in)


def test_mean_divides_by_all_replicas_and_sums_in_replica_order():
    # unquantised messages let the test choose the addends
    n, kappa, chunk = 8, 1, 8
    def msg(idx, v):
        return np.array([idx], np.uint16), np.array([v], np.float32)
    # index 2: 1e8, 1, -1e8 in replica order -> (1e8 + 1) rounds to 1e8, minus 1e8 = 0; other orders give 1/3
    # index 5: only one of three replicas sends 3.0 -> mean 1.0 (divide by M, not by the contributor count)
    (p0, v0), (p1, v1), (p2, v2) = msg(2, 1e8), msg(2, 1.0), msg(2, -1e8)
    out = oracle.aggregate([n], [p0, p1, p2], [v0, v1, v2], kappa, chunk=chunk, quant=False)[0]
    assert out[2] == 0.0 and not out.any()
    (p0, v0), (p1, v1), (p2, v2) = msg(5, 3.0), msg(0, 0.0), msg(1, 0.0)
    out = oracle.aggregate([n], [p0, p1, p2], [v0, v1, v2], kappa, chunk=chunk, quant=False)[0]
    assert out.tolist() == [0, 0, 0, 0, 0, 1.0, 0, 0]
    # one IEEE division, not a multiplication by a rounded reciprocal: 5/3 and 7/3 differ between the two
    vals = np.float32([5.0, 7.0, 11.0, 13.0])
    for v in vals:
        (p0, v0), (p1, v1), (p2, v2) = msg(3, v), msg(0, 0.0), msg(1, 0.0)
        out = oracle.aggregate([n], [p0, p1, p2], [v0, v1, v2], kappa, chunk=chunk, quant=False)[0]
        assert Fraction(float(out[3])) == rn(F(v) / 3)


@pytest.mark.parametrize("quant", [False, True])
@pytest.mark.parametrize("R", [1, 2, 3, 8])
def test_aggregate_equals_dense_mean_of_decoded_messages(quant, R):
    rng = np.random.default_rng(5 + R)
    chunk, kappa = 64, 8
    numels = [64 * 4, 100, 7]
    pairs, aux, dense = [], [], []
    for r in range(R):
        e = [(rng.standard_normal(n) * 1e-4).astype(np.float32) for n in numels]
        d = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for n in numels]
        p, a = oracle.compress(e, kappa, 0.95, delta=d, chunk=chunk, quant=quant)
        pairs.append(p), aux.append(a)
        dense.append(oracle.decode(numels, p, a, kappa, chunk=chunk, quant=quant))
    got = oracle.aggregate(numels, pairs, aux, kappa, chunk=chunk, quant=quant)
    for t, n in enumerate(numels):
        mean64 = sum(dense[r][t].astype(np.float64) for r in range(R)) / R
        assert np.allclose(got[t], mean64, rtol=2e-7 * R, atol=1e-12)
        if R == 1:
            assert np.array_equal(got[t], dense[0][t])
    # two identical replicas: x + x and the halving are both exact, so the mean is the message itself
    # (for more replicas the running sum 3x, 5x, ... already rounds, so this holds for M = 2 only)
    if R == 2:
        same = oracle.aggregate(numels, [pairs[0]] * R, [aux[0]] * R, kappa, chunk=chunk, quant=quant)
        for t in range(len(numels)):
            assert np.array_equal(same[t], dense[0][t])


def test_outer_update_is_theta_minus_lr_times_mean():
    rng = np.random.default_rng(9)
    n = 300
    theta = (rng.standard_normal(n) * 0.02).astype(np.float32)
    dbar = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    dbar[::3] = 0
    for lr in (1.0, 0.8):
        th = theta.copy()
        oracle.outer_update([th], [dbar], lr)
        lr32 = np.float32(lr)
        for i in range(n):
            want = rn(F(theta[i]) - rn(F(lr32) * F(dbar[i])))
            assert Fraction(float(th[i])) == want
        assert np.array_equal(th[::3].view(np.uint32), theta[::3].view(np.uint32))     # untouched where the mean is zero
    th = np.array([1.0, -2.0], np.float32)
    oracle.outer_update([th], [np.array([0.25, -0.5], np.float32)], 1.0)
    assert th.tolist() == [0.75, -1.5]                                                # descent direction: minus


def test_beta_is_the_binary32_nearest_to_0_95():
    assert bits(BETA) == 0x3F733333
    e0 = np.array([3.0], np.float32)
    values, _ = send_everything(e0, 0.95, delta=[np.zeros(1, np.float32)])
    assert Fraction(float(values[0])) == rn(Fraction(0x733333 + 0x800000, 2 ** 24) * 3)
    assert f32(rn(Fraction(0x733333 + 0x800000, 2 ** 24) * 3)) == values[0]


def test_heterogeneous_mean_carries_the_predicted_bias():
    """The analysis of heterogeneous aggregation (end of section 2.4): with a fraction alpha of the replicas
    sending the unbiased pseudo-gradient D and the others its projection onto a subspace, the mean is
    D - (1 - alpha) B with B = D - proj(D).  Checked through the oracle's own compress (Q = identity, kappa = chunk,
    so that every entry is sent) and aggregate; D, its projection and the mean are exact in binary32 here
    (small dyadic values, M a power of two), so the identity must hold bit for bit."""
    rng = np.random.default_rng(11)
    n, chunk, M, n_full = 64, 16, 8, 2                       # alpha = 2/8
    d_star = (rng.integers(-64, 65, n) / 64.0).astype(np.float32)
    keep = np.arange(n) % 4 == 0                             # projection onto a coordinate subspace: exact
    d_proj = np.where(keep, d_star, 0).astype(np.float32)
    bias = (d_star - d_proj).astype(np.float32)
    pairs, vals = [], []
    for m in range(M):
        ef = [np.zeros(n, np.float32)]
        p, v = oracle.compress(ef, chunk, 1.0, delta=[d_star if m < n_full else d_proj], chunk=chunk, quant=False)
        assert not ef[0].any()                               # everything was sent: the buffer is empty again
        pairs.append(p), vals.append(v)
    mean = oracle.aggregate([n], pairs, vals, chunk, chunk=chunk, quant=False)[0]
    alpha = n_full / M
    assert np.array_equal(mean, (d_star - (1 - alpha) * bias).astype(np.float32))
    assert np.array_equal(mean, (alpha * d_star + (1 - alpha) * d_proj).astype(np.float32))
