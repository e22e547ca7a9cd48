"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on seeded inputs spanning several chunks and ragged tails, every
source mode, both quantiser modes, both selection algorithms, and the
degenerate cases (ties, zeros, constant chunks, denormals, kappa >= n_c)."""
import numpy as np
import pytest
import torch

from paper_2601_02360_amd import binding as B
from paper_2601_02360_amd import workloads as W

import parity

pytestmark = pytest.mark.gpu

RAGGED = [4096 * 5, 4096 * 3 + 17, 100, 4096, 1, 2047, 4096 * 2 + 4, 0, 4096 * 2 - 1]


TILED_SHAPES = [(128, 192), (130, 70), (64, 64), (1, 5000), (63, 65), (200, 3), (3, 200), (65, 129), (1, 1), (70, 66)]


# matrices wide enough for strips (four complete tiles taken by one workgroup), with leftovers and edges around them
STRIP_SHAPES = [(128, 1030), (64, 264), (70, 520), (200, 322), (130, 254), (64, 513), (1, 3000), (66, 2050), (3, 258),
                (65, 450)]


def gaussian_case(numels, R, seed, direct=None, heavy=False, shapes=None):
    """shapes: run with the 64 x 64 tile layout over these (rows, cols) matrices instead of flat chunks."""
    if shapes is not None:
        numels = [r * c for r, c in shapes]
    rng = np.random.default_rng(seed)
    draw = (lambda n: rng.standard_t(3, n)) if heavy else (lambda n: rng.standard_normal(n))
    th = [(rng.standard_normal(n) * 0.02).astype(np.float32) for n in numels]
    ef = [[(rng.standard_normal(n) * 1e-4).astype(np.float32) for n in numels] for _ in range(R)]
    deltas = [[(draw(n) * 1e-3).astype(np.float32) for n in numels] for _ in range(R)]
    if direct is None:
        tl = [[(th[t] - deltas[r][t]).astype(np.float32) for t in range(len(numels))] for r in range(R)]
        return parity.HostCase(th, ef, theta_local=tl, shapes=shapes)
    if direct == "bf16":
        deltas = [[(d.view(np.uint32) >> 16).astype(np.uint16) for d in r] for r in deltas]
    return parity.HostCase(th, ef, delta=deltas, shapes=shapes)


@pytest.mark.parametrize("select", [B.SPLC_SELECT_AUTO, B.SPLC_SELECT_RADIX])
@pytest.mark.parametrize("kappa", [1, 32, 64, 128, 256, 300, 4096])
def test_ragged_tensor_list_params_mode(kappa, select):
    case = gaussian_case(RAGGED, R=3, seed=kappa)
    parity.check(case, kappa, select=select, what="ragged kappa=%d" % kappa)


@pytest.mark.parametrize("select", [B.SPLC_SELECT_AUTO, B.SPLC_SELECT_RADIX])
@pytest.mark.parametrize("kappa", [1, 32, 64, 200, 4096])
def test_tiled_layout_params_mode(kappa, select):
    """64 x 64 tiles: full tiles, edge tiles on both sides, column counts that are odd or not
    multiples of four, 1-D tensors, tiles smaller than kappa."""
    case = gaussian_case(None, R=3, seed=300 + kappa, shapes=TILED_SHAPES)
    parity.check(case, kappa, select=select, what="tiled kappa=%d" % kappa)


@pytest.mark.parametrize("select", [B.SPLC_SELECT_AUTO, B.SPLC_SELECT_RADIX])
@pytest.mark.parametrize("kappa", [1, 32, 64, 200, 300])
def test_tiled_layout_with_strips(kappa, select):
    """Runs of four complete tiles go to one 1024-lane workgroup: row lengths that are and are not multiples of
    32 floats, leftover tiles at the end of a tile row, edge tiles below and to the right, odd row lengths (no
    strips), with both selection algorithms and wide messages."""
    case = gaussian_case(None, R=3, seed=700 + kappa, shapes=STRIP_SHAPES)
    parity.check(case, kappa, select=select, what="strips kappa=%d" % kappa)


@pytest.mark.parametrize("direct,quant,fused", [("f32", True, None), ("bf16", True, "no_mean"), ("bf16", False, "with_mean"),
                                                (None, False, "with_mean")])
def test_tiled_layout_with_strips_modes(direct, quant, fused):
    case = gaussian_case(None, R=9, seed=731, direct=direct, heavy=True, shapes=STRIP_SHAPES)
    parity.check(case, 48, lr=0.8, quant=quant, fused=fused, outer_steps=2, what="strips %s quant=%s" % (direct, quant))


def test_strip_with_one_degenerate_tile():
    """Inside one strip, one tile is constant (a 4096-way tie: the candidate filter gives up and the radix
    select runs), one is all zero, one has few distinct values and one is ordinary: the four groups of the
    workgroup must agree on the path and each still get its own tile right."""
    rng = np.random.default_rng(9)
    rows, cols = 64, 2 * 256 + 70
    x = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    x[:, 0:64] = -7.25
    x[:, 64:128] = 0.0
    x[:, 128:192] = (rng.integers(0, 3, (rows, 64)) * 0.125).astype(np.float32)
    x[:, 256 + 64:256 + 128] = 3.0                       # second strip: one constant tile among ordinary ones
    y = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    th = [np.zeros(rows * cols, np.float32)]
    ef = [[np.zeros(rows * cols, np.float32)] for _ in range(2)]
    case = parity.HostCase(th, ef, delta=[[x.reshape(-1)], [y.reshape(-1)]], shapes=[(rows, cols)])
    for kappa in (1, 32, 200):
        parity.check(case, kappa, beta=1.0, what="degenerate strip kappa=%d" % kappa)
        parity.check(case, kappa, beta=1.0, quant=False, fused="with_mean", what="degenerate strip, identity, kappa=%d" % kappa)


@pytest.mark.parametrize("direct,quant", [("f32", True), ("bf16", True), ("bf16", False)])
def test_tiled_layout_direct_modes(direct, quant):
    case = gaussian_case(None, R=2, seed=331, direct=direct, heavy=True, shapes=TILED_SHAPES)
    parity.check(case, 32, quant=quant, fused="no_mean", outer_steps=2, what="tiled direct %s" % direct)


@pytest.mark.parametrize("shapes", [TILED_SHAPES, STRIP_SHAPES], ids=["small", "strips"])
def test_tiled_layout_batched_and_fused(shapes):
    case = gaussian_case(None, R=5, seed=337, shapes=shapes)
    parity.check(case, 64, batch=True, fused="with_mean", outer_steps=2, what="tiled batched")


def test_four_byte_aligned_views():
    """Tensor pointers need only 4-byte alignment: views that start one element into an allocation."""
    import torch
    from paper_2601_02360_amd import binding
    rng = np.random.default_rng(41)
    n = 4096 * 3 + 10
    host = [(rng.standard_normal(n) * s).astype(np.float32) for s in (0.02, 0.02, 1e-4)]
    host[1] = (host[0] - (rng.standard_normal(n) * 1e-3).astype(np.float32)).astype(np.float32)
    case = parity.HostCase([host[0]], [[host[2]]], theta_local=[[host[1]]])
    want = parity.run_oracle(case, 32, 0.95, 1.0)
    bufs = [torch.zeros(n + 1, device="cuda") for _ in range(4)]
    views = [b[1:] for b in bufs]
    for v, h in zip(views, host):
        v.copy_(torch.from_numpy(h))
    assert all(v.data_ptr() % 16 == 4 for v in views)
    plan = binding.Plan([n], 32)
    p, a = plan.message_buffers()
    binding.sparseloco_compress(plan, [views[2]], p, a, 0.95, theta_outer=[views[0]], theta_local=[views[1]])
    binding.sparseloco_aggregate(plan, [p], [views[3]], aux=[a])
    binding.sparseloco_outer_update(plan, [views[0]], [views[3]], 1.0)
    torch.cuda.synchronize()
    got = [dict(pairs=[parity.to_np(p)], aux=[parity.to_np(a)], ef=[[parity.to_np(views[2])]],
                dbar=[parity.to_np(views[3])], theta=[parity.to_np(views[0])])]
    parity.compare(got, want, "4-byte aligned views")
    plan.close()


@pytest.mark.parametrize("quant", [True, False])
@pytest.mark.parametrize("direct", ["f32", "bf16"])
def test_direct_modes_and_identity_quantiser(direct, quant):
    case = gaussian_case(RAGGED, R=2, seed=17, direct=direct, heavy=True)
    parity.check(case, 64, quant=quant, what="direct %s quant=%s" % (direct, quant))


@pytest.mark.parametrize("quant", [True, False])
def test_identity_quantiser_params_mode_two_steps(quant):
    case = gaussian_case([4096 * 4 + 5, 777], R=4, seed=5)
    parity.check(case, 32, lr=0.8, quant=quant, outer_steps=2, what="two steps")


@pytest.mark.parametrize("select", [B.SPLC_SELECT_AUTO, B.SPLC_SELECT_RADIX])
def test_ties_zeros_and_constant_chunks(select):
    rng = np.random.default_rng(3)
    n_chunks = 12
    n = 4096 * n_chunks + 1000
    x = np.zeros(n, np.float32)
    few = np.array([0.0, -0.0, 0.5, -0.5, 1.0, -1.0, 2.0, 3.0, -3.0], np.float32)
    x[:4096 * 4] = few[rng.integers(0, len(few), 4096 * 4)]           # few distinct magnitudes: ties everywhere
    x[4096 * 4:4096 * 5] = 0.0                                          # all zero
    x[4096 * 5:4096 * 6] = -7.25                                        # constant: 4096-way tie
    x[4096 * 6:4096 * 7] = 0.0
    x[4096 * 6 + np.array([5, 900, 4000])] = [1.0, -2.0, 3.0]           # fewer non-zeros than kappa
    x[4096 * 7:4096 * 8] = np.array([1, 2, 3, 0x7FFFFF] * 1024, np.uint32).view(np.float32)   # subnormals
    x[4096 * 8:4096 * 9] = (rng.integers(0, 3, 4096) * 0.125).astype(np.float32)              # ~1365-way ties
    x[4096 * 9:] = (rng.standard_normal(n - 4096 * 9) * 1e-3).astype(np.float32)
    # bf16-rounded values and a zero mask: ties at the threshold are common
    y = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    y = ((y.view(np.uint32) >> 16) << 16).view(np.float32) * (rng.random(n) < 0.5)
    th = [np.zeros(n, np.float32), np.zeros(n, np.float32)]
    ef = [[np.zeros(n, np.float32), np.zeros(n, np.float32)] for _ in range(2)]
    deltas = [[x, y.astype(np.float32)], [y.astype(np.float32), x]]
    case = parity.HostCase(th, ef, delta=deltas)
    for kappa in (1, 32, 64, 200):
        parity.check(case, kappa, beta=1.0, select=select, what="ties kappa=%d" % kappa)


@pytest.mark.parametrize("fused", ["with_mean", "no_mean"])
@pytest.mark.parametrize("kappa,R,quant", [(32, 3, True), (64, 8, True), (128, 9, True), (200, 2, True),
                                           (300, 5, True), (64, 17, False), (4096, 2, True)])
def test_fused_aggregate_update(kappa, R, quant, fused):
    case = gaussian_case(RAGGED, R=R, seed=100 + kappa + R)
    parity.check(case, kappa, lr=0.8, quant=quant, fused=fused, outer_steps=2, what="fused %s" % fused)


@pytest.mark.parametrize("select", [B.SPLC_SELECT_AUTO, B.SPLC_SELECT_RADIX])
@pytest.mark.parametrize("kappa,R,quant", [(32, 1, True), (64, 8, True), (128, 5, False), (300, 3, True)])
def test_batched_compress_matches_the_oracle(kappa, R, quant, select):
    case = gaussian_case(RAGGED, R=R, seed=200 + kappa + R, heavy=True)
    parity.check(case, kappa, quant=quant, select=select, batch=True, outer_steps=2, what="batched compress")


@pytest.mark.parametrize("select", [B.SPLC_SELECT_AUTO, B.SPLC_SELECT_RADIX])
@pytest.mark.parametrize("kappa,R,quant,fused", [(32, 1, True, "with_mean"), (64, 8, True, "no_mean"),
                                                 (128, 5, False, "with_mean"), (300, 3, True, "no_mean"),
                                                 (4096, 2, False, "with_mean"), (1, 9, True, "with_mean")])
def test_one_launch_outer_step_matches_the_oracle(kappa, R, quant, fused, select):
    case = gaussian_case(RAGGED, R=R, seed=900 + kappa + R, heavy=True)
    parity.check(case, kappa, lr=0.8, quant=quant, select=select, batch="step", fused=fused, outer_steps=2,
                 what="one-launch step")


@pytest.mark.parametrize("shapes", [TILED_SHAPES, STRIP_SHAPES], ids=["small", "strips"])
def test_one_launch_outer_step_tiled(shapes):
    case = gaussian_case(None, R=5, seed=937, shapes=shapes)
    parity.check(case, 64, batch="step", fused="with_mean", outer_steps=2, what="tiled one-launch step")


@pytest.mark.parametrize("R", [33, 64])
def test_one_launch_outer_step_many_replicas(R):
    case = gaussian_case([4096 * 2 + 77, 300], R=R, seed=960 + R, heavy=True)
    parity.check(case, 32, batch="step", fused="with_mean", what="one-launch step R=%d" % R)


def test_one_launch_outer_step_equals_the_two_calls_and_resets():
    """Bit for bit the outputs of sparseloco_compress_batch + sparseloco_aggregate_update (ties, zeros and constant
    chunks included), and with reset every participating theta_local becomes the new theta_outer while a further
    set of the binding is left alone."""
    rng = np.random.default_rng(77)
    numels = RAGGED + [4096 * 3]
    th = [(rng.standard_normal(n) * 0.02).astype(np.float32) for n in numels]
    R = 4
    tl = [[(th[t] - np.round(rng.standard_normal(n) * 3).astype(np.float32) * 2.0 ** -12).astype(np.float32)
           for t, n in enumerate(numels)] for _ in range(R)]                      # few distinct values: many ties
    for r in range(R):
        tl[r][-1][:4096] = th[-1][:4096]                                          # an all-zero chunk
    ef = [[np.zeros(n, np.float32) for n in numels] for _ in range(R)]
    for quant in (True, False):
        plan = B.Plan(numels, 32, quant)
        outs = []
        for one_launch in (False, True):
            g_th = [parity._dev(x) for x in th]
            g_ef = [[parity._dev(x) for x in r] for r in ef]
            g_tl = [[parity._dev(x) for x in r] for r in tl]
            msgs = [plan.message_buffers() for _ in range(R)]
            b_msgs = plan.bind_messages([m[0] for m in msgs], [m[1] for m in msgs])
            b_tl = plan.bind(g_tl)
            dbar = [torch.full((n,), float("nan"), device="cuda") for n in numels]
            if one_launch:
                B.sparseloco_outer_step_batch(plan, g_th, b_tl, g_ef, b_msgs, 0.95, 0.7, delta_bar_out=dbar, reset=True,
                                              n_replicas=R - 1)
            else:
                B.sparseloco_compress_batch(plan, g_th, b_tl, g_ef, b_msgs, 0.95, n_replicas=R - 1)
                first = plan.bind_messages([m[0] for m in msgs[:R - 1]], [m[1] for m in msgs[:R - 1]])
                B.sparseloco_aggregate_update(plan, first, g_th, 0.7, delta_bar_out=dbar, reset=g_tl[:R - 1])
            torch.cuda.synchronize()
            outs.append([parity.to_np(x).tobytes() for x in g_th + dbar + [x for r in g_ef[:R - 1] for x in r]
                         + [x for m in msgs[:R - 1] for x in m] + [x for r in g_tl for x in r]])
            if one_launch:
                for t in range(len(numels)):
                    new = parity.to_np(g_th[t]).tobytes()
                    assert all(parity.to_np(g_tl[r][t]).tobytes() == new for r in range(R - 1))
                    assert parity.to_np(g_tl[R - 1][t]).tobytes() == tl[R - 1][t].tobytes()
        assert outs[0] == outs[1]
        plan.close()


def test_fused_update_resets_the_replicas():
    """sparseloco_aggregate_update with reset tables: every theta_local becomes the new theta_outer, bit for
    bit, on flat and tiled layouts, full and edge chunks."""
    import torch
    for shapes in (None, TILED_SHAPES + STRIP_SHAPES[:4]):
        case = gaussian_case(RAGGED, R=3, seed=401, shapes=shapes)
        want = parity.run_oracle(case, 32, 0.95, 0.8)
        plan = B.Plan(case.shapes if shapes else case.numels, 32, True, tiled=shapes is not None)
        th = [parity._dev(x) for x in case.theta_outer]
        ef = [[parity._dev(x) for x in r] for r in case.ef]
        tl = [[parity._dev(x) for x in r] for r in case.theta_local]
        msgs = [plan.message_buffers() for _ in range(case.R)]
        b_msgs = plan.bind_messages([m[0] for m in msgs], [m[1] for m in msgs])
        B.sparseloco_compress_batch(plan, th, tl, ef, b_msgs, 0.95)
        B.sparseloco_aggregate_update(plan, b_msgs, th, 0.8, reset=tl[:2])
        torch.cuda.synchronize()
        for t in range(len(case.numels)):
            new = parity.to_np(th[t])
            parity.assert_close_fp32(new, want[0]["theta"][t], "theta[%d]" % t)
            for r in range(2):
                assert parity.to_np(tl[r][t]).tobytes() == new.tobytes()
            assert parity.to_np(tl[2][t]).tobytes() == case.theta_local[2][t].tobytes()      # not in the reset list
        plan.close()


def test_colliding_indices_many_replicas():
    """All replicas send (almost) the same indices: every accumulator entry gets R addends."""
    rng = np.random.default_rng(77)
    numels = [4096 * 3 + 100]
    R = 33
    shared = (rng.standard_normal(numels[0]) * 1e-3).astype(np.float32)
    th = [np.zeros(numels[0], np.float32)]
    ef = [[np.zeros(numels[0], np.float32)] for _ in range(R)]
    deltas = [[(shared + (rng.standard_normal(numels[0]) * 1e-5).astype(np.float32)).astype(np.float32)]
              for _ in range(R)]
    case = parity.HostCase(th, ef, delta=deltas)
    for kappa in (16, 64, 128):
        parity.check(case, kappa, what="collisions kappa=%d" % kappa)
        parity.check(case, kappa, fused="no_mean", what="collisions fused kappa=%d" % kappa)


def colliding_case(numels, R, seed, noise=1e-5):
    """Replicas that send (almost) the same indices: shared pseudo-gradient plus a little noise of their own."""
    rng = np.random.default_rng(seed)
    shared = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for n in numels]
    th = [np.zeros(n, np.float32) for n in numels]
    ef = [[np.zeros(n, np.float32) for n in numels] for _ in range(R)]
    deltas = [[(shared[t] + (rng.standard_normal(n) * noise).astype(np.float32)).astype(np.float32)
               for t, n in enumerate(numels)] for _ in range(R)]
    return parity.HostCase(th, ef, delta=deltas)


@pytest.mark.parametrize("quant", [True, False])
@pytest.mark.parametrize("R", [9, 17, 40])
@pytest.mark.parametrize("kappa", [200, 256])
def test_wide_messages_many_replicas(kappa, R, quant):
    """kappa in 129..256 (four pairs per lane in the aggregation) with several batches of eight replicas, so
    that the prefetch of batch g + 4 and the hand-over between the four waves run; heavy collisions; separate
    and fused line 5; a partial chunk with kappa_c < kappa."""
    case = colliding_case([4096 * 2 + 230, 150], R, seed=kappa + R)
    parity.check(case, kappa, quant=quant, what="wide kappa=%d R=%d" % (kappa, R))
    parity.check(case, kappa, lr=0.8, quant=quant, fused="with_mean", what="wide fused kappa=%d R=%d" % (kappa, R))


@pytest.mark.parametrize("R", [33, 64])
def test_batched_compress_many_replicas(R):
    case = gaussian_case([4096 * 2 + 77, 300], R=R, seed=600 + R, heavy=True)
    parity.check(case, 32, batch=True, fused="no_mean", what="batched R=%d" % R)


def test_declared_limits_of_replica_counts():
    """SPLC_MAX_REPLICAS = 1024 replicas on a two-chunk tensor: bound as 1024 sets and 1024 messages, one batched
    compress launch, the mean over 1024 messages, and the reset of all 1024 local parameter sets."""
    R = B.SPLC_MAX_REPLICAS
    n = 4096 + 500
    rng = np.random.default_rng(1024)
    shared = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    th = [(rng.standard_normal(n) * 0.02).astype(np.float32)]
    ef = [[(rng.standard_normal(n) * 1e-4).astype(np.float32)] for _ in range(R)]
    tl = [[(th[0] - (shared + (rng.standard_normal(n) * 3e-4).astype(np.float32))).astype(np.float32)] for _ in range(R)]
    case = parity.HostCase(th, ef, theta_local=tl)
    want = parity.run_oracle(case, 16, 0.95, 1.0)
    plan = B.Plan(case.numels, 16)
    g_th = [parity._dev(th[0])]
    g_ef = [[parity._dev(e[0])] for e in ef]
    g_tl = [[parity._dev(t[0])] for t in tl]
    msgs = [plan.message_buffers() for _ in range(R)]
    b_msgs = plan.bind_messages([m[0] for m in msgs], [m[1] for m in msgs])
    b_tl = plan.bind(g_tl)
    B.sparseloco_compress_batch(plan, g_th, b_tl, g_ef, b_msgs, 0.95)
    dbar = [torch.full((n,), float("nan"), device="cuda")]
    B.sparseloco_aggregate_update(plan, b_msgs, g_th, 1.0, delta_bar_out=dbar, reset=b_tl)
    torch.cuda.synchronize()
    got = [dict(pairs=[parity.to_np(m[0]) for m in msgs], aux=[parity.to_np(m[1]) for m in msgs],
                ef=[[parity.to_np(e[0])] for e in g_ef], dbar=[parity.to_np(dbar[0])], theta=[parity.to_np(g_th[0])])]
    parity.compare(got, want, "1024 replicas")
    new = parity.to_np(g_th[0]).tobytes()
    assert all(parity.to_np(t[0]).tobytes() == new for t in g_tl)
    with pytest.raises(B.SparseLoCoError) as ei:            # one more than the limit is refused at bind time
        plan.bind(g_tl + [g_tl[0]])
    assert ei.value.status == B.SPLC_EINVAL
    plan.close()


def test_reset_of_64_replicas_on_ragged_tensors():
    case = gaussian_case([4096 + 9, 100, 4096 * 2], R=64, seed=64)
    want = parity.run_oracle(case, 32, 0.95, 1.0)
    plan = B.Plan(case.numels, 32)
    th = [parity._dev(x) for x in case.theta_outer]
    ef = [[parity._dev(x) for x in r] for r in case.ef]
    tl = [[parity._dev(x) for x in r] for r in case.theta_local]
    msgs = [plan.message_buffers() for _ in range(case.R)]
    b_msgs = plan.bind_messages([m[0] for m in msgs], [m[1] for m in msgs])
    B.sparseloco_compress_batch(plan, th, tl, ef, b_msgs, 0.95)
    B.sparseloco_aggregate_update(plan, b_msgs, th, 1.0, reset=tl)
    torch.cuda.synchronize()
    for t in range(len(case.numels)):
        new = parity.to_np(th[t])
        parity.assert_close_fp32(new, want[0]["theta"][t], "theta[%d]" % t)
        assert all(parity.to_np(tl[r][t]).tobytes() == new.tobytes() for r in range(64))
    plan.close()


@pytest.mark.parametrize("variant", ["three_calls", "batched_fused", "one_launch"])
@pytest.mark.parametrize("tiled", [False, True])
def test_outer_step_replays_from_a_hip_graph(variant, tiled):
    """The operations only enqueue kernels, so a whole outer step can be recorded into a HIP graph.  Three
    replays, each after fresh local parameters were written by eager work and a synchronisation, each compared
    bit for bit with the same step run eagerly on a copy of the state; the first also against the oracle."""
    R, kappa, beta, lr = 5, 48, 0.95, 0.8
    shapes = TILED_SHAPES + STRIP_SHAPES[:3] if tiled else None
    case = gaussian_case(RAGGED, R=R, seed=808, shapes=shapes)
    want = parity.run_oracle(case, kappa, beta, lr)
    plan = B.Plan(case.shapes if tiled else case.numels, kappa, True, tiled=tiled)

    class State:
        def __init__(self):
            self.th = [parity._dev(x) for x in case.theta_outer]
            self.ef = [[parity._dev(x) for x in r] for r in case.ef]
            self.tl = [[parity._dev(x) for x in r] for r in case.theta_local]
            self.msgs = [plan.message_buffers() for _ in range(R)]
            self.dbar = [torch.zeros(n, device="cuda") for n in case.numels]
            self.b_th, self.b_ef, self.b_tl, self.b_dbar = (plan.bind(x) for x in (self.th, self.ef, self.tl, self.dbar))
            self.b_msgs = plan.bind_messages([m[0] for m in self.msgs], [m[1] for m in self.msgs])

        def step(self):
            if variant == "three_calls":
                for r in range(R):
                    B.sparseloco_compress(plan, self.b_ef, self.msgs[r][0], self.msgs[r][1], beta, theta_outer=self.b_th,
                                          theta_local=self.b_tl, replica=r)
                B.sparseloco_aggregate(plan, self.b_msgs, self.b_dbar)
                B.sparseloco_outer_update(plan, self.b_th, self.b_dbar, lr)
            elif variant == "batched_fused":
                B.sparseloco_compress_batch(plan, self.b_th, self.b_tl, self.b_ef, self.b_msgs, beta)
                B.sparseloco_aggregate_update(plan, self.b_msgs, self.b_th, lr, delta_bar_out=self.b_dbar)
            else:
                B.sparseloco_outer_step_batch(plan, self.b_th, self.b_tl, self.b_ef, self.b_msgs, beta, lr,
                                              delta_bar_out=self.b_dbar)

        def tensors(self):
            return self.th + [x for r in self.ef for x in r] + [x for m in self.msgs for x in m] + self.dbar

    warm, a, b = State(), State(), State()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        warm.step()                                                  # loads the kernels outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        a.step()
    gen = torch.Generator(device="cuda").manual_seed(5)
    for rep in range(3):
        if rep > 0:                                                  # the replicas' next inner phase, eagerly
            for r in range(R):
                for t, n in enumerate(case.numels):
                    fresh = a.th[t] - torch.randn(n, generator=gen, device="cuda") * 1e-3
                    a.tl[r][t].copy_(fresh)
                    b.tl[r][t].copy_(fresh)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        b.step()
        torch.cuda.synchronize()
        for x, y in zip(a.tensors(), b.tensors()):
            assert torch.equal(x, y), "replay %d differs from the eager step" % rep
        if rep == 0:
            got = [dict(pairs=[parity.to_np(m[0]) for m in a.msgs], aux=[parity.to_np(m[1]) for m in a.msgs],
                        ef=[[parity.to_np(x) for x in r] for r in a.ef], dbar=[parity.to_np(x) for x in a.dbar],
                        theta=[parity.to_np(x) for x in a.th])]
            parity.compare(got, want, "graph replay 0")
    plan.close()


def test_workload0_full():
    cfg = W.WORKLOADS[0]
    rs = W.ReplicaSet(0, device="cuda")
    case = parity.HostCase([parity.to_np(t) for t in rs.theta_outer],
                           [[parity.to_np(t) for t in r] for r in rs.ef],
                           theta_local=[[parity.to_np(t) for t in r] for r in rs.theta_local])
    parity.check(case, cfg["kappa"], cfg["beta"], cfg["outer_lr"], what="workload 0")


def test_workload1_full():
    """The whole ~150M set (110 tensors, 151.9M parameters), all R = 8 replicas, element by element."""
    cfg = W.WORKLOADS[1]
    rs = W.ReplicaSet(1, device="cuda")
    case = parity.HostCase([parity.to_np(t) for t in rs.theta_outer],
                           [[parity.to_np(t) for t in r] for r in rs.ef],
                           theta_local=[[parity.to_np(t) for t in r] for r in rs.theta_local])
    del rs
    parity.check(case, cfg["kappa"], cfg["beta"], cfg["outer_lr"], what="workload 1")


def test_same_inputs_twice_give_identical_bytes():
    case = gaussian_case([4096 * 9 + 3], R=5, seed=23)
    a = parity.run_gpu(case, 64, 0.95, 1.0)
    b = parity.run_gpu(case, 64, 0.95, 1.0)
    for key in ("pairs", "aux"):
        for x, y in zip(a[0][key], b[0][key]):
            assert x.tobytes() == y.tobytes()
    for x, y in zip(a[0]["dbar"] + a[0]["theta"], b[0]["dbar"] + b[0]["theta"]):
        assert x.tobytes() == y.tobytes()


def test_runs_on_a_side_stream():
    case = gaussian_case([4096 * 3 + 9, 50], R=2, seed=29)
    want = parity.run_oracle(case, 32, 0.95, 1.0)
    s = torch.cuda.Stream()
    got = parity.run_gpu(case, 32, 0.95, 1.0, stream=s)
    parity.compare(got, want, "side stream")


@pytest.mark.parametrize("kw", [dict(), dict(slots=1), dict(run=16), dict(slots=1, run=4), dict(max_groups_per_unit=1),
                                dict(run=2, max_groups_per_unit=3)], ids=str)
def test_stream_probe_shapes_cover_every_element(kw):
    """The measurement aid touches every element exactly once whatever the launch shape: the write pattern fills
    the whole array, the compress pattern leaves (a - b) + c everywhere."""
    n = 4096 * 8 * 16 * 3
    g = torch.Generator(device="cuda").manual_seed(12)
    a, b, c = (torch.randn(n, generator=g, device="cuda") for _ in range(3))
    sink = torch.zeros(1, device="cuda")
    want = (a - b) + c
    B.sparseloco_stream_probe(B.SPLC_STREAM_R3W1, a, b, c, sink, **kw)
    assert torch.equal(c, want)
    B.sparseloco_stream_probe(B.SPLC_STREAM_WRITE, a, b, c, sink, **kw)
    assert torch.equal(c, torch.tensor([1.0, 2.0, 3.0, 4.0], device="cuda").repeat(n // 4))
    B.sparseloco_stream_probe(B.SPLC_STREAM_COPY, a, b, c, sink, **kw)
    assert torch.equal(c, a)


def test_error_returns_do_not_launch():
    plan = B.Plan([4096, 10], 32)
    e = [torch.zeros(4096, device="cuda"), torch.zeros(10, device="cuda")]
    p, a = plan.message_buffers()
    with pytest.raises(ValueError):                     # the binding refuses a missing tensor on the host
        B.sparseloco_compress(plan, e, p, a, 0.95, theta_outer=e, theta_local=[e[0], None])
    L = B.lib()
    import ctypes
    h = ctypes.c_void_p()
    ptrs = (ctypes.c_void_p * 2)(e[0].data_ptr(), None)
    assert L.sparseloco_tensors_bind(ctypes.byref(h), plan.handle, 1, ptrs, B.SPLC_F32, None) == B.SPLC_EINVAL
    big = torch.zeros(2 * (4096 + 8), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(B.SparseLoCoError) as ei:        # a bf16 source that starts at an odd element: 2-byte aligned
        B.sparseloco_compress(plan, e, p, a, 0.95, delta=[big[1:4097], big[4100:4110]])
    assert ei.value.status == B.SPLC_EALIGN
    with pytest.raises(B.SparseLoCoError) as ei:
        B.sparseloco_compress(plan, e, p, a, float("inf"), delta=e)
    assert ei.value.status == B.SPLC_EINVAL
    with pytest.raises(B.SparseLoCoError) as ei:
        B.sparseloco_aggregate(plan, [], e, aux=[])
    assert ei.value.status == B.SPLC_EINVAL
    with pytest.raises(B.SparseLoCoError) as ei:        # replica index beyond the sets of a multi-set binding
        B.sparseloco_compress(plan, plan.bind([e, e]), p, a, 0.95, delta=e, replica=2)
    assert ei.value.status == B.SPLC_EINVAL
    two = [plan.message_buffers() for _ in range(2)]
    m2 = plan.bind_messages([m[0] for m in two], [m[1] for m in two])
    th0 = [t.clone() for t in e]
    for kwargs in (dict(n_replicas=3), dict(n_replicas=0)):      # more replicas than bound sets / messages; none
        with pytest.raises(B.SparseLoCoError) as ei:
            B.sparseloco_outer_step_batch(plan, th0, [e, e], plan.bind([e, e]), m2, 0.95, 1.0, **kwargs)
        assert ei.value.status == B.SPLC_EINVAL
    with pytest.raises(B.SparseLoCoError) as ei:
        B.sparseloco_outer_step_batch(plan, th0, [e, e], plan.bind([e, e]), m2, 0.95, float("nan"))
    assert ei.value.status == B.SPLC_EINVAL
    torch.cuda.synchronize()
    assert all(torch.equal(a_, b_) for a_, b_ in zip(th0, e))     # nothing was launched
    other = B.Plan([4096], 32)
    with pytest.raises(B.SparseLoCoError) as ei:        # a binding made for another plan
        B.sparseloco_outer_update(plan, other.bind([e[0]]), e, 1.0)
    assert ei.value.status == B.SPLC_EPLAN
    other.close()
    plan.close()


@pytest.mark.parametrize("seed", range(24))
def test_random_configurations(seed):
    """Seeded random tensor lists, kappa, replica counts, source modes, quantiser modes, layouts and
    entry-point variants, each compared with the oracle element by element."""
    rng = np.random.default_rng(9000 + seed)
    tiled = bool(rng.integers(0, 2))
    n_t = int(rng.integers(1, 6))
    if tiled:
        shapes = [(int(rng.integers(1, 200)), int(rng.integers(1, 200))) for _ in range(n_t)]
        numels = None
    else:
        shapes = None
        numels = [int(rng.choice([0, 1, 63, 64, 65, 4095, 4096, 4097, 8192, 3 * 4096 + int(rng.integers(0, 4096))]))
                  for _ in range(n_t)]
        if not any(numels):
            numels[0] = 4096
    kappa = int(rng.choice([1, 2, 7, 31, 32, 33, 64, 100, 128, 255, 256, 257, 1000]))
    R = int(rng.integers(1, 6))
    direct = [None, "f32", "bf16"][int(rng.integers(0, 3))]
    quant = bool(rng.integers(0, 2))
    heavy = bool(rng.integers(0, 2))
    select = [B.SPLC_SELECT_AUTO, B.SPLC_SELECT_RADIX][int(rng.integers(0, 4) == 0)]
    fused = [None, "with_mean", "no_mean"][int(rng.integers(0, 3))]
    batch = direct is None and bool(rng.integers(0, 2))
    case = gaussian_case(numels, R=R, seed=int(rng.integers(0, 1 << 30)), direct=direct, heavy=heavy, shapes=shapes)
    parity.check(case, kappa, lr=float(rng.choice([1.0, 0.8])), quant=quant, select=select, fused=fused, batch=batch,
                 outer_steps=int(rng.integers(1, 3)),
                 what="random case %d (tiled=%s kappa=%d R=%d direct=%s quant=%s)" % (seed, tiled, kappa, R, direct, quant))


def test_aggregate_survives_malformed_messages():
    """Pairs that no compress call would emit (duplicate indices, spare bits set, indices beyond a partial
    chunk): indices are masked to 12 bits and only present positions are written, so the call completes;
    the values themselves are unspecified, positions outside every chunk's extent stay untouched."""
    import torch
    numels = [4096 * 2 + 100, 50]
    kappa, R = 64, 3
    plan = B.Plan(numels, kappa)
    g = torch.Generator(device="cuda").manual_seed(1)
    pairs = [torch.randint(-32768, 32767, (plan.num_chunks * kappa,), generator=g, device="cuda",
                           dtype=torch.int16) for _ in range(R)]
    scales = [torch.rand(plan.num_chunks * 2, generator=g, device="cuda") for _ in range(R)]
    guard = 7.0
    bufs = [torch.full((n + 64,), guard, device="cuda") for n in numels]
    dbar = [b[:n] for b, n in zip(bufs, numels)]
    B.sparseloco_aggregate(plan, pairs, dbar, aux=scales)
    torch.cuda.synchronize()
    for b, n in zip(bufs, numels):
        assert bool(torch.isfinite(b[:n]).all()) and bool((b[n:] == guard).all())
    plan.close()
