"""Parity at the benchmark's full sizes and launch configuration.

The whole parameter set of a workload lives on the GPU and goes through the
library exactly as bench.py drives it (one compress launch per replica over all
tensors, then aggregate, then outer update).  The oracle cannot sort a billion
elements in test time, so it recomputes SAMPLED chunks one by one -- every
chunk is independent in the method -- chosen as: the first and the last chunk
of every tensor (so every partial chunk), plus random ones.  Properties that
hold at any size are checked over all chunks on the device.
"""
import numpy as np
import pytest
import torch

from paper_2601_02360_amd import binding as B
from paper_2601_02360_amd import workloads as W

import parity

pytestmark = pytest.mark.gpu
CH = 4096


def chunks_of(shape, tiled):
    rows, cols = B.rows_cols(shape)
    if tiled and rows > 1:
        return ((rows + 63) // 64) * ((cols + 63) // 64)
    return (rows * cols + CH - 1) // CH


def sample_chunks(shapes, n_random, seed, tiled=False):
    rng = np.random.default_rng(seed)
    picks = []                                   # (tensor, chunk-in-tensor)
    total = [chunks_of(s, tiled) for s in shapes]
    for t, nc in enumerate(total):
        if nc == 0:
            continue
        picks.append((t, 0))
        if nc > 1:
            picks.append((t, nc - 1))
        if tiled and B.rows_cols(shapes[t])[0] > 1:          # right edge of the first tile row, left edge of the last
            nbj = (B.rows_cols(shapes[t])[1] + 63) // 64
            picks += [(t, nbj - 1), (t, nc - nbj)]
    cum = np.cumsum([0] + total)
    for g in rng.integers(0, cum[-1], n_random):
        t = int(np.searchsorted(cum, g, side="right") - 1)
        picks.append((t, int(g - cum[t])))
    return sorted(set(picks)), cum


def gather(tensors, picks, shapes=None):
    """The picked chunks as host arrays; with shapes (tiled layout) a 2-D tensor's chunk is its 64 x 64 tile."""
    out = []
    for t, c in picks:
        flat = tensors[t].view(-1)
        rows, cols = B.rows_cols(shapes[t]) if shapes is not None else (1, flat.numel())
        if rows > 1:
            nbj = (cols + 63) // 64
            bi, bj = c // nbj, c % nbj
            tile = flat.view(rows, cols)[bi * 64:(bi + 1) * 64, bj * 64:(bj + 1) * 64]
            out.append(parity.to_np(tile.contiguous()))
        else:
            out.append(parity.to_np(flat[c * CH:min((c + 1) * CH, flat.numel())]).reshape(1, -1))
    return out


def gather_msg(msg, picks, cum, kappa, quant=True):
    p, a = msg
    gi = torch.tensor([int(cum[t] + c) for t, c in picks], device=p.device)
    pp = p.view(-1, kappa)[gi].reshape(-1)
    aa = a.view(-1, 2 if quant else kappa)[gi].reshape(-1)
    return parity.to_np(pp), parity.to_np(aa)


def all_chunk_properties(plan, msg, numels, kappa):
    """Every chunk (flat layout): exactly kappa_c valid pairs, ascending in-range indices, spare bits zero, lo <= hi."""
    p, a = msg
    total = [(n + CH - 1) // CH for n in numels]
    n_c = torch.full((sum(total),), CH, dtype=torch.int32, device=p.device)
    cum = np.cumsum(total)
    for t, n in enumerate(numels):
        if n % CH and total[t]:
            n_c[cum[t] - 1] = n % CH
    kc = torch.clamp(n_c, max=kappa)
    pv = p.view(-1, kappa).to(torch.int32) & 0xFFFF
    slot = torch.arange(kappa, device=p.device, dtype=torch.int32)[None, :]
    valid = slot < kc[:, None]
    assert bool(((pv == 0xFFFF) == ~valid).all())
    idx = pv & 0xFFF
    assert bool((((pv >> 14) == 0) | ~valid).all())
    assert bool(((idx < n_c[:, None]) | ~valid).all())
    asc = (idx[:, 1:] > idx[:, :-1]) | ~valid[:, 1:]
    assert bool(asc.all())
    s = a.view(-1, 2)
    assert bool((s[:, 0] <= s[:, 1]).all()) and bool((s[:, 0] >= 0).all()) and bool(torch.isfinite(s).all())


def fullsize_check(workload, R, kappa, tensors=None, n_random=300, outer_steps=1, seed=0, tiled=False,
                   one_launch=False):
    """one_launch: the step goes through sparseloco_outer_step_batch instead of the three calls."""
    cfg = W.WORKLOADS[workload]
    rs = W.ReplicaSet(workload, device="cuda", replicas=R, tensors=tensors)
    shapes = [W.tensor_shapes(workload)[t] for t in rs.tensor_ids] if tiled else None
    picks, cum = sample_chunks(shapes if tiled else rs.numels, n_random, seed, tiled)
    gather_ = lambda tensors, picks: gather(tensors, picks, shapes)
    th0 = gather_(rs.theta_outer, picks)
    ef0 = [gather_(rs.ef[r], picks) for r in range(R)]
    plan = B.Plan(shapes if tiled else rs.numels, kappa, True, tiled=tiled)
    dbar = [torch.empty(n, device="cuda") for n in rs.numels]
    got, deltas_per_step = [], []
    tl0 = None
    b_theta, b_dbar, b_ef = plan.bind(rs.theta_outer), plan.bind(dbar), plan.bind(rs.ef)
    b_tl = None if rs.direct else plan.bind(rs.theta_local)
    for step in range(outer_steps):
        if rs.direct:
            if step > 0:
                for r in range(R):
                    for i, t in enumerate(rs.tensor_ids):
                        rs.delta[r][i] = W.replica_inputs(workload, t, r, None, "cuda", outer_step=step)[1]
            deltas_per_step.append([gather_(rs.delta[r], picks) for r in range(R)])
        elif step == 0:
            tl0 = [gather_(rs.theta_local[r], picks) for r in range(R)]
        msgs = [plan.message_buffers() for _ in range(R)]
        b_msgs = plan.bind_messages([m[0] for m in msgs], [m[1] for m in msgs])
        if one_launch:
            B.sparseloco_outer_step_batch(plan, b_theta, b_tl, b_ef, b_msgs, cfg["beta"], cfg["outer_lr"],
                                          delta_bar_out=b_dbar)
        for r in range(0 if one_launch else R):
            if rs.direct:
                B.sparseloco_compress(plan, b_ef, msgs[r][0], msgs[r][1], cfg["beta"], delta=rs.delta[r], replica=r)
            else:
                B.sparseloco_compress(plan, b_ef, msgs[r][0], msgs[r][1], cfg["beta"],
                                      theta_outer=b_theta, theta_local=b_tl, replica=r)
        if not one_launch:
            B.sparseloco_aggregate(plan, b_msgs, b_dbar)
            B.sparseloco_outer_update(plan, b_theta, b_dbar, cfg["outer_lr"])
        torch.cuda.synchronize()
        b_msgs.close()
        for r in (0, R - 1):
            if not tiled:
                all_chunk_properties(plan, msgs[r], rs.numels, kappa)
        gm = [gather_msg(msgs[r], picks, cum, kappa) for r in range(R)]
        got.append(dict(pairs=[g[0] for g in gm], aux=[g[1] for g in gm],
                        ef=[gather_(rs.ef[r], picks) for r in range(R)],
                        dbar=gather_(dbar, picks), theta=gather_(rs.theta_outer, picks)))
        del msgs
    plan.close()
    sample_shapes = [x.shape for x in th0] if tiled else None      # every sampled tile is one tile of its own
    if rs.direct:
        case = parity.HostCase(th0, ef0, delta=deltas_per_step[0], shapes=sample_shapes)
        want = parity.run_oracle(case, kappa, cfg["beta"], cfg["outer_lr"], True, outer_steps, deltas_per_step)
    else:
        case = parity.HostCase(th0, ef0, theta_local=tl0, shapes=sample_shapes)
        want = parity.run_oracle(case, kappa, cfg["beta"], cfg["outer_lr"], True, outer_steps)
    parity.compare(got, want, "workload %d full size (%d sampled chunks)" % (workload, len(picks)))


def test_workload2_full_size_as_benchmarked():
    """~0.9B parameters, kappa 64, R 8: the configuration bench.py times."""
    cfg = W.WORKLOADS[2]
    fullsize_check(2, cfg["replicas"], cfg["kappa"], n_random=400)


def test_workload2_full_size_in_one_launch():
    """The same configuration through sparseloco_outer_step_batch (bench.py's one-launch variant), two outer steps."""
    cfg = W.WORKLOADS[2]
    fullsize_check(2, cfg["replicas"], cfg["kappa"], n_random=300, outer_steps=2, seed=3, one_launch=True)


def test_workload2_tiled_in_one_launch():
    fullsize_check(2, 4, W.WORKLOADS[2]["kappa"], n_random=200, seed=4, tiled=True, one_launch=True)


@pytest.mark.parametrize("kappa", [16, 32, 64, 128])
def test_workload3_density_sweep_correlated_replicas(kappa):
    """R 16 replicas sharing most of their pseudo-gradient: heavy index collisions in the mean.
    One transformer layer and the embedding of the ~0.9B shape."""
    fullsize_check(3, 16, kappa, tensors=list(range(9)) + [144, 145], n_random=150, seed=kappa)


def test_workload4_ragged_bf16_two_outer_steps():
    """Every tensor ends in a partial chunk; bf16 pseudo-gradients given directly, half zeros, many
    ties.  Full shapes, 4 of the 32 replicas, two outer steps (the second sees a non-trivial buffer)."""
    fullsize_check(4, 4, W.WORKLOADS[4]["kappa"], n_random=300, outer_steps=2)


def test_workload4_all_replicas_on_two_layers():
    fullsize_check(4, 32, W.WORKLOADS[4]["kappa"], tensors=list(range(18)) + [144, 145], n_random=100)


def test_workload2_full_size_tiled_layout():
    """The ~0.9B set with 64 x 64 tile chunks (every matrix dimension is a multiple of 64; vectors stay flat)."""
    cfg = W.WORKLOADS[2]
    fullsize_check(2, 4, cfg["kappa"], n_random=300, tiled=True)


def test_workload4_ragged_shapes_tiled_layout():
    """2050 x 5630 and 32001 x 2048 matrices: edge tiles on both sides, odd row starts for the bf16 source."""
    fullsize_check(4, 2, W.WORKLOADS[4]["kappa"], tensors=list(range(9)) + [144, 145], n_random=200, tiled=True)


def test_one_tensor_with_more_than_2_31_elements():
    """64-bit addressing: a single tensor of 2^31 + 10000 elements (byte offsets beyond 2^33), R = 1.
    The oracle recomputes the chunks around the 2^31-element mark, the first and the last (partial) chunk
    and random ones."""
    n = (1 << 31) + 10000
    g = torch.Generator(device="cuda").manual_seed(5)
    theta_o = torch.randn(n, generator=g, device="cuda") * 0.02
    theta_l = theta_o - torch.randn(n, generator=g, device="cuda") * 1e-3
    ef = torch.randn(n, generator=g, device="cuda") * 1e-4
    kappa = 32
    n_chunks = (n + CH - 1) // CH
    rng = np.random.default_rng(1)
    mark = (1 << 31) // CH
    picks = sorted(set([(0, 0), (0, n_chunks - 1), (0, mark - 1), (0, mark), (0, mark + 1), (0, (1 << 30) // CH)] +
                       [(0, int(c)) for c in rng.integers(0, n_chunks, 60)]))
    cum = np.array([0, n_chunks])
    th0, tl0, ef0 = gather([theta_o], picks), gather([theta_l], picks), gather([ef], picks)
    plan = B.Plan([n], kappa)
    assert plan.num_chunks == n_chunks and plan.num_params == n
    msg = plan.message_buffers()
    dbar = torch.empty(n, device="cuda")
    B.sparseloco_compress(plan, [ef], msg[0], msg[1], 0.95, theta_outer=[theta_o], theta_local=[theta_l])
    B.sparseloco_aggregate(plan, [msg[0]], [dbar], aux=[msg[1]])
    B.sparseloco_outer_update(plan, [theta_o], [dbar], 1.0)
    torch.cuda.synchronize()
    all_chunk_properties(plan, msg, [n], kappa)
    gp, ga = gather_msg(msg, picks, cum, kappa)
    got = [dict(pairs=[gp], aux=[ga], ef=[gather([ef], picks)], dbar=gather([dbar], picks),
                theta=gather([theta_o], picks))]
    plan.close()
    case = parity.HostCase(th0, [ef0], theta_local=[tl0])
    want = parity.run_oracle(case, kappa, 0.95, 1.0)
    parity.compare(got, want, "2^31+ elements")
