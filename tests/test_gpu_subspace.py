"""GPU parity of the embedding re-projection (paper section 2.4) against the float64 oracle.

Tolerance, derived from the arithmetic: the GPU forms two fp32 dot products per output (length d,
then length k) with fp32 accumulation in an unspecified order.  With rounding errors of the partial
sums modelled as independent, a dot product of length n has relative error about sqrt(n) * eps
(eps = 2^-24) with respect to |x| |u|; the bar below is 8 (sqrt(d) + sqrt(k)) eps per ROW in the
2-norm, relative to the row norm of T_S, for the projection, and the same plus one rounding of the
sum for T_perp.  The worst-case bound (d + k) eps is also asserted element-wise.

Every test runs twice: with fp32 MFMA products and with SPLC_MATMUL_BF16X3 (operands split exactly into three
bf16 pieces, six piece products per product).  The split drops less than 3 * 2^-24 |x y| per product --
part of a rounding step, far inside the bars above -- and products with an exact result (a coordinate
subspace) stay exact, so both modes are held to the same bars.
"""
import numpy as np
import pytest
import torch

from oracle import subspace
from paper_2601_02360_amd import binding as B

pytestmark = pytest.mark.gpu
EPS = 2.0 ** -24


@pytest.fixture(autouse=True, params=[B.SPLC_MATMUL_FP32, B.SPLC_MATMUL_BF16X3], ids=["fp32", "bf16x3"])
def matmul_mode(request):
    B.sparseloco_set_matmul_mode(request.param)
    assert B.sparseloco_get_matmul_mode() == request.param
    yield request.param
    B.sparseloco_set_matmul_mode(B.SPLC_MATMUL_FP32)


def run_case(vocab, d, k, seed):
    rng = np.random.default_rng(seed)
    u64 = subspace.orthonormal_basis(d, k, seed)
    u = u64.astype(np.float32)
    ts = (rng.standard_normal((vocab, d)) * 0.02).astype(np.float32)
    tp = (rng.standard_normal((vocab, d)) * 0.02).astype(np.float32)
    want_ts, want_tp = subspace.reproject(ts, tp, u)             # the oracle sees the same fp32 inputs
    g_ts, g_tp, g_u = (torch.from_numpy(x.copy()).cuda() for x in (ts, tp, u))
    ws = torch.full((max(vocab * k, 1),), float("nan"), device="cuda")
    B.sparseloco_reproject_embedding(g_ts, g_tp, g_u, ws)
    torch.cuda.synchronize()
    got_ts, got_tp = g_ts.cpu().numpy().astype(np.float64), g_tp.cpu().numpy().astype(np.float64)
    row = np.linalg.norm(ts.astype(np.float64), axis=1)
    tol_row = 8 * (np.sqrt(d) + np.sqrt(k)) * EPS * row + 1e-30
    assert np.all(np.linalg.norm(got_ts - want_ts, axis=1) <= tol_row), "projection"
    assert np.all(np.linalg.norm(got_tp - want_tp, axis=1) <= tol_row + 4 * EPS * np.linalg.norm(want_tp, axis=1)), "T_perp"
    worst = (d + k + 4) * EPS * row[:, None] * 1.0 + 4 * EPS * np.abs(want_tp)
    assert np.all(np.abs(got_ts - want_ts) <= worst) and np.all(np.abs(got_tp - want_tp) <= worst)
    # the identities of the section hold on the GPU result as well
    assert np.all(np.linalg.norm((got_ts + got_tp) - (ts.astype(np.float64) + tp), axis=1) <= tol_row)
    resid = np.linalg.norm(got_ts - (got_ts @ u64) @ u64.T, axis=1)
    assert np.all(resid <= tol_row)
    coeff = ws[:vocab * k].cpu().numpy().reshape(vocab, k).astype(np.float64)
    assert np.all(np.linalg.norm(coeff - ts.astype(np.float64) @ u.astype(np.float64), axis=1) <= tol_row)


@pytest.mark.parametrize("vocab,d,k", [(128, 128, 128), (256, 256, 32), (300, 200, 7), (1, 64, 2), (129, 130, 131),
                                       (1000, 768, 96), (517, 1536, 2), (64, 2048, 256), (2000, 1024, 128),
                                       # narrow bases: both passes (k <= 32 in fours, or k <= 8), pass 1 only (k <= 64)
                                       (100, 64, 8), (33, 96, 20), (2000, 1024, 16), (70, 32, 32), (300, 128, 64),
                                       (17, 160, 5), (4097, 512, 4), (250, 2048, 48)])
def test_reproject_matches_the_oracle(vocab, d, k):
    if k > d:
        k = d
    run_case(vocab, d, k, seed=vocab + d + k)


def test_coordinate_subspace_is_exact():
    """U = columns of the identity: every product is x * 1 or x * 0, so the result is exact."""
    vocab, d, k = 200, 192, 64
    rng = np.random.default_rng(5)
    cols = rng.permutation(d)[:k]
    u = np.zeros((d, k), np.float32)
    u[cols, np.arange(k)] = 1.0
    ts = rng.standard_normal((vocab, d)).astype(np.float32)
    tp = rng.standard_normal((vocab, d)).astype(np.float32)
    g_ts, g_tp, g_u = (torch.from_numpy(x.copy()).cuda() for x in (ts, tp, u))
    ws = torch.empty(vocab * k, device="cuda")
    B.sparseloco_reproject_embedding(g_ts, g_tp, g_u, ws)
    keep = np.zeros(d, bool)
    keep[cols] = True
    out_ts, out_tp = g_ts.cpu().numpy(), g_tp.cpu().numpy()
    assert np.array_equal(out_ts[:, keep], ts[:, keep]) and not out_ts[:, ~keep].any()
    assert np.array_equal(out_tp[:, ~keep], tp[:, ~keep] + ts[:, ~keep])
    assert np.array_equal(out_tp[:, keep], tp[:, keep])


def test_matmul_mode_argument():
    assert B.lib().sparseloco_set_matmul_mode(7) == B.SPLC_EINVAL


def test_argument_checks():
    t = torch.zeros(4, 8, device="cuda")
    u = torch.zeros(8, 2, device="cuda")
    L = B.lib()
    assert L.sparseloco_reproject_embedding(None, t.data_ptr(), u.data_ptr(), t.data_ptr(), 4, 8, 2, None) == B.SPLC_EINVAL
    assert L.sparseloco_reproject_embedding(t.data_ptr(), t.data_ptr(), u.data_ptr(), t.data_ptr(), 4, 8, 9, None) == B.SPLC_EINVAL
    assert L.sparseloco_reproject_embedding(t.data_ptr(), t.data_ptr(), u.data_ptr(), t.data_ptr(), 0, 8, 2, None) == B.SPLC_OK


@pytest.mark.parametrize("rows,seq,d,k,vocab,use_perp,use_pos", [
    (256, 64, 128, 16, 50, True, True), (300, 100, 200, 7, 33, True, True), (129, 43, 130, 130, 5, True, False),
    (512, 128, 768, 96, 1000, False, True), (1000, 250, 1536, 2, 64, True, True), (640, 64, 2048, 256, 512, False, False),
    # narrow bases (the narrow kernel up to 32 columns, or 16 with both tables; the 64 x 64 GEMM tile otherwise):
    # reduction lengths that leave some of a workgroup's waves without a tile or end inside a tile, row counts
    # off the 16-row grid
    (257, 64, 100, 33, 20, True, False), (64, 16, 36, 36, 7, False, True), (1000, 128, 512, 64, 100, True, True),
    (33, 33, 70, 48, 9, True, True), (500, 50, 2048, 17, 30, False, False), (16, 16, 1, 1, 3, True, True),
    (4099, 1024, 1536, 8, 3000, True, True), (15, 5, 257, 64, 4, False, False), (2048, 512, 768, 32, 500, False, True),
    # more narrow bases, single rows and single tiles
    (77, 11, 64, 3, 9, True, False), (200, 40, 96, 5, 50, False, False), (333, 37, 256, 24, 100, True, True),
    (50, 50, 32, 12, 5, False, True), (1, 1, 32, 4, 2, True, True), (130, 13, 160, 1, 7, True, True),
    (1000, 100, 1024, 20, 300, True, False),
    # the GEMM kernel with a basis whose width is no multiple of four: its loads run past column k into the next
    # row of U, except in the guarded last tiles
    (700, 70, 512, 42, 60, True, True), (300, 30, 1024, 21, 10, True, True), (90, 9, 64, 63, 5, False, True),
    (64, 8, 48, 1, 3, True, True), (2000, 200, 2048, 170, 100, True, False)])
def test_project_and_reconstruct_match_the_oracle(rows, seq, d, k, vocab, use_perp, use_pos):
    rng = np.random.default_rng(rows + d + k)
    u64 = subspace.orthonormal_basis(d, k, rows)
    u = u64.astype(np.float32)
    x = rng.standard_normal((rows, d)).astype(np.float32)
    tp = (rng.standard_normal((vocab, d)) * 0.5).astype(np.float32) if use_perp else None
    tok = rng.integers(0, vocab, rows).astype(np.int32) if use_perp else None
    pos = (rng.standard_normal((seq, d)) * 0.5).astype(np.float32) if use_pos else None
    dev = lambda a: None if a is None else torch.from_numpy(a.copy()).cuda()
    g_x, g_u, g_tp, g_tok, g_pos = dev(x), dev(u), dev(tp), dev(tok), dev(pos)
    out_t = torch.full((rows, k), float("nan"), device="cuda")
    B.sparseloco_subspace_project(g_x, g_u, out_t, t_perp=g_tp, token_ids=g_tok, pos_embed=g_pos)
    want_t = subspace.project(x, u, tp, tok, pos)
    high = np.zeros((rows, d)) if (tp is None and pos is None) else subspace.reconstruct(np.zeros((rows, k)), u, tp, tok, pos)
    scale = np.linalg.norm(x.astype(np.float64), axis=1) + np.linalg.norm(high, axis=1)
    tol = 8 * (np.sqrt(d) + np.sqrt(k)) * EPS * scale
    got_t = out_t.cpu().numpy().astype(np.float64)
    assert np.all(np.linalg.norm(got_t - want_t, axis=1) <= tol), "project"
    # reconstruct from the GPU's own x_tilde, compared with the oracle applied to the same x_tilde
    out_h = torch.full((rows, d), float("nan"), device="cuda")
    B.sparseloco_subspace_reconstruct(out_t, g_u, out_h, t_perp=g_tp, token_ids=g_tok, pos_embed=g_pos)
    want_h = subspace.reconstruct(out_t.cpu().numpy(), u, tp, tok, pos)
    got_h = out_h.cpu().numpy().astype(np.float64)
    assert np.all(np.linalg.norm(got_h - want_h, axis=1) <= tol), "reconstruct"


def test_subspace_calls_replay_from_a_hip_graph():
    """The matrix entry points only enqueue kernels, so they can be recorded into a HIP graph: three replays on
    fresh inputs, with eager work and synchronisation in between, each equal to the eager result bit for bit."""
    rows, seq, d, k, vocab = 500, 50, 256, 40, 64
    gen = torch.Generator(device="cuda").manual_seed(17)
    u = torch.from_numpy(subspace.orthonormal_basis(d, k, 3).astype(np.float32)).cuda()
    x = torch.randn(rows, d, generator=gen, device="cuda")
    tp = torch.randn(vocab, d, generator=gen, device="cuda") * 0.5
    pos = torch.randn(seq, d, generator=gen, device="cuda") * 0.5
    tok = torch.randint(0, vocab, (rows,), generator=gen, device="cuda", dtype=torch.int32)
    ts = torch.randn(vocab, d, generator=gen, device="cuda")
    xt, xh = torch.empty(rows, k, device="cuda"), torch.empty(rows, d, device="cuda")
    ws = torch.empty(vocab * k, device="cuda")

    def work(x_in, ts_io, tp_io, xt_out, xh_out):
        B.sparseloco_subspace_project(x_in, u, xt_out, t_perp=tp_io, token_ids=tok, pos_embed=pos)
        B.sparseloco_subspace_reconstruct(xt_out, u, xh_out, t_perp=tp_io, token_ids=tok, pos_embed=pos)
        B.sparseloco_reproject_embedding(ts_io, tp_io, u, ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    ts_g, tp_g = ts.clone(), tp.clone()
    with torch.cuda.stream(side):
        work(x, ts_g.clone(), tp_g.clone(), xt, xh)                 # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        work(x, ts_g, tp_g, xt, xh)
    for rep in range(3):
        x.copy_(torch.randn(rows, d, generator=gen, device="cuda"))
        ts_g.copy_(torch.randn(vocab, d, generator=gen, device="cuda"))
        tp_g.copy_(tp)
        ts_e, tp_e = ts_g.clone(), tp_g.clone()
        xt_e, xh_e = torch.empty_like(xt), torch.empty_like(xh)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        work(x, ts_e, tp_e, xt_e, xh_e)                              # eager, same inputs
        torch.cuda.synchronize()
        # the eager project / reconstruct ran before the eager re-projection changed tp_e, as in the graph
        assert torch.equal(xt, xt_e) and torch.equal(xh, xh_e), "replay %d: stage boundary" % rep
        assert torch.equal(ts_g, ts_e) and torch.equal(tp_g, tp_e), "replay %d: re-projection" % rep


def test_random_shapes_of_all_three_calls():
    """Eighty seeded random shapes around the tile sizes (rows, d and k on, just below and just above multiples of
    16, 32, 64 and 128; either table present or absent), each call held to the bars of the tests above."""
    rng = np.random.default_rng(12345)
    for it in range(80):
        rows = int(rng.choice([1, 7, 16, 17, 63, 64, 65, 129, 300, 1000, 2049]))
        d = int(rng.choice([1, 4, 31, 32, 33, 64, 96, 100, 128, 160, 256, 257, 512, 1024]))
        k = int(min(d, rng.choice([1, 2, 3, 4, 5, 8, 15, 16, 17, 31, 32, 33, 48, 63, 64, 65, 100, 128, 129, 200, 256])))
        seq, vocab = int(rng.integers(1, rows + 1)), int(rng.integers(1, 200))
        use_perp, use_pos = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        what = "case %d: rows %d d %d k %d seq %d vocab %d perp %d pos %d" % (it, rows, d, k, seq, vocab, use_perp, use_pos)
        u = subspace.orthonormal_basis(d, k, it).astype(np.float32)
        x = rng.standard_normal((rows, d)).astype(np.float32)
        tp = (rng.standard_normal((vocab, d)) * 0.5).astype(np.float32) if use_perp else None
        tok = rng.integers(0, vocab, rows).astype(np.int32) if use_perp else None
        pos = (rng.standard_normal((seq, d)) * 0.5).astype(np.float32) if use_pos else None
        dev = lambda a: None if a is None else torch.from_numpy(a.copy()).cuda()
        g_x, g_u, g_tp, g_tok, g_pos = dev(x), dev(u), dev(tp), dev(tok), dev(pos)
        out_t = torch.full((rows, k), float("nan"), device="cuda")
        B.sparseloco_subspace_project(g_x, g_u, out_t, t_perp=g_tp, token_ids=g_tok, pos_embed=g_pos)
        # the roundings of fl(fl(x - t) - p) scale with the operands, not with t + p (which may cancel)
        scale = np.linalg.norm(x.astype(np.float64), axis=1)
        if tp is not None:
            scale = scale + np.linalg.norm(tp[tok].astype(np.float64), axis=1)
        if pos is not None:
            scale = scale + np.linalg.norm(pos[np.arange(rows) % seq].astype(np.float64), axis=1)
        tol = 8 * (np.sqrt(d) + np.sqrt(k)) * EPS * scale
        got_t = out_t.cpu().numpy()
        assert np.all(np.linalg.norm(got_t.astype(np.float64) - subspace.project(x, u, tp, tok, pos), axis=1) <= tol), what
        out_h = torch.full((rows, d), float("nan"), device="cuda")
        B.sparseloco_subspace_reconstruct(out_t, g_u, out_h, t_perp=g_tp, token_ids=g_tok, pos_embed=g_pos)
        want_h = subspace.reconstruct(got_t, u, tp, tok, pos)
        assert np.all(np.linalg.norm(out_h.cpu().numpy().astype(np.float64) - want_h, axis=1) <= tol), what
        ts = (rng.standard_normal((vocab, d)) * 0.02).astype(np.float32)
        tq = (rng.standard_normal((vocab, d)) * 0.02).astype(np.float32)
        want_ts, want_tq = subspace.reproject(ts, tq, u)
        g_ts, g_tq = dev(ts), dev(tq)
        B.sparseloco_reproject_embedding(g_ts, g_tq, g_u, torch.empty(vocab * k, device="cuda"))
        tol_r = 8 * (np.sqrt(d) + np.sqrt(k)) * EPS * np.linalg.norm(ts.astype(np.float64), axis=1)
        assert np.all(np.linalg.norm(g_ts.cpu().numpy().astype(np.float64) - want_ts, axis=1) <= tol_r), what
        assert np.all(np.linalg.norm(g_tq.cpu().numpy().astype(np.float64) - want_tq, axis=1) <=
                      tol_r + 2 * EPS * np.linalg.norm(tq.astype(np.float64), axis=1)), what
