"""GPU parity of the dense products around the outer step -- the embedding re-projection (paper section 2.4)
and the stage boundary (section 2.2) -- against the float64 oracle, ELEMENT BY ELEMENT.

Bar, from the arithmetic.  The GPU forms every output as an fp32 dot product with fp32 accumulation in an
unspecified order.  For any order, |fl(sum a_i b_i) - sum a_i b_i| <= gamma_n (|a| . |b|) with gamma_n ~ n u,
u = 2^-24; that worst case needs every rounding to err the same way.  With roundings of either sign the error of
n sequential accumulations has standard deviation of the order of u (|a| . |b|) whatever n is (each step errs by
at most u |partial sum|, partial sums grow like sqrt(j), and |a| . |b| grows like n).  Measured on the matrix
cores at the benchmarked shapes (some 10^8 outputs each): the largest error is 7 u (|A| |B|)_ij.  The bar is
C u (|A| |B|)_ij  with C = 16 -- twice the largest error seen -- propagated through the chain of operations of
each call:
  re-projection  coeff = T U:            C u (|T| |U|)
                 R = coeff U^T:          C u ((|T| |U|) |U|^T  +  |coeff| |U|^T)      (error of coeff carried along)
                 T_perp' = T_perp + (T - R): bar(R) + 2 u (|T| + |R| + |T_perp'|)
  project        A = fl(fl(x - t) - p):  2 u (|x| + |t| + |p|) per element, then C u (|A| |U|) for the product
  reconstruct    fl(fl(v + t) + p):      C u (|x~| |U|^T) + 2 u (|v| + |t| + |p|)
A dropped or misplaced product term changes an output by about (|A| |B|)_ij / n >= 5e-4 (|A| |B|)_ij at
n = 2048, five hundred times the bar of 1e-6 (|A| |B|)_ij.

Every test runs twice: with fp32 MFMA products and with SPLC_MATMUL_BF16X3 (operands split exactly into three
bf16 pieces, six piece products per product).  The split drops less than 3 * 2^-24 |x y| per product, of either
sign -- inside the same bar -- and products with an exact result (a coordinate subspace) stay exact.

The shapes are chosen so that every tile shape of the GEMM kernel (128 or 64 rows by 128 or 64 columns, with
the second operand given as K x N and as N x K) and both widths of the narrow projection kernel run against the
oracle in both modes: test_every_kernel_variant_is_reached asserts it with the library's own launch rule.
"""
import numpy as np
import pytest
import torch

from oracle import subspace
from paper_2601_02360_amd import binding as B
from paper_2601_02360_amd import workloads as W

pytestmark = pytest.mark.gpu
U24 = 2.0 ** -24
C = 16.0


@pytest.fixture(autouse=True, params=[B.SPLC_MATMUL_FP32, B.SPLC_MATMUL_BF16X3], ids=["fp32", "bf16x3"])
def matmul_mode(request):
    return request.param


def gpu_randn(shape, seed, std=1.0):
    g = torch.Generator(device="cuda").manual_seed(int(seed))
    return torch.randn(*shape, generator=g, device="cuda") * std


def f64(t):
    return t.detach().cpu().numpy().astype(np.float64)


def assert_within(got, want, bar, what):
    err = np.abs(got - want)
    bad = err > bar
    if bad.any():
        i = np.unravel_index(np.argmax(err - bar), err.shape)
        raise AssertionError("%s: %d of %d elements beyond the bar; worst at %r: got %.9g want %.9g, |diff| %.3g, bar %.3g"
                             % (what, int(bad.sum()), err.size, i, got[i], want[i], err[i], bar[i]))
    with np.errstate(divide="ignore", invalid="ignore"):
        return float(np.nanmax(np.where(bar > 0, err / bar, 0.0)))


# ---------------------------------------------------------------- re-projection (section 2.4)

def check_reproject(vocab, d, k, seed, mode, rows=None):
    """rows: check these rows only (the oracle's products are row-independent); default all."""
    u32 = W.orthonormal_basis(d, k, seed, "cuda")
    ts, tp = gpu_randn((vocab, d), seed + 1, 0.02), gpu_randn((vocab, d), seed + 2, 0.02)
    g_ts, g_tp = ts.clone(), tp.clone()
    ws = torch.full((max(vocab * k, 1),), float("nan"), device="cuda")
    B.sparseloco_reproject_embedding(g_ts, g_tp, u32, ws, matmul=mode)
    torch.cuda.synchronize()
    sel = slice(None) if rows is None else torch.as_tensor(rows, device="cuda")
    T, P, U = f64(ts[sel]), f64(tp[sel]), f64(u32)
    want_ts, want_tp = subspace.reproject(T, P, U)                # the oracle sees the same fp32 inputs
    absU = np.abs(U)
    bar_c = C * U24 * (np.abs(T) @ absU)
    coeff = f64(ws[:vocab * k].view(vocab, k)[sel])
    worst = [assert_within(coeff, T @ U, bar_c, "coefficients T_S U")]
    bar_r = bar_c @ absU.T + C * U24 * (np.abs(coeff) @ absU.T)
    worst.append(assert_within(f64(g_ts[sel]), want_ts, bar_r, "T_S"))
    bar_p = bar_r + 2 * U24 * (np.abs(T) + np.abs(want_ts) + np.abs(want_tp))
    worst.append(assert_within(f64(g_tp[sel]), want_tp, bar_p, "T_perp"))
    # T_S + T_perp is conserved up to the roundings of the update itself
    assert_within(f64(g_ts[sel]) + f64(g_tp[sel]), T + P, 4 * U24 * (np.abs(T) + np.abs(want_ts) + np.abs(want_tp)) + 1e-300,
                  "T_S + T_perp")
    return max(worst)


REPROJECT_SHAPES = [(128, 128, 128), (256, 256, 32), (300, 200, 7), (1, 64, 2), (129, 130, 130),
                    (1000, 768, 96), (517, 1536, 2), (64, 2048, 256), (2000, 1024, 128),
                    # narrow bases: both passes (k <= 32 in fours, or k <= 8), pass 1 only (k <= 64)
                    (100, 64, 8), (33, 96, 20), (2000, 1024, 16), (70, 32, 32), (300, 128, 64),
                    (17, 160, 5), (4097, 512, 4), (250, 2048, 48),
                    # the 128-row tiles: pass 2 on 128 x 128 (512 workgroups, K = 256) and on 128 x 64 (d = 17 blocks
                    # of 64), pass 1 on 128 x 64 (k = 192) -- and a K tail on the tall tile (k = 250)
                    (8192, 1024, 256), (4096, 1088, 256), (22000, 256, 192), (8200, 1024, 250)]


@pytest.mark.parametrize("vocab,d,k", REPROJECT_SHAPES)
def test_reproject_matches_the_oracle(vocab, d, k, matmul_mode):
    check_reproject(vocab, d, k, seed=vocab + d + k, mode=matmul_mode)


@pytest.mark.parametrize("k", [256, 192])
def test_reproject_at_the_benchmarked_shape(k, matmul_mode):
    """Vocabulary 32000, d 2048 (the 1B shape bench.py --op reproject times), every row and element."""
    worst = check_reproject(32000, 2048, k, seed=7 + k, mode=matmul_mode)
    print("largest error / bar at 32000 x 2048, k = %d: %.3f" % (k, worst))


def test_coordinate_subspace_is_exact(matmul_mode):
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
    B.sparseloco_reproject_embedding(g_ts, g_tp, g_u, ws, matmul=matmul_mode)
    keep = np.zeros(d, bool)
    keep[cols] = True
    out_ts, out_tp = g_ts.cpu().numpy(), g_tp.cpu().numpy()
    assert np.array_equal(out_ts[:, keep], ts[:, keep]) and not out_ts[:, ~keep].any()
    assert np.array_equal(out_tp[:, ~keep], tp[:, ~keep] + ts[:, ~keep])
    assert np.array_equal(out_tp[:, keep], tp[:, keep])


def test_argument_checks():
    t = torch.zeros(4, 8, device="cuda")
    u = torch.zeros(8, 2, device="cuda")
    L = B.lib()
    p = t.data_ptr()
    assert L.sparseloco_reproject_embedding(None, p, u.data_ptr(), p, 4, 8, 2, 0, None) == B.SPLC_EINVAL
    assert L.sparseloco_reproject_embedding(p, p, u.data_ptr(), p, 4, 8, 9, 0, None) == B.SPLC_EINVAL
    assert L.sparseloco_reproject_embedding(p, p, u.data_ptr(), p, 4, 8, 2, 7, None) == B.SPLC_EINVAL     # matmul mode
    assert L.sparseloco_reproject_embedding(p, p, u.data_ptr(), p, 0, 8, 2, 0, None) == B.SPLC_OK
    assert L.sparseloco_subspace_project(p, None, None, 0, None, 0, u.data_ptr(), p, 4, 8, 2, 2, None) == B.SPLC_EINVAL


# ---------------------------------------------------------------- stage boundary (section 2.2)

def check_stage_boundary(rows, seq, d, k, vocab, use_perp, use_pos, seed, mode, what=""):
    u32 = W.orthonormal_basis(d, k, seed, "cuda")
    x = gpu_randn((rows, d), seed + 1)
    tp = gpu_randn((vocab, d), seed + 2, 0.5) if use_perp else None
    pos = gpu_randn((seq, d), seed + 3, 0.5) if use_pos else None
    tok = None
    if use_perp:
        g = torch.Generator(device="cuda").manual_seed(seed + 4)
        tok = torch.randint(0, vocab, (rows,), generator=g, device="cuda", dtype=torch.int32)
    out_t = torch.full((rows, k), float("nan"), device="cuda")
    B.sparseloco_subspace_project(x, u32, out_t, t_perp=tp, token_ids=tok, pos_embed=pos, matmul=mode)
    X, U = f64(x), f64(u32)
    TP = None if tp is None else f64(tp)
    PS = None if pos is None else f64(pos)
    TK = None if tok is None else tok.cpu().numpy()
    want_t = subspace.project(X, U, TP, TK, PS)
    t_rows = np.zeros_like(X) if TP is None else TP[TK]
    p_rows = np.zeros_like(X) if PS is None else PS[np.arange(rows) % seq]
    absU = np.abs(U)
    a_exact = X - t_rows - p_rows
    bar_t = U24 * ((C * np.abs(a_exact) + 2 * (np.abs(X) + np.abs(t_rows) + np.abs(p_rows))) @ absU)
    worst = [assert_within(f64(out_t), want_t, bar_t, "project " + what)]
    # reconstruct from the GPU's own x_tilde, compared with the oracle applied to the same x_tilde
    out_h = torch.full((rows, d), float("nan"), device="cuda")
    B.sparseloco_subspace_reconstruct(out_t, u32, out_h, t_perp=tp, token_ids=tok, pos_embed=pos, matmul=mode)
    XT = f64(out_t)
    want_h = subspace.reconstruct(XT, U, TP, TK, PS)
    v = XT @ U.T
    bar_h = C * U24 * (np.abs(XT) @ absU.T) + 2 * U24 * (np.abs(v) + np.abs(t_rows) + np.abs(p_rows))
    worst.append(assert_within(f64(out_h), want_h, bar_h, "reconstruct " + what))
    return max(worst)


STAGE_SHAPES = [
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
    (64, 8, 48, 1, 3, True, True), (2000, 200, 2048, 170, 100, True, False),
    # 128-row tiles of the projection: 128 x 128 (k = 256, 32768 rows) and 128 x 64 (k = 192), with and without tables
    (32768, 1024, 512, 256, 1000, True, True), (22016, 512, 384, 192, 300, False, False),
    (33000, 1000, 320, 250, 77, False, True)]


@pytest.mark.parametrize("rows,seq,d,k,vocab,use_perp,use_pos", STAGE_SHAPES)
def test_project_and_reconstruct_match_the_oracle(rows, seq, d, k, vocab, use_perp, use_pos, matmul_mode):
    check_stage_boundary(rows, seq, d, k, vocab, use_perp, use_pos, seed=rows + d + k, mode=matmul_mode)


def test_stage_boundary_at_the_benchmarked_shape(matmul_mode):
    """16384 tokens, d 2048, k 256, vocabulary 32000, both tables: what bench.py --op project times."""
    worst = check_stage_boundary(16384, 1024, 2048, 256, 32000, True, True, seed=3, mode=matmul_mode)
    print("largest error / bar at the stage-boundary bench shape: %.3f" % worst)


def test_every_kernel_variant_is_reached(matmul_mode):
    """The shapes above, run through the library's own launch rule, cover all eight tile shapes of the GEMM
    kernel (rows x columns x operand form) and both narrow kernels, in this matmul mode."""
    reached = set()
    for vocab, d, k in REPROJECT_SHAPES + [(32000, 2048, 256), (32000, 2048, 192)]:
        reached.add(("KxN",) + B.subspace_kernel_choice(B.SPLC_OP_REPROJECT_PASS1, vocab, d, k, 0, matmul_mode))
        reached.add(("NxK",) + B.subspace_kernel_choice(B.SPLC_OP_REPROJECT_PASS2, vocab, d, k, 0, matmul_mode))
    for rows, seq, d, k, vocab, use_perp, use_pos in STAGE_SHAPES + [(16384, 1024, 2048, 256, 32000, True, True)]:
        tables = int(use_perp) + int(use_pos)
        reached.add(("KxN",) + B.subspace_kernel_choice(B.SPLC_OP_PROJECT, rows, d, k, tables, matmul_mode))
        reached.add(("NxK",) + B.subspace_kernel_choice(B.SPLC_OP_RECONSTRUCT, rows, d, k, tables, matmul_mode))
    want = {(form, tm, tn) for form in ("KxN", "NxK") for tm in (64, 128) for tn in (64, 128)}
    if matmul_mode == B.SPLC_MATMUL_BF16X3:          # with split operands an N x K product always takes 128 rows
        want -= {("NxK", 64, 64), ("NxK", 64, 128)}
    want |= {("KxN", 16, 16), ("KxN", 16, 32)}
    assert want <= reached, "not reached: %r" % sorted(want - reached)


def test_subspace_calls_replay_from_a_hip_graph(matmul_mode):
    """The matrix entry points only enqueue kernels, so they can be recorded into a HIP graph: three replays on
    fresh inputs, with eager work and synchronisation in between, each equal to the eager result bit for bit."""
    rows, seq, d, k, vocab = 500, 50, 256, 40, 64
    gen = torch.Generator(device="cuda").manual_seed(17)
    u = W.orthonormal_basis(d, k, 3, "cuda")
    x = torch.randn(rows, d, generator=gen, device="cuda")
    tp = torch.randn(vocab, d, generator=gen, device="cuda") * 0.5
    pos = torch.randn(seq, d, generator=gen, device="cuda") * 0.5
    tok = torch.randint(0, vocab, (rows,), generator=gen, device="cuda", dtype=torch.int32)
    ts = torch.randn(vocab, d, generator=gen, device="cuda")
    xt, xh = torch.empty(rows, k, device="cuda"), torch.empty(rows, d, device="cuda")
    ws = torch.empty(vocab * k, device="cuda")

    def work(x_in, ts_io, tp_io, xt_out, xh_out):
        B.sparseloco_subspace_project(x_in, u, xt_out, t_perp=tp_io, token_ids=tok, pos_embed=pos, matmul=matmul_mode)
        B.sparseloco_subspace_reconstruct(xt_out, u, xh_out, t_perp=tp_io, token_ids=tok, pos_embed=pos,
                                          matmul=matmul_mode)
        B.sparseloco_reproject_embedding(ts_io, tp_io, u, ws, matmul=matmul_mode)

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


def test_random_shapes_of_all_three_calls(matmul_mode):
    """Eighty seeded random shapes around the tile sizes (rows, d and k on, just below and just above multiples of
    16, 32, 64 and 128; either table present or absent), each call held to the element-wise bars above."""
    rng = np.random.default_rng(12345)
    for it in range(80):
        rows = int(rng.choice([1, 7, 16, 17, 63, 64, 65, 129, 300, 1000, 2049]))
        d = int(rng.choice([1, 4, 31, 32, 33, 64, 96, 100, 128, 160, 256, 257, 512, 1024]))
        k = int(min(d, rng.choice([1, 2, 3, 4, 5, 8, 15, 16, 17, 31, 32, 33, 48, 63, 64, 65, 100, 128, 129, 200, 256])))
        seq, vocab = int(rng.integers(1, rows + 1)), int(rng.integers(1, 200))
        use_perp, use_pos = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        what = "case %d: rows %d d %d k %d seq %d vocab %d perp %d pos %d" % (it, rows, d, k, seq, vocab, use_perp, use_pos)
        check_stage_boundary(rows, seq, d, k, vocab, use_perp, use_pos, seed=1000 + 7 * it, mode=matmul_mode, what=what)
        check_reproject(vocab, d, k, seed=5000 + 7 * it, mode=matmul_mode)
