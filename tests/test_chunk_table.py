"""Host-side bounds check of the chunk table the kernels walk (no GPU: sparseloco_chunk_table computes the
table of a plan on the host).  For the tensor shapes of the five workloads and for fuzzed shapes, in both
layouts: every present local index of every chunk maps inside its tensor, every element of every tensor belongs
to exactly one chunk, chunk numbers follow the documented order, and the streaming path (4-element vector
accesses) is only promised for complete chunks."""
import numpy as np
import pytest

from paper_2601_02360_amd import binding as B
from paper_2601_02360_amd import workloads as W

IDX = np.arange(4096, dtype=np.int64)
LR, LC = IDX >> 6, IDX & 63


def check_table(shapes, tiled, batch=1024):
    rc = [B.rows_cols(s) for s in shapes]
    numels = [r * c for r, c in rc]
    tab = B.chunk_table(shapes, tiled)
    # chunk numbers: a permutation, tensor by tensor in list order
    assert np.array_equal(np.sort(tab["id"]), np.arange(len(tab)))
    by_id = tab[np.argsort(tab["id"])]
    assert np.all(np.diff(by_id["tensor"].astype(np.int64)) >= 0)
    expect_chunks = [(((r + 63) // 64) * ((c + 63) // 64) if (tiled and r > 1) else (r * c + 4095) // 4096) for r, c in rc]
    assert np.array_equal(np.bincount(tab["tensor"], minlength=len(shapes)), expect_chunks)
    assert int(tab["n_c"].sum()) == sum(numels)
    # processing order of the chunks taken one by one: element-wise chunks first, then fp32-only vector chunks,
    # then the rest; the members of four-tile strips follow, strip by strip
    n_single = int((tab["strip"] == 0).sum())
    single, members = tab[:n_single], tab[n_single:]
    assert np.all(single["strip"] == 0)
    cls = np.where(single["vec"] == 0, 0, np.where(single["vec"] == 1, 1, 2))
    assert np.all(np.diff(cls) >= 0) and set(np.unique(tab["vec"])) <= {0, 1, 3}
    if not tiled:
        assert len(members) == 0
    assert len(members) % 4 == 0
    if len(members):
        m4 = members.reshape(-1, 4)
        assert np.array_equal(m4["strip"], np.tile(np.arange(1, 5, dtype=np.uint32), (len(m4), 1)))
        assert np.all(m4["vec"] == 3) and np.all(m4["n_c"] == 4096)            # complete tiles, even row length
        assert np.all(m4["tensor"] == m4["tensor"][:, :1]) and np.all(m4["stride"] == m4["stride"][:, :1])
        assert np.array_equal(m4["id"], m4["id"][:, :1] + np.arange(4, dtype=np.uint32))
        assert np.array_equal(m4["offset"], m4["offset"][:, :1] + 64 * np.arange(4, dtype=np.uint64))
        # a strip's rows (256 floats from the first tile's origin, 64 rows) stay inside the tensor
        last = m4["offset"][:, 0].astype(np.int64) + 63 * m4["stride"][:, 0].astype(np.int64) + 255
        assert np.all(last < np.asarray(numels, dtype=np.int64)[m4["tensor"][:, 0]])
    first = np.concatenate([[0], np.cumsum(expect_chunks)])
    for t, (r, c) in enumerate(rc):
        mine = by_id[first[t]:first[t + 1]]
        if len(mine) == 0:
            continue
        k = np.arange(len(mine), dtype=np.int64)
        if tiled and r > 1:
            nbj = (c + 63) // 64
            bi, bj = k // nbj, k % nbj
            assert np.array_equal(mine["offset"].astype(np.int64), bi * 64 * c + bj * 64)
            assert np.all(mine["stride"] == c)
            assert np.array_equal(mine["h"], np.minimum(64, r - 64 * bi)) and np.array_equal(mine["w"], np.minimum(64, c - 64 * bj))
            assert np.array_equal(mine["last_w"], mine["w"])
            full = (mine["h"] == 64) & (mine["w"] == 64)
            assert np.array_equal(mine["vec"], np.where(full, 1 + 2 * (c % 2 == 0), 0))
        else:
            assert np.array_equal(mine["offset"].astype(np.int64), 4096 * k) and np.all(mine["stride"] == 64)
            assert np.array_equal(mine["vec"], np.where(mine["n_c"] == 4096, 3, 0))
        cover = np.zeros(numels[t], np.uint8)
        for s in range(0, len(mine), batch):
            m = mine[s:s + batch]
            h, w, lw = (m[f].astype(np.int64)[:, None] for f in ("h", "w", "last_w"))
            present = ((LR[None, :] < h - 1) & (LC[None, :] < w)) | ((LR[None, :] == h - 1) & (LC[None, :] < lw))
            assert np.array_equal(present.sum(axis=1), m["n_c"])
            at = m["offset"].astype(np.int64)[:, None] + LR[None, :] * m["stride"].astype(np.int64)[:, None] + LC[None, :]
            at = at[present]
            assert at.min() >= 0 and at.max() < numels[t], "chunk element outside tensor %d" % t
            cover[at] += 1
        assert cover.min() == 1 and cover.max() == 1, "tensor %d not covered exactly once" % t


@pytest.mark.parametrize("tiled", [False, True], ids=["flat", "tile"])
@pytest.mark.parametrize("workload", [0, 1, 2, 4])
def test_every_distinct_shape_of_the_workloads(workload, tiled):
    shapes = sorted(set(W.tensor_shapes(workload)))
    check_table(shapes, tiled)


@pytest.mark.parametrize("tiled", [False, True], ids=["flat", "tile"])
def test_whole_tensor_lists_of_the_workloads(tiled):
    """All 110 / 146 tensors at once: counts, numbering and ordering (the per-element check runs above)."""
    for workload in (1, 2, 4):
        shapes = W.tensor_shapes(workload)
        tab = B.chunk_table(shapes, tiled)
        assert np.array_equal(np.sort(tab["id"]), np.arange(len(tab)))
        assert int(tab["n_c"].sum()) == sum(W.numels(workload))
        if not tiled:
            assert len(tab) == sum((n + 4095) // 4096 for n in W.numels(workload))


@pytest.mark.parametrize("seed", range(6))
def test_fuzzed_shapes(seed):
    rng = np.random.default_rng(seed)
    edge = [0, 1, 2, 3, 63, 64, 65, 127, 128, 129, 200, 257]
    shapes = []
    for _ in range(12):
        kind = rng.integers(0, 3)
        if kind == 0:
            shapes.append((int(rng.choice(edge + [4095, 4096, 4097, 9000])),))
        else:
            shapes.append((int(rng.choice(edge)), int(rng.choice(edge + [1000]))))
    if not any(np.prod(s) for s in shapes):
        shapes.append((5,))
    check_table(shapes, False)
    check_table(shapes, True)


def test_strips_take_every_run_of_four_complete_tiles():
    tab = B.chunk_table([(128, 1030), (130, 255), (64, 264), (64, 513), (7,), (64, 256)], True)
    strips = tab[tab["strip"] == 1]
    # 128 x 1030: 2 tile rows x 16 complete tiles -> 8 strips; 130 x 255: 3 complete tiles per row -> none;
    # 64 x 264: one strip; 64 x 513: odd row length -> none; 64 x 256: rows are whole cache lines -> none
    assert np.array_equal(np.bincount(strips["tensor"], minlength=6), [8, 0, 1, 0, 0, 0])
    assert len(tab) == 2 * 17 + 3 * 4 + 5 + 9 + 1 + 4


def test_rejections():
    with pytest.raises(B.SparseLoCoError):
        B.chunk_table([], False)
    with pytest.raises(B.SparseLoCoError):
        B.chunk_table([(70, 1 << 24)], True)          # a tile row must span less than 2^32 bytes
    assert len(B.chunk_table([(0,), (0, 5)], True)) == 0
