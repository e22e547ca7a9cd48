"""CPU oracle of the SparseLoCo outer step (paper section 2.1) -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares nothing with the GPU library: the arithmetic lives in
sparseloco_oracle.c (plain C, full sort per chunk), compiled with gcc and
called through ctypes on numpy arrays.  Multi-tensor loops are done here in
Python, tensor by tensor, chunk numbering in list order.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparseloco_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

# -ffp-contract=off: one rounding per written operation (no fused multiply-add).
CFLAGS = ["-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (about a second)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_f = ctypes.POINTER(ctypes.c_float)
        c_u16 = ctypes.POINTER(ctypes.c_uint16)
        lib.oracle_compress.restype = ctypes.c_int
        i64, ci = ctypes.c_int64, ctypes.c_int
        lib.oracle_compress.argtypes = [i64, i64, ci, ci, ci, ctypes.c_float, ci,
                                        c_f, c_f, c_f, c_u16, c_f, c_u16, c_f, c_f]
        lib.oracle_decode.restype = ctypes.c_int
        lib.oracle_decode.argtypes = [i64, i64, ci, ci, ci, ci, c_u16, c_f, c_f, c_f]
        lib.oracle_aggregate.restype = ctypes.c_int
        lib.oracle_aggregate.argtypes = [i64, i64, ci, ci, ci, ci, ci,
                                         ctypes.POINTER(c_u16), ctypes.POINTER(c_f), ctypes.POINTER(c_f), c_f]
        lib.oracle_outer_update.restype = ctypes.c_int
        lib.oracle_outer_update.argtypes = [ctypes.c_int64, c_f, c_f, ctypes.c_float]
        _lib = lib
    return _lib


def _fp(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _u16p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.uint16 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _rc(shape) -> tuple:
    """(rows, cols) of a tensor given its numel or its shape: 1-D -> (1, n); N-D -> (prod(leading), last)."""
    if isinstance(shape, (int, np.integer)):
        return 1, int(shape)
    shape = tuple(int(v) for v in shape)
    if len(shape) == 0:
        return 1, 1
    if len(shape) == 1:
        return 1, shape[0]
    rows = 1
    for v in shape[:-1]:
        rows *= v
    return rows, shape[-1]


def tensor_chunks(shape, chunk: int = 4096, tile: Optional[int] = None) -> int:
    """Chunks of one tensor.  tile=None: flat chunks of `chunk` elements; tile=T: T x T blocks of the
    (rows, cols) matrix (1-D tensors flat with chunk T*T)."""
    rows, cols = _rc(shape)
    if rows * cols == 0:
        return 0
    if tile is None or rows == 1:
        ch = chunk if tile is None else tile * tile
        return (rows * cols + ch - 1) // ch
    return ((rows + tile - 1) // tile) * ((cols + tile - 1) // tile)


def num_chunks(shapes: Sequence, chunk: int = 4096, tile: Optional[int] = None) -> int:
    return sum(tensor_chunks(s, chunk, tile) for s in shapes)


def chunk_offsets(shapes: Sequence, chunk: int = 4096, tile: Optional[int] = None) -> List[int]:
    """First chunk number of every tensor (chunks are numbered tensor by tensor)."""
    out, c = [], 0
    for s in shapes:
        out.append(c)
        c += tensor_chunks(s, chunk, tile)
    return out


def _geom(shape, chunk, tile):
    rows, cols = _rc(shape)
    return (rows, cols, tile, 1) if tile is not None else (1, rows * cols, chunk, 0)


def set_threads(n: int) -> None:
    """OpenMP thread count for the chunk loop (used by the cpu_baseline timing)."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def compress(ef: Sequence[np.ndarray], kappa: int, beta: float, *,
             theta_outer: Optional[Sequence[np.ndarray]] = None,
             theta_local: Optional[Sequence[np.ndarray]] = None,
             delta: Optional[Sequence[np.ndarray]] = None,
             chunk: int = 4096, quant: bool = True, shapes: Optional[Sequence] = None,
             tile: Optional[int] = None):
    """One replica's compress over a list of tensors (flat views are taken).

    Geometry: flat chunks of `chunk` elements, or, with tile=T and shapes (default: the arrays' own
    shapes), T x T blocks of every tensor seen as a (rows, cols) matrix.

    ef: fp32 arrays, updated in place.  Either (theta_outer, theta_local) fp32,
    or delta: fp32 arrays, or uint16 arrays holding bfloat16 bit patterns.
    Returns (pairs u16[n_chunks*kappa], scales f32[n_chunks*2]) when quant, else
    (pairs, values f32[n_chunks*kappa]).
    """
    lib = _load()
    numels = [int(e.size) for e in ef]
    shapes = [e.shape for e in ef] if shapes is None else list(shapes)
    nch = num_chunks(shapes, chunk, tile)
    offs = chunk_offsets(shapes, chunk, tile)
    pairs = np.empty(nch * kappa, np.uint16)
    scales = np.zeros(nch * 2, np.float32) if quant else None
    values = None if quant else np.zeros(nch * kappa, np.float32)
    for t, e in enumerate(ef):
        assert e.dtype == np.float32 and e.flags.c_contiguous
        c0 = offs[t]
        tc = tensor_chunks(shapes[t], chunk, tile)
        p = pairs[c0 * kappa:(c0 + tc) * kappa]
        s = scales[c0 * 2:(c0 + tc) * 2] if quant else None
        v = None if quant else values[c0 * kappa:(c0 + tc) * kappa]
        to = tl = d32 = d16 = None
        if delta is not None:
            d = np.ascontiguousarray(delta[t]).reshape(-1)
            if d.dtype == np.uint16:
                d16 = d
            else:
                assert d.dtype == np.float32
                d32 = d
            assert d.size == numels[t]
        else:
            to = np.ascontiguousarray(theta_outer[t]).reshape(-1)
            tl = np.ascontiguousarray(theta_local[t]).reshape(-1)
            assert to.size == numels[t] and tl.size == numels[t]
        rc = lib.oracle_compress(*_geom(shapes[t], chunk, tile), kappa, beta, 1 if quant else 0,
                                 _fp(to), _fp(tl), _fp(d32), _u16p(d16),
                                 _fp(e.reshape(-1)), _u16p(p), _fp(s), _fp(v))
        if rc != 0:
            raise ValueError("oracle_compress failed: %d" % rc)
    return (pairs, scales) if quant else (pairs, values)


def decode(shapes: Sequence, pairs: np.ndarray, aux: np.ndarray, kappa: int, *,
           chunk: int = 4096, quant: bool = True, tile: Optional[int] = None) -> List[np.ndarray]:
    """Dense flat fp32 arrays of one replica's message (zeros where nothing was sent).
    shapes: per tensor its numel or its shape."""
    lib = _load()
    offs = chunk_offsets(shapes, chunk, tile)
    out = []
    for t, shp in enumerate(shapes):
        rows, cols = _rc(shp)
        n = rows * cols
        c0 = offs[t]
        tc = tensor_chunks(shp, chunk, tile)
        dense = np.empty(n, np.float32)
        p = pairs[c0 * kappa:(c0 + tc) * kappa]
        s = aux[c0 * 2:(c0 + tc) * 2] if quant else None
        v = None if quant else aux[c0 * kappa:(c0 + tc) * kappa]
        rc = lib.oracle_decode(*_geom(shp, chunk, tile), kappa, 1 if quant else 0, _u16p(p), _fp(s), _fp(v),
                               _fp(dense))
        if rc != 0:
            raise ValueError("oracle_decode failed: %d" % rc)
        out.append(dense)
    return out


def aggregate(shapes: Sequence, pairs: Sequence[np.ndarray], aux: Sequence[np.ndarray], kappa: int, *,
              chunk: int = 4096, quant: bool = True, tile: Optional[int] = None) -> List[np.ndarray]:
    """Mean over replicas of the decoded messages; returns dense flat fp32 arrays per tensor.
    shapes: per tensor its numel or its shape."""
    lib = _load()
    R = len(pairs)
    offs = chunk_offsets(shapes, chunk, tile)
    c_f = ctypes.POINTER(ctypes.c_float)
    c_u16 = ctypes.POINTER(ctypes.c_uint16)
    out = []
    for t, shp in enumerate(shapes):
        rows, cols = _rc(shp)
        n = rows * cols
        c0 = offs[t]
        tc = tensor_chunks(shp, chunk, tile)
        ps = [pairs[r][c0 * kappa:(c0 + tc) * kappa] for r in range(R)]
        if quant:
            ss = [aux[r][c0 * 2:(c0 + tc) * 2] for r in range(R)]
            vs = None
        else:
            ss = None
            vs = [aux[r][c0 * kappa:(c0 + tc) * kappa] for r in range(R)]
        pp = (c_u16 * R)(*[_u16p(p) for p in ps])
        sp = (c_f * R)(*[_fp(s) for s in ss]) if ss is not None else None
        vp = (c_f * R)(*[_fp(v) for v in vs]) if vs is not None else None
        dense = np.empty(n, np.float32)
        rc = lib.oracle_aggregate(*_geom(shp, chunk, tile), kappa, 1 if quant else 0, R, pp, sp, vp, _fp(dense))
        if rc != 0:
            raise ValueError("oracle_aggregate failed: %d" % rc)
        out.append(dense)
    return out


def outer_update(theta_outer: Sequence[np.ndarray], delta_bar: Sequence[np.ndarray], outer_lr: float) -> None:
    """theta_outer -= outer_lr * delta_bar, in place, tensor by tensor."""
    lib = _load()
    for th, db in zip(theta_outer, delta_bar):
        assert th.dtype == np.float32 and th.flags.c_contiguous and db.size == th.size
        rc = lib.oracle_outer_update(int(th.size), _fp(th.reshape(-1)),
                                     _fp(np.ascontiguousarray(db).reshape(-1)), outer_lr)
        if rc != 0:
            raise ValueError("oracle_outer_update failed: %d" % rc)


def unpack(pairs: np.ndarray):
    """(index, code, valid) of packed pairs: index = bits 0-11, code = bits 12-13, 0xFFFF = empty slot."""
    p = pairs.astype(np.uint32)
    return p & 0xFFF, (p >> 12) & 3, pairs != 0xFFFF
