"""Thin ctypes binding of libsparseloco.so: argument marshalling only.

Every step of the outer step (paper section 2.1) runs in the library's HIP
kernels; this module turns torch tensors into device pointers and passes the
current HIP stream.  There is no fallback: if the library has not been built
(`python -m paper_2601_02360_amd.build`) importing `lib()` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsparseloco.so")

SPLC_CHUNK = 4096
SPLC_OK, SPLC_EINVAL, SPLC_EALIGN, SPLC_ENOMEM, SPLC_EHIP, SPLC_EPLAN, SPLC_ETOOBIG = 0, -1, -2, -3, -4, -5, -6
SPLC_NOALLOC_MAX_COEFF = 8 * 1024 * 1024
SPLC_F32, SPLC_BF16 = 0, 1
SPLC_DELTA_FROM_PARAMS, SPLC_DELTA_DIRECT = 0, 1
SPLC_QUANT_NONE, SPLC_QUANT_2BIT = 0, 1
SPLC_SELECT_AUTO, SPLC_SELECT_RADIX = 0, 1
SPLC_LAYOUT_FLAT, SPLC_LAYOUT_TILE64 = 0, 1
SPLC_MATMUL_FP32, SPLC_MATMUL_BF16X3 = 0, 1

EXPORTS = [
    "sparseloco_plan_create", "sparseloco_plan_create_2d", "sparseloco_plan_destroy", "sparseloco_plan_num_chunks",
    "sparseloco_plan_layout",
    "sparseloco_plan_num_params", "sparseloco_plan_kappa", "sparseloco_plan_quant_mode",
    "sparseloco_plan_set_select", "sparseloco_compress", "sparseloco_aggregate",
    "sparseloco_outer_update", "sparseloco_aggregate_update", "sparseloco_compress_batch",
    "sparseloco_reproject_embedding", "sparseloco_reproject_embedding_noalloc", "sparseloco_subspace_project", "sparseloco_subspace_reconstruct",
    "sparseloco_set_matmul_mode", "sparseloco_get_matmul_mode", "sparseloco_strerror",
]

_lib = None


class SparseLoCoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().sparseloco_strerror(status).decode()
        super().__init__("%s: %s (%d)" % (where, msg, status))


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libsparseloco.so is not built; run `python -m paper_2601_02360_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float
        pp = ctypes.POINTER(ctypes.c_void_p)
        L.sparseloco_plan_create.restype = i32
        L.sparseloco_plan_create.argtypes = [pp, i32, ctypes.POINTER(i64), i32, i32]
        L.sparseloco_plan_create_2d.restype = i32
        L.sparseloco_plan_create_2d.argtypes = [pp, i32, ctypes.POINTER(i64), ctypes.POINTER(i64), i32, i32]
        L.sparseloco_plan_layout.restype = i32
        L.sparseloco_plan_layout.argtypes = [vp]
        L.sparseloco_plan_destroy.restype = None
        L.sparseloco_plan_destroy.argtypes = [vp]
        L.sparseloco_plan_num_chunks.restype = i64
        L.sparseloco_plan_num_chunks.argtypes = [vp]
        L.sparseloco_plan_num_params.restype = i64
        L.sparseloco_plan_num_params.argtypes = [vp]
        L.sparseloco_plan_kappa.restype = i32
        L.sparseloco_plan_kappa.argtypes = [vp]
        L.sparseloco_plan_quant_mode.restype = i32
        L.sparseloco_plan_quant_mode.argtypes = [vp]
        L.sparseloco_plan_set_select.restype = i32
        L.sparseloco_plan_set_select.argtypes = [vp, i32]
        L.sparseloco_set_matmul_mode.restype = i32
        L.sparseloco_set_matmul_mode.argtypes = [i32]
        L.sparseloco_get_matmul_mode.restype = i32
        L.sparseloco_get_matmul_mode.argtypes = []
        L.sparseloco_compress.restype = i32
        L.sparseloco_compress.argtypes = [vp, i32, i32, pp, pp, pp, f32, vp, vp, vp]
        L.sparseloco_aggregate.restype = i32
        L.sparseloco_aggregate.argtypes = [vp, i32, pp, pp, pp, vp]
        L.sparseloco_outer_update.restype = i32
        L.sparseloco_outer_update.argtypes = [vp, pp, pp, f32, vp]
        L.sparseloco_aggregate_update.restype = i32
        L.sparseloco_aggregate_update.argtypes = [vp, i32, pp, pp, pp, f32, pp, i32, ctypes.POINTER(pp), vp]
        L.sparseloco_compress_batch.restype = i32
        L.sparseloco_compress_batch.argtypes = [vp, i32, pp, ctypes.POINTER(pp), ctypes.POINTER(pp), f32, pp, pp, vp]
        L.sparseloco_reproject_embedding.restype = i32
        L.sparseloco_reproject_embedding.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp]
        L.sparseloco_reproject_embedding_noalloc.restype = i32
        L.sparseloco_reproject_embedding_noalloc.argtypes = [vp, vp, vp, i64, i32, i32, vp]
        for fn in (L.sparseloco_subspace_project, L.sparseloco_subspace_reconstruct):
            fn.restype = i32
            fn.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp, i64, i32, i32, vp]
        L.sparseloco_strerror.restype = ctypes.c_char_p
        L.sparseloco_strerror.argtypes = [i32]
        _lib = L
    return _lib


def ptr_table(tensors: Sequence[Optional[torch.Tensor]]):
    """Host array of device pointers for a list of tensors (build once, reuse across calls)."""
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None or t.numel() == 0 else t.data_ptr()
    return arr


def _table(x):
    return x if isinstance(x, ctypes.Array) else ptr_table(x)


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return h or None


def rows_cols(shape):
    """(rows, cols) of a tensor for the tiled layout: leading dimensions fold into rows; 1-D -> (1, n)."""
    if isinstance(shape, int):
        return 1, int(shape)
    shape = tuple(int(v) for v in shape)
    if len(shape) <= 1:
        return 1, (shape[0] if shape else 1)
    rows = 1
    for v in shape[:-1]:
        rows *= v
    return rows, shape[-1]


class Plan:
    """Chunk table and staging slots for a list of tensors.

    shapes: per tensor its numel (int) or its shape.  tiled=False: chunks are 4096 consecutive
    elements (sparseloco_plan_create); tiled=True: 64 x 64 tiles of each tensor seen as a
    (rows, cols) matrix (sparseloco_plan_create_2d)."""

    def __init__(self, shapes: Sequence, kappa: int, quant: bool = True, tiled: bool = False):
        self._h = ctypes.c_void_p()
        n = len(shapes)
        rc_list = [rows_cols(s) for s in shapes]
        numels = [r * c for r, c in rc_list]
        q = SPLC_QUANT_2BIT if quant else SPLC_QUANT_NONE
        if tiled:
            rows = (ctypes.c_int64 * max(n, 1))(*[r for r, _ in rc_list])
            cols = (ctypes.c_int64 * max(n, 1))(*[c for _, c in rc_list])
            rc = lib().sparseloco_plan_create_2d(ctypes.byref(self._h), n, rows, cols, int(kappa), q)
        else:
            arr = (ctypes.c_int64 * max(n, 1))(*numels)
            rc = lib().sparseloco_plan_create(ctypes.byref(self._h), n, arr, int(kappa), q)
        if rc != SPLC_OK:
            self._h = ctypes.c_void_p()
            raise SparseLoCoError(rc, "sparseloco_plan_create")
        self.numels = numels
        self.tiled = bool(tiled)
        self.kappa = int(kappa)
        self.quant = bool(quant)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().sparseloco_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    @property
    def num_chunks(self) -> int:
        return int(lib().sparseloco_plan_num_chunks(self._h))

    @property
    def num_params(self) -> int:
        return int(lib().sparseloco_plan_num_params(self._h))

    def set_select(self, mode: int) -> None:
        rc = lib().sparseloco_plan_set_select(self._h, int(mode))
        if rc != SPLC_OK:
            raise SparseLoCoError(rc, "sparseloco_plan_set_select")

    def message_buffers(self, device="cuda"):
        """Freshly allocated (pairs, aux) for one replica's message."""
        nch = self.num_chunks
        pairs = torch.empty(nch * self.kappa, dtype=torch.int16, device=device)
        aux = torch.empty(nch * 2 if self.quant else nch * self.kappa, dtype=torch.float32, device=device)
        return pairs, aux


def sparseloco_compress(plan: Plan, ef, pairs_out: torch.Tensor, aux_out: torch.Tensor, beta: float, *,
                        theta_outer=None, theta_local=None, delta=None, delta_dtype=SPLC_F32, stream=None) -> None:
    """Lines 1-4 of the update equations for one replica.  ef / theta_* / delta: lists of
    tensors or prebuilt ptr_table()s."""
    if delta is not None:
        mode, a, b = SPLC_DELTA_DIRECT, _table(delta), None
        if not isinstance(delta, ctypes.Array) and len(delta) and delta[0].dtype == torch.bfloat16:
            delta_dtype = SPLC_BF16
    else:
        mode, a, b, delta_dtype = SPLC_DELTA_FROM_PARAMS, _table(theta_outer), _table(theta_local), SPLC_F32
    rc = lib().sparseloco_compress(plan.handle, mode, delta_dtype, a, b, _table(ef), float(beta),
                                   pairs_out.data_ptr(), aux_out.data_ptr(), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_compress")


def sparseloco_aggregate(plan: Plan, pairs, aux, delta_bar_out, *, stream=None) -> None:
    """Mean over replicas of the decoded messages into dense fp32 tensors."""
    pt, at = _table(pairs), _table(aux)
    rc = lib().sparseloco_aggregate(plan.handle, len(pt), pt, at, _table(delta_bar_out), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_aggregate")


def sparseloco_outer_update(plan: Plan, theta_outer, delta_bar, outer_lr: float, *, stream=None) -> None:
    """theta_outer -= outer_lr * delta_bar, in place."""
    rc = lib().sparseloco_outer_update(plan.handle, _table(theta_outer), _table(delta_bar), float(outer_lr),
                                       _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_outer_update")


def sparseloco_aggregate_update(plan: Plan, pairs, aux, theta_outer, outer_lr: float, *, delta_bar_out=None,
                                reset=None, stream=None) -> None:
    """Mean over replicas and outer update in one pass (theta_outer in place); delta_bar_out optional;
    reset: per replica a list of theta_local tensors (or a ptr_table_2d) that receive the new theta_outer."""
    pt, at = _table(pairs), _table(aux)
    rt = None
    if reset is not None:
        rt = reset if isinstance(reset, ctypes.Array) and hasattr(reset, "_keepalive") else ptr_table_2d(reset)
    rc = lib().sparseloco_aggregate_update(plan.handle, len(pt), pt, at, _table(theta_outer), float(outer_lr),
                                           None if delta_bar_out is None else _table(delta_bar_out),
                                           0 if rt is None else len(rt), rt, _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_aggregate_update")


def ptr_table_2d(tables):
    """Host array of host pointer tables (one ptr_table per replica)."""
    tabs = [_table(t) for t in tables]
    pp = ctypes.POINTER(ctypes.c_void_p)
    arr = (pp * len(tabs))(*[ctypes.cast(t, pp) for t in tabs])
    arr._keepalive = tabs
    return arr


def sparseloco_compress_batch(plan: Plan, theta_outer, theta_local, ef, pairs_out, aux_out, beta: float, *,
                              stream=None) -> None:
    """Lines 1-4 for R replicas sharing theta_outer, one launch.  theta_local / ef: per replica a list of
    tensors (or ptr_table), or a prebuilt ptr_table_2d; pairs_out / aux_out: per replica message buffers."""
    tl = theta_local if isinstance(theta_local, ctypes.Array) and hasattr(theta_local, "_keepalive") \
        else ptr_table_2d(theta_local)
    e = ef if isinstance(ef, ctypes.Array) and hasattr(ef, "_keepalive") else ptr_table_2d(ef)
    rc = lib().sparseloco_compress_batch(plan.handle, len(tl), _table(theta_outer), tl, e, float(beta),
                                         _table(pairs_out), _table(aux_out), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_compress_batch")


def sparseloco_reproject_embedding(t_s: torch.Tensor, t_perp: torch.Tensor, u: torch.Tensor,
                                   coeff_ws: torch.Tensor, *, stream=None) -> None:
    """T_perp += T_S - T_S U U^T; T_S = T_S U U^T (in place).  t_s, t_perp: [vocab, d]; u: [d, k];
    coeff_ws: at least vocab * k floats."""
    vocab, d = t_s.shape
    k = u.shape[1]
    assert t_perp.shape == t_s.shape and u.shape[0] == d and coeff_ws.numel() >= vocab * k
    assert all(x.dtype == torch.float32 and x.is_contiguous() for x in (t_s, t_perp, u, coeff_ws))
    rc = lib().sparseloco_reproject_embedding(t_s.data_ptr(), t_perp.data_ptr(), u.data_ptr(), coeff_ws.data_ptr(),
                                              int(vocab), int(d), int(k), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_reproject_embedding")


def sparseloco_reproject_embedding_noalloc(t_s: torch.Tensor, t_perp: torch.Tensor, u: torch.Tensor, *,
                                           stream=None) -> None:
    """sparseloco_reproject_embedding with the coefficients in the library's fixed per-GPU array (no allocation,
    no caller workspace); vocab * k <= SPLC_NOALLOC_MAX_COEFF."""
    vocab, d = t_s.shape
    k = u.shape[1]
    assert t_perp.shape == t_s.shape and u.shape[0] == d
    assert all(x.dtype == torch.float32 and x.is_contiguous() for x in (t_s, t_perp, u))
    rc = lib().sparseloco_reproject_embedding_noalloc(t_s.data_ptr(), t_perp.data_ptr(), u.data_ptr(), int(vocab),
                                                      int(d), int(k), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_reproject_embedding_noalloc")


def sparseloco_set_matmul_mode(mode: int) -> None:
    """SPLC_MATMUL_FP32 (default) or SPLC_MATMUL_BF16X3 for the dense products of the three calls around here."""
    rc = lib().sparseloco_set_matmul_mode(int(mode))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_set_matmul_mode")


def sparseloco_get_matmul_mode() -> int:
    return int(lib().sparseloco_get_matmul_mode())


def _opt(t):
    return None if t is None else t.data_ptr()


def sparseloco_subspace_project(x: torch.Tensor, u: torch.Tensor, out: torch.Tensor, *, t_perp=None, token_ids=None,
                                pos_embed=None, stream=None) -> None:
    """out[rows, k] = (x - t_perp[token_ids] - pos_embed[row % seq_len]) @ u;  x: [rows, d], u: [d, k]."""
    rows, d = x.shape
    k = u.shape[1]
    assert out.shape == (rows, k) and x.is_contiguous() and u.is_contiguous() and out.is_contiguous()
    assert token_ids is None or token_ids.dtype == torch.int32
    rc = lib().sparseloco_subspace_project(x.data_ptr(), _opt(t_perp), _opt(token_ids),
                                           0 if t_perp is None else t_perp.shape[0], _opt(pos_embed),
                                           0 if pos_embed is None else pos_embed.shape[0], u.data_ptr(),
                                           out.data_ptr(), int(rows), int(d), int(k), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_subspace_project")


def sparseloco_subspace_reconstruct(x_tilde: torch.Tensor, u: torch.Tensor, out: torch.Tensor, *, t_perp=None,
                                    token_ids=None, pos_embed=None, stream=None) -> None:
    """out[rows, d] = x_tilde @ u.T + t_perp[token_ids] + pos_embed[row % seq_len]."""
    rows, k = x_tilde.shape
    d = u.shape[0]
    assert out.shape == (rows, d) and x_tilde.is_contiguous() and u.is_contiguous() and out.is_contiguous()
    assert token_ids is None or token_ids.dtype == torch.int32
    rc = lib().sparseloco_subspace_reconstruct(x_tilde.data_ptr(), _opt(t_perp), _opt(token_ids),
                                               0 if t_perp is None else t_perp.shape[0], _opt(pos_embed),
                                               0 if pos_embed is None else pos_embed.shape[0], u.data_ptr(),
                                               out.data_ptr(), int(rows), int(d), int(k), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_subspace_reconstruct")
