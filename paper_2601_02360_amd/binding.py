"""Thin ctypes binding of libsparseloco.so: argument marshalling only.

Every step of the outer step (paper section 2.1) runs in the library's HIP
kernels; this module turns torch tensors into device pointers (checking sizes,
dtypes, contiguity and device on the way, so that a wrong tensor is refused on the
host instead of becoming an out-of-bounds device access) and passes the current
HIP stream.  There is no fallback: if the library has not been built
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
    "sparseloco_plan_layout", "sparseloco_plan_num_tensors",
    "sparseloco_plan_num_params", "sparseloco_plan_kappa", "sparseloco_plan_quant_mode",
    "sparseloco_plan_set_select", "sparseloco_plan_set_radix_counter", "sparseloco_chunk_table", "sparseloco_stream_probe",
    "sparseloco_stream_probe_shaped",
    "sparseloco_tensors_bind", "sparseloco_tensors_release", "sparseloco_messages_bind", "sparseloco_messages_release",
    "sparseloco_compress", "sparseloco_aggregate",
    "sparseloco_outer_update", "sparseloco_aggregate_update", "sparseloco_compress_batch",
    "sparseloco_outer_step_batch",
    "sparseloco_reproject_embedding", "sparseloco_reproject_embedding_noalloc", "sparseloco_subspace_project",
    "sparseloco_subspace_reconstruct", "sparseloco_subspace_kernel_choice", "sparseloco_strerror",
]

SPLC_OP_PROJECT, SPLC_OP_RECONSTRUCT, SPLC_OP_REPROJECT_PASS1, SPLC_OP_REPROJECT_PASS2 = 0, 1, 2, 3
SPLC_MAX_REPLICAS = 1024
SPLC_STREAM_READ, SPLC_STREAM_WRITE, SPLC_STREAM_COPY, SPLC_STREAM_R2W1, SPLC_STREAM_R3W1 = 0, 1, 2, 3, 4

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
        p64 = ctypes.POINTER(i64)
        sig = {
            "sparseloco_plan_create": (i32, [pp, i32, p64, i32, i32, i32, vp]),
            "sparseloco_plan_create_2d": (i32, [pp, i32, p64, p64, i32, i32, i32, vp]),
            "sparseloco_plan_destroy": (None, [vp]),
            "sparseloco_plan_num_chunks": (i64, [vp]),
            "sparseloco_plan_num_params": (i64, [vp]),
            "sparseloco_plan_num_tensors": (i32, [vp]),
            "sparseloco_plan_kappa": (i32, [vp]),
            "sparseloco_plan_quant_mode": (i32, [vp]),
            "sparseloco_plan_layout": (i32, [vp]),
            "sparseloco_plan_set_select": (i32, [vp, i32]),
            "sparseloco_plan_set_radix_counter": (i32, [vp, vp]),
            "sparseloco_stream_probe": (i32, [i32, vp, vp, vp, vp, i64, vp]),
            "sparseloco_stream_probe_shaped": (i32, [i32, vp, vp, vp, vp, i64, i32, i32, i32, vp]),
            "sparseloco_chunk_table": (i64, [i32, p64, p64, i32, vp, i64]),
            "sparseloco_tensors_bind": (i32, [pp, vp, i32, pp, i32, vp]),
            "sparseloco_tensors_release": (None, [vp]),
            "sparseloco_messages_bind": (i32, [pp, vp, i32, pp, pp, vp]),
            "sparseloco_messages_release": (None, [vp]),
            "sparseloco_compress": (i32, [vp, i32, vp, vp, vp, i32, f32, vp, vp, vp]),
            "sparseloco_compress_batch": (i32, [vp, i32, vp, vp, vp, f32, vp, vp]),
            "sparseloco_outer_step_batch": (i32, [vp, i32, vp, vp, vp, f32, f32, vp, vp, i32, vp]),
            "sparseloco_aggregate": (i32, [vp, vp, vp, vp]),
            "sparseloco_outer_update": (i32, [vp, vp, vp, f32, vp]),
            "sparseloco_aggregate_update": (i32, [vp, vp, vp, f32, vp, vp, vp]),
            "sparseloco_reproject_embedding": (i32, [vp, vp, vp, vp, i64, i32, i32, i32, vp]),
            "sparseloco_reproject_embedding_noalloc": (i32, [vp, vp, vp, i64, i32, i32, i32, vp]),
            "sparseloco_subspace_project": (i32, [vp, vp, vp, i32, vp, i32, vp, vp, i64, i32, i32, i32, vp]),
            "sparseloco_subspace_reconstruct": (i32, [vp, vp, vp, i32, vp, i32, vp, vp, i64, i32, i32, i32, vp]),
            "sparseloco_subspace_kernel_choice": (i32, [i32, i64, i32, i32, i32, i32]),
            "sparseloco_strerror": (ctypes.c_char_p, [i32]),
        }
        assert sorted(sig) == sorted(EXPORTS)
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


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


def chunk_table(shapes: Sequence, tiled: bool):
    """The chunk table of a plan over these tensors as a numpy structured array (host only, no GPU)."""
    import numpy as np
    rc_list = [rows_cols(s) for s in shapes]
    n = len(rc_list)
    rows = (ctypes.c_int64 * max(n, 1))(*[r for r, _ in rc_list])
    cols = (ctypes.c_int64 * max(n, 1))(*[c for _, c in rc_list])
    layout = SPLC_LAYOUT_TILE64 if tiled else SPLC_LAYOUT_FLAT
    total = lib().sparseloco_chunk_table(n, rows, cols, layout, None, 0)
    if total < 0:
        raise SparseLoCoError(int(total), "sparseloco_chunk_table")
    dt = np.dtype([("tensor", "<u4"), ("n_c", "<u4"), ("offset", "<u8"), ("stride", "<u4"), ("h", "u1"), ("w", "u1"),
                   ("last_w", "u1"), ("vec", "u1"), ("id", "<u4"), ("strip", "<u4")])
    assert dt.itemsize == 32
    out = np.zeros(int(total), dt)
    got = lib().sparseloco_chunk_table(n, rows, cols, layout, out.ctypes.data_as(ctypes.c_void_p), int(total))
    assert got == total
    return out


def _check_tensor(t, numel: int, dtype, what: str, device: bool = True):
    """Host-side refusal of anything that would turn into an out-of-bounds device access.  device=False leaves
    the device check to a later pass (lists are checked for sizes first, then for where they live)."""
    if numel == 0 and t is None:
        return
    if t is None:
        raise ValueError("%s: missing (the plan expects %d elements)" % (what, numel))
    if not isinstance(t, torch.Tensor):
        raise TypeError("%s: expected a tensor, got %r" % (what, type(t)))
    if t.numel() != numel:
        raise ValueError("%s: %d elements, the plan expects %d" % (what, t.numel(), numel))
    if t.dtype != dtype:
        raise ValueError("%s: dtype %s, expected %s" % (what, t.dtype, dtype))
    if not t.is_contiguous():
        raise ValueError("%s: not contiguous" % what)
    if device and not t.is_cuda:
        raise ValueError("%s: not on a GPU" % what)


class Tensors:
    """A bound list (or R lists) of the plan's tensors: sparseloco_tensors_bind / _release."""

    def __init__(self, plan: "Plan", sets, dtype=torch.float32, stream=None):
        if len(sets) and isinstance(sets[0], torch.Tensor) or (len(sets) and sets[0] is None):
            sets = [sets]
        nt = len(plan.numels)
        for s, tensors in enumerate(sets):
            if len(tensors) != nt:
                raise ValueError("set %d: %d tensors, the plan has %d" % (s, len(tensors), nt))
            for i, t in enumerate(tensors):
                _check_tensor(t, plan.numels[i], dtype, "set %d tensor %d" % (s, i), device=False)
        for s, tensors in enumerate(sets):
            for i, t in enumerate(tensors):
                _check_tensor(t, plan.numels[i], dtype, "set %d tensor %d" % (s, i))
        arr = (ctypes.c_void_p * max(nt * len(sets), 1))()
        for s, tensors in enumerate(sets):
            for i, t in enumerate(tensors):
                arr[s * nt + i] = None if t is None or t.numel() == 0 else t.data_ptr()
        self._h = ctypes.c_void_p()
        self.n_sets = len(sets)
        self.dtype = dtype
        self._keep = [list(t) for t in sets]        # the tensors stay alive as long as the binding
        rc = lib().sparseloco_tensors_bind(ctypes.byref(self._h), plan.handle, len(sets), arr,
                                           SPLC_BF16 if dtype == torch.bfloat16 else SPLC_F32, _stream(stream))
        if rc != SPLC_OK:
            self._h = ctypes.c_void_p()
            raise SparseLoCoError(rc, "sparseloco_tensors_bind")

    @property
    def handle(self):
        return self._h

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().sparseloco_tensors_release(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Messages:
    """Bound message buffers of R replicas: sparseloco_messages_bind / _release."""

    def __init__(self, plan: "Plan", pairs, aux, stream=None):
        if len(pairs) != len(aux):
            raise ValueError("%d pair buffers, %d level/value buffers" % (len(pairs), len(aux)))
        nch = plan.num_chunks
        for device in (False, True):
            for r, (p, a) in enumerate(zip(pairs, aux)):
                _check_tensor(p, nch * plan.kappa, torch.int16, "pairs of replica %d" % r, device)
                _check_tensor(a, nch * (2 if plan.quant else plan.kappa), torch.float32,
                              "levels/values of replica %d" % r, device)
        n = len(pairs)
        pa = (ctypes.c_void_p * max(n, 1))(*[p.data_ptr() for p in pairs])
        aa = (ctypes.c_void_p * max(n, 1))(*[a.data_ptr() for a in aux])
        self._h = ctypes.c_void_p()
        self.n_replicas = n
        self._keep = (list(pairs), list(aux))
        rc = lib().sparseloco_messages_bind(ctypes.byref(self._h), plan.handle, n, pa, aa, _stream(stream))
        if rc != SPLC_OK:
            self._h = ctypes.c_void_p()
            raise SparseLoCoError(rc, "sparseloco_messages_bind")

    @property
    def handle(self):
        return self._h

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().sparseloco_messages_release(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Plan:
    """Chunk table for a list of tensors.

    shapes: per tensor its numel (int) or its shape.  tiled=False: chunks are 4096 consecutive
    elements (sparseloco_plan_create); tiled=True: 64 x 64 tiles of each tensor seen as a
    (rows, cols) matrix (sparseloco_plan_create_2d)."""

    def __init__(self, shapes: Sequence, kappa: int, quant: bool = True, tiled: bool = False, stream=None):
        self._h = ctypes.c_void_p()
        n = len(shapes)
        rc_list = [rows_cols(s) for s in shapes]
        numels = [r * c for r, c in rc_list]
        q = SPLC_QUANT_2BIT if quant else SPLC_QUANT_NONE
        st = _stream(stream)
        if tiled:
            rows = (ctypes.c_int64 * max(n, 1))(*[r for r, _ in rc_list])
            cols = (ctypes.c_int64 * max(n, 1))(*[c for _, c in rc_list])
            rc = lib().sparseloco_plan_create_2d(ctypes.byref(self._h), n, rows, cols, SPLC_CHUNK, int(kappa), q, st)
        else:
            arr = (ctypes.c_int64 * max(n, 1))(*numels)
            rc = lib().sparseloco_plan_create(ctypes.byref(self._h), n, arr, SPLC_CHUNK, int(kappa), q, st)
        if rc != SPLC_OK:
            self._h = ctypes.c_void_p()
            raise SparseLoCoError(rc, "sparseloco_plan_create")
        self.numels = numels
        self.tiled = bool(tiled)
        self.kappa = int(kappa)
        self.quant = bool(quant)
        self._temps = []           # bindings made on the fly by the convenience wrappers below

    def close(self):
        for t in getattr(self, "_temps", []):
            t.close()
        self._temps = []
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

    def set_radix_counter(self, counter: Optional[torch.Tensor]) -> None:
        """Diagnostic: an int32 device tensor of one element that every compress launch adds the number of
        selections on the general radix path to; None switches it off."""
        if counter is not None and (counter.dtype != torch.int32 or counter.numel() != 1 or not counter.is_cuda):
            raise ValueError("counter: one int32 element on the GPU")
        self._counter = counter
        rc = lib().sparseloco_plan_set_radix_counter(self._h, None if counter is None else counter.data_ptr())
        if rc != SPLC_OK:
            raise SparseLoCoError(rc, "sparseloco_plan_set_radix_counter")

    def message_buffers(self, device="cuda"):
        """Freshly allocated (pairs, aux) for one replica's message."""
        nch = self.num_chunks
        pairs = torch.empty(nch * self.kappa, dtype=torch.int16, device=device)
        aux = torch.empty(nch * 2 if self.quant else nch * self.kappa, dtype=torch.float32, device=device)
        return pairs, aux

    def bind(self, sets, dtype=torch.float32, stream=None) -> Tensors:
        """Bind one list of tensors, or a list of per-replica lists (sets)."""
        return Tensors(self, sets, dtype, stream)

    def bind_messages(self, pairs, aux, stream=None) -> Messages:
        return Messages(self, pairs, aux, stream)

    # Convenience for callers that pass plain lists: bound on the fly, released with the plan.
    def _tensors(self, x, dtype=torch.float32, stream=None) -> Optional[Tensors]:
        if x is None or isinstance(x, Tensors):
            return x
        t = Tensors(self, x, dtype, stream)
        self._temps.append(t)
        return t

    def _messages(self, pairs, aux, stream=None) -> Messages:
        if isinstance(pairs, Messages):
            return pairs
        m = Messages(self, pairs, aux, stream)
        self._temps.append(m)
        return m


def _h(x):
    return None if x is None else x.handle


def _opt(t):
    return None if t is None else t.data_ptr()


def sparseloco_compress(plan: Plan, ef, pairs_out: torch.Tensor, aux_out: torch.Tensor, beta: float, *,
                        theta_outer=None, theta_local=None, delta=None, replica: int = 0, stream=None) -> None:
    """Lines 1-4 of the update equations for one replica.  ef / theta_* / delta: Tensors bindings or lists of
    tensors (bound on the fly); replica: which set of multi-set bindings."""
    nch = plan.num_chunks
    _check_tensor(pairs_out, nch * plan.kappa, torch.int16, "pairs_out")
    _check_tensor(aux_out, nch * (2 if plan.quant else plan.kappa), torch.float32, "aux_out")
    if delta is not None:
        dt = delta.dtype if isinstance(delta, Tensors) else next((t.dtype for t in delta if t is not None), torch.float32)
        mode, a, b = SPLC_DELTA_DIRECT, plan._tensors(delta, dt, stream), None
    else:
        mode, a, b = SPLC_DELTA_FROM_PARAMS, plan._tensors(theta_outer, stream=stream), plan._tensors(theta_local, stream=stream)
    e = plan._tensors(ef, stream=stream)
    rc = lib().sparseloco_compress(plan.handle, mode, _h(a), _h(b), _h(e), int(replica), float(beta),
                                   pairs_out.data_ptr(), aux_out.data_ptr(), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_compress")


def sparseloco_aggregate(plan: Plan, messages, delta_bar_out, *, aux=None, stream=None) -> None:
    """Mean over replicas of the decoded messages into dense fp32 tensors.  messages: a Messages binding, or the
    list of pair buffers with aux= the list of level/value buffers."""
    m = plan._messages(messages, aux, stream)
    rc = lib().sparseloco_aggregate(plan.handle, m.handle, _h(plan._tensors(delta_bar_out, stream=stream)),
                                    _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_aggregate")


def sparseloco_outer_update(plan: Plan, theta_outer, delta_bar, outer_lr: float, *, stream=None) -> None:
    """theta_outer -= outer_lr * delta_bar, in place."""
    rc = lib().sparseloco_outer_update(plan.handle, _h(plan._tensors(theta_outer, stream=stream)),
                                       _h(plan._tensors(delta_bar, stream=stream)), float(outer_lr), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_outer_update")


def sparseloco_aggregate_update(plan: Plan, messages, theta_outer, outer_lr: float, *, aux=None, delta_bar_out=None,
                                reset=None, stream=None) -> None:
    """Mean over replicas and outer update in one pass (theta_outer in place); delta_bar_out optional;
    reset: a Tensors binding (or per replica a list of theta_local tensors) that receives the new theta_outer."""
    m = plan._messages(messages, aux, stream)
    rc = lib().sparseloco_aggregate_update(plan.handle, m.handle, _h(plan._tensors(theta_outer, stream=stream)),
                                           float(outer_lr), _h(plan._tensors(delta_bar_out, stream=stream)),
                                           _h(plan._tensors(reset, stream=stream)), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_aggregate_update")


def sparseloco_compress_batch(plan: Plan, theta_outer, theta_local, ef, messages_out, beta: float, *, aux_out=None,
                              n_replicas: Optional[int] = None, stream=None) -> None:
    """Lines 1-4 for R replicas sharing theta_outer, one launch.  theta_local / ef: multi-set bindings or per
    replica a list of tensors; messages_out: a Messages binding, or the pair buffers with aux_out= the others."""
    tl, e = plan._tensors(theta_local, stream=stream), plan._tensors(ef, stream=stream)
    m = plan._messages(messages_out, aux_out, stream)
    n = tl.n_sets if n_replicas is None else int(n_replicas)
    rc = lib().sparseloco_compress_batch(plan.handle, n, _h(plan._tensors(theta_outer, stream=stream)), tl.handle,
                                         e.handle, float(beta), m.handle, _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_compress_batch")


def sparseloco_outer_step_batch(plan: Plan, theta_outer, theta_local, ef, messages_out, beta: float,
                                outer_lr: float, *, aux_out=None, delta_bar_out=None, reset: bool = False,
                                n_replicas: Optional[int] = None, stream=None) -> None:
    """The whole outer step of a single-node simulation in one launch: sparseloco_compress_batch followed by
    sparseloco_aggregate_update over the same replicas, bit for bit.  reset=True also writes the new theta_outer
    into the replicas' theta_local."""
    tl, e = plan._tensors(theta_local, stream=stream), plan._tensors(ef, stream=stream)
    m = plan._messages(messages_out, aux_out, stream)
    n = tl.n_sets if n_replicas is None else int(n_replicas)
    rc = lib().sparseloco_outer_step_batch(plan.handle, n, _h(plan._tensors(theta_outer, stream=stream)), tl.handle,
                                           e.handle, float(beta), float(outer_lr), m.handle,
                                           _h(plan._tensors(delta_bar_out, stream=stream)), 1 if reset else 0,
                                           _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_outer_step_batch")


def sparseloco_stream_probe(pattern: int, a, b, c, sink, *, slots: int = 4, run: int = 0, max_groups_per_unit: int = 0,
                            stream=None) -> None:
    """One launch of a streaming probe (SPLC_STREAM_*) over flat fp32 device tensors of equal length; slots, run and
    max_groups_per_unit vary the launch shape (sparseloco_stream_probe_shaped)."""
    n = next(t.numel() for t in (a, b, c) if t is not None)
    for t in (a, b, c):
        if t is not None and (t.numel() != n or t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda):
            raise ValueError("probe arrays: contiguous fp32 GPU tensors of equal length")
    rc = lib().sparseloco_stream_probe_shaped(int(pattern), _opt(a), _opt(b), _opt(c), _opt(sink), int(n), int(slots),
                                              int(run), int(max_groups_per_unit), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_stream_probe")


def _check_matrices(specs):
    """specs: (tensor, shape, name[, dtype]).  Shapes, dtypes and strides of all first, then where they live."""
    for spec in specs:
        t, shape, what = spec[:3]
        dtype = spec[3] if len(spec) > 3 else torch.float32
        if not isinstance(t, torch.Tensor) or tuple(t.shape) != tuple(shape):
            raise ValueError("%s: expected shape %r, got %r"
                             % (what, tuple(shape), tuple(t.shape) if isinstance(t, torch.Tensor) else None))
        if t.dtype != dtype or not t.is_contiguous():
            raise ValueError("%s: must be a contiguous %s tensor" % (what, dtype))
    for spec in specs:
        if not spec[0].is_cuda:
            raise ValueError("%s: not on a GPU" % spec[2])


def sparseloco_reproject_embedding(t_s: torch.Tensor, t_perp: torch.Tensor, u: torch.Tensor,
                                   coeff_ws: torch.Tensor, *, matmul: int = SPLC_MATMUL_FP32, stream=None) -> None:
    """T_perp += T_S - T_S U U^T; T_S = T_S U U^T (in place).  t_s, t_perp: [vocab, d]; u: [d, k];
    coeff_ws: at least vocab * k floats."""
    if t_s.dim() != 2 or u.dim() != 2:
        raise ValueError("t_s and u must be matrices")
    vocab, d = t_s.shape
    k = u.shape[1]
    if coeff_ws.numel() < vocab * k or coeff_ws.dtype != torch.float32 or not coeff_ws.is_contiguous():
        raise ValueError("coeff_ws: needs %d contiguous fp32 elements" % (vocab * k))
    _check_matrices([(t_s, (vocab, d), "t_s"), (t_perp, (vocab, d), "t_perp"), (u, (d, k), "u"),
                     (coeff_ws, coeff_ws.shape, "coeff_ws")])
    rc = lib().sparseloco_reproject_embedding(t_s.data_ptr(), t_perp.data_ptr(), u.data_ptr(), coeff_ws.data_ptr(),
                                              int(vocab), int(d), int(k), int(matmul), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_reproject_embedding")


def sparseloco_reproject_embedding_noalloc(t_s: torch.Tensor, t_perp: torch.Tensor, u: torch.Tensor, *,
                                           matmul: int = SPLC_MATMUL_FP32, stream=None) -> None:
    """sparseloco_reproject_embedding with the coefficients in the library's fixed per-GPU array (no allocation,
    no caller workspace); vocab * k <= SPLC_NOALLOC_MAX_COEFF."""
    if t_s.dim() != 2 or u.dim() != 2:
        raise ValueError("t_s and u must be matrices")
    vocab, d = t_s.shape
    k = u.shape[1]
    _check_matrices([(t_s, (vocab, d), "t_s"), (t_perp, (vocab, d), "t_perp"), (u, (d, k), "u")])
    rc = lib().sparseloco_reproject_embedding_noalloc(t_s.data_ptr(), t_perp.data_ptr(), u.data_ptr(), int(vocab),
                                                      int(d), int(k), int(matmul), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_reproject_embedding_noalloc")


def subspace_kernel_choice(op: int, rows: int, d: int, k: int, tables: int = 0, matmul: int = SPLC_MATMUL_FP32):
    """(tile_rows, tile_cols) of the kernel variant a matrix call takes for this shape (host logic only)."""
    rc = lib().sparseloco_subspace_kernel_choice(int(op), int(rows), int(d), int(k), int(tables), int(matmul))
    if rc < 0:
        raise SparseLoCoError(rc, "sparseloco_subspace_kernel_choice")
    return rc >> 8, rc & 255


def _check_stage_boundary(rows, d, k, wide, narrow, u, t_perp, token_ids, pos_embed):
    specs = [(wide, (rows, d), "activations"), (narrow, (rows, k), "projected activations"), (u, (d, k), "u")]
    if t_perp is not None:
        if t_perp.dim() != 2:
            raise ValueError("t_perp must be a matrix")
        if token_ids is None:
            raise ValueError("t_perp needs token_ids")
        specs += [(t_perp, (t_perp.shape[0], d), "t_perp"), (token_ids, (rows,), "token_ids", torch.int32)]
    if pos_embed is not None:
        if pos_embed.dim() != 2:
            raise ValueError("pos_embed must be a matrix")
        specs.append((pos_embed, (pos_embed.shape[0], d), "pos_embed"))
    _check_matrices(specs)


def sparseloco_subspace_project(x: torch.Tensor, u: torch.Tensor, out: torch.Tensor, *, t_perp=None, token_ids=None,
                                pos_embed=None, matmul: int = SPLC_MATMUL_FP32, stream=None) -> None:
    """out[rows, k] = (x - t_perp[token_ids] - pos_embed[row % seq_len]) @ u;  x: [rows, d], u: [d, k]."""
    if x.dim() != 2 or u.dim() != 2:
        raise ValueError("x and u must be matrices")
    rows, d = x.shape
    k = u.shape[1]
    _check_stage_boundary(rows, d, k, x, out, u, t_perp, token_ids, pos_embed)
    rc = lib().sparseloco_subspace_project(x.data_ptr(), _opt(t_perp), _opt(token_ids),
                                           0 if t_perp is None else t_perp.shape[0], _opt(pos_embed),
                                           0 if pos_embed is None else pos_embed.shape[0], u.data_ptr(),
                                           out.data_ptr(), int(rows), int(d), int(k), int(matmul), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_subspace_project")


def sparseloco_subspace_reconstruct(x_tilde: torch.Tensor, u: torch.Tensor, out: torch.Tensor, *, t_perp=None,
                                    token_ids=None, pos_embed=None, matmul: int = SPLC_MATMUL_FP32,
                                    stream=None) -> None:
    """out[rows, d] = x_tilde @ u.T + t_perp[token_ids] + pos_embed[row % seq_len]."""
    if x_tilde.dim() != 2 or u.dim() != 2:
        raise ValueError("x_tilde and u must be matrices")
    rows, k = x_tilde.shape
    d = u.shape[0]
    _check_stage_boundary(rows, d, k, out, x_tilde, u, t_perp, token_ids, pos_embed)
    rc = lib().sparseloco_subspace_reconstruct(x_tilde.data_ptr(), _opt(t_perp), _opt(token_ids),
                                               0 if t_perp is None else t_perp.shape[0], _opt(pos_embed),
                                               0 if pos_embed is None else pos_embed.shape[0], u.data_ptr(),
                                               out.data_ptr(), int(rows), int(d), int(k), int(matmul), _stream(stream))
    if rc != SPLC_OK:
        raise SparseLoCoError(rc, "sparseloco_subspace_reconstruct")
