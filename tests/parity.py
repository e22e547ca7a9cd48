"""Shared driver of the GPU parity tests: run the same host inputs through the
C-ABI library (via the thin binding) and through the CPU oracle, and compare.

Bars: selected indices, codes, pairs and the per-chunk levels (or sent values)
bit-exact; error-feedback buffer, mean and updated parameters within
1e-6 relative / 1e-7 absolute in fp32 (in practice they differ at most in the
sign of a zero, which the strict check below also asserts).
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

import oracle
from paper_2601_02360_amd import binding as B

RTOL, ATOL = 1e-6, 1e-7


def to_np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.int16:
        return t.numpy().view(np.uint16)
    return t.numpy()


def assert_close_fp32(got: np.ndarray, want: np.ndarray, what: str):
    got, want = got.reshape(-1), want.reshape(-1)
    assert got.shape == want.shape, what
    assert np.allclose(got, want, rtol=RTOL, atol=ATOL), what
    # stronger than the stated tolerance: equal as numbers (only the sign of a zero may differ)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, "%s: %d values differ, first at %d: %r vs %r" % (
        what, bad.size, bad[0], got[bad[0]], want[bad[0]])


class HostCase:
    """Inputs on the host: theta_outer[t]; per replica theta_local[r][t] (fp32) or
    delta[r][t] (fp32, or uint16 holding bf16 bits); ef[r][t]."""

    def __init__(self, theta_outer, ef, theta_local=None, delta=None, shapes=None):
        # shapes: per tensor (rows, cols) etc. for the tiled layout; None = flat chunks
        self.shapes = None if shapes is None else [tuple(s) for s in shapes]
        self.theta_outer = [np.ascontiguousarray(x, np.float32).reshape(-1) for x in theta_outer]
        self.ef = [[np.ascontiguousarray(x, np.float32).reshape(-1) for x in r] for r in ef]
        self.theta_local = None if theta_local is None else \
            [[np.ascontiguousarray(x, np.float32).reshape(-1) for x in r] for r in theta_local]
        self.delta = None if delta is None else [[np.ascontiguousarray(x).reshape(-1) for x in r] for r in delta]
        self.numels = [int(x.size) for x in self.theta_outer]
        self.R = len(self.ef)


def run_oracle(case: HostCase, kappa, beta, lr, quant=True, outer_steps=1, deltas_per_step=None):
    geo = dict(shapes=case.shapes, tile=64) if case.shapes is not None else {}
    shapes = case.shapes if case.shapes is not None else case.numels
    th = [x.copy() for x in case.theta_outer]
    ef = [[x.copy() for x in r] for r in case.ef]
    out = []
    for step in range(outer_steps):
        pairs, aux = [], []
        for r in range(case.R):
            if case.delta is not None:
                d = case.delta[r] if deltas_per_step is None else deltas_per_step[step][r]
                p, a = oracle.compress(ef[r], kappa, beta, delta=d, quant=quant, **geo)
            else:
                p, a = oracle.compress(ef[r], kappa, beta, theta_outer=th, theta_local=case.theta_local[r],
                                       quant=quant, **geo)
            pairs.append(p), aux.append(a)
        dbar = oracle.aggregate(shapes, pairs, aux, kappa, quant=quant,
                                tile=64 if case.shapes is not None else None)
        oracle.outer_update(th, dbar, lr)
        out.append(dict(pairs=pairs, aux=aux, ef=[[x.copy() for x in r] for r in ef], dbar=dbar,
                        theta=[x.copy() for x in th]))
    return out


def _dev(x: np.ndarray, bf16: bool = False) -> torch.Tensor:
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(x.copy()).cuda()


def run_gpu(case: HostCase, kappa, beta, lr, quant=True, select=B.SPLC_SELECT_AUTO, outer_steps=1,
            deltas_per_step=None, stream: Optional[torch.cuda.Stream] = None, fused=None, batch=False):
    """fused: None = aggregate then outer_update; "with_mean" / "no_mean" = sparseloco_aggregate_update
    with / without the dense mean output (without it, the returned mean is recomputed by a separate
    sparseloco_aggregate call, which the fused call must agree with anyway).
    batch: False = one compress launch per replica; True = sparseloco_compress_batch; "step" = the whole outer
    step in one launch (sparseloco_outer_step_batch; its mean output follows `fused` as above)."""
    ctx = torch.cuda.stream(stream) if stream is not None else torch.cuda.stream(torch.cuda.current_stream())
    out = []
    with ctx:
        plan = B.Plan(case.shapes if case.shapes is not None else case.numels, kappa, quant,
                      tiled=case.shapes is not None)
        plan.set_select(select)
        th = [_dev(x) for x in case.theta_outer]
        ef = [[_dev(x) for x in r] for r in case.ef]
        tl = None if case.theta_local is None else [[_dev(x) for x in r] for r in case.theta_local]
        b_th, b_ef = plan.bind(th), plan.bind(ef)
        b_tl = None if tl is None else plan.bind(tl)
        for step in range(outer_steps):
            msgs = [plan.message_buffers() for _ in range(case.R)]
            for p, a in msgs:                       # poison: the library must overwrite everything
                p.fill_(0x5A5A)
                a.fill_(float("nan"))
            b_msgs = plan.bind_messages([m[0] for m in msgs], [m[1] for m in msgs])
            dbar = [torch.full((n,), float("nan"), device="cuda") for n in case.numels]
            b_dbar = plan.bind(dbar)
            if batch == "step":                     # the whole step in one launch
                B.sparseloco_outer_step_batch(plan, b_th, b_tl, b_ef, b_msgs, beta, lr,
                                              delta_bar_out=b_dbar if fused == "with_mean" else None)
            elif batch:
                B.sparseloco_compress_batch(plan, b_th, b_tl, b_ef, b_msgs, beta)
            for r in range(case.R if not batch else 0):
                p, a = msgs[r]
                if case.delta is not None:
                    src = case.delta[r] if deltas_per_step is None else deltas_per_step[step][r]
                    d = [_dev(x) for x in src]
                    B.sparseloco_compress(plan, b_ef, p, a, beta, delta=d, replica=r)
                else:
                    B.sparseloco_compress(plan, b_ef, p, a, beta, theta_outer=b_th, theta_local=b_tl, replica=r)
            if batch == "step":
                if fused != "with_mean":
                    B.sparseloco_aggregate(plan, b_msgs, b_dbar)
            elif fused is None:
                B.sparseloco_aggregate(plan, b_msgs, b_dbar)
                B.sparseloco_outer_update(plan, b_th, b_dbar, lr)
            elif fused == "with_mean":
                B.sparseloco_aggregate_update(plan, b_msgs, b_th, lr, delta_bar_out=b_dbar)
            else:
                B.sparseloco_aggregate_update(plan, b_msgs, b_th, lr)
                B.sparseloco_aggregate(plan, b_msgs, b_dbar)
            torch.cuda.synchronize()
            out.append(dict(pairs=[to_np(m[0]) for m in msgs], aux=[to_np(m[1]) for m in msgs],
                            ef=[[to_np(x) for x in r] for r in ef], dbar=[to_np(x) for x in dbar],
                            theta=[to_np(x) for x in th]))
            b_msgs.close(), b_dbar.close()
        for b in (b_th, b_ef, b_tl):
            if b is not None:
                b.close()
        plan.close()
    return out


def compare(got, want, what=""):
    assert len(got) == len(want)
    for step, (g, w) in enumerate(zip(got, want)):
        tag = "%s step %d" % (what, step)
        for r, (a, b) in enumerate(zip(g["pairs"], w["pairs"])):
            bad = np.nonzero(a != b)[0]
            assert bad.size == 0, "%s replica %d: %d pairs differ, first at slot %d: %#x vs %#x" % (
                tag, r, bad.size, bad[0], a[bad[0]], b[bad[0]])
        for r, (a, b) in enumerate(zip(g["aux"], w["aux"])):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), "%s replica %d: levels/values differ" % (tag, r)
        for r in range(len(w["ef"])):
            for t in range(len(w["ef"][r])):
                assert_close_fp32(g["ef"][r][t], w["ef"][r][t], "%s ef[%d][%d]" % (tag, r, t))
        for t in range(len(w["dbar"])):
            assert_close_fp32(g["dbar"][t], w["dbar"][t], "%s delta_bar[%d]" % (tag, t))
            assert_close_fp32(g["theta"][t], w["theta"][t], "%s theta[%d]" % (tag, t))


def check(case: HostCase, kappa, beta=0.95, lr=1.0, quant=True, select=B.SPLC_SELECT_AUTO, outer_steps=1,
          deltas_per_step=None, what="", fused=None, batch=False):
    want = run_oracle(case, kappa, beta, lr, quant, outer_steps, deltas_per_step)
    got = run_gpu(case, kappa, beta, lr, quant, select, outer_steps, deltas_per_step, fused=fused, batch=batch)
    compare(got, want, what)
    return got, want
