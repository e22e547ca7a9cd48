"""Seeded synthetic inputs shaped like the paper's models (appendix: LLaMA-style
decoder-only transformers with SwiGLU, 178M-1B parameters; SparseLoCo with
chunk 4096, Top-32 per chunk, beta 0.95, M = 8 replicas).

This module only DRAWS inputs -- parameter tensors, per-replica local
parameters or pseudo-gradients, error-feedback buffers.  It holds none of the
method's arithmetic and is used by the tests, the benchmark and the smoke check
to feed the same bits to the GPU library and to the CPU oracle.  The trained
weights and corpora of the paper are not needed: the cost of the outer step
does not depend on the values except through ties and zeros, which workload 4
stresses on purpose.

Workloads (index = position in the benchmark's config list):
  0  one 2048x2048 tensor, kappa 32, R 4
  1  ~150M set: d 768, 12 layers, FFN 3072, vocabulary 50304; kappa 32, R 8
  2  ~0.9B set: d 2048, 16 layers, FFN 5632, vocabulary 32000; heavy-tailed
     pseudo-gradients (Student-t, 3 degrees of freedom); kappa 64, R 8
  3  shapes of 2; replicas share most of their pseudo-gradient (index
     collisions in the aggregation); kappa in {16, 32, 64, 128}, R 16
  4  shapes not multiples of 64, bf16 pseudo-gradients given directly, half of
     them exact zeros, many ties; kappa 32, R 32
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import torch

WORKLOADS: Dict[int, dict] = {
    0: dict(name="single-2048x2048", kappa=32, replicas=4, beta=0.95, outer_lr=1.0, direct_bf16=False),
    1: dict(name="llama-150M", kappa=32, replicas=8, beta=0.95, outer_lr=1.0, direct_bf16=False),
    2: dict(name="llama-0.9B", kappa=64, replicas=8, beta=0.95, outer_lr=1.0, direct_bf16=False),
    3: dict(name="llama-0.9B-correlated", kappa=64, replicas=16, beta=0.95, outer_lr=1.0, direct_bf16=False,
            kappa_sweep=(16, 32, 64, 128)),
    4: dict(name="llama-0.9B-ragged-bf16", kappa=32, replicas=32, beta=0.95, outer_lr=1.0, direct_bf16=True),
}


def _llama(d: int, layers: int, ffn: int, vocab: int, emb_cols: Optional[int] = None,
           gain: Optional[int] = None) -> List[Tuple[int, ...]]:
    gain = d if gain is None else gain
    shapes: List[Tuple[int, ...]] = []
    for _ in range(layers):
        shapes += [(d, d)] * 4                      # Wq Wk Wv Wo
        shapes += [(d, ffn), (d, ffn), (ffn, d)]    # SwiGLU W1 W3 W2
        shapes += [(gain,), (gain,)]                # two RMSNorm gains
    shapes.append((vocab, emb_cols or d))           # tied embedding
    shapes.append((gain,))                          # final norm
    return shapes


def tensor_shapes(workload: int) -> List[Tuple[int, ...]]:
    if workload == 0:
        return [(2048, 2048)]
    if workload == 1:
        return _llama(768, 12, 3072, 50304)
    if workload in (2, 3):
        return _llama(2048, 16, 5632, 32000)
    if workload == 4:
        return _llama(2050, 16, 5630, 32001, emb_cols=2048, gain=2047)
    raise ValueError("unknown workload %r" % (workload,))


def numels(workload: int) -> List[int]:
    return [math.prod(s) for s in tensor_shapes(workload)]


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _seed(workload: int, tensor: int, replica: int) -> int:
    """Per-replica draws use replica = 0..R-1; draws shared by all replicas use 999."""
    return 1_000_000 * workload + 1000 * tensor + replica


def _randn(n: int, std: float, device, seed: int) -> torch.Tensor:
    return torch.randn(n, generator=_gen(device, seed), device=device, dtype=torch.float32) * std


def theta_outer(workload: int, tensor: int, device="cpu") -> torch.Tensor:
    n = numels(workload)[tensor]
    return _randn(n, 0.02, device, _seed(workload, tensor, 999))


def replica_inputs(workload: int, tensor: int, replica: int, theta_o: torch.Tensor, device="cpu", *,
                   outer_step: int = 0):
    """Returns (theta_local or None, delta or None, ef) for one tensor of one replica, flat.

    Workloads 0-3 give theta_local = fl(theta_outer - delta); workload 4 gives the
    pseudo-gradient directly in bfloat16.  `ef` is the buffer before the first
    outer step; for outer_step > 0 only a fresh pseudo-gradient is drawn (the
    caller carries its own buffer) and ef is None.
    """
    shape = tensor_shapes(workload)[tensor]
    n = math.prod(shape)
    seed = _seed(workload, tensor, replica) + 500 * outer_step
    g = _gen(device, seed)
    rn = lambda: torch.randn(n, generator=g, device=device, dtype=torch.float32)
    ef = None
    if workload == 0:
        delta = rn() * 1e-3
        ef = rn() * 1e-4
    elif workload == 1:
        fan_in = shape[1] if len(shape) == 2 else 1
        delta = rn() * (1e-3 / math.sqrt(fan_in))
        ef = rn() * 1e-4
    elif workload == 2:
        z = rn()
        chi2 = rn() ** 2 + rn() ** 2 + rn() ** 2
        delta = z / torch.sqrt(chi2 / 3.0) * 1e-3
        del z, chi2
        ef = rn() * 1e-4
    elif workload == 3:
        shared = _randn(n, 1e-3, device, _seed(workload, tensor, 999) + 1 + 500 * outer_step)
        delta = shared + rn() * 3e-4
        ef = rn() * 1e-4
    elif workload == 4:
        delta = (rn() * 1e-3).to(torch.bfloat16)
        keep = torch.rand(n, generator=g, device=device) < 0.5
        delta = torch.where(keep, delta, torch.zeros_like(delta))
        ef = torch.zeros(n, device=device, dtype=torch.float32)
        return None, delta, (ef if outer_step == 0 else None)
    else:
        raise ValueError("unknown workload %r" % (workload,))
    theta_l = theta_o - delta
    return theta_l, None, (ef if outer_step == 0 else None)


def orthonormal_basis(d: int, k: int, seed: int, device="cpu") -> torch.Tensor:
    """A seeded random d x k fp32 matrix with orthonormal columns (the fixed random basis U of section 2.2):
    Gaussian draw, QR in float64 on the host, signs fixed so that the result is reproducible."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    q, r = torch.linalg.qr(torch.randn(d, k, generator=g, dtype=torch.float64))
    q = q * torch.sign(torch.diagonal(r))[None, :]
    return q.to(torch.float32).contiguous().to(device)


class ReplicaSet:
    """All inputs of a workload resident on one device: theta_outer, and per
    replica theta_local (or bf16 delta) and the error-feedback buffer."""

    def __init__(self, workload: int, device="cuda", replicas: Optional[int] = None,
                 tensors: Optional[Sequence[int]] = None):
        cfg = WORKLOADS[workload]
        self.workload = workload
        self.cfg = cfg
        self.R = cfg["replicas"] if replicas is None else replicas
        self.tensor_ids = list(range(len(tensor_shapes(workload)))) if tensors is None else list(tensors)
        all_n = numels(workload)
        self.numels = [all_n[t] for t in self.tensor_ids]
        self.theta_outer = [theta_outer(workload, t, device) for t in self.tensor_ids]
        self.theta_local: List[List[torch.Tensor]] = []
        self.delta: List[List[torch.Tensor]] = []
        self.ef: List[List[torch.Tensor]] = []
        for r in range(self.R):
            tl, dl, ef = [], [], []
            for i, t in enumerate(self.tensor_ids):
                a, b, e = replica_inputs(workload, t, r, self.theta_outer[i], device)
                tl.append(a), dl.append(b), ef.append(e)
            self.theta_local.append(tl), self.delta.append(dl), self.ef.append(ef)
        self.direct = cfg["direct_bf16"]

    @property
    def num_params(self) -> int:
        return sum(self.numels)
