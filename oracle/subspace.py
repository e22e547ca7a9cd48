"""CPU oracle of the post-synchronisation token-embedding re-projection
(paper section 2.4) -- TEST INFRASTRUCTURE, same rules as the rest of oracle/.

After every SparseLoCo outer synchronisation the embedding component T_S is
projected back onto the compression subspace S = Col(U), and what the
projection removes is accumulated into T_perp, so that TE = T_S + T_perp is
unchanged:

    T_perp <- T_perp + (T_S - Pi_S(T_S))
    T_S    <- Pi_S(T_S),          Pi_S(X) = X U U^T   (U: d x k, orthonormal columns)

The same operation with T_perp = 0 is the initialisation before training
(T_S <- TE U U^T, T_perp <- TE - T_S).

Plain numpy in float64, the definition written out; the GPU path computes in
fp32 and is compared within a tolerance derived from the arithmetic.
"""
from __future__ import annotations

import numpy as np


def orthonormal_basis(d: int, k: int, seed: int) -> np.ndarray:
    """A random d x k matrix orthonormalised by QR (section 2.2), float64."""
    rng = np.random.default_rng(seed)
    q, r = np.linalg.qr(rng.standard_normal((d, k)))
    return q * np.sign(np.diag(r))            # fix the sign convention so the basis is reproducible


def reproject(t_s: np.ndarray, t_perp: np.ndarray, u: np.ndarray):
    """Returns (new T_S, new T_perp) in float64; inputs are not modified."""
    t_s = np.asarray(t_s, np.float64)
    t_perp = np.asarray(t_perp, np.float64)
    u = np.asarray(u, np.float64)
    coeff = t_s @ u                            # coordinates in the subspace, vocab x k
    proj = coeff @ u.T                         # Pi_S(T_S), vocab x d
    return proj, t_perp + (t_s - proj)


def _high_rank(rows, d, t_perp, token_ids, pos_embed):
    """T_perp[x] + PosEmbed of every row of a [batch, seq_len, d] activation tensor (section 2.2)."""
    h = np.zeros((rows, d), np.float64)
    if t_perp is not None:
        h += np.asarray(t_perp, np.float64)[np.asarray(token_ids)]
    if pos_embed is not None:
        pos_embed = np.asarray(pos_embed, np.float64)
        h += pos_embed[np.arange(rows) % pos_embed.shape[0]]
    return h


def project(x, u, t_perp=None, token_ids=None, pos_embed=None):
    """What a stage transmits: x_tilde = (x - T_perp[x] - PosEmbed) U, float64.  With no tables this is the
    product applied to activation gradients in the backward pass."""
    x = np.asarray(x, np.float64)
    return (x - _high_rank(x.shape[0], x.shape[1], t_perp, token_ids, pos_embed)) @ np.asarray(u, np.float64)


def reconstruct(x_tilde, u, t_perp=None, token_ids=None, pos_embed=None):
    """What the next stage rebuilds: x_hat = x_tilde U^T + T_perp[x] + PosEmbed, float64."""
    u = np.asarray(u, np.float64)
    x_tilde = np.asarray(x_tilde, np.float64)
    return x_tilde @ u.T + _high_rank(x_tilde.shape[0], u.shape[0], t_perp, token_ids, pos_embed)
