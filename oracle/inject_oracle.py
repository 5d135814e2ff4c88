"""fp64 CPU oracle for the gated injection of target features into the draft's input
embeddings (Sec.3.3, "Stochastic Gating for Target Features").

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library and is never imported by it.

  t      = Proj([x_1; ...; x_F])      the target model's hidden states of F layers (the paper
                                      names three, low / middle / high, and trains with four),
                                      concatenated along the feature axis and projected to the
                                      draft's width
  e'     = e + xi * t                 xi ~ Bernoulli(1 - rho), drawn per training instance

Readings (the paper calls Proj "a lightweight projection module" and says no more; parity
unpinned by the paper): Proj is one linear map without bias, t = [x_1; ...; x_F] . P^T with
P[d, F*dt]; the gate is an input, one value per token row (the caller repeats an instance's
draw over its rows), and any real value is accepted, not only 0 and 1.  The target model is
frozen, so the backward produces the gradient of the draft embeddings (the identity), of the
projected feature, dt_feat = xi * de', and of the projection, dP = dt_feat^T . [x_1; ...; x_F].
"""
from __future__ import annotations

import numpy as np


def inject_forward(E, feats, P, xi):
    """e'[T, d] = E + xi[:, None] * (concat(feats, axis=1) @ P^T), float64."""
    X = np.concatenate([np.asarray(f, dtype=np.float64) for f in feats], axis=1)
    t = X @ np.asarray(P, dtype=np.float64).T
    return np.asarray(E, dtype=np.float64) + np.asarray(xi, dtype=np.float64)[:, None] * t


def inject_backward(dEout, feats, xi):
    """Returns (dT[T, d], dP[d, F*dt]) for upstream gradient dEout[T, d]; dE equals dEout."""
    X = np.concatenate([np.asarray(f, dtype=np.float64) for f in feats], axis=1)
    dT = np.asarray(xi, dtype=np.float64)[:, None] * np.asarray(dEout, dtype=np.float64)
    return dT, dT.T @ X
