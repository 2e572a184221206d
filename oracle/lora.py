"""fp64 oracle: the decoder layer with low-rank adapters on its projection matrices.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper trains its largest model with rank-32 low-rank adapters and computes
only the adapter gradients (App. D, experiment setup).  An adapted matrix acts as
    y = x W^T + s (x A^T) B^T = x (W + s B A)^T,      A [r, in], B [out, r],
with W frozen.  StreamBP is exact for any parameterisation (Sec. 3.1), so the
oracle is again the plain definition: the ordinary full-sequence layer of
oracle/layer.py evaluated at the effective matrices W + s B A, and the chain rule
through the product B A:
    dA = s B^T dW_eff,      dB = s dW_eff A^T,
where dW_eff is the ordinary weight gradient at the effective matrix.  The
gradient wrt the layer input is the ordinary one at the effective matrices.
"""
from __future__ import annotations

import numpy as np

from . import layer

F64 = np.float64
MATRICES = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def effective_weights(w, adapters, scale):
    """w: dict of base weights; adapters: dict name -> (A [r, in], B [out, r]) for the adapted matrices."""
    out = {k: np.asarray(v, F64) for k, v in w.items()}
    for name, (A, B) in adapters.items():
        assert name in MATRICES
        out[name] = out[name] + scale * (np.asarray(B, F64) @ np.asarray(A, F64))
    return out


def layer_forward_backward(x, w, adapters, scale, cfg, dy, first_valid=None):
    """Returns (y, dx, dA, dB): dA / dB dicts over the adapted matrices, summed over the batch."""
    w_eff = effective_weights(w, adapters, scale)
    y, dx, g = layer.layer_forward_backward(x, w_eff, cfg, dy, first_valid)
    dA = {n: scale * (np.asarray(B, F64).T @ g[n]) for n, (A, B) in adapters.items()}
    dB = {n: scale * (g[n] @ np.asarray(A, F64).T) for n, (A, B) in adapters.items()}
    return y, dx, dA, dB
