"""moe_expert_dense.py -- TEST INFRASTRUCTURE ONLY.

One expert of the layer on the rows routed to it, forward and backward, as dense fp64 matrix expressions with
numpy's matmul as the only library step (FastMoE paper, Section 5.1: the expert is two linear layers d_m x d_h and
d_h x d_m; Section 4: an expert processes its samples as one batch; Algorithm 1: its output enters y with the
score as weight).  The activation is the erf GeLU (scipy's erf), as in moe_oracle.c.

It states for a whole segment what the per-token loop of moe_oracle.c states row by row, so that the weight
gradients of an expert with ten thousand rows can be checked at full size in seconds instead of minutes.  It shares
nothing with the HIP library and is used by tests only.

Pins (tests/test_oracle_pins.py): equality with the per-token oracle, an independent implementation in C, for every
returned tensor on seeded problems with and without biases; the full-size GPU test repeats that comparison on one
expert of the large workload at its real shape.
"""
import numpy as np
from scipy.special import erf


def _gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def _gelu_grad(z):
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def expert_segment(Xe, W1e, W2e, we=None, dYe=None, b1e=None, b2e=None):
    """Xe [m,d]: the inputs of the m assignments of one expert; W1e [d,h], W2e [h,d]; optional biases b1e [h], b2e [d].
    we [m]: the scores of those assignments, dYe [m,d]: dL/dy of their tokens (both None: forward only).
    Returns dict(Z, H, O) and, with gradients, dO = we * dYe, dZ, dXs = dZ W1e^T, dW1 = Xe^T dZ, dW2 = H^T dO,
    db1 = column sums of dZ, db2 = column sums of dO."""
    Xe = np.asarray(Xe, np.float64)
    Z = Xe @ W1e
    if b1e is not None:
        Z = Z + b1e
    H = _gelu(Z)
    O = H @ W2e
    if b2e is not None:
        O = O + b2e
    out = dict(Z=Z, H=H, O=O)
    if dYe is not None:
        dO = np.asarray(we, np.float64)[:, None] * np.asarray(dYe, np.float64)
        dZ = (dO @ W2e.T) * _gelu_grad(Z)
        out.update(dO=dO, dZ=dZ, dXs=dZ @ W1e.T, dW1=Xe.T @ dZ, dW2=H.T @ dO, db1=dZ.sum(0), db2=dO.sum(0))
    return out
