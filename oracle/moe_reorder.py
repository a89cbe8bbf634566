"""moe_reorder.py -- TEST INFRASTRUCTURE ONLY.

Plain fp64 numpy statements of the two data-movement steps of the layer taken on their own
(FastMoE paper, Section 4: the samples are "scattered" into per-expert contiguous buffers before
the experts run and "gathered" back afterwards; Algorithm 1: the outputs of the chosen experts are
summed with their scores; Section 2.1: the gate is trained through that score), and of their
gradients with the top-k indices held constant.

Every function is the definition written out with one row per assignment a = t*k + j; there is no
blocking or reordering.  They share nothing with the HIP library and are used by tests only.

Pins (tests/test_oracle_pins.py): scatter then gather with weights that sum to one returns X; the
composition scatter -> per-expert FFN (numpy) -> gather and its gradients reproduce the per-token
oracle of moe_oracle.c, an independent implementation; gradients against central finite differences.
"""
import numpy as np


def scatter(X, pos, k):
    """Xs[pos[a], :] = X[a // k, :]"""
    X = np.asarray(X, np.float64)
    M = pos.size
    Xs = np.empty((M, X.shape[1]))
    for a in range(M):
        Xs[pos[a]] = X[a // k]
    return Xs


def gather(Ys, w, pos):
    """Y[t, :] = sum_j w[t, j] * Ys[pos[t*k + j], :]   (j ascending)"""
    Ys = np.asarray(Ys, np.float64)
    N, k = w.shape
    Y = np.zeros((N, Ys.shape[1]))
    for t in range(N):
        for j in range(k):
            Y[t] += w[t, j] * Ys[pos[t * k + j]]
    return Y


def gather_backward(dY, Ys, w, pos):
    """dYs[pos[a], :] = w[a] * dY[t, :];  dw[t, j] = <dY[t], Ys[pos[t*k+j]]>;
    dl[t, j] = w[t, j] * (dw[t, j] - sum_i w[t, i] * dw[t, i])  (softmax over the k selected logits)."""
    dY = np.asarray(dY, np.float64)
    Ys = np.asarray(Ys, np.float64)
    N, k = w.shape
    dYs = np.empty_like(Ys)
    dl = np.empty((N, k))
    for t in range(N):
        dw = np.empty(k)
        for j in range(k):
            r = pos[t * k + j]
            dYs[r] = w[t, j] * dY[t]
            dw[j] = float(np.dot(dY[t], Ys[r]))
        s = float(np.dot(w[t], dw))
        dl[t] = w[t] * (dw - s)
    return dYs, dl


def scatter_backward(Wg, Xs, dXs, dl, idx, pos):
    """dX[t] = sum_j dXs[pos[t*k+j]] + sum_j dl[t, j] * Wg[:, idx[t, j]];
    dWg[:, e] = sum over assignments of e of dl * x;  dbg[e] = sum of dl  (x = Xs[pos[a]] = X[t])."""
    Wg = np.asarray(Wg, np.float64)
    Xs = np.asarray(Xs, np.float64)
    dXs = np.asarray(dXs, np.float64)
    N, k = idx.shape
    d, E = Wg.shape
    dX = np.zeros((N, d))
    dWg = np.zeros((d, E))
    dbg = np.zeros(E)
    for t in range(N):
        for j in range(k):
            r = pos[t * k + j]
            e = idx[t, j]
            dX[t] += dXs[r] + dl[t, j] * Wg[:, e]
            dWg[:, e] += dl[t, j] * Xs[r]
            dbg[e] += dl[t, j]
    return dX, dWg, dbg
