"""What rounding the stored tensors to bfloat16 costs by itself -- CPU only, numpy fp64.

`ideal_bf16_layer` runs the layer the way any bf16 implementation has to: every tensor the method keeps in memory
between two steps (Z, H, Ys, Y, dYs, dZ, dXs, dX and the weight gradients) is computed EXACTLY, in fp64 with exact
sums, from the bf16 values of the tensors before it, and then rounded to bf16 once (round to nearest even).  Nothing
else is approximated: no fp32 accumulation, no table, no reordering.  Its distance from the fp64 oracle is therefore
a floor for the error of every path that stores these tensors in bf16, whatever its kernels look like; the parity
tests use it to tell which error metric the stated bound of 2e-2 can be held to for which tensor.

It follows the routing of the oracle (indices and weights are taken from it) and is test support, not an oracle:
no expected value of a parity test comes from here.
"""
import numpy as np
from scipy.special import erf

import oracle as orc
from paper_2103_13262_amd.synth import f32_to_bf16_bits


def rb(a):
    """fp64 -> nearest bfloat16 (ties to even, via fp32: exact for values that fp32 holds to 24 bits first) -> fp64."""
    return orc.bf16_bits_to_f64(f32_to_bf16_bits(np.asarray(a, np.float64).astype(np.float32)))


def gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def strict_err(got, ref, rms=None):
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref)): elementwise relative error with the tensor's RMS as floor."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    if rms is None:
        rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return 0.0 if not np.any(got) else float("inf")
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))


def ideal_bf16_layer(w, inputs, idx, wt, score_all_logits=None):
    """Returns the bf16-stored tensors of the ideal path as fp64 arrays, by assignment a = t*k + j where a tensor has
    one row per assignment: Z, H [M,h]; Ys, dYs, dXs [M,d]; Y, dX [N,d]; dl [N,k]; dW1 [E,d,h]; dW2 [E,h,d];
    dWg [d,E]; dbg [E].  idx [N,k], wt [N,k]: the oracle's routing.  score_all_logits: the oracle's logits [N,E]
    when the scores are the softmax over all experts (then the experts outside the selection receive gradient)."""
    wide = orc.bf16_bits_to_f64
    X, Wg, W1, W2, dY = (wide(inputs[n]) for n in ("X", "Wg", "W1", "W2", "dY"))
    b1 = wide(inputs["b1"]) if "b1" in inputs else None
    b2 = wide(inputs["b2"]) if "b2" in inputs else None
    N, k, E, M = w.N, w.k, w.E, w.M
    e_of = idx.reshape(-1)
    Xa = np.repeat(X, k, axis=0)                       # the scatter is a copy: exact
    wa = wt.reshape(-1, 1)
    Z, H, Ys = np.zeros((M, w.h)), np.zeros((M, w.h)), np.zeros((M, w.d))
    for e in range(E):
        m = e_of == e
        z = Xa[m] @ W1[e] + (b1[e] if b1 is not None else 0.0)
        Z[m], H[m] = rb(z), rb(gelu(z))
        Ys[m] = rb(H[m] @ W2[e] + (b2[e] if b2 is not None else 0.0))
    Y = rb((wa * Ys).reshape(N, k, -1).sum(1))
    dYa = np.repeat(dY, k, axis=0)
    dYs = rb(wa * dYa)
    dw = np.einsum("ad,ad->a", dYa, Ys).reshape(N, k)
    S = (wt * dw).sum(1, keepdims=True)
    dl = wt * (dw - S)
    dZ, dXs = np.zeros((M, w.h)), np.zeros((M, w.d))
    dW1, dW2 = np.zeros((E, w.d, w.h)), np.zeros((E, w.h, w.d))
    for e in range(E):
        m = e_of == e
        dZ[m] = rb((dYs[m] @ W2[e].T) * gelu_grad(Z[m]))     # the saved pre-activation is the bf16 one
        dW2[e] = rb(H[m].T @ dYs[m])
        dXs[m] = rb(dZ[m] @ W1[e].T)
        dW1[e] = rb(Xa[m].T @ dZ[m])
    dLfull = np.zeros((N, E))
    np.put_along_axis(dLfull, idx, dl, axis=1)
    if score_all_logits is not None:
        p = np.exp(score_all_logits - score_all_logits.max(1, keepdims=True))
        p /= p.sum(1, keepdims=True)
        dense = -p * S
        np.put_along_axis(dense, idx, 0.0, axis=1)
        dLfull += dense
    dX = rb(dXs.reshape(N, k, -1).sum(1) + dLfull @ Wg.T)
    return dict(Z=Z, H=H, Ys=Ys, Y=Y, dYs=dYs, dl=dl, dZ=dZ, dXs=dXs, dX=dX, dW1=dW1, dW2=dW2,
                dWg=rb(X.T @ dLfull), dbg=dLfull.sum(0))
