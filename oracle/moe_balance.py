"""Load-balance monitor of a routed batch -- TEST INFRASTRUCTURE ONLY (numpy, fp64).

The paper leaves a load-balance monitor and loss to future work (Section 6); the two statistics such a monitor
is built from are the fraction of assignments every expert receives and the mean probability the gate gives it,
and the usual scalar made of them is E * sum_e fraction_e * mean_probability_e (1 for a uniform gate, E when one
expert gets everything).  Written out from those definitions; shares nothing with the HIP library.
"""
import numpy as np


def balance_stats(logits, idx, E):
    """logits [N,E] float64, idx [N,k] selected experts.  Returns fraction[E], mean_prob[E], loss."""
    logits = np.asarray(logits, np.float64)
    N = logits.shape[0]
    idx = np.asarray(idx).reshape(N, -1)
    frac = np.zeros(E)
    for t in range(N):
        for e in idx[t]:
            frac[e] += 1.0
    frac /= idx.size
    prob = np.zeros(E)
    for t in range(N):
        ex = np.exp(logits[t] - logits[t].max())
        prob += ex / ex.sum()
    prob /= N
    return frac, prob, float(E * np.dot(frac, prob))
