"""The arithmetic that the bf16 gate kernel's selection rests on (Algorithm 1: indices = ArgMax_k(score)), checked on the CPU.

The kernel ranks fp32 logits and keeps as candidates every expert that its error bound cannot separate from the k-th
largest; the candidates are then ranked in fp64.  Three facts carry that:
  (1) the product of two bf16 values is exact in fp32;
  (2) an fp32 sum of n such products, in any order and association, is off by at most n 2^-24 sum|terms|;
  (3) if every logit is known to within err, the experts with  approx >= (k-th largest approx) - 2 err  contain
      every expert that can be among the exact k largest, whatever the ties.
"""
import numpy as np


def _bf16(x):
    """Round fp32 values to bf16 (nearest even), returned as fp32."""
    u = np.asarray(x, np.float32).view(np.uint32)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def test_products_of_bf16_values_are_exact_in_fp32():
    g = np.random.default_rng(1)
    x = _bf16(g.standard_normal(200000) * np.exp(g.uniform(-20, 20, 200000)))
    w = _bf16(g.standard_normal(200000) * np.exp(g.uniform(-20, 20, 200000)))
    p32 = x * w
    assert p32.dtype == np.float32
    np.testing.assert_array_equal(p32.astype(np.float64), x.astype(np.float64) * w.astype(np.float64))


def _sum_in_order(t, order, tree):
    """fp32 sum of t[order]: sequential, or pairwise (a balanced tree) - two associations a matrix unit may use."""
    v = t[order].astype(np.float32)
    if not tree:
        s = np.float32(0)
        for a in v:
            s = np.float32(s + a)
        return s
    while v.size > 1:
        if v.size & 1:
            v = np.append(v, np.float32(0))
        v = (v[0::2] + v[1::2]).astype(np.float32)
    return v[0]


def test_fp32_sum_of_exact_products_stays_within_the_bound_in_any_order():
    g = np.random.default_rng(2)
    worst = 0.0
    for d in (32, 64, 512, 1024):
        for trial in range(6):
            x = _bf16(g.standard_normal(d) * (1 + 3 * g.random()))
            w = _bf16(g.standard_normal(d) * 0.05)
            if trial == 0:                          # heavy cancellation: the sum is tiny against S
                w[1::2] = -w[0::2] * x[0::2] / np.where(x[1::2] == 0, 1, x[1::2])
                w = _bf16(w)
            b = np.float32(g.standard_normal() * 0.1)
            t = np.append(x * w, b)                 # d exact products and the bias
            exact = float(np.sum(t.astype(np.float64)))
            S = float(np.sum(np.abs(t.astype(np.float64))))
            bound = (d + 1) * 2.0 ** -24 * S
            for tree in (False, True):
                for _ in range(3):
                    got = float(_sum_in_order(t, g.permutation(d + 1), tree))
                    assert abs(got - exact) <= bound, (d, tree, got, exact, bound)
                    worst = max(worst, abs(got - exact) / bound)
    assert worst > 1e-3                             # the bound is not vacuous: sums do get a visible share of it


def test_candidate_band_contains_every_possible_member_of_the_exact_top_k():
    g = np.random.default_rng(3)
    for trial in range(3000):
        E = int(g.integers(2, 40))
        k = int(g.integers(1, min(E, 8) + 1))
        exact = np.round(g.standard_normal(E) * 2, int(g.integers(0, 3)))   # coarse values: many exact ties
        err = float(g.choice([0.0, 0.01, 0.3, 1.0]))
        approx = exact + g.uniform(-err, err, E)
        if g.random() < 0.3:                        # the adversarial corners of the error box
            approx = exact + err * g.choice([-1.0, 1.0], E)
        kth_approx = np.sort(approx)[::-1][k - 1]
        cand = approx >= kth_approx - 2 * err - 1e-12          # (1e-12: the rounding of this test's own fp64 arithmetic at the corners)
        assert cand.sum() >= k
        # every expert whose exact logit reaches the exact k-th largest (the selected ones and all that tie with the
        # last of them) must be a candidate: then ranking the candidates exactly, ties to the lower id, is the exact answer
        kth_exact = np.sort(exact)[::-1][k - 1]
        assert np.all(cand[exact >= kth_exact]), (E, k, err)
        order = np.lexsort((np.arange(E), -exact))[:k]                       # exact top-k, ties to the lower id
        c = np.nonzero(cand)[0]
        order_c = c[np.lexsort((c, -exact[c]))[:k]]
        np.testing.assert_array_equal(order, order_c)
