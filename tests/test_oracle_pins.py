"""Pins of the fp64 oracle against things other than itself (CPU only).

Algorithm 1 of the paper is a definition; the paper prints no numbers for it.  So
the oracle is pinned by (a) a hand-worked instance (tests/golden), (b) special cases
in which the layer collapses to a textbook routine evaluated with numpy / scipy
library calls, (c) numpy's stable sort for the selection and the permutation,
(d) central finite differences of the oracle's own forward for every gradient, and
(e) invariances.  Shapes are non-square (d != h != E) so a transposed operand fails.
"""
import os

import numpy as np
import pytest
from scipy.special import softmax
from scipy.stats import norm

import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")


def _rand_problem(seed, N=7, d=5, h=6, E=4, k=2, bias=True, dy=True, dtype=np.float64):
    g = np.random.default_rng(seed)
    X = g.standard_normal((N, d))
    Wg = g.standard_normal((d, E))
    W1 = g.standard_normal((E, d, h)) * 0.7
    W2 = g.standard_normal((E, h, d)) * 0.7
    bg = g.standard_normal(E) * 0.3 if bias else None
    dY = g.standard_normal((N, d)) if dy else None
    c = lambda a: None if a is None else a.astype(dtype)
    return orc.OracleProblem(c(X), c(Wg), c(W1), c(W2), k, bg=bg, dY=c(dY))


def _gelu(z):          # z * Phi(z) through scipy's normal CDF (library routine, not erf)
    return z * norm.cdf(z)


def _gelu_grad(z):
    return norm.cdf(z) + z * norm.pdf(z)


def _ffn(x, W1, W2):
    return _gelu(x @ W1) @ W2


# ------------------------------------------------------------------ (a) hand-worked instance
def _golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *nums = line.split()
            vals[key] = np.array([float(v) for v in nums])
    return vals


def _worked_problem(k, dY=None):
    X = np.array([[1.0, 2.0]])
    Wg = np.eye(2)
    W1 = np.array([[[1.0, 0.0], [0.0, 0.0]], [[0.0, 0.0], [0.5, -0.5]]])
    W2 = np.array([[[2.0, 0.0], [0.0, 0.0]], [[1.0, 1.0], [0.0, 2.0]]])
    return orc.OracleProblem(X, Wg, W1, W2, k, dY=dY)


def test_worked_example_k2():
    gold = _golden()
    out = orc.layer(_worked_problem(2, dY=np.array([[1.0, 0.0]])), want_internals=True)
    assert out["idx"].tolist() == [gold["idx_k2"].astype(int).tolist()]
    np.testing.assert_allclose(out["w"][0], gold["w_k2"], rtol=0, atol=2e-16)
    np.testing.assert_allclose(out["Z"][0, 0], gold["z_slot0"], rtol=0, atol=0)
    np.testing.assert_allclose(out["Z"][0, 1], gold["z_slot1"], rtol=0, atol=0)
    np.testing.assert_allclose(out["O"][0, 0], gold["o_slot0"], rtol=0, atol=3e-16)
    np.testing.assert_allclose(out["O"][0, 1], gold["o_slot1"], rtol=0, atol=3e-16)
    np.testing.assert_allclose(out["Y"][0], gold["y_k2"], rtol=0, atol=5e-16)
    np.testing.assert_allclose(out["dl"][0], gold["dl_k2"], rtol=0, atol=5e-16)


def test_worked_example_k1():
    gold = _golden()
    out = orc.layer(_worked_problem(1))
    assert out["idx"].tolist() == [[1]]
    assert out["w"][0, 0] == 1.0
    np.testing.assert_allclose(out["Y"][0], gold["y_k1"], rtol=0, atol=3e-16)


# ------------------------------------------------------------------ (b) collapses to textbook routines
def test_single_expert_is_dense_ffn_forward_and_backward():
    p = _rand_problem(1, N=9, d=5, h=7, E=1, k=1)
    out = orc.layer(p)
    X, W1, W2, dY = p.X, p.W1[0], p.W2[0], p.dY
    Z = X @ W1
    G = _gelu(Z)
    np.testing.assert_allclose(out["Y"], G @ W2, rtol=1e-12, atol=1e-13)
    assert np.all(out["w"] == 1.0) and np.all(out["idx"] == 0)
    dG = dY @ W2.T
    dZ = dG * _gelu_grad(Z)
    np.testing.assert_allclose(out["dW2"][0], G.T @ dY, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["dW1"][0], X.T @ dZ, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["dX"], dZ @ W1.T, rtol=1e-12, atol=1e-12)   # gate term is 0 for k=1
    assert np.all(out["dl"] == 0.0) and np.all(out["dWg"] == 0.0) and np.all(out["dbg"] == 0.0)


def test_single_expert_with_biases_is_dense_ffn_with_biases():
    # E = 1, k = 1: Y = GeLU(X W1 + b1) W2 + b2, and the textbook gradients of that dense network
    p0 = _rand_problem(21, N=9, d=5, h=7, E=1, k=1)
    g = np.random.default_rng(21)
    b1, b2 = g.standard_normal((1, 7)), g.standard_normal((1, 5))
    p = orc.OracleProblem(p0.X, p0.Wg, p0.W1, p0.W2, 1, bg=p0.bg, dY=p0.dY, b1=b1, b2=b2)
    out = orc.layer(p)
    X, W1, W2, dY = p.X, p.W1[0], p.W2[0], p.dY
    Z = X @ W1 + b1[0]
    G = _gelu(Z)
    np.testing.assert_allclose(out["Y"], G @ W2 + b2[0], rtol=1e-12, atol=1e-13)
    dZ = (dY @ W2.T) * _gelu_grad(Z)
    np.testing.assert_allclose(out["dW2"][0], G.T @ dY, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["dW1"][0], X.T @ dZ, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["dX"], dZ @ W1.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["db2"][0], dY.sum(0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["db1"][0], dZ.sum(0), rtol=1e-12, atol=1e-12)


def test_zero_biases_change_nothing_and_b2_shifts_the_output_by_the_weighted_biases():
    p0 = _rand_problem(22, N=7, d=4, h=6, E=4, k=2)
    base = orc.layer(p0)
    z = orc.layer(orc.OracleProblem(p0.X, p0.Wg, p0.W1, p0.W2, 2, bg=p0.bg, dY=p0.dY, b1=np.zeros((4, 6)),
                                    b2=np.zeros((4, 4))))
    for n in ("Y", "dX", "dW1", "dW2", "dWg", "dbg"):
        np.testing.assert_array_equal(z[n], base[n])
    # Y is affine in b2: Y(b2) - Y(0) = sum_j w_j b2[idx_j]  (Algorithm 1's weighted sum)
    b2 = np.random.default_rng(22).standard_normal((4, 4))
    out = orc.layer(orc.OracleProblem(p0.X, p0.Wg, p0.W1, p0.W2, 2, bg=p0.bg, b2=b2))
    shift = (base["w"][:, :, None] * b2[base["idx"]]).sum(1)
    np.testing.assert_allclose(out["Y"] - base["Y"], shift, rtol=1e-11, atol=1e-13)
    # each expert's db2 is the sum of w_j dY over the slots routed to it; db1, db2 rows of unused experts are zero
    ob = orc.layer(orc.OracleProblem(p0.X, p0.Wg, p0.W1, p0.W2, 2, bg=p0.bg, dY=p0.dY, b2=b2))
    ref = np.zeros((4, 4))
    for t in range(7):
        for j in range(2):
            ref[base["idx"][t, j]] += base["w"][t, j] * p0.dY[t]
    np.testing.assert_allclose(ob["db2"], ref, rtol=1e-12, atol=1e-13)


def test_k_equals_E_is_dense_softmax_mixture():
    p = _rand_problem(2, N=6, d=4, h=5, E=3, k=3, dy=False)
    out = orc.layer(p)
    logits = p.X @ p.Wg + p.bg
    prob = softmax(logits, axis=1)
    ref = sum(prob[:, [e]] * _ffn(p.X, p.W1[e], p.W2[e]) for e in range(p.E))
    np.testing.assert_allclose(out["Y"], ref, rtol=1e-12, atol=1e-13)
    # slots are in descending-logit order and the weights are the softmax probabilities
    np.testing.assert_array_equal(out["idx"], np.argsort(-logits, axis=1, kind="stable"))
    np.testing.assert_allclose(out["w"], -np.sort(-prob, axis=1), rtol=1e-13)


def test_identical_experts_make_the_gate_irrelevant():
    p0 = _rand_problem(3, N=8, d=4, h=6, E=5, k=3)
    W1 = np.repeat(p0.W1[:1], p0.E, axis=0)
    W2 = np.repeat(p0.W2[:1], p0.E, axis=0)
    p = orc.OracleProblem(p0.X, p0.Wg, W1, W2, 3, bg=p0.bg, dY=p0.dY)
    out = orc.layer(p)
    np.testing.assert_allclose(out["Y"], _ffn(p.X, W1[0], W2[0]), rtol=1e-12, atol=1e-13)
    # sum over experts of dW equals the dense FFN weight gradient
    Z = p.X @ W1[0]
    dZ = (p.dY @ W2[0].T) * _gelu_grad(Z)
    np.testing.assert_allclose(out["dW1"].sum(0), p.X.T @ dZ, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(out["dW2"].sum(0), _gelu(Z).T @ p.dY, rtol=1e-11, atol=1e-12)
    # every expert gives the same output, so dL/dw_j are equal and the softmax passes no gradient
    np.testing.assert_allclose(out["dl"], 0.0, atol=1e-13)


def test_output_is_linear_in_W2():
    p = _rand_problem(4, dy=False)
    y = orc.layer(p)["Y"]
    y3 = orc.layer(orc.OracleProblem(p.X, p.Wg, p.W1, -3.0 * p.W2, p.k, bg=p.bg))["Y"]
    y0 = orc.layer(orc.OracleProblem(p.X, p.Wg, p.W1, 0.0 * p.W2, p.k, bg=p.bg))["Y"]
    np.testing.assert_allclose(y3, -3.0 * y, rtol=1e-13, atol=1e-14)
    assert np.all(y0 == 0.0)


def test_top1_of_two_experts_selects_by_sign():
    # E=2,k=1 with Wg = (+v, -v): expert 0 iff <x,v> >= 0 (tie -> lower id); output is that expert's FFN
    g = np.random.default_rng(5)
    X = g.standard_normal((20, 3))
    X[3] = 0.0                                        # exact tie
    v = g.standard_normal(3)
    Wg = np.stack([v, -v], axis=1)
    W1 = g.standard_normal((2, 3, 4))
    W2 = g.standard_normal((2, 4, 3))
    out = orc.layer(orc.OracleProblem(X, Wg, W1, W2, 1))
    sel = np.where(X @ v >= 0, 0, 1)
    np.testing.assert_array_equal(out["idx"][:, 0], sel)
    ref = np.stack([_ffn(X[t], W1[sel[t]], W2[sel[t]]) for t in range(20)])
    np.testing.assert_allclose(out["Y"], ref, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ (c) selection and permutation
def test_topk_matches_numpy_stable_sort_with_engineered_ties():
    g = np.random.default_rng(6)
    N, d, E, k = 64, 6, 9, 4
    X = g.integers(-3, 4, (N, d)).astype(np.float64)      # small integers: all sums exact, many ties
    Wg = g.integers(-2, 3, (d, E)).astype(np.float64)
    Wg[:, 5] = Wg[:, 2]                                   # duplicate columns: exact ties everywhere
    Wg[:, 7] = Wg[:, 0]
    X[10] = 0.0                                           # all logits equal -> 0,1,2,3
    W1 = np.zeros((E, d, 2))
    W2 = np.zeros((E, 2, d))
    p = orc.OracleProblem(X, Wg, W1, W2, k)
    idx, w, logits = orc.gate(p)
    np.testing.assert_array_equal(logits, X @ Wg)
    ref = np.argsort(-logits, axis=1, kind="stable")[:, :k]
    np.testing.assert_array_equal(idx, ref)
    assert idx[10].tolist() == [0, 1, 2, 3]
    sel = np.take_along_axis(logits, ref, axis=1)
    np.testing.assert_allclose(w, softmax(sel, axis=1), rtol=1e-14)
    np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-15)
    assert np.all(np.diff(w, axis=1) <= 0) and np.all(w > 0)
    assert all(len(set(r)) == k for r in idx.tolist())


def test_gate_bias_enters_the_logits():
    p = _rand_problem(7, N=12, d=5, E=6, k=2, dy=False)
    idx, w, logits = orc.gate(p)
    np.testing.assert_allclose(logits, p.X @ p.Wg + p.bg, rtol=1e-13, atol=1e-14)


def test_plan_is_numpy_stable_counting_sort():
    g = np.random.default_rng(8)
    E, N, k = 7, 500, 2
    idx = g.integers(0, E, (N, k)).astype(np.int32)
    idx[idx == 4] = 3                                      # expert 4 stays empty
    counts, offsets, pos, perm = orc.plan(idx, E)
    flat = idx.reshape(-1)
    np.testing.assert_array_equal(counts, np.bincount(flat, minlength=E))
    np.testing.assert_array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    np.testing.assert_array_equal(perm, np.argsort(flat, kind="stable"))
    np.testing.assert_array_equal(perm[pos], np.arange(N * k))           # bijection
    assert counts[4] == 0 and counts.sum() == N * k and offsets[-1] == N * k
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)


def test_plan_rejects_out_of_range_expert():
    with pytest.raises(ValueError):
        orc.plan(np.array([[0, 5]], np.int32), 4)


# ------------------------------------------------------------------ (d) gradients by finite differences
def _loss(p):
    return float((orc.layer(orc.OracleProblem(p.X, p.Wg, p.W1, p.W2, p.k, bg=p.bg, b1=p.b1, b2=p.b2))["Y"] * p.dY).sum())


@pytest.mark.parametrize("k,E", [(2, 4), (1, 3), (3, 3)])
def test_gradients_match_central_differences(k, E):
    for seed in range(40, 60):
        p = _rand_problem(seed, N=4, d=3, h=5, E=E, k=k)
        _, _, logits = orc.gate(p)
        srt = -np.sort(-logits, axis=1)
        if k == E or np.min(srt[:, :k] - srt[:, 1:k + 1]) > 5e-2:       # selection locally constant
            break
    else:
        pytest.skip("no seed with a safe decision gap")
    g = np.random.default_rng(k * 10 + E)
    p = orc.OracleProblem(p.X, p.Wg, p.W1, p.W2, p.k, bg=p.bg, dY=p.dY, b1=0.3 * g.standard_normal((E, 5)),
                          b2=0.3 * g.standard_normal((E, 3)))
    out = orc.layer(p)
    eps = 1e-6
    for name, grad in (("X", out["dX"]), ("Wg", out["dWg"]), ("bg", out["dbg"]),
                       ("W1", out["dW1"]), ("W2", out["dW2"]), ("b1", out["db1"]), ("b2", out["db2"])):
        arr = getattr(p, name)
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + eps
            lp = _loss(p)
            arr[i] = old - eps
            lm = _loss(p)
            arr[i] = old
            num[i] = (lp - lm) / (2 * eps)
        scale = max(1.0, np.abs(num).max())
        assert np.max(np.abs(num - grad)) / scale < 2e-8, name
        if k > 1 and name in ("Wg", "bg"):
            assert np.abs(grad).max() > 1e-3          # the gate really receives gradient via the score


# ------------------------------------------------------------------ scores = softmax over all experts
def _all(p, **kw):
    return orc.OracleProblem(p.X, p.Wg, p.W1, p.W2, p.k, bg=p.bg, dY=p.dY, b1=p.b1, b2=p.b2, score_all=True, **kw)


def test_scores_over_all_experts_are_the_softmax_probabilities_of_the_selected():
    p = _rand_problem(61, N=9, d=4, h=5, E=6, k=2)
    base, out = orc.layer(p), orc.layer(_all(p))
    prob = softmax(p.X @ p.Wg + p.bg, axis=1)
    np.testing.assert_array_equal(out["idx"], base["idx"])                     # the selection does not change
    np.testing.assert_allclose(out["w"], np.take_along_axis(prob, out["idx"], 1), rtol=1e-13)
    assert np.all(out["w"].sum(1) < 1.0)
    # the two score modes differ by one factor per token: the probability mass of the selected experts
    mass = out["w"].sum(1, keepdims=True)
    np.testing.assert_allclose(out["w"], base["w"] * mass, rtol=1e-12)
    np.testing.assert_allclose(out["Y"], base["Y"] * mass, rtol=1e-11, atol=1e-13)


def test_scores_over_all_experts_equal_the_other_mode_when_every_expert_is_selected():
    p = _rand_problem(62, N=6, d=4, h=5, E=3, k=3)
    a, b = orc.layer(p), orc.layer(_all(p))
    for n in ("Y", "dX", "dW1", "dW2", "dWg", "dbg", "w", "dl"):
        np.testing.assert_allclose(b[n], a[n], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("k,E", [(2, 5), (1, 4)])
def test_scores_over_all_experts_gradients_match_central_differences(k, E):
    for seed in range(70, 90):
        p = _rand_problem(seed, N=4, d=3, h=5, E=E, k=k)
        _, _, logits = orc.gate(p)
        srt = -np.sort(-logits, axis=1)
        if np.min(srt[:, :k] - srt[:, 1:k + 1]) > 5e-2:
            break
    else:
        pytest.skip("no seed with a safe decision gap")
    p = _all(p)
    out = orc.layer(p)
    loss = lambda: float((orc.layer(orc.OracleProblem(p.X, p.Wg, p.W1, p.W2, p.k, bg=p.bg, score_all=True))["Y"] * p.dY).sum())
    eps = 1e-6
    for name, grad in (("X", out["dX"]), ("Wg", out["dWg"]), ("bg", out["dbg"]), ("W1", out["dW1"]), ("W2", out["dW2"])):
        arr = getattr(p, name)
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + eps
            lp = loss()
            arr[i] = old - eps
            lm = loss()
            arr[i] = old
            num[i] = (lp - lm) / (2 * eps)
        scale = max(1.0, np.abs(num).max())
        assert np.max(np.abs(num - grad)) / scale < 2e-8, name
    # in this mode the gate is trained through the score even with one expert per token, and every expert's
    # column of the gate matrix receives gradient, selected or not
    assert np.abs(out["dWg"]).min(axis=0).max() > 0 and np.all(np.abs(out["dWg"]).max(axis=0) > 1e-6)
    assert np.abs(out["dbg"]).sum() > 1e-3 and abs(out["dbg"].sum()) < 1e-12 * max(1.0, np.abs(out["dbg"]).sum()) * 1e3


def test_k1_passes_no_gradient_to_the_gate():
    out = orc.layer(_rand_problem(9, k=1))
    assert np.all(out["dl"] == 0) and np.all(out["dWg"] == 0) and np.all(out["dbg"] == 0)


# ------------------------------------------------------------------ (e) invariances and API consistency
def test_token_permutation_equivariance_and_expert_relabelling():
    p = _rand_problem(10, N=10, d=4, h=5, E=4, k=2)
    out = orc.layer(p)
    g = np.random.default_rng(0)
    tp = g.permutation(p.N)
    q = orc.OracleProblem(p.X[tp], p.Wg, p.W1, p.W2, p.k, bg=p.bg, dY=p.dY[tp])
    oq = orc.layer(q)
    np.testing.assert_allclose(oq["Y"], out["Y"][tp], rtol=0, atol=0)
    np.testing.assert_allclose(oq["dX"], out["dX"][tp], rtol=0, atol=0)
    np.testing.assert_allclose(oq["dW1"], out["dW1"], rtol=1e-12, atol=1e-13)
    ep = np.array([2, 0, 3, 1])                               # new expert e' holds old expert ep[e']
    r = orc.OracleProblem(p.X, p.Wg[:, ep], p.W1[ep], p.W2[ep], p.k, bg=p.bg[ep], dY=p.dY)
    orr = orc.layer(r)
    np.testing.assert_allclose(orr["Y"], out["Y"], rtol=1e-13, atol=1e-14)
    np.testing.assert_array_equal(ep[orr["idx"]], out["idx"])
    np.testing.assert_allclose(orr["dW2"], out["dW2"][ep], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(orr["dWg"], out["dWg"][:, ep], rtol=1e-13, atol=1e-14)


def test_storage_types_are_widened_exactly():
    from paper_2103_13262_amd.synth import f32_to_bf16_bits, bf16_bits_to_f32

    g = np.random.default_rng(11)
    mk = lambda *s: g.standard_normal(s).astype(np.float32)
    X, Wg, W1, W2, dY = mk(6, 8), mk(8, 3), mk(3, 8, 4), mk(3, 4, 8), mk(6, 8)
    bits = [f32_to_bf16_bits(a) for a in (X, Wg, W1, W2, dY)]
    wide = [orc.bf16_bits_to_f64(b) for b in bits]
    for b, wd in zip(bits, wide):
        np.testing.assert_array_equal(bf16_bits_to_f32(b).astype(np.float64), wd)
    ob = orc.layer(orc.OracleProblem(*bits[:4], 2, dY=bits[4]))
    ow = orc.layer(orc.OracleProblem(*wide[:4], 2, dY=wide[4]))
    of = orc.layer(orc.OracleProblem(*[a.astype(np.float32) for a in wide[:4]], 2, dY=wide[4].astype(np.float32)))
    for key in ("Y", "dX", "dW1", "dW2", "dWg", "dbg", "w"):
        np.testing.assert_array_equal(ob[key], ow[key])
        np.testing.assert_array_equal(of[key], ow[key])
    # bf16 rounding itself: round-to-nearest-even on a half-way case and a plain case
    assert f32_to_bf16_bits(np.array([1.00390625], np.float32))[0] == 0x3F80      # tie -> even
    assert f32_to_bf16_bits(np.array([1.01171875], np.float32))[0] == 0x3F82      # tie -> even (up)
    assert f32_to_bf16_bits(np.array([-2.5], np.float32))[0] == 0xC020


def test_token_subsets_and_tracked_experts_are_consistent():
    p = _rand_problem(12, N=12, d=4, h=5, E=4, k=2)
    full = orc.layer(p)
    a, b = np.array([0, 3, 4, 9, 11], np.int32), np.array([1, 2, 5, 6, 7, 8, 10], np.int32)
    oa, ob = orc.layer(p, tokens=a), orc.layer(p, tokens=b)
    np.testing.assert_array_equal(oa["Y"], full["Y"][a])
    np.testing.assert_array_equal(ob["dX"], full["dX"][b])
    np.testing.assert_allclose(oa["dW1"] + ob["dW1"], full["dW1"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oa["dWg"] + ob["dWg"], full["dWg"], rtol=1e-12, atol=1e-13)
    trk = np.array([2, 0], np.int32)
    ot = orc.layer(p, track=trk, only_tracked=True)
    np.testing.assert_array_equal(ot["dW1"], full["dW1"][trk])
    np.testing.assert_array_equal(ot["dW2"], full["dW2"][trk])
    assert "Y" not in ot and "dWg" not in ot


# ------------------------------------------------------------------ scatter / gather on their own
def _reorder_setup(seed, N=9, d=5, h=6, E=4, k=2):
    from oracle import moe_reorder as ro

    p = _rand_problem(seed, N=N, d=d, h=h, E=E, k=k)
    ref = orc.layer(p, want_internals=True)
    idx, w, _ = orc.gate(p)
    counts, offsets, pos, perm = orc.plan(idx, E)
    return ro, p, ref, idx, w, counts, offsets, pos, perm


def test_scatter_then_gather_with_unit_weight_sums_is_identity():
    ro, p, ref, idx, w, counts, offsets, pos, perm = _reorder_setup(71)
    X = p.X
    Xs = ro.scatter(X, pos, p.k)
    np.testing.assert_array_equal(Xs[pos], np.repeat(X, p.k, axis=0))     # a pure copy, row by row
    for e in range(p.E):                                                   # segments hold the rows of their expert
        assert np.all(idx.reshape(-1)[perm[offsets[e]:offsets[e + 1]]] == e)
    np.testing.assert_allclose(ro.gather(Xs, w, pos), X, rtol=0, atol=1e-14)   # the weights sum to one


def test_scatter_experts_gather_reproduces_the_per_token_oracle():
    """Batched route (scatter, one dense FFN per expert segment in numpy, gather, and the same backwards)
    against the per-token loop of moe_oracle.c: two independent statements of Algorithm 1."""
    ro, p, ref, idx, w, counts, offsets, pos, perm = _reorder_setup(72, N=11, E=5, k=3)
    X, Wg, W1, W2, dY = p.X, p.Wg, p.W1, p.W2, p.dY      # float64 in this problem
    Xs = ro.scatter(X, pos, p.k)
    Ys = np.empty_like(Xs)
    for e in range(p.E):
        seg = slice(offsets[e], offsets[e + 1])
        Ys[seg] = _ffn(Xs[seg], W1[e], W2[e])
    np.testing.assert_allclose(ro.gather(Ys, w, pos), ref["Y"], rtol=1e-12, atol=1e-13)
    dYs, dl = ro.gather_backward(dY, Ys, w, pos)
    np.testing.assert_allclose(dl, ref["dl"], rtol=1e-10, atol=1e-12)
    dXs = np.empty_like(Xs)
    for e in range(p.E):
        seg = slice(offsets[e], offsets[e + 1])
        Z = Xs[seg] @ W1[e]
        dZ = (dYs[seg] @ W2[e].T) * _gelu_grad(Z)
        dXs[seg] = dZ @ W1[e].T
    dX, dWg, dbg = ro.scatter_backward(Wg, Xs, dXs, dl, idx, pos)
    np.testing.assert_allclose(dX, ref["dX"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dWg, ref["dWg"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dbg, ref["dbg"], rtol=1e-10, atol=1e-12)


def test_gather_gradients_match_central_differences():
    ro, p, ref, idx, w, counts, offsets, pos, perm = _reorder_setup(73, N=4, d=3, E=3, k=2)
    g = np.random.default_rng(5)
    Ys = g.standard_normal((p.N * p.k, p.d))
    dY = g.standard_normal((p.N, p.d))
    logits = g.standard_normal((p.N, p.k))          # the k selected logits of each token
    sm = lambda l: softmax(l, axis=1)
    loss = lambda ys, l: float(np.sum(dY * ro.gather(ys, sm(l), pos)))
    dYs, dl = ro.gather_backward(dY, Ys, sm(logits), pos)
    eps = 1e-6
    num = np.zeros_like(Ys)
    for i in np.ndindex(*Ys.shape):
        a, b = Ys.copy(), Ys.copy()
        a[i] += eps
        b[i] -= eps
        num[i] = (loss(a, logits) - loss(b, logits)) / (2 * eps)
    np.testing.assert_allclose(dYs, num, rtol=1e-6, atol=1e-8)
    numl = np.zeros_like(logits)
    for i in np.ndindex(*logits.shape):
        a, b = logits.copy(), logits.copy()
        a[i] += eps
        b[i] -= eps
        numl[i] = (loss(Ys, a) - loss(Ys, b)) / (2 * eps)
    np.testing.assert_allclose(dl, numl, rtol=1e-6, atol=1e-8)


# ------------------------------------------------------------------ load-balance monitor
def test_balance_stats_closed_forms_and_library_softmax():
    from oracle.moe_balance import balance_stats

    g = np.random.default_rng(5)
    N, E, k = 40, 6, 2
    logits = g.standard_normal((N, E))
    idx = np.argsort(-logits, axis=1, kind="stable")[:, :k]
    frac, prob, loss = balance_stats(logits, idx, E)
    np.testing.assert_allclose(frac, np.bincount(idx.reshape(-1), minlength=E) / (N * k), rtol=0, atol=1e-15)
    np.testing.assert_allclose(prob, softmax(logits, axis=1).mean(0), rtol=1e-13)
    assert abs(frac.sum() - 1) < 1e-14 and abs(prob.sum() - 1) < 1e-14
    np.testing.assert_allclose(loss, E * (frac * prob).sum(), rtol=1e-14)
    # a gate that cannot tell the experts apart: every probability is 1/E and the scalar is 1 whatever the routing
    _, p0, l0 = balance_stats(np.zeros((N, E)), idx, E)
    np.testing.assert_allclose(p0, 1.0 / E, rtol=1e-15)
    assert abs(l0 - 1.0) < 1e-14
    # a gate that sends everything to one expert with certainty: the scalar is E
    hot = np.full((N, E), -50.0)
    hot[:, 3] = 50.0
    f1, p1, l1 = balance_stats(hot, np.full((N, 1), 3), E)
    assert f1[3] == 1.0 and abs(p1[3] - 1.0) < 1e-12 and abs(l1 - E) < 1e-10



# ------------------------------------------------------------------ the per-slot values the loop holds (H, dL/dE_i, dL/dz, W1 dz)
def test_per_slot_intermediates_of_a_single_expert_are_the_dense_network_s():
    # E = 1, k = 1: the values per slot are the hidden activations and gradients of the dense FFN (numpy + scipy)
    p = _rand_problem(31, N=9, d=5, h=7, E=1, k=1)
    out = orc.layer(p, want_internals=True)
    X, W1, W2, dY = p.X, p.W1[0], p.W2[0], p.dY
    Z = X @ W1
    dZ = (dY @ W2.T) * _gelu_grad(Z)
    np.testing.assert_allclose(out["H"][:, 0], _gelu(Z), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out["dO"][:, 0], dY, rtol=0, atol=0)                  # w = 1 exactly
    np.testing.assert_allclose(out["dZ"][:, 0], dZ, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out["dXs"][:, 0], dZ @ W1.T, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("score_all", [False, True])
def test_per_slot_intermediates_follow_their_definitions_slot_by_slot(score_all):
    # general routing: every slot (t, j) with expert e = idx[t, j] against the dense expression of that one expert
    # on that one token, and the slots' shares of dX add up to dX minus the gate's share
    p0 = _rand_problem(32, N=11, d=5, h=6, E=4, k=3)
    p = orc.OracleProblem(p0.X, p0.Wg, p0.W1, p0.W2, 3, bg=p0.bg, dY=p0.dY, score_all=score_all)
    out = orc.layer(p, want_internals=True)
    idx, w = out["idx"], out["w"]
    for t in range(p.N):
        for j in range(p.k):
            e = idx[t, j]
            z = p.X[t] @ p.W1[e]
            do = w[t, j] * p.dY[t]
            dz = (p.W2[e] @ do) * _gelu_grad(z)
            np.testing.assert_allclose(out["Z"][t, j], z, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(out["H"][t, j], _gelu(z), rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(out["O"][t, j], _gelu(z) @ p.W2[e], rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(out["dO"][t, j], do, rtol=1e-15, atol=0)
            np.testing.assert_allclose(out["dZ"][t, j], dz, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(out["dXs"][t, j], p.W1[e] @ dz, rtol=1e-12, atol=1e-13)
    _, _, logits = orc.gate(p)
    dL = np.zeros((p.N, p.E))
    np.put_along_axis(dL, idx, out["dl"], axis=1)
    if score_all:
        S = (w * np.einsum("td,tjd->tj", p.dY, out["O"])).sum(1, keepdims=True)
        dense = -softmax(logits, axis=1) * S
        np.put_along_axis(dense, idx, 0.0, axis=1)
        dL += dense
    np.testing.assert_allclose(out["dXs"].sum(1) + dL @ p.Wg.T, out["dX"], rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ the dense per-expert statement (oracle/moe_expert_dense.py)
@pytest.mark.parametrize("bias", [False, True])
def test_dense_expert_segment_equals_the_per_token_oracle(bias):
    from oracle.moe_expert_dense import expert_segment

    p0 = _rand_problem(41, N=40, d=5, h=7, E=4, k=2)
    g = np.random.default_rng(41)
    b1, b2 = (g.standard_normal((4, 7)), g.standard_normal((4, 5))) if bias else (None, None)
    p = orc.OracleProblem(p0.X, p0.Wg, p0.W1, p0.W2, 2, bg=p0.bg, dY=p0.dY, b1=b1, b2=b2)
    out = orc.layer(p, want_internals=True)
    idx, w = out["idx"], out["w"]
    for e in range(p.E):
        t, j = np.nonzero(idx == e)                      # the expert's assignments in ascending assignment order
        assert t.size > 0
        seg = expert_segment(p.X[t], p.W1[e], p.W2[e], w[t, j], p.dY[t], None if b1 is None else b1[e],
                             None if b2 is None else b2[e])
        for name, key in (("Z", "Z"), ("H", "H"), ("O", "O"), ("dO", "dO"), ("dZ", "dZ"), ("dXs", "dXs")):
            np.testing.assert_allclose(seg[name], out[key][t, j], rtol=1e-12, atol=1e-13, err_msg=name)
        for name in ("dW1", "dW2", "db1", "db2"):
            np.testing.assert_allclose(seg[name], out[name][e], rtol=1e-11, atol=1e-12, err_msg=name)
