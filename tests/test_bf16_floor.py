"""What storing the path's tensors in bfloat16 costs by itself, worked out on the CPU from the oracle (no GPU).

The stated parity bound for bf16 is a max relative error of 2e-2.  These tests rebuild, from the fp64 oracle's own
intermediates, the figures that decide how that bound can be read: an IDEAL bf16 path (tests/bf16_floor.py: every
stored tensor computed exactly from the bf16 tensors before it and rounded once, nothing else approximated) is
compared with the oracle under the strict metric |T - R| / max(|R|, rms(R)) and the relaxed one |T - R| / (|R| + rms(R)).

What they establish (and the parity tests rely on):
  * Z, H, dYs are one rounding away from exact values: 2^-8 = 3.9e-3, far inside the bound;
  * Ys, Y, dl stay inside the bound with room to spare (0.8-1.6e-2), so the HIP path is held to the stated bound there;
  * dZ, dXs, dX and the weight gradients of large experts come within 25 % of the bound or cross it, under either metric;
  * per-expert weight gradients judged against the whole tensor's RMS reach 4e-2 under a skewed load; against the
    expert's own block 1.4-1.8e-2 for experts with at least 64 rows and 2.5e-2 and more for experts with fewer;
  * a gate-bias entry that is a small remainder of cancelling sums is moved by 1e-1 of the vector's size by the
    rounding of Ys alone.
So no bf16 implementation can be held to 2e-2 on every tensor of every shape; the parity tests hold the HIP path to
max(2e-2, 1.5 x the ideal path's error on the same case) and print both.
"""
import numpy as np
import pytest

import oracle as orc
from bf16_floor import ideal_bf16_layer
from harness import oracle_problem, rel_err, strict_err
from paper_2103_13262_amd.synth import Workload, make_inputs


def _floor_errors(w):
    inputs = make_inputs(w)
    p = oracle_problem(w, inputs)
    ref = orc.layer(p, want_internals=True)
    idx, wt, logits = orc.gate(p)
    counts, _, _, _ = orc.plan(idx, w.E)
    got = ideal_bf16_layer(w, inputs, idx, wt, logits if w.score_all else None)
    M = w.M
    pairs = dict(Z=ref["Z"], H=ref["H"], Ys=ref["O"], dYs=ref["dO"], dZ=ref["dZ"], dXs=ref["dXs"])
    out = {n: (strict_err(got[n], r.reshape(M, -1)), rel_err(got[n], r.reshape(M, -1))) for n, r in pairs.items()}
    for n in ("Y", "dl", "dX", "dW1", "dW2", "dWg", "dbg"):
        out[n] = (strict_err(got[n], ref[n]), rel_err(got[n], ref[n]))
    for n in ("dW1", "dW2"):        # per expert: against the whole tensor's RMS, and against the expert's own
        rms = float(np.sqrt(np.mean(ref[n] ** 2)))
        live = [e for e in range(w.E) if counts[e] > 0]
        out[n + "/whole"] = max(rel_err(got[n][e], ref[n][e], rms=rms) for e in live)
        out[n + "/block, 64 rows or more"] = max([strict_err(got[n][e], ref[n][e]) for e in live if counts[e] >= 64] or [0.0])
        out[n + "/block, fewer rows"] = max([strict_err(got[n][e], ref[n][e]) for e in live if counts[e] < 64] or [0.0])
    print(w.name, {k: (f"{v[0]:.2e}/{v[1]:.2e}" if isinstance(v, tuple) else f"{v:.2e}") for k, v in out.items()})
    return out


def test_one_rounding_tensors_and_the_forward_have_room():
    e = _floor_errors(Workload("tiles_skew_bf16", 1024, 256, 512, 8, 2, "bf16", 1.2, 12))
    for n in ("Z", "H", "dYs"):
        assert e[n][0] <= 2.0 ** -8 * 1.001          # a single rounding to 8 significant bits
    for n in ("Ys", "Y", "dl"):
        assert e[n][0] <= 1.3e-2                     # strict metric, well inside 2e-2
    # the backward tensors and the weight gradients leave the stated bound little or no room, under either metric
    for n in ("dZ", "dXs", "dX"):
        assert 1.1e-2 <= e[n][1] <= e[n][0] <= 2e-2
    assert e["dW1"][0] >= 1.9e-2 and e["dW2"][0] >= 1.8e-2        # strict: at the bound before any kernel exists
    assert e["dW1"][1] >= 1.6e-2                                  # relaxed: within 20 % of it


def test_per_expert_gradients_under_a_skewed_load():
    e = _floor_errors(Workload("rand12", 399, 384, 512, 40, 3, "bf16", 0.8, 9012, 0.1))
    assert e["dW2/whole"] >= 3.9e-2 and e["dW1/whole"] >= 3.0e-2   # against the whole tensor's RMS: twice the bound
    # against the expert's own block: inside the bound for experts with 64 rows or more ...
    assert e["dW2/block, 64 rows or more"] <= 1.9e-2 and e["dW1/block, 64 rows or more"] <= 1.9e-2
    # ... and beyond it for experts with few rows, whose elements are sums of few products with no averaging
    assert e["dW2/block, fewer rows"] >= 2.5e-2


def test_short_reductions_put_dx_beyond_the_bound():
    e = _floor_errors(Workload("short_reduction_wide_dx_bf16", 1537, 2048, 256, 16, 1, "bf16", 1.2, 8025, 0.1, True))
    assert e["dX"][1] >= 2.0e-2 and e["dX"][0] >= 2.3e-2 and e["dXs"][0] >= 2.4e-2


def test_a_cancelling_gate_bias_entry_has_no_accuracy_in_bf16():
    e = _floor_errors(Workload("cancelling_gate_bias_bf16", 2503, 512, 256, 3, 2, "bf16", 2.0, 8022, 0.0, True))
    assert e["dbg"][1] >= 1.0e-1
    assert e["dWg"][0] <= 1.2e-2                     # the matrix gradient itself is fine
