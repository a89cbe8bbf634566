"""Thin ctypes binding of libmoe355.so: same names as the C ABI in include/moe355.h.

Argument marshalling only.  torch supplies device memory and the stream; every step
of the layer runs in the library's kernels.  There is no fallback: if the library is
missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe355.so")

MOE_OK, MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_WORKSPACE, MOE_ERR_HIP = 0, -1, -2, -3, -4
MOE_F32, MOE_BF16 = 0, 1
EXPORTS = ("moe_workspace_bytes", "moe_workspace_region", "moe_check_status", "moe_plan", "moe_forward", "moe_backward",
           "moe_bias_backward", "moe_balance_stats", "moe_scatter", "moe_gather", "moe_gather_backward", "moe_scatter_backward", "moe_scatter_backward_static",
           "moe_last_error", "moe_profile_enable", "moe_profile_read")


class MoeDesc(C.Structure):
    _fields_ = [("N", C.c_int32), ("d", C.c_int32), ("h", C.c_int32), ("E", C.c_int32), ("k", C.c_int32),
                ("dtype", C.c_int32), ("grad_dtype", C.c_int32), ("accumulate", C.c_int32),
                ("score_all", C.c_int32), ("balance_stats", C.c_int32), ("reserved", C.c_int32 * 6)]


class MoePlan(C.Structure):
    _fields_ = [("topk_idx", C.c_void_p), ("topk_w", C.c_void_p), ("counts", C.c_void_p),
                ("offsets", C.c_void_p), ("pos", C.c_void_p), ("perm", C.c_void_p)]


class MoeKernelTime(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int32), ("total_ms", C.c_double)]


class MoeError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"libmoe355 status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """Loads the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2103_13262_amd.build` "
                "(there is no fallback path)")
        # torch first: its bundled HIP runtime must be the one this process initialises, so that the
        # library's kernels run on the same runtime (and devices, streams) as torch's allocations.
        import torch  # noqa: F401

        L = C.CDLL(LIB_PATH)
        L.moe_workspace_bytes.restype = C.c_size_t
        L.moe_workspace_bytes.argtypes = [C.POINTER(MoeDesc)]
        L.moe_last_error.restype = C.c_char_p
        L.moe_last_error.argtypes = []
        vp = C.c_void_p
        L.moe_plan.restype = C.c_int
        L.moe_plan.argtypes = [C.POINTER(MoeDesc), vp, vp, vp, C.POINTER(MoePlan), vp, C.c_size_t, vp]
        L.moe_forward.restype = C.c_int
        L.moe_forward.argtypes = [C.POINTER(MoeDesc), C.POINTER(MoePlan), vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.moe_backward.restype = C.c_int
        L.moe_backward.argtypes = [C.POINTER(MoeDesc), C.POINTER(MoePlan)] + [vp] * 11 + [C.c_size_t, vp]
        for name, nptr in (("moe_scatter", 3), ("moe_gather", 3), ("moe_gather_backward", 5)):
            getattr(L, name).argtypes = [C.POINTER(MoeDesc), C.POINTER(MoePlan)] + [vp] * nptr
            getattr(L, name).restype = C.c_int
        L.moe_scatter_backward.argtypes = [C.POINTER(MoeDesc), C.POINTER(MoePlan)] + [vp] * 8 + [C.c_size_t, vp]
        L.moe_scatter_backward.restype = C.c_int
        L.moe_scatter_backward_static.argtypes = [C.POINTER(MoeDesc), C.POINTER(MoePlan)] + [vp] * 8
        L.moe_scatter_backward_static.restype = C.c_int
        L.moe_workspace_region.restype = C.c_int
        L.moe_workspace_region.argtypes = [C.POINTER(MoeDesc), C.c_char_p, C.POINTER(C.c_size_t),
                                           C.POINTER(C.c_size_t)]
        L.moe_check_status.restype = C.c_int
        L.moe_check_status.argtypes = [C.POINTER(MoeDesc), vp, C.c_size_t, vp, C.POINTER(C.c_int32)]
        L.moe_profile_enable.restype = C.c_int
        L.moe_profile_enable.argtypes = [C.c_int]
        L.moe_profile_read.restype = C.c_int
        L.moe_profile_read.argtypes = [C.POINTER(MoeKernelTime), C.c_int]
        _lib = L
    return _lib


def _p(t):
    """Device (or raw integer) pointer of a torch tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _check(status):
    if status != MOE_OK:
        raise MoeError(status, lib().moe_last_error().decode())


def make_desc(N, d, h, E, k, dtype=MOE_BF16, grad_dtype=None, accumulate=0, score_all=0, balance_stats=0):
    return MoeDesc(N, d, h, E, k, dtype, dtype if grad_dtype is None else grad_dtype, accumulate, score_all, balance_stats)


def moe_workspace_bytes(desc):
    return int(lib().moe_workspace_bytes(C.byref(desc)))


def moe_workspace_region(desc, name):
    """(offset, bytes) of a named intermediate inside the workspace."""
    off, n = C.c_size_t(0), C.c_size_t(0)
    _check(lib().moe_workspace_region(C.byref(desc), name.encode(), C.byref(off), C.byref(n)))
    return int(off.value), int(n.value)


def moe_check_status(desc, workspace, workspace_bytes, stream=0):
    """The workspace's status word (0 = fine); waits for the stream."""
    out = C.c_int32(-1)
    _check(lib().moe_check_status(C.byref(desc), _p(workspace), C.c_size_t(workspace_bytes), C.c_void_p(stream), C.byref(out)))
    return int(out.value)


def moe_profile_enable(on):
    _check(lib().moe_profile_enable(1 if on else 0))


def moe_profile_read():
    """{kernel group: (launches, total_ms)} since the last read; waits for the recorded work."""
    buf = (MoeKernelTime * 32)()
    n = lib().moe_profile_read(buf, 32)
    if n < 0:
        _check(n)
    return {buf[i].name.decode(): (int(buf[i].launches), float(buf[i].total_ms)) for i in range(n)}


def moe_last_error():
    return lib().moe_last_error().decode()


def make_plan(topk_idx, topk_w, counts, offsets, pos, perm):
    return MoePlan(_p(topk_idx), _p(topk_w), _p(counts), _p(offsets), _p(pos), _p(perm))


def moe_plan(desc, X, Wg, bg, plan, workspace, workspace_bytes, stream=0):
    _check(lib().moe_plan(C.byref(desc), _p(X), _p(Wg), _p(bg), C.byref(plan), _p(workspace),
                          C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def moe_forward(desc, plan, X, W1, W2, b1, b2, Y, workspace, workspace_bytes, stream=0):
    _check(lib().moe_forward(C.byref(desc), C.byref(plan), _p(X), _p(W1), _p(W2), _p(b1), _p(b2), _p(Y),
                             _p(workspace), C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def moe_backward(desc, plan, X, Wg, W1, W2, dY, dX, dWg, dbg, dW1, dW2, workspace, workspace_bytes, stream=0):
    _check(lib().moe_backward(C.byref(desc), C.byref(plan), _p(X), _p(Wg), _p(W1), _p(W2), _p(dY), _p(dX),
                              _p(dWg), _p(dbg), _p(dW1), _p(dW2), _p(workspace), C.c_size_t(workspace_bytes),
                              C.c_void_p(stream)))


def moe_bias_backward(desc, plan, db1, db2, workspace, workspace_bytes, stream=0):
    _check(lib().moe_bias_backward(C.byref(desc), None if plan is None else C.byref(plan), _p(db1), _p(db2), _p(workspace),
                                   C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def moe_balance_stats(desc, plan, fraction, mean_prob, loss, workspace, workspace_bytes, stream=0):
    _check(lib().moe_balance_stats(C.byref(desc), None if plan is None else C.byref(plan), _p(fraction), _p(mean_prob),
                                   _p(loss), _p(workspace), C.c_size_t(workspace_bytes), C.c_void_p(stream)))


def moe_scatter(desc, plan, X, Xs, stream=0):
    _check(lib().moe_scatter(C.byref(desc), None if plan is None else C.byref(plan), _p(X), _p(Xs), C.c_void_p(stream)))


def moe_gather(desc, plan, Ys, Y, stream=0):
    _check(lib().moe_gather(C.byref(desc), None if plan is None else C.byref(plan), _p(Ys), _p(Y), C.c_void_p(stream)))


def moe_gather_backward(desc, plan, dY, Ys, dYs, dl, stream=0):
    _check(lib().moe_gather_backward(C.byref(desc), None if plan is None else C.byref(plan), _p(dY), _p(Ys), _p(dYs), _p(dl),
                                     C.c_void_p(stream)))


def moe_scatter_backward(desc, plan, Wg, Xs, dXs, dl, dX, dWg, dbg, workspace, workspace_bytes, stream=0):
    _check(lib().moe_scatter_backward(C.byref(desc), None if plan is None else C.byref(plan), _p(Wg), _p(Xs), _p(dXs), _p(dl), _p(dX),
                                      _p(dWg), _p(dbg), _p(workspace), C.c_size_t(workspace_bytes),
                                      C.c_void_p(stream)))


def moe_scatter_backward_static(desc, plan, Wg, Xs, dXs, dl, dX, dWg, dbg, stream=0):
    _check(lib().moe_scatter_backward_static(C.byref(desc), None if plan is None else C.byref(plan), _p(Wg), _p(Xs), _p(dXs),
                                             _p(dl), _p(dX), _p(dWg), _p(dbg), C.c_void_p(stream)))


class MoeLayerBuffers:
    """Convenience holder of the device buffers of one problem (allocation through torch only).

    Not part of the ABI: it just allocates what the three calls need and keeps the tensors alive.
    """

    def __init__(self, desc, device="cuda:0"):
        import torch

        self.torch = torch
        self.desc = desc
        self.device = torch.device(device)
        M = desc.N * desc.k
        i32 = dict(dtype=torch.int32, device=self.device)
        self.topk_idx = torch.empty((desc.N, desc.k), **i32)
        self.topk_w = torch.empty((desc.N, desc.k), dtype=torch.float32, device=self.device)
        self.counts = torch.empty(max(desc.E, 4), **i32)
        self.offsets = torch.empty(desc.E + 4, **i32)
        self.pos = torch.empty(max(M, 4), **i32)
        self.perm = torch.empty(max(M, 4), **i32)
        self.plan = make_plan(self.topk_idx if M else self.pos, self.topk_w if M else self.pos, self.counts,
                              self.offsets, self.pos, self.perm)
        self.ws_bytes = moe_workspace_bytes(desc)
        if self.ws_bytes == 0:
            raise MoeError(MOE_ERR_UNSUPPORTED, moe_last_error())
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)

    def stream(self):
        return self.torch.cuda.current_stream(self.device).cuda_stream
