"""ctypes front end of the C oracle (moe_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Argument marshalling only: every number is produced by the C file.  Inputs are
numpy arrays of dtype float32, float64 or uint16 (bfloat16 bit patterns); all
outputs are float64 / int32.
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, build_oracle

_F32, _BF16, _F64 = 0, 1, 2
_lib = None


class _Problem(C.Structure):
    _fields_ = [
        ("N", C.c_int32), ("d", C.c_int32), ("h", C.c_int32), ("E", C.c_int32), ("k", C.c_int32),
        ("dtype", C.c_int32),
        ("X", C.c_void_p), ("Wg", C.c_void_p), ("bg", C.c_void_p),
        ("W1", C.c_void_p), ("W2", C.c_void_p), ("dY", C.c_void_p),
        ("b1", C.c_void_p), ("b2", C.c_void_p), ("score_all", C.c_int32),
    ]


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build_oracle()
        _lib = C.CDLL(LIB)
        _lib.orc_gate.restype = C.c_int
        _lib.orc_plan.restype = C.c_int
        _lib.orc_layer.restype = C.c_int
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _code(a):
    if a.dtype == np.float32:
        return _F32
    if a.dtype == np.uint16:
        return _BF16
    if a.dtype == np.float64:
        return _F64
    raise TypeError(f"unsupported storage dtype {a.dtype}")


def _ptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def bf16_bits_to_f64(a):
    """Exact widening of bfloat16 bit patterns (uint16) to float64."""
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


class OracleProblem:
    """X[N,d], Wg[d,E], W1[E,d,h], W2[E,h,d], optional bg[E], b1[E,h], b2[E,d] (float64), optional dY[N,d]."""

    def __init__(self, X, Wg, W1, W2, k, bg=None, dY=None, b1=None, b2=None, score_all=False):
        arrs = [np.ascontiguousarray(a) for a in (X, Wg, W1, W2)]
        self.X, self.Wg, self.W1, self.W2 = arrs
        self.dY = None if dY is None else np.ascontiguousarray(dY)
        self.bg = None if bg is None else np.ascontiguousarray(bg, dtype=np.float64)
        code = _code(self.X)
        for a in arrs + ([self.dY] if self.dY is not None else []):
            if _code(a) != code:
                raise TypeError("all tensors must share one storage dtype")
        self.N, self.d = self.X.shape
        self.E, d2, self.h = self.W1.shape
        assert d2 == self.d and self.W2.shape == (self.E, self.h, self.d)
        assert self.Wg.shape == (self.d, self.E)
        assert self.bg is None or self.bg.shape == (self.E,)
        assert self.dY is None or self.dY.shape == self.X.shape
        self.b1 = None if b1 is None else np.ascontiguousarray(b1, dtype=np.float64)
        self.b2 = None if b2 is None else np.ascontiguousarray(b2, dtype=np.float64)
        assert self.b1 is None or self.b1.shape == (self.E, self.h)
        assert self.b2 is None or self.b2.shape == (self.E, self.d)
        self.k = int(k)
        self._c = _Problem(self.N, self.d, self.h, self.E, self.k, code, _ptr(self.X), _ptr(self.Wg),
                           _ptr(self.bg), _ptr(self.W1), _ptr(self.W2), _ptr(self.dY), _ptr(self.b1), _ptr(self.b2),
                           1 if score_all else 0)
        self.score_all = bool(score_all)


def num_threads():
    return int(_load().orc_num_threads())


def gate(p: OracleProblem):
    """Returns idx[N,k] int32, w[N,k] float64, logits[N,E] float64."""
    idx = np.empty((p.N, p.k), np.int32)
    w = np.empty((p.N, p.k), np.float64)
    logits = np.empty((p.N, p.E), np.float64)
    rc = _load().orc_gate(C.byref(p._c), _ptr(logits), _ptr(idx), _ptr(w))
    if rc:
        raise ValueError(f"orc_gate failed ({rc})")
    return idx, w, logits


def plan(idx, E):
    """idx[...]: expert of each assignment a = t*k + j.  Returns counts, offsets, pos, perm."""
    flat = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1)
    M = flat.size
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    pos = np.empty(M, np.int32)
    perm = np.empty(M, np.int32)
    rc = _load().orc_plan(C.c_int64(M), C.c_int32(E), _ptr(flat), _ptr(counts), _ptr(offsets), _ptr(pos),
                          _ptr(perm))
    if rc:
        raise ValueError(f"orc_plan failed ({rc})")
    return counts, offsets, pos, perm


def layer(p: OracleProblem, tokens=None, track=None, only_tracked=False, want_internals=False,
          want_dw=True):
    """Algorithm 1 (and its gradient when p.dY is given) on the listed tokens.

    tokens: token ids (default all).  track: expert ids whose dW1/dW2 are returned
    (default all, natural order).  only_tracked: compute only the slots routed to a
    tracked expert (then only dW1/dW2 are meaningful and returned).
    """
    tokens = np.arange(p.N, dtype=np.int32) if tokens is None else np.ascontiguousarray(tokens, np.int32)
    nt = tokens.size
    backward = p.dY is not None
    if track is None:
        trk, ntrk, nslots = None, -1, p.E
    else:
        trk = np.ascontiguousarray(track, np.int32)
        ntrk = nslots = trk.size
    out = {}
    full = not only_tracked

    def alloc(name, shape, cond=True, dtype=np.float64):
        if cond:
            out[name] = np.empty(shape, dtype)
            return out[name]
        return None

    Y = alloc("Y", (nt, p.d), full)
    dX = alloc("dX", (nt, p.d), full and backward)
    idx = alloc("idx", (nt, p.k), True, np.int32)
    w = alloc("w", (nt, p.k))
    dl = alloc("dl", (nt, p.k), full and backward)
    Z = alloc("Z", (nt, p.k, p.h), want_internals and full)
    O = alloc("O", (nt, p.k, p.d), want_internals and full)
    G = alloc("H", (nt, p.k, p.h), want_internals and full)
    dO = alloc("dO", (nt, p.k, p.d), want_internals and full and backward)
    dZ = alloc("dZ", (nt, p.k, p.h), want_internals and full and backward)
    dXs = alloc("dXs", (nt, p.k, p.d), want_internals and full and backward)
    dW1 = alloc("dW1", (nslots, p.d, p.h), backward and want_dw)
    dW2 = alloc("dW2", (nslots, p.h, p.d), backward and want_dw)
    dWg = alloc("dWg", (p.d, p.E), full and backward)
    dbg = alloc("dbg", (p.E,), full and backward)
    db1 = alloc("db1", (nslots, p.h), backward and want_dw)
    db2 = alloc("db2", (nslots, p.d), backward and want_dw)
    rc = _load().orc_layer(C.byref(p._c), _ptr(tokens), C.c_int32(nt), _ptr(trk), C.c_int32(ntrk),
                           C.c_int32(1 if only_tracked else 0), _ptr(Y), _ptr(dX), _ptr(idx), _ptr(w),
                           _ptr(dl), _ptr(Z), _ptr(O), _ptr(dW1), _ptr(dW2), _ptr(dWg), _ptr(dbg), _ptr(db1),
                           _ptr(db2), _ptr(G), _ptr(dO), _ptr(dZ), _ptr(dXs))
    if rc:
        raise ValueError(f"orc_layer failed ({rc})")
    out["tokens"] = tokens
    return out
