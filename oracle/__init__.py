"""ctypes front end of the CPU oracle in ``moe_oracle.c``.

TEST INFRASTRUCTURE: imported only by the tests, by the smoke check and by the CPU-baseline leg
of the benchmark.  The GPU library never imports it and it never imports the GPU library.

Two builds of the same C file are loaded: ``f64`` (FFN and combine in double, the reference the
GPU outputs are compared with) and ``f32`` (the same steps in float, used to show how little the
reference itself moves with precision).  The routing decision is fp32 in both.

All array arguments are numpy arrays (float32 for activations/weights: bf16 values are widened
exactly before they get here).  The functions keep the C names without the ``oracle_`` prefix.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")


def lib_path(prec: str) -> str:
    return os.path.join(_HERE, f"libmoe_oracle_{prec}.so")


def build(force: bool = True) -> None:
    """Compile both precisions with gcc (plain -O2, no fast-math, no contraction)."""
    for prec, real in (("f64", "double"), ("f32", "float")):
        out = lib_path(prec)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-mfma", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
               "-fPIC", f"-DREAL={real}", _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class Oracle:
    """One precision of the oracle.  ``Oracle('f64')`` is the reference."""

    def __init__(self, prec: str = "f64"):
        assert prec in ("f64", "f32")
        if not os.path.exists(lib_path(prec)) or os.path.getmtime(lib_path(prec)) < os.path.getmtime(_SRC):
            build(force=False)
        self.prec = prec
        self.real = np.float64 if prec == "f64" else np.float32
        self.lib = ctypes.CDLL(lib_path(prec))
        self.lib.oracle_real_bytes.restype = ctypes.c_int
        assert self.lib.oracle_real_bytes() == np.dtype(self.real).itemsize
        self.lib.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_route", "oracle_permute", "oracle_gather", "oracle_expert_group_forward",
                     "oracle_shared_forward", "oracle_combine", "oracle_token_forward",
                     "oracle_set_num_threads", "oracle_residual_norm"):
            getattr(self.lib, name).restype = None

    # -- helpers -------------------------------------------------------------------------
    def num_threads(self) -> int:
        return int(self.lib.oracle_num_threads())

    def set_num_threads(self, n: int) -> None:
        self.lib.oracle_set_num_threads(ctypes.c_int(int(n)))

    def _real(self, a):
        return np.ascontiguousarray(a, dtype=self.real)

    # -- the steps of the path -----------------------------------------------------------
    def route(self, x, Wr, bias, K, renorm, want_logits=False):
        x, Wr = _f32(x), _f32(Wr)
        T, H = x.shape
        E = Wr.shape[0]
        assert Wr.shape[1] == H and H % 8 == 0 and 1 <= K <= E
        bias = None if bias is None else _f32(bias)
        ids = np.empty((T, K), np.int32)
        w = np.empty((T, K), np.float32)
        logits = np.empty((T, E), np.float32) if want_logits else None
        self.lib.oracle_route(_p(x), _p(Wr), _p(bias), T, H, E, K, int(bool(renorm)), _p(ids), _p(w),
                              _p(logits))
        return (ids, w, logits) if want_logits else (ids, w)

    def permute(self, ids, E):
        ids = _i32(ids)
        T, K = ids.shape
        assert ids.size == 0 or (ids.min() >= 0 and ids.max() < E)
        offsets = np.empty(E + 1, np.int32)
        src_of_row = np.empty(T * K, np.int32)
        row_of_pair = np.empty(T * K, np.int32)
        self.lib.oracle_permute(_p(ids), T, K, E, _p(offsets), _p(src_of_row), _p(row_of_pair))
        return offsets, src_of_row, row_of_pair

    def gather(self, x, src_of_row, K):
        x, src_of_row = _f32(x), _i32(src_of_row)
        P, H = src_of_row.shape[0], x.shape[1]
        Xp = np.empty((P, H), np.float32)
        self.lib.oracle_gather(_p(x), _p(src_of_row), P, K, H, _p(Xp))
        return Xp

    def expert_group_forward(self, lo, hi, Xp, offsets, Wg, Wu, Wd, Yp=None):
        Xp, offsets, Wg, Wu, Wd = _f32(Xp), _i32(offsets), _f32(Wg), _f32(Wu), _f32(Wd)
        P, H = Xp.shape
        E, I, _ = Wg.shape
        assert Wg.shape == (E, I, H) and Wu.shape == (E, I, H) and Wd.shape == (E, H, I)
        assert 0 <= lo < hi <= E and offsets.shape[0] == E + 1
        if Yp is None:
            Yp = np.zeros((P, H), self.real)
        assert Yp.dtype == self.real and Yp.flags.c_contiguous and Yp.shape == (P, H)
        self.lib.oracle_expert_group_forward(int(lo), int(hi), _p(Xp), _p(offsets), _p(Wg), _p(Wu),
                                             _p(Wd), P, H, E, I, _p(Yp))
        return Yp

    def shared_forward(self, x, Wsg, Wsu, Wsd, wgate):
        x, Wsg, Wsu, Wsd = _f32(x), _f32(Wsg), _f32(Wsu), _f32(Wsd)
        wgate = None if wgate is None else _f32(wgate)
        T, H = x.shape
        Is = Wsg.shape[0]
        assert Wsg.shape == (Is, H) and Wsu.shape == (Is, H) and Wsd.shape == (H, Is)
        S = np.empty((T, H), self.real)
        sg = np.empty(T, self.real)
        self.lib.oracle_shared_forward(_p(x), _p(Wsg), _p(Wsu), _p(Wsd), _p(wgate), T, H, Is, _p(S),
                                       _p(sg))
        return S, sg

    def combine(self, Yp, row_of_pair, w, S, sg, K):
        Yp, row_of_pair, w = self._real(Yp), _i32(row_of_pair), _f32(w)
        P, H = Yp.shape
        T = P // K
        S = None if S is None else self._real(S)
        sg = None if sg is None else self._real(sg)
        out = np.empty((T, H), self.real)
        self.lib.oracle_combine(_p(Yp), _p(row_of_pair), _p(w), _p(S), _p(sg), T, H, K, _p(out))
        return out

    def residual_norm(self, x, y, eps=1e-6):
        """bf16( (x + y) / sqrt(mean((x + y)^2) + eps) ) per row; returns float32 holding bf16 values."""
        x, y = _f32(x), self._real(y)
        T, H = x.shape
        out = np.empty((T, H), np.float32)
        self.lib.oracle_residual_norm(_p(x), _p(y), T, H, ctypes.c_double(eps), _p(out))
        return out

    def token_forward(self, tokens, x, Wr, bias, Wg, Wu, Wd, shared, K, renorm):
        """Per-token definition for the listed tokens.  shared = (Wsg, Wsu, Wsd, wgate) or None."""
        tok = _i32(tokens)
        x, Wr, Wg, Wu, Wd = _f32(x), _f32(Wr), _f32(Wg), _f32(Wu), _f32(Wd)
        bias = None if bias is None else _f32(bias)
        H = x.shape[1]
        E, I, _ = Wg.shape
        if shared is not None:
            Wsg, Wsu, Wsd, wgate = (_f32(a) if a is not None else None for a in shared)
            Is = Wsg.shape[0]
        else:
            Wsg = Wsu = Wsd = wgate = None
            Is = 0
        n = tok.shape[0]
        out = np.empty((n, H), self.real)
        ids = np.empty((n, K), np.int32)
        w = np.empty((n, K), np.float32)
        self.lib.oracle_token_forward(_p(tok), n, _p(x), _p(Wr), _p(bias), _p(Wg), _p(Wu), _p(Wd),
                                      _p(Wsg), _p(Wsu), _p(Wsd), _p(wgate), H, E, K, I, Is,
                                      int(bool(renorm)), _p(out), _p(ids), _p(w))
        return out, ids, w

    # -- the whole path, in the paper's order --------------------------------------------
    def layer(self, x, Wr, bias, Wg, Wu, Wd, shared, K, renorm, groups=None):
        """route -> permute -> one expert_group_forward per block -> shared -> combine.

        groups: list of (lo, hi) covering [0, E); default one block of all experts.
        Returns a dict with every intermediate array."""
        E = Wg.shape[0]
        ids, w = self.route(x, Wr, bias, K, renorm)
        offsets, src_of_row, row_of_pair = self.permute(ids, E)
        Xp = self.gather(x, src_of_row, K)
        Yp = np.zeros((Xp.shape[0], Xp.shape[1]), self.real)
        for lo, hi in (groups or [(0, E)]):
            self.expert_group_forward(lo, hi, Xp, offsets, Wg, Wu, Wd, Yp)
        S = sg = None
        if shared is not None:
            S, sg = self.shared_forward(x, *shared)
        out = self.combine(Yp, row_of_pair, w, S, sg, K)
        return dict(ids=ids, w=w, offsets=offsets, src_of_row=src_of_row, row_of_pair=row_of_pair,
                    Xp=Xp, Yp=Yp, S=S, sg=sg, out=out)
