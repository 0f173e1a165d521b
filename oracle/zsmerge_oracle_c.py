"""ctypes face of the plain-C oracle (zsmerge_oracle_c.c).  TEST INFRASTRUCTURE ONLY.

Argument marshalling and nothing else: every number comes out of the C file.  `BatchCache`
holds the state of many units in NumPy arrays that the C code updates in place; `UnitCache`
is a one-unit view with the attributes and methods of the Python oracle's class of the same
name, so that the same pins can be run against both.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

from .zsmerge_oracle import StepInfo

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "zsmerge_oracle_c.c")
LIB = os.path.join(HERE, "libzsm_oracle_c.so")

_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int32)
_lp = C.POINTER(C.c_int64)


class _Batch(C.Structure):
    _fields_ = [("n_units", C.c_int32), ("d", C.c_int32), ("G", C.c_int32), ("B_r", C.c_int32), ("cap", C.c_int32),
                ("pad_", C.c_int32), ("lam", C.c_double), ("alpha", C.c_double), ("scale", C.c_double),
                ("K", _dp), ("V", _dp), ("pos", _lp), ("w", _lp), ("s", _dp), ("n_seen", _lp),
                ("B_p", _ip), ("B_c", _ip)]


def build() -> str:
    """Compile the C oracle (IEEE arithmetic as written: no fast-math, no contraction)."""
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        L = C.CDLL(LIB)
        L.zso_decode_step.argtypes = [C.POINTER(_Batch), _dp, _dp, _dp, _dp, _ip, _ip, _ip, _dp, _ip, _dp, _lp]
        L.zso_prompt_scores.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, _dp, _dp, C.c_double, C.c_double, _dp]
        L.zso_prefill_compress.argtypes = [C.POINTER(_Batch), C.c_int, C.c_int, _ip, _dp, _dp, _dp, _dp]
        L.zso_full_attention_row.argtypes = [C.c_int, C.c_int, _dp, _dp, _dp, C.c_double, _dp, _dp]
        for f in (L.zso_decode_step, L.zso_prompt_scores, L.zso_prefill_compress,
                  L.zso_full_attention_row, L.zso_threads):
            f.restype = C.c_int
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().zso_threads())


def _d(a):
    return a.ctypes.data_as(_dp)


def _f64(x, *shape):
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    return a.reshape(shape) if shape else a


class BatchCache:
    """State of n units side by side.  B_p, B_c: one int for all units or one per unit."""

    def __init__(self, n_units: int, d: int, G: int, B_p, B_c, B_r: int, lam: float = 0.98, alpha: float = 1.0,
                 scale: Optional[float] = None, cap: Optional[int] = None):
        self.n, self.d, self.G, self.B_r = int(n_units), int(d), int(G), int(B_r)
        self.B_p = np.ascontiguousarray(np.broadcast_to(np.asarray(B_p, dtype=np.int32), (self.n,)))
        self.B_c = np.ascontiguousarray(np.broadcast_to(np.asarray(B_c, dtype=np.int32), (self.n,)))
        if (self.B_p < 1).any():
            raise ValueError("B_p >= 1 required (the incoming token must not evict itself)")
        need = int((self.B_p + self.B_c).max()) + self.B_r
        self.cap = int(cap) if cap else need
        assert self.cap >= need
        self.lam, self.alpha = float(lam), float(alpha)
        self.scale = float(scale) if scale else 1.0 / np.sqrt(d)
        n, cp = self.n, self.cap
        self.K = np.zeros((n, cp, d))
        self.V = np.zeros((n, cp, d))
        self.pos = np.full((n, cp), -1, dtype=np.int64)
        self.w = np.zeros((n, cp), dtype=np.int64)
        self.s = np.zeros((n, cp))
        self.n_seen = np.zeros(n, dtype=np.int64)
        self._b = _Batch(n, d, G, B_r, cp, 0, self.lam, self.alpha, self.scale, _d(self.K), _d(self.V),
                         self.pos.ctypes.data_as(_lp), self.w.ctypes.data_as(_lp), _d(self.s),
                         self.n_seen.ctypes.data_as(_lp), self.B_p.ctypes.data_as(_ip), self.B_c.ctypes.data_as(_ip))

    def decode_step(self, q, k_new, v_new, debug: bool = False):
        """q [n, G, d], k_new, v_new [n, d] -> out [n, G, d], write_slot, evicted_pos, merged_slot [n]
        (and, with debug, the probabilities [n, G, cap + 1], the candidate lists [n, cap + 1] = count then
        slots, and the candidates' scores and positions [n, cap] as the choice saw them)."""
        n, G, d = self.n, self.G, self.d
        q, k_new, v_new = _f64(q, n, G, d), _f64(k_new, n, d), _f64(v_new, n, d)
        out = np.empty((n, G, d))
        ws, ev, mg = (np.empty(n, dtype=np.int32) for _ in range(3))
        a = np.empty((n, G, self.cap + 1)) if debug else None
        cand = np.empty((n, self.cap + 1), dtype=np.int32) if debug else None
        cs = np.empty((n, self.cap)) if debug else None
        cp = np.empty((n, self.cap), dtype=np.int64) if debug else None
        e = lib().zso_decode_step(C.byref(self._b), _d(q), _d(k_new), _d(v_new), _d(out), ws.ctypes.data_as(_ip),
                                  ev.ctypes.data_as(_ip), mg.ctypes.data_as(_ip), _d(a) if debug else None,
                                  cand.ctypes.data_as(_ip) if debug else None, _d(cs) if debug else None,
                                  cp.ctypes.data_as(_lp) if debug else None)
        if e:
            raise RuntimeError(f"zso_decode_step: error {e}")
        return (out, ws, ev, mg, a, cand, cs, cp) if debug else (out, ws, ev, mg)

    def prefill_compress(self, Qw, K, V, T: Optional[Sequence[int]] = None):
        """Qw [n, G, W, d]; K, V [n, T_max, d]; T [n] prompt lengths (default: all T_max).
        Returns the prompt scores [n, T_max] (fp32 values, 0 past a unit's length)."""
        n, G, d = self.n, self.G, self.d
        K = _f64(K)
        T_max = K.shape[1]
        K, V = K.reshape(n, T_max, d), _f64(V, n, T_max, d)
        Qw = _f64(Qw)
        W = Qw.size // (n * G * d)
        Qw = Qw.reshape(n, G, W, d)
        Tn = np.ascontiguousarray(np.broadcast_to(np.asarray(T_max if T is None else T, dtype=np.int32), (n,)))
        s = np.zeros((n, T_max))
        e = lib().zso_prefill_compress(C.byref(self._b), W, T_max, Tn.ctypes.data_as(_ip), _d(Qw), _d(K), _d(V), _d(s))
        if e:
            raise RuntimeError(f"zso_prefill_compress: error {e}")
        return s


class UnitCache:
    """One unit of the C oracle behind the interface of the Python oracle's UnitCache."""

    def __init__(self, d: int, G: int, B_p: int, B_c: int, B_r: int, lam: float = 0.98, alpha: float = 1.0,
                 scale: Optional[float] = None):
        self._b = BatchCache(1, d, G, B_p, B_c, B_r, lam, alpha, scale)
        b = self._b
        self.d, self.G, self.B_p, self.B_c, self.B_r = d, G, B_p, B_c, B_r
        self.B = B_p + B_c + B_r
        self.lam, self.alpha, self.scale = b.lam, b.alpha, b.scale
        self.K, self.V, self.pos, self.w, self.s = b.K[0], b.V[0], b.pos[0], b.w[0], b.s[0]

    n_seen = property(lambda self: int(self._b.n_seen[0]))

    # The sets of Alg. 1, read off the state as the C code does: retained tokens by position, the B_p most recent
    # are the proximity set (oldest first), the others the context set; the residual slots in use.
    def _tokens_by_position(self):
        tok = [j for j in range(self.B_r, self.B) if self.w[j] > 0]
        return sorted(tok, key=lambda j: self.pos[j])

    @property
    def Kp(self):
        tok = self._tokens_by_position()
        return tok[max(0, len(tok) - self.B_p):]

    @property
    def Kc(self):
        tok = self._tokens_by_position()
        return tok[:max(0, len(tok) - self.B_p)]

    @property
    def Kr(self):
        return [r for r in range(self.B_r) if self.w[r] > 0]

    def decode_step(self, q, k_new, v_new):
        occ = np.flatnonzero(self.w > 0)
        out, ws, ev, mg, a, cand, cand_s, cand_pos = self._b.decode_step(np.asarray(q, dtype=np.float64).reshape(1, self.G, self.d),
                                                       np.asarray(k_new, dtype=np.float64).reshape(1, self.d),
                                                       np.asarray(v_new, dtype=np.float64).reshape(1, self.d), debug=True)
        self.last_occ = occ
        self.last_a = np.concatenate([a[0][:, occ], a[0][:, -1:]], axis=1)
        nc = int(cand[0, 0])
        info = StepInfo(int(ws[0]), int(ev[0]), int(mg[0]), cand[0, 1:1 + nc].astype(np.int64), cand_s[0, :nc].copy(),
                        cand_pos[0, :nc].copy())
        return out[0], info

    def prefill_compress(self, Qw, K, V):
        K = np.asarray(K, dtype=np.float64)
        return self._b.prefill_compress(np.asarray(Qw, dtype=np.float64).reshape(1, self.G, -1, self.d), K[None], np.asarray(V, dtype=np.float64)[None])[0]

    def online_prefill(self, Q, K, V):
        Q = np.asarray(Q, dtype=np.float64).reshape(self.G, -1, self.d)
        return np.stack([self.decode_step(Q[:, t], K[t], V[t])[0] for t in range(np.asarray(K).shape[0])])

    def export_state(self):
        return dict(K=self.K.copy(), V=self.V.copy(), pos=self.pos.copy(), w=self.w.copy(), s=self.s.copy(),
                    n_seen=self.n_seen)

    def import_state(self, K, V, pos, w, s, n_seen):
        self.K[:], self.V[:] = K, V
        self.pos[:], self.w[:], self.s[:] = pos, w, s
        self._b.n_seen[0] = int(n_seen)


def prompt_scores(Qw, K, lam, scale):
    Qw = _f64(Qw)
    G, W, d = Qw.shape
    K = _f64(K)
    s = np.empty(K.shape[0])
    e = lib().zso_prompt_scores(G, W, K.shape[0], d, _d(Qw), _d(K), float(lam), float(scale), _d(s))
    if e:
        raise RuntimeError(f"zso_prompt_scores: error {e}")
    return s


def full_attention_row(q, K, V, scale):
    q, K, V = _f64(q), _f64(K), _f64(V)
    T, d = K.shape
    out, a = np.empty(d), np.empty(T)
    lib().zso_full_attention_row(T, d, _d(q), _d(K), _d(V), float(scale), _d(out), _d(a))
    return out, a
