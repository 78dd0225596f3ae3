"""ctypes front end of the CPU oracle (``lshe_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, the smoke check and the
benchmark's CPU-baseline leg.  The HIP library and its Python binding never
import this package, and this package never imports them.

The wrapper only marshals NumPy arrays; all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lshe_oracle.c")
_LIB = os.path.join(_HERE, "liblshe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP only for the multi-unit driver)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _declare(L):
    for name in ("lsheo_select", "lsheo_l2_select", "lsheo_apply", "lsheo_decode_step",
                 "lsheo_l2_decode_step", "lsheo_max_threads"):
        getattr(L, name).restype = C.c_int
    L.lsheo_norm2.restype = C.c_double
    return L


def lib():
    """The oracle built from ``lshe_oracle.c`` beside this file -- nothing else is ever loaded
    implicitly (no environment variable, no search path)."""
    global _lib
    if _lib is None:
        _lib = _declare(C.CDLL(build()))
    return _lib


def load(path: str):
    """Replace the library by the one at ``path`` for the rest of this process.  Only the
    mutation test calls this (in a child process that runs the pins on a deliberately broken
    copy of the source); it refuses to run on a machine with a GPU device node, so the parity
    tests can never be pointed at another oracle."""
    global _lib
    if os.path.exists("/dev/kfd"):
        raise RuntimeError("oracle.load() is for CPU-only mutation tests")
    _lib = _declare(C.CDLL(path))
    return _lib


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def words(r: int) -> int:
    return (r + 31) // 32


def hash_codes(X, R, with_margin=False):
    """eq. (2).  X [n][d], R [d][r] -> codes uint32 [n][W] (and margins [n][r])."""
    X = _f32(X)
    R = _f32(R)
    n, d = X.shape
    assert R.shape[0] == d
    r = R.shape[1]
    codes = np.zeros((n, words(r)), dtype=np.uint32)
    margin = np.zeros((n, r), dtype=np.float64) if with_margin else None
    lib().lsheo_hash(_p(X, C.c_float), C.c_int64(n), C.c_int(d), _p(R, C.c_float), C.c_int(r),
                     _p(codes, C.c_uint32), _p(margin, C.c_double))
    return (codes, margin) if with_margin else codes


def score(codes, cq):
    """eq. (5), summed over the group.  codes [n][W], cq [G][W] -> int32 [n]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    cq = np.ascontiguousarray(cq, dtype=np.uint32)
    n, W = codes.shape
    G = cq.shape[0]
    assert cq.shape[1] == W
    out = np.zeros(n, dtype=np.int32)
    lib().lsheo_score(_p(codes, C.c_uint32), C.c_int(n), C.c_int(W), _p(cq, C.c_uint32),
                      C.c_int(G), _p(out, C.c_int32))
    return out


def select(scores, slot_pos, n_valid, t, n_sink=0, n_recent=0):
    """eq. (6) / Algorithm 1 step 1."""
    scores = np.ascontiguousarray(scores, dtype=np.int32)
    slot_pos = np.ascontiguousarray(slot_pos, dtype=np.int32)
    Cn = scores.shape[0]
    return int(lib().lsheo_select(_p(scores, C.c_int32), _p(slot_pos, C.c_int32), C.c_int(Cn),
                                  C.c_int(n_valid), C.c_int(t), C.c_int(n_sink),
                                  C.c_int(n_recent)))


def attend(q, K, V, n_valid=None, with_prob=False):
    """eq. (1).  q [G][d], K, V [>=n_valid][d] -> float64 [G][d]."""
    q = _f32(q)
    K = _f32(K)
    V = _f32(V)
    G, d = q.shape
    if n_valid is None:
        n_valid = K.shape[0]
    out = np.zeros((G, d), dtype=np.float64)
    prob = np.zeros((G, max(n_valid, 1)), dtype=np.float64) if with_prob else None
    lib().lsheo_attend(_p(q, C.c_float), _p(K, C.c_float), _p(V, C.c_float), C.c_int(n_valid),
                       C.c_int(d), C.c_int(G), _p(out, C.c_double), _p(prob, C.c_double))
    return (out, prob[:, :n_valid]) if with_prob else out


def evicted_mass(q, K, k_new, e):
    """Section 4.8 per step: attention probability on slot e among the C cached keys and the new key."""
    q = _f32(q)
    K = _f32(K)
    k_new = _f32(k_new).ravel()
    G, d = q.shape
    mass = np.zeros(G, dtype=np.float64)
    lib().lsheo_evicted_mass(_p(q, C.c_float), _p(K, C.c_float), C.c_int(K.shape[0]), C.c_int(d),
                             C.c_int(G), _p(k_new, C.c_float), C.c_int(int(e)), _p(mass, C.c_double))
    return mass


def norm2(x) -> float:
    """Squared L2 norm of one vector, accumulated in double (the L2-norm comparator's score)."""
    x = _f32(x).ravel()
    return float(lib().lsheo_norm2(_p(x, C.c_float), C.c_int(x.shape[0])))


def norm2_rows(X) -> np.ndarray:
    """norm2 of every row of X [n][d] -> float64 [n]."""
    X = _f32(X)
    return np.array([norm2(row) for row in X], dtype=np.float64)


def l2_select(norm2_slots, slot_pos, n_valid, t, n_sink=0, n_recent=0) -> int:
    """The comparator's victim: append while filling, else the lowest evictable slot with the
    largest squared norm."""
    nn = np.ascontiguousarray(norm2_slots, dtype=np.float64)
    slot_pos = np.ascontiguousarray(slot_pos, dtype=np.int32)
    return int(lib().lsheo_l2_select(_p(nn, C.c_double), _p(slot_pos, C.c_int32),
                                     C.c_int(nn.shape[0]), C.c_int(n_valid), C.c_int(t),
                                     C.c_int(n_sink), C.c_int(n_recent)))


class UnitCache:
    """State of one (sequence, layer, KV head) unit: fixed-budget K/V/code slots.

    policy "hash" is HashEvict (Algorithm 1); "l2" is the L2-norm comparator, which keeps the
    squared norm of each cached key in ``norm2`` (float64) instead of hash codes (R and
    hash_bits are then unused)."""

    def __init__(self, budget, head_dim, hash_bits, gqa_group, R, n_sink=0, n_recent=0,
                 policy="hash"):
        self.C, self.d, self.r, self.G = int(budget), int(head_dim), int(hash_bits), int(gqa_group)
        self.policy = policy
        assert policy in ("hash", "l2")
        self.W = words(self.r) if policy == "hash" else 1
        self.n_sink, self.n_recent = int(n_sink), int(n_recent)
        if self.C <= self.n_sink + self.n_recent:
            raise ValueError("budget %d leaves no evictable slot beside %d first and %d recent "
                             "always-kept tokens" % (self.C, self.n_sink, self.n_recent))
        self.R = _f32(R) if R is not None else np.zeros((self.d, self.r), np.float32)
        assert self.R.shape == (self.d, self.r)
        self.K = np.zeros((self.C, self.d), dtype=np.float32)
        self.V = np.zeros((self.C, self.d), dtype=np.float32)
        self.codes = np.zeros((self.C, self.W), dtype=np.uint32)
        self.norm2 = np.zeros(self.C, dtype=np.float64)     # policy "l2" only
        self.slot_pos = np.full(self.C, -1, dtype=np.int32)
        self.n_valid = np.zeros(1, dtype=np.int32)

    def l2_select(self, t) -> int:
        """The comparator's own victim for token index t (state untouched)."""
        return l2_select(self.norm2, self.slot_pos, int(self.n_valid[0]), t, self.n_sink,
                         self.n_recent)

    def decode_step(self, q, k_new, v_new, t, codes_in=None, attend=True, victim_in=-1):
        """Algorithm 1 at token index t.  Returns dict(out, evicted, scores, codes, mass);
        policy "l2": dict(out, evicted, norms (squared norms before the step), mass), and
        ``victim_in`` >= 0 makes the step write that slot instead of choosing one."""
        q = _f32(q).reshape(self.G, self.d)
        k_new = _f32(k_new).reshape(self.d)
        v_new = _f32(v_new).reshape(self.d)
        out = np.zeros((self.G, self.d), dtype=np.float64)
        ev = np.zeros(1, dtype=np.int32)
        sc = np.zeros(self.C, dtype=np.int32)
        co = np.zeros((self.G + 1, self.W), dtype=np.uint32)
        mass = np.zeros(self.G, dtype=np.float64)
        if self.policy == "l2":
            norms = self.norm2.copy()
            norms[int(self.n_valid[0]):] = -1.0
            rc = lib().lsheo_l2_decode_step(
                _p(self.K, C.c_float), _p(self.V, C.c_float), _p(self.norm2, C.c_double),
                _p(self.slot_pos, C.c_int32), _p(self.n_valid, C.c_int32),
                C.c_int(self.C), C.c_int(self.d), C.c_int(self.G), C.c_int(self.n_sink),
                C.c_int(self.n_recent), _p(q, C.c_float), _p(k_new, C.c_float),
                _p(v_new, C.c_float), C.c_int(int(t)), C.c_int(int(victim_in)),
                C.c_int(1 if attend else 0), _p(out, C.c_double), _p(ev, C.c_int32),
                _p(mass, C.c_double))
            if rc != 0:
                raise RuntimeError("no evictable slot")
            return {"out": out, "evicted": int(ev[0]), "norms": norms, "mass": mass}
        if codes_in is not None:
            codes_in = np.ascontiguousarray(codes_in, dtype=np.uint32).reshape(self.G + 1, self.W)
        rc = lib().lsheo_decode_step(
            _p(self.K, C.c_float), _p(self.V, C.c_float), _p(self.codes, C.c_uint32),
            _p(self.slot_pos, C.c_int32), _p(self.n_valid, C.c_int32),
            C.c_int(self.C), C.c_int(self.d), C.c_int(self.r), C.c_int(self.G),
            C.c_int(self.n_sink), C.c_int(self.n_recent), _p(self.R, C.c_float),
            _p(q, C.c_float), _p(k_new, C.c_float), _p(v_new, C.c_float), C.c_int(int(t)),
            _p(codes_in, C.c_uint32), C.c_int(1 if attend else 0),
            _p(out, C.c_double), _p(ev, C.c_int32), _p(sc, C.c_int32), _p(co, C.c_uint32),
            _p(mass, C.c_double))
        if rc != 0:
            raise RuntimeError("no evictable slot")
        return {"out": out, "evicted": int(ev[0]), "scores": sc, "codes": co, "mass": mass}

    def prefill(self, Kp, Vp, Qp, codes_k=None, codes_q=None):
        """Prompt Encoding Stage.  Kp, Vp [N][d]; Qp [G][N][d].  Returns the eviction log."""
        Kp = _f32(Kp)
        Vp = _f32(Vp)
        Qp = _f32(Qp)
        N = Kp.shape[0]
        assert Kp.shape == (N, self.d) and Vp.shape == (N, self.d)
        assert Qp.shape == (self.G, N, self.d)
        if codes_k is not None:
            codes_k = np.ascontiguousarray(codes_k, dtype=np.uint32).reshape(N, self.W)
            codes_q = np.ascontiguousarray(codes_q, dtype=np.uint32).reshape(self.G, N, self.W)
        log = np.zeros(max(N - self.C, 0), dtype=np.int32)
        if self.policy == "l2":
            lib().lsheo_l2_prefill(
                _p(Kp, C.c_float), _p(Vp, C.c_float), C.c_int(N), _p(self.K, C.c_float),
                _p(self.V, C.c_float), _p(self.norm2, C.c_double), _p(self.slot_pos, C.c_int32),
                _p(self.n_valid, C.c_int32), C.c_int(self.C), C.c_int(self.d),
                C.c_int(self.n_sink), C.c_int(self.n_recent), _p(log, C.c_int32))
            return log
        lib().lsheo_prefill(
            _p(Kp, C.c_float), _p(Vp, C.c_float), _p(Qp, C.c_float), C.c_int(N),
            _p(self.K, C.c_float), _p(self.V, C.c_float), _p(self.codes, C.c_uint32),
            _p(self.slot_pos, C.c_int32), _p(self.n_valid, C.c_int32),
            C.c_int(self.C), C.c_int(self.d), C.c_int(self.r), C.c_int(self.G),
            C.c_int(self.n_sink), C.c_int(self.n_recent), _p(self.R, C.c_float),
            _p(codes_k, C.c_uint32), _p(codes_q, C.c_uint32), _p(log, C.c_int32))
        return log


def decode_step_units(K, V, codes, slot_pos, n_valid, R, q, k_new, v_new, t, gqa_group,
                      hash_bits, n_sink=0, n_recent=0, n_threads=0):
    """Algorithm 1 for many independent units at once (in place on the state arrays).

    K, V [U][C][d] float32; codes [U][C][W]; slot_pos [U][C]; n_valid [U]; q [U][G][d];
    k_new, v_new [U][d]; t [U].  Returns (out float64 [U][G][d], evicted int32 [U]).
    """
    U, Cn, d = K.shape
    for a, ty in ((K, np.float32), (V, np.float32), (codes, np.uint32), (slot_pos, np.int32),
                  (n_valid, np.int32)):
        assert a.dtype == ty and a.flags.c_contiguous
    R = _f32(R)
    q = _f32(q)
    k_new = _f32(k_new)
    v_new = _f32(v_new)
    t = np.ascontiguousarray(t, dtype=np.int32)
    out = np.zeros((U, gqa_group, d), dtype=np.float64)
    ev = np.zeros(U, dtype=np.int32)
    if n_threads <= 0:
        n_threads = max_threads()
    lib().lsheo_decode_step_units(
        C.c_int(U), _p(K, C.c_float), _p(V, C.c_float), _p(codes, C.c_uint32),
        _p(slot_pos, C.c_int32), _p(n_valid, C.c_int32), C.c_int(Cn), C.c_int(d),
        C.c_int(hash_bits), C.c_int(gqa_group), C.c_int(n_sink), C.c_int(n_recent),
        _p(R, C.c_float), _p(q, C.c_float), _p(k_new, C.c_float), _p(v_new, C.c_float),
        _p(t, C.c_int32), _p(out, C.c_double), _p(ev, C.c_int32), C.c_int(n_threads))
    return out, ev


def max_threads() -> int:
    return int(lib().lsheo_max_threads())
