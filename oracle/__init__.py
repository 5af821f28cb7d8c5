"""Float64 CPU oracle (TEST INFRASTRUCTURE ONLY).

Thin ctypes loader around ``ada_oracle.c`` plus the paper's bookkeeping formulas
(``oracle.metrics``).  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product path never does, and this
package never imports the product.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

from . import metrics  # noqa: F401  (re-export)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ada_oracle.c")
_LIB = os.path.join(_HERE, "libada_oracle.so")

CROSS_EARLIER_ONLY = 1
ATTN_CAUSAL = 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (about a second).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-fno-fast-math", "-ffp-contract=off", _SRC, "-o", tmp, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c_dp = ctypes.POINTER(ctypes.c_double)
        c_ip = ctypes.POINTER(ctypes.c_int32)
        c_u8p = ctypes.POINTER(ctypes.c_uint8)
        c_i8p = ctypes.POINTER(ctypes.c_int8)
        c_u64p = ctypes.POINTER(ctypes.c_uint64)
        lib.ada_oracle_threads.restype = ctypes.c_int
        lib.ada_oracle_set_threads.restype = ctypes.c_int
        lib.ada_oracle_set_threads.argtypes = [ctypes.c_int]
        lib.ada_oracle_normalize.argtypes = [c_dp, ctypes.c_int, ctypes.c_int, c_dp, c_dp]
        lib.ada_oracle_gram.argtypes = [c_dp, ctypes.c_int, ctypes.c_int, c_dp]
        lib.ada_oracle_select_full.argtypes = [c_dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                               c_i8p, c_u8p, c_dp, c_ip, c_u64p]
        lib.ada_oracle_gamma_full_rows.argtypes = [c_dp, ctypes.c_int, ctypes.c_int, c_ip, ctypes.c_int, c_dp]
        lib.ada_oracle_cascade_step.argtypes = [c_dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, c_ip,
                                                ctypes.c_int, ctypes.c_uint, c_i8p, c_ip, c_ip, c_ip, c_ip,
                                                c_u64p, c_dp, c_dp]
        lib.ada_oracle_assign_nearest.argtypes = [c_dp, ctypes.c_int, ctypes.c_int, c_ip, ctypes.c_int, c_ip, c_dp]
        lib.ada_oracle_attention_compressed.argtypes = [c_dp, c_dp, c_dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, c_ip,
                                                        ctypes.c_int, c_ip, ctypes.c_uint, c_dp]
        _lib = lib
    return _lib


def _p(a: Optional[np.ndarray], ctype):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctype))


def _as_f64(X) -> np.ndarray:
    X = np.ascontiguousarray(np.asarray(X, dtype=np.float64))
    if X.ndim != 2:
        raise ValueError("X must be T x d")
    return X


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError("%s failed with oracle status %d" % (what, rc))


def threads() -> int:
    return int(_load().ada_oracle_threads())


def set_threads(n: int) -> int:
    """Number of OpenMP threads for later calls (timing only: results do not depend on it); returns the previous one."""
    return int(_load().ada_oracle_set_threads(int(n)))


def normalize(X):
    X = _as_f64(X)
    T, d = X.shape
    Xhat = np.empty_like(X)
    norms = np.empty(T, dtype=np.float64)
    _check(_load().ada_oracle_normalize(_p(X, ctypes.c_double), T, d, _p(Xhat, ctypes.c_double),
                                        _p(norms, ctypes.c_double)), "normalize")
    return Xhat, norms


def gram(X) -> np.ndarray:
    X = _as_f64(X)
    T, d = X.shape
    G = np.empty((T, T), dtype=np.float64)
    _check(_load().ada_oracle_gram(_p(X, ctypes.c_double), T, d, _p(G, ctypes.c_double)), "gram")
    return G


def select_full(X, tau: float, greedy: bool = False, force: Optional[Sequence[int]] = None):
    """Definition "Gram threshold".  Returns dict(mask, idx, gamma, r, gram_ops)."""
    X = _as_f64(X)
    T, d = X.shape
    mask = np.zeros(T, dtype=np.uint8)
    gamma = np.zeros(T, dtype=np.float64)
    r = ctypes.c_int32(0)
    ops = ctypes.c_uint64(0)
    f = None if force is None else np.ascontiguousarray(np.asarray(force, dtype=np.int8))
    _check(_load().ada_oracle_select_full(_p(X, ctypes.c_double), T, d, float(tau), int(bool(greedy)),
                                          _p(f, ctypes.c_int8), _p(mask, ctypes.c_uint8),
                                          _p(gamma, ctypes.c_double), ctypes.byref(r), ctypes.byref(ops)),
           "select_full")
    return dict(mask=mask, idx=np.flatnonzero(mask).astype(np.int32), gamma=gamma, r=int(r.value),
                gram_ops=int(ops.value))


def gamma_full_rows(X, rows) -> np.ndarray:
    X = _as_f64(X)
    T, d = X.shape
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
    out = np.zeros(rows.shape[0], dtype=np.float64)
    _check(_load().ada_oracle_gamma_full_rows(_p(X, ctypes.c_double), T, d, _p(rows, ctypes.c_int32),
                                              int(rows.shape[0]), _p(out, ctypes.c_double)), "gamma_full_rows")
    return out


def cascade_step(X, tau: float, prev_idx, flags: int = 0, force: Optional[Sequence[int]] = None):
    """Algorithm 1.  Returns dict(idx, adds, removes, r_new, gram_ops, gamma, gamma_all)."""
    X = _as_f64(X)
    T, d = X.shape
    prev = np.ascontiguousarray(np.asarray(prev_idx, dtype=np.int32))
    r = int(prev.shape[0])
    idx = np.zeros(T, dtype=np.int32)
    adds = np.zeros(T, dtype=np.int32)
    removes = np.zeros(max(r, 1), dtype=np.int32)
    counts = np.zeros(3, dtype=np.int32)
    ops = ctypes.c_uint64(0)
    gamma = np.zeros(T, dtype=np.float64)
    gamma_all = np.zeros(T, dtype=np.float64)
    f = None if force is None else np.ascontiguousarray(np.asarray(force, dtype=np.int8))
    _check(_load().ada_oracle_cascade_step(_p(X, ctypes.c_double), T, d, float(tau), _p(prev, ctypes.c_int32), r,
                                           int(flags), _p(f, ctypes.c_int8), _p(idx, ctypes.c_int32),
                                           _p(adds, ctypes.c_int32), _p(removes, ctypes.c_int32),
                                           _p(counts, ctypes.c_int32), ctypes.byref(ops),
                                           _p(gamma, ctypes.c_double), _p(gamma_all, ctypes.c_double)),
           "cascade_step")
    return dict(idx=idx[:counts[0]].copy(), adds=adds[:counts[1]].copy(), removes=removes[:counts[2]].copy(),
                r_new=int(counts[0]), gram_ops=int(ops.value), gamma=gamma, gamma_all=gamma_all)


def assign_nearest(X, idx):
    """Section 2.3: nearest representative of every token.  Returns dict(assign, corr)."""
    X = _as_f64(X)
    T, d = X.shape
    R = np.ascontiguousarray(np.asarray(idx, dtype=np.int32))
    assign = np.zeros(T, dtype=np.int32)
    corr = np.zeros(T, dtype=np.float64)
    _check(_load().ada_oracle_assign_nearest(_p(X, ctypes.c_double), T, d, _p(R, ctypes.c_int32), int(R.shape[0]),
                                             _p(assign, ctypes.c_int32), _p(corr, ctypes.c_double)), "assign_nearest")
    return dict(assign=assign, corr=corr)


def attention_compressed(Q, K, V, H: int, idx, assign, flags: int = 0) -> np.ndarray:
    """eq. (1): attention on the representative rows, every token taking its representative's output row.
    Q, K, V: T x (H * d_h).  Returns out, T x (H * d_h), float64."""
    Q, K, V = _as_f64(Q), _as_f64(K), _as_f64(V)
    T, D = Q.shape
    if K.shape != (T, D) or V.shape != (T, D) or D % int(H) != 0:
        raise ValueError("Q, K, V must share the shape T x (H * d_h)")
    R = np.ascontiguousarray(np.asarray(idx, dtype=np.int32))
    a = np.ascontiguousarray(np.asarray(assign, dtype=np.int32))
    if a.shape != (T,):
        raise ValueError("assign must have T entries")
    out = np.empty((T, D), dtype=np.float64)
    _check(_load().ada_oracle_attention_compressed(_p(Q, ctypes.c_double), _p(K, ctypes.c_double), _p(V, ctypes.c_double),
                                                   T, int(H), D // int(H), _p(R, ctypes.c_int32), int(R.shape[0]),
                                                   _p(a, ctypes.c_int32), int(flags), _p(out, ctypes.c_double)),
           "attention_compressed")
    return out


def cascade_layers_adaptive(Xs, tau0: float, kappa: float, eta_target: float, tau_min: float, tau_max: float,
                            flags: int = 0):
    """The layer loop of Section 4.1 with the threshold of Section 8.1 (see metrics.adapt_tau for the reading):
    full selection at layer 0 with tau0, Algorithm 1 afterwards; layer 1 also uses tau0 (no turnover is known yet),
    layer l + 1 the tau adapted from the turnover (eq. (8)) of the step made at layer l.
    Returns (taus, results): the tau each layer used, and the select_full / cascade_step result of each layer."""
    tau = float(np.float32(tau0))                       # the library takes tau0 as a float
    taus, results = [tau], [select_full(Xs[0], tau)]
    prev = results[0]["idx"]
    for X in Xs[1:]:
        taus.append(tau)
        step = cascade_step(X, tau, prev, flags)
        results.append(step)
        eta = metrics.turnover(len(step["adds"]), len(step["removes"]), len(prev))
        tau = metrics.adapt_tau(tau, eta, kappa, eta_target, tau_min, tau_max)
        prev = step["idx"]
    return taus, results
