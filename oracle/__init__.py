"""CPU oracle package -- TEST INFRASTRUCTURE ONLY.

Holds the slow, plain fp64 reference computations that define correctness for
the GPU library: the classical sequential recursions (``hmm_oracle.c``, loaded
through ctypes), the literal brute-force definitions (``brute_force.py``) and
the paper's own element/operator/scan formulation in fp64 numpy
(``scan_formulation.py``).  It shares no code with the GPU path and must only be
imported by tests, the smoke check and the benchmark's CPU-baseline leg.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hmm_oracle.c")
_LIB = os.path.join(_HERE, "libhmm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, strict IEEE arithmetic: no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.hmm_oracle_smooth.argtypes = [fp, fp, fp, ctypes.c_long, ctypes.c_int, dp, dp, dp]
        lib.hmm_oracle_smooth.restype = ctypes.c_int
        lib.hmm_oracle_viterbi.argtypes = [fp, fp, fp, ctypes.c_long, ctypes.c_int, ip, dp]
        lib.hmm_oracle_viterbi.restype = ctypes.c_int
        lib.hmm_oracle_score.argtypes = [fp, fp, fp, ctypes.c_long, ctypes.c_int, ip]
        lib.hmm_oracle_score.restype = ctypes.c_double
        lib.hmm_oracle_max_product.argtypes = [fp, fp, fp, ctypes.c_long, ctypes.c_int, dp, ip, dp]
        lib.hmm_oracle_max_product.restype = ctypes.c_int
        lib.hmm_oracle_transition_counts.argtypes = [fp, fp, fp, ctypes.c_long, ctypes.c_int, dp]
        lib.hmm_oracle_transition_counts.restype = ctypes.c_int
        lib.hmm_oracle_block_element.argtypes = [fp, fp, ctypes.c_long, ctypes.c_int, ctypes.c_int, dp, dp]
        lib.hmm_oracle_block_element.restype = ctypes.c_int
        lib.hmm_oracle_block_carries.argtypes = [fp, fp, fp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, dp, dp, dp]
        lib.hmm_oracle_block_carries.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def smooth(prior, A, loglik, want_filtered: bool = True):
    """One sequence: prior[D], A[D][D], loglik[T][D] (float32).
    Returns (marginals[T][D] f64, filtered[T][D] f64 or None, loglik f64)."""
    lib = _load()
    prior, pp = _f32(prior)
    A, pa = _f32(A)
    loglik, pl = _f32(loglik)
    T, D = loglik.shape
    assert prior.shape == (D,) and A.shape == (D, D)
    marg = np.empty((T, D), dtype=np.float64)
    filt = np.empty((T, D), dtype=np.float64) if want_filtered else None
    L = ctypes.c_double(0.0)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = lib.hmm_oracle_smooth(pp, pa, pl, T, D, marg.ctypes.data_as(dp),
                               filt.ctypes.data_as(dp) if want_filtered else None, ctypes.byref(L))
    if rc != 0:
        raise RuntimeError("hmm_oracle_smooth failed")
    return marg, filt, float(L.value)


def viterbi(prior, A, loglik):
    """One sequence. Returns (path[T] int32, logprob f64)."""
    lib = _load()
    prior, pp = _f32(prior)
    A, pa = _f32(A)
    loglik, pl = _f32(loglik)
    T, D = loglik.shape
    assert prior.shape == (D,) and A.shape == (D, D)
    path = np.empty(T, dtype=np.int32)
    lp = ctypes.c_double(0.0)
    rc = lib.hmm_oracle_viterbi(pp, pa, pl, T, D, path.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                ctypes.byref(lp))
    if rc != 0:
        raise RuntimeError("hmm_oracle_viterbi failed")
    return path, float(lp.value)


def score(prior, A, loglik, path) -> float:
    """fp64 log joint log p(y_{1:T}, x_{1:T}) of a given state sequence (Sec. II joint)."""
    lib = _load()
    prior, pp = _f32(prior)
    A, pa = _f32(A)
    loglik, pl = _f32(loglik)
    T, D = loglik.shape
    path = np.ascontiguousarray(path, dtype=np.int32)
    assert path.shape == (T,) and path.min() >= 0 and path.max() < D
    return float(lib.hmm_oracle_score(pp, pa, pl, T, D, path.ctypes.data_as(ctypes.POINTER(ctypes.c_int))))


def max_product(prior, A, loglik):
    """One sequence: the max-product forward/backward recursions (Sec. IV-C) and Theorem 4.
    Returns (maxmarg[T][D] f64 = log p*(x_k) - log max joint weight, path[T] int32, logprob f64)."""
    lib = _load()
    prior, pp = _f32(prior)
    A, pa = _f32(A)
    loglik, pl = _f32(loglik)
    T, D = loglik.shape
    assert prior.shape == (D,) and A.shape == (D, D)
    mm = np.empty((T, D), dtype=np.float64)
    path = np.empty(T, dtype=np.int32)
    lp = ctypes.c_double(0.0)
    rc = lib.hmm_oracle_max_product(pp, pa, pl, T, D, mm.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                    path.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), ctypes.byref(lp))
    if rc != 0:
        raise RuntimeError("hmm_oracle_max_product failed")
    return mm, path, float(lp.value)


def transition_counts(prior, A, loglik):
    """One sequence: expected transition counts sum_k p(x_{k-1}=i, x_k=j | y_{1:T}) (the Baum-Welch
    expectation step's statistic for the transition matrix).  Returns counts[D][D] f64."""
    lib = _load()
    prior, pp = _f32(prior)
    A, pa = _f32(A)
    loglik, pl = _f32(loglik)
    T, D = loglik.shape
    assert prior.shape == (D,) and A.shape == (D, D)
    counts = np.empty((D, D), dtype=np.float64)
    rc = lib.hmm_oracle_transition_counts(pp, pa, pl, T, D, counts.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise RuntimeError("hmm_oracle_transition_counts failed")
    return counts


def block_element(A, loglik, max_product: bool = False):
    """Element of a block of consecutive steps (Sec. V-B): W(i,j) = joint weight of the block's
    observations and its last state j given its first state i (sum or max over the states between).
    Returns (element[D][D] f64, log_scale f64): sum-product element = W / max W, log_scale = log max W;
    max-product element = log W - max, log_scale = max log W."""
    lib = _load()
    A, pa = _f32(A)
    loglik, pl = _f32(loglik)
    T, D = loglik.shape
    assert A.shape == (D, D)
    el = np.empty((D, D), dtype=np.float64)
    ls = ctypes.c_double(0.0)
    rc = lib.hmm_oracle_block_element(pa, pl, T, D, 1 if max_product else 0,
                                      el.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), ctypes.byref(ls))
    if rc != 0:
        raise RuntimeError("hmm_oracle_block_element failed")
    return el, float(ls.value)


def block_carries(prior, A, elements, log_scales, max_product: bool = False):
    """Carries between the S blocks of one sequence from their elements (float32 elements[S][D][D],
    float64 log_scales[S]).  Returns (carry_rows[S][D], lookahead_rows[S][D], total): the
    log-domain pseudo-observation rows to put in front of / behind each block, and log Z
    (sum-product) or the log of the largest joint weight (max-product)."""
    lib = _load()
    prior, pp = _f32(prior)
    A, pa = _f32(A)
    elements, pe = _f32(elements)
    S, D, _ = elements.shape
    log_scales = np.ascontiguousarray(log_scales, dtype=np.float64)
    assert prior.shape == (D,) and A.shape == (D, D) and log_scales.shape == (S,)
    cr = np.empty((S, D), dtype=np.float64)
    lr = np.empty((S, D), dtype=np.float64)
    tot = ctypes.c_double(0.0)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = lib.hmm_oracle_block_carries(pp, pa, pe, log_scales.ctypes.data_as(dp), S, D, 1 if max_product else 0,
                                      cr.ctypes.data_as(dp), lr.ctypes.data_as(dp), ctypes.byref(tot))
    if rc != 0:
        raise RuntimeError("hmm_oracle_block_carries failed")
    return cr, lr, float(tot.value)


def transition_counts_batch(prior, A, loglik, shared_model: bool):
    B = loglik.shape[0]
    return np.stack([transition_counts(prior[0 if shared_model else b], A[0 if shared_model else b], loglik[b])
                     for b in range(B)])


def max_product_batch(prior, A, loglik, shared_model: bool):
    B = loglik.shape[0]
    outs = [max_product(prior[0 if shared_model else b], A[0 if shared_model else b], loglik[b]) for b in range(B)]
    return np.stack([o[0] for o in outs]), np.stack([o[1] for o in outs]), np.array([o[2] for o in outs])


def smooth_batch(prior, A, loglik, shared_model: bool, want_filtered: bool = True):
    """Batched convenience wrapper: prior[Bm][D], A[Bm][D][D], loglik[B][T][D]."""
    B = loglik.shape[0]
    outs = [smooth(prior[0 if shared_model else b], A[0 if shared_model else b], loglik[b], want_filtered)
            for b in range(B)]
    marg = np.stack([o[0] for o in outs])
    filt = np.stack([o[1] for o in outs]) if want_filtered else None
    return marg, filt, np.array([o[2] for o in outs])


def viterbi_batch(prior, A, loglik, shared_model: bool):
    B = loglik.shape[0]
    outs = [viterbi(prior[0 if shared_model else b], A[0 if shared_model else b], loglik[b]) for b in range(B)]
    return np.stack([o[0] for o in outs]), np.array([o[1] for o in outs])
