"""The paper's element/operator/scan formulation (fp64, CPU) against the classical
recursions and the brute-force definitions: Lemma 1 / Definition 5
associativity, Theorems 1-2 (scan prefixes are the forward/backward
potentials), Algorithm 3 marginals, Algorithm 5 with Theorem 4's argmax."""
import numpy as np
import pytest

import oracle
from oracle import brute_force as bf
from oracle import scan_formulation as sf
from paper_2102_05743_amd import workloads as wl


def _value(a):
    return a[0] * np.exp(a[1])


def test_sum_product_operator_is_associative_in_value():
    p = wl.random_problem(4, 6, seed=30)
    elems, last = sf.sum_product_elements(p.prior[0], p.A[0], p.loglik[0])
    a, b, c = elems[0], elems[2], elems[4]          # includes the rank-one first element
    left = sf.sp_combine(sf.sp_combine(a, b), c)
    right = sf.sp_combine(a, sf.sp_combine(b, c))
    assert np.abs(_value(left) - _value(right)).max() < 1e-15
    ident = sf.sp_identity(4)
    assert np.abs(_value(sf.sp_combine(ident, b)) - _value(b)).max() < 1e-16
    assert np.abs(_value(sf.sp_combine(b, ident)) - _value(b)).max() < 1e-16
    assert np.abs(_value(sf.sp_combine(c, last)) - _value(c).sum(1, keepdims=True)).max() < 1e-15


def test_max_product_operator_is_associative():
    p = wl.random_problem(5, 6, seed=31, zero_frac=0.3)
    elems, last = sf.max_product_elements(p.prior[0], p.A[0], p.loglik[0])
    a, b, c = elems[1], elems[2], elems[3]
    l = sf.mp_combine(sf.mp_combine(a, b), c)
    r = sf.mp_combine(a, sf.mp_combine(b, c))
    fin = np.isfinite(l)
    assert (fin == np.isfinite(r)).all() and np.abs(l[fin] - r[fin]).max() < 1e-13
    I = sf.mp_identity(5)
    assert (sf.mp_combine(I, b) == b).all() and (sf.mp_combine(b, I) == b).all()


def test_parallel_scan_equals_sequential_fold_for_a_noncommutative_operator():
    rng = np.random.default_rng(5)
    for T in (1, 2, 3, 5, 8, 13, 16, 33):
        mats = [rng.normal(size=(3, 3)) for _ in range(T)]
        out = sf.parallel_scan(mats, lambda x, y: x @ y, np.eye(3))
        acc = np.eye(3)
        for k in range(T):
            acc = acc @ mats[k]
            assert np.abs(out[k] - acc).max() < 1e-9 * max(1.0, np.abs(acc).max())
        rev = sf.reversed_parallel_scan(mats, lambda x, y: x @ y, np.eye(3))
        acc = np.eye(3)
        for k in range(T - 1, -1, -1):
            acc = mats[k] @ acc
            assert np.abs(rev[k] - acc).max() < 1e-9 * max(1.0, np.abs(acc).max())


@pytest.mark.parametrize("D,T,seed", [(3, 8, 40), (2, 11, 41), (4, 64, 42), (4, 100, 43), (7, 37, 44)])
def test_algorithm3_equals_classical_smoother(D, T, seed):
    p = wl.random_problem(D, T, seed=seed)
    prior, A, ll = p.prior[0], p.A[0], p.loglik[0]
    marg, filt, logZ, logZk = sf.parallel_sum_product(prior, A, ll)
    m0, f0, L0 = oracle.smooth(prior, A, ll)
    assert np.abs(marg - m0).max() < 1e-12
    assert np.abs(filt - f0).max() < 1e-12
    assert abs(logZ - L0) < 1e-10 * max(1.0, abs(L0))
    assert np.abs(logZk - L0).max() < 1e-10 * max(1.0, abs(L0))     # Z_k does not depend on k
    if D ** T <= 7000:
        mb, Lb = bf.marginals_and_loglik(prior, A, ll)
        assert np.abs(marg - mb).max() < 1e-12 and abs(logZ - Lb) < 1e-12 * max(1, abs(Lb))


@pytest.mark.parametrize("D,T,seed", [(3, 8, 50), (2, 11, 51), (4, 64, 52), (4, 100, 53), (7, 37, 54)])
def test_algorithm5_equals_classical_viterbi(D, T, seed):
    p = wl.random_problem(D, T, seed=seed)
    prior, A, ll = p.prior[0], p.A[0], p.loglik[0]
    path, lp, tab = sf.parallel_max_product(prior, A, ll)
    p0, lp0 = oracle.viterbi(prior, A, ll)
    assert (path == p0).all()
    assert abs(lp - lp0) < 1e-10 * max(1.0, abs(lp0))
    assert np.abs(tab.max(1) - lp0).max() < 1e-10 * max(1.0, abs(lp0))   # max_k-independent optimum
    if D ** T <= 7000:
        mm = bf.max_marginals(prior, A, ll)
        with np.errstate(divide="ignore"):
            assert np.abs(tab - np.log(mm)).max() < 1e-11
    # the sequential max-product recursions (the oracle of hmm_max_product) give the same table
    mm_o, path_o, lp_o = oracle.max_product(prior, A, ll)
    assert np.abs((tab - lp) - mm_o).max() < 1e-9 and (path_o == path).all() and abs(lp_o - lp) < 1e-10 * max(1.0, abs(lp))


def test_gilbert_elliott_long_sequence():
    p = wl.gilbert_elliott(T=4096)
    prior, A, ll = p.prior[0], p.A[0], p.loglik[0]
    marg, filt, logZ, _ = sf.parallel_sum_product(prior, A, ll)
    m0, f0, L0 = oracle.smooth(prior, A, ll)
    assert np.abs(marg - m0).max() < 1e-11 and abs(logZ - L0) < 1e-9 * abs(L0)
    path, lp, tab = sf.parallel_max_product(prior, A, ll)
    p0, lp0 = oracle.viterbi(prior, A, ll)
    assert abs(lp - lp0) < 1e-9 * abs(lp0)
    # binary evidence allows exact ties between different sequences; where the per-step argmax is
    # unambiguous (gap to the runner-up above rounding) it must equal the classical path
    srt = np.sort(tab, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 1e-7
    assert clear.mean() > 0.9 and (path[clear] == p0[clear]).all()
