"""Pins for the CPU oracle (no GPU): the oracle is checked against things other
than itself -- the literal brute-force definitions, closed forms, library
routines on special cases, and invariants -- before anything is compared to it.
"""
import numpy as np
import pytest
from scipy.special import logsumexp

import oracle
from oracle import brute_force as bf
from paper_2102_05743_amd import workloads as wl


def _tiny(D, T, seed, zero_frac=0.0):
    p = wl.random_problem(D, T, seed=seed, zero_frac=zero_frac)
    return p.prior[0], p.A[0], p.loglik[0]


# ------------------------------------------------------------------ brute force (definitions of Sec. II)
@pytest.mark.parametrize("D,T,seed,zf", [(3, 8, 0, 0.0), (3, 8, 1, 0.3), (2, 1, 2, 0.0), (2, 2, 3, 0.0),
                                         (2, 5, 4, 0.0), (2, 12, 5, 0.0), (4, 5, 6, 0.25), (5, 4, 7, 0.0)])
def test_smoother_matches_enumeration(D, T, seed, zf):
    prior, A, ll = _tiny(D, T, seed, zf)
    marg, filt, L = oracle.smooth(prior, A, ll)
    marg_bf, logZ_bf = bf.marginals_and_loglik(prior, A, ll)
    assert np.abs(marg - marg_bf).max() < 1e-12
    assert abs(L - logZ_bf) < 1e-12 * max(1.0, abs(logZ_bf))
    assert np.abs(filt - bf.filtered(prior, A, ll)).max() < 1e-12


@pytest.mark.parametrize("D,T,seed,zf", [(3, 8, 10, 0.0), (3, 8, 11, 0.3), (2, 1, 12, 0.0), (2, 12, 13, 0.0),
                                         (4, 5, 14, 0.25), (5, 4, 15, 0.0), (2, 7, 16, 0.0)])
def test_viterbi_matches_enumeration(D, T, seed, zf):
    prior, A, ll = _tiny(D, T, seed, zf)
    path, lp = oracle.viterbi(prior, A, ll)
    best_seqs, best_lp = bf.map_sequence(prior, A, ll)
    assert abs(lp - best_lp) < 1e-12 * max(1.0, abs(best_lp))
    assert best_seqs.shape[0] == 1, "random inputs should have a unique MAP sequence"
    assert (path == best_seqs[0]).all()
    assert abs(oracle.score(prior, A, ll, path) - best_lp) < 1e-12 * max(1.0, abs(best_lp))


def test_score_matches_enumerated_weight():
    prior, A, ll = _tiny(3, 6, 20)
    seqs, w = bf.enumerate_weights(prior, A, ll)
    for idx in (0, 17, 100, 500, 728):
        assert abs(oracle.score(prior, A, ll, seqs[idx]) - np.log(w[idx])) < 1e-12


def test_asymmetric_transition_orientation():
    """A[i][j] is row = from, column = to: a deterministic cycle 0->1->2->0."""
    A = np.array([[0, 1, 0], [0, 0, 1], [1, 0, 0]], np.float32)
    prior = np.array([1, 0, 0], np.float32)
    ll = np.zeros((7, 3), np.float32)
    marg, filt, L = oracle.smooth(prior, A, ll)
    expect = np.eye(3)[[0, 1, 2, 0, 1, 2, 0]]
    assert np.abs(marg - expect).max() < 1e-15 and abs(L) < 1e-15
    path, lp = oracle.viterbi(prior, A, ll)
    assert (path == [0, 1, 2, 0, 1, 2, 0]).all() and abs(lp) < 1e-15


# ------------------------------------------------------------------ closed forms
def test_identical_rows_is_independent_mixture():
    rng = np.random.default_rng(1)
    D, T = 5, 200
    r = rng.dirichlet(np.ones(D)).astype(np.float32)
    A = np.tile(r, (D, 1))
    prior = rng.dirichlet(np.ones(D)).astype(np.float32)
    ll = (-3.0 * rng.random((T, D))).astype(np.float32)
    marg, filt, L = oracle.smooth(prior, A, ll)
    w = np.vstack([prior.astype(np.float64)[None], np.tile(r.astype(np.float64), (T - 1, 1))])
    post = w * np.exp(ll.astype(np.float64))
    assert np.abs(marg - post / post.sum(1, keepdims=True)).max() < 1e-13
    assert np.abs(filt - marg).max() < 1e-13
    assert abs(L - np.log(post.sum(1)).sum()) < 1e-10
    path, lp = oracle.viterbi(prior, A, ll)
    assert (path == post.argmax(1)).all()
    assert abs(lp - np.log(post.max(1)).sum()) < 1e-10


@pytest.mark.parametrize("perm", [None, [2, 0, 3, 1]])
def test_identity_and_permutation_transitions(perm):
    rng = np.random.default_rng(2)
    D, T = 4, 60
    P = np.eye(D, dtype=np.float32) if perm is None else np.eye(D, dtype=np.float32)[perm]
    prior = rng.dirichlet(np.ones(D)).astype(np.float32)
    ll = (-2.0 * rng.random((T, D))).astype(np.float32)
    nxt = P.argmax(1)
    # trajectory started in state j is deterministic
    traj = np.empty((D, T), dtype=np.int64)
    for j in range(D):
        s = j
        for k in range(T):
            traj[j, k] = s
            s = nxt[s]
    logw = np.log(prior.astype(np.float64)) + np.array(
        [ll[np.arange(T), traj[j]].astype(np.float64).sum() for j in range(D)])
    marg, filt, L = oracle.smooth(prior, P, ll)
    assert abs(L - logsumexp(logw)) < 1e-11
    post0 = np.exp(logw - logsumexp(logw))
    expect = np.zeros((T, D))
    for j in range(D):
        expect[np.arange(T), traj[j]] += post0[j]
    assert np.abs(marg - expect).max() < 1e-13
    path, lp = oracle.viterbi(prior, P, ll)
    assert (path == traj[logw.argmax()]).all()
    assert abs(lp - logw.max()) < 1e-11


def test_constant_evidence_is_matrix_power():
    rng = np.random.default_rng(3)
    D, T, c = 6, 40, -1.25
    A = rng.dirichlet(np.ones(D), size=D).astype(np.float32)
    prior = rng.dirichlet(np.ones(D)).astype(np.float32)
    ll = np.full((T, D), c, np.float32)
    marg, filt, L = oracle.smooth(prior, A, ll)
    A64, p64 = A.astype(np.float64), prior.astype(np.float64)
    rs = A64.sum(1)            # float32 rows do not sum to exactly 1: track the mass
    for k in range(T):
        v = p64 @ np.linalg.matrix_power(A64, k)
        assert np.abs(filt[k] - v / v.sum()).max() < 1e-13
    total = p64 @ np.linalg.matrix_power(A64, T - 1)
    assert abs(L - (T * c + np.log(total.sum()))) < 1e-11
    # with exactly stochastic A the smoother equals the filter; here within float32 row error
    assert np.abs(marg - filt).max() < 1e-5 and abs(rs - 1).max() < 1e-6


def test_single_state_and_single_step():
    ll = np.array([[-0.5], [-1.5], [-0.25]], np.float32)
    marg, filt, L = oracle.smooth(np.ones(1, np.float32), np.ones((1, 1), np.float32), ll)
    assert (marg == 1).all() and (filt == 1).all() and abs(L + 2.25) < 1e-15
    path, lp = oracle.viterbi(np.ones(1, np.float32), np.ones((1, 1), np.float32), ll)
    assert (path == 0).all() and abs(lp + 2.25) < 1e-15
    prior = np.array([0.2, 0.5, 0.3], np.float32)
    ll1 = np.array([[-1.0, -2.0, -0.1]], np.float32)
    A = np.full((3, 3), np.nan, np.float32)          # T = 1 must not touch the transition matrix
    marg, filt, L = oracle.smooth(prior, A, ll1)
    w = prior.astype(np.float64) * np.exp(ll1[0].astype(np.float64))
    assert np.abs(marg[0] - w / w.sum()).max() < 1e-15 and abs(L - np.log(w.sum())) < 1e-15
    path, lp = oracle.viterbi(prior, np.ones((3, 3), np.float32), ll1)
    assert path[0] == w.argmax() and abs(lp - np.log(w.max())) < 1e-15


# ------------------------------------------------------------------ invariants
@pytest.mark.parametrize("gen", [lambda: wl.config1(), lambda: wl.config2(T=5000), lambda: wl.gilbert_elliott(T=3000),
                                 lambda: wl.config3(T=500), lambda: wl.config5(T=300)])
def test_invariants(gen):
    p = gen()
    prior, A, ll = p.prior[0], p.A[0], p.loglik[0]
    marg, filt, L = oracle.smooth(prior, A, ll)
    assert np.abs(marg.sum(1) - 1).max() < 1e-12
    assert np.abs(filt.sum(1) - 1).max() < 1e-12
    assert np.abs(marg[-1] - filt[-1]).max() < 1e-15          # psi^b_{T,T} = 1
    assert (marg >= 0).all() and np.isfinite(L)
    # a per-step shift of the log-likelihoods moves log Z by the total shift and nothing else
    rng = np.random.default_rng(0)
    c = (rng.integers(-16, 17, size=(p.T, 1)) * 0.25).astype(np.float32)
    ll2 = ll + c
    marg2, _, L2 = oracle.smooth(prior, A, ll2)
    assert np.abs(marg2 - marg).max() < 1e-5
    assert abs((L2 - L) - float(c.astype(np.float64).sum())) < 1e-6 * p.T
    path, lp = oracle.viterbi(prior, A, ll)
    assert abs(oracle.score(prior, A, ll, path) - lp) < 1e-9 * abs(lp)
    assert lp <= L + 1e-9
    # the sampled hidden sequence is a valid sequence, so it cannot beat the MAP one
    assert oracle.score(prior, A, ll, p.states[0]) <= lp + 1e-9


def test_log_evidence_chains_over_a_split():
    """log p(y_{1:T}) = log p(y_{1:k}) + log p(y_{k+1:T} | y_{1:k}); the second term is the
    evidence of the suffix problem whose prior is the one-step prediction f_k A."""
    p = wl.gilbert_elliott(T=20000)
    prior, A, ll = p.prior[0], p.A[0], p.loglik[0]
    _, filt, L = oracle.smooth(prior, A, ll)
    k = 7777
    _, _, L1 = oracle.smooth(prior, A, ll[:k])
    pred = filt[k - 1] @ A.astype(np.float64)
    # feed the fp64 prediction through a log-likelihood offset so float32 rounding of the prior cancels
    pred32 = pred.astype(np.float32)
    corr = np.log(pred) - np.log(pred32.astype(np.float64))
    assert np.abs(corr).max() < 1e-6
    _, _, L2 = oracle.smooth(pred32, A, ll[k:])
    assert abs(L - (L1 + L2)) < 1e-5
    assert abs(L - (L1 + L2)) / abs(L) < 1e-8


def test_gilbert_elliott_matrices_match_the_printed_model():
    rows = [r.split() for r in open(__file__.rsplit("/", 1)[0] + "/golden/gilbert_elliott_model.txt")
            if r.strip() and not r.startswith("#")]
    Pi = np.array(rows[1:5], dtype=np.float64)
    O = np.array(rows[6:10], dtype=np.float64)
    Pi_g, O_g = wl.gilbert_elliott_matrices()
    assert np.abs(Pi - Pi_g).max() < 1e-15 and np.abs(O - O_g).max() < 1e-15
    assert np.abs(Pi.sum(1) - 1).max() < 1e-15 and np.abs(O.sum(1) - 1).max() < 1e-15


def test_ties_resolve_to_the_lowest_state():
    """The paper assumes a unique MAP sequence; with every sequence tied the reading
    taken here (lowest index at every argmax) must give the all-zero path."""
    D, T = 3, 9
    prior = np.full(D, 1.0 / D, np.float32)
    A = np.full((D, D), 1.0 / D, np.float32)
    ll = np.zeros((T, D), np.float32)
    path, lp = oracle.viterbi(prior, A, ll)
    assert (path == 0).all()
    assert abs(lp - T * np.log(np.float64(np.float32(1.0 / 3)))) < 1e-12
    seqs, best = bf.map_sequence(prior, A, ll)
    assert seqs.shape[0] == D ** T and abs(best - lp) < 1e-12


# ------------------------------------------------------------------ max-product forward/backward (Sec. IV-C, Theorem 4)
@pytest.mark.parametrize("D,T,seed,zf", [(3, 8, 30, 0.0), (3, 8, 31, 0.3), (2, 1, 32, 0.0), (2, 12, 33, 0.0),
                                         (4, 5, 34, 0.25), (5, 4, 35, 0.0), (2, 2, 36, 0.0)])
def test_max_product_matches_enumeration(D, T, seed, zf):
    """log p*(x_k) (the max-marginal of Sec. II) by enumeration of all D^T sequences."""
    prior, A, ll = _tiny(D, T, seed, zf)
    mm, path, lp = oracle.max_product(prior, A, ll)
    pstar = bf.max_marginals(prior, A, ll)
    best_seqs, best_lp = bf.map_sequence(prior, A, ll)
    assert abs(lp - best_lp) < 1e-12 * max(1.0, abs(best_lp))
    with np.errstate(divide="ignore"):
        want = np.log(pstar) - best_lp
    finite = np.isfinite(want)
    assert (np.isneginf(mm[~finite])).all()
    assert np.abs(mm[finite] - want[finite]).max() < 1e-11
    assert best_seqs.shape[0] == 1 and (path == best_seqs[0]).all()


@pytest.mark.parametrize("gen", [lambda: wl.config1(), lambda: wl.config2(T=5000), lambda: wl.gilbert_elliott(T=3000),
                                 lambda: wl.config3(T=500), lambda: wl.config5(T=300)])
def test_max_product_invariants(gen):
    """max_x [f_k(x) + b_k(x)] is the same for every k (proof of Theorem 4) and equals the Viterbi
    log-probability; on inputs with a unique MAP sequence the per-step maximiser is the Viterbi path."""
    p = gen()
    prior, A, ll = p.prior[0], p.A[0], p.loglik[0]
    mm, path, lp = oracle.max_product(prior, A, ll)
    vpath, vlp = oracle.viterbi(prior, A, ll)
    assert abs(lp - vlp) < 1e-9 * abs(vlp)
    assert np.abs(mm.max(axis=1)).max() < 1e-7          # every step's best max-marginal is the MAP weight
    assert (mm <= 1e-7).all()
    k = np.arange(p.T)
    assert np.abs(mm[k, vpath]).max() < 1e-7            # the Viterbi path runs through maximisers only
    unique = (mm > -1e-9).sum(axis=1) == 1              # steps whose maximiser is unique (all of them without ties;
    assert (path[unique] == vpath[unique]).all()        # the Gilbert-Elliott model has exactly tied sequences)
    if p.name != "GE":
        assert unique.all()
    # the max-marginal of a state dominates the weight of any sequence through it: here the sampled one
    sc = oracle.score(prior, A, ll, p.states[0])
    assert (mm[k, p.states[0]] + lp >= sc - 1e-6).all()


def test_max_product_single_state_and_single_step():
    ll = np.array([[-0.3], [-1.2], [-0.1]], np.float32)
    mm, path, lp = oracle.max_product(np.ones(1, np.float32), np.ones((1, 1), np.float32), ll)
    assert (mm == 0).all() and (path == 0).all() and abs(lp - float(ll.astype(np.float64).sum())) < 1e-12
    prior = np.array([0.2, 0.5, 0.3], np.float32)
    ll1 = np.array([[-1.0, -2.0, -0.5]], np.float32)
    mm, path, lp = oracle.max_product(prior, np.full((3, 3), 1 / 3, np.float32), ll1)
    w = np.log(prior.astype(np.float64)) + ll1[0]
    assert path[0] == w.argmax() and abs(lp - w.max()) < 1e-15 and np.abs(mm[0] - (w - w.max())).max() < 1e-15


# ------------------------------------------------------------------ expected transition counts (Sec. V-C, E-step)
@pytest.mark.parametrize("D,T,seed,zf", [(3, 8, 40, 0.0), (3, 8, 41, 0.3), (2, 1, 42, 0.0), (2, 2, 43, 0.0),
                                         (2, 12, 44, 0.0), (4, 5, 45, 0.25), (5, 4, 46, 0.0)])
def test_transition_counts_match_enumeration(D, T, seed, zf):
    prior, A, ll = _tiny(D, T, seed, zf)
    N = oracle.transition_counts(prior, A, ll)
    assert np.abs(N - bf.transition_counts(prior, A, ll)).max() < 1e-12


@pytest.mark.parametrize("gen", [lambda: wl.config1(), lambda: wl.gilbert_elliott(T=3000), lambda: wl.config3(T=400),
                                 lambda: wl.random_problem(6, 700, seed=3, zero_frac=0.4)])
def test_transition_counts_invariants(gen):
    """Row sums are the summed marginals of steps 1..T-1, column sums those of steps 2..T, the total is
    T-1, and a transition the model forbids is never counted."""
    p = gen()
    prior, A, ll = p.prior[0], p.A[0], p.loglik[0]
    N = oracle.transition_counts(prior, A, ll)
    marg, _, _ = oracle.smooth(prior, A, ll)
    assert np.abs(N.sum(axis=1) - marg[:-1].sum(axis=0)).max() < 1e-8 * p.T
    assert np.abs(N.sum(axis=0) - marg[1:].sum(axis=0)).max() < 1e-8 * p.T
    assert abs(N.sum() - (p.T - 1)) < 1e-8 * p.T
    assert (N[A == 0] == 0).all() and (N >= 0).all()


def test_transition_counts_identical_rows_closed_form():
    """With identical transition rows the steps are independent: p(x_{k-1}, x_k | y) = gamma_{k-1} gamma_k^T."""
    rng = np.random.default_rng(9)
    D, T = 4, 60
    r = rng.dirichlet(np.ones(D)).astype(np.float32)
    A = np.tile(r, (D, 1))
    prior = rng.dirichlet(np.ones(D)).astype(np.float32)
    ll = np.log(rng.uniform(0.05, 1.0, size=(T, D))).astype(np.float32)
    N = oracle.transition_counts(prior, A, ll)
    marg, _, _ = oracle.smooth(prior, A, ll)
    want = sum(np.outer(marg[k - 1], marg[k]) for k in range(1, T))
    assert np.abs(N - want).max() < 1e-10
