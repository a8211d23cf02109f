"""Pins for the oracle's block-wise elements and block carries (Sec. V-B), no GPU: enumeration of the
definition, closed forms, the classical recursions they must reduce to, and the property that matters
to a user -- a sequence processed block by block gives the whole sequence's results.
"""
import numpy as np
import pytest

import oracle
from oracle import brute_force as bf
from paper_2102_05743_amd import workloads as wl


def _tiny(D, T, seed, zero_frac=0.0):
    p = wl.random_problem(D, T, seed=seed, zero_frac=zero_frac)
    return p.prior[0], p.A[0], p.loglik[0]


def _true_element(el, ls, mp):
    return el + ls if mp else el * np.exp(ls)


@pytest.mark.parametrize("mp", [False, True])
@pytest.mark.parametrize("D,T,seed,zf", [(3, 6, 0, 0.0), (3, 6, 1, 0.3), (2, 1, 2, 0.0), (2, 2, 3, 0.0), (4, 4, 4, 0.25),
                                         (2, 10, 5, 0.0)])
def test_block_element_matches_enumeration(D, T, seed, zf, mp):
    _, A, ll = _tiny(D, T, seed, zf)
    el, ls = oracle.block_element(A, ll, mp)
    W = bf.block_element(A, ll, mp)
    if mp:
        with np.errstate(divide="ignore"):
            ref = np.log(W)
        got = _true_element(el, ls, True)
        fin = np.isfinite(ref)
        assert (np.isfinite(got) == fin).all()
        assert np.abs(got[fin] - ref[fin]).max() < 1e-12 * max(1.0, np.abs(ref[fin]).max())
        assert el.max() == 0.0
    else:
        assert np.abs(_true_element(el, ls, False) - W).max() < 1e-12 * W.max()
        assert el.max() == 1.0


@pytest.mark.parametrize("mp", [False, True])
def test_single_step_block_is_the_diagonal_of_its_emission_factors(mp):
    _, A, ll = _tiny(4, 1, 7)
    el, ls = oracle.block_element(A, ll, mp)
    got = _true_element(el, ls, mp)
    ref = np.diag(np.exp(ll[0].astype(np.float64)))
    if mp:
        assert np.allclose(np.diag(got), ll[0]) and np.isneginf(got[~np.eye(4, dtype=bool)]).all()
    else:
        assert np.allclose(got, ref, rtol=1e-12, atol=0)


def test_identity_transitions_give_the_product_of_the_emission_factors():
    _, _, ll = _tiny(3, 9, 8)
    el, ls = oracle.block_element(np.eye(3, dtype=np.float32), ll, False)
    ref = np.diag(np.exp(ll.astype(np.float64).sum(axis=0)))
    assert np.allclose(_true_element(el, ls, False), ref, rtol=1e-12, atol=0)


def test_identical_rows_closed_form():
    # A(i, j) = a(j): W(i, j) = e_1(i) * prod_{1<k<T} (sum_x a(x) e_k(x)) * a(j) e_T(j)
    rng = np.random.default_rng(9)
    a = rng.dirichlet(np.ones(4)).astype(np.float32)
    A = np.tile(a, (4, 1))
    _, _, ll = _tiny(4, 7, 10)
    e = np.exp(ll.astype(np.float64))
    ref = np.outer(e[0], a.astype(np.float64) * e[-1]) * np.prod((e[1:-1] * a.astype(np.float64)).sum(axis=1))
    el, ls = oracle.block_element(A, ll, False)
    assert np.allclose(_true_element(el, ls, False), ref, rtol=1e-12, atol=0)


@pytest.mark.parametrize("mp", [False, True])
def test_adjacent_blocks_combine_through_one_transition(mp):
    # W_{1..T} = W_{1..m} (x) A (x) W_{m+1..T} under the operator of Definition 3 / Definition 5
    _, A, ll = _tiny(3, 11, 11)
    full = _true_element(*oracle.block_element(A, ll, mp), mp)
    for m in (1, 4, 10):
        a = _true_element(*oracle.block_element(A, ll[:m], mp), mp)
        b = _true_element(*oracle.block_element(A, ll[m:], mp), mp)
        if mp:
            with np.errstate(divide="ignore"):
                lA = np.log(A.astype(np.float64))
            ab = (a[:, :, None] + lA[None, :, :]).max(axis=1)
            comb = (ab[:, :, None] + b[None, :, :]).max(axis=1)
            assert np.allclose(comb, full, rtol=1e-12, atol=1e-12)
        else:
            assert np.allclose(a @ A.astype(np.float64) @ b, full, rtol=1e-12, atol=0)


def test_block_element_contracts_to_the_evidence_and_the_best_weight():
    prior, A, ll = _tiny(4, 300, 12)
    el, ls = oracle.block_element(A, ll, False)
    _, _, L = oracle.smooth(prior, A, ll)
    assert abs(np.log(prior.astype(np.float64) @ el @ np.ones(4)) + ls - L) < 1e-10 * abs(L)
    el, ls = oracle.block_element(A, ll, True)
    _, lp = oracle.viterbi(prior, A, ll)
    assert abs((np.log(prior.astype(np.float64))[:, None] + el).max() + ls - lp) < 1e-10 * abs(lp)


def _blocks(ll, cuts):
    edges = [0] + list(cuts) + [ll.shape[0]]
    return [ll[a:b] for a, b in zip(edges[:-1], edges[1:])]


def _carries(prior, A, blocks, mp):
    els = [oracle.block_element(A, b, mp) for b in blocks]
    E = np.stack([e[0] for e in els]).astype(np.float32)
    return oracle.block_carries(prior, A, E, np.array([e[1] for e in els]), mp)


def _framed(blocks, cr, lr, s):
    """[carry; block; lookahead] rows of block s, the prior to use with them, and the slice of real steps."""
    rows = []
    if s > 0:
        rows.append(cr[s][None, :])
    rows.append(blocks[s].astype(np.float64))
    if s + 1 < len(blocks):
        rows.append(lr[s][None, :])
    lo = 1 if s > 0 else 0
    return np.concatenate(rows).astype(np.float32), slice(lo, lo + blocks[s].shape[0])


@pytest.mark.parametrize("D,T,cuts,seed,zf", [(3, 9, (3, 6), 20, 0.0), (2, 10, (1, 2, 9), 21, 0.0), (3, 8, (4,), 22, 0.3),
                                              (4, 6, (2, 4), 23, 0.0)])
def test_blockwise_smoothing_reproduces_the_enumerated_marginals(D, T, cuts, seed, zf):
    prior, A, ll = _tiny(D, T, seed, zf)
    marg_bf, logZ_bf = bf.marginals_and_loglik(prior, A, ll)
    filt_bf = bf.filtered(prior, A, ll)
    blocks = _blocks(ll, cuts)
    cr, lr, total = _carries(prior, A, blocks, False)
    assert abs(total - logZ_bf) < 1e-6 * max(1.0, abs(logZ_bf))     # the elements went through float32
    t0 = 0
    for s, b in enumerate(blocks):
        rows, sl = _framed(blocks, cr, lr, s)
        pr = prior if s == 0 else np.ones(D, dtype=np.float32)
        marg, filt, _ = oracle.smooth(pr, A, rows)
        assert np.abs(marg[sl] - marg_bf[t0:t0 + b.shape[0]]).max() < 1e-6
        assert np.abs(filt[sl] - filt_bf[t0:t0 + b.shape[0]]).max() < 1e-6
        t0 += b.shape[0]


@pytest.mark.parametrize("D,T,cuts,seed", [(3, 9, (3, 6), 30), (2, 10, (1, 2, 9), 31), (4, 6, (2, 4), 32)])
def test_blockwise_decoding_reproduces_the_enumerated_map_sequence(D, T, cuts, seed):
    prior, A, ll = _tiny(D, T, seed)
    best, best_lp = bf.map_sequence(prior, A, ll)
    assert best.shape[0] == 1
    mm_bf = bf.max_marginals(prior, A, ll)
    blocks = _blocks(ll, cuts)
    cr, lr, total = _carries(prior, A, blocks, True)
    assert abs(total - best_lp) < 1e-6 * max(1.0, abs(best_lp))
    t0 = 0
    for s, b in enumerate(blocks):
        rows, sl = _framed(blocks, cr, lr, s)
        pr = prior if s == 0 else np.ones(D, dtype=np.float32)
        path, _ = oracle.viterbi(pr, A, rows)
        assert (path[sl] == best[0][t0:t0 + b.shape[0]]).all()
        mm, _, _ = oracle.max_product(pr, A, rows)
        ref = np.log(mm_bf[t0:t0 + b.shape[0]]) - best_lp
        assert np.abs(mm[sl] - ref).max() < 1e-5
        t0 += b.shape[0]


def test_block_carries_on_a_long_sequence_match_the_one_shot_recursions():
    p = wl.config2(T=6000)
    prior, A, ll = p.prior[0], p.A[0], p.loglik[0]
    marg, filt, L = oracle.smooth(prior, A, ll)
    blocks = _blocks(ll, (1000, 1001, 4500))
    cr, lr, total = _carries(prior, A, blocks, False)
    assert abs(total - L) < 1e-6 * abs(L)
    # carry rows are the logarithms of the filtering distribution at the last step of the previous block
    assert np.abs(np.exp(cr[1]) - filt[999]).max() < 1e-6
    assert np.abs(np.exp(cr[3]) - filt[4499]).max() < 1e-6
    rows, sl = _framed(blocks, cr, lr, 2)
    m2, _, _ = oracle.smooth(np.ones(4, dtype=np.float32), A, rows)
    assert np.abs(m2[sl] - marg[1001:4500]).max() < 1e-6
