"""Brute-force definitions -- TEST INFRASTRUCTURE ONLY.

Evaluates the defining sums and maxima of Sec. II literally, by enumerating all
D**T state sequences: the joint weight psi_1(x_1) * prod_k psi_k(x_{k-1}, x_k),
the partition function Z (sum of all weights), the marginals p(x_k) (sum over
all other variables, divided by Z), the max-marginals p*(x_k), and the MAP
sequence of Sec. IV-A (argmax of the joint).  fp64, probability domain; only for
tiny D and T.  Independent of every other implementation in the repository.
"""
from __future__ import annotations

import itertools

import numpy as np


def enumerate_weights(prior, A, loglik):
    prior = np.asarray(prior, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    lik = np.exp(np.asarray(loglik, dtype=np.float64))      # p(y_k | x_k)
    T, D = lik.shape
    seqs = np.array(list(itertools.product(range(D), repeat=T)), dtype=np.int64)   # [D**T][T]
    w = prior[seqs[:, 0]] * lik[0, seqs[:, 0]]              # psi_1(x_1)
    for k in range(1, T):
        w = w * A[seqs[:, k - 1], seqs[:, k]] * lik[k, seqs[:, k]]   # psi_k(x_{k-1}, x_k)
    return seqs, w


def marginals_and_loglik(prior, A, loglik):
    """Returns (marginals[T][D], log Z)."""
    seqs, w = enumerate_weights(prior, A, loglik)
    T = seqs.shape[1]
    D = np.asarray(prior).shape[0]
    Z = w.sum()
    marg = np.zeros((T, D))
    for k in range(T):
        for j in range(D):
            marg[k, j] = w[seqs[:, k] == j].sum() / Z
    return marg, float(np.log(Z))


def filtered(prior, A, loglik):
    """p(x_k | y_{1:k}) for every k: the marginal of the last variable of the
    length-k prefix problem."""
    T = np.asarray(loglik).shape[0]
    return np.stack([marginals_and_loglik(prior, A, loglik[:k + 1])[0][k] for k in range(T)])


def map_sequence(prior, A, loglik):
    """Returns (all maximising sequences [n][T], log of the maximal joint weight)."""
    seqs, w = enumerate_weights(prior, A, loglik)
    best = w.max()
    return seqs[w == best], float(np.log(best))


def max_marginals(prior, A, loglik):
    """p*(x_k) = max over all other variables of the joint weight (Sec. II)."""
    seqs, w = enumerate_weights(prior, A, loglik)
    T = seqs.shape[1]
    D = np.asarray(prior).shape[0]
    out = np.zeros((T, D))
    for k in range(T):
        for j in range(D):
            sel = w[seqs[:, k] == j]
            out[k, j] = sel.max() if sel.size else 0.0
    return out


def transition_counts(prior, A, loglik):
    """sum_k p(x_{k-1} = i, x_k = j | y_{1:T}) straight from the joint of Sec. II."""
    seqs, w = enumerate_weights(prior, A, loglik)
    T = seqs.shape[1]
    D = np.asarray(prior).shape[0]
    Z = w.sum()
    out = np.zeros((D, D))
    for k in range(1, T):
        np.add.at(out, (seqs[:, k - 1], seqs[:, k]), w / Z)
    return out


def block_element(A, loglik, max_product=False):
    """Element of a block of consecutive steps (Sec. V-B) from the definition: W(i, j) = the sum (or
    the maximum) over all state sequences of the block with first state i and last state j of
    e_1(x_1) prod_{k>=2} A(x_{k-1}, x_k) e_k(x_k) -- no transition into the first step."""
    D = np.asarray(A).shape[0]
    seqs, w = enumerate_weights(np.ones(D), A, loglik)
    W = np.zeros((D, D))
    for i in range(D):
        for j in range(D):
            sel = w[(seqs[:, 0] == i) & (seqs[:, -1] == j)]
            W[i, j] = (sel.max() if sel.size else 0.0) if max_product else sel.sum()
    return W
