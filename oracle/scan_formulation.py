"""The paper's parallel formulation in fp64 numpy -- TEST INFRASTRUCTURE ONLY.

Follows the paper's own steps and notation so that it can be checked against it
by eye: elements a_{k-1:k} and the operator (x) of Definition 3, the path-free
max-product elements and operator (v) of Definition 5, the up-sweep / down-sweep
parallel scan of Algorithm 2 (run sequentially here), the reversed scan by the
recipe of Sec. III-B (reverse inputs, reverse outputs, swap the operator's
arguments), and the parallel sum-product / max-product procedures of
Algorithms 3 and 5 with the per-step argmax of Theorem 4.

Two readings the paper leaves open are fixed here:
  * raw products of potentials underflow, so a sum-product element is stored as
    a pair (M, s) standing for M * exp(s) with max(M) = 1; the operator
    multiplies the matrices, renormalises and adds the scales.  The represented
    value is unchanged, so associativity (Lemma 1) still holds in value;
  * the max-product operator acts on logarithms of the potentials (max, +),
    a monotone transform of Definition 5's (max, x).
Algorithm 2 assumes T is a power of two; shorter inputs are padded on the right
with the operator's neutral element.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- operators
def sp_normalise(M, s):
    c = M.max()
    if c > 0.0 and np.isfinite(c):
        return M / c, s + np.log(c)
    return M, s


def sp_combine(a, b):
    """Definition 3: (a_{i:j} (x) a_{j:k})(x_i, x_k) = sum_{x_j} psi_{i,j}(x_i,x_j) psi_{j,k}(x_j,x_k)."""
    return sp_normalise(a[0] @ b[0], a[1] + b[1])


def sp_identity(D):
    return (np.eye(D), 0.0)


def mp_combine(a, b):
    """Definition 5 in the log domain: max_{x_j} [A_{i:j}(x_i,x_j) + A_{j:k}(x_j,x_k)]."""
    return (a[:, :, None] + b[None, :, :]).max(axis=1)


def mp_identity(D):
    I = np.full((D, D), -np.inf)
    np.fill_diagonal(I, 0.0)
    return I


# ----------------------------------------------------------------------------- Algorithm 2
def parallel_scan(elems, op, identity):
    """All-prefix-sums (Definition 1) by Algorithm 2: save the inputs, up-sweep,
    replace the root by the neutral element, down-sweep, final pass a_i (x) b_i.
    Positions are 1-based in the paper; index p here is position p+1."""
    T = len(elems)
    n = 1
    while n < T:
        n *= 2
    a = list(elems) + [identity] * (n - T)
    b = list(a)
    levels = n.bit_length() - 1
    for d in range(levels):                       # up-sweep
        for i in range(0, n, 2 ** (d + 1)):
            j = i + 2 ** d - 1
            k = i + 2 ** (d + 1) - 1
            a[k] = op(a[j], a[k])
    a[n - 1] = identity
    for d in range(levels - 1, -1, -1):           # down-sweep
        for i in range(0, n, 2 ** (d + 1)):
            j = i + 2 ** d - 1
            k = i + 2 ** (d + 1) - 1
            t = a[j]
            a[j] = a[k]
            a[k] = op(a[k], t)
    return [op(a[i], b[i]) for i in range(T)]     # final pass: exclusive prefix (x) own element


def reversed_parallel_scan(elems, op, identity):
    """Reversed all-prefix-sums (Definition 2): reverse the inputs, run the scan
    with the operator's arguments swapped, reverse the outputs."""
    out = parallel_scan(list(elems)[::-1], lambda x, y: op(y, x), identity)
    return out[::-1]


# ----------------------------------------------------------------------------- Algorithm 3
def sum_product_elements(prior, A, loglik):
    """a_{0:1} = psi_1 (a matrix with identical rows: no dependence on x_0),
    a_{k-1:k} = psi_k(x_{k-1},x_k) = A[x_{k-1}][x_k] p(y_k|x_k), a_{T:T+1} = 1."""
    prior = np.asarray(prior, np.float64)
    A = np.asarray(A, np.float64)
    ll = np.asarray(loglik, np.float64)
    T, D = ll.shape
    elems = []
    for k in range(T):
        m = ll[k].max()
        e = np.exp(ll[k] - m)
        if k == 0:
            M = np.tile(prior * e, (D, 1))
        else:
            M = A * e[None, :]
        elems.append(sp_normalise(M, m))
    last = (np.ones((D, D)), 0.0)
    return elems, last


def parallel_sum_product(prior, A, loglik):
    """Algorithm 3.  Returns (marginals[T][D], filtered[T][D], log Z, log Z_k[T])."""
    elems, last = sum_product_elements(prior, A, loglik)
    T = len(elems)
    D = elems[0][0].shape[0]
    fwd = parallel_scan(elems, sp_combine, sp_identity(D))            # a_{0:k}, k = 1..T
    bwd_in = elems[1:] + [last]                                        # a_{k:k+1}, k = 1..T
    bwd = reversed_parallel_scan(bwd_in, sp_combine, sp_identity(D))   # a_{k:T+1}
    marg = np.empty((T, D))
    filt = np.empty((T, D))
    logZk = np.empty(T)
    for k in range(T):
        f = fwd[k][0][0, :]          # psi^f_{1,k}(x_k): any row (x_0 is notational)
        b = bwd[k][0][:, 0]          # psi^b_{k,T}(x_k): any column (x_{T+1} is notational)
        Zk = (f * b).sum()
        marg[k] = f * b / Zk
        filt[k] = f / f.sum()
        logZk[k] = np.log(Zk) + fwd[k][1] + bwd[k][1]
    logZ = np.log(fwd[T - 1][0][0, :].sum()) + fwd[T - 1][1]
    return marg, filt, float(logZ), logZk


# ----------------------------------------------------------------------------- Algorithm 5
def max_product_elements(prior, A, loglik):
    prior = np.asarray(prior, np.float64)
    A = np.asarray(A, np.float64)
    ll = np.asarray(loglik, np.float64)
    T, D = ll.shape
    with np.errstate(divide="ignore"):
        logA = np.log(A)
        logp = np.log(prior)
    elems = [np.tile(logp + ll[0], (D, 1))] + [logA + ll[k][None, :] for k in range(1, T)]
    last = np.zeros((D, D))
    return elems, last


def parallel_max_product(prior, A, loglik):
    """Algorithm 5 with Theorem 4's per-step argmax (lowest index on ties).
    Returns (path[T], log of the maximal joint, max-marginal table[T][D])."""
    elems, last = max_product_elements(prior, A, loglik)
    T = len(elems)
    D = elems[0].shape[0]
    fwd = parallel_scan(elems, mp_combine, mp_identity(D))
    bwd = reversed_parallel_scan(elems[1:] + [last], mp_combine, mp_identity(D))
    tab = np.stack([fwd[k][0, :] + bwd[k][:, 0] for k in range(T)])    # log psi~^f_k + log psi~^b_k
    path = tab.argmax(axis=1).astype(np.int32)
    return path, float(fwd[T - 1][0, :].max()), tab
