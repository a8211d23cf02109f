"""The classical forward-backward recursion (Alg. 1 with per-step scaling) carried out step by step in numpy
float32: what plain single-precision arithmetic can and cannot hold, independently of any scan.  Test-side
helper; the product never sees it."""
import numpy as np

f32 = np.float32


def smooth_f32(prior, A, ll):
    """Marginals and log-likelihood; forward potentials scaled to sum one, backward ones to maximum one."""
    T, D = ll.shape
    A = A.astype(f32)
    m = ll.max(axis=1, keepdims=True)
    e = np.exp((ll - m).astype(f32)).astype(f32)
    F = np.zeros((T, D), f32)
    g = (prior.astype(f32) * e[0]).astype(f32)
    s = g.sum(dtype=f32)
    L = float(m[0, 0]) + float(np.log(np.float64(s)))
    f = (g / s).astype(f32)
    F[0] = f
    for k in range(1, T):
        g = ((f @ A).astype(f32) * e[k]).astype(f32)
        s = g.sum(dtype=f32)
        L += float(m[k, 0]) + float(np.log(np.float64(s)))
        f = (g / s).astype(f32)
        F[k] = f
    G = np.zeros((T, D), f32)
    b = np.ones(D, f32)
    for k in range(T - 1, -1, -1):
        gam = (F[k] * b).astype(f32)
        G[k] = gam / gam.sum(dtype=f32)
        if k > 0:
            r = (A @ (e[k] * b).astype(f32)).astype(f32)
            b = (r / r.max()).astype(f32)
    return G, L


def smooth_f32_lifted(prior, A, ll, bias=50):
    """The same recursion with both potentials held near 2^bias instead of one (exact power-of-two rescalings):
    an entry 2^-126 below a step's largest is then still a normal number.  This is the arithmetic of the
    library's step-by-step repair pass for more than eight states."""
    T, D = ll.shape
    A = A.astype(f32)
    m = ll.max(axis=1, keepdims=True)
    e = np.exp((ll - m).astype(f32)).astype(f32)
    U = np.zeros((T, D), f32)
    L, s_prev = 0.0, f32(1.0)
    g = (prior.astype(f32) * e[0]).astype(f32)
    for k in range(T):
        if k > 0:
            g = ((U[k - 1] @ A).astype(f32) * e[k]).astype(f32)
        s = g.sum(dtype=f32)
        shift = bias - int(np.frexp(s)[1])
        U[k] = np.ldexp(g, shift).astype(f32)
        L += float(m[k, 0]) + float(np.log(np.float64(s))) - float(np.log(np.float64(s_prev)))
        s_prev = np.ldexp(s, shift).astype(f32)
    G = np.zeros((T, D), f32)
    b = np.ones(D, f32)
    for k in range(T - 1, -1, -1):
        gam = (U[k] * b).astype(f32)
        G[k] = gam / gam.sum(dtype=f32)
        if k > 0:
            r = (A @ (e[k] * b).astype(f32)).astype(f32)
            b = np.ldexp(r, bias - int(np.frexp(r.max())[1])).astype(f32)
    return G, L
