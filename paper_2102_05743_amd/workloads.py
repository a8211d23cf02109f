"""Seeded synthetic HMM workloads (inputs only; no inference arithmetic lives here).

Every generator returns an :class:`HmmProblem` whose arrays are float32 and
C-contiguous: ``prior[Bm][D]``, ``A[Bm][D][D]`` (row-stochastic,
``A[i][j] = p(x_k = j | x_{k-1} = i)``), ``loglik[B][T][D]`` with
``loglik[b][t][j] = log p(y_t | x_t = j)``; ``Bm`` is 1 when the model is shared
by the whole batch and ``B`` otherwise.  All draws are made in float64 from a
counter-based generator (Philox) keyed by the seed, then rounded to float32, so
the CPU oracle and the GPU path consume bit-identical inputs.

The shapes follow the paper's experiment (Sec. VI: a 4-state Gilbert-Elliott
channel with binary observations, long horizons) and scaled-up variants of it;
they stand in for the paper's simulated data, which is itself synthetic.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 210205743


@dataclass
class HmmProblem:
    name: str
    prior: np.ndarray      # [Bm][D] float32
    A: np.ndarray          # [Bm][D][D] float32
    loglik: np.ndarray     # [B][T][D] float32
    shared_model: bool
    states: np.ndarray | None = None   # [B][T] sampled hidden states (int32), for reference only
    obs: np.ndarray | None = None      # [B][T] sampled observations

    @property
    def batch(self) -> int:
        return int(self.loglik.shape[0])

    @property
    def T(self) -> int:
        return int(self.loglik.shape[1])

    @property
    def D(self) -> int:
        return int(self.loglik.shape[2])


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def _sample_chain(rng: np.random.Generator, prior: np.ndarray, A: np.ndarray, T: int) -> np.ndarray:
    """Draw x_1 ~ prior, x_k ~ A[x_{k-1}] by inverse-CDF on one uniform per step."""
    D = prior.shape[0]
    u = rng.random(T)
    cum_prior = np.cumsum(prior)
    cum_A = np.cumsum(A, axis=1)
    cum_prior[-1] = 1.0
    cum_A[:, -1] = 1.0
    # nxt[k][i] = state reached from i when the step's uniform is u[k]
    nxt = np.empty((T, D), dtype=np.int32)
    for i in range(D):
        nxt[:, i] = np.searchsorted(cum_A[i], u, side="right")
    np.minimum(nxt, D - 1, out=nxt)
    x = np.empty(T, dtype=np.int32)
    x[0] = min(int(np.searchsorted(cum_prior, u[0], side="right")), D - 1)
    nl = nxt.tolist()
    cur = int(x[0])
    xs = [cur]
    for k in range(1, T):
        cur = nl[k][cur]
        xs.append(cur)
    x[:] = xs
    return x


def _dirichlet_rows(rng: np.random.Generator, alpha: float, rows: int, cols: int) -> np.ndarray:
    g = rng.standard_gamma(alpha, size=(rows, cols))
    g = np.maximum(g, 1e-300)
    return g / g.sum(axis=1, keepdims=True)


def _f32_stochastic(M: np.ndarray) -> np.ndarray:
    """Round to float32 (rows then sum to 1 within float32 rounding)."""
    return np.ascontiguousarray(M, dtype=np.float32)


def _discrete_problem(name, rng, prior, A, E, T):
    """Sample one sequence from (prior, A, E[j][y]) and tabulate log E[j][y_t]."""
    x = _sample_chain(rng, prior, A, T)
    K = E.shape[1]
    cumE = np.cumsum(E, axis=1)
    cumE[:, -1] = 1.0
    v = rng.random(T)
    y = np.empty(T, dtype=np.int32)
    for j in range(E.shape[0]):
        m = x == j
        y[m] = np.minimum(np.searchsorted(cumE[j], v[m], side="right"), K - 1)
    with np.errstate(divide="ignore"):
        logE = np.log(E)
    ll = logE.T[y]                      # [T][D]
    return x, y, ll


def config1(T: int = 1024, seed: int = BASE_SEED + 1) -> HmmProblem:
    """D=4, uniform prior, Dirichlet(1) transition rows, binary observations."""
    D = 4
    rng = _rng(seed)
    prior = np.full(D, 1.0 / D)
    A = _dirichlet_rows(rng, 1.0, D, D)
    u = rng.uniform(0.05, 0.95, size=D)
    E = np.stack([1.0 - u, u], axis=1)
    x, y, ll = _discrete_problem("c1", rng, prior, A, E, T)
    return HmmProblem("C1", _f32_stochastic(prior[None]), _f32_stochastic(A[None]),
                      np.ascontiguousarray(ll[None], dtype=np.float32), True, x[None], y[None])


def config2(T: int = 1 << 20, seed: int = BASE_SEED + 2) -> HmmProblem:
    """Burst-channel-style D=4 model in the shape of Sec. VI: sticky states
    (self-transition U(0.9, 0.99), rest spread evenly), transmitted bit
    b(j) = j // 2, observed bit flipped with a state-dependent probability
    U(0.01, 0.3)."""
    D = 4
    rng = _rng(seed)
    prior = np.full(D, 1.0 / D)
    stay = rng.uniform(0.9, 0.99, size=D)
    A = np.empty((D, D))
    for i in range(D):
        A[i, :] = (1.0 - stay[i]) / (D - 1)
        A[i, i] = stay[i]
    flip = rng.uniform(0.01, 0.3, size=D)
    E = np.empty((D, 2))
    for j in range(D):
        b = j // 2
        E[j, b] = 1.0 - flip[j]
        E[j, 1 - b] = flip[j]
    x, y, ll = _discrete_problem("c2", rng, prior, A, E, T)
    return HmmProblem("C2", _f32_stochastic(prior[None]), _f32_stochastic(A[None]),
                      np.ascontiguousarray(ll[None], dtype=np.float32), True, x[None], y[None])


def _gaussian_ll(rng, prior, A, mu, T):
    x = _sample_chain(rng, prior, A, T)
    y = mu[x] + rng.standard_normal(T)
    ll = -0.5 * (y[:, None] - mu[None, :]) ** 2 - 0.5 * np.log(2.0 * np.pi)
    return x, y, ll


def config3(T: int = 1 << 18, seed: int = BASE_SEED + 3) -> HmmProblem:
    """D=32, Dirichlet(0.5) rows, unit-variance Gaussian emissions with state
    means ~ N(0, variance 4), log-likelihoods tabulated."""
    D = 32
    rng = _rng(seed)
    prior = np.full(D, 1.0 / D)
    A = _dirichlet_rows(rng, 0.5, D, D)
    mu = 2.0 * rng.standard_normal(D)
    x, y, ll = _gaussian_ll(rng, prior, A, mu, T)
    return HmmProblem("C3", _f32_stochastic(prior[None]), _f32_stochastic(A[None]),
                      np.ascontiguousarray(ll[None], dtype=np.float32), True, x[None], y[None])


def config4(batch: int = 256, T: int = 4096, seed: int = BASE_SEED + 4) -> HmmProblem:
    """Batch of independent D=16 models: per-sequence Dirichlet(1) transition rows and
    categorical emissions over 8 symbols with Dirichlet(1) rows."""
    D, K = 16, 8
    rng = _rng(seed)
    priors = np.full((batch, D), 1.0 / D)
    As = np.empty((batch, D, D))
    lls = np.empty((batch, T, D), dtype=np.float32)
    xs = np.empty((batch, T), dtype=np.int32)
    ys = np.empty((batch, T), dtype=np.int32)
    for b in range(batch):
        As[b] = _dirichlet_rows(rng, 1.0, D, D)
        E = _dirichlet_rows(rng, 1.0, D, K)
        x, y, ll = _discrete_problem("c4", rng, priors[b], As[b], E, T)
        lls[b] = ll
        xs[b] = x
        ys[b] = y
    return HmmProblem("C4", _f32_stochastic(priors), _f32_stochastic(As), lls, False, xs, ys)


def config5(T: int = 1 << 16, seed: int = BASE_SEED + 5, D: int = 128) -> HmmProblem:
    """Banded-plus-noise transitions (self 0.5; in-range neighbours at distance
    1..4 share 0.4 equally, no wrap-around; 0.1/D added everywhere) and
    unit-variance Gaussian emissions with state means on a grid of spacing 0.25."""
    rng = _rng(seed)
    prior = np.full(D, 1.0 / D)
    A = np.full((D, D), 0.1 / D)
    for i in range(D):
        A[i, i] += 0.5
        nb = [j for j in range(i - 4, i + 5) if j != i and 0 <= j < D]
        for j in nb:
            A[i, j] += 0.4 / len(nb)
    mu = (np.arange(D) - (D - 1) / 2.0) * 0.25
    x, y, ll = _gaussian_ll(rng, prior, A, mu, T)
    return HmmProblem("C5", _f32_stochastic(prior[None]), _f32_stochastic(A[None]),
                      np.ascontiguousarray(ll[None], dtype=np.float32), True, x[None], y[None])


def gilbert_elliott_matrices(p0=0.03, p1=0.1, p2=0.05, q0=0.01, q1=0.1):
    """Transition matrix and observation model of the Gilbert-Elliott channel
    exactly as printed in Sec. VI (the equation giving Pi and O), with the
    section's parameter values as defaults."""
    Pi = np.array([
        [(1 - p0) * (1 - p2), p0 * (1 - p2), (1 - p0) * p2, p0 * p2],
        [p1 * (1 - p2), (1 - p1) * (1 - p2), p1 * p2, (1 - p1) * p2],
        [(1 - p0) * p2, p0 * p2, (1 - p0) * (1 - p2), p0 * (1 - p2)],
        [p1 * p2, (1 - p1) * p2, p1 * (1 - p2), (1 - p1) * (1 - p2)],
    ])
    O = np.array([[1 - q0, q0], [1 - q1, q1], [q0, 1 - q0], [q1, 1 - q1]])
    return Pi, O


def gilbert_elliott(T: int = 100000, seed: int = BASE_SEED + 6) -> HmmProblem:
    """The paper's own workload (Sec. VI): D=4, binary observations, uniform prior."""
    rng = _rng(seed)
    Pi, O = gilbert_elliott_matrices()
    prior = np.full(4, 0.25)
    x, y, ll = _discrete_problem("ge", rng, prior, Pi, O, T)
    return HmmProblem("GE", _f32_stochastic(prior[None]), _f32_stochastic(Pi[None]),
                      np.ascontiguousarray(ll[None], dtype=np.float32), True, x[None], y[None])


def random_problem(D: int, T: int, batch: int = 1, shared_model: bool = True, seed: int = 0,
                   alpha: float = 1.0, ll_scale: float = 2.0, zero_frac: float = 0.0) -> HmmProblem:
    """Generic random model for parity sweeps: Dirichlet(alpha) prior and rows,
    log-likelihoods drawn directly as -|N(0, ll_scale)| (no sampled sequence);
    ``zero_frac`` of the transition entries are zeroed (rows renormalised, the
    diagonal kept) to exercise log 0 in the max-product path."""
    rng = _rng(BASE_SEED * 7 + seed)
    Bm = 1 if shared_model else batch
    prior = np.stack([_dirichlet_rows(rng, alpha, 1, D)[0] for _ in range(Bm)])
    A = np.stack([_dirichlet_rows(rng, alpha, D, D) for _ in range(Bm)])
    if zero_frac > 0.0:
        mask = rng.random(A.shape) < zero_frac
        idx = np.arange(D)
        mask[:, idx, idx] = False
        A = np.where(mask, 0.0, A)
        A = A / A.sum(axis=2, keepdims=True)
    ll = -np.abs(rng.standard_normal((batch, T, D))) * ll_scale
    return HmmProblem(f"rand_D{D}_T{T}_B{batch}", _f32_stochastic(prior), _f32_stochastic(A),
                      np.ascontiguousarray(ll, dtype=np.float32), shared_model)


CONFIGS = {"C1": config1, "C2": config2, "C3": config3, "C4": config4, "C5": config5,
           "GE": gilbert_elliott}
