"""Baum-Welch parameter estimation (Sec. V-C) with the library as its expectation step: hmm_smooth for the
marginals and the evidence, hmm_transition_counts for the expected transitions; the maximisation step is a
few lines of array arithmetic in the test.  Checked against the same iterations run with the CPU oracle as
the expectation step, and against EM's own guarantee that the evidence never decreases."""
import numpy as np
import pytest
import torch

import oracle
import paper_2102_05743_amd as hmm
from paper_2102_05743_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _m_step(xp, gamma, counts, obs_onehot):
    """gamma [T][D], counts [D][D], obs_onehot [T][K] -> prior [D], A [D][D], E [D][K] (xp: numpy or torch)."""
    A = counts / counts.sum(-1, keepdims=True) if xp is np else counts / counts.sum(-1, keepdim=True)
    prior = gamma[0] / gamma[0].sum()
    num = gamma.T @ obs_onehot
    E = num / (num.sum(-1, keepdims=True) if xp is np else num.sum(-1, keepdim=True))
    return prior, A, E


@pytest.mark.parametrize("D,K,T", [(4, 2, 20000), (3, 5, 3000), (12, 6, 8000)])
def test_baum_welch_iterations_follow_the_oracle_and_never_lose_evidence(D, K, T):
    rng = np.random.default_rng(100 * D + K)
    # data from a random model, start from another one
    A_true = rng.dirichlet(np.full(D, 0.5), size=D)
    E_true = rng.dirichlet(np.full(K, 0.5), size=D)
    x = np.zeros(T, dtype=np.int64)
    y = np.zeros(T, dtype=np.int64)
    x[0] = rng.integers(D)
    for t in range(T):
        if t:
            x[t] = rng.choice(D, p=A_true[x[t - 1]])
        y[t] = rng.choice(K, p=E_true[x[t]])
    onehot = np.eye(K)[y]
    prior0 = np.full(D, 1.0 / D)
    A0 = rng.dirichlet(np.full(D, 2.0), size=D)
    E0 = rng.dirichlet(np.full(K, 2.0), size=D)

    # oracle-driven EM (fp64 throughout)
    prior, A, E = prior0.copy(), A0.copy(), E0.copy()
    L_ref = []
    for _ in range(6):
        ll = np.log(E[:, y].T)
        p32 = prior.astype(np.float32)[None]; A32 = A.astype(np.float32)[None]; ll32 = ll.astype(np.float32)[None]
        m, f, L = oracle.smooth_batch(p32, A32, ll32, True, want_filtered=True)
        N = oracle.transition_counts_batch(p32, A32, ll32, True)
        L_ref.append(float(L[0]))
        prior, A, E = _m_step(np, m[0].astype(np.float64), N[0], onehot)

    # library-driven EM: the same arithmetic around the GPU calls
    dev = torch.device("cuda:0")
    oh = torch.from_numpy(onehot).to(dev)
    yd = torch.from_numpy(y).to(dev)
    prior, A, E = (torch.from_numpy(v).to(dev) for v in (prior0, A0, E0))
    L_gpu = []
    for _ in range(6):
        ll = torch.log(E[:, yd].T).to(torch.float32)[None].contiguous()
        p32 = prior.to(torch.float32)[None].contiguous(); A32 = A.to(torch.float32)[None].contiguous()
        marg, filt, L = hmm.hmm_smooth(p32, A32, ll, want_filtered=True)
        N = hmm.hmm_transition_counts(A32, filt, marg)
        L_gpu.append(float(L[0]))
        prior, A, E = _m_step(torch, marg[0].to(torch.float64), N[0], oh)
    print(f"[EM D={D} K={K} T={T}] evidence per iteration: gpu {np.round(L_gpu, 3).tolist()} oracle {np.round(L_ref, 3).tolist()}",
          flush=True)
    for it, (a, b) in enumerate(zip(L_gpu, L_ref)):
        assert abs(a - b) <= 1e-4 * abs(b), f"iteration {it}: evidence {a} vs {b} with the oracle as E-step"
    for it in range(1, len(L_gpu)):
        assert L_gpu[it] >= L_gpu[it - 1] - 2e-6 * abs(L_gpu[it]), f"evidence fell at iteration {it}: {L_gpu}"
    assert L_gpu[-1] > L_gpu[0]


@pytest.mark.parametrize("plan", ["single", "multi"])
@pytest.mark.parametrize("D,T,B,shared", [(4, 20000, 1, True), (4, 4097, 5, False), (3, 100, 17, False), (8, 6100, 2, False),
                                          (2, 9000, 2, True), (6, 1, 3, True), (4, 1 << 20, 1, True), (16, 5000, 2, True)])
def test_expectation_step_in_one_call(D, T, B, shared, plan, monkeypatch):
    """hmm_smooth_counts: marginals, evidence and expected transition counts from one call.  Up to eight states the
    counts come out of the smoother's own backward recursion (both launch plans, any length); above that (here
    D = 16) the call takes the two-call form inside the library."""
    import gpu_util
    if D > 8 and plan == "multi":
        pytest.skip("one plan above eight states")
    monkeypatch.setenv("HMMSCAN_PLAN", plan)
    p = wl.config2() if T == 1 << 20 else wl.random_problem(D, T, batch=B, shared_model=shared, seed=5 * D + B)
    gpu_util.check_smooth_counts(p, label=f"D={D} T={T} B={B} plan={plan}")
