"""Helpers shared by the GPU parity tests: run the HIP library through its C ABI binding and
compare with the CPU oracle under the tolerances stated for this build:
marginals 1e-4 absolute, log-likelihood 1e-4 relative, Viterbi path exact except at numerical
near-ties, where the fp64 score of the returned path and the returned log-probability must both
agree with the oracle's optimum within 1e-5 relative."""
import numpy as np
import torch

import oracle
import paper_2102_05743_amd as hmm

MARG_ATOL = 1e-4
LOGLIK_RTOL = 1e-4
LOGPROB_RTOL = 1e-5


def to_dev(p):
    dev = torch.device("cuda:0")
    return (torch.from_numpy(p.prior).to(dev), torch.from_numpy(p.A).to(dev), torch.from_numpy(p.loglik).to(dev))


def run_smooth(p, want_filtered=False):
    prior, A, ll = to_dev(p)
    marg, filt, L = hmm.hmm_smooth(prior, A, ll, want_filtered=want_filtered)
    torch.cuda.synchronize()
    return marg.cpu().numpy(), (filt.cpu().numpy() if filt is not None else None), L.cpu().numpy()


def run_viterbi(p):
    prior, A, ll = to_dev(p)
    path, lp = hmm.hmm_viterbi(prior, A, ll)
    torch.cuda.synchronize()
    return path.cpu().numpy(), lp.cpu().numpy()


def check_smooth(p, want_filtered=False, label=""):
    marg, filt, L = run_smooth(p, want_filtered)
    m0, f0, L0 = oracle.smooth_batch(p.prior, p.A, p.loglik, p.shared_model, want_filtered=True)
    assert np.isfinite(marg).all(), f"{label}: non-finite marginals"
    err = float(np.abs(marg - m0).max())
    rel = float(np.abs((L - L0) / L0).max()) if np.all(L0 != 0) else float(np.abs(L - L0).max())
    print(f"[smooth {label or p.name}] B={p.batch} T={p.T} D={p.D} max|dmarg|={err:.3e} rel dloglik={rel:.3e}", flush=True)
    assert err <= MARG_ATOL, f"{label}: marginals off by {err}"
    assert rel <= LOGLIK_RTOL, f"{label}: loglik rel err {rel} ({L} vs {L0})"
    if want_filtered:
        ferr = float(np.abs(filt - f0).max())
        print(f"    max|dfiltered|={ferr:.3e}", flush=True)
        assert ferr <= MARG_ATOL
    return err, rel


def check_viterbi(p, label=""):
    path, lp = run_viterbi(p)
    assert path.min() >= 0 and path.max() < p.D, f"{label}: state out of range"
    p0, lp0 = oracle.viterbi_batch(p.prior, p.A, p.loglik, p.shared_model)
    total_mismatch = 0
    for b in range(p.batch):
        mb = 0 if p.shared_model else b
        tol = LOGPROB_RTOL * max(abs(lp0[b]), 1e-30)
        assert abs(lp[b] - lp0[b]) <= tol, f"{label}: logprob {lp[b]} vs oracle {lp0[b]} (seq {b})"
        nm = int((path[b] != p0[b]).sum())
        if nm:
            # numerical near-tie: the returned path must itself be (numerically) optimal
            sc = oracle.score(p.prior[mb], p.A[mb], p.loglik[b], path[b])
            assert abs(sc - lp0[b]) <= tol, f"{label}: path differs at {nm} steps and scores {sc} vs {lp0[b]}"
            total_mismatch += nm
    rel = float(np.abs((lp - lp0) / np.where(lp0 == 0, 1, lp0)).max())
    print(f"[viterbi {label or p.name}] B={p.batch} T={p.T} D={p.D} path mismatches={total_mismatch} "
          f"rel dlogprob={rel:.3e}", flush=True)
    return total_mismatch
