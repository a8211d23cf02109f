"""The library's calls under HIP graph capture: a serving loop records hmm_smooth + hmm_viterbi (+ hmm_max_product)
once and replays the graph on new inputs.  Every launch of the library is a kernel (the exchange slots of the
single-launch plan are reset by a fill kernel, not a memset), so the recorded graph must reproduce the eager
results exactly, replay after replay, with eager work on the same workspace in between."""
import numpy as np
import pytest
import torch

import paper_2102_05743_amd as hmm
from paper_2102_05743_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _problems(kind):
    if kind == "c2":
        return wl.config2(T=200000), wl.config2(T=200000, seed=991)
    if kind == "c2_multi":   # more tiles than the single-launch plan takes: the multi-launch kernels
        return wl.config2(T=(1 << 20) + 4097), wl.config2(T=(1 << 20) + 4097, seed=992)
    if kind == "c3":
        return wl.config3(T=30000), wl.config3(T=30000, seed=993)
    if kind == "short":      # several short sequences per workgroup, no workspace
        return (wl.random_problem(4, 300, batch=500, shared_model=True, seed=5),
                wl.random_problem(4, 300, batch=500, shared_model=True, seed=6))
    if kind == "c4_full":    # enough chunks for the one-pass vector recursions
        return wl.config4(), wl.config4(seed=995)
    return wl.config4(batch=8, T=1000), wl.config4(batch=8, T=1000, seed=994)


@pytest.mark.parametrize("kind", ["c2", "c2_multi", "c3", "c4", "short", "c4_full"])
def test_captured_calls_replay_exactly(kind):
    pa, pb = _problems(kind)
    dev = torch.device("cuda:0")
    prior, A = torch.from_numpy(pa.prior).to(dev), torch.from_numpy(pa.A).to(dev)
    lla, llb = torch.from_numpy(pa.loglik).to(dev), torch.from_numpy(pb.loglik).to(dev)
    B, T, D = lla.shape
    ws_s, ws_v = hmm.hmm_workspace_bytes(T, D, B)
    ws = hmm.new_workspace(max(ws_s, ws_v), dev)

    def eager(ll):
        m, _, L = hmm.hmm_smooth(prior, A, ll, workspace=ws)
        p, lp = hmm.hmm_viterbi(prior, A, ll, workspace=ws)
        mm, am, lp2 = hmm.hmm_max_product(prior, A, ll, workspace=ws)
        torch.cuda.synchronize()
        return [t.clone() for t in (m, L, p, lp, mm, am, lp2)]

    ref = {"a": eager(lla), "b": eager(llb)}

    ll_in = lla.clone()
    marg, L = torch.empty_like(lla), torch.empty(B, dtype=torch.float64, device=dev)
    path, lp = torch.empty((B, T), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.float64, device=dev)
    mm, am = torch.empty_like(lla), torch.empty((B, T), dtype=torch.int32, device=dev)
    lp2 = torch.empty(B, dtype=torch.float64, device=dev)
    outs = (marg, L, path, lp, mm, am, lp2)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        hmm.hmm_smooth(prior, A, ll_in, marginals=marg, loglik_out=L, workspace=ws)
        hmm.hmm_viterbi(prior, A, ll_in, path=path, logprob_out=lp, workspace=ws)
        hmm.hmm_max_product(prior, A, ll_in, max_marginals=mm, path=am, logprob_out=lp2, workspace=ws)
    for rep, which in enumerate(["a", "b", "b", "a", "b"]):
        ll_in.copy_(lla if which == "a" else llb)
        for o in outs:
            o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs, ref[which]):
            assert torch.equal(got, want), f"{kind}: replay {rep} on input {which} differs from the eager result"
        eager(lla if rep % 2 else llb)   # eager work on the same workspace between replays
    print(f"[graph {kind}] B={B} T={T} D={D}: 5 replays equal the eager results bit for bit", flush=True)
