"""hmm_smooth_static (the entry point for callers that cannot allocate: its scratch memory is a device array
inside the library) against hmm_smooth on the same inputs, through the C ABI: two calls in a row on the shared
array, the second on a smaller input; too large a shape is refused on the host."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2102_05743_amd as hmm
from paper_2102_05743_amd import binding
from paper_2102_05743_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _both(p, want_filtered):
    dev = torch.device("cuda:0")
    prior, A, ll = (torch.from_numpy(x).to(dev) for x in (p.prior, p.A, p.loglik))
    ref_m, ref_f, ref_L = hmm.hmm_smooth(prior, A, ll, want_filtered=want_filtered)
    torch.cuda.synchronize()
    marg = torch.full_like(ll, float("nan"))
    filt = torch.full_like(ll, float("nan")) if want_filtered else None
    L = torch.full((p.batch,), float("nan"), dtype=torch.float64, device=dev)
    hmm.hmm_smooth_static(prior, A, ll, marg, L, filtered=filt)
    torch.cuda.synchronize()
    # the same kernels on the same inputs: the outputs agree bit for bit
    assert np.array_equal(marg.cpu().numpy(), ref_m.cpu().numpy())
    assert np.array_equal(L.cpu().numpy(), ref_L.cpu().numpy())
    assert np.isfinite(L.cpu().numpy()).all()
    if want_filtered:
        assert np.array_equal(filt.cpu().numpy(), ref_f.cpu().numpy())
    print(f"[static scratch] D={p.D} T={p.T} B={p.batch} loglik={L.cpu().numpy()[:2]}", flush=True)


def test_static_scratch_two_calls_second_smaller():
    # exchange between tiles of one long sequence, then a smaller call that finds the first call's leftovers
    _both(wl.config2(T=300_000), want_filtered=False)
    _both(wl.config2(T=70_001), want_filtered=True)
    # several sequences, multi-tile, and the matrix-core path at a size whose scratch still fits
    _both(wl.random_problem(3, 9000, batch=5, shared_model=False, seed=77), want_filtered=True)
    _both(wl.random_problem(16, 3000, batch=2, shared_model=True, seed=78), want_filtered=False)
    _both(wl.config1(), want_filtered=False)


def test_static_scratch_refuses_large_shapes_on_the_host():
    lib = hmm.load_library()
    need = hmm.hmm_workspace_bytes(1 << 16, 128, 1)[0]
    assert need > binding.STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: the size check comes first
    rc = lib.hmm_smooth_static(fake, fake, fake, 1 << 16, 128, 1, 1, fake, None, fake, None)
    assert rc == 3
