"""GPU parity, register-resident path (D <= 8): the HIP library through its C ABI against the
CPU oracle, element by element, on seeded inputs spanning several tiles and ragged tails."""
import numpy as np
import pytest

from paper_2102_05743_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


@pytest.fixture(autouse=True, params=["single", "multi"])
def plan(request, monkeypatch):
    """Every case runs under both launch plans: the single-launch one (tiles exchange their aggregates
    through self-validating workspace slots) where the shape allows it, and the multi-launch one forced through HMMSCAN_PLAN."""
    monkeypatch.setenv("HMMSCAN_PLAN", request.param)
    return request.param


def test_config1(gu):
    p = wl.config1()
    gu.check_smooth(p, want_filtered=True)
    gu.check_viterbi(p)
    gu.check_max_product(p)
    gu.check_transition_counts(p)


@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 4095, 4096, 4097, 10000])
def test_config2_shapes_ragged(gu, T):
    p = wl.config2(T=T)
    gu.check_smooth(p, want_filtered=(T % 2 == 1), label=f"C2 T={T}")
    gu.check_viterbi(p, label=f"C2 T={T}")
    gu.check_max_product(p, label=f"C2 T={T}")
    gu.check_transition_counts(p, label=f"C2 T={T}")


def test_gilbert_elliott_paper_model(gu):
    p = wl.gilbert_elliott(T=100000)
    gu.check_smooth(p)
    gu.check_viterbi(p)
    gu.check_max_product(p)     # binary evidence: exactly tied sequences, many ambiguous steps
    gu.check_transition_counts(p)


@pytest.mark.parametrize("D", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("T", [1, 7, 300, 4500, 20011])
def test_random_models_every_small_D(gu, D, T):
    p = wl.random_problem(D, T, seed=100 * D + T % 97)
    gu.check_smooth(p, want_filtered=(T == 300))
    gu.check_viterbi(p)
    gu.check_max_product(p)
    gu.check_transition_counts(p)


@pytest.mark.parametrize("D,T,B,shared", [(4, 5000, 3, True), (4, 4097, 5, False), (3, 100, 17, False),
                                          (8, 2100, 4, False), (2, 9000, 2, True)])
def test_batched(gu, D, T, B, shared):
    p = wl.random_problem(D, T, batch=B, shared_model=shared, seed=7 * D + B)
    gu.check_smooth(p, want_filtered=True)
    gu.check_viterbi(p)
    gu.check_max_product(p)
    gu.check_transition_counts(p)


@pytest.mark.parametrize("D,T", [(4, 6000), (6, 3000), (3, 4100)])
def test_zero_transitions_and_impossible_emissions(gu, D, T):
    """Zero entries in A (log 0 in the max-product path) and -inf log-likelihood entries
    (every step keeps at least one possible state)."""
    p = wl.random_problem(D, T, seed=900 + D, zero_frac=0.35)
    rng = np.random.default_rng(D)
    mask = rng.random(p.loglik.shape) < 0.15
    mask[..., 0] = False
    # keep the model consistent: forbid an emission only where the diagonal keeps the chain alive
    p.loglik[mask] = -np.inf
    gu.check_smooth(p)
    gu.check_viterbi(p)
    gu.check_max_product(p)
    gu.check_transition_counts(p)


def test_config2_full_size(gu):
    """The headline workload at its full size, compared element by element with the oracle."""
    p = wl.config2()
    gu.check_smooth(p, want_filtered=False, label="C2 full")
    gu.check_viterbi(p, label="C2 full")
    gu.check_max_product(p, label="C2 full")
    gu.check_transition_counts(p, label="C2 full")


def test_expired_wait_is_reported_not_hung(gu, plan, monkeypatch):
    """Failure handling of the single-launch plan, forced from the host: with a poll limit of zero every
    inter-tile wait gives up at once, all kernels still run to completion, the evidence outputs are NaN and
    the workspace is marked; later calls on it report NaN at once until it has been re-initialised, after
    which they are correct again."""
    import torch
    import paper_2102_05743_amd as hmm
    if plan != "single":
        pytest.skip("the multi-launch plan has no inter-workgroup waits")
    p = wl.config2(T=50000)
    prior, A, ll = gu.to_dev(p)
    ws_s, ws_v = hmm.hmm_workspace_bytes(p.T, p.D, 1)
    ws = hmm.new_workspace(max(ws_s, ws_v), ll.device)
    assert hmm.hmm_workspace_status(ws) == 0
    monkeypatch.setenv("HMMSCAN_SPIN_LIMIT", "0")
    _, _, L = hmm.hmm_smooth(prior, A, ll, workspace=ws)
    torch.cuda.synchronize()
    assert np.isnan(L.cpu().numpy()).all() and hmm.hmm_workspace_status(ws) == 1
    hmm.hmm_workspace_init(ws)
    _, lp = hmm.hmm_viterbi(prior, A, ll, workspace=ws)
    hmm.hmm_workspace_init(ws)
    _, _, lpm = hmm.hmm_max_product(prior, A, ll, workspace=ws)
    torch.cuda.synchronize()
    assert np.isnan(lp.cpu().numpy()).all() and np.isnan(lpm.cpu().numpy()).all()
    monkeypatch.delenv("HMMSCAN_SPIN_LIMIT")
    # still marked: an ordinary call now gives up at once instead of trusting what the failed call left behind
    _, _, L = hmm.hmm_smooth(prior, A, ll, workspace=ws)
    torch.cuda.synchronize()
    assert np.isnan(L.cpu().numpy()).all()
    hmm.hmm_workspace_init(ws)
    assert hmm.hmm_workspace_status(ws) == 0
    marg, _, L = hmm.hmm_smooth(prior, A, ll, workspace=ws)
    torch.cuda.synchronize()
    m0, _, L0 = gu.oracle.smooth(p.prior[0], p.A[0], p.loglik[0], want_filtered=False)
    assert np.abs(marg.cpu().numpy()[0] - m0).max() <= gu.MARG_ATOL and abs(float(L[0]) - L0) <= gu.LOGLIK_RTOL * abs(L0)


@pytest.mark.parametrize("D,T,B,shared", [
    (4, 16, 300, True), (4, 17, 129, False), (4, 31, 64, False), (4, 32, 7, True), (4, 33, 1000, False),
    (4, 127, 50, True), (4, 129, 33, False), (4, 511, 9, False), (4, 513, 5, True), (4, 1023, 3, False),
    (4, 1024, 6, True), (4, 1025, 6, False), (1, 5, 999, True), (2, 16, 257, False), (3, 100, 70, False),
    (5, 8, 400, False), (5, 9, 401, True), (6, 63, 100, False), (7, 65, 31, True), (8, 511, 4, False),
    (8, 512, 5, True), (8, 513, 5, False), (4, 1100, 1200, True), (6, 1030, 1030, False)])
def test_short_sequences_packed_into_workgroups(gu, D, T, B, shared):
    """Sequences of at most 64 chunks (1024 steps at D <= 4, 512 above) share workgroups, a power-of-two
    group of lanes each: lengths at and around the group sizes' limits, batches that do not fill the last
    workgroup, per-sequence models; one step beyond the limit the one-sequence-per-workgroup form takes over."""
    p = wl.random_problem(D, T, batch=B, shared_model=shared, seed=11 * D + T + B)
    label = f"packed D={D} T={T} B={B} shared={shared}"
    gu.check_smooth(p, want_filtered=(T % 2 == 0), label=label)
    gu.check_viterbi(p, label=label)
    gu.check_max_product(p, label=label)
    gu.check_transition_counts(p, label=label)


def test_two_workgroups_per_compute_unit(gu):
    """Two sequences of 2^20 - 3 steps in one call: 512 tiles, which fit the device only with two workgroups
    resident per compute unit; the single-launch plan takes them, every tile waits for the 255 others of its
    own sequence, and the two sequences' exchanges must not mix."""
    import paper_2102_05743_amd as hmm
    p = wl.random_problem(4, (1 << 20) - 3, batch=2, shared_model=False, seed=4242)
    hmm.hmm_kernel_timing_enable(True)
    try:
        gu.check_smooth(p, label="2 x (2^20 - 3), D=4")
        gu.check_viterbi(p, label="2 x (2^20 - 3), D=4")
        print("kernels:", sorted(hmm.hmm_kernel_timing_get()), flush=True)
    finally:
        hmm.hmm_kernel_timing_enable(False)


def test_very_long_sequence(gu, plan):
    """2^23 + 5 steps in one sequence: 2049 tiles, far more than fit the device at once, so the multi-launch
    kernels run whatever plan is asked for; every marginal and the whole path against the oracle."""
    if plan == "multi":
        pytest.skip("the same kernels as under the default plan at this length")
    p = wl.config2(T=(1 << 23) + 5, seed=77)
    gu.check_smooth(p, label="C2 model, T=2^23+5")
    gu.check_viterbi(p, label="C2 model, T=2^23+5")


@pytest.mark.parametrize("T,B", [(2048 * 5 + 77, 1), (4096 * 3, 2), (1 << 18, 1), (100, 3)])
def test_results_do_not_depend_on_the_tile_size(gu, T, B, monkeypatch):
    """The same calls through a second build of the library whose tiles are half as long (8 steps per lane
    instead of 16, D = 4 only): tile boundaries, chunk boundaries and the number of exchanged aggregates all
    move, the results must not.  Each build is checked against the oracle; between the builds the decoded
    paths must be identical and the marginals agree to rounding."""
    import os

    import numpy as np
    import torch

    import paper_2102_05743_amd as hmm
    from paper_2102_05743_amd import binding

    variant = os.path.join(os.path.dirname(binding.LIB_PATH), "libhmmscan_tile8.so")
    if not os.path.exists(variant):
        pytest.skip("the tile-size variant library is not built")
    p = wl.random_problem(4, T, batch=B, shared_model=(B == 1), seed=900 + B)

    def run():
        dev = torch.device("cuda:0")
        prior, A, ll = (torch.from_numpy(x).to(dev) for x in (p.prior, p.A, p.loglik))
        marg, _, L = hmm.hmm_smooth(prior, A, ll)
        path, lp = hmm.hmm_viterbi(prior, A, ll)
        torch.cuda.synchronize()
        return marg.cpu().numpy(), L.cpu().numpy(), path.cpu().numpy(), lp.cpu().numpy()

    main = run()
    gu.check_smooth(p, label=f"main build T={T} B={B}")
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", variant)
    other = run()
    gu.check_smooth(p, label=f"tile-size variant T={T} B={B}")
    gu.check_viterbi(p, label=f"tile-size variant T={T} B={B}")
    monkeypatch.setattr(binding, "_lib", None)   # the next user loads the main library again
    assert np.array_equal(main[2], other[2]), "decoded paths differ between tile sizes"
    assert float(np.abs(main[0] - other[0]).max()) <= 2e-5
    assert np.allclose(main[1], other[1], rtol=1e-7) and np.allclose(main[3], other[3], rtol=1e-7)   # single-precision sums in another order
