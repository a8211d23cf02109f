"""GPU parity on randomly drawn shapes: state counts that are not padded sizes, lengths around tile and
chunk boundaries, small and large batches, shared and per-sequence models -- every call of the library
against the CPU oracle on each."""
import numpy as np
import pytest

from paper_2102_05743_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


def _draw(seed):
    rng = np.random.default_rng(seed)
    D = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 11, 15, 16, 17, 24, 31, 32, 33, 48, 63, 64, 65, 96, 127, 128]))
    budget = 3_000_000                      # D^2 * T * B kept small enough for the oracle
    B = int(rng.choice([1, 1, 1, 2, 3, 7, 19]))
    tmax = max(1, min(30000, budget // (D * D * B)))
    T = int(rng.integers(1, tmax + 1))
    if rng.random() < 0.4:                  # snap to a boundary of the tiling and step around it
        base = int(rng.choice([16, 32, 64, 128, 256, 2048, 4096]))
        T = max(1, min(tmax, base * int(rng.integers(1, 5)) + int(rng.integers(-1, 2))))
    shared = bool(rng.random() < 0.5) or B == 1
    zf = float(rng.choice([0.0, 0.0, 0.3]))
    return D, T, B, shared, zf


@pytest.mark.parametrize("seed", list(range(100)))
def test_random_shape(gu, seed):
    D, T, B, shared, zf = _draw(seed)
    p = wl.random_problem(D, T, batch=B, shared_model=shared, seed=5000 + seed, zero_frac=zf)
    label = f"seed {seed}: D={D} T={T} B={B} shared={shared} zero_frac={zf}"
    print(label, flush=True)
    gu.check_smooth(p, want_filtered=(seed % 2 == 0), label=label)
    gu.check_viterbi(p, label=label)
    gu.check_max_product(p, label=label)
    gu.check_transition_counts(p, label=label)


@pytest.mark.parametrize("D,T,B,shared", [(4, 1, 70000, True), (4, 3, 70000, False), (2, 40, 20000, True),
                                          (16, 2, 3000, False), (128, 1, 5, True), (128, 2, 5, False),
                                          (8, 17, 9000, False), (32, 33, 700, True), (64, 1, 100, True)])
def test_many_short_sequences(gu, D, T, B, shared):
    """The other extreme from the long-horizon workloads: very many sequences of a few steps."""
    p = wl.random_problem(D, T, batch=B, shared_model=shared, seed=D + T + B)
    label = f"D={D} T={T} B={B} shared={shared}"
    gu.check_smooth(p, want_filtered=True, label=label)
    gu.check_viterbi(p, label=label)
    gu.check_max_product(p, label=label)
    gu.check_transition_counts(p, label=label)


@pytest.mark.parametrize("D,T,B,ll_scale,zero_frac", [(16, 3000, 4, 30.0, 0.0), (16, 3000, 4, 8.0, 0.5), (32, 5000, 2, 30.0, 0.3),
                                                      (12, 40000, 1, 20.0, 0.2), (4, 50000, 1, 40.0, 0.0), (64, 3000, 1, 30.0, 0.0),
                                                      (128, 3000, 1, 30.0, 0.3), (24, 200, 50, 15.0, 0.6)])
def test_wide_dynamic_range(gu, D, T, B, ll_scale, zero_frac):
    """Log-likelihoods spread over tens of nats per step (emission factors down to e^-90 and below single-precision
    range after a few steps) and models with many forbidden transitions: every rescaling in the kernels is exercised."""
    p = wl.random_problem(D, T, batch=B, shared_model=(B == 1), seed=D + T + B, ll_scale=ll_scale, zero_frac=zero_frac)
    label = f"D={D} T={T} B={B} ll_scale={ll_scale} zero_frac={zero_frac}"
    gu.check_smooth(p, want_filtered=True, label=label)
    gu.check_viterbi(p, label=label)
    gu.check_max_product(p, label=label)
    gu.check_transition_counts(p, label=label)


@pytest.mark.parametrize("D", [4, 10, 40, 100])
def test_state_fading_through_the_subnormal_range(gu, D):
    """A state that can only be reached from itself and that the evidence disfavours at every step: its filtered
    probability decays through the subnormal range to zero (at e^-7 per step, after about a dozen steps), and so does
    the predicted probability that the transition statistic divides by."""
    p = wl.random_problem(D, 40, batch=3, shared_model=True, seed=90 + D)
    k = D // 2
    A = p.A.copy()
    A[0, :, k] = 0.0
    A[0, k, :] = 0.0
    A[0, k, k] = 1.0
    A[0] /= A[0].sum(axis=1, keepdims=True)
    p.A[...] = A.astype(np.float32)
    p.loglik[:, :, k] -= 7.0
    label = f"fading state D={D}"
    gu.check_smooth(p, want_filtered=True, label=label)
    gu.check_viterbi(p, label=label)
    gu.check_max_product(p, label=label)
    gu.check_transition_counts(p, label=label)


@pytest.mark.parametrize("D,T", [(17, 3000), (20, 700), (40, 2000), (100, 1500)])
def test_start_states_barely_possible_at_the_first_step(gu, D, T):
    """The first observation leaves the states of the last 16- or 32-state strip with emission factors just above
    the smallest normal number (e^-85): the part of the first chunk's aggregate that starts from them turns subnormal
    within a few steps, before its first rescaling."""
    p = wl.random_problem(D, T, batch=2, shared_model=True, seed=300 + D, ll_scale=10.0)
    strip = 16 if D <= 32 else 32
    lo = (D - 1) // strip * strip
    p.loglik[:, 0, lo:] = p.loglik[:, 0, :lo].max(axis=1, keepdims=True) - 85.0
    label = f"barely possible start states D={D}"
    gu.check_smooth(p, want_filtered=True, label=label)
    gu.check_max_product(p, label=label)
    gu.check_transition_counts(p, label=label)


def test_subnormal_strip_in_a_drawn_problem(gu):
    """The drawn problem in which the case above was met: log-likelihoods spread over 40 nats, D = 17 (one real
    state in the second strip), whose factor at the first step of one sequence is 1.4e-37."""
    p = wl.random_problem(17, 17235, batch=7, shared_model=True, seed=9242, ll_scale=40.0)
    gu.check_smooth(p, want_filtered=True, label="drawn D=17")
    gu.check_transition_counts(p, label="drawn D=17")


@pytest.mark.parametrize("D", [3, 4, 16, 40])
@pytest.mark.parametrize("kind", ["identical_rows", "permutation", "identity", "constant_evidence", "one_way_chain"])
def test_degenerate_models(gu, D, kind):
    """Transition structures at the corners of the method: independent steps (identical rows: every element has
    rank one), deterministic dynamics (a permutation, the identity: elements are scaled permutation matrices and
    log A is -inf almost everywhere), evidence that says nothing, and a left-to-right chain with an absorbing end.
    Lengths and likelihood spreads keep the exact posterior inside single-precision range."""
    rng = np.random.default_rng(17 * D + len(kind))
    T, B, scale = 3000, 2, 2.0
    p = wl.random_problem(D, T, batch=B, shared_model=True, seed=400 + D)
    A = np.zeros((D, D))
    if kind == "identical_rows":
        A[:] = rng.dirichlet(np.ones(D))[None, :]
    elif kind == "permutation":
        A[np.arange(D), rng.permutation(D)] = 1.0
        T, scale = 160, 0.3
    elif kind == "identity":
        A[np.arange(D), np.arange(D)] = 1.0
        T, scale = 120, 0.3
    elif kind == "constant_evidence":
        A = rng.dirichlet(np.ones(D), size=D)
        scale = 0.0
    else:
        for i in range(D):
            A[i, i] = 0.9 if i + 1 < D else 1.0
            if i + 1 < D:
                A[i, i + 1] = 0.1
        T, scale = 40 * D, 0.5
    p = wl.random_problem(D, T, batch=B, shared_model=True, seed=400 + D, ll_scale=max(scale, 1e-3))
    if kind == "constant_evidence":
        p.loglik[...] = -1.25
    p.A[0] = A.astype(np.float32)
    if kind == "one_way_chain":
        p.prior[0] = 0.0
        p.prior[0, 0] = 1.0
    label = f"{kind} D={D}"
    gu.check_smooth(p, want_filtered=True, label=label)
    gu.check_viterbi(p, label=label)
    gu.check_max_product(p, label=label)
    gu.check_transition_counts(p, label=label)
