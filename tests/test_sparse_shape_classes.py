"""CPU pin for the two lists of tests/test_gpu_sparse_models.py: the classical recursion run step by step in
single precision (tests/fp32_recursion.py) stays within the tolerances of the fp64 oracle on every
WITHIN_RANGE shape it is asked about and leaves them on every BEYOND_SINGLE_PRECISION shape -- so what the GPU
tests demand of the scan formulation is exactly what the arithmetic type can deliver."""
import numpy as np
import pytest

import oracle
from fp32_recursion import smooth_f32, smooth_f32_lifted
from paper_2102_05743_amd import workloads as wl
from test_gpu_sparse_models import BEYOND_SINGLE_PRECISION, WITHIN_RANGE, _problem


def _worst(shape, recursion=smooth_f32):
    p = _problem(shape)
    bad = 0
    for b in range(p.batch):
        mb = 0 if p.shared_model else b
        m0, _, L0 = oracle.smooth(p.prior[mb], p.A[mb], p.loglik[b], want_filtered=False)
        with np.errstate(all="ignore"):
            g, L = recursion(p.prior[mb], p.A[mb], p.loglik[b])
        ok = np.isfinite(g).all() and float(np.abs(g - m0).max()) <= 1e-4 and abs(L - L0) <= 1e-4 * abs(L0)
        bad += 0 if ok else 1
    return bad


# the small-state shapes are enough for the pin (the oracle and the recursion cost D^2 T per sequence in Python)
@pytest.mark.parametrize("shape", [s for s in BEYOND_SINGLE_PRECISION if s[1] <= 4 and s[2] <= 7000],
                         ids=lambda s: f"seed{s[0]}")
def test_single_precision_recursion_loses_these(shape):
    assert _worst(shape) > 0


# (35688 needs potentials held far above one, which the library does and this plain recursion does not)
@pytest.mark.parametrize("shape", [s for s in WITHIN_RANGE if s[1] <= 4 and s[0] != 35688], ids=lambda s: f"seed{s[0]}")
def test_single_precision_recursion_keeps_these(shape):
    assert _worst(shape) == 0


# above eight states the library falls back on the step-by-step recursion with lifted potentials for such sequences:
# that arithmetic holds these shapes (two of which the plain recursion above does not), and still not the last one
@pytest.mark.parametrize("shape", [s for s in WITHIN_RANGE if s[1] > 8], ids=lambda s: f"seed{s[0]}")
def test_lifted_single_precision_recursion_keeps_these(shape):
    assert _worst(shape, smooth_f32_lifted) == 0


@pytest.mark.parametrize("shape", [s for s in BEYOND_SINGLE_PRECISION if s[1] > 8], ids=lambda s: f"seed{s[0]}")
def test_lifted_single_precision_recursion_loses_these(shape):
    assert _worst(shape, smooth_f32_lifted) > 0
