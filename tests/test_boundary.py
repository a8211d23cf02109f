"""Boundary checks that need no GPU: the C-ABI library loads, exports every symbol the public
header declares, its pure-host functions work, and argument errors are reported before any launch."""
import ctypes
import os
import re

import pytest

import paper_2102_05743_amd as hmm
from paper_2102_05743_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            src = open(os.path.join(ROOT, "include", fn)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names += re.findall(r"\b(hmm_[a-z_]+)\s*\(", src)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = hmm.load_library()
    declared = _declared_functions()
    assert set(declared) == set(binding.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings():
    assert hmm.status_string(0) == "HMM_OK"
    assert hmm.status_string(1) == "HMM_ERR_INVALID_ARG"
    assert hmm.status_string(2) == "HMM_ERR_UNSUPPORTED"
    assert hmm.status_string(3) == "HMM_ERR_WORKSPACE"
    assert hmm.status_string(4) == "HMM_ERR_DEVICE"


def test_workspace_query():
    s, v = hmm.hmm_workspace_bytes(1 << 20, 4, 1)
    assert 0 < s < (1 << 22) and 0 < v < (1 << 23)
    s2, v2 = hmm.hmm_workspace_bytes(1 << 20, 4, 8)
    assert s2 > s and v2 > v
    for bad in [(0, 4, 1), (10, 0, 1), (10, 4, 0)]:
        with pytest.raises(hmm.HmmError) as e:
            hmm.hmm_workspace_bytes(*bad)
        assert e.value.code == 1
    with pytest.raises(hmm.HmmError) as e:
        hmm.hmm_workspace_bytes(10, 129, 1)
    assert e.value.code == 2


def test_argument_errors_are_caught_on_the_host():
    lib = hmm.load_library()
    fake = ctypes.c_void_p(0x1000)       # never dereferenced: every call below fails validation first
    null = ctypes.c_void_p(0)
    # null required pointers
    assert lib.hmm_smooth(null, fake, fake, 8, 4, 1, 1, fake, null, fake, fake, 1 << 20, null) == 1
    assert lib.hmm_smooth(fake, fake, fake, 8, 4, 1, 1, null, null, fake, fake, 1 << 20, null) == 1
    assert lib.hmm_viterbi(fake, fake, fake, 8, 4, 1, 1, null, fake, fake, 1 << 20, null) == 1
    # bad sizes
    assert lib.hmm_smooth(fake, fake, fake, 0, 4, 1, 1, fake, null, fake, fake, 1 << 20, null) == 1
    assert lib.hmm_viterbi(fake, fake, fake, 8, 0, 1, 1, fake, fake, fake, 1 << 20, null) == 1
    assert lib.hmm_viterbi(fake, fake, fake, 8, 4, -1, 1, fake, fake, fake, 1 << 20, null) == 1
    assert lib.hmm_smooth(fake, fake, fake, 8, 1000, 1, 1, fake, null, fake, fake, 1 << 20, null) == 2
    # misaligned log-likelihoods
    assert lib.hmm_smooth(fake, fake, ctypes.c_void_p(0x1004), 8, 4, 1, 1, fake, null, fake, fake, 1 << 20, null) == 1
    # workspace: null, too small, misaligned
    assert lib.hmm_smooth(fake, fake, fake, 8, 4, 1, 1, fake, null, fake, null, 1 << 20, null) == 3
    assert lib.hmm_smooth(fake, fake, fake, 8, 4, 1, 1, fake, null, fake, fake, 16, null) == 3
    assert lib.hmm_viterbi(fake, fake, fake, 8, 4, 1, 1, fake, fake, ctypes.c_void_p(0x1010), 1 << 20, null) == 3
    # hmm_max_product: same rules; the path output is optional
    aligned_ws = ctypes.c_void_p(0x2000)
    assert lib.hmm_max_product(fake, fake, fake, 8, 4, 1, 1, null, null, fake, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_max_product(fake, fake, fake, 8, 4, 1, 1, fake, null, null, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_max_product(fake, fake, fake, 8, 4, 1, 1, ctypes.c_void_p(0x1008), null, fake, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_max_product(fake, fake, fake, 8, 1000, 1, 1, fake, null, fake, aligned_ws, 1 << 20, null) == 2
    assert lib.hmm_max_product(fake, fake, fake, 8, 4, 1, 1, fake, null, fake, aligned_ws, 16, null) == 3
    # hmm_transition_counts
    assert lib.hmm_transition_counts(null, fake, fake, 8, 4, 1, 1, fake, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_transition_counts(fake, fake, fake, 8, 4, 1, 1, null, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_transition_counts(fake, fake, fake, 0, 4, 1, 1, fake, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_transition_counts(fake, fake, fake, 8, 200, 1, 1, fake, aligned_ws, 1 << 20, null) == 2
    assert lib.hmm_transition_counts(fake, fake, fake, 8, 4, 1, 1, fake, aligned_ws, 8, null) == 3
    assert hmm.hmm_transition_counts_workspace_bytes(1 << 20, 4, 1) >= 64
    assert hmm.hmm_transition_counts_workspace_bytes(1, 128, 3) == 3 * 128 * 128 * 4 + binding.WORKSPACE_RESERVED_BYTES
    # hmm_smooth_counts
    assert lib.hmm_smooth_counts(fake, fake, fake, 8, 4, 1, 1, fake, fake, null, aligned_ws, 1 << 22, null) == 1
    assert lib.hmm_smooth_counts(fake, fake, fake, 8, 4, 1, 1, null, fake, fake, aligned_ws, 1 << 22, null) == 1
    assert lib.hmm_smooth_counts(fake, fake, fake, 8, 200, 1, 1, fake, fake, fake, aligned_ws, 1 << 22, null) == 2
    assert lib.hmm_smooth_counts(fake, fake, fake, 8, 4, 1, 1, fake, fake, fake, aligned_ws, 64, null) == 3
    assert hmm.hmm_smooth_counts_workspace_bytes(1 << 20, 4, 1) > hmm.hmm_workspace_bytes(1 << 20, 4, 1)[0]
    # workspace preparation and state query
    assert lib.hmm_workspace_init(null, 1 << 20, null) == 3
    assert lib.hmm_workspace_init(ctypes.c_void_p(0x1010), 1 << 20, null) == 3
    assert lib.hmm_workspace_status(null, null, ctypes.byref(ctypes.c_int32(0))) == 1
    assert lib.hmm_workspace_status(fake, null, None) == 1
    # every workspace size includes the bytes the library keeps across calls
    assert min(hmm.hmm_workspace_bytes(1, 1, 1)) >= binding.WORKSPACE_RESERVED_BYTES
    assert min(hmm.hmm_workspace_bytes(100, 64, 2)) >= binding.WORKSPACE_RESERVED_BYTES
    # hmm_block_element / hmm_block_carries
    assert lib.hmm_block_element(null, fake, 8, 4, 1, 1, 0, fake, fake, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_block_element(fake, fake, 8, 4, 1, 1, 0, fake, null, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_block_element(fake, fake, 0, 4, 1, 1, 1, fake, fake, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_block_element(fake, ctypes.c_void_p(0x1004), 8, 4, 1, 1, 0, fake, fake, aligned_ws, 1 << 20, null) == 1
    assert lib.hmm_block_element(fake, fake, 8, 300, 1, 1, 0, fake, fake, aligned_ws, 1 << 20, null) == 2
    assert lib.hmm_block_element(fake, fake, 8, 4, 1, 1, 0, fake, fake, aligned_ws, 8, null) == 3
    assert lib.hmm_block_element(fake, fake, 8, 64, 1, 1, 1, fake, fake, null, 1 << 30, null) == 3
    assert lib.hmm_block_carries(fake, fake, null, fake, 3, 4, 1, 1, 0, fake, fake, fake, null) == 1
    assert lib.hmm_block_carries(fake, fake, fake, fake, 0, 4, 1, 1, 0, fake, fake, fake, null) == 1
    assert lib.hmm_block_carries(fake, fake, fake, fake, 3, 129, 1, 1, 1, fake, fake, fake, null) == 2
    for shape in [(1 << 20, 4, 1), (1 << 16, 128, 1), (4096, 16, 256), (1, 9, 1)]:
        assert hmm.hmm_block_element_workspace_bytes(*shape) >= 256


def test_a_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """The product path has no CPU fallback: without the built HIP library every call must fail loudly."""
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libhmmscan.so"))
    with pytest.raises(RuntimeError, match="missing"):
        binding.load_library()
    with pytest.raises(RuntimeError, match="missing"):
        hmm.hmm_workspace_bytes(1024, 4, 1)
    # and nothing in the package reaches for the oracle
    pkg = os.path.join(ROOT, "paper_2102_05743_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in text and "from oracle" not in text and "hmm_oracle" not in text, fn
