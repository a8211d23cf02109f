"""ctypes binding of libhmmscan.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device memory; the stream
is torch's current stream.  Every step of the computation runs in the HIP
library; there is no fallback of any kind -- a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhmmscan.so")

HMM_OK = 0
_lib = None

EXPORTED_SYMBOLS = ("hmm_workspace_bytes", "hmm_workspace_init", "hmm_workspace_status", "hmm_smooth", "hmm_smooth_static", "hmm_viterbi", "hmm_max_product",
                    "hmm_transition_counts_workspace_bytes", "hmm_transition_counts",
                    "hmm_smooth_counts_workspace_bytes", "hmm_smooth_counts",
                    "hmm_block_element_workspace_bytes", "hmm_block_element", "hmm_block_carries", "hmm_status_string",
                    "hmm_kernel_timing_enable", "hmm_kernel_timing_count", "hmm_kernel_timing_get")


class HmmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)}")


def load_library():
    """Load the HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2102_05743_amd.build` "
                "(or __graft_entry__.build()); the library has no non-HIP fallback")
        lib = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        lib.hmm_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                            ctypes.POINTER(sz), ctypes.POINTER(sz)]
        lib.hmm_workspace_bytes.restype = ctypes.c_int
        lib.hmm_workspace_init.argtypes = [vp, sz, vp]
        lib.hmm_workspace_init.restype = ctypes.c_int
        lib.hmm_workspace_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int32)]
        lib.hmm_workspace_status.restype = ctypes.c_int
        lib.hmm_smooth.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                   vp, vp, vp, vp, sz, vp]
        lib.hmm_smooth.restype = ctypes.c_int
        lib.hmm_smooth_static.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          vp, vp, vp, vp]
        lib.hmm_smooth_static.restype = ctypes.c_int
        lib.hmm_viterbi.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                    vp, vp, vp, sz, vp]
        lib.hmm_viterbi.restype = ctypes.c_int
        lib.hmm_max_product.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                        vp, vp, vp, vp, sz, vp]
        lib.hmm_max_product.restype = ctypes.c_int
        lib.hmm_transition_counts_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                                              ctypes.POINTER(sz)]
        lib.hmm_transition_counts_workspace_bytes.restype = ctypes.c_int
        lib.hmm_transition_counts.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                              vp, vp, sz, vp]
        lib.hmm_transition_counts.restype = ctypes.c_int
        lib.hmm_smooth_counts_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(sz)]
        lib.hmm_smooth_counts_workspace_bytes.restype = ctypes.c_int
        lib.hmm_smooth_counts.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          vp, vp, vp, vp, sz, vp]
        lib.hmm_smooth_counts.restype = ctypes.c_int
        lib.hmm_block_element_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(sz)]
        lib.hmm_block_element_workspace_bytes.restype = ctypes.c_int
        lib.hmm_block_element.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, vp, vp, vp, sz, vp]
        lib.hmm_block_element.restype = ctypes.c_int
        lib.hmm_block_carries.argtypes = [vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, vp, vp, vp, vp]
        lib.hmm_block_carries.restype = ctypes.c_int
        lib.hmm_status_string.argtypes = [ctypes.c_int]
        lib.hmm_status_string.restype = ctypes.c_char_p
        lib.hmm_kernel_timing_enable.argtypes = [ctypes.c_int32]
        lib.hmm_kernel_timing_enable.restype = ctypes.c_int
        lib.hmm_kernel_timing_count.argtypes = []
        lib.hmm_kernel_timing_count.restype = ctypes.c_int32
        lib.hmm_kernel_timing_get.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_char_p),
                                              ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        lib.hmm_kernel_timing_get.restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(code: int) -> str:
    return load_library().hmm_status_string(int(code)).decode()


def hmm_workspace_bytes(T: int, D: int, batch: int):
    """Returns (smooth_bytes, viterbi_bytes)."""
    lib = load_library()
    s, v = ctypes.c_size_t(0), ctypes.c_size_t(0)
    rc = lib.hmm_workspace_bytes(int(T), int(D), int(batch), ctypes.byref(s), ctypes.byref(v))
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_workspace_bytes")
    return int(s.value), int(v.value)


WORKSPACE_RESERVED_BYTES = 384 * 1024


def hmm_workspace_init(workspace) -> None:
    """Zeroes the workspace's reserved leading bytes on torch's current stream (required once before the
    workspace's first use, and again after a call whose bounded wait ran out)."""
    rc = load_library().hmm_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_workspace_init")


def hmm_workspace_status(workspace) -> int:
    """0: ready; 1: a bounded wait ran out in an earlier call on this workspace (re-initialise it).  Synchronises."""
    state = ctypes.c_int32(0)
    rc = load_library().hmm_workspace_status(_ptr(workspace), _stream(), ctypes.byref(state))
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_workspace_status")
    return int(state.value)


def new_workspace(nbytes: int, device):
    """A device buffer of at least nbytes, prepared for its first use (allocation and hmm_workspace_init)."""
    import torch
    ws = torch.empty((max(int(nbytes), 256),), dtype=torch.uint8, device=device)
    hmm_workspace_init(ws)
    return ws


def hmm_kernel_timing_enable(on: bool) -> None:
    rc = load_library().hmm_kernel_timing_enable(1 if on else 0)
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_kernel_timing_enable")


def hmm_kernel_timing_get():
    """Returns {kernel name: (total_ms, launches)} for everything recorded since the last enable."""
    lib = load_library()
    out = {}
    for i in range(lib.hmm_kernel_timing_count()):
        name, ms, n = ctypes.c_char_p(), ctypes.c_double(0.0), ctypes.c_int64(0)
        rc = lib.hmm_kernel_timing_get(i, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(n))
        if rc != HMM_OK:
            raise HmmError(rc, "hmm_kernel_timing_get")
        out[name.value.decode()] = (float(ms.value), int(n.value))
    return out


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _check(t, dtype, shape, name):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous() \
            or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected contiguous device tensor {dtype} {tuple(shape)}, got "
                         f"{getattr(t, 'dtype', None)} {tuple(getattr(t, 'shape', ()))}")


def _shapes(prior, A, loglik):
    B, T, D = loglik.shape
    Bm = prior.shape[0]
    if Bm not in (1, B):
        raise ValueError("prior/A leading dimension must be 1 (shared) or batch")
    shared = 1 if (Bm == 1) else 0
    return B, T, D, Bm, shared


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class PreparedCall:
    """One C-ABI call with its arguments marshalled once: calling the object enqueues it again on the
    stream that was current at preparation.  For loops that repeat a call on the same buffers, where
    re-validating tensors and rebuilding ctypes arguments would cost more host time than the call."""

    def __init__(self, fn, where, cargs, keep, result):
        self._fn, self._where, self._cargs, self._keep, self.result = fn, where, cargs, keep, result

    def __call__(self):
        rc = self._fn(*self._cargs)
        if rc != HMM_OK:
            raise HmmError(rc, self._where)
        return self.result


def hmm_smooth_prepare(prior, A, loglik, marginals=None, filtered=None, loglik_out=None, workspace=None,
                       want_filtered: bool = False) -> PreparedCall:
    """Validates and marshals an hmm_smooth call; see hmm_smooth for the arguments."""
    import torch
    lib = load_library()
    B, T, D, Bm, shared = _shapes(prior, A, loglik)
    f32 = torch.float32
    _check(prior, f32, (Bm, D), "prior")
    _check(A, f32, (Bm, D, D), "A")
    _check(loglik, f32, (B, T, D), "loglik")
    dev = loglik.device
    if marginals is None:
        marginals = torch.empty((B, T, D), dtype=f32, device=dev)
    if filtered is None and want_filtered:
        filtered = torch.empty((B, T, D), dtype=f32, device=dev)
    if loglik_out is None:
        loglik_out = torch.empty((B,), dtype=torch.float64, device=dev)
    _check(marginals, f32, (B, T, D), "marginals")
    if filtered is not None:
        _check(filtered, f32, (B, T, D), "filtered")
    _check(loglik_out, torch.float64, (B,), "loglik_out")
    if workspace is None:
        workspace = new_workspace(hmm_workspace_bytes(T, D, B)[0], dev)
    cargs = (_ptr(prior), _ptr(A), _ptr(loglik), T, D, B, shared, _ptr(marginals), _ptr(filtered),
             _ptr(loglik_out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    return PreparedCall(lib.hmm_smooth, "hmm_smooth", cargs, (prior, A, loglik, workspace),
                        (marginals, filtered, loglik_out))


def hmm_smooth(prior, A, loglik, marginals=None, filtered=None, loglik_out=None, workspace=None,
               want_filtered: bool = False):
    """prior[Bm][D], A[Bm][D][D], loglik[B][T][D] float32 device tensors (Bm = 1 or B).
    Returns (marginals[B][T][D] f32, filtered or None, loglik_out[B] f64); asynchronous on
    torch's current stream."""
    return hmm_smooth_prepare(prior, A, loglik, marginals, filtered, loglik_out, workspace, want_filtered)()


STATIC_SCRATCH_BYTES = 4 << 20


def hmm_smooth_static(prior, A, loglik, marginals, loglik_out, filtered=None):
    """hmm_smooth on the library's own static scratch array: the caller passes every output (nothing is
    allocated here either).  Returns (marginals, filtered, loglik_out); asynchronous on torch's current stream."""
    import torch
    lib = load_library()
    B, T, D, Bm, shared = _shapes(prior, A, loglik)
    f32 = torch.float32
    _check(prior, f32, (Bm, D), "prior")
    _check(A, f32, (Bm, D, D), "A")
    _check(loglik, f32, (B, T, D), "loglik")
    _check(marginals, f32, (B, T, D), "marginals")
    if filtered is not None:
        _check(filtered, f32, (B, T, D), "filtered")
    _check(loglik_out, torch.float64, (B,), "loglik_out")
    rc = lib.hmm_smooth_static(_ptr(prior), _ptr(A), _ptr(loglik), T, D, B, shared, _ptr(marginals), _ptr(filtered),
                               _ptr(loglik_out), _stream())
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_smooth_static")
    return marginals, filtered, loglik_out


def hmm_viterbi_prepare(prior, A, loglik, path=None, logprob_out=None, workspace=None) -> PreparedCall:
    """Validates and marshals an hmm_viterbi call; see hmm_viterbi for the arguments."""
    import torch
    lib = load_library()
    B, T, D, Bm, shared = _shapes(prior, A, loglik)
    f32 = torch.float32
    _check(prior, f32, (Bm, D), "prior")
    _check(A, f32, (Bm, D, D), "A")
    _check(loglik, f32, (B, T, D), "loglik")
    dev = loglik.device
    if path is None:
        path = torch.empty((B, T), dtype=torch.int32, device=dev)
    if logprob_out is None:
        logprob_out = torch.empty((B,), dtype=torch.float64, device=dev)
    _check(path, torch.int32, (B, T), "path")
    _check(logprob_out, torch.float64, (B,), "logprob_out")
    if workspace is None:
        workspace = new_workspace(hmm_workspace_bytes(T, D, B)[1], dev)
    cargs = (_ptr(prior), _ptr(A), _ptr(loglik), T, D, B, shared, _ptr(path), _ptr(logprob_out),
             _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    return PreparedCall(lib.hmm_viterbi, "hmm_viterbi", cargs, (prior, A, loglik, workspace), (path, logprob_out))


def hmm_viterbi(prior, A, loglik, path=None, logprob_out=None, workspace=None):
    """Returns (path[B][T] int32, logprob_out[B] f64); asynchronous on torch's current stream."""
    return hmm_viterbi_prepare(prior, A, loglik, path, logprob_out, workspace)()


def hmm_max_product_prepare(prior, A, loglik, max_marginals=None, path=None, logprob_out=None, workspace=None,
                            want_path: bool = True) -> PreparedCall:
    """Validates and marshals an hmm_max_product call; see hmm_max_product for the arguments."""
    import torch
    lib = load_library()
    B, T, D, Bm, shared = _shapes(prior, A, loglik)
    f32 = torch.float32
    _check(prior, f32, (Bm, D), "prior")
    _check(A, f32, (Bm, D, D), "A")
    _check(loglik, f32, (B, T, D), "loglik")
    dev = loglik.device
    if max_marginals is None:
        max_marginals = torch.empty((B, T, D), dtype=f32, device=dev)
    if path is None and want_path:
        path = torch.empty((B, T), dtype=torch.int32, device=dev)
    if logprob_out is None:
        logprob_out = torch.empty((B,), dtype=torch.float64, device=dev)
    _check(max_marginals, f32, (B, T, D), "max_marginals")
    if path is not None:
        _check(path, torch.int32, (B, T), "path")
    _check(logprob_out, torch.float64, (B,), "logprob_out")
    if workspace is None:
        workspace = new_workspace(hmm_workspace_bytes(T, D, B)[0], dev)
    cargs = (_ptr(prior), _ptr(A), _ptr(loglik), T, D, B, shared, _ptr(max_marginals), _ptr(path),
             _ptr(logprob_out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    return PreparedCall(lib.hmm_max_product, "hmm_max_product", cargs, (prior, A, loglik, workspace),
                        (max_marginals, path, logprob_out))


def hmm_max_product(prior, A, loglik, max_marginals=None, path=None, logprob_out=None, workspace=None,
                    want_path: bool = True):
    """Returns (max_marginals[B][T][D] f32 (log, largest entry of a step is 0), path[B][T] int32 or None,
    logprob_out[B] f64); asynchronous on torch's current stream."""
    return hmm_max_product_prepare(prior, A, loglik, max_marginals, path, logprob_out, workspace, want_path)()


def hmm_transition_counts_workspace_bytes(T: int, D: int, batch: int) -> int:
    lib = load_library()
    n = ctypes.c_size_t(0)
    rc = lib.hmm_transition_counts_workspace_bytes(int(T), int(D), int(batch), ctypes.byref(n))
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_transition_counts_workspace_bytes")
    return int(n.value)


def hmm_transition_counts(A, filtered, marginals, counts=None, workspace=None):
    """A[Bm][D][D], filtered[B][T][D] and marginals[B][T][D] as returned by hmm_smooth.
    Returns counts[B][D][D] f64 (expected transition counts); asynchronous on torch's current stream."""
    import torch
    lib = load_library()
    B, T, D = marginals.shape
    Bm = A.shape[0]
    if Bm not in (1, B):
        raise ValueError("A's leading dimension must be 1 (shared) or batch")
    f32 = torch.float32
    _check(A, f32, (Bm, D, D), "A")
    _check(filtered, f32, (B, T, D), "filtered")
    _check(marginals, f32, (B, T, D), "marginals")
    dev = marginals.device
    if counts is None:
        counts = torch.empty((B, D, D), dtype=torch.float64, device=dev)
    _check(counts, torch.float64, (B, D, D), "counts")
    if workspace is None:
        workspace = new_workspace(hmm_transition_counts_workspace_bytes(T, D, B), dev)
    rc = lib.hmm_transition_counts(_ptr(A), _ptr(filtered), _ptr(marginals), T, D, B, 1 if Bm == 1 else 0, _ptr(counts),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_transition_counts")
    return counts


def hmm_smooth_counts_workspace_bytes(T: int, D: int, batch: int) -> int:
    lib = load_library()
    n = ctypes.c_size_t(0)
    rc = lib.hmm_smooth_counts_workspace_bytes(int(T), int(D), int(batch), ctypes.byref(n))
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_smooth_counts_workspace_bytes")
    return int(n.value)


def hmm_smooth_counts(prior, A, loglik, marginals=None, loglik_out=None, counts=None, workspace=None):
    """The expectation step in one call.  Returns (marginals[B][T][D] f32, loglik_out[B] f64, counts[B][D][D] f64);
    asynchronous on torch's current stream."""
    import torch
    lib = load_library()
    B, T, D, Bm, shared = _shapes(prior, A, loglik)
    f32 = torch.float32
    _check(prior, f32, (Bm, D), "prior")
    _check(A, f32, (Bm, D, D), "A")
    _check(loglik, f32, (B, T, D), "loglik")
    dev = loglik.device
    if marginals is None:
        marginals = torch.empty((B, T, D), dtype=f32, device=dev)
    if loglik_out is None:
        loglik_out = torch.empty((B,), dtype=torch.float64, device=dev)
    if counts is None:
        counts = torch.empty((B, D, D), dtype=torch.float64, device=dev)
    _check(marginals, f32, (B, T, D), "marginals")
    _check(loglik_out, torch.float64, (B,), "loglik_out")
    _check(counts, torch.float64, (B, D, D), "counts")
    if workspace is None:
        workspace = new_workspace(hmm_smooth_counts_workspace_bytes(T, D, B), dev)
    rc = lib.hmm_smooth_counts(_ptr(prior), _ptr(A), _ptr(loglik), T, D, B, shared, _ptr(marginals), _ptr(loglik_out),
                               _ptr(counts), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_smooth_counts")
    return marginals, loglik_out, counts


def hmm_block_element_workspace_bytes(T: int, D: int, batch: int) -> int:
    lib = load_library()
    n = ctypes.c_size_t(0)
    rc = lib.hmm_block_element_workspace_bytes(int(T), int(D), int(batch), ctypes.byref(n))
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_block_element_workspace_bytes")
    return int(n.value)


def hmm_block_element(A, loglik, max_product: bool = False, element=None, log_scale=None, workspace=None):
    """A[Bm][D][D], loglik[B][T][D]: the rows of one block of each sequence.  Returns (element[B][D][D] f32,
    log_scale[B] f64), the block's element under the sum-product or the max-product operator;
    asynchronous on torch's current stream."""
    import torch
    lib = load_library()
    B, T, D = loglik.shape
    Bm = A.shape[0]
    if Bm not in (1, B):
        raise ValueError("A's leading dimension must be 1 (shared) or batch")
    f32 = torch.float32
    _check(A, f32, (Bm, D, D), "A")
    _check(loglik, f32, (B, T, D), "loglik")
    dev = loglik.device
    if element is None:
        element = torch.empty((B, D, D), dtype=f32, device=dev)
    if log_scale is None:
        log_scale = torch.empty((B,), dtype=torch.float64, device=dev)
    _check(element, f32, (B, D, D), "element")
    _check(log_scale, torch.float64, (B,), "log_scale")
    if workspace is None:
        workspace = new_workspace(hmm_block_element_workspace_bytes(T, D, B), dev)
    rc = lib.hmm_block_element(_ptr(A), _ptr(loglik), T, D, B, 1 if Bm == 1 else 0, 1 if max_product else 0, _ptr(element),
                               _ptr(log_scale), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_block_element")
    return element, log_scale


def hmm_block_carries(prior, A, elements, log_scales, max_product: bool = False):
    """prior[Bm][D], A[Bm][D][D], elements[S][B][D][D] f32 and log_scales[S][B] f64 (hmm_block_element's
    outputs for the S consecutive blocks, stacked).  Returns (carry_rows[S][B][D], lookahead_rows[S][B][D],
    total[B] f64); asynchronous on torch's current stream."""
    import torch
    lib = load_library()
    S, B, D, _ = elements.shape
    Bm = prior.shape[0]
    if Bm not in (1, B):
        raise ValueError("prior/A leading dimension must be 1 (shared) or batch")
    f32 = torch.float32
    _check(prior, f32, (Bm, D), "prior")
    _check(A, f32, (Bm, D, D), "A")
    _check(elements, f32, (S, B, D, D), "elements")
    _check(log_scales, torch.float64, (S, B), "log_scales")
    dev = elements.device
    carry = torch.empty((S, B, D), dtype=f32, device=dev)
    look = torch.empty((S, B, D), dtype=f32, device=dev)
    total = torch.empty((B,), dtype=torch.float64, device=dev)
    rc = lib.hmm_block_carries(_ptr(prior), _ptr(A), _ptr(elements), _ptr(log_scales), S, D, B, 1 if Bm == 1 else 0,
                               1 if max_product else 0, _ptr(carry), _ptr(look), _ptr(total), _stream())
    if rc != HMM_OK:
        raise HmmError(rc, "hmm_block_carries")
    return carry, look, total
