"""HMM smoothing and Viterbi decoding as parallel scans on AMD MI355X (gfx950).

``binding`` wraps the C-ABI HIP library (libhmmscan.so); ``workloads`` holds the
seeded synthetic inputs; ``build`` compiles the library in-tree.
"""
from .binding import (HmmError, hmm_kernel_timing_enable, hmm_kernel_timing_get, hmm_smooth,  # noqa: F401
                      hmm_viterbi, hmm_workspace_bytes, load_library, status_string)
