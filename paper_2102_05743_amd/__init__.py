"""HMM smoothing and Viterbi decoding as parallel scans on AMD MI355X (gfx950).

``binding`` wraps the C-ABI HIP library (libhmmscan.so); ``workloads`` holds the
seeded synthetic inputs; ``build`` compiles the library in-tree.
"""
from .binding import (HmmError, hmm_smooth, hmm_viterbi, hmm_workspace_bytes, load_library,  # noqa: F401
                      status_string)
