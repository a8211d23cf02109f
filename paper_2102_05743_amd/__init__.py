"""HMM smoothing and Viterbi decoding as parallel scans on AMD MI355X (gfx950).

``binding`` wraps the C-ABI HIP library (libhmmscan.so); ``workloads`` holds the
seeded synthetic inputs; ``build`` compiles the library in-tree.
"""
from .binding import (HmmError, PreparedCall, hmm_block_carries, hmm_block_element, hmm_block_element_workspace_bytes, hmm_kernel_timing_enable, hmm_kernel_timing_get,  # noqa: F401
                      hmm_max_product, hmm_max_product_prepare, hmm_smooth, hmm_smooth_prepare, hmm_smooth_counts, hmm_smooth_counts_workspace_bytes, hmm_smooth_static, hmm_transition_counts, hmm_transition_counts_workspace_bytes, hmm_viterbi, hmm_viterbi_prepare, hmm_workspace_bytes, hmm_workspace_init, hmm_workspace_status, new_workspace,
                      load_library, status_string)
