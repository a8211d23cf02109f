/*
 * hmmscan -- HMM smoothing and Viterbi decoding as all-prefix-sums on AMD MI355X (gfx950).
 *
 * C ABI.  Every array argument is DEVICE memory owned by the caller; the library
 * allocates nothing and never synchronises: all work is enqueued on the caller's HIP
 * stream and outputs are valid once that stream has been synchronised.  Inputs are
 * never written; outputs and the workspace must not alias the inputs or each other.
 * All arrays are contiguous and row-major.
 *
 * Model (Sec. II of the paper): x_1 ~ prior, x_k ~ A[x_{k-1}][.], y_k ~ p(y_k | x_k),
 * states are 0-based, potentials psi_1(x_1) = p(y_1|x_1) p(x_1) and
 * psi_k(x_{k-1},x_k) = p(y_k|x_k) A[x_{k-1}][x_k].  Observations enter only
 * through loglik[b][t][j] = log p(y_{t+1} | x_{t+1} = j), which may hold -inf
 * (impossible) entries.  Zero entries in prior and A are legal.
 *
 * Errors are return codes only.  Argument errors are detected on the host before
 * anything is launched; a failed launch is reported as HMM_ERR_DEVICE.  A step
 * whose evidence is impossible under every state (a log-likelihood row that is
 * all -inf, or Z = 0) is not an error: the returned log-likelihood /
 * log-probability is then -inf or NaN and the marginals / path are unspecified.
 * Range: hmm_smooth works on probabilities in single precision, rescaled by exact
 * powers of two; the scale of every vector is kept apart from the mantissas, so the
 * only states lost are those a step-by-step forward-backward recursion in single
 * precision loses as well: a state whose filtered (or backward) probability falls
 * below 2^-126 of the step's largest becomes exactly zero.  For D <= 8 every ROW of
 * an aggregated product of potentials has its own scale (while all rows of an
 * aggregate stay within 2^20 of one another the kernels run a shorter code path
 * with one scale, and fall back per phase and wavefront otherwise).  Above eight
 * states the rows of an aggregate share a scale per strip of 16 or 32 rows; a
 * sequence whose carries meet rows far below that scale (a product of a carry and
 * an aggregate that comes out more than 2^32 below its factors, or a result that
 * is not a number) is computed again inside the same call by the step-by-step
 * recursion itself, one workgroup walking its T steps twice -- correct, and slow
 * for that sequence only.  The max-product calls work on logarithms.
 *
 * Workspaces.  The first HMM_WORKSPACE_RESERVED_BYTES of every workspace belong to
 * the library across calls: they MUST BE ZERO before the workspace's first use
 * (hmm_workspace_init does it on a stream; a zero-filled allocation is as good),
 * and nothing but this library may write there afterwards.  The rest of a workspace
 * is plain scratch: contents on entry are ignored, on exit undefined.  One
 * workspace may serve any sequence of calls of any shapes, one call at a time:
 * two calls must not use one workspace concurrently.
 *
 * Concurrency.  Calls may be enqueued back to back on one stream.  For small state
 * spaces (D <= 8), sequences longer than one tile (4096 steps at D <= 4, 2048
 * above) and shapes whose tiles all fit the device at once, a call is a
 * single kernel whose workgroups wait for one another's partial results (exchanged
 * through the reserved bytes), which needs them all resident together; the host
 * checks this against an otherwise idle device.  (Shorter sequences never wait for
 * one another.)  If other work (another stream, another process) occupies compute
 * units for the whole duration, the wait is bounded: the kernel then terminates by
 * itself, the call's log-likelihood / log-probability output is NaN (its other
 * outputs are then meaningless) and the workspace is marked: every later call of
 * this kind on it reports NaN at once until hmm_workspace_init has been called on
 * it again (hmm_workspace_status tells).  HMMSCAN_SPIN_LIMIT=<polls> overrides the
 * bound (0: give up at once, for exercising this path).  Setting the environment
 * variable HMMSCAN_PLAN=multi selects the plan without such waits for every shape.
 */
#ifndef HMMSCAN_H
#define HMMSCAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HMM_OK = 0,
    HMM_ERR_INVALID_ARG = 1,   /* null required pointer, T < 1, D < 1, batch < 1, misaligned array */
    HMM_ERR_UNSUPPORTED = 2,   /* D above HMM_MAX_STATES, or a shape the launch grid cannot hold  */
    HMM_ERR_WORKSPACE = 3,     /* workspace null or smaller than hmm_workspace_bytes reports      */
    HMM_ERR_DEVICE = 4         /* a HIP call or kernel launch failed                              */
} hmm_status;

/* Largest supported number of states D. */
#define HMM_MAX_STATES 128

/* Leading bytes of every workspace that the library keeps across calls (see "Workspaces" above). */
#define HMM_WORKSPACE_RESERVED_BYTES (384u * 1024u)

/*
 * Scratch size, in bytes, that hmm_smooth and hmm_viterbi need for this shape (the reserved
 * leading bytes included).  Pure host function (no device access).  Either output pointer may be NULL.
 */
hmm_status hmm_workspace_bytes(int64_t T, int32_t D, int32_t batch,
                               size_t* smooth_bytes, size_t* viterbi_bytes);

/*
 * Prepares a workspace for its first use, or for reuse after a call whose bounded wait ran out:
 * enqueues a zero fill of its first min(workspace_bytes, HMM_WORKSPACE_RESERVED_BYTES) bytes on the
 * stream (a kernel: it can be captured into a HIP graph like every other launch of the library).
 * workspace must be 256-byte aligned device memory.
 *
 * hmm_workspace_status copies the workspace's state word back to the host (it synchronises the
 * stream): *state = 0 ready, 1 a bounded wait ran out in an earlier call (re-initialise).
 */
hmm_status hmm_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);
hmm_status hmm_workspace_status(const void* workspace, void* hip_stream, int32_t* state);

/*
 * Smoothing marginals and log-likelihood by the parallel sum-product method
 * (Algorithm 3: element initialisation, forward all-prefix-sums and reversed
 * all-prefix-sums under the operator of Definition 3, then the marginal
 * p(x_k) = a_{0:k} a_{k:T+1} / Z_k).
 *
 *   prior      [shared_model ? 1 : batch][D]     p(x_1)
 *   A          [shared_model ? 1 : batch][D][D]  A[i][j] = p(x_k = j | x_{k-1} = i)
 *   loglik     [batch][T][D]
 *   marginals  [batch][T][D]  out: p(x_t | y_{1:T})
 *   filtered   [batch][T][D]  out, may be NULL: p(x_t | y_{1:t}) (the normalised forward potential)
 *   loglik_out [batch]        out: log p(y_{1:T}) = log Z (the partition function of Sec. II)
 *   workspace / workspace_bytes: device scratch of at least hmm_workspace_bytes(...).smooth_bytes,
 *              256-byte aligned, prepared once as described under "Workspaces" above
 *   hip_stream a hipStream_t (NULL = the default stream)
 *
 * loglik, marginals and filtered must be 16-byte aligned.  fp32 arithmetic
 * throughout, scale factors accumulated in fp64.
 */
hmm_status hmm_smooth(const float* prior, const float* A, const float* loglik,
                      int64_t T, int32_t D, int32_t batch, int32_t shared_model,
                      float* marginals, float* filtered, double* loglik_out,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * MAP state sequence (Viterbi path) by the parallel max-product method
 * (Algorithm 5's forward all-prefix-sums under the operator of Definition 5,
 * taken on logarithms), with the path recovered from the back-pointers
 * u_{k-1}(x_k) of Sec. IV-A by a reversed all-prefix-sums under function
 * composition, seeded with x*_T = argmax V_T.  Ties resolve to the lowest state.
 *
 *   path        [batch][T]  out: 0-based states x*_1..x*_T
 *   logprob_out [batch]     out: log p(y_{1:T}, x*_{1:T}) (Corollary 1: the joint, not the posterior)
 *   workspace: at least hmm_workspace_bytes(...).viterbi_bytes, 256-byte aligned
 * Other arguments as for hmm_smooth.
 */
hmm_status hmm_viterbi(const float* prior, const float* A, const float* loglik,
                       int64_t T, int32_t D, int32_t batch, int32_t shared_model,
                       int32_t* path, double* logprob_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Max-marginals and the per-step MAP states by the paper's parallel max-product
 * algorithm as printed (Algorithm 5): forward all-prefix-sums and reversed
 * all-prefix-sums under the operator of Definition 5 (on logarithms) give the
 * maximum forward and backward potentials psi~^f_k and psi~^b_k (the lemma of
 * Sec. IV-C), and Theorem 4 takes x*_k = argmax_{x_k} psi~^f_k(x_k) psi~^b_k(x_k).
 *
 *   max_marginals [batch][T][D]  out: log p*(x_t = j) - logprob_out, where p*(x_t) is the
 *                 max-marginal of Sec. II (the largest joint weight of a state sequence that
 *                 passes through j at step t): every entry is <= 0 and the step's largest is 0
 *   path          [batch][T]     out, may be NULL: per-step maximiser (lowest state on ties).
 *                 With a unique MAP sequence this is the Viterbi path (Theorem 4); with tied
 *                 sequences the per-step choice may splice several of them -- use hmm_viterbi
 *                 when one consistent path is required
 *   logprob_out   [batch]        out: log of the largest joint weight, as in hmm_viterbi
 *   workspace: at least hmm_workspace_bytes(...).smooth_bytes, 256-byte aligned
 * Other arguments as for hmm_smooth; loglik and max_marginals must be 16-byte aligned.
 */
hmm_status hmm_max_product(const float* prior, const float* A, const float* loglik,
                           int64_t T, int32_t D, int32_t batch, int32_t shared_model,
                           float* max_marginals, int32_t* path, double* logprob_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Expected transition counts, the statistic of the Baum-Welch expectation step for
 * the transition matrix (Sec. V-C: the expectation step is the forward-backward
 * recursion, i.e. hmm_smooth, followed by this sum):
 *     counts[b][i][j] = sum_{k=2..T} p(x_{k-1} = i, x_k = j | y_{1:T}).
 * It is formed from hmm_smooth's own outputs: with pred_k(j) = sum_i filtered_{k-1}(i) A[i][j],
 *     counts[i][j] = A[i][j] * sum_k filtered_{k-1}(i) * marginals_k(j) / pred_k(j).
 * (The other statistics of the expectation step are the marginals themselves: their first row
 * for the prior, their sums against the observations for the emission model.)
 *
 *   A          as for hmm_smooth
 *   filtered   [batch][T][D]  hmm_smooth's filtered output
 *   marginals  [batch][T][D]  hmm_smooth's marginals output
 *   counts     [batch][D][D]  out, fp64; all zero for T = 1
 *   workspace: at least hmm_transition_counts_workspace_bytes(...), 256-byte aligned
 */
hmm_status hmm_transition_counts_workspace_bytes(int64_t T, int32_t D, int32_t batch, size_t* bytes);
hmm_status hmm_transition_counts(const float* A, const float* filtered, const float* marginals,
                                 int64_t T, int32_t D, int32_t batch, int32_t shared_model,
                                 double* counts,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * hmm_smooth and the expected transition counts in one call (the whole expectation step of Sec. V-C).
 *   marginals[B][T][D], loglik_out[B]: as hmm_smooth.  counts[B][D][D] (fp64): as hmm_transition_counts.
 * Up to eight states the smoother's backward recursion itself sums the pairwise posteriors
 * p(x_{k-1}=i, x_k=j | y) = psi^f_{k-1}(i) psi_k(i,j) psi^b_k(j) / Z from the scaled potentials it holds in
 * registers: no filtering distributions in memory, no second pass, and a state whose normalised probability
 * lies below single-precision range still contributes (sequences of at most 1024 steps at D <= 4, 512 above,
 * take a workgroup each here instead of sharing one).  Above eight states the call runs hmm_smooth (filtering
 * distributions into the workspace) followed by hmm_transition_counts.
 * Workspace: hmm_smooth_counts_workspace_bytes (includes the reserved bytes); same rules as hmm_smooth.
 * Errors as hmm_smooth, plus HMM_ERR_INVALID_ARG for a null counts pointer.
 */
hmm_status hmm_smooth_counts_workspace_bytes(int64_t T, int32_t D, int32_t batch, size_t* bytes);
hmm_status hmm_smooth_counts(const float* prior, const float* A, const float* loglik,
                             int64_t T, int32_t D, int32_t batch, int32_t shared_model,
                             float* marginals, double* loglik_out, double* counts,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Block-wise processing (Sec. V-B: a block of consecutive observations and states is ONE element of
 * the scan).  For sequences that are not resident in device memory as a whole, or whose blocks are
 * processed in different places: every block is reduced to its element, the elements give the
 * carries between blocks, and each block is then processed on its own with the calls above.
 *
 * hmm_block_element: the element of the block with log-likelihood rows loglik[b][0..T-1],
 *     W(i, j) = sum (max_product = 0; Definition 3) or max (max_product != 0; Definition 5) over the
 *               states between of  e_1(x_1) prod_{k=2..T} A[x_{k-1}][x_k] e_k(x_k),  x_1 = i, x_T = j,
 * with e_k(x) = exp(loglik[k-1][x]): the joint weight of the block's observations and its last state
 * given its first state.  No transition enters the block's first step: adjacent blocks combine as
 * W_a (x) A (x) W_b.
 *   element   [batch][D][D]  out: W * exp(-log_scale) with its largest entry in [0.5, 1)  (sum-product),
 *                                 log W - log_scale with its largest entry 0              (max-product)
 *   log_scale [batch]        out (fp64); -inf if no state sequence of the block has any weight
 *   workspace: at least hmm_block_element_workspace_bytes(...), 256-byte aligned
 * A, loglik, shared_model, hip_stream as for hmm_smooth (loglik 16-byte aligned).
 *
 * hmm_block_carries: from the elements of the num_blocks consecutive blocks of each sequence,
 *   elements   [num_blocks][batch][D][D], log_scales [num_blocks][batch]   (hmm_block_element's outputs, stacked)
 *   carry_rows     [num_blocks][batch][D]  out: row s (s >= 1) = log of the forward potential at the last
 *                  step of block s-1 (sum-product: log p(x | y up to there); max-product: V shifted to
 *                  maximum 0); row 0 = log of the prior scaled to maximum one, for completeness
 *   lookahead_rows [num_blocks][batch][D]  out: row s (s <= num_blocks-2) = log of the backward potential
 *                  at the first step of block s+1 including that step's emission factor, shifted to
 *                  maximum 0; the last row is zero
 *   total      [batch]  out (fp64): log p(y_{1:T}) (sum-product) / log of the largest joint weight (max-product)
 * No workspace.  Rows may hold -inf.
 *
 * Using the rows: block s of a sequence is processed by hmm_smooth / hmm_viterbi / hmm_max_product on the
 * rows [carry_rows[s] ; the block's own rows ; lookahead_rows[s]] (no carry row and the true prior for
 * s = 0, a prior of all ones otherwise; no lookahead row for the last block).  The results on the
 * block's own steps are then those of the whole sequence: marginals, filtered distributions,
 * max-marginals, and the MAP path if it is unique (with tied MAP sequences, pass the one-hot row of the
 * next block's first decoded state as lookahead instead, last block first, to get one consistent
 * path).  The per-block log-likelihood / log-probability outputs of those calls refer to the framed
 * rows and are superseded by `total`.
 */
hmm_status hmm_block_element_workspace_bytes(int64_t T, int32_t D, int32_t batch, size_t* bytes);
hmm_status hmm_block_element(const float* A, const float* loglik, int64_t T, int32_t D, int32_t batch,
                             int32_t shared_model, int32_t max_product,
                             float* element, double* log_scale,
                             void* workspace, size_t workspace_bytes, void* hip_stream);
hmm_status hmm_block_carries(const float* prior, const float* A, const float* elements, const double* log_scales,
                             int32_t num_blocks, int32_t D, int32_t batch, int32_t shared_model, int32_t max_product,
                             float* carry_rows, float* lookahead_rows, double* total, void* hip_stream);

/*
 * hmm_smooth for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Identical to hmm_smooth (same kernels, same
 * outputs) except that the scratch memory is not an argument: it is a device array of
 * HMM_STATIC_SCRATCH_BYTES bytes inside the library itself, one copy on every GPU that loads the
 * library, held until the process ends.  The call allocates and frees nothing.
 *
 *   Shapes whose hmm_workspace_bytes(...).smooth_bytes exceeds HMM_STATIC_SCRATCH_BYTES are refused
 *   with HMM_ERR_WORKSPACE before anything is launched (every D <= 8 shape up to millions of steps
 *   fits; large D needs per-step scratch and fits only short sequences).
 *   The first call on a device looks the array's address up once (no allocation, but make that
 *   call outside a graph capture).
 *   All calls on one GPU share that GPU's array, whose contents carry over from call to call (it
 *   starts out zero, as a workspace must, and the library keeps its reserved bytes consistent from
 *   then on): calls that overlap on one GPU -- two streams, two host threads -- race and must be
 *   serialised by the caller.  Calls on different GPUs are independent.
 * Other arguments, alignment rules and error codes as for hmm_smooth.
 */
#define HMM_STATIC_SCRATCH_BYTES (4u << 20)
hmm_status hmm_smooth_static(const float* prior, const float* A, const float* loglik,
                             int64_t T, int32_t D, int32_t batch, int32_t shared_model,
                             float* marginals, float* filtered, double* loglik_out,
                             void* hip_stream);

/* Static, human-readable name of a status code (an hmm_status; any other integer gives "HMM_ERR_UNKNOWN"). */
const char* hmm_status_string(int32_t status);

/*
 * Measurement aid (not part of the method): per-kernel timing with HIP events.
 * hmm_kernel_timing_enable(1) clears earlier records and makes every later kernel launch of the
 * library carry a start and a stop HIP event attached to that kernel's own dispatch on the
 * caller's stream (hipExtLaunchKernel), so their difference is the kernel's execution time;
 * hmm_kernel_timing_enable(0) switches recording off and clears the records.
 * hmm_kernel_timing_count() waits for the recorded events and returns the number of distinct
 * kernels seen; hmm_kernel_timing_get(i, ...) returns, for the i-th of them, a static name, the
 * summed elapsed time in milliseconds and the number of launches.  Process-global, not
 * thread-safe, and the only state the library keeps; events are created on first use and reused.
 */
hmm_status hmm_kernel_timing_enable(int32_t on);
int32_t hmm_kernel_timing_count(void);
hmm_status hmm_kernel_timing_get(int32_t index, const char** name, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* HMMSCAN_H */
