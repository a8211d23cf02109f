// C ABI of the library: argument validation and dispatch by state-space size.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hmmscan.h"
#include "blocks.hpp"
#include "estep.hpp"
#include "large_d.hpp"
#include "small_d.hpp"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Every workspace starts with HMM_WORKSPACE_RESERVED_BYTES that only the single-launch kernels of the
// small state spaces write (tagged exchange words); all other scratch lies behind it.
constexpr size_t RESERVED = hmm::XCH_REGION_BYTES;
static_assert(RESERVED == HMM_WORKSPACE_RESERVED_BYTES, "header and library disagree on the reserved region");
char* behind_reserved(void* ws) { return static_cast<char*>(ws) + RESERVED; }

hmm_status check_common(const float* prior, const float* A, const float* loglik, int64_t T, int32_t D,
                        int32_t batch) {
    if (!prior || !A || !loglik) return HMM_ERR_INVALID_ARG;
    if (T < 1 || D < 1 || batch < 1) return HMM_ERR_INVALID_ARG;
    if (D > HMM_MAX_STATES) return HMM_ERR_UNSUPPORTED;
    if (!aligned16(loglik)) return HMM_ERR_INVALID_ARG;
    return HMM_OK;
}

}  // namespace

extern "C" {

hmm_status hmm_workspace_bytes(int64_t T, int32_t D, int32_t batch, size_t* smooth_bytes, size_t* viterbi_bytes) {
    if (T < 1 || D < 1 || batch < 1) return HMM_ERR_INVALID_ARG;
    if (D > HMM_MAX_STATES) return HMM_ERR_UNSUPPORTED;
    size_t s = 0, v = 0;
    if (D <= hmm::SMALL_D_MAX) {
        s = hmm::small_d_smooth_ws_bytes(D, T, batch);     // these include the reserved region
        v = hmm::small_d_viterbi_ws_bytes(D, T, batch);
    } else {
        s = hmm::large_d_smooth_ws_bytes(D, T, batch);
        const size_t mp = hmm::large_d_max_product_ws_bytes(D, T, batch);   // hmm_max_product shares smooth_bytes
        if (mp > s) s = mp;
        v = hmm::large_d_viterbi_ws_bytes(D, T, batch);
        s += RESERVED;
        v += RESERVED;
    }
    if (smooth_bytes) *smooth_bytes = s;
    if (viterbi_bytes) *viterbi_bytes = v;
    return HMM_OK;
}

hmm_status hmm_smooth(const float* prior, const float* A, const float* loglik, int64_t T, int32_t D, int32_t batch,
                      int32_t shared_model, float* marginals, float* filtered, double* loglik_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    hmm_status st = check_common(prior, A, loglik, T, D, batch);
    if (st != HMM_OK) return st;
    if (!marginals || !loglik_out) return HMM_ERR_INVALID_ARG;
    if (!aligned16(marginals) || (filtered && !aligned16(filtered))) return HMM_ERR_INVALID_ARG;
    size_t need = 0;
    st = hmm_workspace_bytes(T, D, batch, &need, nullptr);
    if (st != HMM_OK) return st;
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return HMM_ERR_WORKSPACE;
    if (D > hmm::SMALL_D_MAX) {
        hmm::LargeArgs la{prior, A, loglik, (long long)T, D, batch, shared_model ? 1 : 0, behind_reserved(workspace),
                          workspace_bytes - RESERVED, static_cast<hipStream_t>(hip_stream)};
        return static_cast<hmm_status>(hmm::large_d_smooth(la, marginals, filtered, loglik_out));
    }
    hmm::SmallArgs a{prior, A, loglik, (long long)T, batch, shared_model ? 1 : 0, workspace, workspace_bytes,
                     static_cast<hipStream_t>(hip_stream)};
    return static_cast<hmm_status>(hmm::small_d_smooth(D, a, marginals, filtered, loglik_out));
}

hmm_status hmm_viterbi(const float* prior, const float* A, const float* loglik, int64_t T, int32_t D, int32_t batch,
                       int32_t shared_model, int32_t* path, double* logprob_out, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
    hmm_status st = check_common(prior, A, loglik, T, D, batch);
    if (st != HMM_OK) return st;
    if (!path || !logprob_out) return HMM_ERR_INVALID_ARG;
    size_t need = 0;
    st = hmm_workspace_bytes(T, D, batch, nullptr, &need);
    if (st != HMM_OK) return st;
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return HMM_ERR_WORKSPACE;
    if (D > hmm::SMALL_D_MAX) {
        hmm::LargeArgs la{prior, A, loglik, (long long)T, D, batch, shared_model ? 1 : 0, behind_reserved(workspace),
                          workspace_bytes - RESERVED, static_cast<hipStream_t>(hip_stream)};
        return static_cast<hmm_status>(hmm::large_d_viterbi(la, path, logprob_out));
    }
    hmm::SmallArgs a{prior, A, loglik, (long long)T, batch, shared_model ? 1 : 0, workspace, workspace_bytes,
                     static_cast<hipStream_t>(hip_stream)};
    return static_cast<hmm_status>(hmm::small_d_viterbi(D, a, path, logprob_out));
}

hmm_status hmm_max_product(const float* prior, const float* A, const float* loglik, int64_t T, int32_t D,
                           int32_t batch, int32_t shared_model, float* max_marginals, int32_t* path,
                           double* logprob_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    hmm_status st = check_common(prior, A, loglik, T, D, batch);
    if (st != HMM_OK) return st;
    if (!max_marginals || !logprob_out) return HMM_ERR_INVALID_ARG;
    if (!aligned16(max_marginals)) return HMM_ERR_INVALID_ARG;
    size_t need = 0;
    st = hmm_workspace_bytes(T, D, batch, &need, nullptr);
    if (st != HMM_OK) return st;
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return HMM_ERR_WORKSPACE;
    if (D > hmm::SMALL_D_MAX) {
        hmm::LargeArgs la{prior, A, loglik, (long long)T, D, batch, shared_model ? 1 : 0, behind_reserved(workspace),
                          workspace_bytes - RESERVED, static_cast<hipStream_t>(hip_stream)};
        return static_cast<hmm_status>(hmm::large_d_max_product(la, max_marginals, path, logprob_out));
    }
    hmm::SmallArgs a{prior, A, loglik, (long long)T, batch, shared_model ? 1 : 0, workspace, workspace_bytes,
                     static_cast<hipStream_t>(hip_stream)};
    return static_cast<hmm_status>(hmm::small_d_max_product(D, a, max_marginals, path, logprob_out));
}

hmm_status hmm_transition_counts_workspace_bytes(int64_t T, int32_t D, int32_t batch, size_t* bytes) {
    if (T < 1 || D < 1 || batch < 1 || !bytes) return HMM_ERR_INVALID_ARG;
    if (D > HMM_MAX_STATES) return HMM_ERR_UNSUPPORTED;
    *bytes = hmm::transition_counts_ws_bytes(D, T, batch) + RESERVED;
    return HMM_OK;
}

hmm_status hmm_transition_counts(const float* A, const float* filtered, const float* marginals, int64_t T, int32_t D,
                                 int32_t batch, int32_t shared_model, double* counts, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
    if (!A || !filtered || !marginals || !counts) return HMM_ERR_INVALID_ARG;
    if (T < 1 || D < 1 || batch < 1) return HMM_ERR_INVALID_ARG;
    if (D > HMM_MAX_STATES) return HMM_ERR_UNSUPPORTED;
    const size_t need = hmm::transition_counts_ws_bytes(D, T, batch) + RESERVED;
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return HMM_ERR_WORKSPACE;
    hmm::EstepArgs a{A, filtered, marginals, (long long)T, D, batch, shared_model ? 1 : 0, behind_reserved(workspace),
                     workspace_bytes - RESERVED, static_cast<hipStream_t>(hip_stream)};
    return static_cast<hmm_status>(hmm::transition_counts(a, counts));
}

namespace {
size_t align256(size_t x) { return (x + 255) / 256 * 256; }
// Workspace of hmm_smooth_counts: the smoother's own, then either the per-tile pair sums (D <= 8, sequences
// longer than the packed plan takes) or, for the two-call form, the filtering distributions and the scratch of
// the counting kernels.
struct CountsWs { size_t smooth, extra, total; };
CountsWs counts_ws(int64_t T, int32_t D, int32_t batch) {
    CountsWs w{0, 0, 0};
    hmm_workspace_bytes(T, D, batch, &w.smooth, nullptr);
    w.extra = align256(w.smooth);
    const size_t two_calls = align256((size_t)T * D * batch * sizeof(float)) + hmm::transition_counts_ws_bytes(D, T, batch);
    size_t pairs = 0;
    if (D <= hmm::SMALL_D_MAX) pairs = (size_t)hmm::small_d_tiles(D, T) * batch * D * D * sizeof(float);
    w.total = w.extra + (two_calls > pairs ? two_calls : pairs);
    return w;
}
}  // namespace

hmm_status hmm_smooth_counts_workspace_bytes(int64_t T, int32_t D, int32_t batch, size_t* bytes) {
    if (T < 1 || D < 1 || batch < 1 || !bytes) return HMM_ERR_INVALID_ARG;
    if (D > HMM_MAX_STATES) return HMM_ERR_UNSUPPORTED;
    *bytes = counts_ws(T, D, batch).total;
    return HMM_OK;
}

hmm_status hmm_smooth_counts(const float* prior, const float* A, const float* loglik, int64_t T, int32_t D, int32_t batch,
                             int32_t shared_model, float* marginals, double* loglik_out, double* counts, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
    hmm_status st = check_common(prior, A, loglik, T, D, batch);
    if (st != HMM_OK) return st;
    if (!marginals || !loglik_out || !counts || !aligned16(marginals)) return HMM_ERR_INVALID_ARG;
    const CountsWs w = counts_ws(T, D, batch);
    if (!workspace || workspace_bytes < w.total || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return HMM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char* extra = static_cast<char*>(workspace) + w.extra;
    if (D <= hmm::SMALL_D_MAX) {
        // one pass: the smoother's backward recursion sums the pairwise posteriors where it has both potentials
        hmm::SmallArgs a{prior, A, loglik, (long long)T, batch, shared_model ? 1 : 0, workspace, w.smooth, stream};
        long long tiles = 0;
        const int rc = hmm::small_d_smooth_pairs(D, a, marginals, loglik_out, reinterpret_cast<float*>(extra), &tiles);
        if (rc != 0) return static_cast<hmm_status>(rc);
        return static_cast<hmm_status>(
            hmm::reduce_pair_partials(reinterpret_cast<const float*>(extra), (int)tiles, D, batch, counts, stream));
    }
    float* filtered = reinterpret_cast<float*>(extra);
    st = hmm_smooth(prior, A, loglik, T, D, batch, shared_model, marginals, filtered, loglik_out, workspace, w.smooth, hip_stream);
    if (st != HMM_OK) return st;
    char* tc = extra + align256((size_t)T * D * batch * sizeof(float));
    hmm::EstepArgs e{A, filtered, marginals, (long long)T, D, batch, shared_model ? 1 : 0, tc,
                     workspace_bytes - (size_t)(tc - static_cast<char*>(workspace)), stream};
    return static_cast<hmm_status>(hmm::transition_counts(e, counts));
}

hmm_status hmm_block_element_workspace_bytes(int64_t T, int32_t D, int32_t batch, size_t* bytes) {
    if (T < 1 || D < 1 || batch < 1 || !bytes) return HMM_ERR_INVALID_ARG;
    if (D > HMM_MAX_STATES) return HMM_ERR_UNSUPPORTED;
    if (D <= hmm::SMALL_D_MAX) {
        *bytes = hmm::small_d_element_ws_bytes(D, T, batch);
    } else {
        const size_t sp = hmm::large_d_element_sp_ws_bytes(D, T, batch), mp = hmm::large_d_element_mp_ws_bytes(D, T, batch);
        *bytes = (sp > mp ? sp : mp) + RESERVED;
    }
    return HMM_OK;
}

hmm_status hmm_block_element(const float* A, const float* loglik, int64_t T, int32_t D, int32_t batch,
                             int32_t shared_model, int32_t max_product, float* element, double* log_scale,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!A || !loglik || !element || !log_scale) return HMM_ERR_INVALID_ARG;
    if (T < 1 || D < 1 || batch < 1) return HMM_ERR_INVALID_ARG;
    if (D > HMM_MAX_STATES) return HMM_ERR_UNSUPPORTED;
    if (!aligned16(loglik)) return HMM_ERR_INVALID_ARG;
    size_t need = 0;
    hmm_status st = hmm_block_element_workspace_bytes(T, D, batch, &need);
    if (st != HMM_OK) return st;
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return HMM_ERR_WORKSPACE;
    if (D > hmm::SMALL_D_MAX) {
        hmm::LargeArgs la{nullptr, A, loglik, (long long)T, D, batch, shared_model ? 1 : 0, behind_reserved(workspace),
                          workspace_bytes - RESERVED, static_cast<hipStream_t>(hip_stream)};
        return static_cast<hmm_status>(max_product ? hmm::large_d_element_mp(la, element, log_scale)
                                                   : hmm::large_d_element_sp(la, element, log_scale));
    }
    hmm::SmallArgs a{nullptr, A, loglik, (long long)T, batch, shared_model ? 1 : 0, workspace, workspace_bytes,
                     static_cast<hipStream_t>(hip_stream)};
    return static_cast<hmm_status>(hmm::small_d_block_element(D, a, max_product ? 1 : 0, element, log_scale));
}

hmm_status hmm_block_carries(const float* prior, const float* A, const float* elements, const double* log_scales,
                             int32_t num_blocks, int32_t D, int32_t batch, int32_t shared_model, int32_t max_product,
                             float* carry_rows, float* lookahead_rows, double* total, void* hip_stream) {
    if (!prior || !A || !elements || !log_scales || !carry_rows || !lookahead_rows || !total) return HMM_ERR_INVALID_ARG;
    if (num_blocks < 1 || D < 1 || batch < 1) return HMM_ERR_INVALID_ARG;
    if (D > HMM_MAX_STATES) return HMM_ERR_UNSUPPORTED;
    hmm::BlockCarryArgs a{prior, A, elements, log_scales, num_blocks, D, batch, shared_model ? 1 : 0, max_product ? 1 : 0,
                          static_cast<hipStream_t>(hip_stream)};
    return static_cast<hmm_status>(hmm::block_carries(a, carry_rows, lookahead_rows, total));
}

hmm_status hmm_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return HMM_ERR_WORKSPACE;
    const size_t n = workspace_bytes < RESERVED ? workspace_bytes : RESERVED;
    return static_cast<hmm_status>(hmm::small_d_zero_region(workspace, n, static_cast<hipStream_t>(hip_stream)));
}

hmm_status hmm_workspace_status(const void* workspace, void* hip_stream, int32_t* state) {
    if (!workspace || !state) return HMM_ERR_INVALID_ARG;
    uint32_t header[4] = {0u, 0u, 0u, 0u};   // generation, poison flag, finished-sequence counter, padding
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(header, workspace, sizeof(header), hipMemcpyDeviceToHost, st) != hipSuccess) return HMM_ERR_DEVICE;
    if (hipStreamSynchronize(st) != hipSuccess) return HMM_ERR_DEVICE;
    *state = header[1] != 0u ? 1 : 0;
    return HMM_OK;
}

const char* hmm_status_string(int32_t status) {   // (an integer, not the enum: callers may pass anything)
    switch (status) {
        case HMM_OK: return "HMM_OK";
        case HMM_ERR_INVALID_ARG: return "HMM_ERR_INVALID_ARG";
        case HMM_ERR_UNSUPPORTED: return "HMM_ERR_UNSUPPORTED";
        case HMM_ERR_WORKSPACE: return "HMM_ERR_WORKSPACE";
        case HMM_ERR_DEVICE: return "HMM_ERR_DEVICE";
    }
    return "HMM_ERR_UNKNOWN";
}

}  // extern "C"
