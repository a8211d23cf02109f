// Dispatch of the register-resident path by state-space size.
#include "small_d.hpp"

namespace hmm {

#ifdef HMM_ONLY_SMALL_D
// A library that holds one state-space size only (the tile-size variant that the tests compare with the full
// library): every other size is reported as unsupported.
extern template struct SmallD<HMM_ONLY_SMALL_D>;

#define HMM_DISPATCH_SMALL_D(D_, CALL) \
    if ((D_) == HMM_ONLY_SMALL_D) return SmallD<HMM_ONLY_SMALL_D>::CALL;
#else
extern template struct SmallD<1>;
extern template struct SmallD<2>;
extern template struct SmallD<3>;
extern template struct SmallD<4>;
extern template struct SmallD<5>;
extern template struct SmallD<6>;
extern template struct SmallD<7>;
extern template struct SmallD<8>;

#define HMM_DISPATCH_SMALL_D(D_, CALL) \
    switch (D_) {                      \
        case 1: return SmallD<1>::CALL; \
        case 2: return SmallD<2>::CALL; \
        case 3: return SmallD<3>::CALL; \
        case 4: return SmallD<4>::CALL; \
        case 5: return SmallD<5>::CALL; \
        case 6: return SmallD<6>::CALL; \
        case 7: return SmallD<7>::CALL; \
        case 8: return SmallD<8>::CALL; \
        default: break;                \
    }
#endif

size_t small_d_smooth_ws_bytes(int D, long long T, int batch) {
    HMM_DISPATCH_SMALL_D(D, smooth_ws_bytes(T, batch))
    return 0;
}

size_t small_d_viterbi_ws_bytes(int D, long long T, int batch) {
    HMM_DISPATCH_SMALL_D(D, viterbi_ws_bytes(T, batch))
    return 0;
}

int small_d_smooth(int D, const SmallArgs& a, float* marg, float* filt, double* loglik_out) {
    HMM_DISPATCH_SMALL_D(D, smooth(a, marg, filt, loglik_out))
    return 2;
}

int small_d_smooth_pairs(int D, const SmallArgs& a, float* marg, double* loglik_out, float* pair_partial, long long* tiles) {
    HMM_DISPATCH_SMALL_D(D, smooth_pairs(a, marg, loglik_out, pair_partial, tiles))
    return 2;
}

long long small_d_tiles(int D, long long T) {
    HMM_DISPATCH_SMALL_D(D, tiles(T))
    return 0;
}

int small_d_viterbi(int D, const SmallArgs& a, int32_t* path, double* logprob_out) {
    HMM_DISPATCH_SMALL_D(D, viterbi(a, path, logprob_out))
    return 2;
}

int small_d_max_product(int D, const SmallArgs& a, float* maxmarg, int32_t* path, double* logprob_out) {
    HMM_DISPATCH_SMALL_D(D, max_product(a, maxmarg, path, logprob_out))
    return 2;
}

size_t small_d_element_ws_bytes(int D, long long T, int batch) {
    HMM_DISPATCH_SMALL_D(D, element_ws_bytes(T, batch))
    return 0;
}

int small_d_block_element(int D, const SmallArgs& a, int max_product, float* element, double* log_scale) {
    HMM_DISPATCH_SMALL_D(D, block_element(a, max_product, element, log_scale))
    return 2;
}

}  // namespace hmm
