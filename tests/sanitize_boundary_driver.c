/* Host-only sanitizer driver for the C ABI: every entry point is called with arguments that fail validation
 * (so nothing is launched and no GPU is needed), and the pure-host size queries are swept over many shapes.
 * Built with the boundary's host code under AddressSanitizer and UndefinedBehaviorSanitizer and run by
 * tests/test_boundary_sanitizers.py; exit status 0 = every return code as expected and no report. */
#include <stdint.h>
#include <stdio.h>

#include "../include/hmmscan.h"

static int failures = 0;
#define EXPECT(call, code) do { int rc_ = (int)(call); if (rc_ != (code)) { printf("line %d: got %d, expected %d\n", __LINE__, rc_, (code)); ++failures; } } while (0)

int main(void)
{
    float *fake = (float *)0x1000, *odd = (float *)0x1004;
    double *fd = (double *)0x1000;
    int32_t *fi = (int32_t *)0x1000;
    void *ws = (void *)0x2000, *badws = (void *)0x1010;
    const size_t big = (size_t)1 << 20;

    /* size queries: pure host arithmetic over the planners of every path */
    static const int Ds[] = {1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 32, 33, 64, 100, 128};
    static const long long Ts[] = {1, 2, 63, 64, 1000, 4096, 4097, 65536, 1 << 20, (1 << 23) + 5, 1LL << 31};
    static const int Bs[] = {1, 2, 19, 256, 70000};
    for (unsigned a = 0; a < sizeof Ds / sizeof *Ds; ++a)
        for (unsigned b = 0; b < sizeof Ts / sizeof *Ts; ++b)
            for (unsigned c = 0; c < sizeof Bs / sizeof *Bs; ++c) {
                size_t s = 0, v = 0, e = 0, t = 0;
                int rc = (int)hmm_workspace_bytes(Ts[b], Ds[a], Bs[c], &s, &v);
                if (rc == HMM_OK && (s < HMM_WORKSPACE_RESERVED_BYTES || v < HMM_WORKSPACE_RESERVED_BYTES)) {
                    printf("workspace below the reserved bytes at D=%d T=%lld B=%d\n", Ds[a], Ts[b], Bs[c]);
                    ++failures;
                }
                if (rc != HMM_OK && rc != HMM_ERR_UNSUPPORTED) { printf("hmm_workspace_bytes rc %d\n", rc); ++failures; }
                (void)hmm_transition_counts_workspace_bytes(Ts[b], Ds[a], Bs[c], &t);
                (void)hmm_block_element_workspace_bytes(Ts[b], Ds[a], Bs[c], &e);
            }
    {
        size_t s = 0, v = 0;
        EXPECT(hmm_workspace_bytes(0, 4, 1, &s, &v), HMM_ERR_INVALID_ARG);
        EXPECT(hmm_workspace_bytes(10, 0, 1, &s, &v), HMM_ERR_INVALID_ARG);
        EXPECT(hmm_workspace_bytes(10, 4, 0, &s, &v), HMM_ERR_INVALID_ARG);
        EXPECT(hmm_workspace_bytes(10, 129, 1, &s, &v), HMM_ERR_UNSUPPORTED);
    }
    for (int c = -1; c < 7; ++c)
        if (hmm_status_string(c) == NULL) { printf("no status string for %d\n", c); ++failures; }

    /* argument errors: reported before anything is launched */
    EXPECT(hmm_smooth(NULL, fake, fake, 8, 4, 1, 1, fake, NULL, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_smooth(fake, fake, fake, 8, 4, 1, 1, NULL, NULL, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_smooth(fake, fake, fake, 0, 4, 1, 1, fake, NULL, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_smooth(fake, fake, odd, 8, 4, 1, 1, fake, NULL, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_smooth(fake, fake, fake, 8, 1000, 1, 1, fake, NULL, fd, ws, big, NULL), HMM_ERR_UNSUPPORTED);
    EXPECT(hmm_smooth(fake, fake, fake, 8, 4, 1, 1, fake, NULL, fd, NULL, big, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_smooth(fake, fake, fake, 8, 4, 1, 1, fake, NULL, fd, ws, 16, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_smooth(fake, fake, fake, 1 << 20, 128, 1, 1, fake, NULL, fd, ws, big, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_smooth_static(NULL, fake, fake, 8, 4, 1, 1, fake, NULL, fd, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_smooth_static(fake, fake, fake, 1 << 20, 128, 1, 1, fake, NULL, fd, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_viterbi(fake, fake, fake, 8, 4, 1, 1, NULL, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_viterbi(fake, fake, fake, 8, 0, 1, 1, fi, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_viterbi(fake, fake, fake, 8, 4, -1, 1, fi, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_viterbi(fake, fake, fake, 8, 4, 1, 1, fi, fd, badws, big, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_max_product(fake, fake, fake, 8, 4, 1, 1, NULL, NULL, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_max_product(fake, fake, fake, 8, 1000, 1, 1, fake, NULL, fd, ws, big, NULL), HMM_ERR_UNSUPPORTED);
    EXPECT(hmm_max_product(fake, fake, fake, 8, 4, 1, 1, fake, NULL, fd, ws, 16, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_transition_counts(NULL, fake, fake, 8, 4, 1, 1, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_transition_counts(fake, fake, fake, 8, 200, 1, 1, fd, ws, big, NULL), HMM_ERR_UNSUPPORTED);
    EXPECT(hmm_transition_counts(fake, fake, fake, 8, 4, 1, 1, fd, ws, 8, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_block_element(NULL, fake, 8, 4, 1, 1, 0, fake, fd, ws, big, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_block_element(fake, fake, 8, 300, 1, 1, 0, fake, fd, ws, big, NULL), HMM_ERR_UNSUPPORTED);
    EXPECT(hmm_block_element(fake, fake, 8, 4, 1, 1, 0, fake, fd, ws, 8, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_block_carries(fake, fake, NULL, fd, 3, 4, 1, 1, 0, fake, fake, fd, NULL), HMM_ERR_INVALID_ARG);
    EXPECT(hmm_block_carries(fake, fake, fake, fd, 3, 129, 1, 1, 1, fake, fake, fd, NULL), HMM_ERR_UNSUPPORTED);
    EXPECT(hmm_workspace_init(NULL, big, NULL), HMM_ERR_WORKSPACE);
    EXPECT(hmm_workspace_init(badws, big, NULL), HMM_ERR_WORKSPACE);
    {
        int32_t state = 0;
        EXPECT(hmm_workspace_status(NULL, NULL, &state), HMM_ERR_INVALID_ARG);
        EXPECT(hmm_workspace_status(ws, NULL, NULL), HMM_ERR_INVALID_ARG);
    }
    printf("boundary sanitizer driver: %s\n", failures ? "FAILED" : "ok");
    return failures ? 1 : 0;
}
