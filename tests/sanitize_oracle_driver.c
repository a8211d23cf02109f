/* Host-only sanitizer driver for the C oracle: calls every entry point on small seeded inputs that cover
 * the edge sizes (T = 1, D = 1, zero transitions, -inf log-likelihoods) so that AddressSanitizer and
 * UndefinedBehaviorSanitizer see every loop bound and every allocation.  Built and run by
 * tests/test_oracle_sanitizers.py; exit status 0 means every call returned without a report. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int hmm_oracle_smooth(const float *, const float *, const float *, long, int, double *, double *, double *);
int hmm_oracle_viterbi(const float *, const float *, const float *, long, int, int *, double *);
double hmm_oracle_score(const float *, const float *, const float *, long, int, const int *);
int hmm_oracle_max_product(const float *, const float *, const float *, long, int, double *, int *, double *);
int hmm_oracle_transition_counts(const float *, const float *, const float *, long, int, double *);
int hmm_oracle_block_element(const float *, const float *, long, int, int, double *, double *);
int hmm_oracle_block_carries(const float *, const float *, const float *, const double *, int, int, int, double *,
                             double *, double *);

static unsigned long long state = 0x9e3779b97f4a7c15ull;
static double uniform(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0;
}

static int run_case(long T, int D, double zero_frac, double neginf_frac)
{
    const size_t dd = (size_t)D * D, td = (size_t)T * D;
    float *prior = malloc(sizeof(float) * D), *A = malloc(sizeof(float) * dd), *ll = malloc(sizeof(float) * td);
    double *marg = malloc(sizeof(double) * td), *filt = malloc(sizeof(double) * td), *mm = malloc(sizeof(double) * td);
    double *counts = malloc(sizeof(double) * dd), *elem = malloc(sizeof(double) * dd);
    int *path = malloc(sizeof(int) * T), *path2 = malloc(sizeof(int) * T);
    if (!prior || !A || !ll || !marg || !filt || !mm || !counts || !elem || !path || !path2) return 2;
    double s = 0.0;
    for (int i = 0; i < D; ++i) { prior[i] = (float)(uniform() + 1e-3); s += prior[i]; }
    for (int i = 0; i < D; ++i) prior[i] = (float)(prior[i] / s);
    for (int i = 0; i < D; ++i) {
        s = 0.0;
        for (int j = 0; j < D; ++j) {
            double a = (uniform() < zero_frac && j != i) ? 0.0 : uniform() + 1e-3;
            A[(size_t)i * D + j] = (float)a; s += a;
        }
        for (int j = 0; j < D; ++j) A[(size_t)i * D + j] = (float)(A[(size_t)i * D + j] / s);
    }
    for (size_t e = 0; e < td; ++e) ll[e] = (uniform() < neginf_frac) ? -INFINITY : (float)(-8.0 * uniform());
    double L = 0.0, lp = 0.0, lp2 = 0.0, ls = 0.0;
    int rc = 0;
    rc |= hmm_oracle_smooth(prior, A, ll, T, D, marg, filt, &L);
    rc |= hmm_oracle_smooth(prior, A, ll, T, D, marg, NULL, &L);
    rc |= hmm_oracle_viterbi(prior, A, ll, T, D, path, &lp);
    (void)hmm_oracle_score(prior, A, ll, T, D, path);
    rc |= hmm_oracle_max_product(prior, A, ll, T, D, mm, path2, &lp2);
    rc |= hmm_oracle_transition_counts(prior, A, ll, T, D, counts);
    rc |= hmm_oracle_block_element(A, ll, T, D, 0, elem, &ls);
    rc |= hmm_oracle_block_element(A, ll, T, D, 1, elem, &ls);
    /* blocks: split the sequence into S pieces, elements of each, then the carries */
    int S = T >= 3 ? 3 : 1;
    float *els = malloc(sizeof(float) * dd * S);
    double *lsc = malloc(sizeof(double) * S), *cr = malloc(sizeof(double) * (size_t)S * D), *lr = malloc(sizeof(double) * (size_t)S * D);
    if (!els || !lsc || !cr || !lr) return 2;
    for (int mp = 0; mp < 2; ++mp) {
        for (int b = 0; b < S; ++b) {
            long t0 = T * b / S, t1 = T * (b + 1) / S;
            rc |= hmm_oracle_block_element(A, ll + (size_t)t0 * D, t1 - t0, D, mp, elem, &lsc[b]);
            for (size_t e = 0; e < dd; ++e) els[(size_t)b * dd + e] = (float)elem[e];
        }
        double tot = 0.0;
        rc |= hmm_oracle_block_carries(prior, A, els, lsc, S, D, mp, cr, lr, &tot);
    }
    /* bad sizes are refused, not executed */
    if (hmm_oracle_smooth(prior, A, ll, 0, D, marg, filt, &L) != 1) rc |= 4;
    if (hmm_oracle_viterbi(prior, A, ll, T, 0, path, &lp) != 1) rc |= 4;
    free(prior); free(A); free(ll); free(marg); free(filt); free(mm); free(counts); free(elem); free(path); free(path2);
    free(els); free(lsc); free(cr); free(lr);
    return rc;
}

int main(void)
{
    static const long Ts[] = {1, 2, 3, 17, 257};
    static const int Ds[] = {1, 2, 3, 4, 7, 16, 33};
    int bad = 0;
    for (unsigned a = 0; a < sizeof Ts / sizeof *Ts; ++a)
        for (unsigned b = 0; b < sizeof Ds / sizeof *Ds; ++b) {
            bad |= run_case(Ts[a], Ds[b], 0.0, 0.0);
            bad |= run_case(Ts[a], Ds[b], 0.4, 0.2);   /* sparse transitions and impossible observations */
        }
    printf("oracle sanitizer driver: %s\n", bad ? "FAILED" : "ok");
    return bad ? 1 : 0;
}
