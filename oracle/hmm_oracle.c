/*
 * CPU oracle for HMM smoothing and Viterbi decoding -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, sequential, single-threaded fp64 implementations of the two classical
 * recursions that the paper's parallel-scan method is algebraically equivalent to
 * (Sec. VI states the parallel and sequential methods are algebraically
 * equivalent; Theorems 1-2 and Propositions 2-3 identify the scan results with
 * the forward/backward potentials).  Nothing here is shared with the GPU library:
 * no headers, no helpers, no tables.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it.
 *
 * Inputs are the same float32 arrays the GPU path consumes, widened to double.
 *   prior[D]         p(x_1)
 *   A[D][D]          A[i][j] = p(x_k = j | x_{k-1} = i)
 *   ll[T][D]         ll[t][j] = log p(y_{t+1} | x_{t+1} = j)   (t is 0-based)
 * Potentials (Sec. II): psi_1(x_1) = p(y_1|x_1) p(x_1),
 *                       psi_k(x_{k-1}, x_k) = p(y_k|x_k) p(x_k|x_{k-1}).
 *
 * Pins (see tests/test_oracle_*.py): brute-force enumeration of all D^T sequences
 * (the definitions of the marginals, of Z and of the MAP sequence in Sec. II and
 * Sec. IV-A), closed forms (identical transition rows, identity transitions,
 * constant evidence), D = 1, T = 1, and invariants.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

/*
 * Forward-backward recursion of Algorithm 1 with the marginal of the equation
 * p(x_k) = psi^f_{1,k}(x_k) psi^b_{k,T}(x_k) / Z_k (Sec. III-A).
 *
 * The paper's recursion is stated on raw potentials, which underflow for long
 * sequences; the only change made here is the classical per-step rescaling:
 * the forward vector is divided by its sum (making it the filtering
 * distribution p(x_k | y_{1:k})) and the removed factors are accumulated in the
 * log domain, so that log Z = log p(y_{1:T}) is their total; the backward
 * vector is divided by its largest entry (its scale cancels in Z_k).
 *
 * marginals[T][D], filtered[T][D] (may be NULL), *loglik.  Returns 0, or 1 on
 * allocation failure / bad sizes.
 */
int hmm_oracle_smooth(const float *prior, const float *A, const float *ll,
                      long T, int D, double *marginals, double *filtered, double *loglik)
{
    if (T < 1 || D < 1) return 1;
    double *f = (double *)malloc(sizeof(double) * (size_t)T * D);   /* scaled psi^f_{1,k} */
    double *b = (double *)malloc(sizeof(double) * D);               /* scaled psi^b_{k,T} */
    double *bn = (double *)malloc(sizeof(double) * D);
    double *g = (double *)malloc(sizeof(double) * D);
    if (!f || !b || !bn || !g) { free(f); free(b); free(bn); free(g); return 1; }

    double L = 0.0;
    /* forward pass: psi^f_{1,1} = psi_1; psi^f_{1,k}(x_k) = sum_{x_{k-1}} psi^f_{1,k-1} psi_k */
    for (long k = 0; k < T; ++k) {
        const float *llk = ll + (size_t)k * D;
        double m = -INFINITY;
        for (int j = 0; j < D; ++j) if ((double)llk[j] > m) m = (double)llk[j];
        double c = 0.0;
        for (int j = 0; j < D; ++j) {
            double pred;
            if (k == 0) {
                pred = (double)prior[j];
            } else {
                const double *fp = f + (size_t)(k - 1) * D;
                pred = 0.0;
                for (int i = 0; i < D; ++i) pred += fp[i] * (double)A[(size_t)i * D + j];
            }
            g[j] = pred * exp((double)llk[j] - m);
            c += g[j];
        }
        for (int j = 0; j < D; ++j) f[(size_t)k * D + j] = g[j] / c;
        L += m + log(c);
    }
    *loglik = L;
    if (filtered) memcpy(filtered, f, sizeof(double) * (size_t)T * D);

    /* backward pass: psi^b_{T,T} = 1; psi^b_{k,T}(x_k) = sum_{x_{k+1}} psi_{k+1}(x_k,x_{k+1}) psi^b_{k+1,T} */
    for (int j = 0; j < D; ++j) b[j] = 1.0;
    for (long k = T - 1; k >= 0; --k) {
        /* marginal at step k from f_k and b_k */
        double z = 0.0;
        for (int j = 0; j < D; ++j) z += f[(size_t)k * D + j] * b[j];
        for (int j = 0; j < D; ++j) marginals[(size_t)k * D + j] = f[(size_t)k * D + j] * b[j] / z;
        if (k == 0) break;
        const float *llk = ll + (size_t)k * D;
        double m = -INFINITY;
        for (int j = 0; j < D; ++j) if ((double)llk[j] > m) m = (double)llk[j];
        for (int j = 0; j < D; ++j) g[j] = exp((double)llk[j] - m) * b[j];
        double hm = 0.0;
        for (int i = 0; i < D; ++i) {
            double h = 0.0;
            for (int j = 0; j < D; ++j) h += (double)A[(size_t)i * D + j] * g[j];
            bn[i] = h;
            if (h > hm) hm = h;
        }
        for (int i = 0; i < D; ++i) b[i] = bn[i] / hm;
    }
    free(f); free(b); free(bn); free(g);
    return 0;
}

static double log_or_neginf(double p) { return p > 0.0 ? log(p) : -INFINITY; }

/*
 * Classical Viterbi recursion of Algorithm 4, carried out on logarithms of the
 * potentials (a monotone transform, so every max and argmax is unchanged):
 *   V_1(x_1) = log psi_1(x_1)
 *   V_k(x_k) = max_{x_{k-1}} [log psi_k(x_{k-1},x_k) + V_{k-1}(x_{k-1})],  u_{k-1}(x_k) = argmax
 *   x*_T = argmax V_T,  x*_{k-1} = u_{k-1}(x*_k).
 * Ties (which the paper excludes by assuming a unique MAP sequence) are resolved
 * towards the lowest state index.  *logprob = V_T(x*_T) = log p(y_{1:T}, x*_{1:T})
 * (Corollary 1: the first component of a~_{0:T+1}).
 */
int hmm_oracle_viterbi(const float *prior, const float *A, const float *ll,
                       long T, int D, int *path, double *logprob)
{
    if (T < 1 || D < 1) return 1;
    unsigned char *u8 = NULL; int *u32 = NULL;
    size_t nu = (size_t)(T > 1 ? T - 1 : 1) * D;
    if (D <= 256) u8 = (unsigned char *)malloc(nu); else u32 = (int *)malloc(sizeof(int) * nu);
    double *V = (double *)malloc(sizeof(double) * D);
    double *Vn = (double *)malloc(sizeof(double) * D);
    double *logA = (double *)malloc(sizeof(double) * (size_t)D * D);
    if ((!u8 && !u32) || !V || !Vn || !logA) { free(u8); free(u32); free(V); free(Vn); free(logA); return 1; }
    for (size_t e = 0; e < (size_t)D * D; ++e) logA[e] = log_or_neginf((double)A[e]);
    for (int j = 0; j < D; ++j) V[j] = log_or_neginf((double)prior[j]) + (double)ll[j];
    for (long k = 1; k < T; ++k) {
        const float *llk = ll + (size_t)k * D;
        for (int j = 0; j < D; ++j) {
            double best = -INFINITY; int arg = 0;
            for (int i = 0; i < D; ++i) {
                double v = V[i] + logA[(size_t)i * D + j];
                if (v > best) { best = v; arg = i; }
            }
            Vn[j] = best + (double)llk[j];
            if (u8) u8[(size_t)(k - 1) * D + j] = (unsigned char)arg; else u32[(size_t)(k - 1) * D + j] = arg;
        }
        double *t = V; V = Vn; Vn = t;
    }
    double best = -INFINITY; int arg = 0;
    for (int j = 0; j < D; ++j) if (V[j] > best) { best = V[j]; arg = j; }
    *logprob = best;
    path[T - 1] = arg;
    for (long k = T - 1; k >= 1; --k) {
        arg = u8 ? (int)u8[(size_t)(k - 1) * D + arg] : u32[(size_t)(k - 1) * D + arg];
        path[k - 1] = arg;
    }
    free(u8); free(u32); free(V); free(Vn); free(logA);
    return 0;
}

/*
 * log of the joint of Sec. II evaluated on a given state sequence:
 * log psi_1(x_1) + sum_{k>=2} log psi_k(x_{k-1}, x_k).  Used to adjudicate
 * decodings that differ from the oracle's only at numerical near-ties.
 */
double hmm_oracle_score(const float *prior, const float *A, const float *ll,
                        long T, int D, const int *path)
{
    double s = log_or_neginf((double)prior[path[0]]) + (double)ll[path[0]];
    for (long k = 1; k < T; ++k) {
        s += log_or_neginf((double)A[(size_t)path[k - 1] * D + path[k]]) + (double)ll[(size_t)k * D + path[k]];
    }
    return s;
}

/*
 * Max-product forward/backward recursions (the lemma of Sec. IV-C) on logarithms
 * of the potentials, and the per-step maximiser of Theorem 4:
 *   f_1(x_1) = log psi_1(x_1),  f_k(x_k) = max_{x_{k-1}} [log psi_k(x_{k-1},x_k) + f_{k-1}(x_{k-1})]
 *   b_T(x_T) = 0,               b_k(x_k) = max_{x_{k+1}} [log psi_{k+1}(x_k,x_{k+1}) + b_{k+1}(x_{k+1})]
 *   x*_k = argmax_{x_k} [f_k(x_k) + b_k(x_k)]        (lowest index on ties)
 * f_k + b_k is the logarithm of the max-marginal p*(x_k) of Sec. II (the largest
 * joint weight over all sequences that pass through x_k at step k).  It is
 * returned relative to its own maximum over x_k, which is the same for every k
 * and equals *logprob = log of the largest joint weight:
 *   maxmarg[k][j] = f_k(j) + b_k(j) - logprob   (<= 0, and 0 at x*_k).
 * Returns 0, or 1 on allocation failure / bad sizes.
 */
int hmm_oracle_max_product(const float *prior, const float *A, const float *ll,
                           long T, int D, double *maxmarg, int *path, double *logprob)
{
    if (T < 1 || D < 1) return 1;
    double *f = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *b = (double *)malloc(sizeof(double) * D);
    double *bn = (double *)malloc(sizeof(double) * D);
    double *logA = (double *)malloc(sizeof(double) * (size_t)D * D);
    if (!f || !b || !bn || !logA) { free(f); free(b); free(bn); free(logA); return 1; }
    for (size_t e = 0; e < (size_t)D * D; ++e) logA[e] = log_or_neginf((double)A[e]);
    for (int j = 0; j < D; ++j) f[j] = log_or_neginf((double)prior[j]) + (double)ll[j];
    for (long k = 1; k < T; ++k) {
        const double *fp = f + (size_t)(k - 1) * D;
        double *fk = f + (size_t)k * D;
        for (int j = 0; j < D; ++j) {
            double best = -INFINITY;
            for (int i = 0; i < D; ++i) {
                double v = fp[i] + logA[(size_t)i * D + j];
                if (v > best) best = v;
            }
            fk[j] = best + (double)ll[(size_t)k * D + j];
        }
    }
    double top = -INFINITY;
    for (int j = 0; j < D; ++j) if (f[(size_t)(T - 1) * D + j] > top) top = f[(size_t)(T - 1) * D + j];
    *logprob = top;
    for (int j = 0; j < D; ++j) b[j] = 0.0;
    for (long k = T - 1; k >= 0; --k) {
        const double *fk = f + (size_t)k * D;
        double best = -INFINITY; int arg = 0;
        for (int j = 0; j < D; ++j) {
            double v = fk[j] + b[j];
            if (v > best) { best = v; arg = j; }
        }
        path[k] = arg;
        for (int j = 0; j < D; ++j) maxmarg[(size_t)k * D + j] = fk[j] + b[j] - top;
        if (k > 0) {
            for (int i = 0; i < D; ++i) {
                double m = -INFINITY;
                for (int j = 0; j < D; ++j) {
                    double v = logA[(size_t)i * D + j] + (double)ll[(size_t)k * D + j] + b[j];
                    if (v > m) m = v;
                }
                bn[i] = m;
            }
            double *t = b; b = bn; bn = t;
        }
    }
    free(f); free(b); free(bn); free(logA);
    return 0;
}

/*
 * Expected transition counts of the Baum-Welch expectation step (Sec. V-C names the
 * forward-backward recursion as its core): the pairwise posterior of the chain of Sec. II,
 *   p(x_{k-1}, x_k | y_{1:T}) = psi^f_{1,k-1}(x_{k-1}) psi_k(x_{k-1}, x_k) psi^b_{k,T}(x_k) / Z,
 * summed over k = 2..T:  counts[i][j] = sum_k p(x_{k-1} = i, x_k = j | y_{1:T}).
 * Same scaled forward and backward vectors as in hmm_oracle_smooth; each step's table is
 * normalised by its own total (every scale factor cancels).  counts[D][D]; returns 0 or 1.
 */
int hmm_oracle_transition_counts(const float *prior, const float *A, const float *ll,
                                 long T, int D, double *counts)
{
    if (T < 1 || D < 1) return 1;
    double *f = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *b = (double *)malloc(sizeof(double) * D);
    double *bn = (double *)malloc(sizeof(double) * D);
    double *g = (double *)malloc(sizeof(double) * D);
    double *xi = (double *)malloc(sizeof(double) * (size_t)D * D);
    if (!f || !b || !bn || !g || !xi) { free(f); free(b); free(bn); free(g); free(xi); return 1; }
    for (size_t e = 0; e < (size_t)D * D; ++e) counts[e] = 0.0;
    for (long k = 0; k < T; ++k) {
        const float *llk = ll + (size_t)k * D;
        double m = -INFINITY;
        for (int j = 0; j < D; ++j) if ((double)llk[j] > m) m = (double)llk[j];
        double c = 0.0;
        for (int j = 0; j < D; ++j) {
            double pred = 0.0;
            if (k == 0) pred = (double)prior[j];
            else for (int i = 0; i < D; ++i) pred += f[(size_t)(k - 1) * D + i] * (double)A[(size_t)i * D + j];
            g[j] = pred * exp((double)llk[j] - m);
            c += g[j];
        }
        for (int j = 0; j < D; ++j) f[(size_t)k * D + j] = g[j] / c;
    }
    for (int j = 0; j < D; ++j) b[j] = 1.0;
    for (long k = T - 1; k >= 1; --k) {
        const float *llk = ll + (size_t)k * D;
        double m = -INFINITY;
        for (int j = 0; j < D; ++j) if ((double)llk[j] > m) m = (double)llk[j];
        for (int j = 0; j < D; ++j) g[j] = exp((double)llk[j] - m) * b[j];     /* e_k(x_k) psi^b_{k,T}(x_k) */
        double tot = 0.0;
        for (int i = 0; i < D; ++i)
            for (int j = 0; j < D; ++j) {
                double v = f[(size_t)(k - 1) * D + i] * (double)A[(size_t)i * D + j] * g[j];
                xi[(size_t)i * D + j] = v;
                tot += v;
            }
        for (size_t e = 0; e < (size_t)D * D; ++e) counts[e] += xi[e] / tot;
        double hm = 0.0;
        for (int i = 0; i < D; ++i) {
            double h = 0.0;
            for (int j = 0; j < D; ++j) h += (double)A[(size_t)i * D + j] * g[j];
            bn[i] = h;
            if (h > hm) hm = h;
        }
        for (int i = 0; i < D; ++i) b[i] = bn[i] / hm;
    }
    free(f); free(b); free(bn); free(g); free(xi);
    return 0;
}

/*
 * Block-wise element (Sec. V-B: a block of consecutive observations and states taken as ONE element
 * of the scan).  For a block with log-likelihood rows ll[0..T-1] its element is, by Definition 3
 * (sum-product) or Definition 5 (max-product) applied to the block's own per-step elements,
 *   W(i, j) = sum / max over x_2..x_{T-1} of  e_1(i) prod_{k=2..T} A(x_{k-1}, x_k) e_k(x_k),
 *   x_1 = i, x_T = j, e_k(x) = exp(ll[k-1][x]),
 * the joint weight of the block's observations and its last state given its first state (T = 1:
 * diag(e_1)).  There is no transition into the block's first step: two adjacent blocks combine as
 * W_a (x) A (x) W_b.  Written out as the plain left-to-right product, rescaled every step:
 *   sum-product:  element = W / max W,      *log_scale = log max W   (element 0, -inf if W = 0)
 *   max-product:  element = log W - max,    *log_scale = max log W
 * element[D][D]; returns 0, or 1 on allocation failure / bad sizes.
 */
int hmm_oracle_block_element(const float *A, const float *ll, long T, int D, int max_product,
                             double *element, double *log_scale)
{
    if (T < 1 || D < 1) return 1;
    const size_t n = (size_t)D * D;
    double *X = (double *)malloc(sizeof(double) * n);
    double *Y = (double *)malloc(sizeof(double) * n);
    double *M = (double *)malloc(sizeof(double) * n);
    if (!X || !Y || !M) { free(X); free(Y); free(M); return 1; }
    double ls = 0.0;
    if (max_product) {
        for (size_t e = 0; e < n; ++e) M[e] = log_or_neginf((double)A[e]);
        for (int i = 0; i < D; ++i)
            for (int j = 0; j < D; ++j) X[(size_t)i * D + j] = (i == j) ? (double)ll[j] : -INFINITY;
    } else {
        for (size_t e = 0; e < n; ++e) M[e] = (double)A[e];
        for (int i = 0; i < D; ++i)
            for (int j = 0; j < D; ++j) X[(size_t)i * D + j] = (i == j) ? exp((double)ll[j]) : 0.0;
    }
    for (long k = 0; k < T; ++k) {
        if (k > 0) {
            const float *llk = ll + (size_t)k * D;
            for (int i = 0; i < D; ++i)
                for (int j = 0; j < D; ++j) {
                    double acc = max_product ? -INFINITY : 0.0;
                    for (int h = 0; h < D; ++h) {
                        if (max_product) {
                            double v = X[(size_t)i * D + h] + M[(size_t)h * D + j];
                            if (v > acc) acc = v;
                        } else {
                            acc += X[(size_t)i * D + h] * M[(size_t)h * D + j];
                        }
                    }
                    Y[(size_t)i * D + j] = max_product ? acc + (double)llk[j] : acc * exp((double)llk[j]);
                }
            double *t = X; X = Y; Y = t;
        }
        double m = max_product ? -INFINITY : 0.0;
        for (size_t e = 0; e < n; ++e) if (X[e] > m) m = X[e];
        if (max_product) {
            if (m > -INFINITY) { for (size_t e = 0; e < n; ++e) X[e] -= m; ls += m; }
            else ls = -INFINITY;
        } else {
            if (m > 0.0) { for (size_t e = 0; e < n; ++e) X[e] /= m; ls += log(m); }
            else ls = -INFINITY;
        }
    }
    for (size_t e = 0; e < n; ++e) element[e] = X[e];
    *log_scale = ls;
    free(X); free(Y); free(M);
    return 0;
}

/*
 * Carries between the blocks of one sequence from the blocks' elements (Sec. V-B; Theorems 1-2 and
 * the lemma of Sec. IV-C at block granularity).  elements[S][D][D] and log_scales[S] are as
 * returned by hmm_oracle_block_element (given here as float / double, the arrays the GPU path
 * consumes).  With p_0 = prior, for s = 0..S-1:
 *     c_s = p_s (x) W_s      forward potential at the last step of block s, scaled to sum to one
 *                            (sum-product: the filtering distribution) or to maximum zero (max-product)
 *     p_{s+1} = c_s (x) A    its prediction for the first step of block s+1
 * and with r_{S-1} = 1 (the neutral backward potential at the sequence's end), for s = S-1..1:
 *     u_s = W_s (x) r_s      backward potential at the first step of block s INCLUDING that step's
 *                            emission factor, scaled to maximum one (zero on logarithms)
 *     r_{s-1} = A (x) u_s    backward potential at the last step of block s-1.
 * carry_rows[s] = log c_{s-1} for s >= 1 (row 0: log of the prior scaled to maximum one);
 * lookahead_rows[s] = log u_{s+1} for s <= S-2 (row S-1: zeros).  These are the rows that, put
 * in front of / behind block s's own log-likelihood rows as one more pseudo-observation each,
 * make a stand-alone recursion over [carry; block; lookahead] reproduce the whole sequence's
 * results on the block's steps (with a uniform prior of ones for s >= 1, the true prior for s = 0).
 * *total = log Z (sum-product) or the log of the largest joint weight (max-product).
 */
int hmm_oracle_block_carries(const float *prior, const float *A, const float *elements,
                             const double *log_scales, int S, int D, int max_product,
                             double *carry_rows, double *lookahead_rows, double *total)
{
    if (S < 1 || D < 1) return 1;
    double *p = (double *)malloc(sizeof(double) * D);
    double *c = (double *)malloc(sizeof(double) * D);
    if (!p || !c) { free(p); free(c); return 1; }
    double tot = 0.0, pm = 0.0;
    for (int j = 0; j < D; ++j) if ((double)prior[j] > pm) pm = (double)prior[j];
    for (int j = 0; j < D; ++j) {
        p[j] = max_product ? log_or_neginf((double)prior[j]) : (double)prior[j];
        carry_rows[j] = log_or_neginf((double)prior[j] / pm);
    }
    for (int s = 0; s < S; ++s) {
        const float *W = elements + (size_t)s * D * D;
        double nrm = max_product ? -INFINITY : 0.0;
        for (int j = 0; j < D; ++j) {
            double acc = max_product ? -INFINITY : 0.0;
            for (int i = 0; i < D; ++i) {
                if (max_product) { double v = p[i] + (double)W[(size_t)i * D + j]; if (v > acc) acc = v; }
                else acc += p[i] * (double)W[(size_t)i * D + j];
            }
            c[j] = acc;
            if (max_product) { if (acc > nrm) nrm = acc; } else nrm += acc;
        }
        tot += (max_product ? nrm : log(nrm)) + log_scales[s];
        for (int j = 0; j < D; ++j) c[j] = max_product ? c[j] - nrm : c[j] / nrm;
        if (s + 1 < S)
            for (int j = 0; j < D; ++j) carry_rows[(size_t)(s + 1) * D + j] = max_product ? c[j] : log_or_neginf(c[j]);
        for (int j = 0; j < D; ++j) {
            double acc = max_product ? -INFINITY : 0.0;
            for (int i = 0; i < D; ++i) {
                if (max_product) { double v = c[i] + log_or_neginf((double)A[(size_t)i * D + j]); if (v > acc) acc = v; }
                else acc += c[i] * (double)A[(size_t)i * D + j];
            }
            p[j] = acc;
        }
    }
    *total = tot;
    /* backward: p holds r_s, c holds u_s */
    for (int i = 0; i < D; ++i) { p[i] = max_product ? 0.0 : 1.0; lookahead_rows[(size_t)(S - 1) * D + i] = 0.0; }
    for (int s = S - 1; s >= 1; --s) {
        const float *W = elements + (size_t)s * D * D;
        double m = max_product ? -INFINITY : 0.0;
        for (int i = 0; i < D; ++i) {
            double acc = max_product ? -INFINITY : 0.0;
            for (int j = 0; j < D; ++j) {
                if (max_product) { double v = (double)W[(size_t)i * D + j] + p[j]; if (v > acc) acc = v; }
                else acc += (double)W[(size_t)i * D + j] * p[j];
            }
            c[i] = acc;
            if (acc > m) m = acc;
        }
        for (int i = 0; i < D; ++i) {
            c[i] = max_product ? c[i] - m : c[i] / m;
            lookahead_rows[(size_t)(s - 1) * D + i] = max_product ? c[i] : log_or_neginf(c[i]);
        }
        for (int i = 0; i < D; ++i) {
            double acc = max_product ? -INFINITY : 0.0;
            for (int j = 0; j < D; ++j) {
                if (max_product) { double v = log_or_neginf((double)A[(size_t)i * D + j]) + c[j]; if (v > acc) acc = v; }
                else acc += (double)A[(size_t)i * D + j] * c[j];
            }
            p[i] = acc;
        }
    }
    free(p); free(c);
    return 0;
}
