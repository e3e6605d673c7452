/*
 * fp64 streaming oracle for RACE Attention, plain C.  TEST INFRASTRUCTURE ONLY.
 *
 * The same mathematics as oracle/race_oracle.py (which holds the explicit N x N
 * definition), written as the linear-time algorithms of the paper so that it can be
 * run, and timed, at sequence lengths where the quadratic form cannot:
 *   - non-causal forward : Algorithm 1, steps 4, 5, 7, 8
 *   - causal forward     : Algorithm 2, one left-to-right scan per table, each table
 *                          with its own cumulative bucket arrays (update, then read)
 *   - backward           : the paper prints none; two scans per table, derived from
 *                          Algorithms 1/2 (prefix statistics for the query side, suffix
 *                          statistics of the read-out cotangents for the key/value side)
 * It shares no code with the HIP library and is never linked into it.  The tests pin it
 * to the N x N definition and to finite differences through race_oracle.py.
 *
 * Layout: Q, K, V, O, dO, dQ, dK, dV are (B, H, N, d) row-major doubles, den is (B, H, N),
 * W is (H, L*P, d): row l*P+t of head h is hyperplane t of table l.  Corner r has
 * v_{r,t} = +1 iff bit t of r is set.  Parallelism: OpenMP over (batch*head, table);
 * per-table partial results are summed over tables in table order afterwards, so the
 * result does not depend on the number of threads.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* phi[r] = softmax_r(beta * tanh(W x) . v_r), and u[t] = tanh(<w_t, x>)  (Algorithm 1, step 4) */
static void soft_hash(const double *x, const double *Wl, int d, int P, double beta,
                      double *u, double *phi)
{
    const int R = 1 << P;
    for (int t = 0; t < P; ++t) {
        double z = 0.0;
        for (int c = 0; c < d; ++c) z += Wl[(size_t)t * d + c] * x[c];
        u[t] = tanh(z);
    }
    double mx = -INFINITY;
    for (int r = 0; r < R; ++r) {
        double s = 0.0;
        for (int t = 0; t < P; ++t) s += ((r >> t) & 1) ? u[t] : -u[t];
        phi[r] = beta * s;
        if (phi[r] > mx) mx = phi[r];
    }
    double sum = 0.0;
    for (int r = 0; r < R; ++r) { phi[r] = exp(phi[r] - mx); sum += phi[r]; }
    for (int r = 0; r < R; ++r) phi[r] /= sum;
}

/* cotangent of phi -> cotangent of x, added into dx: softmax, corner logits, tanh, W.
 * The corner logits are beta * (u . v_r): the cotangent of beta, sum_r ds_r (u . v_r), is added to *dbeta. */
static void soft_hash_vjp(const double *Wl, int d, int P, double beta, const double *u,
                          const double *phi, const double *dphi, double *dx, double *dbeta)
{
    const int R = 1 << P;
    double mean = 0.0;
    for (int r = 0; r < R; ++r) mean += phi[r] * dphi[r];
    for (int t = 0; t < P; ++t) {
        double du = 0.0;
        for (int r = 0; r < R; ++r) {
            double ds = phi[r] * (dphi[r] - mean);
            du += ((r >> t) & 1) ? ds : -ds;
        }
        *dbeta += du * u[t];
        double dz = beta * du * (1.0 - u[t] * u[t]);
        for (int c = 0; c < d; ++c) dx[c] += dz * Wl[(size_t)t * d + c];
    }
}

int race_oracle_threads(void) { return oracle_threads(); }

/* Forward.  Returns 0 on success, 1 on allocation failure, 2 on a bad argument.
 * state: NULL, or (B*H, L, R, d+1) doubles, per bucket row the d value sums then the mass (Algorithm 2's
 * cumulative arrays): the scan starts from it and leaves the arrays after the last token there, so that a long
 * sequence can be run slice by slice in bounded memory (causal only: Algorithm 1's statistics are over all N).
 * The additions are the same, in the same order, whether a sequence is run whole or in slices. */
int race_oracle_forward_carry(int B, int H, long N, int d, int L, int P, double beta, int causal,
                              const double *Q, const double *K, const double *V, const double *W,
                              double *state, double *O, double *den)
{
    if (state && !causal) return 2;
    const int R = 1 << P;
    const int BH = B * H;
    int group = (oracle_threads() + L - 1) / L;       /* heads processed together */
    if (group < 1) group = 1;
    if (group > BH) group = BH;
    const size_t per_tab = (size_t)N * (d + 1);
    double *part = (double *)malloc(sizeof(double) * per_tab * (size_t)L * group);
    if (!part) return 1;
    int fail = 0;

    for (int bh0 = 0; bh0 < BH; bh0 += group) {
        const int g = (bh0 + group <= BH) ? group : BH - bh0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int gi = 0; gi < g; ++gi) {
            for (int l = 0; l < L; ++l) {
                const int bh = bh0 + gi, h = bh % H;
                const double *q = Q + (size_t)bh * N * d, *k = K + (size_t)bh * N * d;
                const double *v = V + (size_t)bh * N * d;
                const double *Wl = W + ((size_t)h * L + l) * P * d;
                double *out = part + ((size_t)gi * L + l) * per_tab;   /* [N][d+1]: num | den */
                double *A = state ? state + ((size_t)bh * L + l) * R * (d + 1)
                                  : (double *)calloc((size_t)R * (d + 1), sizeof(double));
                double *phi = (double *)malloc(sizeof(double) * (R + P));
                if (!A || !phi) {
#pragma omp atomic write
                    fail = 1;
                    if (!state) free(A);
                    free(phi);
                    continue;
                }
                double *u = phi + R;
                if (!causal) {                      /* Algorithm 1, step 5: all-N statistics */
                    for (long j = 0; j < N; ++j) {
                        soft_hash(k + j * d, Wl, d, P, beta, u, phi);
                        for (int r = 0; r < R; ++r) {
                            double *row = A + (size_t)r * (d + 1);
                            for (int c = 0; c < d; ++c) row[c] += phi[r] * v[j * d + c];
                            row[d] += phi[r];
                        }
                    }
                }
                for (long t = 0; t < N; ++t) {
                    if (causal) {                   /* Algorithm 2: add key/value t first ... */
                        soft_hash(k + t * d, Wl, d, P, beta, u, phi);
                        for (int r = 0; r < R; ++r) {
                            double *row = A + (size_t)r * (d + 1);
                            for (int c = 0; c < d; ++c) row[c] += phi[r] * v[t * d + c];
                            row[d] += phi[r];
                        }
                    }
                    soft_hash(q + t * d, Wl, d, P, beta, u, phi);   /* ... then query t reads */
                    double *o = out + (size_t)t * (d + 1);
                    for (int c = 0; c <= d; ++c) o[c] = 0.0;
                    for (int r = 0; r < R; ++r) {
                        const double *row = A + (size_t)r * (d + 1);
                        for (int c = 0; c <= d; ++c) o[c] += phi[r] * row[c];
                    }
                }
                if (!state) free(A);
                free(phi);
            }
        }
        /* Num = (1/L) sum_l num_l, Den = (1/L) sum_l den_l, O = Num / Den */
#pragma omp parallel for collapse(2) schedule(static)
        for (int gi = 0; gi < g; ++gi) {
            for (long t = 0; t < N; ++t) {
                const int bh = bh0 + gi;
                double dn = 0.0;
                for (int l = 0; l < L; ++l)
                    dn += part[((size_t)gi * L + l) * per_tab + (size_t)t * (d + 1) + d];
                dn /= L;
                for (int c = 0; c < d; ++c) {
                    double nm = 0.0;
                    for (int l = 0; l < L; ++l)
                        nm += part[((size_t)gi * L + l) * per_tab + (size_t)t * (d + 1) + c];
                    O[((size_t)bh * N + t) * d + c] = (nm / L) / dn;
                }
                den[(size_t)bh * N + t] = dn;
            }
        }
    }
    free(part);
    return fail;
}

int race_oracle_forward(int B, int H, long N, int d, int L, int P, double beta, int causal,
                        const double *Q, const double *K, const double *V, const double *W,
                        double *O, double *den)
{
    return race_oracle_forward_carry(B, H, N, d, L, P, beta, causal, Q, K, V, W, NULL, O, den);
}

/* Backward of loss = sum(dO * O), given O and den of the forward pass on the same inputs.
 * dbeta: (B*H) cotangents of the temperature, one per (batch, head).
 * Slices of a long causal sequence: S_state / dS_state are NULL or (B*H, L, R, d+1) doubles, the prefix statistics
 * (B | A) before the slice's first token and the suffix statistics (dB | dA) of the read-out cotangents after its
 * last token; each pass starts from its array and leaves it advanced over the slice.  do_query runs pass 1 (dQ),
 * do_keyvalue pass 2 (dK, dV): a sliced run sweeps the slices left to right with do_query, then right to left with
 * do_keyvalue.  A pass that is not run leaves zeros in its outputs, and dbeta holds the share of the passes run. */
int race_oracle_backward_carry(int B, int H, long N, int d, int L, int P, double beta, int causal,
                               const double *Q, const double *K, const double *V, const double *W,
                               const double *O, const double *den, const double *dO,
                               double *S_state, double *dS_state, int do_query, int do_keyvalue,
                               double *dQ, double *dK, double *dV, double *dbeta)
{
    if ((S_state || dS_state || !do_query || !do_keyvalue) && !causal) return 2;
    const int R = 1 << P;
    const int BH = B * H;
    int group = (oracle_threads() + L - 1) / L;
    if (group < 1) group = 1;
    if (group > BH) group = BH;
    const size_t per_tab = (size_t)N * d;
    double *part = (double *)malloc(sizeof(double) * per_tab * 3 * (size_t)L * group);
    double *gn = (double *)malloc(sizeof(double) * (size_t)N * (d + 1) * group);
    double *pbeta = (double *)malloc(sizeof(double) * (size_t)L * group);      /* per (head of the group, table) */
    if (!part || !gn || !pbeta) { free(part); free(gn); free(pbeta); return 1; }
    int fail = 0;

    for (int bh0 = 0; bh0 < BH; bh0 += group) {
        const int g = (bh0 + group <= BH) ? group : BH - bh0;
        /* cotangents of the un-averaged numerator and normaliser: e_i = L * Den_i,
           gn_i = dO_i / e_i,  ge_i = -(dO_i . O_i) / e_i  (stored as column d) */
#pragma omp parallel for collapse(2) schedule(static)
        for (int gi = 0; gi < g; ++gi) {
            for (long t = 0; t < N; ++t) {
                const size_t row = ((size_t)(bh0 + gi) * N + t) * d;
                const double e = den[(size_t)(bh0 + gi) * N + t] * L;
                double dot = 0.0;
                double *o = gn + ((size_t)gi * N + t) * (d + 1);
                for (int c = 0; c < d; ++c) { o[c] = dO[row + c] / e; dot += dO[row + c] * O[row + c]; }
                o[d] = -dot / e;
            }
        }
        memset(part, 0, sizeof(double) * per_tab * 3 * (size_t)L * g);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int gi = 0; gi < g; ++gi) {
            for (int l = 0; l < L; ++l) {
                const int bh = bh0 + gi, h = bh % H;
                const double *q = Q + (size_t)bh * N * d, *k = K + (size_t)bh * N * d;
                const double *v = V + (size_t)bh * N * d;
                const double *gt = gn + (size_t)gi * N * (d + 1);
                const double *Wl = W + ((size_t)h * L + l) * P * d;
                double *pQ = part + (((size_t)gi * L + l) * 3 + 0) * per_tab;
                double *pK = part + (((size_t)gi * L + l) * 3 + 1) * per_tab;
                double *pV = part + (((size_t)gi * L + l) * 3 + 2) * per_tab;
                const size_t soff = ((size_t)bh * L + l) * R * (d + 1);
                double *S = S_state ? S_state + soff : (double *)calloc((size_t)R * (d + 1), sizeof(double));      /* B | A  */
                double *dS = dS_state ? dS_state + soff : (double *)calloc((size_t)R * (d + 1), sizeof(double));   /* dB | dA */
                double *phi = (double *)malloc(sizeof(double) * (2 * R + P));
                if (!S || !dS || !phi) {
#pragma omp atomic write
                    fail = 1;
                    if (!S_state) free(S);
                    if (!dS_state) free(dS);
                    free(phi);
                    continue;
                }
                double *dphi = phi + R, *u = phi + 2 * R;
                double db = 0.0;
                if (!causal) {
                    for (long j = 0; j < N; ++j) {
                        soft_hash(k + j * d, Wl, d, P, beta, u, phi);
                        for (int r = 0; r < R; ++r) {
                            double *row = S + (size_t)r * (d + 1);
                            for (int c = 0; c < d; ++c) row[c] += phi[r] * v[j * d + c];
                            row[d] += phi[r];
                        }
                        soft_hash(q + j * d, Wl, d, P, beta, u, phi);
                        for (int r = 0; r < R; ++r) {
                            double *row = dS + (size_t)r * (d + 1);
                            for (int c = 0; c <= d; ++c) row[c] += phi[r] * gt[j * (d + 1) + c];
                        }
                    }
                }
                /* pass 1, left to right: prefix statistics -> cotangent of phi_Q -> dQ */
                for (long i = 0; do_query && i < N; ++i) {
                    if (causal) {
                        soft_hash(k + i * d, Wl, d, P, beta, u, phi);
                        for (int r = 0; r < R; ++r) {
                            double *row = S + (size_t)r * (d + 1);
                            for (int c = 0; c < d; ++c) row[c] += phi[r] * v[i * d + c];
                            row[d] += phi[r];
                        }
                    }
                    soft_hash(q + i * d, Wl, d, P, beta, u, phi);
                    for (int r = 0; r < R; ++r) {
                        const double *row = S + (size_t)r * (d + 1);
                        double acc = 0.0;
                        for (int c = 0; c <= d; ++c) acc += row[c] * gt[i * (d + 1) + c];
                        dphi[r] = acc;
                    }
                    soft_hash_vjp(Wl, d, P, beta, u, phi, dphi, pQ + i * d, &db);
                }
                /* pass 2, right to left: suffix statistics of the read-out cotangents -> dV, dK */
                for (long j = N - 1; do_keyvalue && j >= 0; --j) {
                    if (causal) {
                        soft_hash(q + j * d, Wl, d, P, beta, u, phi);
                        for (int r = 0; r < R; ++r) {
                            double *row = dS + (size_t)r * (d + 1);
                            for (int c = 0; c <= d; ++c) row[c] += phi[r] * gt[j * (d + 1) + c];
                        }
                    }
                    soft_hash(k + j * d, Wl, d, P, beta, u, phi);
                    for (int r = 0; r < R; ++r) {
                        const double *row = dS + (size_t)r * (d + 1);
                        double acc = row[d];
                        for (int c = 0; c < d; ++c) {
                            pV[j * d + c] += phi[r] * row[c];
                            acc += row[c] * v[j * d + c];
                        }
                        dphi[r] = acc;
                    }
                    soft_hash_vjp(Wl, d, P, beta, u, phi, dphi, pK + j * d, &db);
                }
                pbeta[(size_t)gi * L + l] = db;
                if (!S_state) free(S);
                if (!dS_state) free(dS);
                free(phi);
            }
        }
#pragma omp parallel for collapse(2) schedule(static)
        for (int gi = 0; gi < g; ++gi) {
            for (long t = 0; t < N; ++t) {
                const size_t row = ((size_t)(bh0 + gi) * N + t) * d;
                for (int c = 0; c < d; ++c) {
                    double a = 0.0, b = 0.0, cc = 0.0;
                    for (int l = 0; l < L; ++l) {
                        const double *p = part + ((size_t)gi * L + l) * 3 * per_tab + (size_t)t * d + c;
                        a += p[0]; b += p[per_tab]; cc += p[2 * per_tab];
                    }
                    dQ[row + c] = a; dK[row + c] = b; dV[row + c] = cc;
                }
            }
        }
        if (dbeta) {                    /* tables added up in table order: independent of the thread count */
            for (int gi = 0; gi < g; ++gi) {
                double sb = 0.0;
                for (int l = 0; l < L; ++l) sb += pbeta[(size_t)gi * L + l];
                dbeta[bh0 + gi] = sb;
            }
        }
    }
    free(part); free(gn); free(pbeta);
    return fail;
}

int race_oracle_backward(int B, int H, long N, int d, int L, int P, double beta, int causal,
                         const double *Q, const double *K, const double *V, const double *W,
                         const double *O, const double *den, const double *dO,
                         double *dQ, double *dK, double *dV, double *dbeta)
{
    return race_oracle_backward_carry(B, H, N, d, L, P, beta, causal, Q, K, V, W, O, den, dO, NULL, NULL, 1, 1,
                                      dQ, dK, dV, dbeta);
}
