/*
 * Dictionary Annealing (DA) -- plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what
 * the GPU library computes.  It shares no code, header, table or helper with the HIP
 * path; only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Paper: "HCLAE: High Capacity Locally Aggregating Encodings for Approximate Nearest
 * Neighbor Search" (arXiv 1509.05194).  Passages followed:
 *   - Sec. 3.1 (Dictionary Annealing): heat  x' = e_x + c_m(i_m(x));  cool = refit C_m to
 *     {x'}; one dictionary per iteration, then re-encode to get the next residue; learning
 *     from scratch = DA on all-zero dictionaries (footnote: then x' equals the residue).
 *   - Sec. 3.2: the previously learned dictionary is the initial point of the k-means
 *     that cools (plain full-dimension Lloyd here; the PCA / dimension-adding variant is
 *     not part of this oracle).
 *   - Sec. 3.3, Eq. 1 first line: E = || x - sum_m c_m(i_m(x)) ||^2 ; Eq. 3 with L = 1 is
 *     greedy residual encoding; with L > 1 it is the multi-path (beam) encoding of
 *     da_beam_step / da_encode_beam.
 *   - Table 1 magnitudes fix E as the mean over vectors of the squared residual norm.
 *
 * Readings where the paper is silent: fixed number T of Lloyd iterations per cool-down;
 * argmin ties go to the lowest index (ascending k, strict <); an empty cluster keeps its
 * previous codeword; a stage re-encodes only its own code column; an all-zero dictionary
 * is seeded with K rows of x' picked by caller-supplied indices.
 *
 * Arithmetic: IEEE double everywhere, every sum in ascending index order, distances in
 * the direct form sum_d (x_d - c_d)^2.  Build WITHOUT fast-math and without FP contraction.
 * OpenMP is used only across vectors, where results do not depend on the thread count;
 * the centroid sums are accumulated serially in vector order.
 *
 * Layouts (row-major): r, xp: double[N][D]; C: double[M][K][D]; codes: uint8[N][M].
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int da_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void da_oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* Sec. 3.1, heat-up: x'_n = e_n + c_m(i_m(n)), in place over r. */
void da_heat(double *r, const uint8_t *codes, const double *C,
             int64_t N, int D, int M, int K, int m)
{
    const double *Cm = C + (size_t)m * K * D;
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const double *c = Cm + (size_t)codes[n * M + m] * D;
        double *rn = r + (size_t)n * D;
        for (int d = 0; d < D; ++d) rn[d] = rn[d] + c[d];
    }
}

/* Sec. 3.1, "obtain the new residue": e_n = x'_n - c_m(i_m(n)), in place over xp. */
void da_cool(double *xp, const uint8_t *codes, const double *C,
             int64_t N, int D, int M, int K, int m)
{
    const double *Cm = C + (size_t)m * K * D;
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const double *c = Cm + (size_t)codes[n * M + m] * D;
        double *xn = xp + (size_t)n * D;
        for (int d = 0; d < D; ++d) xn[d] = xn[d] - c[d];
    }
}

/*
 * Nearest codeword of dictionary m for every x'_n (the assignment half of the k-means
 * that cools, Sec. 3.1/3.2; also the L = 1 case of Eq. 3).
 * Writes codes[n][m].  Optional outputs (may be NULL):
 *   d1[n]  smallest squared distance, d2[n] second smallest (+inf when K == 1),
 *   i2[n]  index attaining d2 (-1 when K == 1).
 */
void da_assign(const double *xp, const double *C, int64_t N, int D, int M, int K, int m,
               uint8_t *codes, double *d1, double *d2, int32_t *i2)
{
    const double *Cm = C + (size_t)m * K * D;
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const double *x = xp + (size_t)n * D;
        double best = INFINITY, second = INFINITY;
        int ibest = 0, isecond = -1;
        for (int k = 0; k < K; ++k) {
            const double *c = Cm + (size_t)k * D;
            double s = 0.0;
            for (int d = 0; d < D; ++d) {
                double t = x[d] - c[d];
                s = s + t * t;
            }
            if (k == 0 || s < best) {
                if (k != 0) { second = best; isecond = ibest; }
                best = s; ibest = k;
            } else if (s < second) {
                second = s; isecond = k;
            }
        }
        codes[n * M + m] = (uint8_t)ibest;
        if (d1) d1[n] = best;
        if (d2) d2[n] = second;
        if (i2) i2[n] = isecond;
    }
}

/* Squared distance from x'_n to one given codeword k of dictionary m (test helper for
 * judging a code that differs from the oracle's own choice). */
double da_dist_to(const double *xp, const double *C, int64_t n, int D, int K, int m, int k)
{
    const double *x = xp + (size_t)n * D;
    const double *c = C + ((size_t)m * K + k) * D;
    double s = 0.0;
    for (int d = 0; d < D; ++d) {
        double t = x[d] - c[d];
        s = s + t * t;
    }
    return s;
}

/*
 * Centroid half of the k-means that cools: c_m(k) <- mean of the x'_n assigned to k;
 * a codeword with no member is left as it was.  counts[K] (may be NULL) receives n_k.
 * Returns the number of empty clusters.
 */
int da_update(const double *xp, const uint8_t *codes, double *C,
              int64_t N, int D, int M, int K, int m, int64_t *counts)
{
    double *Cm = C + (size_t)m * K * D;
    double *S = (double *)calloc((size_t)K * D, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)K, sizeof(int64_t));
    for (int64_t n = 0; n < N; ++n) {
        int k = codes[n * M + m];
        const double *x = xp + (size_t)n * D;
        double *s = S + (size_t)k * D;
        for (int d = 0; d < D; ++d) s[d] = s[d] + x[d];
        cnt[k] += 1;
    }
    int empty = 0;
    for (int k = 0; k < K; ++k) {
        if (cnt[k] > 0) {
            for (int d = 0; d < D; ++d)
                Cm[(size_t)k * D + d] = S[(size_t)k * D + d] / (double)cnt[k];
        } else {
            ++empty;
        }
        if (counts) counts[k] = cnt[k];
    }
    free(S);
    free(cnt);
    return empty;
}

/* Eq. 1, first line, averaged over the vectors: E = (1/N) sum_n ||e_n||^2. */
double da_quant_error(const double *r, int64_t N, int D)
{
    double total = 0.0;
    for (int64_t n = 0; n < N; ++n) {
        const double *rn = r + (size_t)n * D;
        double s = 0.0;
        for (int d = 0; d < D; ++d) s = s + rn[d] * rn[d];
        total = total + s;
    }
    return N > 0 ? total / (double)N : 0.0;
}

/*
 * Greedy residual encoding = multi-path encoding with a single path (Eq. 3, L = 1):
 * r <- x; for m = 1..M: i_m = argmin_k ||r - c_m(k)||^2, r <- r - c_m(i_m).
 * X is the fp32 input, widened exactly.
 */
void da_encode(const float *X, const double *C, int64_t N, int D, int M, int K,
               uint8_t *codes, double *r)
{
    for (size_t i = 0; i < (size_t)N * D; ++i) r[i] = (double)X[i];
    for (int m = 0; m < M; ++m) {
        da_assign(r, C, N, D, M, K, m, codes, NULL, NULL, NULL);
        da_cool(r, codes, C, N, D, M, K, m);
    }
}

/*
 * Multi-path encoding, one dictionary (Sec. 3.3, the left-hand side of Eq. 3).
 *
 * The beam holds Lc approximations a_l of every vector on the dictionaries before this one
 * (A: double[N][Lc][D]; Lc = 1 with a = 0 before the first dictionary).  All K*Lc sums
 * a_l + c(k) are scored by  e(l,k) = || x - a_l - c(k) ||^2  in its direct form and the
 * Ln = min(L, K*Lc) smallest are kept, in ascending order of e.
 * Reading where the paper is silent: equal e are ordered by (l, k) ascending, i.e. a stable
 * sort of the candidates enumerated l-major.
 *
 * Outputs per vector: parent[Ln] = l and code[Ln] = k of every kept sum, err[Ln] = its e,
 * A_next[Ln][D] = a_l + c(k).  gap (may be NULL) receives the smallest relative difference
 * (e_{i+1} - e_i) / e_{i+1} between neighbours among the first Ln + 1 sorted candidates (a
 * pair with e_{i+1} = 0 counts as 0; +inf when there is a single candidate): the tests use it
 * to tell a genuine near-tie from an error.
 */
typedef struct { double e; int l, k; } beam_cand;

static int beam_cmp(const void *pa, const void *pb)
{
    const beam_cand *a = (const beam_cand *)pa, *b = (const beam_cand *)pb;
    if (a->e < b->e) return -1;
    if (a->e > b->e) return 1;
    if (a->l != b->l) return a->l < b->l ? -1 : 1;
    return (a->k > b->k) - (a->k < b->k);
}

void da_beam_step(const float *X, const double *Cm, int64_t N, int D, int K, int Lc, int L,
                  const double *A, uint8_t *parent, uint8_t *code, double *err,
                  double *A_next, double *gap)
{
    const int total = K * Lc;
    const int Ln = L < total ? L : total;
#pragma omp parallel
    {
        beam_cand *cand = (beam_cand *)malloc(sizeof(beam_cand) * (size_t)total);
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            const float *x = X + (size_t)n * D;
            for (int l = 0; l < Lc; ++l) {
                const double *a = A + ((size_t)n * Lc + l) * D;
                for (int k = 0; k < K; ++k) {
                    const double *c = Cm + (size_t)k * D;
                    double e = 0.0;
                    for (int d = 0; d < D; ++d) {
                        const double t = (double)x[d] - a[d] - c[d];
                        e += t * t;
                    }
                    cand[l * K + k].e = e;
                    cand[l * K + k].l = l;
                    cand[l * K + k].k = k;
                }
            }
            qsort(cand, (size_t)total, sizeof(beam_cand), beam_cmp);   /* total order: no ties left */
            for (int i = 0; i < Ln; ++i) {
                parent[(size_t)n * Ln + i] = (uint8_t)cand[i].l;
                code[(size_t)n * Ln + i] = (uint8_t)cand[i].k;
                err[(size_t)n * Ln + i] = cand[i].e;
                const double *a = A + ((size_t)n * Lc + cand[i].l) * D;
                const double *c = Cm + (size_t)cand[i].k * D;
                double *an = A_next + ((size_t)n * Ln + i) * D;
                for (int d = 0; d < D; ++d) an[d] = a[d] + c[d];
            }
            if (gap) {
                double g = INFINITY;
                const int last = Ln < total ? Ln : total - 1;        /* index of the last right neighbour */
                for (int i = 0; i < last; ++i) {
                    const double hi = cand[i + 1].e, lo = cand[i].e;
                    const double rel = hi > 0.0 ? (hi - lo) / hi : 0.0;
                    if (rel < g) g = rel;
                }
                gap[n] = g;
            }
        }
        free(cand);
    }
}

/*
 * Multi-path encoding of X on all M dictionaries in order (Sec. 3.3): da_beam_step for
 * m = 1..M starting from the single empty sum, carrying the code prefix of every kept sum;
 * the answer is the best sum of the last beam.  codes: uint8[N][M]; r: double[N][D] receives
 * x - sum_m c_m(i_m); err (may be NULL): double[N] its squared norm as scored; gap (may be
 * NULL): double[N], the smallest da_beam_step gap over the M steps.
 */
void da_encode_beam(const float *X, const double *C, int64_t N, int D, int M, int K, int L,
                    uint8_t *codes, double *r, double *err, double *gap)
{
    int Lc = 1;
    double *A = (double *)calloc((size_t)N * D, sizeof(double));
    uint8_t *pre = (uint8_t *)calloc((size_t)N * (M > 0 ? M : 1), 1);      /* [N][Lc][M] */
    double *g = gap ? (double *)malloc(sizeof(double) * (size_t)N) : NULL;
    double *e = NULL;
    if (gap) for (int64_t n = 0; n < N; ++n) gap[n] = INFINITY;
    for (int m = 0; m < M; ++m) {
        const long total = (long)K * Lc;
        const int Ln = L < total ? L : (int)total;
        uint8_t *parent = (uint8_t *)malloc((size_t)N * Ln);
        uint8_t *code = (uint8_t *)malloc((size_t)N * Ln);
        double *en = (double *)malloc(sizeof(double) * (size_t)N * Ln);
        double *An = (double *)malloc(sizeof(double) * (size_t)N * Ln * D);
        uint8_t *pn = (uint8_t *)calloc((size_t)N * Ln * M, 1);
        da_beam_step(X, C + (size_t)m * K * D, N, D, K, Lc, L, A, parent, code, en, An, g);
        for (int64_t n = 0; n < N; ++n) {
            for (int i = 0; i < Ln; ++i) {
                const uint8_t *src = pre + ((size_t)n * Lc + parent[(size_t)n * Ln + i]) * M;
                uint8_t *dst = pn + ((size_t)n * Ln + i) * M;
                memcpy(dst, src, (size_t)m);
                dst[m] = code[(size_t)n * Ln + i];
            }
            if (gap && g[n] < gap[n]) gap[n] = g[n];
        }
        free(A); free(pre); free(parent); free(code); free(e);
        A = An; pre = pn; e = en; Lc = Ln;
    }
    for (int64_t n = 0; n < N; ++n) {
        memcpy(codes + (size_t)n * M, pre + (size_t)n * Lc * M, (size_t)M);
        const double *a = A + (size_t)n * Lc * D;
        for (int d = 0; d < D; ++d) r[(size_t)n * D + d] = (double)X[(size_t)n * D + d] - a[d];
        if (err) {
            double q = 0.0;                                            /* M == 0: nothing subtracted */
            for (int d = 0; d < D; ++d) q += r[(size_t)n * D + d] * r[(size_t)n * D + d];
            err[n] = e ? e[(size_t)n * Lc] : q;
        }
    }
    free(A); free(pre); free(e); free(g);
}

/*
 * One DA iteration on dictionary m (Sec. 3.1): heat, optional seeding of an all-zero
 * dictionary from rows of x' (init_idx[K], may be NULL), T x (assign, update), a final
 * assign against the final C_m (the stage-local re-encode), cool.
 * Precondition: r == x - sum_j C_j[codes[:,j]].
 * J (may be NULL) receives 2T+2 values of (1/N) sum ||x' - C_m[i]||^2: at stage entry,
 * after every assign and every update, and after the final assign.
 * Returns E after the stage.
 */
double da_anneal_stage(int m, double *C, uint8_t *codes, double *r,
                       int64_t N, int D, int M, int K, int T,
                       const int64_t *init_idx, double *J)
{
    double *Cm = C + (size_t)m * K * D;
    int j = 0;
    if (J) J[j++] = da_quant_error(r, N, D);
    da_heat(r, codes, C, N, D, M, K, m);               /* r now holds x' */
    if (init_idx) {
        for (int k = 0; k < K; ++k)
            memcpy(Cm + (size_t)k * D, r + (size_t)init_idx[k] * D, sizeof(double) * D);
    }
    for (int t = 0; t < T; ++t) {
        da_assign(r, C, N, D, M, K, m, codes, NULL, NULL, NULL);
        if (J) {
            da_cool(r, codes, C, N, D, M, K, m);
            J[j++] = da_quant_error(r, N, D);
            da_heat(r, codes, C, N, D, M, K, m);
        }
        da_update(r, codes, C, N, D, M, K, m, NULL);
        if (J) {
            da_cool(r, codes, C, N, D, M, K, m);
            J[j++] = da_quant_error(r, N, D);
            da_heat(r, codes, C, N, D, M, K, m);
        }
    }
    da_assign(r, C, N, D, M, K, m, codes, NULL, NULL, NULL);
    da_cool(r, codes, C, N, D, M, K, m);               /* r holds the residue again */
    double E = da_quant_error(r, N, D);
    if (J) J[j++] = E;
    return E;
}

/*
 * One sweep: DA iteration on m = 0..M-1 in order (Sec. 3.1, "multiple iterations").
 * init_idx: NULL or int64[M][K].  err_per_stage: NULL or double[M].
 */
void da_sweep(double *C, uint8_t *codes, double *r,
              int64_t N, int D, int M, int K, int T,
              const int64_t *init_idx, double *err_per_stage)
{
    for (int m = 0; m < M; ++m) {
        double E = da_anneal_stage(m, C, codes, r, N, D, M, K, T,
                                   init_idx ? init_idx + (size_t)m * K : NULL, NULL);
        if (err_per_stage) err_per_stage[m] = E;
    }
}

/*
 * Sec. 3.4, online learning: keep fitting the learned dictionaries to newly arriving data.
 * The paper gives no update rule; the reading taken is running per-codeword sums S and counts
 * cnt over everything seen so far.  For one chunk X (uint8 [n][D], as SIFT descriptors are
 * stored) and each dictionary m in order, with r the chunk's residue so far (r = x for m = 0):
 *   assign r to C_m;  S_m[k] += sum of its members, cnt_m[k] += their number;
 *   c_m(k) <- S_m[k] / cnt_m[k] where cnt_m[k] > 0;  assign again;  r <- r - c_m(i_m).
 * S: double[M][K][D], cnt: int64[M][K] are updated in place.  Returns E of the chunk.
 */
double da_online_chunk(const uint8_t *X, int64_t n, int D, int M, int K,
                       double *C, double *S, int64_t *cnt, uint8_t *codes, double *r)
{
    for (size_t i = 0; i < (size_t)n * D; ++i) r[i] = (double)X[i];
    for (int m = 0; m < M; ++m) {
        double *Cm = C + (size_t)m * K * D;
        double *Sm = S + (size_t)m * K * D;
        int64_t *cm = cnt + (size_t)m * K;
        da_assign(r, C, n, D, M, K, m, codes, NULL, NULL, NULL);
        for (int64_t v = 0; v < n; ++v) {
            const int k = codes[v * M + m];
            const double *x = r + (size_t)v * D;
            for (int d = 0; d < D; ++d) Sm[(size_t)k * D + d] = Sm[(size_t)k * D + d] + x[d];
            cm[k] += 1;
        }
        for (int k = 0; k < K; ++k)
            if (cm[k] > 0)
                for (int d = 0; d < D; ++d) Cm[(size_t)k * D + d] = Sm[(size_t)k * D + d] / (double)cm[k];
        da_assign(r, C, n, D, M, K, m, codes, NULL, NULL, NULL);
        da_cool(r, codes, C, n, D, M, K, m);
    }
    return da_quant_error(r, n, D);
}

/*
 * Sec. 3.2, step 1 / step 3: y_n = R x_n (transpose == 0) or y_n = R^T x_n (transpose != 0),
 * R: double[D][D] row-major, its rows are the principal axes.  y may not alias x.
 */
void da_rotate(const double *x, int64_t N, int D, const double *R, int transpose, double *y)
{
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const double *xn = x + (size_t)n * D;
        double *yn = y + (size_t)n * D;
        for (int i = 0; i < D; ++i) {
            double s = 0.0;
            for (int j = 0; j < D; ++j)
                s = s + (transpose ? R[(size_t)j * D + i] : R[(size_t)i * D + j]) * xn[j];
            yn[i] = s;
        }
    }
}

/* Nearest codeword using only the first dact coordinates (Sec. 3.2, step 2); Cm: double[K][D]. */
static void assign_prefix(const double *xr, const double *Cm, int64_t N, int D, int dact, int K,
                          uint8_t *codes, int M, int m)
{
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const double *x = xr + (size_t)n * D;
        double best = INFINITY;
        int ibest = 0;
        for (int k = 0; k < K; ++k) {
            const double *c = Cm + (size_t)k * D;
            double s = 0.0;
            for (int d = 0; d < dact; ++d) {
                double t = x[d] - c[d];
                s = s + t * t;
            }
            if (k == 0 || s < best) { best = s; ibest = k; }
        }
        codes[n * M + m] = (uint8_t)ibest;
    }
}

/*
 * Sec. 3.2, improved k-means as the cool-down of one DA iteration on dictionary m:
 *   heat (Sec. 3.1); optional seeding; x^r = R x', C' = R C_m;
 *   for each d in dims[0] < ... < dims[I-1] = D:  T Lloyd iterations whose assignment uses only the
 *   first d coordinates of x^r and C' and whose centroid update takes the mean over all D
 *   coordinates (so the clustering found on few dimensions is what the next, larger prefix starts from);
 *   C_m = R^T C';  final assign in the original space; new residue.
 * R is an input (principal axes of {x'} as rows, most variance first).  Returns E after the stage.
 */
double da_anneal_stage_pca(int m, double *C, uint8_t *codes, double *r,
                           int64_t N, int D, int M, int K, const double *R,
                           const int *dims, int I, int T, const int64_t *init_idx)
{
    double *Cm = C + (size_t)m * K * D;
    da_heat(r, codes, C, N, D, M, K, m);
    if (init_idx)
        for (int k = 0; k < K; ++k)
            memcpy(Cm + (size_t)k * D, r + (size_t)init_idx[k] * D, sizeof(double) * D);
    double *xr = (double *)malloc(sizeof(double) * (size_t)N * D);
    double *Cp = (double *)malloc(sizeof(double) * (size_t)K * D);
    double *S = (double *)malloc(sizeof(double) * (size_t)K * D);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)K);
    da_rotate(r, N, D, R, 0, xr);
    da_rotate(Cm, K, D, R, 0, Cp);
    for (int i = 0; i < I; ++i) {
        for (int t = 0; t < T; ++t) {
            assign_prefix(xr, Cp, N, D, dims[i], K, codes, M, m);
            memset(S, 0, sizeof(double) * (size_t)K * D);
            memset(cnt, 0, sizeof(int64_t) * (size_t)K);
            for (int64_t n = 0; n < N; ++n) {
                const int k = codes[n * M + m];
                const double *x = xr + (size_t)n * D;
                for (int d = 0; d < D; ++d) S[(size_t)k * D + d] = S[(size_t)k * D + d] + x[d];
                cnt[k] += 1;
            }
            for (int k = 0; k < K; ++k)
                if (cnt[k] > 0)
                    for (int d = 0; d < D; ++d) Cp[(size_t)k * D + d] = S[(size_t)k * D + d] / (double)cnt[k];
        }
    }
    da_rotate(Cp, K, D, R, 1, Cm);
    free(xr); free(Cp); free(S); free(cnt);
    da_assign(r, C, N, D, M, K, m, codes, NULL, NULL, NULL);
    da_cool(r, codes, C, N, D, M, K, m);
    return da_quant_error(r, N, D);
}

/* x_hat_n = sum_m c_m(i_m(n)) (used to check x = x_hat + r). */
void da_reconstruct(const double *C, const uint8_t *codes, int64_t N, int D, int M, int K,
                    double *xhat)
{
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double *o = xhat + (size_t)n * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int m = 0; m < M; ++m) {
            const double *c = C + ((size_t)m * K + codes[n * M + m]) * D;
            for (int d = 0; d < D; ++d) o[d] = o[d] + c[d];
        }
    }
}
