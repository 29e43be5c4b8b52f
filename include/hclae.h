/*
 * libhclae -- Dictionary Annealing (DA) sweep on one AMD MI355X (gfx950).
 *
 * Method: "HCLAE: High Capacity Locally Aggregating Encodings for Approximate Nearest
 * Neighbor Search", arXiv 1509.05194.  The library implements the data-parallel part of
 * Sec. 3.1 (Dictionary Annealing) with the single-path case of Sec. 3.3 (Eq. 3, L = 1)
 * as its encoder and Eq. 1 (first line) as its error measure.
 *
 * Notation (the paper's, with 0-based indices):
 *   N vectors x in R^D;  M dictionaries C_m of K codewords c_m(k);  code i_m(x) in [0,K);
 *   residue e_x = x - sum_m c_m(i_m(x));  intermediate vector x' = e_x + c_m(i_m(x)).
 *
 * Layouts (all row-major, all DEVICE memory unless marked HOST):
 *   X, residue : float   [N][D]      (D % 4 == 0)
 *   C          : float   [M][K][D]
 *   Every float array (these, beam rows, R, rotated copies) is read and written four floats at a
 *   time: its base must be 16-byte aligned, else the call returns HCLAE_EINVAL.
 *   Values must be finite: the library does not scan its inputs, and with a NaN or an infinity in
 *   X, residue or C the behaviour is undefined.
 *   codes      : uint8_t [N][M]      (the paper's M-byte code; K <= 256)
 *
 * Ownership: every data pointer is caller-owned; the library neither allocates nor frees
 * them and keeps no pointer after a call returns.  An hclae_ctx owns scratch memory only.
 *
 * Ordering: all work is enqueued on the HIP stream given to hclae_create.  Calls return
 * after enqueueing, except where a HOST output is requested (stats, err_per_stage, out):
 * those synchronise that stream before returning.  One ctx must not be used from two
 * threads at once.
 *
 * Errors: every entry point returns HCLAE_OK or a negative code.  Arguments are checked
 * before any HIP call; on HCLAE_EINVAL nothing was enqueued and no state changed.
 * A failing HIP call gives HCLAE_EHIP; hclae_last_error(ctx) then holds its text.
 * With N == 0 every call is a no-op that returns HCLAE_OK (data pointers may then be NULL).
 * Argmin ties go to the lowest index.  A codeword whose cluster is empty keeps its value.
 */
#ifndef HCLAE_H
#define HCLAE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hclae_ctx hclae_ctx;

enum {
    HCLAE_OK     = 0,
    HCLAE_EINVAL = -1,   /* bad argument (null pointer, size out of range, shape mismatch) */
    HCLAE_ENOMEM = -2,   /* scratch allocation failed                                       */
    HCLAE_EHIP   = -3,   /* a HIP runtime call failed                                       */
    HCLAE_ESTATE = -4    /* call exceeds what the ctx was created for                       */
};

/* Limits checked by every entry point. */
#define HCLAE_MAX_K 256
#define HCLAE_MAX_D 4096
#define HCLAE_MAX_M 256

typedef struct {
    double  err_before;      /* (1/N) sum ||e_x||^2 at stage entry                          */
    double  err_after;       /* same at stage exit                                          */
    int64_t codes_changed;   /* vectors whose i_m differs from its value at stage entry     */
    int64_t refined;         /* vectors of the final assign decided by the fp64 re-check
                                (with pruning: among the vectors that assign recomputed)    */
    int32_t empty_clusters;  /* codewords with no member at the last centroid update        */
    int32_t iters_run;       /* Lloyd iterations executed                                   */
} hclae_stage_stats;

/* Shape check shared by all entry points: HCLAE_OK iff 0 <= N < 2^31, 4 <= D <= HCLAE_MAX_D
 * with D % 4 == 0, 1 <= M <= HCLAE_MAX_M, 1 <= K <= HCLAE_MAX_K.  Needs no device. */
int hclae_check_shape(int64_t N, int D, int M, int K);

/* Create a context whose scratch fits calls with N <= N_max and exactly this D, M, K.
 * hip_stream: a hipStream_t (NULL = the default stream).  The current device is used. */
int hclae_create(hclae_ctx **out, int64_t N_max, int D, int M, int K, void *hip_stream);
int hclae_destroy(hclae_ctx *ctx);
/* Text of the last error of this ctx (never NULL; valid until the next call on it).
 * With ctx == NULL: text of the last error of a failed hclae_create on this thread. */
const char *hclae_last_error(const hclae_ctx *ctx);

/*
 * Sec. 3.3, Eq. 3 with one path (greedy residual encoding) under the objective of Eq. 1:
 *   r <- x;  for m = 0..M-1:  i_m = argmin_k ||r - c_m(k)||^2,  r <- r - c_m(i_m).
 * Reads X and C; writes codes[N][M] and residue[N][D] (residue may not alias X).
 */
int hclae_encode(hclae_ctx *ctx, const float *X, int64_t N, int D,
                 const float *C, int M, int K, uint8_t *codes, float *residue);

/*
 * Sec. 3.1, one DA iteration on dictionary m:
 *   heat   x' = e_x + c_m(i_m(x))                              (in place over residue)
 *   [seed  c_m(k) <- x'[init_idx[k]] : the "all-zeros dictionary" start, where x' = e_x]
 *   cool   iters x ( i_m = argmin_k ||x' - c_m(k)||^2 ;  c_m(k) <- mean of its members )
 *   re-encode  i_m = argmin_k ||x' - c_m(k)||^2 ;  e_x = x' - c_m(i_m)
 * Updates C[m], column m of codes and residue in place.
 * Precondition: residue == X - sum_j C[j][codes[:,j]].
 * init_idx: HOST int64[K] of row indices in [0,N), or NULL.  stats: HOST, or NULL.
 */
int hclae_anneal_stage(hclae_ctx *ctx, int m, int64_t N, int D, float *C, int M, int K,
                       uint8_t *codes, float *residue, int iters,
                       const int64_t *init_idx, hclae_stage_stats *stats);

/*
 * Sec. 3.1, "multiple iterations": hclae_anneal_stage for m = 0..M-1 in order.
 * reencode_mode 0: each stage re-encodes only its own column (keeps E non-increasing).
 * reencode_mode 1: after each stage all M parts are re-encoded greedily from X
 *                  (hclae_encode); X must then be non-NULL.
 * reencode_mode 2: as 1 with the multi-path encoder (hclae_encode_beam) of the width set by
 *                  hclae_set_beam_width (10 unless set).
 * init_idx: HOST int64[M][K] or NULL.  err_per_stage: HOST double[M] or NULL
 * (mean ||e_x||^2 after each stage).
 * The k-means that cools each stage is the one hclae_set_cooldown chose (plain Lloyd iterations unless set).
 * With the plain cool-down, reencode_mode 0, init_idx == NULL and err_per_stage == NULL the call only enqueues kernels on the
 * context's stream (no allocation, copy, memset or synchronisation; all data-dependent sizes are read on the
 * device), so it may be recorded into a HIP graph on that stream and replayed.
 */
int hclae_sweep(hclae_ctx *ctx, const float *X, int64_t N, int D, float *C, int M, int K,
                uint8_t *codes, float *residue, int iters, int reencode_mode,
                const int64_t *init_idx, double *err_per_stage);

/*
 * Sec. 3.1, "multiple iterations" of the whole method: n_sweeps sweeps over the dictionaries
 * (hclae_sweep with reencode_mode 0, n_sweeps times; init_idx, if given, seeds the all-zero dictionaries of the
 * first sweep as it does there, NULL for the others).  C, codes and residue end with the very
 * bits those calls give; what the single call adds is speed in late sweeps: every stage but the last passes
 * into the next through the fused row pass, from one sweep to the next as well, and (plain Lloyd cool-down with
 * the exact shortcuts on, iters > 0, at least two sweeps that do not seed) each stage keeps the distance bounds it
 * ends with and starts its next visit from them, widened by how far x' has moved since, so that the first assignment
 * of a stage also runs only over the vectors the bounds cannot settle.  The arrays this needs (16 * M + 8 bytes per
 * vector of N_max) are allocated at the first such call and kept by the ctx.
 *   C: DEVICE float[M][K][D], codes: DEVICE uint8[N][M], residue: DEVICE float[N][D], all updated in place.
 *   Precondition: residue == X - sum_j C[j][codes[:,j]].
 *   init_idx: HOST int64[M][K] or NULL.  err_per_stage: HOST double[n_sweeps][M] (mean ||e_x||^2 after each stage;
 *   the stream is synchronised once per sweep) or NULL (without init_idx the call then only enqueues, apart from
 *   that first allocation; with it, it synchronises once at the end).
 */
int hclae_anneal(hclae_ctx *ctx, int64_t N, int D, float *C, int M, int K, uint8_t *codes, float *residue,
                 int iters, int n_sweeps, const int64_t *init_idx, double *err_per_stage);

/* Eq. 1, first line, averaged over the vectors (Table 1 reports such means):
 *   *out = (1/N) sum_n ||residue_n||^2, accumulated in fp64.  out: HOST.  N == 0 gives 0. */
int hclae_quant_error(hclae_ctx *ctx, const float *residue, int64_t N, int D, double *out);

/*
 * hclae_quant_error for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Needs no hclae_ctx and calls no hipMalloc, hipFree or other allocating
 * routine; its scratch (one fp64 partial sum per block of the reduction, 32 KB) is a static device array
 * inside the library, which every GPU the library runs on holds until the process ends.
 *   residue: DEVICE float[N][D], 16-byte aligned.  out: DEVICE double (8-byte aligned), receives
 *   (1/N) sum_n ||residue_n||^2 (0 when N == 0) -- the same bits hclae_quant_error returns on a 256-CU device.
 *   hip_stream: the hipStream_t the two kernels are enqueued on (NULL = the default stream); the call does
 *   not synchronise.  The current device is used.
 * Limits: 0 <= N < 2^31, 4 <= D <= 4096, D % 4 == 0; anything beyond is rejected with HCLAE_EINVAL before a
 * launch (text via hclae_last_error(NULL)).  All calls on one GPU share that GPU's scratch: calls that may
 * overlap on one GPU (different streams or threads) race and must be ordered by the caller.  Nothing in the
 * scratch has to start at zero (every partial read has been written by the same call), so it is not cleared.
 */
int hclae_quant_error_noalloc(const float *residue, int64_t N, int D, double *out, void *hip_stream);

/* ---- single steps of a stage (Sec. 3.1), exported so each can be checked on its own ---- */

/* heat: residue_n += C[m][codes[n][m]] */
int hclae_heat(hclae_ctx *ctx, int m, int64_t N, int D, const float *C, int M, int K,
               const uint8_t *codes, float *residue);
/* new residue: xp_n -= C[m][codes[n][m]] */
int hclae_cool(hclae_ctx *ctx, int m, int64_t N, int D, const float *C, int M, int K,
               const uint8_t *codes, float *xp);
/* assignment half of the cooling k-means: codes[n][m] = argmin_k ||xp_n - C[m][k]||^2.
 * dmin: DEVICE float[N] or NULL; receives ||xp_n - C[m][codes[n][m]]||^2 (direct form). */
int hclae_assign(hclae_ctx *ctx, int m, int64_t N, int D, const float *xp, const float *C,
                 int M, int K, uint8_t *codes, float *dmin);
/* centroid half: C[m][k] = mean of xp_n with codes[n][m] == k (unchanged when empty).
 * counts: DEVICE int32[K] or NULL; receives the cluster sizes. */
int hclae_update(hclae_ctx *ctx, int m, int64_t N, int D, const float *xp, float *C,
                 int M, int K, const uint8_t *codes, int32_t *counts);

/* Number of vectors the last hclae_assign (or the last assign inside a stage / encode) sent
 * to the fp64 re-check because their two best fp32 scores were closer than the rounding
 * bound of the fp32 contraction.  Synchronises the stream.  out: HOST. */
int hclae_last_refined(hclae_ctx *ctx, int64_t *out);

/* ---- online learning (Sec. 3.4: keep fitting learned dictionaries to newly arriving data) ---- */

/*
 * The paper states no update rule; the reading taken is running per-codeword sums and counts over
 * everything seen so far, held by the ctx.  hclae_online_begin sets them from the current
 * dictionaries: sums = C * n0, counts = n0 (n0: HOST int64[M][K] weights of what C was learned
 * from, or NULL for all zero, in which case the first chunk replaces every codeword it touches).
 */
int hclae_online_begin(hclae_ctx *ctx, const float *C, int M, int K, int D, const int64_t *n0);

/*
 * One chunk of n new vectors, given as stored descriptors Xu8 (DEVICE uint8 [n][D], 16-byte aligned,
 * else HCLAE_EINVAL).  For each
 * dictionary m in order, with r the chunk's residue so far (r = x for m = 0):
 *   assign r to C_m;  add its members to the running sums and counts;  c_m(k) <- sum / count
 *   where count > 0;  assign again;  r <- r - c_m(i_m).
 * Updates C in place; writes codes [n][M] and residue [n][D] (both DEVICE, caller-owned, required).
 * codes_first: DEVICE uint8 [n][M] or NULL; receives the codes of each stage's FIRST assignment,
 * i.e. the memberships that entered the running sums (codes holds the re-assigned ones).
 * err: HOST, receives (1/n) sum ||residue||^2 and synchronises the stream; or NULL (no sync).
 * The caller may overlap the host-to-device copy of the next chunk on another stream.
 */
int hclae_online_chunk(hclae_ctx *ctx, const uint8_t *Xu8, int64_t n, int D, float *C, int M, int K,
                       uint8_t *codes, float *residue, uint8_t *codes_first, double *err);

/* Checkpoint / resume of the online state at a chunk boundary: running sums (HOST double[M][K][D])
 * and counts (HOST int64[M][K]).  Both synchronise the stream.  Together with C they are the
 * whole state of the learner. */
int hclae_online_export(hclae_ctx *ctx, double *run_sum, int64_t *run_cnt);
int hclae_online_import(hclae_ctx *ctx, const double *run_sum, const int64_t *run_cnt);

/* ---- choice of the matrix-core arithmetic of the distance contraction ------------------------- */

#define HCLAE_CONTRACT_F32        0   /* fp32 MFMA (default)                                         */
#define HCLAE_CONTRACT_SPLIT_BF16 1   /* fp32 operands split into two bf16 terms, three bf16 MFMAs   */

/*
 * Selects how the nearest-codeword kernels (Sec. 3.1 / 3.2 assignment; every entry point that assigns)
 * form the scores x'.c - ||c||^2/2.  Either way the scores only pre-select candidates within an error margin
 * (mode 0: a rigorous bound of the fp32 accumulation; mode 1: the dropped terms bounded rigorously, the
 * accumulation of a bf16 MFMA by a measured constant with a fourfold allowance) and the decision is the fp64
 * direct-form re-check, so codes, dictionaries and residues do not depend on the mode; only the number of
 * vectors that take the re-check does.  Mode 1 applies to the
 * assignments and to the multi-path scoring (hclae_beam_step, hclae_encode_beam) of every shape.
 */
int hclae_set_contraction(hclae_ctx *ctx, int mode);

/*
 * Exact shortcuts of the Lloyd iterations of hclae_anneal_stage / hclae_sweep (on by default; on = 0 makes
 * every assignment and every centroid sum of a stage run over all N vectors).  x' is fixed during a stage, so
 * (1) per vector an upper bound on the distance to its codeword and a lower bound on the distance to all
 *     others are kept, aged by how far the codewords move in each centroid update (triangle inequality), and
 *     only vectors whose bounds stop separating are assigned again;
 * (2) the integer totals of the first centroid update are kept and later updates add only the vectors that
 *     changed cluster.
 * The bounds include the rounding bounds of the kernels and the sums are exact integers, so the results are
 * those of the full passes, bit for bit; only the work differs.
 */
int hclae_set_pruning(hclae_ctx *ctx, int on);

/* ---- multi-path encoding (Sec. 3.3, Eq. 3) ---------------------------------------------------- */

#define HCLAE_MAX_L 32     /* paths kept per vector */

/*
 * One dictionary of the multi-path encoding.  The beam of every vector is held as residuals
 * r_l = x - a_l of its Lc kept sums a_l:  rows DEVICE float[N][Lc][D], err DEVICE double[N][Lc] =
 * ||r_l||^2 (NULL means all zero and is allowed when Lc == 1, where it only shifts every score).
 * All K * Lc candidates are scored by ||r_l - c(k)||^2 (the left-hand side of Eq. 3) and the
 * Ln = min(L, K * Lc) smallest are kept in ascending order, equal errors in (l, k) order:
 *   rows_next DEVICE float[N][Ln][D] = r_l - c(k) (must not alias rows), err_next DEVICE double[N][Ln],
 *   parent / code DEVICE uint8[N][Ln] = l / k.  err_next, parent and code may be NULL.
 * Cm: DEVICE float[K][D].  1 <= Lc <= L <= HCLAE_MAX_L, N * L < 2^31.
 * Decisions are taken on fp64 direct-form errors of the fp32 rows (candidates pre-selected on the
 * fp32 matrix cores with a rigorous rounding margin).
 */
int hclae_beam_step(hclae_ctx *ctx, const float *rows, const double *err, const float *Cm,
                    int64_t N, int D, int K, int Lc, int L,
                    float *rows_next, double *err_next, uint8_t *parent, uint8_t *code);

/*
 * Multi-path encoding of X on dictionaries 0..M-1 in order with L paths; the answer is the best
 * sum of the last beam.  Writes codes[N][M], residue[N][D] = x - sum_m c_m(i_m) (must not alias X)
 * and, when err != NULL, err DEVICE double[N] = its squared norm as scored.  L = 1 is hclae_encode.
 * Scratch for batches of vectors is allocated by the first call and kept by the ctx.
 */
int hclae_encode_beam(hclae_ctx *ctx, const float *X, int64_t N, int D, const float *C, int M, int K, int L,
                      uint8_t *codes, float *residue, double *err);

/* Width of the multi-path re-encode that hclae_sweep runs with reencode_mode 2. */
int hclae_set_beam_width(hclae_ctx *ctx, int L);

/* ---- improved k-means for high-dimensional residue (Sec. 3.2) --------------------------------- */

/* Second moments of {x'} for its PCA: mean (DEVICE double[D]) and centred covariance (DEVICE
 * double[D][D], divided by N). */
int hclae_covariance(hclae_ctx *ctx, const float *xp, int64_t N, int D, double *mean, double *cov);

/* Step 1 of Sec. 3.2, the PCA space of {x'}: R (DEVICE float[D][D]) receives the principal axes of the N rows
 * of xp as its rows, most variance first, each signed so that its entry of largest magnitude is positive;
 * eigenvalues (HOST double[D], descending; may be NULL) the variances along them.  Second moments on the device
 * (hclae_covariance), eigen-decomposition of the D x D matrix on the host in fp64 (Householder tridiagonal form,
 * implicit-shift QR).  Synchronises the stream. */
int hclae_pca_axes(hclae_ctx *ctx, const float *xp, int64_t N, int D, float *R, double *eigenvalues);

/* The eigen-solver of hclae_pca_axes on its own; needs no device.  A: HOST double[n][n], symmetric, not
 * modified.  w: HOST double[n], eigenvalues descending.  Vt: HOST double[n][n], row i = unit eigenvector of
 * w[i] with its entry of largest magnitude positive.  1 <= n <= HCLAE_MAX_D.  HCLAE_ESTATE if the iteration
 * does not converge. */
int hclae_symmetric_eigen(const double *A, int n, double *w, double *Vt);

/* Step 1 / step 3 of Sec. 3.2: out_n = R x_n (transpose == 0) or R^T x_n (transpose != 0) for the N rows
 * of x.  R: DEVICE float[D][D] row-major.  out: DEVICE float[N][D], must not alias x. */
int hclae_rotate(hclae_ctx *ctx, const float *x, int64_t N, int D, const float *R, int transpose, float *out);

/* Assignment on a prefix (step 2 of Sec. 3.2): codes[n][m] = argmin_k of the squared distance over the
 * first dact coordinates of xp_n and C[m][k]; rows keep their stride D. */
int hclae_assign_prefix(hclae_ctx *ctx, int m, int64_t N, int D, const float *xp, const float *C,
                        int M, int K, int dact, uint8_t *codes);

/*
 * hclae_anneal_stage with the improved k-means as cool-down:
 *   heat; [seed]; x^r = R x', C' = R C_m;
 *   for d in dims[0] < ... < dims[n_dims-1] = D: iters_per_dim Lloyd iterations whose assignment uses the
 *   first d coordinates and whose centroid update is the mean over all D coordinates;
 *   C_m = R^T C'; re-encode (assign in the original space); new residue.
 * R: DEVICE float[D][D], the principal axes as rows; or NULL, in which case the stage computes them from
 * its own x' (hclae_pca_axes; this synchronises the stream once).  dims: HOST int[n_dims].  xr: DEVICE
 * float[N][D] scratch (caller-owned, holds x^r on return).  Other arguments as hclae_anneal_stage.
 */
int hclae_anneal_stage_pca(hclae_ctx *ctx, int m, int64_t N, int D, float *C, int M, int K,
                           uint8_t *codes, float *residue, const float *R, const int *dims, int n_dims,
                           int iters_per_dim, float *xr, const int64_t *init_idx, hclae_stage_stats *stats);

/* The dimension schedule of Sec. 3.2: d_i = ceil(D^(i/phases)), i = 1..phases (the printed d^(i/I) is no integer:
 * rounded up), equal values once, the last one D.  dims: HOST int[phases]; *n_dims: how many were written.
 * Needs no device.  1 <= phases <= 64. */
int hclae_dimension_schedule(int D, int phases, int *dims, int *n_dims);

#define HCLAE_COOLDOWN_LLOYD    0   /* plain full-dimension Lloyd iterations (default)                       */
#define HCLAE_COOLDOWN_IMPROVED 1   /* the improved k-means of Sec. 3.2                                       */

/*
 * Which k-means cools a dictionary in hclae_anneal_stage and hclae_sweep (Sec. 3.1 cools with "a k-means"; Sec. 3.2
 * gives the improved one for high-dimensional residue).  With HCLAE_COOLDOWN_IMPROVED every stage runs as
 * hclae_anneal_stage_pca does with R = NULL: principal axes of its own x', the schedule of `phases` prefixes
 * (hclae_dimension_schedule; 10 in the paper), ceil(iters / prefixes) Lloyd iterations on each prefix -- `iters`
 * being the argument of the stage or sweep call -- rotation back, re-encode in the original space.  Such a stage
 * synchronises the stream once (the eigen-decomposition runs on the host), keeps heat and new residue as separate
 * passes, and does not use the distance-bound shortcuts; x^r lives in scratch (N_max x D floats) that the first such
 * stage allocates and the ctx keeps.  phases is ignored with HCLAE_COOLDOWN_LLOYD.
 */
int hclae_set_cooldown(hclae_ctx *ctx, int mode, int phases);

/* ---- dictionary order and code statistics (Sec. 3.3, Sec. 2.2) --------------------------------- */

/* Sec. 3.3: dictionaries put in descending order of the variance of their codewords.
 * The variance of dictionary m is read as (1/K) sum_k ||c_m(k) - mean_k c_m||^2.  Writes var (HOST
 * double[M], variances in the OLD order) and order (HOST int[M]: new position j holds old dictionary
 * order[j]; ties keep the lower old index), then permutes C and the columns of codes accordingly, in place.
 * The residue is unchanged (the sum of the selected codewords does not depend on their order).
 * var and order may be NULL.  Synchronises the stream.  Scratch (a copy of C) is allocated by the first call
 * and kept by the ctx. */
int hclae_reorder_by_variance(hclae_ctx *ctx, int64_t N, int D, float *C, int M, int K, uint8_t *codes,
                              double *var, int *order);

/* Sec. 2.2: counts behind the self-information H(I_m) and the mutual information of two code parts.
 * hist: HOST int64[M][K], hist[m][k] = #{n : codes[n][m] == k}.  joint: HOST int64[K][K] for the pair of
 * columns (a, b), joint[i][j] = #{n : codes[n][a] == i and codes[n][b] == j}; may be NULL.  Synchronises. */
int hclae_code_stats(hclae_ctx *ctx, const uint8_t *codes, int64_t N, int M, int K,
                     int64_t *hist, int a, int b, int64_t *joint);

/* ---- measurement: work done, and per-kernel durations from HIP events on the ctx's stream ------------- */

/* Work since hclae_create or the last reset, counted on the device: out[0] = nearest-codeword assignments run
 * (Sec. 3.1 cool-down and re-encode, Eq. 3 with one path), out[1] = vectors those assignments recomputed (all N
 * of a full assignment, the listed ones of an assignment the distance bounds pruned), out[2] = vectors decided by
 * the fp64 re-check.  out: HOST int64[3].  reset != 0 zeroes the counters.  Synchronises the stream. */
int hclae_work_counters(hclae_ctx *ctx, int64_t *out, int reset);


enum {
    HCLAE_T_HEAT = 0,   /* heat pass (Sec. 3.1, x' = e_x + c)                              */
    HCLAE_T_COOL,       /* new-residue pass                                                 */
    HCLAE_T_ASSIGN,     /* fp32-MFMA distance contraction + argmin                          */
    HCLAE_T_REFINE,     /* fp64 re-check of near-ties                                       */
    HCLAE_T_ACCUM,      /* centroid sums and counts                                         */
    HCLAE_T_MERGE,      /* merge of the block partials, division, codeword norms            */
    HCLAE_T_NORMS,      /* codeword norms alone                                             */
    HCLAE_T_ERROR,      /* Eq. 1 reduction alone                                            */
    HCLAE_T_TRANSITION, /* fused stage boundary of hclae_sweep: new residue of m + heat of m+1 */
    HCLAE_T_ROTATE,     /* projection y = R x (Sec. 3.2)                                    */
    HCLAE_T_MOMENTS,    /* mean and covariance of x' (Sec. 3.2)                             */
    HCLAE_T_BEAM_SCORE, /* multi-path encoding: fp32-MFMA scoring and candidate bitmaps     */
    HCLAE_T_BEAM_EXPAND,/* multi-path encoding: fp64 evaluation, top-L, next beam           */
    HCLAE_T_ACCUM_MOVED,/* centroid sums advanced by the vectors that changed cluster       */
    HCLAE_T_ASSIGN_ACTIVE, /* assignment of the vectors the distance bounds could not settle  */
    HCLAE_T_BOUNDS,     /* ageing of the distance bounds and listing of those vectors       */
    HCLAE_T_COUNT
};

typedef struct {
    double  ms[HCLAE_T_COUNT];        /* summed event time per kernel class, milliseconds   */
    int64_t launches[HCLAE_T_COUNT];  /* launches those sums cover                          */
} hclae_kernel_times;

/* Bracket every later launch whose class bit (1 << HCLAE_T_*) is set in class_mask with a
 * pair of events; 0 switches timing off (recorded launches are kept until read).  At most
 * 4096 launches are kept between reads; later ones go untimed. */
int hclae_timing_enable(hclae_ctx *ctx, uint32_t class_mask);
/* Synchronise the stream, sum the recorded launches per class into *out (HOST), forget them. */
int hclae_timing_read(hclae_ctx *ctx, hclae_kernel_times *out);

#ifdef __cplusplus
}
#endif
#endif /* HCLAE_H */
