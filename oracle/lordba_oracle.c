/*
 * LoRDBA adapter branch (forward, and the backward pass of training): CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition that
 * the GPU library is checked against.  Nothing in the product path may call it;
 * it shares no code, header, table or helper with the HIP library, and it has
 * its own fp16 decoder and its own bit packer.
 *
 * What it computes (paper notation; the C ABI's name in brackets):
 *   host projection N x M  [d_in x d_out], carrier rank R [r], T token rows,
 *   B1 in {+-1}^{N x R}  [sign(A) = B1^T, stored as S_A[r, d_in]],
 *   B2 in {+-1}^{R x M}  [sign(B) = B2^T, stored as S_B[d_out, r]],
 *   alpha in R^N [s_in], beta in R^R [s_rank], gamma in R^M [s_out].
 *   Def. 1 / Eq. (lordba), canonical l = 1 envelope:
 *       DeltaW = diag(alpha) B1 diag(beta) B2 diag(gamma)
 *   Eq. (adapter-mode-fwd): Y = Y_base + X DeltaW
 *   evaluated in the order of Eq. (lordba-fwd):
 *       ((((X D_alpha) B1) D_beta) B2) D_gamma
 *
 * Every fp16 input is taken at its exact real value; all arithmetic is IEEE
 * binary64, plain left-to-right loops, no blocking, no fusion, no reordering.
 *
 * Parity pins (tests/test_oracle_*.py, none of them calls back into this file
 * for the expected value): exact rational brute force of the dense DeltaW on
 * tiny shapes, numpy fp64 GEMM special case, closed forms (all-ones, rank-1,
 * unit-vector rows), invariants (zero scales, sign gauge, linearity), the
 * plus-set/minus-set form of Eq. (sign-accum), the 65536-entry fp16 table
 * against numpy, and hand-written packed words.  The multi-envelope forward
 * (Eq. (lordba) with l >= 1) is pinned by the dense DeltaW built term by term
 * in exact rationals and in numpy, by its reduction to the one-envelope
 * function, by the zero-beta envelope that must change nothing (Sec. 3.2,
 * initialisation of additional envelopes), and by additivity over envelopes.
 * The batched forward (one adapter of a pool per token row) is pinned by running
 * the pinned one-adapter function on every group of rows separately, by the
 * pass-through rows, and by its invariance under any permutation of the rows.
 * The backward pass (Sec. 3.2; Eq. (smoothsign); Alg. QAT-LoRDBA) is pinned by
 * torch autograd in fp64 over Eq. (lordba-fwd) with a sign function whose
 * derivative is the smooth-sign factor, by exact unit-step differences of the
 * loss on a dense numpy DeltaW, by the contraction of X^T G in exact rationals,
 * by the adjoint identity with the pinned forward, by Euler's relation for the
 * three scale vectors, and by closed forms of the smooth-sign factor; with
 * several envelopes, by the sum of the pinned one-envelope results over the
 * envelopes (DeltaW is their sum) and again by autograd.  The
 * rank-r intermediate t is pinned by a numpy fp64 GEMM and by the forward
 * oracle with an identity-like second carrier.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- fp16 ---- */

/* IEEE 754 binary16 bit pattern -> exact binary64 value.
 * 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits. */
double lordba_oracle_f16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24);              /* zero and subnormals: f * 2^-24 */
    } else if (e == 31) {
        v = (f == 0) ? INFINITY : NAN;
    } else {
        v = ldexp((double)(1024 + f), e - 25);  /* (1 + f/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

void lordba_oracle_f16_array_to_f64(const uint16_t *h, double *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = lordba_oracle_f16_to_f64(h[i]);
}

/* ------------------------------------------------------------- packing ---- */

/* Canonical packed carrier format (the paper only says "bit-packed", Sec. 3.3;
 * storage R(N+M) bits, Eq. (lordba-bits)).  Reading taken here: a [rows, cols]
 * sign matrix is the row-major bit stream n = row*cols + col; bit n lives in bit
 * (n mod 32) of 32-bit word (n div 32); bit = 1 means -1, bit = 0 means +1 (the
 * IEEE sign-bit convention); pad bits of the last word are 0.
 * Returns 0, or 3 if an entry is not +-1. */
int lordba_oracle_pack(const int8_t *signs, int64_t rows, int64_t cols, uint32_t *words)
{
    int64_t nbits = rows * cols;
    int64_t nwords = (nbits + 31) / 32;
    for (int64_t w = 0; w < nwords; ++w) words[w] = 0u;
    for (int64_t row = 0; row < rows; ++row) {
        for (int64_t col = 0; col < cols; ++col) {
            int8_t s = signs[row * cols + col];
            if (s != 1 && s != -1) return 3;
            int64_t n = row * cols + col;
            if (s == -1) words[n / 32] |= (uint32_t)1 << (n % 32);
        }
    }
    return 0;
}

void lordba_oracle_unpack(const uint32_t *words, int64_t rows, int64_t cols, int8_t *signs)
{
    for (int64_t row = 0; row < rows; ++row) {
        for (int64_t col = 0; col < cols; ++col) {
            int64_t n = row * cols + col;
            int bit = (int)((words[n / 32] >> (n % 32)) & 1u);
            signs[n] = bit ? -1 : 1;
        }
    }
}

/* Binarisation of a real latent carrier: sign(u) with sign(0) = +1 (Sec. 2,
 * Notation).  Compared by value, so -0.0 also maps to +1.  Returns 3 on NaN. */
int lordba_oracle_sign_f64(const double *u, int64_t n, int8_t *signs)
{
    for (int64_t i = 0; i < n; ++i) {
        if (u[i] != u[i]) return 3;
        signs[i] = (u[i] >= 0.0) ? 1 : -1;
    }
    return 0;
}

/* ------------------------------------------------------------- forward ---- */

/* One token row, staged exactly as Eq. (lordba-fwd):
 *   w = x D_alpha;  t = w B1;  u = t D_beta;  v = u B2;  delta = v D_gamma;
 *   y = y_base + delta                                  (Eq. adapter-mode-fwd)
 * sA is S_A[r, d_in] = B1^T, sB is S_B[d_out, r] = B2^T, both int8 +-1. */
static void forward_row(const uint16_t *x_row, const int8_t *sA, const int8_t *sB,
                        const double *alpha, const double *beta, const double *gamma,
                        const uint16_t *ybase_row, double *y_row,
                        int64_t d_in, int64_t d_out, int64_t r,
                        double *w, double *u)
{
    for (int64_t i = 0; i < d_in; ++i)
        w[i] = lordba_oracle_f16_to_f64(x_row[i]) * alpha[i];
    for (int64_t k = 0; k < r; ++k) {
        double t = 0.0;
        for (int64_t i = 0; i < d_in; ++i)
            t += w[i] * (double)sA[k * d_in + i];          /* (w B1)_k, B1[i,k] = S_A[k,i] */
        u[k] = t * beta[k];
    }
    for (int64_t j = 0; j < d_out; ++j) {
        double v = 0.0;
        for (int64_t k = 0; k < r; ++k)
            v += u[k] * (double)sB[j * r + k];             /* (u B2)_j, B2[k,j] = S_B[j,k] */
        y_row[j] = lordba_oracle_f16_to_f64(ybase_row[j]) + v * gamma[j];
    }
}

typedef struct {
    const uint16_t *x; const int8_t *sA; const int8_t *sB;
    const double *alpha, *beta, *gamma;
    const uint16_t *y_base; double *y;
    int64_t t0, t1, d_in, d_out, r;
    int status;
} row_job;

static void *row_worker(void *arg)
{
    row_job *jb = (row_job *)arg;
    double *w = (double *)malloc(sizeof(double) * (size_t)(jb->d_in > 0 ? jb->d_in : 1));
    double *u = (double *)malloc(sizeof(double) * (size_t)(jb->r > 0 ? jb->r : 1));
    if (!w || !u) { jb->status = 9; free(w); free(u); return NULL; }
    for (int64_t t = jb->t0; t < jb->t1; ++t)
        forward_row(jb->x + t * jb->d_in, jb->sA, jb->sB, jb->alpha, jb->beta, jb->gamma,
                    jb->y_base + t * jb->d_out, jb->y + t * jb->d_out,
                    jb->d_in, jb->d_out, jb->r, w, u);
    free(w); free(u);
    jb->status = 0;
    return NULL;
}

/* x[T,d_in], y_base[T,d_out]: fp16 bit patterns, row-major.  signsA[r,d_in],
 * signsB[d_out,r]: int8 +-1.  s_in[d_in], s_rank[r], s_out[d_out]: fp16 bit
 * patterns.  y[T,d_out]: fp64 out.  Token rows are independent, so nthreads > 1
 * only splits the row range; each row is computed by the same plain loops.
 * Returns 0, 2 on a bad dimension, 3 on a sign that is not +-1, 9 on malloc failure. */
int lordba_oracle_forward(const uint16_t *x, const int8_t *signsA, const int8_t *signsB,
                          const uint16_t *s_in, const uint16_t *s_rank, const uint16_t *s_out,
                          const uint16_t *y_base, double *y,
                          int64_t T, int64_t d_in, int64_t d_out, int64_t r, int nthreads)
{
    if (T < 0 || d_in < 1 || d_out < 1 || r < 1) return 2;
    for (int64_t n = 0; n < r * d_in; ++n) if (signsA[n] != 1 && signsA[n] != -1) return 3;
    for (int64_t n = 0; n < d_out * r; ++n) if (signsB[n] != 1 && signsB[n] != -1) return 3;
    if (T == 0) return 0;

    double *alpha = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *beta = (double *)malloc(sizeof(double) * (size_t)r);
    double *gamma = (double *)malloc(sizeof(double) * (size_t)d_out);
    if (!alpha || !beta || !gamma) { free(alpha); free(beta); free(gamma); return 9; }
    lordba_oracle_f16_array_to_f64(s_in, alpha, d_in);
    lordba_oracle_f16_array_to_f64(s_rank, beta, r);
    lordba_oracle_f16_array_to_f64(s_out, gamma, d_out);

    if (nthreads < 1) nthreads = 1;
    if ((int64_t)nthreads > T) nthreads = (int)T;
    row_job *jobs = (row_job *)calloc((size_t)nthreads, sizeof(row_job));
    pthread_t *tids = (pthread_t *)calloc((size_t)nthreads, sizeof(pthread_t));
    int status = 0;
    if (!jobs || !tids) { status = 9; goto done; }
    for (int i = 0; i < nthreads; ++i) {
        row_job *jb = &jobs[i];
        jb->x = x; jb->sA = signsA; jb->sB = signsB;
        jb->alpha = alpha; jb->beta = beta; jb->gamma = gamma;
        jb->y_base = y_base; jb->y = y;
        jb->t0 = T * i / nthreads; jb->t1 = T * (i + 1) / nthreads;
        jb->d_in = d_in; jb->d_out = d_out; jb->r = r; jb->status = 0;
    }
    if (nthreads == 1) {
        row_worker(&jobs[0]);
    } else {
        for (int i = 0; i < nthreads; ++i)
            if (pthread_create(&tids[i], NULL, row_worker, &jobs[i]) != 0) { jobs[i].status = 9; tids[i] = 0; row_worker(&jobs[i]); }
        for (int i = 0; i < nthreads; ++i)
            if (tids[i]) pthread_join(tids[i], NULL);
    }
    for (int i = 0; i < nthreads; ++i) if (jobs[i].status) status = jobs[i].status;
done:
    free(jobs); free(tids); free(alpha); free(beta); free(gamma);
    return status;
}

/* Same map, but the carriers arrive in the canonical packed format and are
 * unpacked with this file's own unpacker first. */
int lordba_oracle_forward_packed(const uint16_t *x, const uint32_t *packedA, const uint32_t *packedB,
                                 const uint16_t *s_in, const uint16_t *s_rank, const uint16_t *s_out,
                                 const uint16_t *y_base, double *y,
                                 int64_t T, int64_t d_in, int64_t d_out, int64_t r, int nthreads)
{
    if (T < 0 || d_in < 1 || d_out < 1 || r < 1) return 2;
    int8_t *sA = (int8_t *)malloc((size_t)(r * d_in));
    int8_t *sB = (int8_t *)malloc((size_t)(d_out * r));
    if (!sA || !sB) { free(sA); free(sB); return 9; }
    lordba_oracle_unpack(packedA, r, d_in, sA);
    lordba_oracle_unpack(packedB, d_out, r, sB);
    int st = lordba_oracle_forward(x, sA, sB, s_in, s_rank, s_out, y_base, y, T, d_in, d_out, r, nthreads);
    free(sA); free(sB);
    return st;
}

/* ------------------------------------------------- multi-envelope forward ---- */

/* Def. 1 / Eq. (lordba) with envelope rank l >= 1: the carriers B1, B2 are shared and
 *   DeltaW = sum_{e=1..l} diag(alpha_e) B1 diag(beta_e) B2 diag(gamma_e),
 *   Y = Y_base + X DeltaW                                 (Eq. adapter-mode-fwd).
 * One token row: each envelope is staged as in Eq. (lordba-fwd) and added to the
 * row in envelope order, y = ((y_base + delta_1) + delta_2) + ...
 * alpha is [l, d_in], beta [l, r], gamma [l, d_out], row-major. */
static void forward_row_multi(const uint16_t *x_row, const int8_t *sA, const int8_t *sB,
                              const double *alpha, const double *beta, const double *gamma,
                              const uint16_t *ybase_row, double *y_row,
                              int64_t d_in, int64_t d_out, int64_t r, int64_t ell,
                              double *w, double *u)
{
    for (int64_t j = 0; j < d_out; ++j)
        y_row[j] = lordba_oracle_f16_to_f64(ybase_row[j]);
    for (int64_t e = 0; e < ell; ++e) {
        const double *al = alpha + e * d_in, *be = beta + e * r, *ga = gamma + e * d_out;
        for (int64_t i = 0; i < d_in; ++i)
            w[i] = lordba_oracle_f16_to_f64(x_row[i]) * al[i];
        for (int64_t k = 0; k < r; ++k) {
            double t = 0.0;
            for (int64_t i = 0; i < d_in; ++i)
                t += w[i] * (double)sA[k * d_in + i];
            u[k] = t * be[k];
        }
        for (int64_t j = 0; j < d_out; ++j) {
            double v = 0.0;
            for (int64_t k = 0; k < r; ++k)
                v += u[k] * (double)sB[j * r + k];
            y_row[j] += v * ga[j];
        }
    }
}

typedef struct {
    row_job base;
    int64_t ell;
} row_job_multi;

static void *row_worker_multi(void *arg)
{
    row_job_multi *jm = (row_job_multi *)arg;
    row_job *jb = &jm->base;
    double *w = (double *)malloc(sizeof(double) * (size_t)(jb->d_in > 0 ? jb->d_in : 1));
    double *u = (double *)malloc(sizeof(double) * (size_t)(jb->r > 0 ? jb->r : 1));
    if (!w || !u) { jb->status = 9; free(w); free(u); return NULL; }
    for (int64_t t = jb->t0; t < jb->t1; ++t)
        forward_row_multi(jb->x + t * jb->d_in, jb->sA, jb->sB, jb->alpha, jb->beta, jb->gamma,
                          jb->y_base + t * jb->d_out, jb->y + t * jb->d_out,
                          jb->d_in, jb->d_out, jb->r, jm->ell, w, u);
    free(w); free(u);
    jb->status = 0;
    return NULL;
}

/* As lordba_oracle_forward, with s_in[ell, d_in], s_rank[ell, r], s_out[ell, d_out] (fp16 bit
 * patterns, row-major) and ell >= 1 envelopes over the same carriers. */
int lordba_oracle_forward_multi(const uint16_t *x, const int8_t *signsA, const int8_t *signsB,
                                const uint16_t *s_in, const uint16_t *s_rank, const uint16_t *s_out,
                                const uint16_t *y_base, double *y,
                                int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, int nthreads)
{
    if (T < 0 || d_in < 1 || d_out < 1 || r < 1 || ell < 1) return 2;
    for (int64_t n = 0; n < r * d_in; ++n) if (signsA[n] != 1 && signsA[n] != -1) return 3;
    for (int64_t n = 0; n < d_out * r; ++n) if (signsB[n] != 1 && signsB[n] != -1) return 3;
    if (T == 0) return 0;

    double *alpha = (double *)malloc(sizeof(double) * (size_t)(ell * d_in));
    double *beta = (double *)malloc(sizeof(double) * (size_t)(ell * r));
    double *gamma = (double *)malloc(sizeof(double) * (size_t)(ell * d_out));
    if (!alpha || !beta || !gamma) { free(alpha); free(beta); free(gamma); return 9; }
    lordba_oracle_f16_array_to_f64(s_in, alpha, ell * d_in);
    lordba_oracle_f16_array_to_f64(s_rank, beta, ell * r);
    lordba_oracle_f16_array_to_f64(s_out, gamma, ell * d_out);

    if (nthreads < 1) nthreads = 1;
    if ((int64_t)nthreads > T) nthreads = (int)T;
    row_job_multi *jobs = (row_job_multi *)calloc((size_t)nthreads, sizeof(row_job_multi));
    pthread_t *tids = (pthread_t *)calloc((size_t)nthreads, sizeof(pthread_t));
    int status = 0;
    if (!jobs || !tids) { status = 9; goto done; }
    for (int i = 0; i < nthreads; ++i) {
        row_job *jb = &jobs[i].base;
        jb->x = x; jb->sA = signsA; jb->sB = signsB;
        jb->alpha = alpha; jb->beta = beta; jb->gamma = gamma;
        jb->y_base = y_base; jb->y = y;
        jb->t0 = T * i / nthreads; jb->t1 = T * (i + 1) / nthreads;
        jb->d_in = d_in; jb->d_out = d_out; jb->r = r; jb->status = 0;
        jobs[i].ell = ell;
    }
    if (nthreads == 1) {
        row_worker_multi(&jobs[0]);
    } else {
        for (int i = 0; i < nthreads; ++i)
            if (pthread_create(&tids[i], NULL, row_worker_multi, &jobs[i]) != 0) { tids[i] = 0; row_worker_multi(&jobs[i]); }
        for (int i = 0; i < nthreads; ++i)
            if (tids[i]) pthread_join(tids[i], NULL);
    }
    for (int i = 0; i < nthreads; ++i) if (jobs[i].base.status) status = jobs[i].base.status;
done:
    free(jobs); free(tids); free(alpha); free(beta); free(gamma);
    return status;
}

/* ------------------------------------------------ multi-adapter batch ---- */

/* Several adapters of the same shape served in one batch (Sec. 3.3, hot-swappable adapters served concurrently):
 * token row t uses adapter id[t] of a pool,
 *   y[t] = y_base[t] + x[t] DeltaW(theta_{id[t]})            (Eq. adapter-mode-fwd, row by row)
 * and a row whose id is not in [0, n_adapters) has no adapter: y[t] = y_base[t].
 * Pools are contiguous arrays over the adapter index: signsA[n, r, d_in], signsB[n, d_out, r], s_in[n, d_in],
 * s_rank[n, r], s_out[n, d_out].  Plain loop over rows; each row is the one-adapter row function. */
int lordba_oracle_forward_batched(const uint16_t *x, const int8_t *signsA, const int8_t *signsB,
                                  const uint16_t *s_in, const uint16_t *s_rank, const uint16_t *s_out,
                                  const int32_t *id, const uint16_t *y_base, double *y,
                                  int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t n_adapters)
{
    if (T < 0 || d_in < 1 || d_out < 1 || r < 1 || n_adapters < 0) return 2;
    for (int64_t n = 0; n < n_adapters * r * d_in; ++n) if (signsA[n] != 1 && signsA[n] != -1) return 3;
    for (int64_t n = 0; n < n_adapters * d_out * r; ++n) if (signsB[n] != 1 && signsB[n] != -1) return 3;
    double *alpha = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *beta = (double *)malloc(sizeof(double) * (size_t)r);
    double *gamma = (double *)malloc(sizeof(double) * (size_t)d_out);
    double *w = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *u = (double *)malloc(sizeof(double) * (size_t)r);
    int status = 0;
    if (!alpha || !beta || !gamma || !w || !u) { status = 9; goto done; }
    for (int64_t t = 0; t < T; ++t) {
        const int64_t a = id[t];
        if (a < 0 || a >= n_adapters) {
            for (int64_t j = 0; j < d_out; ++j) y[t * d_out + j] = lordba_oracle_f16_to_f64(y_base[t * d_out + j]);
            continue;
        }
        lordba_oracle_f16_array_to_f64(s_in + a * d_in, alpha, d_in);
        lordba_oracle_f16_array_to_f64(s_rank + a * r, beta, r);
        lordba_oracle_f16_array_to_f64(s_out + a * d_out, gamma, d_out);
        forward_row(x + t * d_in, signsA + a * r * d_in, signsB + a * d_out * r, alpha, beta, gamma,
                    y_base + t * d_out, y + t * d_out, d_in, d_out, r, w, u);
    }
done:
    free(alpha); free(beta); free(gamma); free(w); free(u);
    return status;
}

/* The same batch when every adapter of the pool has `ell` scale envelopes over its own carriers (Def. 1 / Eq. (lordba)
 * with envelope rank l = ell for each adapter; Sec. 3.3):
 *   y[t] = y_base[t] + x[t] sum_e diag(alpha_{a,e}) B1_a diag(beta_{a,e}) B2_a diag(gamma_{a,e}),   a = id[t],
 * pools s_in[n, ell, d_in], s_rank[n, ell, r], s_out[n, ell, d_out].  Plain loop over rows; each row is the
 * multi-envelope row function with its adapter's carriers and envelopes. */
int lordba_oracle_forward_batched_multi(const uint16_t *x, const int8_t *signsA, const int8_t *signsB,
                                        const uint16_t *s_in, const uint16_t *s_rank, const uint16_t *s_out,
                                        const int32_t *id, const uint16_t *y_base, double *y,
                                        int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, int64_t n_adapters)
{
    if (T < 0 || d_in < 1 || d_out < 1 || r < 1 || ell < 1 || n_adapters < 0) return 2;
    for (int64_t n = 0; n < n_adapters * r * d_in; ++n) if (signsA[n] != 1 && signsA[n] != -1) return 3;
    for (int64_t n = 0; n < n_adapters * d_out * r; ++n) if (signsB[n] != 1 && signsB[n] != -1) return 3;
    double *alpha = (double *)malloc(sizeof(double) * (size_t)(ell * d_in));
    double *beta = (double *)malloc(sizeof(double) * (size_t)(ell * r));
    double *gamma = (double *)malloc(sizeof(double) * (size_t)(ell * d_out));
    double *w = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *u = (double *)malloc(sizeof(double) * (size_t)r);
    int status = 0;
    if (!alpha || !beta || !gamma || !w || !u) { status = 9; goto done; }
    for (int64_t t = 0; t < T; ++t) {
        const int64_t a = id[t];
        if (a < 0 || a >= n_adapters) {
            for (int64_t j = 0; j < d_out; ++j) y[t * d_out + j] = lordba_oracle_f16_to_f64(y_base[t * d_out + j]);
            continue;
        }
        lordba_oracle_f16_array_to_f64(s_in + a * ell * d_in, alpha, ell * d_in);
        lordba_oracle_f16_array_to_f64(s_rank + a * ell * r, beta, ell * r);
        lordba_oracle_f16_array_to_f64(s_out + a * ell * d_out, gamma, ell * d_out);
        forward_row_multi(x + t * d_in, signsA + a * r * d_in, signsB + a * d_out * r, alpha, beta, gamma,
                          y_base + t * d_out, y + t * d_out, d_in, d_out, r, ell, w, u);
    }
done:
    free(alpha); free(beta); free(gamma); free(w); free(u);
    return status;
}

/* ------------------------------------------------- rank-r intermediate ---- */

/* t = (X D_alpha) B1, the inner two factors of Eq. (lordba-fwd): t[row, k] = sum_i S_A[k,i] * alpha_i * x[row, i].
 * Training keeps it from the forward pass for the backward pass.  x[T,d_in], s_in[d_in]: fp16 bit patterns;
 * signsA[r,d_in]: int8 +-1; t[T,r]: fp64 out (token-major).  Returns 0, 2 or 3 as the other functions. */
int lordba_oracle_rank_intermediate(const uint16_t *x, const int8_t *signsA, const uint16_t *s_in, double *t,
                                    int64_t T, int64_t d_in, int64_t r)
{
    if (T < 0 || d_in < 1 || r < 1) return 2;
    for (int64_t n = 0; n < r * d_in; ++n) if (signsA[n] != 1 && signsA[n] != -1) return 3;
    for (int64_t row = 0; row < T; ++row) {
        for (int64_t k = 0; k < r; ++k) {
            double s = 0.0;
            for (int64_t i = 0; i < d_in; ++i)
                s += lordba_oracle_f16_to_f64(x[row * d_in + i]) * lordba_oracle_f16_to_f64(s_in[i]) * (double)signsA[k * d_in + i];
            t[row * r + k] = s;
        }
    }
    return 0;
}

/* ------------------------------------------------- backward of the branch ---- */

/* Smooth-sign straight-through factor, Eq. (smoothsign): on the backward pass the derivative of sign(u)
 * is replaced by d/du tanh(kappa u) = kappa (1 - tanh^2(kappa u)).  Written as kappa / cosh^2(kappa u),
 * the same function without the cancellation of 1 - tanh^2 at large |kappa u|. */
double lordba_oracle_smooth_sign_grad(double u, double kappa)
{
    double c = cosh(kappa * u);
    return kappa / (c * c);
}

/* Gradients of a scalar loss through the branch (training of Sec. 3.2, "Forward and backward pass";
 * Alg. QAT-LoRDBA), for given G = dL/dY:
 *   forward, Eq. (lordba-fwd):  w = x D_alpha;  t = w B1;  u = t D_beta;  v = u B2;  y = y_base + v D_gamma
 *   with B1 = sign(U1), B2 = sign(U2) (here S_A = B1^T, S_B = B2^T, and the latents in the same layouts:
 *   latA[r, d_in] = U1^T, latB[d_out, r] = U2^T).
 * Reverse mode, one token row after the other, every product written out:
 *   d_gamma_j += g_j v_j            dv_j = g_j gamma_j
 *   dB2[k,j]  += u_k dv_j           du_k = sum_j dv_j B2[k,j]
 *   d_beta_k  += du_k t_k           dt_k = du_k beta_k
 *   dB1[i,k]  += w_i dt_k           dw_i = sum_k dt_k B1[i,k]
 *   d_alpha_i += dw_i x_i           dx_i = dx_base_i + dw_i alpha_i
 * and at the end the carriers' gradients pass through the smooth-sign factor of Eq. (smoothsign):
 *   d_latA[k,i] = dB1[i,k] * kappa (1 - tanh^2(kappa latA[k,i])),   d_latB[j,k] likewise from dB2[k,j].
 * The carriers used are the given signs (the caller keeps them equal to sign(latent)); the scales are
 * the fp16 values the forward pass used, at their exact values.
 * x[T,d_in], g[T,d_out], dx_base[T,d_in] (may be NULL = 0): fp16 bit patterns.  latA, latB: binary32.
 * Outputs (fp64): dx[T,d_in], d_s_in[d_in], d_s_rank[r], d_s_out[d_out], d_latA[r,d_in], d_latB[d_out,r].
 * Returns 0, 2 on a bad dimension, 3 on a sign that is not +-1, 9 on malloc failure. */
int lordba_oracle_backward(const uint16_t *x, const uint16_t *g, const int8_t *signsA, const int8_t *signsB,
                           const uint16_t *s_in, const uint16_t *s_rank, const uint16_t *s_out,
                           const float *latA, const float *latB, double kappa,
                           const uint16_t *dx_base, double *dx,
                           double *d_s_in, double *d_s_rank, double *d_s_out, double *d_latA, double *d_latB,
                           int64_t T, int64_t d_in, int64_t d_out, int64_t r)
{
    if (T < 0 || d_in < 1 || d_out < 1 || r < 1) return 2;
    for (int64_t n = 0; n < r * d_in; ++n) if (signsA[n] != 1 && signsA[n] != -1) return 3;
    for (int64_t n = 0; n < d_out * r; ++n) if (signsB[n] != 1 && signsB[n] != -1) return 3;

    double *alpha = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *beta = (double *)malloc(sizeof(double) * (size_t)r);
    double *gamma = (double *)malloc(sizeof(double) * (size_t)d_out);
    double *w = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *dw = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *v = (double *)malloc(sizeof(double) * (size_t)d_out);
    double *dv = (double *)malloc(sizeof(double) * (size_t)d_out);
    double *t = (double *)malloc(sizeof(double) * (size_t)r);
    double *u = (double *)malloc(sizeof(double) * (size_t)r);
    double *du = (double *)malloc(sizeof(double) * (size_t)r);
    double *dt = (double *)malloc(sizeof(double) * (size_t)r);
    int status = 0;
    if (!alpha || !beta || !gamma || !w || !dw || !v || !dv || !t || !u || !du || !dt) { status = 9; goto done; }
    lordba_oracle_f16_array_to_f64(s_in, alpha, d_in);
    lordba_oracle_f16_array_to_f64(s_rank, beta, r);
    lordba_oracle_f16_array_to_f64(s_out, gamma, d_out);

    for (int64_t i = 0; i < d_in; ++i) d_s_in[i] = 0.0;
    for (int64_t k = 0; k < r; ++k) d_s_rank[k] = 0.0;
    for (int64_t j = 0; j < d_out; ++j) d_s_out[j] = 0.0;
    for (int64_t n = 0; n < r * d_in; ++n) d_latA[n] = 0.0;      /* holds dB1 (as [r, d_in]) until the end */
    for (int64_t n = 0; n < d_out * r; ++n) d_latB[n] = 0.0;     /* holds dB2 (as [d_out, r]) until the end */

    for (int64_t row = 0; row < T; ++row) {
        const uint16_t *xr = x + row * d_in, *gr = g + row * d_out;
        /* forward intermediates of this row */
        for (int64_t i = 0; i < d_in; ++i) w[i] = lordba_oracle_f16_to_f64(xr[i]) * alpha[i];
        for (int64_t k = 0; k < r; ++k) {
            double s = 0.0;
            for (int64_t i = 0; i < d_in; ++i) s += w[i] * (double)signsA[k * d_in + i];
            t[k] = s;
            u[k] = s * beta[k];
        }
        for (int64_t j = 0; j < d_out; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < r; ++k) s += u[k] * (double)signsB[j * r + k];
            v[j] = s;
        }
        /* reverse */
        for (int64_t j = 0; j < d_out; ++j) {
            double gj = lordba_oracle_f16_to_f64(gr[j]);
            d_s_out[j] += gj * v[j];
            dv[j] = gj * gamma[j];
        }
        for (int64_t k = 0; k < r; ++k) {
            double s = 0.0;
            for (int64_t j = 0; j < d_out; ++j) {
                d_latB[j * r + k] += u[k] * dv[j];
                s += dv[j] * (double)signsB[j * r + k];
            }
            du[k] = s;
            d_s_rank[k] += s * t[k];
            dt[k] = s * beta[k];
        }
        for (int64_t i = 0; i < d_in; ++i) {
            double s = 0.0;
            for (int64_t k = 0; k < r; ++k) {
                d_latA[k * d_in + i] += w[i] * dt[k];
                s += dt[k] * (double)signsA[k * d_in + i];
            }
            dw[i] = s;
            d_s_in[i] += s * lordba_oracle_f16_to_f64(xr[i]);
            double base = dx_base ? lordba_oracle_f16_to_f64(dx_base[row * d_in + i]) : 0.0;
            dx[row * d_in + i] = base + s * alpha[i];
        }
    }
    for (int64_t n = 0; n < r * d_in; ++n) d_latA[n] *= lordba_oracle_smooth_sign_grad((double)latA[n], kappa);
    for (int64_t n = 0; n < d_out * r; ++n) d_latB[n] *= lordba_oracle_smooth_sign_grad((double)latB[n], kappa);
done:
    free(alpha); free(beta); free(gamma); free(w); free(dw); free(v); free(dv); free(t); free(u); free(du); free(dt);
    return status;
}

/* ------------------------------------- backward with several envelopes ---- */

/* As lordba_oracle_backward for an adapter with ell scale envelopes over the same carriers (Def. 1 / Eq. (lordba),
 * l >= 1): Y = Y_base + sum_e X diag(alpha_e) B1 diag(beta_e) B2 diag(gamma_e).  Each envelope is staged forward and
 * reversed exactly as in the one-envelope function, one token row after the other; the input gradient and the carrier
 * gradients add up over the envelopes (in envelope order), every envelope has its own scale gradients.
 * s_in[ell,d_in], s_rank[ell,r], s_out[ell,d_out]: fp16 bit patterns; d_s_in[ell,d_in], d_s_rank[ell,r],
 * d_s_out[ell,d_out]: fp64 out; everything else as lordba_oracle_backward. */
int lordba_oracle_backward_multi(const uint16_t *x, const uint16_t *g, const int8_t *signsA, const int8_t *signsB,
                                 const uint16_t *s_in, const uint16_t *s_rank, const uint16_t *s_out,
                                 const float *latA, const float *latB, double kappa,
                                 const uint16_t *dx_base, double *dx,
                                 double *d_s_in, double *d_s_rank, double *d_s_out, double *d_latA, double *d_latB,
                                 int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell)
{
    if (T < 0 || d_in < 1 || d_out < 1 || r < 1 || ell < 1) return 2;
    for (int64_t n = 0; n < r * d_in; ++n) if (signsA[n] != 1 && signsA[n] != -1) return 3;
    for (int64_t n = 0; n < d_out * r; ++n) if (signsB[n] != 1 && signsB[n] != -1) return 3;

    double *alpha = (double *)malloc(sizeof(double) * (size_t)(ell * d_in));
    double *beta = (double *)malloc(sizeof(double) * (size_t)(ell * r));
    double *gamma = (double *)malloc(sizeof(double) * (size_t)(ell * d_out));
    double *w = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *v = (double *)malloc(sizeof(double) * (size_t)d_out);
    double *dv = (double *)malloc(sizeof(double) * (size_t)d_out);
    double *t = (double *)malloc(sizeof(double) * (size_t)r);
    double *u = (double *)malloc(sizeof(double) * (size_t)r);
    double *dt = (double *)malloc(sizeof(double) * (size_t)r);
    int status = 0;
    if (!alpha || !beta || !gamma || !w || !v || !dv || !t || !u || !dt) { status = 9; goto done; }
    lordba_oracle_f16_array_to_f64(s_in, alpha, ell * d_in);
    lordba_oracle_f16_array_to_f64(s_rank, beta, ell * r);
    lordba_oracle_f16_array_to_f64(s_out, gamma, ell * d_out);

    for (int64_t n = 0; n < ell * d_in; ++n) d_s_in[n] = 0.0;
    for (int64_t n = 0; n < ell * r; ++n) d_s_rank[n] = 0.0;
    for (int64_t n = 0; n < ell * d_out; ++n) d_s_out[n] = 0.0;
    for (int64_t n = 0; n < r * d_in; ++n) d_latA[n] = 0.0;      /* dB1 (as [r, d_in]) until the end */
    for (int64_t n = 0; n < d_out * r; ++n) d_latB[n] = 0.0;     /* dB2 (as [d_out, r]) until the end */

    for (int64_t row = 0; row < T; ++row) {
        const uint16_t *xr = x + row * d_in, *gr = g + row * d_out;
        for (int64_t i = 0; i < d_in; ++i)
            dx[row * d_in + i] = dx_base ? lordba_oracle_f16_to_f64(dx_base[row * d_in + i]) : 0.0;
        for (int64_t e = 0; e < ell; ++e) {
            const double *al = alpha + e * d_in, *be = beta + e * r, *ga = gamma + e * d_out;
            /* forward intermediates of this row and envelope */
            for (int64_t i = 0; i < d_in; ++i) w[i] = lordba_oracle_f16_to_f64(xr[i]) * al[i];
            for (int64_t k = 0; k < r; ++k) {
                double s = 0.0;
                for (int64_t i = 0; i < d_in; ++i) s += w[i] * (double)signsA[k * d_in + i];
                t[k] = s;
                u[k] = s * be[k];
            }
            for (int64_t j = 0; j < d_out; ++j) {
                double s = 0.0;
                for (int64_t k = 0; k < r; ++k) s += u[k] * (double)signsB[j * r + k];
                v[j] = s;
            }
            /* reverse */
            for (int64_t j = 0; j < d_out; ++j) {
                double gj = lordba_oracle_f16_to_f64(gr[j]);
                d_s_out[e * d_out + j] += gj * v[j];
                dv[j] = gj * ga[j];
            }
            for (int64_t k = 0; k < r; ++k) {
                double s = 0.0;
                for (int64_t j = 0; j < d_out; ++j) {
                    d_latB[j * r + k] += u[k] * dv[j];
                    s += dv[j] * (double)signsB[j * r + k];
                }
                d_s_rank[e * r + k] += s * t[k];
                dt[k] = s * be[k];
            }
            for (int64_t i = 0; i < d_in; ++i) {
                double s = 0.0;
                for (int64_t k = 0; k < r; ++k) {
                    d_latA[k * d_in + i] += w[i] * dt[k];
                    s += dt[k] * (double)signsA[k * d_in + i];
                }
                d_s_in[e * d_in + i] += s * lordba_oracle_f16_to_f64(xr[i]);
                dx[row * d_in + i] += s * al[i];
            }
        }
    }
    for (int64_t n = 0; n < r * d_in; ++n) d_latA[n] *= lordba_oracle_smooth_sign_grad((double)latA[n], kappa);
    for (int64_t n = 0; n < d_out * r; ++n) d_latB[n] *= lordba_oracle_smooth_sign_grad((double)latB[n], kappa);
done:
    free(alpha); free(beta); free(gamma); free(w); free(v); free(dv); free(t); free(u); free(dt);
    return status;
}
