/*
 * CPU oracle for jagged softmax attention -- TEST INFRASTRUCTURE, not a product path.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 * It shares no code with the HIP library and is written for obviousness, not speed:
 * every (sample, head) pair materialises its full L x L score matrix in fp64.
 *
 * What is computed (paper Section 2: a jagged tensor is a values tensor holding all
 * samples back to back plus an offsets tensor marking sample boundaries; Section 2.1:
 * standard attention, i.e. two matrix products around a row softmax, applied to each
 * sample on its own with no padding; Section 2.2: forward and backward):
 *
 *   sample b owns rows offsets[b] .. offsets[b+1]-1 (length L) of q, k, v [sum_B, H, D];
 *   for every head h, with Q, K, V the L x D slices:
 *     S_ij   = (sum_d Q_id K_jd) / sqrt(D)                 non-causal, all i, j in [0, L)
 *     m_i    = max_j S_ij,  l_i = sum_j exp(S_ij - m_i),  P_ij = exp(S_ij - m_i) / l_i
 *     O_id   = sum_j P_ij V_jd                             -> out[s+i, h, d]
 *     LSE_i  = m_i + ln l_i                                -> lse[h, s+i]   (natural log, scaled scores)
 *   backward for a given dO:
 *     delta_i = sum_d dO_id O_id                           -> delta[h, s+i]
 *     dV_jd  = sum_i P_ij dO_id
 *     dP_ij  = sum_d dO_id V_jd
 *     dS_ij  = P_ij (dP_ij - delta_i)
 *     dQ_id  = (1/sqrt(D)) sum_j dS_ij K_jd
 *     dK_jd  = (1/sqrt(D)) sum_i dS_ij Q_id
 *
 * The online-softmax / tiling of flash attention (Section 2.1) is an exact reformulation
 * of the above, so the oracle is the plain definition.  Readings where the paper is silent
 * (scale 1/sqrt(D), non-causal, one offsets array for Q, K and V, LSE layout [H, sum_B],
 * zero-length samples legal and contributing nothing) are listed in the design notes.
 *
 * Inputs are float32 (bf16 workloads pass bf16 values widened exactly); all arithmetic and
 * all outputs are fp64.  Pins: tests/test_oracle_pins.py (brute-force padded dense attention
 * in numpy, PyTorch fp64 SDPA + autograd on equal-length batches, the unfused three-step
 * formulation, closed forms, invariances and central finite differences).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* index of element (row, h, d) in a [rows, H, D] tensor */
static inline size_t at(int64_t row, int h, int d, int H, int D) {
    return ((size_t)row * (size_t)H + (size_t)h) * (size_t)D + (size_t)d;
}

/* Scores and row statistics of one (sample, head): S (L*L), m (L), l (L). */
static void scores_one(const float *q, const float *k, int64_t s, int64_t L, int h, int H, int D,
                       double *S, double *m, double *l) {
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    for (int64_t i = 0; i < L; ++i) {
        for (int64_t j = 0; j < L; ++j) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += (double)q[at(s + i, h, d, H, D)] * (double)k[at(s + j, h, d, H, D)];
            S[i * L + j] = acc * inv_sqrt_d;
        }
        double mi = S[i * L];
        for (int64_t j = 1; j < L; ++j)
            if (S[i * L + j] > mi) mi = S[i * L + j];
        double li = 0.0;
        for (int64_t j = 0; j < L; ++j) li += exp(S[i * L + j] - mi);
        m[i] = mi;
        l[i] = li;
    }
}

/* Forward of one (sample, head).  `probs` (may be NULL) receives the L*L softmax matrix. */
static void forward_one(const float *q, const float *k, const float *v, int64_t s, int64_t L, int h, int H,
                        int D, int64_t sum_B, double *out, double *lse, double *probs) {
    if (L <= 0) return;
    double *S = (double *)malloc(sizeof(double) * (size_t)L * (size_t)L);
    double *m = (double *)malloc(sizeof(double) * (size_t)L);
    double *l = (double *)malloc(sizeof(double) * (size_t)L);
    scores_one(q, k, s, L, h, H, D, S, m, l);
    for (int64_t i = 0; i < L; ++i) {
        for (int64_t j = 0; j < L; ++j) S[i * L + j] = exp(S[i * L + j] - m[i]) / l[i];
        /* O_i = sum_j P_ij V_j, accumulated row by row of V (unit-stride inner loop) */
        double *o = &out[at(s + i, h, 0, H, D)];
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int64_t j = 0; j < L; ++j)
            for (int d = 0; d < D; ++d) o[d] += S[i * L + j] * (double)v[at(s + j, h, d, H, D)];
        lse[(size_t)h * (size_t)sum_B + (size_t)(s + i)] = m[i] + log(l[i]);
    }
    if (probs) memcpy(probs, S, sizeof(double) * (size_t)L * (size_t)L);
    free(S); free(m); free(l);
}

/* Backward of one (sample, head); recomputes P from the inputs in fp64. */
static void backward_one(const float *q, const float *k, const float *v, const float *dout, int64_t s, int64_t L,
                         int h, int H, int D, int64_t sum_B, double *dq, double *dk, double *dv, double *delta) {
    if (L <= 0) return;
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    double *P = (double *)malloc(sizeof(double) * (size_t)L * (size_t)L);
    double *m = (double *)malloc(sizeof(double) * (size_t)L);
    double *l = (double *)malloc(sizeof(double) * (size_t)L);
    double *dl = (double *)malloc(sizeof(double) * (size_t)L);
    scores_one(q, k, s, L, h, H, D, P, m, l);
    for (int64_t i = 0; i < L; ++i)
        for (int64_t j = 0; j < L; ++j) P[i * L + j] = exp(P[i * L + j] - m[i]) / l[i];
    /* All sums below run with the feature index d innermost (unit stride); the gradient rows of this
       (sample, head) are zeroed first and then accumulated term by term. */
    for (int64_t i = 0; i < L; ++i)
        for (int d = 0; d < D; ++d) {
            dq[at(s + i, h, d, H, D)] = 0.0;
            dk[at(s + i, h, d, H, D)] = 0.0;
            dv[at(s + i, h, d, H, D)] = 0.0;
        }
    double *o = (double *)malloc(sizeof(double) * (size_t)D);
    for (int64_t i = 0; i < L; ++i) {
        /* delta_i = dO_i . O_i with O_i = sum_j P_ij V_j */
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int64_t j = 0; j < L; ++j)
            for (int d = 0; d < D; ++d) o[d] += P[i * L + j] * (double)v[at(s + j, h, d, H, D)];
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += (double)dout[at(s + i, h, d, H, D)] * o[d];
        dl[i] = acc;
        if (delta) delta[(size_t)h * (size_t)sum_B + (size_t)(s + i)] = acc;
    }
    free(o);
    for (int64_t i = 0; i < L; ++i)
        for (int64_t j = 0; j < L; ++j) {
            const double p = P[i * L + j];
            /* dV_jd += P_ij dO_id ;  dP_ij = dO_i . V_j */
            double dp = 0.0;
            for (int d = 0; d < D; ++d) {
                dv[at(s + j, h, d, H, D)] += p * (double)dout[at(s + i, h, d, H, D)];
                dp += (double)dout[at(s + i, h, d, H, D)] * (double)v[at(s + j, h, d, H, D)];
            }
            /* dS_ij = P_ij (dP_ij - delta_i) ;  dQ_id += dS_ij K_jd ;  dK_jd += dS_ij Q_id */
            const double ds = p * (dp - dl[i]);
            for (int d = 0; d < D; ++d) {
                dq[at(s + i, h, d, H, D)] += ds * (double)k[at(s + j, h, d, H, D)];
                dk[at(s + j, h, d, H, D)] += ds * (double)q[at(s + i, h, d, H, D)];
            }
        }
    /* the 1/sqrt(D) of the scaled scores */
    for (int64_t i = 0; i < L; ++i)
        for (int d = 0; d < D; ++d) {
            dq[at(s + i, h, d, H, D)] *= inv_sqrt_d;
            dk[at(s + i, h, d, H, D)] *= inv_sqrt_d;
        }
    free(P); free(m); free(l); free(dl);
}

/*
 * Forward over a list of (sample, head) pairs: pair p is (pair_b[p], pair_h[p]).
 * pair_b == NULL means all B*H pairs.  Rows of out / lse that belong to pairs not
 * listed are left untouched.  Returns the number of threads used.
 */
int jfa_oracle_forward(const float *q, const float *k, const float *v, const int64_t *offsets, int64_t B, int H,
                       int D, const int64_t *pair_b, const int32_t *pair_h, int64_t n_pairs, double *out,
                       double *lse) {
    const int64_t sum_B = offsets[B];
    const int64_t n = pair_b ? n_pairs : B * (int64_t)H;
    int threads = 1;
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        threads = omp_get_num_threads();
#endif
#pragma omp for schedule(dynamic, 1)
        for (int64_t p = 0; p < n; ++p) {
            const int64_t b = pair_b ? pair_b[p] : p / H;
            const int h = pair_b ? pair_h[p] : (int)(p % H);
            forward_one(q, k, v, offsets[b], offsets[b + 1] - offsets[b], h, H, D, sum_B, out, lse, NULL);
        }
    }
    return threads;
}

int jfa_oracle_backward(const float *q, const float *k, const float *v, const float *dout, const int64_t *offsets,
                        int64_t B, int H, int D, const int64_t *pair_b, const int32_t *pair_h, int64_t n_pairs,
                        double *dq, double *dk, double *dv, double *delta) {
    const int64_t sum_B = offsets[B];
    const int64_t n = pair_b ? n_pairs : B * (int64_t)H;
    int threads = 1;
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        threads = omp_get_num_threads();
#endif
#pragma omp for schedule(dynamic, 1)
        for (int64_t p = 0; p < n; ++p) {
            const int64_t b = pair_b ? pair_b[p] : p / H;
            const int h = pair_b ? pair_h[p] : (int)(p % H);
            backward_one(q, k, v, dout, offsets[b], offsets[b + 1] - offsets[b], h, H, D, sum_B, dq, dk, dv, delta);
        }
    }
    return threads;
}

/* Softmax matrix of one (sample, head): probs[L*L], row-major (query, key).  Tiny cases only. */
void jfa_oracle_probs(const float *q, const float *k, const float *v, const int64_t *offsets, int64_t B, int H,
                      int D, int64_t b, int h, double *probs) {
    const int64_t sum_B = offsets[B];
    const int64_t L = offsets[b + 1] - offsets[b];
    if (L <= 0) return;
    double *out = (double *)calloc((size_t)sum_B * (size_t)H * (size_t)D, sizeof(double));
    double *lse = (double *)calloc((size_t)sum_B * (size_t)H, sizeof(double));
    forward_one(q, k, v, offsets[b], L, h, H, D, sum_B, out, lse, probs);
    free(out); free(lse);
}
