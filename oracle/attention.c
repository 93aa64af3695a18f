/*
 * ORACLE -- test infrastructure only.  Plain fp64 CPU attention used to check the HIP path.
 * Nothing in the product path may link, load or call this file; it shares no code with the
 * kernels.  Only tests, the smoke check and the bench's cpu_baseline leg use it.
 *
 * What it computes (paper section 2.1: causal mask; section 2.2: packed sequences keep a
 * per-sequence causal mask; section 4.2: a dependent chunk attends to the key/value state of
 * the earlier chunks of its sequence, and the key/value gradients of those earlier chunks
 * receive contributions from the later chunks; section 4: accumulating the per-chunk
 * gradients gives the same result as ordinary, unsplit training).
 *
 * Two independent formulations live here so that each can be tested against the other:
 *
 *   orc_seq_*    the DEFINITION: ordinary causal softmax attention of one whole sequence,
 *                written straight from the formulas
 *                    S_ij = s <q_i, k_j>  (j <= i),  LSE_i = log sum_j exp S_ij,
 *                    P_ij = exp(S_ij - LSE_i),       O_i = sum_j P_ij v_j,
 *                    delta_i = <dO_i, O_i>,          dV_j = sum_{i>=j} P_ij dO_i,
 *                    dS_ij = P_ij (<dO_i, v_j> - delta_i),
 *                    dQ_i = s sum_j dS_ij k_j,       dK_j = s sum_{i>=j} dS_ij q_i,
 *                with grouped-query heads: query head h reads key/value head h / (Hq/Hkv) and
 *                dK/dV sum over the query heads of the group.
 *
 *   orc_chunk_*  the METHOD: one call per chunk.  A chunk has n_seg segments; segment g has
 *                Lq_g query rows and Lk_g >= Lq_g key rows, and query i of the segment sees key
 *                j iff j <= i + (Lk_g - Lq_g): the first Lk_g - Lq_g keys are the retained
 *                prefix state, the rest are the chunk's own keys.  The backward ADDS into
 *                dK/dV (so that the prefix rows collect the contributions of later chunks when
 *                the chunks of a sequence run in descending order) and overwrites dQ.
 *
 * All tensors are fp64, token-major: X[token][head][d], contiguous.  LSE is [head][token].
 * No blocking, no online softmax, no fusion: every row is computed by the formulas above with
 * a max-subtracted exponential for range safety.  OpenMP only spreads independent rows over
 * the host cores.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double dot(const double *a, const double *b, int64_t D)
{
    double s = 0.0;
    for (int64_t d = 0; d < D; ++d) s += a[d] * b[d];
    return s;
}

/* ------------------------------------------------------------------------------------------
 * Definition: one whole sequence of L tokens.
 * q,o,d_o,dq : [L][Hq][D]   k,v,dk,dv : [L][Hkv][D]   lse : [Hq][L]
 * ---------------------------------------------------------------------------------------- */
void orc_seq_attn_fwd(int64_t L, int64_t Hq, int64_t Hkv, int64_t D, double scale,
                      const double *q, const double *k, const double *v,
                      double *o, double *lse)
{
    const int64_t G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int64_t h = 0; h < Hq; ++h) {
        for (int64_t i = 0; i < L; ++i) {
            const int64_t kh = h / G;
            const double *qi = q + (i * Hq + h) * D;
            double *s = (double *)malloc((size_t)(i + 1) * sizeof(double));
            double m = -INFINITY;
            for (int64_t j = 0; j <= i; ++j) {
                s[j] = scale * dot(qi, k + (j * Hkv + kh) * D, D);
                if (s[j] > m) m = s[j];
            }
            double z = 0.0;
            for (int64_t j = 0; j <= i; ++j) z += exp(s[j] - m);
            const double l = m + log(z);
            lse[h * L + i] = l;
            double *oi = o + (i * Hq + h) * D;
            for (int64_t d = 0; d < D; ++d) oi[d] = 0.0;
            for (int64_t j = 0; j <= i; ++j) {
                const double p = exp(s[j] - l);
                const double *vj = v + (j * Hkv + kh) * D;
                for (int64_t d = 0; d < D; ++d) oi[d] += p * vj[d];
            }
            free(s);
        }
    }
}

/* dq is overwritten; dk and dv are overwritten too (a whole sequence has no earlier state). */
void orc_seq_attn_bwd(int64_t L, int64_t Hq, int64_t Hkv, int64_t D, double scale,
                      const double *q, const double *k, const double *v,
                      const double *o, const double *lse, const double *d_o,
                      double *dq, double *dk, double *dv)
{
    const int64_t G = Hq / Hkv;
    double *delta = (double *)malloc((size_t)(Hq * L) * sizeof(double));
#pragma omp parallel for collapse(2)
    for (int64_t h = 0; h < Hq; ++h)
        for (int64_t i = 0; i < L; ++i)
            delta[h * L + i] = dot(d_o + (i * Hq + h) * D, o + (i * Hq + h) * D, D);

    /* dQ_i = s sum_{j<=i} dS_ij k_j */
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int64_t h = 0; h < Hq; ++h) {
        for (int64_t i = 0; i < L; ++i) {
            const int64_t kh = h / G;
            const double *qi = q + (i * Hq + h) * D;
            const double *doi = d_o + (i * Hq + h) * D;
            double *dqi = dq + (i * Hq + h) * D;
            for (int64_t d = 0; d < D; ++d) dqi[d] = 0.0;
            for (int64_t j = 0; j <= i; ++j) {
                const double *kj = k + (j * Hkv + kh) * D;
                const double *vj = v + (j * Hkv + kh) * D;
                const double p = exp(scale * dot(qi, kj, D) - lse[h * L + i]);
                const double ds = p * (dot(doi, vj, D) - delta[h * L + i]);
                for (int64_t d = 0; d < D; ++d) dqi[d] += scale * ds * kj[d];
            }
        }
    }
    /* dV_j = sum_{h in group} sum_{i>=j} P_ij dO_i ;  dK_j = s sum sum dS_ij q_i */
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int64_t kh = 0; kh < Hkv; ++kh) {
        for (int64_t j = 0; j < L; ++j) {
            const double *kj = k + (j * Hkv + kh) * D;
            const double *vj = v + (j * Hkv + kh) * D;
            double *dkj = dk + (j * Hkv + kh) * D;
            double *dvj = dv + (j * Hkv + kh) * D;
            for (int64_t d = 0; d < D; ++d) { dkj[d] = 0.0; dvj[d] = 0.0; }
            for (int64_t h = kh * G; h < (kh + 1) * G; ++h) {
                for (int64_t i = j; i < L; ++i) {
                    const double *qi = q + (i * Hq + h) * D;
                    const double *doi = d_o + (i * Hq + h) * D;
                    const double p = exp(scale * dot(qi, kj, D) - lse[h * L + i]);
                    const double ds = p * (dot(doi, vj, D) - delta[h * L + i]);
                    for (int64_t d = 0; d < D; ++d) {
                        dvj[d] += p * doi[d];
                        dkj[d] += scale * ds * qi[d];
                    }
                }
            }
        }
    }
    free(delta);
}

/* ------------------------------------------------------------------------------------------
 * Method: one chunk.
 * cu_q[n_seg+1], cu_k[n_seg+1]: exclusive prefix sums of the segments' query / key row counts.
 * q,o,d_o,dq : [Tq][Hq][D] with Tq = cu_q[n_seg];  k,v,dk,dv : [Tk][Hkv][D] with Tk = cu_k[n_seg]
 * lse : [Hq][Tq].   Returns 0, or -1 if a segment has more query rows than key rows.
 * ---------------------------------------------------------------------------------------- */
static int segments_ok(int64_t n_seg, const int64_t *cu_q, const int64_t *cu_k)
{
    for (int64_t g = 0; g < n_seg; ++g) {
        const int64_t lq = cu_q[g + 1] - cu_q[g], lk = cu_k[g + 1] - cu_k[g];
        if (lq < 0 || lk < lq) return 0;
    }
    return 1;
}

int orc_chunk_attn_fwd(int64_t n_seg, const int64_t *cu_q, const int64_t *cu_k,
                       int64_t Hq, int64_t Hkv, int64_t D, double scale,
                       const double *q, const double *k, const double *v,
                       double *o, double *lse)
{
    if (!segments_ok(n_seg, cu_q, cu_k)) return -1;
    const int64_t G = Hq / Hkv, Tq = cu_q[n_seg];
    for (int64_t g = 0; g < n_seg; ++g) {
        const int64_t q0 = cu_q[g], lq = cu_q[g + 1] - q0;
        const int64_t k0 = cu_k[g], lk = cu_k[g + 1] - k0;
        const int64_t prefix = lk - lq;          /* keys every query row of the segment sees */
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
        for (int64_t h = 0; h < Hq; ++h) {
            for (int64_t i = 0; i < lq; ++i) {
                const int64_t kh = h / G, n_vis = prefix + i + 1;
                const double *qi = q + ((q0 + i) * Hq + h) * D;
                double *s = (double *)malloc((size_t)n_vis * sizeof(double));
                double m = -INFINITY;
                for (int64_t j = 0; j < n_vis; ++j) {
                    s[j] = scale * dot(qi, k + ((k0 + j) * Hkv + kh) * D, D);
                    if (s[j] > m) m = s[j];
                }
                double z = 0.0;
                for (int64_t j = 0; j < n_vis; ++j) z += exp(s[j] - m);
                const double l = m + log(z);
                lse[h * Tq + q0 + i] = l;
                double *oi = o + ((q0 + i) * Hq + h) * D;
                for (int64_t d = 0; d < D; ++d) oi[d] = 0.0;
                for (int64_t j = 0; j < n_vis; ++j) {
                    const double p = exp(s[j] - l);
                    const double *vj = v + ((k0 + j) * Hkv + kh) * D;
                    for (int64_t d = 0; d < D; ++d) oi[d] += p * vj[d];
                }
                free(s);
            }
        }
    }
    return 0;
}

/* dq overwritten; dk, dv ACCUMULATED (+=) -- the caller zeroes them once per sequence. */
int orc_chunk_attn_bwd(int64_t n_seg, const int64_t *cu_q, const int64_t *cu_k,
                       int64_t Hq, int64_t Hkv, int64_t D, double scale,
                       const double *q, const double *k, const double *v,
                       const double *o, const double *lse, const double *d_o,
                       double *dq, double *dk, double *dv)
{
    if (!segments_ok(n_seg, cu_q, cu_k)) return -1;
    const int64_t G = Hq / Hkv, Tq = cu_q[n_seg];
    double *delta = (double *)malloc((size_t)(Hq * Tq + 1) * sizeof(double));
#pragma omp parallel for collapse(2)
    for (int64_t h = 0; h < Hq; ++h)
        for (int64_t t = 0; t < Tq; ++t)
            delta[h * Tq + t] = dot(d_o + (t * Hq + h) * D, o + (t * Hq + h) * D, D);

    for (int64_t g = 0; g < n_seg; ++g) {
        const int64_t q0 = cu_q[g], lq = cu_q[g + 1] - q0;
        const int64_t k0 = cu_k[g], lk = cu_k[g + 1] - k0;
        const int64_t prefix = lk - lq;
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
        for (int64_t h = 0; h < Hq; ++h) {
            for (int64_t i = 0; i < lq; ++i) {
                const int64_t kh = h / G, n_vis = prefix + i + 1;
                const double *qi = q + ((q0 + i) * Hq + h) * D;
                const double *doi = d_o + ((q0 + i) * Hq + h) * D;
                const double li = lse[h * Tq + q0 + i], di = delta[h * Tq + q0 + i];
                double *dqi = dq + ((q0 + i) * Hq + h) * D;
                for (int64_t d = 0; d < D; ++d) dqi[d] = 0.0;
                for (int64_t j = 0; j < n_vis; ++j) {
                    const double *kj = k + ((k0 + j) * Hkv + kh) * D;
                    const double *vj = v + ((k0 + j) * Hkv + kh) * D;
                    const double p = exp(scale * dot(qi, kj, D) - li);
                    const double ds = p * (dot(doi, vj, D) - di);
                    for (int64_t d = 0; d < D; ++d) dqi[d] += scale * ds * kj[d];
                }
            }
        }
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
        for (int64_t kh = 0; kh < Hkv; ++kh) {
            for (int64_t j = 0; j < lk; ++j) {
                const double *kj = k + ((k0 + j) * Hkv + kh) * D;
                const double *vj = v + ((k0 + j) * Hkv + kh) * D;
                double *dkj = dk + ((k0 + j) * Hkv + kh) * D;
                double *dvj = dv + ((k0 + j) * Hkv + kh) * D;
                /* first query row that sees key j:  j <= i + prefix  <=>  i >= j - prefix */
                const int64_t i_first = j > prefix ? j - prefix : 0;
                for (int64_t h = kh * G; h < (kh + 1) * G; ++h) {
                    for (int64_t i = i_first; i < lq; ++i) {
                        const double *qi = q + ((q0 + i) * Hq + h) * D;
                        const double *doi = d_o + ((q0 + i) * Hq + h) * D;
                        const double p = exp(scale * dot(qi, kj, D) - lse[h * Tq + q0 + i]);
                        const double ds = p * (dot(doi, vj, D) - delta[h * Tq + q0 + i]);
                        for (int64_t d = 0; d < D; ++d) {
                            dvj[d] += p * doi[d];
                            dkj[d] += scale * ds * qi[d];
                        }
                    }
                }
            }
        }
    }
    free(delta);
    return 0;
}
