/*
 * CPU oracle for exact multi-head self-attention, forward and backward.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the HIP kernels are checked against.  It is not part of the product:
 * only the tests, the smoke check and the benchmark's CPU-baseline leg may call it, and it shares
 * no code with the GPU path.
 *
 * What it computes is the plain definition the paper describes in words (Sec. 3, "Flash
 * Attention": a weighted average of the value features whose weights come from the dot-product
 * similarities of queries and keys).  The memory-efficient block-wise method of the paper reaches
 * exactly this result (Sec. 1: the block-wise results are combined into the final output), so the
 * oracle is the definition written out, per (batch, head), one query row at a time, in fp64:
 *
 *   forward :  s_ij = scale * sum_c q_ic k_jc
 *              m_i  = max_j s_ij ,  e_ij = exp(s_ij - m_i) ,  l_i = sum_j e_ij
 *              P_ij = e_ij / l_i                    (the "weights")
 *              O_ic = sum_j P_ij v_jc               (the "weighted average")
 *              LSE_i = m_i + ln l_i
 *   backward, for a given upstream gradient dO (any loss):
 *              dV_jc = sum_i P_ij dO_ic
 *              dP_ij = sum_c dO_ic v_jc
 *              dS_ij = P_ij * (dP_ij - sum_k P_ik dP_ik)      (Jacobian of a row softmax)
 *              dQ_ic = scale * sum_j dS_ij k_jc
 *              dK_jc = scale * sum_i dS_ij q_ic
 *
 * Causal variant (the *_causal entry points): the paper's text encoder is "GPT-like" (implementation
 * details of the video-language model), i.e. token i attends to tokens 0..i only.  The definition is
 * the same with every sum over keys j restricted to j <= i (weights of later keys are exactly 0),
 * and the dK, dV sums over queries accordingly receive nothing from queries i < j.
 *
 * The paper never writes these formulas; they are the textbook definition of scaled dot-product
 * attention and its analytic gradient.  The inner sum of dS is evaluated as written (not through
 * the rowsum(dO*O) shortcut a fused kernel uses), so that shortcut is itself under test.
 *
 * Layout: every tensor is [B, N, H, d] contiguous (token stride H*d, head stride d); LSE and the
 * optional weight dump are [B, H, N] and [B, H, N, N].  Inputs are fp64, or bf16 bit patterns
 * that are widened exactly.  No blocking, no fusion, no BLAS.  Threads (OpenMP) split the query
 * rows of one (batch, head); dK/dV partials are kept per thread and summed in thread order, so a
 * run with a fixed thread count is reproducible.
 *
 * Pins (tests/test_oracle_pins.py): rows of P sum to one; identical keys give the mean of V;
 * N = 1; Q = 0; N = 2, d = 1 sigmoid case with hand-derived numbers; central finite differences
 * of sum(O*dO) in every coordinate of Q, K, V; gradient invariants; the block-merge identity;
 * shift and permutation invariance; agreement with a dense fp64 softmax(QK^T)V + autograd.
 * Causal: first row returns v_0; last row equals the unmasked result; prefix property; dense masked
 * softmax in numpy; finite differences; last key's gradients come from the last query alone.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)
#define ORACLE_ENOMEM (-2)

static double bf16_to_f64(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static size_t idx4(int b, int n, int h, int N, int H, int d)
{
    return (((size_t)b * N + n) * H + h) * (size_t)d;
}

int avion_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Forward on fp64 inputs.  o: [B,N,H,d]; lse: [B,H,N]; weights: NULL or [B,H,N,N].
   causal != 0: query i sees keys 0..i only. */
static int fwd_core(const double *q, const double *k, const double *v, double *o, double *lse,
                    double *weights, int B, int H, int N, int d, double scale, int nthreads, int causal)
{
    if (!q || !k || !v || !o || !lse || B <= 0 || H <= 0 || N <= 0 || d <= 0) return ORACLE_EINVAL;
    if (nthreads <= 0) nthreads = avion_oracle_max_threads();
    int failed = 0;
#pragma omp parallel num_threads(nthreads)
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)N);
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
            long long rows = (long long)B * H * N;
#pragma omp for schedule(static)
            for (long long r = 0; r < rows; ++r) {
                int i = (int)(r % N);
                int h = (int)((r / N) % H);
                int b = (int)(r / ((long long)N * H));
                const double *qi = q + idx4(b, i, h, N, H, d);
                const int nk = causal ? i + 1 : N; /* keys this query sees */
                double m = -INFINITY;
                for (int j = 0; j < nk; ++j) {
                    const double *kj = k + idx4(b, j, h, N, H, d);
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += qi[c] * kj[c];
                    s[j] = scale * acc;
                    if (s[j] > m) m = s[j];
                }
                double l = 0.0;
                for (int j = 0; j < nk; ++j) {
                    s[j] = exp(s[j] - m);
                    l += s[j];
                }
                double *oi = o + idx4(b, i, h, N, H, d);
                for (int c = 0; c < d; ++c) oi[c] = 0.0;
                for (int j = 0; j < nk; ++j) {
                    double p = s[j] / l;
                    const double *vj = v + idx4(b, j, h, N, H, d);
                    for (int c = 0; c < d; ++c) oi[c] += p * vj[c];
                    if (weights) weights[(((size_t)b * H + h) * N + i) * (size_t)N + j] = p;
                }
                if (weights)
                    for (int j = nk; j < N; ++j) weights[(((size_t)b * H + h) * N + i) * (size_t)N + j] = 0.0;
                lse[((size_t)b * H + h) * N + i] = m + log(l);
            }
        }
        free(s);
    }
    return failed ? ORACLE_ENOMEM : ORACLE_OK;
}

int avion_oracle_fwd_f64(const double *q, const double *k, const double *v, double *o, double *lse,
                         double *weights, int B, int H, int N, int d, double scale, int nthreads)
{
    return fwd_core(q, k, v, o, lse, weights, B, H, N, d, scale, nthreads, 0);
}

int avion_oracle_fwd_causal_f64(const double *q, const double *k, const double *v, double *o, double *lse,
                                double *weights, int B, int H, int N, int d, double scale, int nthreads)
{
    return fwd_core(q, k, v, o, lse, weights, B, H, N, d, scale, nthreads, 1);
}

/* Backward on fp64 inputs, from the definition (P is rebuilt from q, k; o and lse are not inputs).
   dq, dk, dv: [B,N,H,d], fully overwritten.  causal != 0: query i sees keys 0..i only. */
static int bwd_core(const double *q, const double *k, const double *v, const double *dO,
                    double *dq, double *dk, double *dv, int B, int H, int N, int d,
                    double scale, int nthreads, int causal)
{
    if (!q || !k || !v || !dO || !dq || !dk || !dv || B <= 0 || H <= 0 || N <= 0 || d <= 0)
        return ORACLE_EINVAL;
    if (nthreads <= 0) nthreads = avion_oracle_max_threads();
    size_t nd = (size_t)N * d;
    /* per-thread partial dK and dV of the (batch, head) being processed */
    double *part = (double *)malloc(sizeof(double) * 2 * nd * (size_t)nthreads);
    double *rowbuf = (double *)malloc(sizeof(double) * 2 * (size_t)N * (size_t)nthreads);
    if (!part || !rowbuf) {
        free(part);
        free(rowbuf);
        return ORACLE_ENOMEM;
    }
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int used = 1;
#pragma omp parallel num_threads(nthreads)
            {
                int t = 0, nt = 1;
#ifdef _OPENMP
                t = omp_get_thread_num();
                nt = omp_get_num_threads();
#endif
#pragma omp single
                used = nt;
                double *pdk = part + (size_t)t * 2 * nd;
                double *pdv = pdk + nd;
                double *p = rowbuf + (size_t)t * 2 * N; /* weights of row i      */
                double *g = p + N;                      /* dP, then dS, of row i */
                memset(pdk, 0, sizeof(double) * 2 * nd);
#pragma omp for schedule(static)
                for (int i = 0; i < N; ++i) {
                    const double *qi = q + idx4(b, i, h, N, H, d);
                    const double *doi = dO + idx4(b, i, h, N, H, d);
                    const int nk = causal ? i + 1 : N; /* keys this query sees */
                    double m = -INFINITY;
                    for (int j = 0; j < nk; ++j) {
                        const double *kj = k + idx4(b, j, h, N, H, d);
                        double acc = 0.0;
                        for (int c = 0; c < d; ++c) acc += qi[c] * kj[c];
                        p[j] = scale * acc;
                        if (p[j] > m) m = p[j];
                    }
                    double l = 0.0;
                    for (int j = 0; j < nk; ++j) {
                        p[j] = exp(p[j] - m);
                        l += p[j];
                    }
                    double inner = 0.0; /* sum_k P_ik dP_ik */
                    for (int j = 0; j < nk; ++j) {
                        p[j] /= l;
                        const double *vj = v + idx4(b, j, h, N, H, d);
                        double acc = 0.0;
                        for (int c = 0; c < d; ++c) acc += doi[c] * vj[c];
                        g[j] = acc;
                        inner += p[j] * acc;
                    }
                    double *dqi = dq + idx4(b, i, h, N, H, d);
                    for (int c = 0; c < d; ++c) dqi[c] = 0.0;
                    for (int j = 0; j < nk; ++j) {
                        double ds = p[j] * (g[j] - inner);
                        const double *kj = k + idx4(b, j, h, N, H, d);
                        double *dkj = pdk + (size_t)j * d;
                        double *dvj = pdv + (size_t)j * d;
                        for (int c = 0; c < d; ++c) {
                            dqi[c] += ds * kj[c];
                            dkj[c] += ds * qi[c];
                            dvj[c] += p[j] * doi[c];
                        }
                    }
                    for (int c = 0; c < d; ++c) dqi[c] *= scale;
                }
                /* implicit barrier of the omp for: all partials are complete */
#pragma omp for schedule(static)
                for (int j = 0; j < N; ++j) {
                    double *dkj = dk + idx4(b, j, h, N, H, d);
                    double *dvj = dv + idx4(b, j, h, N, H, d);
                    for (int c = 0; c < d; ++c) {
                        double sk = 0.0, sv = 0.0;
                        for (int u = 0; u < nt; ++u) {
                            sk += part[(size_t)u * 2 * nd + (size_t)j * d + c];
                            sv += part[(size_t)u * 2 * nd + nd + (size_t)j * d + c];
                        }
                        dkj[c] = scale * sk;
                        dvj[c] = sv;
                    }
                }
            }
            (void)used;
        }
    }
    free(part);
    free(rowbuf);
    return ORACLE_OK;
}

int avion_oracle_bwd_f64(const double *q, const double *k, const double *v, const double *dO,
                         double *dq, double *dk, double *dv, int B, int H, int N, int d,
                         double scale, int nthreads)
{
    return bwd_core(q, k, v, dO, dq, dk, dv, B, H, N, d, scale, nthreads, 0);
}

int avion_oracle_bwd_causal_f64(const double *q, const double *k, const double *v, const double *dO,
                                double *dq, double *dk, double *dv, int B, int H, int N, int d,
                                double scale, int nthreads)
{
    return bwd_core(q, k, v, dO, dq, dk, dv, B, H, N, d, scale, nthreads, 1);
}

static double *widen(const uint16_t *x, size_t n)
{
    double *y = (double *)malloc(sizeof(double) * n);
    if (y)
        for (size_t i = 0; i < n; ++i) y[i] = bf16_to_f64(x[i]);
    return y;
}

/* Same as the fp64 entry points, on bf16 bit patterns (widened exactly). Outputs stay fp64. */
static int fwd_bits(const uint16_t *q, const uint16_t *k, const uint16_t *v, double *o, double *lse,
                    int B, int H, int N, int d, double scale, int nthreads, int causal)
{
    if (!q || !k || !v || B <= 0 || H <= 0 || N <= 0 || d <= 0) return ORACLE_EINVAL;
    size_t n = (size_t)B * N * H * d;
    double *qd = widen(q, n), *kd = widen(k, n), *vd = widen(v, n);
    int rc = ORACLE_ENOMEM;
    if (qd && kd && vd) rc = fwd_core(qd, kd, vd, o, lse, NULL, B, H, N, d, scale, nthreads, causal);
    free(qd);
    free(kd);
    free(vd);
    return rc;
}

int avion_oracle_fwd(const uint16_t *q, const uint16_t *k, const uint16_t *v, double *o, double *lse,
                     int B, int H, int N, int d, double scale, int nthreads)
{
    return fwd_bits(q, k, v, o, lse, B, H, N, d, scale, nthreads, 0);
}

int avion_oracle_fwd_causal(const uint16_t *q, const uint16_t *k, const uint16_t *v, double *o, double *lse,
                            int B, int H, int N, int d, double scale, int nthreads)
{
    return fwd_bits(q, k, v, o, lse, B, H, N, d, scale, nthreads, 1);
}

static int bwd_bits(const uint16_t *q, const uint16_t *k, const uint16_t *v, const uint16_t *dO,
                    double *dq, double *dk, double *dv, int B, int H, int N, int d, double scale,
                    int nthreads, int causal)
{
    if (!q || !k || !v || !dO || B <= 0 || H <= 0 || N <= 0 || d <= 0) return ORACLE_EINVAL;
    size_t n = (size_t)B * N * H * d;
    double *qd = widen(q, n), *kd = widen(k, n), *vd = widen(v, n), *gd = widen(dO, n);
    int rc = ORACLE_ENOMEM;
    if (qd && kd && vd && gd)
        rc = bwd_core(qd, kd, vd, gd, dq, dk, dv, B, H, N, d, scale, nthreads, causal);
    free(qd);
    free(kd);
    free(vd);
    free(gd);
    return rc;
}

int avion_oracle_bwd(const uint16_t *q, const uint16_t *k, const uint16_t *v, const uint16_t *dO,
                     double *dq, double *dk, double *dv, int B, int H, int N, int d, double scale,
                     int nthreads)
{
    return bwd_bits(q, k, v, dO, dq, dk, dv, B, H, N, d, scale, nthreads, 0);
}

int avion_oracle_bwd_causal(const uint16_t *q, const uint16_t *k, const uint16_t *v, const uint16_t *dO,
                            double *dq, double *dk, double *dv, int B, int H, int N, int d, double scale,
                            int nthreads)
{
    return bwd_bits(q, k, v, dO, dq, dk, dv, B, H, N, d, scale, nthreads, 1);
}
