/*
 * Plain C oracle of one decode step of a transformer attention block.
 *
 * TEST INFRASTRUCTURE ONLY: loaded by tests, the smoke check and the bench's
 * cpu_baseline leg.  It shares nothing with the HIP library.
 *
 * Same definition as the numpy oracle next to it (paper Eq. 1 for one new
 * token per sequence; decode semantics of Sec. 2.1; RoPE with half-split
 * pairing and theta_i = base^(-2i/d); W_qkv columns ordered Q heads, K heads,
 * V heads; query head i uses KV head i / (n_q/n_kv)).  fp16 inputs are widened
 * exactly; every sum is a double accumulated in index order.  OpenMP spreads
 * independent outputs (column chunks, heads) over threads; no output's
 * arithmetic depends on the thread count.
 *
 * Pins: tests compare it against the numpy oracle and run the same
 * invariants on it (empty cache, x = 0 closed form).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double half_to_double(uint16_t h)
{
    /* binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
    uint64_t sign = (uint64_t)(h >> 15) << 63;
    uint32_t e = (h >> 10) & 0x1fu, m = h & 0x3ffu;
    uint64_t bits;
    double v;
    if (e == 0) {                                   /* zero and subnormals: m * 2^-24 */
        v = (double)m * 5.9604644775390625e-08;
        return (h >> 15) ? -v : v;
    }
    if (e == 31)
        bits = sign | 0x7ff0000000000000ull | ((uint64_t)m << 42);
    else
        bits = sign | ((uint64_t)(e - 15 + 1023) << 52) | ((uint64_t)m << 42);
    memcpy(&v, &bits, sizeof v);
    return v;
}

int cfo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void cfo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* y[b][j] = sum_i x[b][i] * w[i][j],  w row-major [rows, cols] */
static void matvec(const double *x, const uint16_t *w, int B, int rows, int cols, double *y)
{
    enum { CH = 256 };
    int nch = (cols + CH - 1) / CH;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < nch; ++c) {
        int j0 = c * CH, j1 = j0 + CH < cols ? j0 + CH : cols;
        for (int b = 0; b < B; ++b) {
            double *yb = y + (size_t)b * cols;
            for (int j = j0; j < j1; ++j) yb[j] = 0.0;
            for (int i = 0; i < rows; ++i) {
                double xi = x[(size_t)b * rows + i];
                const uint16_t *wr = w + (size_t)i * cols;
                for (int j = j0; j < j1; ++j) yb[j] += xi * half_to_double(wr[j]);
            }
        }
    }
}

static void rope_inplace(double *v, int d, int pos, double base)
{
    int h = d / 2;
    for (int i = 0; i < h; ++i) {
        double ang = (double)pos * pow(base, -2.0 * (double)i / (double)d);
        double c = cos(ang), s = sin(ang);
        double lo = v[i], hi = v[i + h];
        v[i] = lo * c - hi * s;
        v[i + h] = hi * c + lo * s;
    }
}

/*
 * The block for an input given as doubles: xd [B,D] (not modified); everything else as in
 * cfo_decode_block below.
 */
int cfo_decode_block_real(const double *xd, const uint16_t *w_qkv, const uint16_t *w_o,
                          const uint16_t *k_cache, const uint16_t *v_cache,
                          int B, int D, int nq, int nkv, int d, int max_seq, int pos, double rope_base,
                          double *out, double *q_rot, double *k_rot, double *v_new, double *attn)
{
    if (B < 1 || D < 1 || nq < 1 || nkv < 1 || nq % nkv || d < 2 || (d & 1) || pos < 0 || pos >= max_seq)
        return -1;
    int G = nq / nkv, nqkv = (nq + 2 * nkv) * d;
    double *y = (double *)malloc(sizeof(double) * (size_t)B * nqkv);
    if (!y) return -1;

    matvec(xd, w_qkv, B, D, nqkv, y);
    for (int b = 0; b < B; ++b) {
        const double *yb = y + (size_t)b * nqkv;
        memcpy(q_rot + (size_t)b * nq * d, yb, sizeof(double) * (size_t)nq * d);
        memcpy(k_rot + (size_t)b * nkv * d, yb + (size_t)nq * d, sizeof(double) * (size_t)nkv * d);
        memcpy(v_new + (size_t)b * nkv * d, yb + (size_t)(nq + nkv) * d, sizeof(double) * (size_t)nkv * d);
        for (int i = 0; i < nq; ++i) rope_inplace(q_rot + ((size_t)b * nq + i) * d, d, pos, rope_base);
        for (int g = 0; g < nkv; ++g) rope_inplace(k_rot + ((size_t)b * nkv + g) * d, d, pos, rope_base);
    }

    double inv_sqrt_d = 1.0 / sqrt((double)d);
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bi = 0; bi < B * nq; ++bi) {
        int b = bi / nq, i = bi % nq, g = i / G;
        const double *q = q_rot + ((size_t)b * nq + i) * d;
        const uint16_t *kc = k_cache + ((size_t)b * nkv + g) * (size_t)max_seq * d;
        const uint16_t *vc = v_cache + ((size_t)b * nkv + g) * (size_t)max_seq * d;
        const double *kn = k_rot + ((size_t)b * nkv + g) * d;
        const double *vn = v_new + ((size_t)b * nkv + g) * d;
        double *s = (double *)malloc(sizeof(double) * (size_t)(pos + 1));
        double *a = attn + ((size_t)b * nq + i) * d;
        if (!s) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        double m = -INFINITY;
        for (int t = 0; t <= pos; ++t) {
            double acc = 0.0;
            if (t < pos)
                for (int c = 0; c < d; ++c) acc += q[c] * half_to_double(kc[(size_t)t * d + c]);
            else
                for (int c = 0; c < d; ++c) acc += q[c] * kn[c];
            s[t] = acc * inv_sqrt_d;
            if (s[t] > m) m = s[t];
        }
        double l = 0.0;
        for (int t = 0; t <= pos; ++t) { s[t] = exp(s[t] - m); l += s[t]; }
        for (int c = 0; c < d; ++c) a[c] = 0.0;
        for (int t = 0; t <= pos; ++t) {
            double w = s[t] / l;
            if (t < pos)
                for (int c = 0; c < d; ++c) a[c] += w * half_to_double(vc[(size_t)t * d + c]);
            else
                for (int c = 0; c < d; ++c) a[c] += w * vn[c];
        }
        free(s);
    }
    if (!fail) matvec(attn, w_o, B, nq * d, D, out);
    free(y);
    return fail ? -1 : 0;
}

/*
 * x [B,D], w_qkv [D,(nq+2nkv)d], w_o [nq d, D], caches [B,nkv,max_seq,d] (fp16 bits).
 * Outputs (double, caller-allocated): out [B,D], q_rot [B,nq,d], k_rot [B,nkv,d],
 * v_new [B,nkv,d], attn [B,nq,d].  The caches are not modified.  Returns 0, or -1
 * on a bad argument or allocation failure.
 */
int cfo_decode_block(const uint16_t *x, const uint16_t *w_qkv, const uint16_t *w_o,
                     const uint16_t *k_cache, const uint16_t *v_cache,
                     int B, int D, int nq, int nkv, int d, int max_seq, int pos, double rope_base,
                     double *out, double *q_rot, double *k_rot, double *v_new, double *attn)
{
    if (B < 1 || D < 1) return -1;
    double *xd = (double *)malloc(sizeof(double) * (size_t)B * D);
    if (!xd) return -1;
    for (size_t i = 0; i < (size_t)B * D; ++i) xd[i] = half_to_double(x[i]);
    int rc = cfo_decode_block_real(xd, w_qkv, w_o, k_cache, v_cache, B, D, nq, nkv, d, max_seq, pos, rope_base,
                                   out, q_rot, k_rot, v_new, attn);
    free(xd);
    return rc;
}

/*
 * The decoder layer around the block: pre-normalisation and residual connection of a Llama-style
 * layer (the paper leaves RMSNorm to other libraries, end of Sec. 3; the block is Eq. 1):
 *   n_b   = x_b / sqrt(mean_j(x_bj^2) + eps) * gamma      (RMSNorm, all in double, nothing rounded)
 *   out_b = x_b + block(n_b)
 * gamma [D] fp16 bits.  Other arguments and outputs as above.
 */
int cfo_decode_layer(const uint16_t *x, const uint16_t *gamma, double eps, const uint16_t *w_qkv, const uint16_t *w_o,
                     const uint16_t *k_cache, const uint16_t *v_cache,
                     int B, int D, int nq, int nkv, int d, int max_seq, int pos, double rope_base,
                     double *out, double *q_rot, double *k_rot, double *v_new, double *attn)
{
    if (B < 1 || D < 1) return -1;
    double *n = (double *)malloc(sizeof(double) * (size_t)B * D);
    if (!n) return -1;
    for (int b = 0; b < B; ++b) {
        double ss = 0.0;
        for (int j = 0; j < D; ++j) {
            double v = half_to_double(x[(size_t)b * D + j]);
            ss += v * v;
        }
        double r = 1.0 / sqrt(ss / (double)D + eps);
        for (int j = 0; j < D; ++j)
            n[(size_t)b * D + j] = half_to_double(x[(size_t)b * D + j]) * r * half_to_double(gamma[j]);
    }
    int rc = cfo_decode_block_real(n, w_qkv, w_o, k_cache, v_cache, B, D, nq, nkv, d, max_seq, pos, rope_base,
                                   out, q_rot, k_rot, v_new, attn);
    if (rc == 0)
        for (size_t i = 0; i < (size_t)B * D; ++i) out[i] += half_to_double(x[i]);
    free(n);
    return rc;
}
