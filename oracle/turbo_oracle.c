/*
 * CPU oracle for the two batch-reduction operations of the TurboTransformers
 * paper (Section 4.1.2, "GPU-based Batch-Reduction").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT PATH.  Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg may call it.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Both operations are exact definitions that the paper's method reaches
 * faster, so the oracle is the plain definition, one row at a time, in
 * double precision:
 *
 *   - Softmax needs a row sum and a row maximum over the low dimension of a
 *     2-D view (Section 4.1.2); in attention it is applied to the scaled
 *     query-key dot products (Section 2.1).  The additive mask is the
 *     padding convention of Section 2.1 (short sequences are zero-padded to
 *     the longest one in the batch).
 *   - LayerNorm needs the row mean and the row variance (Section 4.1.2); the
 *     variance is the population variance of Equation 1.  The fused kernel
 *     ("AddBiasLayerNorm", Section 6.2.1) normalises x + bias + residual.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (hand cases, closed forms, invariants, library special cases).  Nothing is
 * "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of host threads the row loops may use (rows are independent). */
void oracle_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int oracle_get_threads(void) { return g_threads; }

/*
 * Scaled, masked softmax over the last axis of scores[B][H][Sq][Sk].
 *   z_k = scale * s_k + mask_k ;  m = max_k z_k ;  e_k = exp(z_k - m) ;
 *   y_k = e_k / sum_k e_k.
 * mask may be NULL.  Otherwise mask element (b, q, k) lives at
 * mask[b*mask_stride_b + q*mask_stride_q + k] and is shared by all heads.
 * Nothing is special-cased for masked entries: they become 0 only because
 * exp() of a very negative number underflows.
 */
void oracle_masked_softmax(const double *scores, const double *mask, long long mask_stride_b,
                           long long mask_stride_q, int B, int H, int Sq, int Sk, double scale, double *out)
{
    long long n_rows = (long long)B * H * Sq;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long long row = 0; row < n_rows; ++row) {
        long long q = row % Sq;
        long long b = row / ((long long)H * Sq);
        const double *s = scores + row * Sk;
        const double *a = mask ? mask + b * mask_stride_b + q * mask_stride_q : NULL;
        double *y = out + row * Sk;

        double m = -INFINITY;
        for (int k = 0; k < Sk; ++k) {
            double z = scale * s[k] + (a ? a[k] : 0.0);
            y[k] = z;
            if (z > m) m = z;
        }
        double l = 0.0;
        for (int k = 0; k < Sk; ++k) {
            y[k] = exp(y[k] - m);
            l += y[k];
        }
        for (int k = 0; k < Sk; ++k) y[k] /= l;
    }
}

/*
 * out[r][j] = (t_j - mu) / sqrt(var + eps) * gamma_j + beta_j  with
 * t_j = x[r][j] + bias_j + residual[r][j],  mu = mean_j t_j,
 * var = mean_j (t_j - mu)^2   (population variance, first form of Eq. 1).
 * bias and residual may be NULL (treated as zeros).
 */
void oracle_add_bias_layernorm(const double *x, const double *residual, const double *bias, const double *gamma,
                               const double *beta, long long rows, int hidden, double eps, double *out)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long long r = 0; r < rows; ++r) {
        const double *xr = x + r * hidden;
        const double *rr = residual ? residual + r * hidden : NULL;
        double *o = out + r * hidden;

        double sum = 0.0;
        for (int j = 0; j < hidden; ++j) {
            double t = xr[j] + (bias ? bias[j] : 0.0) + (rr ? rr[j] : 0.0);
            o[j] = t;
            sum += t;
        }
        double mu = sum / hidden;
        double ss = 0.0;
        for (int j = 0; j < hidden; ++j) {
            double d = o[j] - mu;
            ss += d * d;
        }
        double var = ss / hidden;
        double inv = 1.0 / sqrt(var + eps);
        for (int j = 0; j < hidden; ++j) o[j] = (o[j] - mu) * inv * gamma[j] + beta[j];
    }
}

/* ---- the three variance algorithms that Equation 1 relates ------------- */

/* E(x - E x)^2: two reductions, the form the paper attributes to the baseline. */
double oracle_variance_two_pass(const double *x, int n)
{
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += x[i];
    double mu = s / n, ss = 0.0;
    for (int i = 0; i < n; ++i) ss += (x[i] - mu) * (x[i] - mu);
    return ss / n;
}

/* E(x^2) - E^2(x): x and x^2 reduced together, the form the paper adopts. */
double oracle_variance_sum_of_squares(const double *x, int n)
{
    double s = 0.0, s2 = 0.0;
    for (int i = 0; i < n; ++i) {
        s += x[i];
        s2 += x[i] * x[i];
    }
    double mu = s / n;
    return s2 / n - mu * mu;
}

/* Welford's running (count, mean, M2) update: one pass like the form above,
 * without the cancellation it suffers when |mean| >> std. */
double oracle_variance_welford(const double *x, int n)
{
    double mean = 0.0, m2 = 0.0;
    for (int i = 0; i < n; ++i) {
        double d = x[i] - mean;
        mean += d / (i + 1);
        m2 += d * (x[i] - mean);
    }
    return m2 / n;
}

/* Merge of two (count, mean, M2) states (Chan et al.), used by tests to check
 * that splitting a row in any way gives the same statistics. */
void oracle_welford_merge(double na, double mean_a, double m2_a, double nb, double mean_b, double m2_b,
                          double *n, double *mean, double *m2)
{
    double nt = na + nb;
    if (nt == 0.0) {
        *n = 0.0; *mean = 0.0; *m2 = 0.0;
        return;
    }
    double d = mean_b - mean_a;
    *n = nt;
    *mean = mean_a + d * (nb / nt);
    *m2 = m2_a + m2_b + d * d * (na * nb / nt);
}

/* ---- element-wise fused kernels (Section 4.1.1 counts the fused activations and the fused transposes as the
 * non-GEMM kernels that are purely element-wise) ---------------------------------------------------------
 * The paper names the two kinds but prints no formula or layout.  Readings taken here:
 *   - the activation is GELU, the feed-forward activation of the BERT family the paper evaluates:
 *     gelu(t) = t * Phi(t), Phi the standard normal distribution function (approximate = 0), or its
 *     usual tanh form 0.5 t (1 + tanh(sqrt(2/pi) (t + 0.044715 t^3))) (approximate = 1);
 *   - the fused transposes are the head split after the Q/K/V projection (bias added on the way) and
 *     the head merge after attention.
 */

/* out[r][j] = gelu(x[r][j] + bias[j]); bias may be NULL. */
void oracle_add_bias_gelu(const double *x, const double *bias, long long rows, int hidden, int approximate,
                          double *out)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long long r = 0; r < rows; ++r) {
        for (int j = 0; j < hidden; ++j) {
            double t = x[r * hidden + j] + (bias ? bias[j] : 0.0);
            double y;
            if (approximate) {
                double u = 0.7978845608028654 * (t + 0.044715 * t * t * t); /* sqrt(2/pi) */
                y = 0.5 * t * (1.0 + tanh(u));
            } else {
                y = t * 0.5 * erfc(-t * 0.7071067811865476); /* Phi(t) = erfc(-t/sqrt 2)/2 */
            }
            out[r * hidden + j] = y;
        }
    }
}

/* Head split with bias: x is [B][S][n_split][H][D] (the output of one fused projection, n_split = 3 for
 * Q, K, V together, 1 for a single projection), bias is [n_split][H][D] or NULL, out is
 * [n_split][B][H][S][D]:  out[k][b][h][s][d] = x[b][s][k][h][d] + bias[k][h][d]. */
void oracle_add_bias_split_heads(const double *x, const double *bias, int B, int S, int n_split, int H, int D,
                                 double *out)
{
    for (int k = 0; k < n_split; ++k)
        for (int b = 0; b < B; ++b)
            for (int h = 0; h < H; ++h)
                for (int s = 0; s < S; ++s)
                    for (int d = 0; d < D; ++d) {
                        long long src = ((((long long)b * S + s) * n_split + k) * H + h) * D + d;
                        long long dst = ((((long long)k * B + b) * H + h) * S + s) * D + d;
                        out[dst] = x[src] + (bias ? bias[((long long)k * H + h) * D + d] : 0.0);
                    }
}

/* Head merge: x is [B][H][S][D], out is [B][S][H][D]:  out[b][s][h][d] = x[b][h][s][d]. */
void oracle_merge_heads(const double *x, int B, int H, int S, int D, double *out)
{
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h)
            for (int s = 0; s < S; ++s)
                for (int d = 0; d < D; ++d)
                    out[(((long long)b * S + s) * H + h) * D + d] = x[(((long long)b * H + h) * S + s) * D + d];
}

/* ---- length-aware variants for zero-padded variable-length batches (Section 2.1) -----------------------
 * The paper pads short requests to the longest one and lets its kernels work on the padding.  These variants
 * take the request lengths instead: what lies beyond a request's length is neither read nor normalised.
 * out is a full copy of the input for everything the operation leaves untouched. */

/* For q < q_len[b] (all q if q_len is NULL) and k_len[b] > 0: softmax over the first k_len[b] keys of
 * scale * scores, exact zeros for the remaining keys.  All other rows: out = scores. */
void oracle_masked_softmax_varlen(const double *scores, const int *q_len, const int *k_len, int B, int H, int Sq,
                                  int Sk, double scale, double *out)
{
    for (int b = 0; b < B; ++b) {
        int kl = k_len[b] < 0 ? 0 : (k_len[b] > Sk ? Sk : k_len[b]);
        for (int h = 0; h < H; ++h)
            for (int q = 0; q < Sq; ++q) {
                long long row = ((long long)b * H + h) * Sq + q;
                const double *s = scores + row * Sk;
                double *y = out + row * Sk;
                int active = kl > 0 && (q_len == NULL || q < q_len[b]);
                if (!active) {
                    for (int k = 0; k < Sk; ++k) y[k] = s[k];
                    continue;
                }
                double m = -INFINITY, l = 0.0;
                for (int k = 0; k < kl; ++k)
                    if (scale * s[k] > m) m = scale * s[k];
                for (int k = 0; k < kl; ++k) {
                    y[k] = exp(scale * s[k] - m);
                    l += y[k];
                }
                for (int k = 0; k < kl; ++k) y[k] /= l;
                for (int k = kl; k < Sk; ++k) y[k] = 0.0;
            }
    }
}

/* Causal variant: query q sees the keys k <= q + (Sk - Sq) (the last query sees every key), further restricted to
 * k < k_len[b] when k_len is given.  Rows with q >= q_len[b] (when q_len is given) and rows without any visible key
 * are copied unchanged; everywhere else the visible keys get softmax(scale * s) and the others exact zeros. */
void oracle_masked_softmax_causal(const double *scores, const int *q_len, const int *k_len, int B, int H, int Sq, int Sk,
                                  double scale, double *out)
{
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h)
            for (int q = 0; q < Sq; ++q) {
                long long row = ((long long)b * H + h) * Sq + q;
                const double *s = scores + row * Sk;
                double *y = out + row * Sk;
                int visible = q + (Sk - Sq) + 1;          /* keys 0 .. q + (Sk - Sq) */
                if (k_len != NULL && k_len[b] < visible) visible = k_len[b];
                if (visible > Sk) visible = Sk;
                if (visible <= 0 || (q_len != NULL && q >= q_len[b])) {
                    for (int k = 0; k < Sk; ++k) y[k] = s[k];
                    continue;
                }
                double m = -INFINITY, l = 0.0;
                for (int k = 0; k < visible; ++k)
                    if (scale * s[k] > m) m = scale * s[k];
                for (int k = 0; k < visible; ++k) {
                    y[k] = exp(scale * s[k] - m);
                    l += y[k];
                }
                for (int k = 0; k < visible; ++k) y[k] /= l;
                for (int k = visible; k < Sk; ++k) y[k] = 0.0;
            }
}

/* Row-packed variable-length batch: no padding in memory.  Request b holds its scores as [H][len_b][len_b],
 * the requests follow one another (request b starts at element H * sum_{i<b} len_i^2).  Every row of len_b keys is
 * normalised: y = softmax(scale * s) over the row.  `scores` and `out` hold H * sum len_b^2 values. */
void oracle_masked_softmax_packed(const double *scores, const int *len, int B, int H, double scale, double *out)
{
    long long base = 0;
    for (int b = 0; b < B; ++b) {
        const long long n = len[b];
        for (int h = 0; h < H; ++h)
            for (long long q = 0; q < n; ++q) {
                const double *s = scores + base + (h * n + q) * n;
                double *y = out + base + (h * n + q) * n;
                double m = -INFINITY, l = 0.0;
                for (long long k = 0; k < n; ++k)
                    if (scale * s[k] > m) m = scale * s[k];
                for (long long k = 0; k < n; ++k) {
                    y[k] = exp(scale * s[k] - m);
                    l += y[k];
                }
                for (long long k = 0; k < n; ++k) y[k] /= l;
            }
        base += (long long)H * n * n;
    }
}

/* x, residual, out_before, out are [B][S][hidden].  Token rows s < len[b] get LayerNorm(x + bias + residual)
 * * gamma + beta; padding rows keep out_before. */
void oracle_add_bias_layernorm_varlen(const double *x, const double *residual, const double *bias,
                                      const double *gamma, const double *beta, const int *len, int B, int S,
                                      int hidden, double eps, const double *out_before, double *out)
{
    for (int b = 0; b < B; ++b)
        for (int s = 0; s < S; ++s) {
            long long r = (long long)b * S + s;
            if (s < len[b])
                oracle_add_bias_layernorm(x + r * hidden, residual ? residual + r * hidden : NULL, bias, gamma, beta, 1,
                                          hidden, eps, out + r * hidden);
            else
                for (int j = 0; j < hidden; ++j) out[r * hidden + j] = out_before[r * hidden + j];
        }
}
