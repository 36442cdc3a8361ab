/*
 * Drives every function of oracle/turbo_oracle.c on exactly sized heap buffers.  Built with
 * -fsanitize=address,undefined by tests/test_oracle_pins.py: a read or write past an operand, a signed overflow in
 * an index or a misaligned access ends the run.  Results are only checked for being finite and, where the
 * definition gives it away, for their row sums; the values themselves are pinned elsewhere.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../oracle/turbo_oracle.c"

static unsigned long long g_state = 88172645463325252ull;
static double draw(void) /* xorshift: uniform on (-1, 1) */
{
    g_state ^= g_state << 13;
    g_state ^= g_state >> 7;
    g_state ^= g_state << 17;
    return (double)(g_state >> 11) / 4503599627370496.0 - 1.0;
}
static double *filled(long long n)
{
    double *p = malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    for (long long i = 0; i < n; ++i) p[i] = 3.0 * draw();
    return p;
}
static int all_finite(const double *p, long long n)
{
    for (long long i = 0; i < n; ++i)
        if (!isfinite(p[i])) return 0;
    return 1;
}
#define CHECK(c)                                                 \
    do {                                                         \
        if (!(c)) {                                              \
            printf("FAILED line %d: %s\n", __LINE__, #c);        \
            return 1;                                            \
        }                                                        \
    } while (0)

int main(void)
{
    const int shapes[][4] = {{1, 1, 1, 1}, {2, 3, 5, 7}, {3, 2, 4, 16}, {1, 2, 9, 33}};
    for (int threads = 1; threads <= 3; threads += 2) {
        oracle_set_threads(threads);
        for (unsigned s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s) {
            const int B = shapes[s][0], H = shapes[s][1], Sq = shapes[s][2], Sk = shapes[s][3];
            const long long n = (long long)B * H * Sq * Sk;
            double *sc = filled(n), *out = filled(n);
            /* no mask, key mask [B,Sk], causal [Sq,Sk], dense [B,Sq,Sk]: each exactly as large as its strides say */
            oracle_masked_softmax(sc, NULL, 0, 0, B, H, Sq, Sk, 0.125, out);
            CHECK(all_finite(out, n));
            double *mk = filled((long long)B * Sk);
            oracle_masked_softmax(sc, mk, Sk, 0, B, H, Sq, Sk, 0.125, out);
            double *mc = filled((long long)Sq * Sk);
            oracle_masked_softmax(sc, mc, 0, Sk, B, H, Sq, Sk, 0.125, out);
            double *md = filled((long long)B * Sq * Sk);
            oracle_masked_softmax(sc, md, (long long)Sq * Sk, Sk, B, H, Sq, Sk, 0.125, out);
            for (long long r = 0; r < (long long)B * H * Sq; ++r) {
                double sum = 0.0;
                for (int k = 0; k < Sk; ++k) sum += out[r * Sk + k];
                CHECK(fabs(sum - 1.0) < 1e-12);
            }
            /* length-aware and causal forms; lengths include 0 and the full length */
            int *ql = malloc(sizeof(int) * B), *kl = malloc(sizeof(int) * B);
            for (int b = 0; b < B; ++b) {
                ql[b] = b % 2 ? Sq : Sq / 2;
                kl[b] = b % 3 == 2 ? 0 : (b % 2 ? Sk : (Sk + 1) / 2);
            }
            oracle_masked_softmax_varlen(sc, ql, kl, B, H, Sq, Sk, 0.5, out);
            oracle_masked_softmax_varlen(sc, NULL, kl, B, H, Sq, Sk, 0.5, out);
            oracle_masked_softmax_causal(sc, ql, kl, B, H, Sq, Sk, 0.5, out);
            oracle_masked_softmax_causal(sc, NULL, NULL, B, H, Sq, Sk, 0.5, out);
            CHECK(all_finite(out, n));
            free(ql); free(kl); free(mk); free(mc); free(md); free(sc); free(out);
        }
        /* row-packed batch: H * sum(len^2) values, a request without tokens among them */
        {
            const int len[4] = {5, 0, 17, 1}, H = 3;
            long long total = 0;
            for (int b = 0; b < 4; ++b) total += (long long)H * len[b] * len[b];
            double *sc = filled(total), *out = filled(total);
            oracle_masked_softmax_packed(sc, len, 4, H, 0.25, out);
            CHECK(all_finite(out, total));
            free(sc); free(out);
        }
        /* LayerNorm with and without its optional operands; one column; length-aware form */
        const int ln_shapes[][2] = {{1, 1}, {4, 3}, {7, 64}, {2, 1000}};
        for (unsigned s = 0; s < sizeof(ln_shapes) / sizeof(ln_shapes[0]); ++s) {
            const int rows = ln_shapes[s][0], hidden = ln_shapes[s][1];
            const long long n = (long long)rows * hidden;
            double *x = filled(n), *r = filled(n), *b = filled(hidden), *g = filled(hidden), *be = filled(hidden),
                   *out = filled(n);
            oracle_add_bias_layernorm(x, r, b, g, be, rows, hidden, 1e-5, out);
            CHECK(all_finite(out, n));
            oracle_add_bias_layernorm(x, NULL, NULL, g, be, rows, hidden, 1e-5, out);
            CHECK(all_finite(out, n));
            CHECK(isfinite(oracle_variance_two_pass(x, hidden)));
            CHECK(isfinite(oracle_variance_sum_of_squares(x, hidden)));
            CHECK(isfinite(oracle_variance_welford(x, hidden)));
            free(x); free(r); free(b); free(g); free(be); free(out);
        }
        {
            const int B = 3, S = 5, hidden = 12, len[3] = {5, 0, 2};
            const long long n = (long long)B * S * hidden;
            double *x = filled(n), *r = filled(n), *b = filled(hidden), *g = filled(hidden), *be = filled(hidden),
                   *before = filled(n), *out = filled(n);
            oracle_add_bias_layernorm_varlen(x, r, b, g, be, len, B, S, hidden, 1e-5, before, out);
            oracle_add_bias_layernorm_varlen(x, NULL, NULL, g, be, len, B, S, hidden, 1e-5, before, out);
            CHECK(all_finite(out, n));
            free(x); free(r); free(b); free(g); free(be); free(before); free(out);
        }
        /* element-wise kernels */
        {
            const int rows = 5, hidden = 9;
            double *x = filled(rows * hidden), *b = filled(hidden), *out = filled(rows * hidden);
            oracle_add_bias_gelu(x, b, rows, hidden, 0, out);
            oracle_add_bias_gelu(x, NULL, rows, hidden, 1, out);
            CHECK(all_finite(out, rows * hidden));
            free(x); free(b); free(out);
            const int B = 2, S = 3, K = 3, H = 2, D = 5;
            const long long n = (long long)B * S * K * H * D;
            double *px = filled(n), *pb = filled((long long)K * H * D), *po = filled(n);
            oracle_add_bias_split_heads(px, pb, B, S, K, H, D, po);
            oracle_add_bias_split_heads(px, NULL, B, S, K, H, D, po);
            oracle_merge_heads(px, B, K * H, S, D, po);
            CHECK(all_finite(po, n));
            free(px); free(pb); free(po);
        }
        double nn, mm, qq;
        oracle_welford_merge(0, 0, 0, 0, 0, 0, &nn, &mm, &qq);
        oracle_welford_merge(3, 1.0, 2.0, 5, -1.0, 0.5, &nn, &mm, &qq);
        CHECK(nn == 8.0 && isfinite(mm) && isfinite(qq));
    }
    printf("ok\n");
    return 0;
}
