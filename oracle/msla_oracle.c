/*
 * msla_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the multi-scale linear attention
 * (MSLA) module of EfficientViT computes (paper Section 3.1, Fig. 2 right).
 * It exists only so that tests, the smoke check and the bench's CPU-baseline
 * leg have something independent to compare the GPU library against.  It
 * shares no code, header, table or helper with the HIP path and is never
 * called by it.
 *
 * Everything is written as the defining sums, one loop nest per definition,
 * in double precision with no intermediate rounding, no blocking and no
 * fusion.  OpenMP (if enabled at compile time) only splits the outermost
 * independent index (token, image, head); it never changes a summation order.
 *
 * Conventions (definitions of the library boundary, shared with the GPU path
 * by specification only):
 *   - token maps are row-major [B, H, W, channels] (a token is one (y,x));
 *   - the 3*heads*d projected channels are ordered o = (h*3 + t)*d + e with
 *     t = 0:Q, 1:K, 2:V, so that every (head, Q/K/V) pair is one contiguous
 *     group of d channels -- the grouping Section 3.1 prescribes for the
 *     grouped 1x1 convolution (3*#heads groups of d channels);
 *   - convolutions are stride 1, zero padded by (k-1)/2, cross-correlation
 *     (no kernel flip); no bias, norm or activation inside the module;
 *   - the denominator of Eq. (3) gets "+ eps" (the equation itself has none;
 *     a token whose rectified query is all zero would otherwise be 0/0).
 *
 * Pins (tests/test_oracle_pins.py): linear form == explicit N x N form of
 * Eq. (1)+(2); constant V returns the constant; convex-hull bound; scale
 * invariances; N = 1; delta / shifted-delta / box depthwise kernels with
 * hand-counted border values; grouped conv == independent d x d blocks;
 * projections vs numpy matmul; whole-module reductions to bare Eq. (3).
 * Parity unpinned: only the conventions above (channel order, conv
 * orientation), which are definitions rather than results.
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int msla_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* y[n, o] = sum_c x[n, c] * w[o, c]        (Section 3.1: Q = x W_Q etc.; the
 * same definition serves the final projection of the concatenated heads).  */
void msla_oracle_linear(const double *x, const double *w, double *y,
                        long n_tokens, int c_in, int c_out)
{
    long n;
#pragma omp parallel for schedule(static)
    for (n = 0; n < n_tokens; ++n) {
        for (int o = 0; o < c_out; ++o) {
            double s = 0.0;
            for (int c = 0; c < c_in; ++c)
                s += x[n * c_in + c] * w[(long)o * c_in + c];
            y[n * c_out + o] = s;
        }
    }
}

/* Depthwise k x k aggregation of nearby tokens (Section 3.1, "small-kernel
 * depthwise-separable convolutions", depthwise half):
 *   out[b,y,x,o] = sum_{u,v<k} w[o,u,v] * in[b, y+u-p, x+v-p, o],  p=(k-1)/2,
 * terms whose source token lies outside the H x W grid contribute nothing.  */
void msla_oracle_dwconv(const double *in, const double *w, double *out,
                        int B, int H, int W, int ch, int k)
{
    const int p = (k - 1) / 2;
    long by;
#pragma omp parallel for schedule(static)
    for (by = 0; by < (long)B * H; ++by) {
        const int b = (int)(by / H), y = (int)(by % H);
        for (int x = 0; x < W; ++x) {
            for (int o = 0; o < ch; ++o) {
                double s = 0.0;
                for (int u = 0; u < k; ++u) {
                    const int yy = y + u - p;
                    if (yy < 0 || yy >= H) continue;
                    for (int v = 0; v < k; ++v) {
                        const int xx = x + v - p;
                        if (xx < 0 || xx >= W) continue;
                        s += w[((long)o * k + u) * k + v] *
                             in[(((long)b * H + yy) * W + xx) * ch + o];
                    }
                }
                out[(((long)b * H + y) * W + x) * ch + o] = s;
            }
        }
    }
}

/* Grouped 1x1 convolution, groups of d channels (Section 3.1: one group per
 * (head, Q/K/V), i.e. 3*#heads groups):
 *   out[n, o] = sum_{e<d} w[o, e] * in[n, (o / d)*d + e].                    */
void msla_oracle_grouped_pw(const double *in, const double *w, double *out,
                            long n_tokens, int ch, int d)
{
    long n;
#pragma omp parallel for schedule(static)
    for (n = 0; n < n_tokens; ++n) {
        for (int o = 0; o < ch; ++o) {
            const int g = o / d;
            double s = 0.0;
            for (int e = 0; e < d; ++e)
                s += w[(long)o * d + e] * in[n * ch + g * d + e];
            out[n * ch + o] = s;
        }
    }
}

static double relu(double v) { return v > 0.0 ? v : 0.0; }

/* The once-per-image state of Eq. (3) for one branch map of one image:
 *   kv[h, e, f] = sum_n relu(K_n[e]) * V_n[f]   (f < d)
 *   kv[h, e, d] = sum_n relu(K_n[e])
 * map is [N, 3*heads*d] in the channel order given at the top.              */
void msla_oracle_kv_state(const double *map, double *kv, long N, int heads, int d)
{
    const int ch = 3 * heads * d;
    int h;
#pragma omp parallel for schedule(static)
    for (h = 0; h < heads; ++h) {
        const int ko = (h * 3 + 1) * d, vo = (h * 3 + 2) * d;
        for (int e = 0; e < d; ++e) {
            for (int f = 0; f <= d; ++f) {
                double s = 0.0;
                for (long n = 0; n < N; ++n) {
                    const double kk = relu(map[n * ch + ko + e]);
                    s += (f < d) ? kk * map[n * ch + vo + f] : kk;
                }
                kv[((long)h * d + e) * (d + 1) + f] = s;
            }
        }
    }
}

/* Eq. (3), last line, for one branch map of one image, given its state:
 *   att[n, h*d + f] = relu(Q_n) . kv[h,:,f] / (relu(Q_n) . kv[h,:,d] + eps). */
void msla_oracle_apply(const double *map, const double *kv, double *att,
                       long N, int heads, int d, double eps,
                       long att_stride, long att_offset)
{
    const int ch = 3 * heads * d;
    long n;
#pragma omp parallel for schedule(static)
    for (n = 0; n < N; ++n) {
        for (int h = 0; h < heads; ++h) {
            const double *q = map + n * ch + (h * 3 + 0) * d;
            double den = 0.0;
            for (int e = 0; e < d; ++e)
                den += relu(q[e]) * kv[((long)h * d + e) * (d + 1) + d];
            for (int f = 0; f < d; ++f) {
                double num = 0.0;
                for (int e = 0; e < d; ++e)
                    num += relu(q[e]) * kv[((long)h * d + e) * (d + 1) + f];
                att[n * att_stride + att_offset + h * d + f] = num / (den + eps);
            }
        }
    }
}

/* Eq. (1) with the similarity of Eq. (2), written out in its quadratic form
 * for ONE head: s_ij = relu(Q_i) . relu(K_j),
 *   O_i = sum_j s_ij V_j / (sum_j s_ij + eps).
 * Q, K, V, O are [N, d].  O(N^2): tiny inputs only.  This is what the linear
 * form must reproduce "without changing its functionality".                */
void msla_oracle_attention_nxn(const double *Q, const double *K, const double *V,
                               double *O, long N, int d, double eps)
{
    for (long i = 0; i < N; ++i) {
        double den = 0.0;
        for (int f = 0; f < d; ++f) O[i * d + f] = 0.0;
        for (long j = 0; j < N; ++j) {
            double s = 0.0;
            for (int e = 0; e < d; ++e)
                s += relu(Q[i * d + e]) * relu(K[j * d + e]);
            den += s;
            for (int f = 0; f < d; ++f) O[i * d + f] += s * V[j * d + f];
        }
        for (int f = 0; f < d; ++f) O[i * d + f] /= (den + eps);
    }
}

/* Multi-scale token aggregation + per-head ReLU linear attention on a given
 * projected map (Section 3.1, Fig. 2 right, without the two projections).
 *   qkv  [B, H, W, 3*heads*d]
 *   w_dw  concatenation over the aggregated scales a of [3*heads*d, k_a, k_a]
 *   w_gpw [A, 3*heads*d, d]
 *   att  [B, H, W, (1+A)*heads*d], column (s*heads + h)*d + f, s = 0 the raw
 *        branch, s = a+1 the branch aggregated with kernel scales[a].
 * Every aggregated branch reads the raw map (parallel branches).  The sum of
 * Eq. (3) runs over the N = H*W tokens of one image and one branch only.
 * If kv_out is not NULL it receives [B, 1+A, heads, d, d+1].
 * Returns 0, or -1 if scratch memory could not be obtained.                 */
int msla_oracle_core_forward(const double *qkv, const double *w_dw,
                             const double *w_gpw, double *att, double *kv_out,
                             int B, int H, int W, int heads, int d,
                             const int *scales, int n_scales, double eps)
{
    const int ch = 3 * heads * d;
    const int S = 1 + n_scales;
    const long N = (long)H * W;
    const long att_stride = (long)S * heads * d;
    const long kv_sz = (long)heads * d * (d + 1);
    double *dw = NULL, *agg = NULL, *kv = NULL;
    int rc = -1;

    kv = (double *)malloc(sizeof(double) * (size_t)kv_sz);
    if (!kv) goto done;
    if (n_scales > 0) {
        dw = (double *)malloc(sizeof(double) * (size_t)B * N * ch);
        agg = (double *)malloc(sizeof(double) * (size_t)B * N * ch);
        if (!dw || !agg) goto done;
    }
    {
        const double *wd = w_dw;
        for (int s = 0; s < S; ++s) {
            const double *map = qkv;
            if (s > 0) {
                const int k = scales[s - 1];
                msla_oracle_dwconv(qkv, wd, dw, B, H, W, ch, k);
                msla_oracle_grouped_pw(dw, w_gpw + (long)(s - 1) * ch * d, agg,
                                       (long)B * N, ch, d);
                wd += (long)ch * k * k;
                map = agg;
            }
            for (int b = 0; b < B; ++b) {
                msla_oracle_kv_state(map + (long)b * N * ch, kv, N, heads, d);
                if (kv_out)
                    memcpy(kv_out + ((long)b * S + s) * kv_sz, kv,
                           sizeof(double) * (size_t)kv_sz);
                msla_oracle_apply(map + (long)b * N * ch, kv,
                                  att + (long)b * N * att_stride, N, heads, d, eps,
                                  att_stride, (long)s * heads * d);
            }
        }
    }
    rc = 0;
done:
    free(dw); free(agg); free(kv);
    return rc;
}

/* The whole module (Fig. 2 right): x [B,H,W,C] -> out [B,H,W,C].
 *   w_qkv [3*heads*d, C], w_proj [C, (1+A)*heads*d].                        */
int msla_oracle_forward(const double *x, const double *w_qkv, const double *w_dw,
                        const double *w_gpw, const double *w_proj, double *out,
                        int B, int C, int H, int W, int heads, int d,
                        const int *scales, int n_scales, double eps)
{
    const int ch = 3 * heads * d;
    const int S = 1 + n_scales;
    const long T = (long)B * H * W;
    double *qkv = (double *)malloc(sizeof(double) * (size_t)T * ch);
    double *att = (double *)malloc(sizeof(double) * (size_t)T * S * heads * d);
    int rc = -1;
    if (qkv && att) {
        msla_oracle_linear(x, w_qkv, qkv, T, C, ch);
        rc = msla_oracle_core_forward(qkv, w_dw, w_gpw, att, NULL, B, H, W, heads, d,
                                      scales, n_scales, eps);
        if (rc == 0)
            msla_oracle_linear(att, w_proj, out, T, S * heads * d, C);
    }
    free(qkv); free(att);
    return rc;
}
