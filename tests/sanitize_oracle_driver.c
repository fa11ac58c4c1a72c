/* Driver for tests/test_oracle_sanitizers.py: calls every entry point of oracle/msla_oracle.c on small
 * inputs held in heap buffers of exactly the documented sizes, so that an address or undefined-behaviour
 * sanitizer build reports any access past an operand (the values are checked elsewhere: the oracle's pins).
 * Prints "sanitizer driver ok" and returns 0 when every call came back. */
#include <stdio.h>
#include <stdlib.h>

void msla_oracle_linear(const double *x, const double *w, double *y, long n, int c_in, int c_out);
void msla_oracle_dwconv(const double *in, const double *w, double *out, int B, int H, int W, int ch, int k);
void msla_oracle_grouped_pw(const double *in, const double *w, double *out, long n, int ch, int d);
void msla_oracle_kv_state(const double *map, double *kv, long N, int heads, int d);
void msla_oracle_apply(const double *map, const double *kv, double *att, long N, int heads, int d, double eps,
                       long att_stride, long att_off);
void msla_oracle_attention_nxn(const double *Q, const double *K, const double *V, double *O, long N, int d, double eps);
int msla_oracle_core_forward(const double *qkv, const double *w_dw, const double *w_gpw, double *att, double *kv_out,
                             int B, int H, int W, int heads, int d, const int *scales, int n_scales, double eps);
int msla_oracle_forward(const double *x, const double *w_qkv, const double *w_dw, const double *w_gpw,
                        const double *w_proj, double *out, int B, int C, int H, int W, int heads, int d,
                        const int *scales, int n_scales, double eps);

static unsigned long long state = 88172645463325252ull;
static double draw(void) {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state % 20001ull) / 10000.0 - 1.0;
}
static double *filled(size_t n) {
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    for (size_t i = 0; i < n; ++i) p[i] = draw();
    return p;
}

static int one_shape(int B, int C, int H, int W, int heads, int d, const int *scales, int n_scales) {
    const int ch = 3 * heads * d, S = 1 + n_scales;
    const long N = (long)H * W, T = N * B;
    size_t dw_elems = 0;
    for (int i = 0; i < n_scales; ++i) dw_elems += (size_t)ch * scales[i] * scales[i];
    double *x = filled((size_t)T * C), *w_qkv = filled((size_t)ch * C), *w_dw = filled(dw_elems);
    double *w_gpw = filled((size_t)n_scales * ch * d), *w_proj = filled((size_t)C * S * heads * d);
    double *out = filled((size_t)T * C), *qkv = filled((size_t)T * ch), *tmp = filled((size_t)T * ch);
    double *att = filled((size_t)T * S * heads * d), *kv = filled((size_t)B * S * heads * d * (d + 1));
    int rc = 0;
    msla_oracle_linear(x, w_qkv, qkv, T, C, ch);
    if (n_scales > 0) {
        msla_oracle_dwconv(qkv, w_dw, tmp, B, H, W, ch, scales[0]);
        msla_oracle_grouped_pw(tmp, w_gpw, qkv, T, ch, d);
    }
    msla_oracle_kv_state(qkv, kv, N, heads, d);
    msla_oracle_apply(qkv, kv, att, N, heads, d, 1e-15, (long)S * heads * d, (long)(S - 1) * heads * d);
    {   /* one head's Q, K, V as [N, d] for the N x N form */
        double *Q = filled((size_t)N * d), *K = filled((size_t)N * d), *V = filled((size_t)N * d), *O = filled((size_t)N * d);
        msla_oracle_attention_nxn(Q, K, V, O, N, d, 1e-15);
        free(Q); free(K); free(V); free(O);
    }
    rc |= msla_oracle_core_forward(qkv, w_dw, w_gpw, att, kv, B, H, W, heads, d, scales, n_scales, 1e-15);
    rc |= msla_oracle_core_forward(qkv, w_dw, w_gpw, att, NULL, B, H, W, heads, d, scales, n_scales, 1e-15);
    rc |= msla_oracle_forward(x, w_qkv, w_dw, w_gpw, w_proj, out, B, C, H, W, heads, d, scales, n_scales, 1e-15);
    free(x); free(w_qkv); free(w_dw); free(w_gpw); free(w_proj); free(out); free(qkv); free(tmp); free(att); free(kv);
    return rc;
}

int main(void) {
    const int s5[1] = {5}, s37[2] = {3, 7};
    int rc = 0;
    rc |= one_shape(1, 16, 1, 1, 1, 16, s5, 1);        /* a single token: the window is all padding */
    rc |= one_shape(2, 32, 5, 7, 2, 16, s37, 2);       /* three branches, windows larger than the image rows */
    rc |= one_shape(1, 24, 9, 4, 3, 8, s5, 1);         /* head size 8, C != heads * d */
    rc |= one_shape(1, 32, 3, 3, 1, 32, s5, 0);        /* head size 32, no aggregated scale */
    if (rc != 0) { fprintf(stderr, "an oracle call failed\n"); return 1; }
    printf("sanitizer driver ok\n");
    return 0;
}
