/*
 * Sanitizer run of the oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A small driver that calls every function of kst_oracle.c on a handful of shapes (edge cases
 * included) so that the test-suite can build both files with -fsanitize=address,undefined and
 * let the sanitizers watch every index the oracle computes.  It checks two closed forms on the
 * way (all-ones input and kernel; the one-pixel layer), prints "ok" and returns 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int kst_oracle_out_size(int N, int n, int P);
int kst_oracle_forward(const double *in, const double *w, double *out, int B, int Cin, int Cout, int N, int n, int P);
int kst_oracle_forward_epilogue(const double *in, const double *w, const double *bias, double *out,
                                int B, int Cin, int Cout, int N, int n, int P, int act);
int kst_oracle_backward_input(const double *g, const double *w, double *din, int B, int Cin, int Cout, int N, int n, int P);
int kst_oracle_backward_weight(const double *in, const double *g, double *dw, int B, int Cin, int Cout, int N, int n, int P);
int kst_oracle_forward_planes(const double *in, const double *w, double *out_planes, const int32_t *b_idx,
                              const int32_t *co_idx, int n_planes, int B, int Cin, int Cout, int N, int n, int P);
void kst_oracle_conventional_ops(int Cin, int Cout, int N, int n, int P, int64_t *mults, int64_t *adds);

static double *filled(size_t count, double v)
{
    double *p = (double *)malloc((count ? count : 1) * sizeof(double));
    if (!p) exit(2);
    for (size_t i = 0; i < count; ++i) p[i] = v;
    return p;
}

static int one_shape(int B, int Cin, int Cout, int N, int n, int P)
{
    const int M = kst_oracle_out_size(N, n, P);
    if (M < 1) return 0;
    double *in = filled((size_t)B * Cin * N * N, 1.0), *w = filled((size_t)Cout * Cin * n * n, 1.0);
    double *out = filled((size_t)B * Cout * M * M, -1.0), *out2 = filled((size_t)B * Cout * M * M, -1.0);
    double *bias = filled((size_t)Cout, 0.5);
    double *din = filled((size_t)B * Cin * N * N, -1.0), *dw = filled((size_t)Cout * Cin * n * n, -1.0);
    double *planes = filled((size_t)2 * M * M, -1.0);
    const int32_t b_idx[2] = {0, B - 1}, co_idx[2] = {Cout - 1, 0};
    int bad = 0;
    bad |= kst_oracle_forward(in, w, out, B, Cin, Cout, N, n, P);
    for (int act = 0; act < 3; ++act) bad |= kst_oracle_forward_epilogue(in, w, bias, out2, B, Cin, Cout, N, n, P, act);
    bad |= kst_oracle_forward_epilogue(in, w, NULL, out2, B, Cin, Cout, N, n, P, 1);
    bad |= kst_oracle_backward_input(out, w, din, B, Cin, Cout, N, n, P);
    bad |= kst_oracle_backward_weight(in, out, dw, B, Cin, Cout, N, n, P);
    bad |= kst_oracle_forward_planes(in, w, planes, b_idx, co_idx, 2, B, Cin, Cout, N, n, P);
    /* all ones: every output is Cin times the number of kernel taps that meet an input pixel,
       so the largest output is Cin * ceil(n/2)^2 when the map is large enough to hold such a window */
    double top = 0.0;
    for (size_t i = 0; i < (size_t)B * Cout * M * M; ++i) top = out[i] > top ? out[i] : top;
    const int t = (n + 1) / 2, fit = N < t ? N : t;
    if (fabs(top - (double)Cin * fit * fit) > 1e-9) bad |= 4;
    for (int k = 0; k < M * M; ++k)
        if (planes[k] != out[((size_t)0 * Cout + (Cout - 1)) * M * M + k]) bad |= 8;
    free(in); free(w); free(out); free(out2); free(bias); free(din); free(dw); free(planes);
    return bad;
}

int main(void)
{
    static const int shapes[][6] = {
        {1, 1, 1, 1, 1, 0}, {1, 1, 1, 1, 5, 2}, {2, 3, 2, 4, 3, 0}, {1, 2, 3, 4, 5, 2}, {1, 1, 2, 4, 5, 3},
        {2, 2, 2, 5, 4, 1}, {1, 3, 1, 7, 7, 0}, {3, 1, 1, 2, 2, 0}, {1, 2, 2, 3, 6, 4}, {2, 1, 3, 6, 1, 0},
    };
    int bad = 0;
    for (size_t k = 0; k < sizeof(shapes) / sizeof(shapes[0]); ++k)
        bad |= one_shape(shapes[k][0], shapes[k][1], shapes[k][2], shapes[k][3], shapes[k][4], shapes[k][5]);
    /* illegal shapes and an unknown activation must be refused, not computed */
    double x = 1.0, y = 0.0;
    if (kst_oracle_forward(&x, &x, &y, 1, 1, 1, 1, 3, 0) != 1) bad |= 16;      /* 2N - n < 1 */
    if (kst_oracle_forward(&x, &x, &y, 0, 1, 1, 1, 1, 0) != 1) bad |= 16;
    if (kst_oracle_forward_epilogue(&x, &x, NULL, &y, 1, 1, 1, 1, 1, 0, 7) != 1) bad |= 16;
    int64_t mults = 0, adds = 0;
    kst_oracle_conventional_ops(1024, 512, 4, 4, 2, &mults, &adds);
    if (mults != 536870912LL || adds != 536838144LL) bad |= 32;                /* Table 4, DCGAN layer 2 */
    printf(bad ? "FAILED %d\n" : "ok\n", bad);
    return bad ? 1 : 0;
}
