/*
 * Oracle for the transpose convolution of arxiv 2209.03704 -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that every GPU result is checked
 * against.  It is not part of the product: only the test-suite, the smoke
 * check and the CPU-baseline leg of the benchmark may call it.  It shares no
 * code with the HIP library.
 *
 * What it computes (Section 1, second paragraph, and Eq. 1 of Section 2):
 *
 *   1. Up-sampling.  An N x N map becomes S x S with S = 2N-1 by embedding a
 *      zero after every row and every column:
 *          U[p][q] = in[p/2][q/2]  if p and q are both even, else 0.
 *      With a padding factor P (Section 3.3 applies P = 2 in its figures; the
 *      benchmark shapes use P = 0) a frame of P zeros is put around U, giving
 *      Sp = S + 2P.
 *   2. Stride-1 correlation with the n x n kernel (Eq. 1, read with 0-based
 *      offsets u,v = 0..n-1, no kernel flip), summed over input channels:
 *          out[b][co][y][x] = sum_ci sum_u sum_v  Upad[b][ci][y+u][x+v] * w[co][ci][u][v]
 *      for 0 <= y,x < M,  M = Sp - n + 1  (= 2N - n when P = 0).
 *
 * U is really built and the zeros are really multiplied: there is no parity
 * shortcut anywhere in this file.  All arithmetic is fp64.  Layouts are dense
 * row-major: in[B][Cin][N][N], w[Cout][Cin][n][n], out[B][Cout][M][M].
 *
 * Parity pins (tests/test_oracle_pins.py): hand-worked 4x4 / 3x3 example of
 * Fig. 2's shapes, all-ones and unit-impulse closed forms, n = 1 and n = 2
 * degenerate cases, agreement with separately coded forms of Eqs. 7-10 and of
 * the scatter (adjoint) form, linearity, the adjoint identity with a strided
 * correlation, library conv routines on fp64, and the operation counts of
 * Table 4; the gradients by the inner-product identities that define an adjoint and
 * by a library autograd of the forward in fp64; the bias + activation form by constant maps
 * (zero kernel), printed values of tanh, the order of bias and activation on a one-pixel
 * layer, the hand-worked example shifted and clipped, and a library layer in fp64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Output edge length for input edge N, kernel edge n, padding factor P. */
int kst_oracle_out_size(int N, int n, int P)
{
    return (2 * N - 1) + 2 * P - n + 1;
}

int kst_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Build the zero-embedded, zero-framed maps of one batch item: Upad[Cin][Sp][Sp]. */
static void upsample_item(const double *in_b, double *Upad, int Cin, int N, int P)
{
    const int S = 2 * N - 1;
    const int Sp = S + 2 * P;
    memset(Upad, 0, (size_t)Cin * Sp * Sp * sizeof(double));
    for (int ci = 0; ci < Cin; ++ci)
        for (int a = 0; a < N; ++a)
            for (int b = 0; b < N; ++b)
                Upad[((size_t)ci * Sp + (P + 2 * a)) * Sp + (P + 2 * b)] =
                    in_b[((size_t)ci * N + a) * N + b];
}

/* Eq. 1 on the up-sampled maps, one output plane (one batch item, one co). */
static void correlate_plane(const double *Upad, const double *w_co, double *out_plane,
                            int Cin, int Sp, int n, int M)
{
    for (int y = 0; y < M; ++y)
        for (int x = 0; x < M; ++x) {
            double acc = 0.0;
            for (int ci = 0; ci < Cin; ++ci)
                for (int u = 0; u < n; ++u)
                    for (int v = 0; v < n; ++v)
                        acc += Upad[((size_t)ci * Sp + (y + u)) * Sp + (x + v)] *
                               w_co[((size_t)ci * n + u) * n + v];
            out_plane[(size_t)y * M + x] = acc;
        }
}

/*
 * Full forward.  Returns 0, or 1 for an illegal shape / failed allocation.
 * out must hold B*Cout*M*M doubles.
 */
int kst_oracle_forward(const double *in, const double *w, double *out,
                       int B, int Cin, int Cout, int N, int n, int P)
{
    if (B < 1 || Cin < 1 || Cout < 1 || N < 1 || n < 1 || P < 0) return 1;
    const int M = kst_oracle_out_size(N, n, P);
    if (M < 1) return 1;
    const int Sp = 2 * N - 1 + 2 * P;
    double *Upad = (double *)malloc((size_t)Cin * Sp * Sp * sizeof(double));
    if (!Upad) return 1;
    for (int b = 0; b < B; ++b) {
        upsample_item(in + (size_t)b * Cin * N * N, Upad, Cin, N, P);
#pragma omp parallel for schedule(dynamic, 1)
        for (int co = 0; co < Cout; ++co)
            correlate_plane(Upad, w + (size_t)co * Cin * n * n,
                            out + ((size_t)b * Cout + co) * M * M, Cin, Sp, n, M);
    }
    free(Upad);
    return 0;
}

/*
 * The layer as a generator uses it: the transpose convolution above, then a bias per output
 * channel, then an activation.  The paper leaves both out (its layers are timed bare; Table 3
 * only lists the generators they come from); this is the usual definition of such a layer,
 * written out on top of kst_oracle_forward:
 *     out[b][co][y][x] = act( T[b][co][y][x] + bias[co] ),   T = kst_oracle_forward(in, w)
 * act: 0 identity, 1 max(v, 0), 2 tanh(v).  bias may be NULL (no bias).  fp64, libm's tanh.
 * Returns 0, or 1 for an illegal shape, an unknown act or a failed allocation.
 */
int kst_oracle_forward_epilogue(const double *in, const double *w, const double *bias, double *out,
                                int B, int Cin, int Cout, int N, int n, int P, int act)
{
    if (act < 0 || act > 2) return 1;
    if (kst_oracle_forward(in, w, out, B, Cin, Cout, N, n, P) != 0) return 1;
    const int M = kst_oracle_out_size(N, n, P);
    for (int b = 0; b < B; ++b)
        for (int co = 0; co < Cout; ++co) {
            double *plane = out + ((size_t)b * Cout + co) * M * M;
            for (size_t e = 0; e < (size_t)M * M; ++e) {
                double v = plane[e];
                if (bias) v += bias[co];
                if (act == 1) v = v > 0.0 ? v : 0.0;
                else if (act == 2) v = tanh(v);
                plane[e] = v;
            }
        }
    return 0;
}

/*
 * Gradients of the forward definition (the paper states, at the end of Section 3.3, that the
 * method also serves the input and kernel gradients of back-propagation, without giving
 * formulas; these are the plain adjoints of the two steps above).  With g = d(loss)/d(out):
 *
 *   input gradient:   every product Upad[y+u][x+v] * w[u][v] of Eq. 1 sends g[y][x] * w[u][v]
 *                     back to Upad[y+u][x+v]; the gradient of zero-embedding is sampling the
 *                     even rows and columns inside the frame:
 *                         dUpad[b][ci][y+u][x+v] += g[b][co][y][x] * w[co][ci][u][v]
 *                         din[b][ci][a][c] = dUpad[b][ci][P+2a][P+2c]
 *   kernel gradient:  dw[co][ci][u][v] = sum_b sum_y sum_x Upad[b][ci][y+u][x+v] * g[b][co][y][x]
 *
 * dUpad and Upad are really built, zeros included.  Return 0, or 1 for an illegal shape or a
 * failed allocation.
 */
int kst_oracle_backward_input(const double *g, const double *w, double *din,
                              int B, int Cin, int Cout, int N, int n, int P)
{
    if (B < 1 || Cin < 1 || Cout < 1 || N < 1 || n < 1 || P < 0) return 1;
    const int M = kst_oracle_out_size(N, n, P);
    if (M < 1) return 1;
    const int Sp = 2 * N - 1 + 2 * P;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int ci = 0; ci < Cin; ++ci) {
            double *dU = (double *)calloc((size_t)Sp * Sp, sizeof(double));
            if (!dU) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            for (int co = 0; co < Cout; ++co) {
                const double *gp = g + ((size_t)b * Cout + co) * M * M;
                const double *wk = w + ((size_t)co * Cin + ci) * n * n;
                for (int y = 0; y < M; ++y)
                    for (int x = 0; x < M; ++x)
                        for (int u = 0; u < n; ++u)
                            for (int v = 0; v < n; ++v)
                                dU[(size_t)(y + u) * Sp + (x + v)] += gp[(size_t)y * M + x] * wk[u * n + v];
            }
            double *d = din + ((size_t)b * Cin + ci) * N * N;
            for (int a = 0; a < N; ++a)
                for (int c = 0; c < N; ++c) d[(size_t)a * N + c] = dU[(size_t)(P + 2 * a) * Sp + (P + 2 * c)];
            free(dU);
        }
    return fail;
}

int kst_oracle_backward_weight(const double *in, const double *g, double *dw,
                               int B, int Cin, int Cout, int N, int n, int P)
{
    if (B < 1 || Cin < 1 || Cout < 1 || N < 1 || n < 1 || P < 0) return 1;
    const int M = kst_oracle_out_size(N, n, P);
    if (M < 1) return 1;
    const int Sp = 2 * N - 1 + 2 * P;
    double *Upad = (double *)malloc((size_t)Cin * Sp * Sp * sizeof(double));
    if (!Upad) return 1;
    memset(dw, 0, (size_t)Cout * Cin * n * n * sizeof(double));
    for (int b = 0; b < B; ++b) {
        upsample_item(in + (size_t)b * Cin * N * N, Upad, Cin, N, P);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int co = 0; co < Cout; ++co)
            for (int ci = 0; ci < Cin; ++ci) {
                const double *gp = g + ((size_t)b * Cout + co) * M * M;
                const double *Up = Upad + (size_t)ci * Sp * Sp;
                double *d = dw + ((size_t)co * Cin + ci) * n * n;
                for (int u = 0; u < n; ++u)
                    for (int v = 0; v < n; ++v) {
                        double acc = 0.0;
                        for (int y = 0; y < M; ++y)
                            for (int x = 0; x < M; ++x)
                                acc += Up[(size_t)(y + u) * Sp + (x + v)] * gp[(size_t)y * M + x];
                        d[u * n + v] += acc;
                    }
            }
    }
    free(Upad);
    return 0;
}

/*
 * The same definition restricted to chosen output planes, for sizes where
 * the whole tensor would take too long: plane k is (b_idx[k], co_idx[k]) and
 * is written, complete, to out_planes[k][M][M].
 */
int kst_oracle_forward_planes(const double *in, const double *w, double *out_planes,
                              const int32_t *b_idx, const int32_t *co_idx, int n_planes,
                              int B, int Cin, int Cout, int N, int n, int P)
{
    if (B < 1 || Cin < 1 || Cout < 1 || N < 1 || n < 1 || P < 0 || n_planes < 0) return 1;
    const int M = kst_oracle_out_size(N, n, P);
    if (M < 1) return 1;
    for (int k = 0; k < n_planes; ++k)
        if (b_idx[k] < 0 || b_idx[k] >= B || co_idx[k] < 0 || co_idx[k] >= Cout) return 1;
    const int Sp = 2 * N - 1 + 2 * P;
    int fail = 0;
#pragma omp parallel
    {
        double *Upad = (double *)malloc((size_t)Cin * Sp * Sp * sizeof(double));
        if (!Upad) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int k = 0; k < n_planes; ++k) {
            if (!Upad) continue;
            upsample_item(in + (size_t)b_idx[k] * Cin * N * N, Upad, Cin, N, P);
            correlate_plane(Upad, w + (size_t)co_idx[k] * Cin * n * n,
                            out_planes + (size_t)k * M * M, Cin, Sp, n, M);
        }
        free(Upad);
    }
    return fail;
}

/*
 * Operation counts of the conventional method as Table 4 counts them: one
 * multiplication per (output element, kernel element, ci, co), and one
 * addition fewer than that per output element of each output channel.
 */
void kst_oracle_conventional_ops(int Cin, int Cout, int N, int n, int P,
                                 int64_t *mults, int64_t *adds)
{
    const int64_t M = kst_oracle_out_size(N, n, P);
    *mults = M * M * (int64_t)n * n * Cin * Cout;
    *adds = *mults - M * M * Cout;
}
