// Gradients of the transpose convolution (end of Section 3.3: the method also serves the input
// and kernel gradients of back-propagation).  With g = d(loss)/d(out), P = 0:
//
//   input gradient    din[b][ci][a][c]  = sum_co sum_u sum_v g[b][co][2a-u][2c-v] * w[co][ci][u][v]
//   kernel gradient   dw[co][ci][u][v]  = sum_b sum_a sum_c in[b][ci][a][c] * g[b][co][2a-u][2c-v]
//
// over the (u, v) / (a, c) whose g index lies inside the M x M map.  Both are the forward's
// products read backwards: only the N^2 n^2 products with an original input pixel exist, the
// ones the segregated forward performs; nothing is multiplied by an embedded zero.  Kernel
// element (u, v) = (2al+r, 2be+s) belongs to sub-kernel K_(r,s) of Section 3.2 and meets the
// output rows of parity r only: g[2a-u] = g[2(a-r-al)+r].
//
// This file: the kernels that take any shape and either operand type (plain ALU work).
#include "kst_igemm_common.h"

namespace kst {

namespace {

// One thread per din element; g is fp32, w is T.
template <typename T>
__global__ void __launch_bounds__(256) backward_input_generic_kernel(const float *__restrict__ g, const T *__restrict__ w,
                                                                      float *__restrict__ din, int B, int Cin, int Cout,
                                                                      int N, int M, int n)
{
    const size_t e = (size_t)blockIdx.x * 256u + threadIdx.x;
    const size_t total = (size_t)B * Cin * N * N;
    if (e >= total) return;
    const int c = (int)(e % (unsigned)N);
    size_t rest = e / (unsigned)N;
    const int a = (int)(rest % (unsigned)N);
    rest /= (unsigned)N;
    const int ci = (int)(rest % (unsigned)Cin);
    const int b = (int)(rest / (unsigned)Cin);
    // rows 2a - u inside [0, M): u in [u_lo, u_hi]
    const int u_lo = max(0, 2 * a - (M - 1)), u_hi = min(n - 1, 2 * a);
    const int v_lo = max(0, 2 * c - (M - 1)), v_hi = min(n - 1, 2 * c);
    float acc = 0.0f;
    for (int co = 0; co < Cout; ++co) {
        const float *gp = g + ((size_t)b * Cout + co) * M * M;
        const T *wk = w + ((size_t)co * Cin + ci) * n * n;
        for (int u = u_lo; u <= u_hi; ++u)
            for (int v = v_lo; v <= v_hi; ++v)
                acc = fmaf(gp[(size_t)(2 * a - u) * M + (2 * c - v)], to_f32(wk[u * n + v]), acc);
    }
    din[e] = acc;
}

// One workgroup per (co, ci) and slice of the positions: each thread sums its share of the
// slice's (b, a, c) for one kernel element at a time, then a tree in LDS.  With more than one
// slice the workgroups write partial sums [slice][co][ci][u][v] that a second pass adds up.
template <typename T>
__global__ void __launch_bounds__(256) backward_weight_generic_kernel(const T *__restrict__ in, const float *__restrict__ g,
                                                                       float *__restrict__ dst, int B, int Cin, int Cout,
                                                                       int N, int M, int n, int per_slice)
{
    __shared__ float red[256];
    const int pairs = Cout * Cin;
    const int slice = blockIdx.x / pairs, pair = blockIdx.x - slice * pairs;
    const int co = pair / Cin, ci = pair - co * Cin;
    const int tid = threadIdx.x;
    const int per_item = N * N;
    const int total = B * per_item;
    const int e_begin = slice * per_slice, e_end = min(total, e_begin + per_slice);
    float *o = dst + (size_t)slice * pairs * n * n;
    for (int uv = 0; uv < n * n; ++uv) {
        const int u = uv / n, v = uv - u * n;
        float acc = 0.0f;
        for (int e = e_begin + tid; e < e_end; e += 256) {
            const int b = e / per_item, rem = e - b * per_item;
            const int a = rem / N, c = rem - a * N;
            const int y = 2 * a - u, x = 2 * c - v;
            if (y >= 0 && y < M && x >= 0 && x < M)
                acc = fmaf(to_f32(in[(((size_t)b * Cin + ci) * N + a) * N + c]),
                           g[(((size_t)b * Cout + co) * M + y) * M + x], acc);
        }
        red[tid] = acc;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) red[tid] += red[tid + s];
            __syncthreads();
        }
        if (tid == 0) o[((size_t)co * Cin + ci) * n * n + uv] = red[0];
        __syncthreads();
    }
}

// Slices of the position range: few (co, ci) pairs alone cannot fill the chip.
int weight_slices(const Shape &s)
{
    const long long pairs = (long long)s.Cout * s.Cin;
    const long long total = (long long)s.B * s.N * s.N;
    long long slices = (1024 + pairs - 1) / pairs;
    if (slices > 256) slices = 256;
    if (slices > (total + 1023) / 1024) slices = (total + 1023) / 1024;   // at least 1024 positions per slice
    return slices < 1 ? 1 : (int)slices;
}

}  // namespace

hipError_t launch_backward_input_generic(const float *g, const void *w, float *din, const Shape &s, kst_dtype dt,
                                         hipStream_t stream)
{
    const size_t total = (size_t)s.B * s.Cin * s.N * s.N;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dt == KST_BF16)
        hipLaunchKernelGGL(backward_input_generic_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream, g,
                           (const uint16_t *)w, din, s.B, s.Cin, s.Cout, s.N, s.M, s.n);
    else
        hipLaunchKernelGGL(backward_input_generic_kernel<float>, dim3(blocks), dim3(256), 0, stream, g, (const float *)w,
                           din, s.B, s.Cin, s.Cout, s.N, s.M, s.n);
    return hipGetLastError();
}

size_t backward_weight_generic_workspace_bytes(const Shape &s)
{
    const int slices = weight_slices(s);
    return slices > 1 ? (((size_t)slices * s.Cout * s.Cin * s.n * s.n * sizeof(float) + 255) & ~(size_t)255) : 0;
}

hipError_t launch_backward_weight_generic(const void *in, const float *g, float *dw, void *ws, const Shape &s,
                                          kst_dtype dt, hipStream_t stream)
{
    const int slices = weight_slices(s);
    const int total = s.B * s.N * s.N;
    const int per_slice = (total + slices - 1) / slices;
    const unsigned blocks = (unsigned)s.Cout * (unsigned)s.Cin * (unsigned)slices;
    float *dst = slices > 1 ? (float *)ws : dw;
    if (dt == KST_BF16)
        hipLaunchKernelGGL(backward_weight_generic_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream,
                           (const uint16_t *)in, g, dst, s.B, s.Cin, s.Cout, s.N, s.M, s.n, per_slice);
    else
        hipLaunchKernelGGL(backward_weight_generic_kernel<float>, dim3(blocks), dim3(256), 0, stream, (const float *)in, g,
                           dst, s.B, s.Cin, s.Cout, s.N, s.M, s.n, per_slice);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || slices == 1) return e;
    return launch_splitk_reduce((const float *)ws, dw, (size_t)s.Cout * s.Cin * s.n * s.n, slices, stream);
}

}  // namespace kst
