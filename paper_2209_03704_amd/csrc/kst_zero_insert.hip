// The conventional method (Section 1; Eq. 1 applied to the up-sampled map),
// kept as the speed-up reference.  Deliberately plain: U is written to HBM
// with all its zeros and every output runs the full n x n x Cin loop over it.
#include "kst_internal.h"

namespace kst {

// U[b][ci][p][q] = in[b][ci][p/2][q/2] when p and q are even, else 0.
template <typename T>
__global__ void __launch_bounds__(256) upsample_kernel(const T *__restrict__ in, T *__restrict__ U,
                                                         unsigned planes, int N, int S)
{
    const size_t e = (size_t)blockIdx.x * 256u + threadIdx.x;
    const size_t total = (size_t)planes * S * S;
    if (e >= total) return;
    const int q = (int)(e % (unsigned)S);
    const size_t rest = e / (unsigned)S;
    const int p = (int)(rest % (unsigned)S);
    const size_t plane = rest / (unsigned)S;
    T v = T(0);
    if (((p | q) & 1) == 0) v = in[(plane * N + (p >> 1)) * N + (q >> 1)];
    U[e] = v;
}

// One thread per output element; Eq. 1 with the channel sum, reading U.
template <typename T>
__global__ void __launch_bounds__(256) conv_on_upsampled_kernel(const T *__restrict__ U, const T *__restrict__ w,
                                                                  float *__restrict__ out, int Cin, int Cout,
                                                                  int S, int n, int M, size_t total)
{
    const size_t e = (size_t)blockIdx.x * 256u + threadIdx.x;
    if (e >= total) return;
    const int x = (int)(e % (unsigned)M);
    size_t rest = e / (unsigned)M;
    const int y = (int)(rest % (unsigned)M);
    rest /= (unsigned)M;
    const int co = (int)(rest % (unsigned)Cout);
    const size_t b = rest / (unsigned)Cout;
    float acc = 0.0f;
    for (int ci = 0; ci < Cin; ++ci) {
        const size_t ub = ((b * Cin + ci) * S + y) * S + x;
        const size_t wb = ((size_t)co * Cin + ci) * n * n;
        for (int u = 0; u < n; ++u)
            for (int v = 0; v < n; ++v)
                acc = fmaf(to_f32(U[ub + (size_t)u * S + v]), to_f32(w[wb + u * n + v]), acc);
    }
    out[e] = acc;
}

template <typename T>
static hipError_t run(const T *in, const T *w, T *U, float *out, const Shape &s, hipStream_t stream)
{
    const int S = 2 * s.N - 1;
    const unsigned planes = (unsigned)s.B * (unsigned)s.Cin;
    const size_t u_total = (size_t)planes * S * S;
    hipLaunchKernelGGL(upsample_kernel<T>, dim3((unsigned)((u_total + 255) / 256)), dim3(256), 0, stream,
                       in, U, planes, s.N, S);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const size_t o_total = (size_t)s.B * s.Cout * s.M * s.M;
    hipLaunchKernelGGL(conv_on_upsampled_kernel<T>, dim3((unsigned)((o_total + 255) / 256)), dim3(256), 0, stream,
                       (const T *)U, w, out, s.Cin, s.Cout, S, s.n, s.M, o_total);
    return hipGetLastError();
}

hipError_t launch_zero_insert(const void *in, const void *w, void *U, float *out, const Shape &s,
                              kst_dtype dt, hipStream_t stream)
{
    if (dt == KST_BF16)
        return run<uint16_t>((const uint16_t *)in, (const uint16_t *)w, (uint16_t *)U, out, s, stream);
    if (dt == KST_F16)
        return run<half_bits>((const half_bits *)in, (const half_bits *)w, (half_bits *)U, out, s, stream);
    return run<float>((const float *)in, (const float *)w, (float *)U, out, s, stream);
}

}  // namespace kst
