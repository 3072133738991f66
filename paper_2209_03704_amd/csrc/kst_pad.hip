// Padding factor P of Section 3.3 (Figs. 5-7): the up-sampled map is framed by P zeros,
// which the segregated method turns into a frame on the ORIGINAL input.
//
// For even P the framed operation is exactly the unframed one on the input framed by P / 2
// zeros (the paper's reduced padding factor).  For odd P the up-sampled frame is one zero
// short of that of P + 1 on every side, so its output is the output for P + 1 without its
// outermost rows and columns; the one-pixel shift is what swaps the roles of the four
// sub-kernels (the paper's reversed order K4, K3, K2, K1).  Both cases therefore run the
// unframed kernels on a framed copy of the input; odd P adds a crop.
#include "kst_internal.h"

namespace kst {

namespace {

// dst[b*c][Nq][Ns] = src[b*c][N][N] framed by q zeros, rows Ns >= Nq = N + 2q elements apart
// (the elements past Nq are zeros too); one thread per element.  I: index type (32 bits while the
// copy has fewer than 2^32 elements: its two divisions per element are what the kernel costs).
template <typename T, typename I>
__global__ void __launch_bounds__(256) frame_input_kernel(const T *__restrict__ src, T *__restrict__ dst, unsigned planes,
                                                          int N, int q, int Ns)
{
    const int Nq = N + 2 * q;
    const I total = (I)planes * (I)Nq * (I)Ns;
    for (I i = (I)blockIdx.x * 256 + threadIdx.x; i < total; i += (I)gridDim.x * 256) {
        const I row = i / (unsigned)Ns;
        const int x = (int)(i - row * (unsigned)Ns) - q;
        const I plane = row / (unsigned)Nq;
        const int y = (int)(row - plane * (unsigned)Nq) - q;
        T v = (T)0;
        if (x >= 0 && x < N && y >= 0 && y < N) v = src[((size_t)plane * N + y) * N + x];
        dst[i] = v;
    }
}

// dst[plane][M][M] = src[plane][M + 2q][M + 2q] without its q outermost rows and columns.
__global__ void __launch_bounds__(256) crop_kernel(const float *__restrict__ src, float *__restrict__ dst, unsigned planes,
                                                   int M, int q)
{
    const int Ms = M + 2 * q;
    const size_t total = (size_t)planes * M * M;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t row = i / (unsigned)M;
        const int x = (int)(i - row * (unsigned)M);
        const size_t plane = row / (unsigned)M;
        const int y = (int)(row - plane * (unsigned)M);
        dst[i] = src[(plane * Ms + y + q) * Ms + x + q];
    }
}

// dst[i] = src[i] widened to fp32 (exact for both 16-bit types).
template <typename T>
__global__ void __launch_bounds__(256) widen_kernel(const T *__restrict__ src, float *__restrict__ dst, size_t total)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) dst[i] = to_f32(src[i]);
}

unsigned grid_for(size_t total)
{
    const size_t blocks = (total + 255) / 256;
    return (unsigned)(blocks < 8192 ? (blocks ? blocks : 1) : 8192);
}

}  // namespace

hipError_t launch_frame_input(const void *in, void *in_framed, int B, int Cin, int N, int q, int Ns, kst_dtype dt,
                              hipStream_t stream)
{
    const unsigned planes = (unsigned)B * (unsigned)Cin;
    const size_t total = (size_t)planes * (N + 2 * q) * Ns;
    const bool small = total + (size_t)8192 * 256 < 0xffffffffu;      // the grid-stride index stays inside 32 bits
    if (is16(dt)) {
        if (small)
            hipLaunchKernelGGL((frame_input_kernel<uint16_t, unsigned>), dim3(grid_for(total)), dim3(256), 0, stream,
                               (const uint16_t *)in, (uint16_t *)in_framed, planes, N, q, Ns);
        else
            hipLaunchKernelGGL((frame_input_kernel<uint16_t, size_t>), dim3(grid_for(total)), dim3(256), 0, stream,
                               (const uint16_t *)in, (uint16_t *)in_framed, planes, N, q, Ns);
    } else {
        if (small)
            hipLaunchKernelGGL((frame_input_kernel<float, unsigned>), dim3(grid_for(total)), dim3(256), 0, stream,
                               (const float *)in, (float *)in_framed, planes, N, q, Ns);
        else
            hipLaunchKernelGGL((frame_input_kernel<float, size_t>), dim3(grid_for(total)), dim3(256), 0, stream,
                               (const float *)in, (float *)in_framed, planes, N, q, Ns);
    }
    return hipGetLastError();
}

hipError_t launch_widen(const void *src, float *dst, size_t elems, kst_dtype dt, hipStream_t stream)
{
    if (dt == KST_BF16)
        hipLaunchKernelGGL(widen_kernel<uint16_t>, dim3(grid_for(elems)), dim3(256), 0, stream, (const uint16_t *)src, dst,
                           elems);
    else if (dt == KST_F16)
        hipLaunchKernelGGL(widen_kernel<half_bits>, dim3(grid_for(elems)), dim3(256), 0, stream, (const half_bits *)src, dst,
                           elems);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_crop(const float *wide, float *out, int B, int Cout, int M, int q, hipStream_t stream)
{
    const unsigned planes = (unsigned)B * (unsigned)Cout;
    const size_t total = (size_t)planes * M * M;
    hipLaunchKernelGGL(crop_kernel, dim3(grid_for(total)), dim3(256), 0, stream, wide, out, planes, M, q);
    return hipGetLastError();
}

}  // namespace kst
