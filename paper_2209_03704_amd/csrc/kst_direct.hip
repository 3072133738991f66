// Direct (bandwidth-bound) segregated forward pass, Section 3.3, Eqs. 7-10.
//
// One lane owns one output quad (2i..2i+1, 2j..2j+1): the four parity
// sub-kernels K1..K4 read the same (fl+1) x (fl+1) window of the ORIGINAL
// input (fl = floor(n/2)), so the window is fetched once from an LDS tile and
// feeds all n*n multiply-adds of the quad.  Nothing is up-sampled.
//
// For odd M the last quad row / column has no odd member (Section 3.3's extra
// row and column): those stores are suppressed, and the input indices a
// phantom member would read still lie inside the map, so loads need no mask
// beyond the tile edge.
#include "kst_internal.h"

namespace kst {

template <typename T>
__device__ __forceinline__ size_t wseg_index(size_t off_p, int Tp, int Cout, int ci, int t, int co)
{
    if constexpr (sizeof(T) == 2)
        return off_p + ((((size_t)(ci >> 3)) * Tp + t) * Cout + co) * 8 + (ci & 7);
    else
        return off_p + ((size_t)ci * Tp + t) * Cout + co;
}

struct DirectParams {
    int B, Cin, Cout, N, M, E;
    int tiles_x, tiles_y;
    unsigned off[4];   // element offset of W_p in the segregated buffer
};

constexpr int D_TJ = 64;                 // quad columns per tile = lanes of a wave
constexpr int D_WAVES = 4;
constexpr int D_RPT = 2;                 // quad rows per lane
constexpr int D_TI = D_WAVES * D_RPT;    // quad rows per tile

template <int n, typename T>
__global__ void __launch_bounds__(256) direct_kernel(const T *__restrict__ in, const T *__restrict__ w_seg,
                                                       float *__restrict__ out, DirectParams p)
{
    constexpr int fl = n / 2;
    constexpr int H = D_TI + fl, W = D_TJ + fl;
    constexpr int Ta0 = (n + 1) / 2, Ta1 = n / 2;   // sub-kernel rows (= columns) for parity 0 / 1
    __shared__ float tile[H * W];

    unsigned id = blockIdx.x;
    const int tx = (int)(id % (unsigned)p.tiles_x);
    id /= (unsigned)p.tiles_x;
    const int ty = (int)(id % (unsigned)p.tiles_y);
    const int plane = (int)(id / (unsigned)p.tiles_y);
    const int b = plane / p.Cout, co = plane - b * p.Cout;
    const int i0 = ty * D_TI, j0 = tx * D_TJ;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    float acc[D_RPT][2][2];
#pragma unroll
    for (int q = 0; q < D_RPT; ++q)
        acc[q][0][0] = acc[q][0][1] = acc[q][1][0] = acc[q][1][1] = 0.0f;

    for (int ci = 0; ci < p.Cin; ++ci) {
        if (ci) __syncthreads();
        const T *src = in + ((size_t)b * p.Cin + ci) * p.N * p.N;
        for (int idx = threadIdx.x; idx < H * W; idx += 256) {
            const int y = idx / W, x = idx - y * W;
            const int gy = i0 + y, gx = j0 + x;
            float v = 0.0f;
            if (gy < p.N && gx < p.N) v = to_f32(src[(size_t)gy * p.N + gx]);
            tile[idx] = v;
        }
        __syncthreads();

        // The n*n weights of (co, ci), sub-kernel by sub-kernel: uniform across the workgroup.
        float wk[2][2][Ta0 * Ta0 > 0 ? Ta0 * Ta0 : 1];
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int Ta = r ? Ta1 : Ta0, Tb = s ? Ta1 : Ta0;
#pragma unroll
                for (int t = 0; t < Ta * Tb; ++t)
                    wk[r][s][t] = to_f32(w_seg[wseg_index<T>(p.off[2 * r + s], Ta * Tb, p.Cout, ci, t, co)]);
            }

        // Window rows shared by the lane's D_RPT vertically adjacent quads.
        float win[D_RPT + fl][fl + 1];
#pragma unroll
        for (int y = 0; y < D_RPT + fl; ++y)
#pragma unroll
            for (int x = 0; x <= fl; ++x)
                win[y][x] = tile[(wave * D_RPT + y) * W + lane + x];

#pragma unroll
        for (int q = 0; q < D_RPT; ++q)
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int Ta = r ? Ta1 : Ta0, Tb = s ? Ta1 : Ta0;
                    float a = acc[q][r][s];
#pragma unroll
                    for (int u = 0; u < Ta; ++u)
#pragma unroll
                        for (int v = 0; v < Tb; ++v)
                            a = fmaf(win[q + r + u][s + v], wk[r][s][u * Tb + v], a);
                    acc[q][r][s] = a;
                }
    }

    const int gj = j0 + lane;
    const int x = 2 * gj;
    if (x >= p.M) return;
#pragma unroll
    for (int q = 0; q < D_RPT; ++q)
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int y = 2 * (i0 + wave * D_RPT + q) + r;
            if (y >= p.M) continue;
            float *o = out + ((size_t)plane * p.M + y) * p.M + x;
            if (x + 1 < p.M) {
                if ((reinterpret_cast<uintptr_t>(o) & 7u) == 0) {
                    *reinterpret_cast<float2 *>(o) = make_float2(acc[q][r][0], acc[q][r][1]);
                } else {
                    o[0] = acc[q][r][0];
                    o[1] = acc[q][r][1];
                }
            } else {
                o[0] = acc[q][r][0];
            }
        }
}

// Any kernel size: one lane per quad, operands read straight from global memory.
template <typename T>
__global__ void __launch_bounds__(256) direct_generic_kernel(const T *__restrict__ in, const T *__restrict__ w_seg,
                                                               float *__restrict__ out, DirectParams p, int n)
{
    const size_t q = (size_t)blockIdx.x * 256u + threadIdx.x;
    const size_t quads = (size_t)p.B * p.Cout * p.E * p.E;
    if (q >= quads) return;
    const int j = (int)(q % (unsigned)p.E);
    size_t rest = q / (unsigned)p.E;
    const int i = (int)(rest % (unsigned)p.E);
    const int plane = (int)(rest / (unsigned)p.E);
    const int b = plane / p.Cout, co = plane - b * p.Cout;
    for (int r = 0; r < 2; ++r)
        for (int s = 0; s < 2; ++s) {
            const int y = 2 * i + r, x = 2 * j + s;
            if (y >= p.M || x >= p.M) continue;
            const int Ta = taps_for_parity(n, r), Tb = taps_for_parity(n, s);
            float a = 0.0f;
            for (int ci = 0; ci < p.Cin; ++ci) {
                const T *src = in + (((size_t)b * p.Cin + ci) * p.N + (i + r)) * p.N + (j + s);
                for (int u = 0; u < Ta; ++u)
                    for (int v = 0; v < Tb; ++v)
                        a = fmaf(to_f32(src[(size_t)u * p.N + v]),
                                 to_f32(w_seg[wseg_index<T>(p.off[2 * r + s], Ta * Tb, p.Cout, ci, u * Tb + v, co)]), a);
            }
            out[((size_t)plane * p.M + y) * p.M + x] = a;
        }
}

template <int n, typename T>
static void launch_tiled(const T *in, const T *w_seg, float *out, const DirectParams &p, unsigned blocks,
                         hipStream_t stream)
{
    hipLaunchKernelGGL((direct_kernel<n, T>), dim3(blocks), dim3(256), 0, stream, in, w_seg, out, p);
}

template <typename T>
static hipError_t run(const T *in, const T *w_seg, float *out, const Shape &s, kst_dtype dt, hipStream_t stream)
{
    DirectParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.N = s.N; p.M = s.M; p.E = s.E;
    p.tiles_x = (s.E + D_TJ - 1) / D_TJ;
    p.tiles_y = (s.E + D_TI - 1) / D_TI;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, dt);
    const size_t blocks = (size_t)s.B * s.Cout * p.tiles_x * p.tiles_y;
    if (s.n <= 7 && blocks < 0x7fffffffu) {
        const unsigned nb = (unsigned)blocks;
        switch (s.n) {
            case 1: launch_tiled<1, T>(in, w_seg, out, p, nb, stream); break;
            case 2: launch_tiled<2, T>(in, w_seg, out, p, nb, stream); break;
            case 3: launch_tiled<3, T>(in, w_seg, out, p, nb, stream); break;
            case 4: launch_tiled<4, T>(in, w_seg, out, p, nb, stream); break;
            case 5: launch_tiled<5, T>(in, w_seg, out, p, nb, stream); break;
            case 6: launch_tiled<6, T>(in, w_seg, out, p, nb, stream); break;
            default: launch_tiled<7, T>(in, w_seg, out, p, nb, stream); break;
        }
    } else {
        const size_t quads = (size_t)s.B * s.Cout * s.E * s.E;
        hipLaunchKernelGGL(direct_generic_kernel<T>, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream,
                           in, w_seg, out, p, s.n);
    }
    return hipGetLastError();
}

hipError_t launch_direct(const void *in, const void *w_seg, float *out, const Shape &s, kst_dtype dt,
                         hipStream_t stream)
{
    if (dt == KST_BF16) return run<uint16_t>((const uint16_t *)in, (const uint16_t *)w_seg, out, s, dt, stream);
    return run<float>((const float *)in, (const float *)w_seg, out, s, dt, stream);
}

}  // namespace kst
