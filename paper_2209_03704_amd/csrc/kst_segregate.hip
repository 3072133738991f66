// Weight pre-segregation (Section 3.2): K -> K1..K4 by (row, column) parity,
// written in the reduction-major layouts that kst.h documents.
#include "kst_internal.h"

namespace kst {

struct SegGeom {
    int Cin, Cout, n;
    int cin_pad;           // Cin rounded up to the layout's channel group (1 or 8)
    int group;             // 1 (fp32) or 8 (bf16)
    unsigned off[5];       // element offset of class p; off[4] = total
    int Tb[4];             // columns of sub-kernel p
    int T[4];              // taps of sub-kernel p
};

// One thread per element of the segregated buffer: coalesced writes, gathered reads.
template <typename T>
__global__ void __launch_bounds__(256) segregate_kernel(const T *__restrict__ w, T *__restrict__ w_seg, SegGeom g)
{
    const unsigned e = blockIdx.x * 256u + threadIdx.x;
    if (e >= g.off[4]) return;
    int p = 0;
    while (p < 3 && e >= g.off[p + 1]) ++p;
    const int Tp = g.T[p];
    if (Tp == 0) return;   // empty class (n = 1): occupies no elements, unreachable
    unsigned ep = e - g.off[p];
    const int c_lo = (int)(ep % (unsigned)g.group);
    ep /= (unsigned)g.group;
    const int co = (int)(ep % (unsigned)g.Cout);
    ep /= (unsigned)g.Cout;
    const int t = (int)(ep % (unsigned)Tp);
    const int c_hi = (int)(ep / (unsigned)Tp);
    const int ci = c_hi * g.group + c_lo;
    const int a = t / g.Tb[p], b = t % g.Tb[p];
    const int u = 2 * a + (p >> 1), v = 2 * b + (p & 1);
    T val = T(0);
    if (ci < g.Cin) val = w[(((size_t)co * g.Cin + ci) * g.n + u) * g.n + v];
    w_seg[e] = val;
}

// fp32 weights of many-channel layers: the permutation is a transpose (w has the output channel
// slowest, the segregated layout has it fastest), done through LDS so that both sides are
// coalesced.  A workgroup takes 64 output channels x a run of S_RUN consecutive floats of
// w[co][.] (whole input channels' kernels are not required: a run element is decoded on its own),
// reads each channel's run as it lies in memory and writes, for every run element, the 64
// output channels side by side.
constexpr int S_CO = 64;
constexpr int S_RUN = 64;

// VEC: a channel's floats in w are a multiple of 4, so runs are read as 16-byte groups (all of a
// lane's loads in flight at once).
template <bool VEC>
__global__ void __launch_bounds__(256) segregate_tiled_f32_kernel(const float *__restrict__ w, float *__restrict__ w_seg,
                                                                  SegGeom g)
{
    __shared__ float tile[S_CO][S_RUN + 1];
    const unsigned per_co = (unsigned)g.Cin * g.n * g.n;          // floats of one output channel in w
    const unsigned runs = (per_co + S_RUN - 1) / S_RUN;
    const unsigned run = blockIdx.x % runs, co0 = (blockIdx.x / runs) * S_CO;
    const unsigned r0 = run * S_RUN;
    const int tid = threadIdx.x;
    if constexpr (VEC) {
        constexpr int G = S_RUN / 4, PER = S_CO * G / 256;        // 16-byte groups per row / per lane
        float4 v[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int idx = tid + k * 256;
            const unsigned co_l = idx / G, r = 4 * (idx % G);
            v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (co0 + co_l < (unsigned)g.Cout && r0 + r < per_co)
                v[k] = *reinterpret_cast<const float4 *>(w + (size_t)(co0 + co_l) * per_co + r0 + r);
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int idx = tid + k * 256;
            const unsigned co_l = idx / G, r = 4 * (idx % G);
            tile[co_l][r] = v[k].x;
            tile[co_l][r + 1] = v[k].y;
            tile[co_l][r + 2] = v[k].z;
            tile[co_l][r + 3] = v[k].w;
        }
    } else {
        for (int idx = tid; idx < S_CO * S_RUN; idx += 256) {
            const unsigned co_l = idx / S_RUN, r = idx % S_RUN;
            float v = 0.0f;
            if (co0 + co_l < (unsigned)g.Cout && r0 + r < per_co) v = w[(size_t)(co0 + co_l) * per_co + r0 + r];
            tile[co_l][r] = v;
        }
    }
    __syncthreads();
    // A wave writes run element r = wave, wave + 4, ... for its 64 output channels (lane = channel).
    // The element's (ci, u, v) follow from those of the one before by a step of four with carries: one
    // division per wave, none per element (u = uv / n by a multiplication, exact for every uv < n * n with n <= 42).
    const unsigned nn = (unsigned)g.n * g.n;
    const unsigned co_l = (unsigned)tid & 63u;
    unsigned r = (unsigned)tid >> 6;
    unsigned e = r0 + r;
    unsigned ci = e / nn, uv = e - ci * nn;
    const unsigned magic = (65536u + (unsigned)g.n - 1u) / (unsigned)g.n;
    const bool co_ok = co0 + co_l < (unsigned)g.Cout;
    for (; r < (unsigned)S_RUN; r += 4, e += 4) {
        if (e < per_co && co_ok) {
            const unsigned u = (uv * magic) >> 16, v = uv - u * g.n;
            const int p = (int)((u & 1u) * 2u + (v & 1u));
            const unsigned t = (u >> 1) * g.Tb[p] + (v >> 1);
            w_seg[g.off[p] + ((size_t)ci * g.T[p] + t) * g.Cout + co0 + co_l] = tile[co_l][r];
        }
        uv += 4;
        while (uv >= nn) { uv -= nn; ++ci; }
    }
}

hipError_t launch_segregate(const void *w, void *w_seg, int Cin, int Cout, int n, kst_dtype dt,
                            hipStream_t stream)
{
    SegGeom g;
    g.Cin = Cin;
    g.Cout = Cout;
    g.n = n;
    g.group = is16(dt) ? 8 : 1;
    g.cin_pad = (int)seg_cin_padded(Cin, dt);
    for (int p = 0; p < 4; ++p) {
        g.off[p] = (unsigned)seg_offset(Cin, Cout, n, p, dt);
        g.Tb[p] = taps_for_parity(n, p & 1);
        g.T[p] = class_taps(n, p);
    }
    g.off[4] = (unsigned)seg_elems(Cin, Cout, n, dt);
    const unsigned blocks = (g.off[4] + 255u) / 256u;
    if (dt == KST_F32 && Cout >= 32 && n <= 32 && (size_t)Cin * n * n >= 64) {     // (n <= 32: the tiled kernel's division by n)
        const size_t runs = ((size_t)Cin * n * n + S_RUN - 1) / S_RUN;
        const size_t tiles = runs * ((Cout + S_CO - 1) / S_CO);
        if (tiles < 0x7fffffffu) {
            if (((size_t)Cin * n * n) % 4 == 0)
                hipLaunchKernelGGL(segregate_tiled_f32_kernel<true>, dim3((unsigned)tiles), dim3(256), 0, stream,
                                   (const float *)w, (float *)w_seg, g);
            else
                hipLaunchKernelGGL(segregate_tiled_f32_kernel<false>, dim3((unsigned)tiles), dim3(256), 0, stream,
                                   (const float *)w, (float *)w_seg, g);
            return hipGetLastError();
        }
    }
    if (is16(dt))
        hipLaunchKernelGGL(segregate_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream,
                           (const uint16_t *)w, (uint16_t *)w_seg, g);
    else
        hipLaunchKernelGGL(segregate_kernel<float>, dim3(blocks), dim3(256), 0, stream,
                           (const float *)w, (float *)w_seg, g);
    return hipGetLastError();
}

}  // namespace kst
