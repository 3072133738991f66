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

hipError_t launch_segregate(const void *w, void *w_seg, int Cin, int Cout, int n, kst_dtype dt,
                            hipStream_t stream)
{
    SegGeom g;
    g.Cin = Cin;
    g.Cout = Cout;
    g.n = n;
    g.group = dt == KST_BF16 ? 8 : 1;
    g.cin_pad = (int)seg_cin_padded(Cin, dt);
    for (int p = 0; p < 4; ++p) {
        g.off[p] = (unsigned)seg_offset(Cin, Cout, n, p, dt);
        g.Tb[p] = taps_for_parity(n, p & 1);
        g.T[p] = class_taps(n, p);
    }
    g.off[4] = (unsigned)seg_elems(Cin, Cout, n, dt);
    const unsigned blocks = (g.off[4] + 255u) / 256u;
    if (dt == KST_BF16)
        hipLaunchKernelGGL(segregate_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream,
                           (const uint16_t *)w, (uint16_t *)w_seg, g);
    else
        hipLaunchKernelGGL(segregate_kernel<float>, dim3(blocks), dim3(256), 0, stream,
                           (const float *)w, (float *)w_seg, g);
    return hipGetLastError();
}

}  // namespace kst
