// Direct segregated forward pass for layers with several input channels and few output channels
// (Section 3.3, Eqs. 7-10 with the sum over input channels; the last layer of the GAN generators
// of Table 3 and the 3-channel image layers of Tables 1-2 have this shape).
//
// One lane owns one output quad (2i..2i+1, 2j..2j+1) of CO output channels (CO <= 4) for the whole
// reduction: 4 * CO accumulators.  A workgroup covers a tile of M_TI x M_TJ quads; the input window
// rows and the weights of M_KC channels at a time are staged in LDS (two stages: the loads of the
// next chunk are in flight in registers while the current one is multiplied, one barrier per
// chunk).  The (fl+1) x (fl+1) window a quad reads from LDS feeds the n*n*CO multiply-adds of its
// four classes and CO channels; the weights of a channel, the same for every lane, are read from
// LDS as whole 16-byte groups (scalar loads were tried first: the n*n*CO values of a channel do not
// fit the scalar registers together with the next channel's, and with one or two waves per SIMD
// every channel then waited for several scalar-load round trips).
//
// Layers with many input channels and few tiles (the 128 -> 3 and 64 -> 3 output layers of the
// generators: one tile per CU at a batch of 64, four tiles in all for one sample) are bound by the
// latency of one chunk's loads per workgroup.  For them a workgroup is KS groups of M_THREADS
// lanes on the same tile: group g takes chunks g, g + KS, ... with staging buffers of its own, so
// that KS chunks are in flight per workgroup, and the groups' accumulators are added through LDS
// in group order at the end (a fixed order: results do not depend on timing).
#include "kst_internal.h"

namespace kst {
namespace {

constexpr int M_TJ = 32;                 // quad columns per tile
constexpr int M_TI = 8;                  // quad rows per tile
constexpr int M_THREADS = M_TI * M_TJ;

struct MultiParams {
    int B, Cin, Cout, M, E;
    int N0, q;                           // edge of the tensor in memory; zero frame around it (virtual)
    int crop;                            // 1: `out` is the interior of the M x M map (edge M - 2)
    int tiles_x, tiles_y;
    unsigned off[4];                     // element offset of W_p in the segregated buffer
    Epilogue epi;
};

template <typename T>
__device__ __forceinline__ size_t wseg_at(size_t off_p, int Tp, int Cout, int ci, int t, int co)
{
    if constexpr (sizeof(T) == 2)
        return off_p + ((((size_t)(ci >> 3)) * Tp + t) * Cout + co) * 8 + (ci & 7);
    else
        return off_p + ((size_t)ci * Tp + t) * Cout + co;
}

// M_KC: input channels per chunk (8, or 4 for layers with at most 4 input channels); KS: groups of
// lanes that share the reduction of a tile.
template <int n, int CO, int M_KC, int KS, typename T>
__global__ void __launch_bounds__(M_THREADS * KS) direct_multi_kernel(const T *__restrict__ in, const T *__restrict__ w_seg,
                                                                       float *__restrict__ out, MultiParams p)
{
    constexpr int fl = n / 2;
    constexpr int XH = M_TI + fl, XW = M_TJ + fl;              // staged rows and columns per channel
    constexpr int PLANE = XH * XW;
    constexpr int CHUNK = M_KC * PLANE;                        // staged elements per chunk
    constexpr int NLD = (CHUNK + M_THREADS - 1) / M_THREADS;   // ... per lane
    constexpr int Ta0 = (n + 1) / 2, Ta1 = n / 2;
    constexpr int NN = n * n;
    constexpr int WPC = (NN * CO + 3) & ~3;                    // staged weights per channel: [tap][k], padded
    constexpr int WCHUNK = M_KC * WPC;
    constexpr int NWL = (WCHUNK + M_THREADS - 1) / M_THREADS;  // ... per lane
    static_assert(CHUNK % 4 == 0 && WCHUNK % 4 == 0, "stages keep 16-byte alignment");
    constexpr int GROUP_FLOATS = 2 * (CHUNK + WCHUNK);         // one group's two stages
    static_assert(KS == 1 || 4 * CO * M_THREADS <= GROUP_FLOATS, "a group's accumulators fit its stages");
    extern __shared__ __attribute__((aligned(16))) float multi_lds[];
    const int grp = KS == 1 ? 0 : (int)threadIdx.x / M_THREADS;       // uniform over a wave
    float(*Xs)[CHUNK] = reinterpret_cast<float(*)[CHUNK]>(multi_lds + grp * GROUP_FLOATS);
    float(*Wsh)[WCHUNK] = reinterpret_cast<float(*)[WCHUNK]>(multi_lds + grp * GROUP_FLOATS + 2 * CHUNK);

    unsigned id = blockIdx.x;
    const int co_groups = p.Cout / CO;              // CO divides Cout
    const int co0 = (int)(id % (unsigned)co_groups) * CO;
    id /= (unsigned)co_groups;
    const int tx = (int)(id % (unsigned)p.tiles_x);
    id /= (unsigned)p.tiles_x;
    const int ty = (int)(id % (unsigned)p.tiles_y);
    const int b = (int)(id / (unsigned)p.tiles_y);

    const int tid = KS == 1 ? (int)threadIdx.x : (int)threadIdx.x - grp * M_THREADS;   // lane within its group
    const int ti = tid / M_TJ, tj = tid - ti * M_TJ;
    const int i0 = ty * M_TI, j0 = tx * M_TJ;
    const int i = i0 + ti, j = j0 + tj;

    // Staging plan: element e = tid + k * M_THREADS of a chunk is (channel c, row, column) of the
    // window; off[k] is its place in the first chunk, or ~0 when it lies outside the map (then
    // the LDS cell is written as zero: it belongs to the zero frame of a padded layer, or only
    // phantom quads past the edge read it).
    unsigned ld_off[NLD];
    int ld_c[NLD];
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
        const int e = tid + k * M_THREADS;
        const int c = e / PLANE;
        const int rem = e - c * PLANE;
        const int row = rem / XW, col = rem - row * XW;
        const int y = i0 + row - p.q, xx = j0 + col - p.q;     // in the tensor as it lies in memory
        const bool ok = e < CHUNK && y >= 0 && y < p.N0 && xx >= 0 && xx < p.N0;
        ld_off[k] = ok ? (((unsigned)b * p.Cin + grp * M_KC + c) * p.N0 + y) * p.N0 + xx : ~0u;
        ld_c[k] = c;
    }
    const unsigned ld_inc = (unsigned)(M_KC * KS) * p.N0 * p.N0;

    // Weights: element e of a chunk is (channel c, tap t in class-major order, output channel k).
    unsigned w_off[NWL], w_inc[NWL];
    int w_c[NWL];
#pragma unroll
    for (int k = 0; k < NWL; ++k) {
        const int e = tid + k * M_THREADS;
        const int c = e / WPC;
        const int rem = e - c * WPC;
        const int t = rem / CO, kk = rem - t * CO;
        const bool ok = e < WCHUNK && t < NN;
        int cls = 0;
#pragma unroll
        for (int q = 1; q < 4; ++q)
            if (t >= class_tap_base(n, q) && class_taps(n, q) > 0) cls = q;
        const int Tp = cls == 0 ? class_taps(n, 0) : cls == 1 ? class_taps(n, 1) : cls == 2 ? class_taps(n, 2) : class_taps(n, 3);
        const int tb = cls == 0 ? 0 : cls == 1 ? class_tap_base(n, 1) : cls == 2 ? class_tap_base(n, 2) : class_tap_base(n, 3);
        w_off[k] = ok ? (unsigned)wseg_at<T>(p.off[cls], Tp, p.Cout, grp * M_KC + c, t - tb, co0 + kk) : ~0u;
        w_inc[k] = (unsigned)(M_KC * KS) * Tp * p.Cout;
        w_c[k] = c;
    }

    float pre[NLD], wpre[NWL];
    auto fetch = [&](int ci0) {
#pragma unroll
        for (int k = 0; k < NWL; ++k) {
            float v = 0.f;
            if (w_off[k] != ~0u) {
                if (ci0 + w_c[k] < p.Cin) v = to_f32(w_seg[w_off[k]]);
                w_off[k] += w_inc[k];
            }
            wpre[k] = v;
        }
#pragma unroll
        for (int k = 0; k < NLD; ++k) {
            float v = 0.f;
            if (ld_off[k] != ~0u) {
                if (ci0 + ld_c[k] < p.Cin) v = to_f32(in[ld_off[k]]);
                ld_off[k] += ld_inc;
            }
            pre[k] = v;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int k = 0; k < NLD; ++k)
            if ((k + 1) * M_THREADS <= CHUNK || tid + k * M_THREADS < CHUNK) Xs[buf][tid + k * M_THREADS] = pre[k];
#pragma unroll
        for (int k = 0; k < NWL; ++k)
            if ((k + 1) * M_THREADS <= WCHUNK || tid + k * M_THREADS < WCHUNK) Wsh[buf][tid + k * M_THREADS] = wpre[k];
    };

    float acc[CO][2][2];
#pragma unroll
    for (int k = 0; k < CO; ++k)
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int s = 0; s < 2; ++s) acc[k][r][s] = 0.f;
    // Every group makes the same number of rounds (and meets the same barriers); a group whose
    // chunk lies past the last channel stages zeros and multiplies nothing.
    const int rounds = (p.Cin + M_KC * KS - 1) / (M_KC * KS);
    fetch(grp * M_KC);
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int round = 0; round < rounds; ++round) {
        const int ci0 = (round * KS + grp) * M_KC;
        const bool more = round + 1 < rounds;                   // uniform over the workgroup
        if (more) fetch(ci0 + M_KC * KS);
        const float *X = &Xs[buf][ti * XW + tj];
#pragma unroll
        for (int c = 0; c < M_KC; ++c) {
            const int ci = ci0 + c;
            if (ci >= p.Cin) break;                             // uniform
            float x[fl + 1][fl + 1];
#pragma unroll
            for (int dy = 0; dy <= fl; ++dy)
#pragma unroll
                for (int dx = 0; dx <= fl; ++dx) x[dy][dx] = X[c * PLANE + dy * XW + dx];
            // This channel's weights: the same address for every lane, 16 bytes at a time.
            float wv[WPC];
#pragma unroll
            for (int g4 = 0; g4 < WPC / 4; ++g4) {
                const float4 v = *reinterpret_cast<const float4 *>(&Wsh[buf][c * WPC + 4 * g4]);
                wv[4 * g4] = v.x;
                wv[4 * g4 + 1] = v.y;
                wv[4 * g4 + 2] = v.z;
                wv[4 * g4 + 3] = v.w;
            }
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int Ta = r ? Ta1 : Ta0, Tb = s ? Ta1 : Ta0;
                    const int tb = class_tap_base(n, 2 * r + s);
#pragma unroll
                    for (int u = 0; u < Ta; ++u)
#pragma unroll
                        for (int v = 0; v < Tb; ++v)
#pragma unroll
                            for (int k = 0; k < CO; ++k)
                                acc[k][r][s] = fmaf(x[r + u][s + v], wv[(tb + u * Tb + v) * CO + k], acc[k][r][s]);
                }
        }
        if (!more) break;
        stage(buf ^ 1);          // the other stage was last read before the previous barrier
        __syncthreads();
        buf ^= 1;
    }

    if constexpr (KS > 1) {
        // Add the groups' accumulators in group order: group g leaves its 4 * CO values per lane
        // in its own (now idle) stages, group 0 collects.
        __syncthreads();                                        // the last stage has been read by all
        float *mine = multi_lds + grp * GROUP_FLOATS;
        if (grp != 0) {
#pragma unroll
            for (int k = 0; k < CO; ++k)
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) mine[((k * 2 + r) * 2 + s2) * M_THREADS + tid] = acc[k][r][s2];
        }
        __syncthreads();
        if (grp != 0) return;
#pragma unroll
        for (int g = 1; g < KS; ++g)
#pragma unroll
            for (int k = 0; k < CO; ++k)
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2)
                        acc[k][r][s2] += multi_lds[g * GROUP_FLOATS + ((k * 2 + r) * 2 + s2) * M_THREADS + tid];
    }
    if (i >= p.E || j >= p.E) return;
    if (epi_on(p.epi)) {                                        // uniform
#pragma unroll
        for (int k = 0; k < CO; ++k) {
            const float bias = epi_bias(p.epi, co0 + k);
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) acc[k][r][s2] = epi_apply(acc[k][r][s2], bias, p.epi.act);
        }
    }
    if (p.crop) {
        // Odd padding factor: only the interior of the map is wanted, and `out` holds just that:
        // element (y, x) of the map is element (y - 1, x - 1) of `out` (edge M - 2).  Seen from `out`
        // the quads start on odd rows and columns: its even rows take the sub-kernels of the odd
        // row parity and the other way round (Fig. 7's swap of roles).
        const int Mo = p.M - 2;
#pragma unroll
        for (int k = 0; k < CO; ++k) {
            float *plane = out + ((size_t)b * p.Cout + co0 + k) * Mo * Mo;
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const int y = 2 * i + r - 1, x = 2 * j + s2 - 1;
                    if (y >= 0 && y < Mo && x >= 0 && x < Mo) plane[(size_t)y * Mo + x] = acc[k][r][s2];
                }
        }
        return;
    }
    const bool x1 = 2 * j + 1 < p.M;
#pragma unroll
    for (int k = 0; k < CO; ++k) {
        float *plane = out + ((size_t)b * p.Cout + co0 + k) * p.M * p.M;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int y = 2 * i + r;
            if (y >= p.M) continue;
            float *q = plane + (size_t)y * p.M + 2 * j;
            if (x1) {
                if ((reinterpret_cast<uintptr_t>(q) & 7u) == 0) {
                    *reinterpret_cast<float2 *>(q) = make_float2(acc[k][r][0], acc[k][r][1]);
                } else {
                    q[0] = acc[k][r][0];
                    q[1] = acc[k][r][1];
                }
            } else {
                q[0] = acc[k][r][0];
            }
        }
    }
}

// Output channels per lane: all of them up to four, else the largest of 4, 3, 2, 1 that divides
// Cout (a lane's channels are then always whole groups).
inline int co_per_lane(int Cout)
{
    if (Cout <= 4) return Cout;
    return Cout % 4 == 0 ? 4 : Cout % 3 == 0 ? 3 : Cout % 2 == 0 ? 2 : 1;
}

// Lane groups per workgroup: several when the tiles alone leave most of the chip's load slots
// empty and there are enough chunks to share (kernels up to 5 x 5: the larger ones need the
// registers a 1024-lane workgroup does not have).
inline int lane_groups(int n, size_t blocks, int Cin)
{
    if (n > 5 || blocks >= 1024) return 1;
    if (Cin >= 64) return 4;
    return Cin >= 32 ? 2 : 1;
}

template <int n, int CO, int M_KC, int KS, typename T>
hipError_t launch_ks(const T *in, const T *w_seg, float *out, const MultiParams &p, unsigned blocks, hipStream_t stream)
{
    constexpr int fl = n / 2;
    constexpr size_t lds = (size_t)KS * 2 * ((size_t)M_KC * (M_TI + fl) * (M_TJ + fl) + (size_t)M_KC * ((n * n * CO + 3) & ~3)) *
                           sizeof(float);
    static_assert(lds <= 160 * 1024, "stages fit the LDS of a CU");
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&direct_multi_kernel<n, CO, M_KC, KS, T>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((direct_multi_kernel<n, CO, M_KC, KS, T>), dim3(blocks), dim3(M_THREADS * KS), lds, stream, in,
                       w_seg, out, p);
    return hipGetLastError();
}

template <int n, int CO, typename T>
hipError_t launch_co(const T *in, const T *w_seg, float *out, const MultiParams &p, hipStream_t stream)
{
    const size_t blocks_l = (size_t)p.B * (p.Cout / CO) * p.tiles_x * p.tiles_y;
    const unsigned blocks = (unsigned)blocks_l;
    // (bf16 weights are stored in groups of 8 input channels: chunks of 8 only.)
    if (p.Cin <= 4 && sizeof(T) == 4) return launch_ks<n, CO, 4, 1, T>(in, w_seg, out, p, blocks, stream);
    if constexpr (n <= 5) {
        const int ks = lane_groups(n, blocks_l, p.Cin);
        // Four groups are 1024 lanes with 128 registers each: enough for up to 50 weights per channel.
        if constexpr (n * n * CO <= 50)
            if (ks == 4) return launch_ks<n, CO, 8, 4, T>(in, w_seg, out, p, blocks, stream);
        if (ks >= 2) return launch_ks<n, CO, 8, 2, T>(in, w_seg, out, p, blocks, stream);
    }
    return launch_ks<n, CO, 8, 1, T>(in, w_seg, out, p, blocks, stream);
}

template <int n, typename T>
hipError_t launch_n(const T *in, const T *w_seg, float *out, const MultiParams &p, hipStream_t stream)
{
    switch (co_per_lane(p.Cout)) {
        case 1: return launch_co<n, 1, T>(in, w_seg, out, p, stream);
        case 2: return launch_co<n, 2, T>(in, w_seg, out, p, stream);
        case 3: return launch_co<n, 3, T>(in, w_seg, out, p, stream);
        default: return launch_co<n, 4, T>(in, w_seg, out, p, stream);
    }
}

template <typename T>
hipError_t launch_t(const T *in, const T *w_seg, float *out, const Shape &s, kst_dtype dt, hipStream_t stream)
{
    MultiParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.M = s.M; p.E = s.E;
    p.q = s.frame;
    p.crop = s.crop;
    p.N0 = s.N - 2 * s.frame;
    p.tiles_x = (s.E + M_TJ - 1) / M_TJ;
    p.tiles_y = (s.E + M_TI - 1) / M_TI;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, dt);
    p.epi = s.epi;
    switch (s.n) {
        case 1: return launch_n<1, T>(in, w_seg, out, p, stream);
        case 2: return launch_n<2, T>(in, w_seg, out, p, stream);
        case 3: return launch_n<3, T>(in, w_seg, out, p, stream);
        case 4: return launch_n<4, T>(in, w_seg, out, p, stream);
        case 5: return launch_n<5, T>(in, w_seg, out, p, stream);
        case 6: return launch_n<6, T>(in, w_seg, out, p, stream);
        case 7: return launch_n<7, T>(in, w_seg, out, p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool direct_multi_supported(const Shape &s)
{
    if (s.Cin < 2 || s.n < 1 || s.n > 7 || s.Ns != s.N) return false;
    const size_t tiles = (size_t)((s.E + M_TJ - 1) / M_TJ) * ((s.E + M_TI - 1) / M_TI);
    return (size_t)s.B * s.Cout * tiles < 0x7fffffffu && (size_t)s.Cin * s.Cout * s.n * s.n < 0x7fffffffu;
}

hipError_t launch_direct_multi(const void *in, const void *w_seg, float *out, const Shape &s, kst_dtype dt,
                               hipStream_t stream)
{
    if (!direct_multi_supported(s)) return hipErrorInvalidValue;
    if (dt == KST_BF16) return launch_t<uint16_t>((const uint16_t *)in, (const uint16_t *)w_seg, out, s, dt, stream);
    if (dt == KST_F16) return launch_t<half_bits>((const half_bits *)in, (const half_bits *)w_seg, out, s, dt, stream);
    return launch_t<float>((const float *)in, (const float *)w_seg, out, s, dt, stream);
}

}  // namespace kst
