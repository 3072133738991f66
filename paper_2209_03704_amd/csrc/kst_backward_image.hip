// Kernel gradient of layers with a handful of channels on large maps (the image layers of
// Tables 1-2: 3 -> 1 channels, 224 x 224), which is a reduction over half a gigabyte of `in` and
// `g` into a few dozen numbers: bound by how fast the two tensors stream in.
//
//   dw[co][ci][u][v] = sum over b, i, j of in[b][ci][i][j] * g[b][co][2 i + P - u][2 j + P - v]
//
// (end of Section 3.3; the products of the segregated forward pass read backwards: every one has
// an original input pixel, none an inserted or padded zero).
//
// A workgroup is persistent over strips of RB input rows of one batch item.  A strip's rows of
// all input channels and the 2 RB + n - 1 rows of g they meet are staged in LDS with coalesced
// loads (each element of both tensors is read once, apart from the g halo between strips); the
// g rows sit between zeroed margins of n - 1 - P columns so that taps beyond the map's edge
// need no test, and rows beyond its top or bottom are staged as zeros.  A lane walks positions
// (i, j) of the strip by a fixed step with a carry, keeps all n * n * Cin sums of its output
// channel in registers, reads an input value once for n * n products and a g value once for Cin;
// at the end the sums are added across the lanes by wave shuffles, across the waves through LDS,
// and every workgroup writes one partial result that the summing pass adds in a fixed order.
// Where a strip's loads fit a lane's registers (maps up to 512 wide) the next strip is fetched
// while this one is multiplied; wider maps stage strip after strip.  The input gradient of
// such layers with one output channel (second kernel below) runs on the same strips of g.
#include "kst_internal.h"

namespace kst {

namespace {

constexpr int BI_THREADS = 256;

struct ImageGradParams {
    int B, Cin, Cout, N0, M, P, n;
    int RB;                 // input rows per strip
    int strips_per_item;    // ceil(N0 / RB)
    int wgs;                // workgroups per output channel (= partial results)
    int GS;                 // floats per staged g row: the map's M between two margins of padc, rounded up to even;
                            // a row is stored as its even columns followed by its odd columns (see g_cell)
    int padc;               // max(0, n - 1 - P)
    int step_i, step_j;     // a lane's step through the positions: threads = step_i * N0 + step_j
    int pre;                // 1: a strip's loads fit a lane's registers (the prefetching variant)
};

// Geometry of a strip.
struct Strip {
    int b, i_lo, rows, y_lo, nrows;
};

template <int n>
__device__ __forceinline__ Strip strip_of(const ImageGradParams &p, int strip)
{
    Strip s;
    s.b = strip / p.strips_per_item;
    const int rblk = strip - s.b * p.strips_per_item;
    s.i_lo = rblk * p.RB;
    s.rows = min(p.RB, p.N0 - s.i_lo);
    s.y_lo = 2 * s.i_lo + p.P - (n - 1);                         // g row staged as row 0
    s.nrows = 2 * s.rows + n - 2;                                // y_lo .. 2 (i_lo + rows - 1) + P
    return s;
}

// Maps up to 512 wide and strips up to 2048 input elements per channel: a strip's loads all fit a lane's
// registers (a wave takes g rows wave, wave + 4, ..., a lane columns lane, lane + 64, ...), so the next
// strip is on its way from memory while this one is multiplied.
constexpr int BI_XK = 8;                                         // columns per lane and g row
constexpr int BI_XE = 8;                                         // input elements per lane and channel
template <int n>
constexpr int bi_rows_per_wave() { return (2 * 8 + n - 1 + 3) / 4; }

// Where column c (margin included) of a staged g row lies: the even columns first, then the odd
// ones.  A lane reads column c0 - v + 2 j for its position j, so with the two parities apart
// neighbouring lanes read neighbouring cells (in one interleaved row they would be two cells
// apart and half of the LDS banks would serve the whole wave).
__device__ __forceinline__ int g_cell(const ImageGradParams &p, int c) { return (c & 1) * (p.GS >> 1) + (c >> 1); }

template <int n>
__device__ __forceinline__ void g_rows_fetch(const ImageGradParams &p, const float *__restrict__ g, const Strip &st, int co,
                                             int tid, float (&gv)[bi_rows_per_wave<n>()][BI_XK])
{
    const int lane = tid & 63, wave = tid >> 6;
    const float *gp = g + ((size_t)st.b * p.Cout + co) * ((size_t)p.M * p.M);
#pragma unroll
    for (int k = 0; k < bi_rows_per_wave<n>(); ++k) {
        const int r = wave + 4 * k, y = st.y_lo + r;
        const bool row_ok = r < st.nrows && y >= 0 && y < p.M;   // uniform over the wave
        const float *grow = gp + (size_t)(row_ok ? y : 0) * p.M;
#pragma unroll
        for (int m = 0; m < BI_XK; ++m) {
            const int x = lane + 64 * m;
            gv[k][m] = row_ok && x < p.M ? grow[x] : 0.0f;
        }
    }
}

template <int n>
__device__ __forceinline__ void g_rows_land(const ImageGradParams &p, float *gs, const Strip &st, int tid,
                                            const float (&gv)[bi_rows_per_wave<n>()][BI_XK])
{
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int k = 0; k < bi_rows_per_wave<n>(); ++k) {
        const int r = wave + 4 * k;
        if (r < st.nrows) {
            float *drow = gs + r * p.GS;
#pragma unroll
            for (int m = 0; m < BI_XK; ++m) {
                const int x = lane + 64 * m;
                if (x < p.M) drow[g_cell(p, p.padc + x)] = gv[k][m];
            }
        }
    }
}

template <int n, int CI, typename T>
__device__ __forceinline__ void strip_fetch(const ImageGradParams &p, const T *__restrict__ in, const float *__restrict__ g,
                                            const Strip &st, int co, int tid, float (&gv)[bi_rows_per_wave<n>()][BI_XK],
                                            float (&xv)[CI][BI_XE])
{
    g_rows_fetch<n>(p, g, st, co, tid, gv);
    const int cnt = st.rows * p.N0;
#pragma unroll
    for (int c = 0; c < CI; ++c) {
        const T *src = in + ((size_t)st.b * p.Cin + c) * ((size_t)p.N0 * p.N0) + (size_t)st.i_lo * p.N0;
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int e4 = tid + h * BI_THREADS;
                float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
                if (e4 < (cnt >> 2)) a = reinterpret_cast<const float4 *>(src)[e4];
                xv[c][4 * h] = a.x; xv[c][4 * h + 1] = a.y; xv[c][4 * h + 2] = a.z; xv[c][4 * h + 3] = a.w;
            }
        } else {
#pragma unroll
            for (int m = 0; m < BI_XE; ++m) {
                const int e = tid + m * BI_THREADS;
                xv[c][m] = e < cnt ? to_f32(src[e]) : 0.0f;
            }
        }
    }
}

template <int n, int CI, typename T>
__device__ __forceinline__ void strip_land(const ImageGradParams &p, float *gs, float *xs, const Strip &st, int tid,
                                           const float (&gv)[bi_rows_per_wave<n>()][BI_XK], const float (&xv)[CI][BI_XE])
{
    g_rows_land<n>(p, gs, st, tid, gv);
    const int cnt = st.rows * p.N0;
#pragma unroll
    for (int c = 0; c < CI; ++c) {
        float *d = xs + c * p.RB * p.N0;
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int e4 = tid + h * BI_THREADS;
                if (e4 < (cnt >> 2))
                    reinterpret_cast<float4 *>(d)[e4] = make_float4(xv[c][4 * h], xv[c][4 * h + 1], xv[c][4 * h + 2], xv[c][4 * h + 3]);
            }
        } else {
#pragma unroll
            for (int m = 0; m < BI_XE; ++m) {
                const int e = tid + m * BI_THREADS;
                if (e < cnt) d[e] = xv[c][m];
            }
        }
    }
}

// PRE: the register-prefetched staging above (the plan says when it fits).
template <int n, int CI, typename T, bool PRE>
__global__ void __launch_bounds__(BI_THREADS) backward_weight_image_kernel(const T *__restrict__ in,
                                                                            const float *__restrict__ g,
                                                                            float *__restrict__ dst, ImageGradParams p)
{
    constexpr int NN = n * n;
    constexpr int S = NN * CI;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int grows = 2 * p.RB + n - 1;
    float *gs = lds;                                // [grows][GS]
    float *xs = lds + ((grows * p.GS + 3) & ~3);    // [CI][RB * N0], 16-byte aligned
    __shared__ float red[BI_THREADS / 64][S];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int co = blockIdx.x % p.Cout, w = blockIdx.x / p.Cout;
    const size_t in_plane = (size_t)p.N0 * p.N0, g_plane = (size_t)p.M * p.M;

    float acc[CI][NN];
#pragma unroll
    for (int c = 0; c < CI; ++c)
#pragma unroll
        for (int t = 0; t < NN; ++t) acc[c][t] = 0.0f;

    // The margins are cells nobody writes again.
    for (int e = tid; e < grows * p.GS; e += BI_THREADS) gs[e] = 0.0f;

    // This lane's first position of a strip.
    const int i0 = tid / p.N0, j0 = tid - i0 * p.N0;
    // Column c0 - v + 2 j of a g row, for tap column v: cell po[v] + j.
    int po[n];
#pragma unroll
    for (int v = 0; v < n; ++v) po[v] = g_cell(p, p.padc + p.P - v);

    const int strips = p.B * p.strips_per_item;
    float gv[bi_rows_per_wave<n>()][BI_XK], xv[CI][BI_XE];       // PRE: the strip on its way
    if constexpr (PRE) {
        if (w < strips) strip_fetch<n, CI, T>(p, in, g, strip_of<n>(p, w), co, tid, gv, xv);
    }
    for (int strip = w; strip < strips; strip += p.wgs) {
        const Strip st = strip_of<n>(p, strip);
        const int b = st.b, i_lo = st.i_lo, rows = st.rows, y_lo = st.y_lo, nrows = st.nrows;
        __syncthreads();                                        // the strip before is done with LDS (and the margins are clear)
        if constexpr (PRE) {
            strip_land<n, CI, T>(p, gs, xs, st, tid, gv, xv);
            __syncthreads();
            if (strip + p.wgs < strips) strip_fetch<n, CI, T>(p, in, g, strip_of<n>(p, strip + p.wgs), co, tid, gv, xv);
        } else {
            // ---- g rows: a wave takes rows wave, wave + 4, ...; four loads in flight per lane ----------
            const float *gp = g + ((size_t)b * p.Cout + co) * g_plane;
            for (int r = wave; r < nrows; r += BI_THREADS / 64) {
                const int y = y_lo + r;
                const bool row_ok = y >= 0 && y < p.M;              // uniform over the wave
                const float *grow = gp + (size_t)(row_ok ? y : 0) * p.M;
                float *drow = gs + r * p.GS;
                for (int x0 = lane; x0 < p.M; x0 += 256) {
                    float v[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int x = x0 + 64 * k;
                        v[k] = row_ok && x < p.M ? grow[x] : 0.0f;
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int x = x0 + 64 * k;
                        if (x < p.M) drow[g_cell(p, p.padc + x)] = v[k];
                    }
                }
            }
            // ---- input rows of the strip: rows * N0 consecutive elements per channel -------------------
            const int cnt = rows * p.N0;
#pragma unroll
            for (int c = 0; c < CI; ++c) {
                const T *src = in + ((size_t)b * p.Cin + c) * in_plane + (size_t)i_lo * p.N0;
                float *d = xs + c * p.RB * p.N0;
                if constexpr (sizeof(T) == 4) {
                    // (N0 is a multiple of 4 for this kernel: 16-byte groups)
                    for (int e4 = tid; e4 < (cnt >> 2); e4 += 2 * BI_THREADS) {
                        const int e4b = e4 + BI_THREADS;
                        const float4 a = reinterpret_cast<const float4 *>(src)[e4];
                        float4 bq = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (e4b < (cnt >> 2)) bq = reinterpret_cast<const float4 *>(src)[e4b];
                        reinterpret_cast<float4 *>(d)[e4] = a;
                        if (e4b < (cnt >> 2)) reinterpret_cast<float4 *>(d)[e4b] = bq;
                    }
                } else {
                    for (int e = tid; e < cnt; e += BI_THREADS) d[e] = to_f32(src[e]);
                }
            }
            __syncthreads();
        }
        // ---- products: position (i, j) meets g rows 2 i + P - u, columns 2 j + P - v ----------------
        // In LDS: row 2 i_rel + (n - 1) - u, column padc + 2 j + P - v.
        int ir = i0, j = j0;
        while (ir < rows) {
            float xin[CI];
#pragma unroll
            for (int c = 0; c < CI; ++c) xin[c] = xs[c * p.RB * p.N0 + ir * p.N0 + j];
            const float *gw = gs + (2 * ir + (n - 1)) * p.GS + j;
#pragma unroll
            for (int u = 0; u < n; ++u)
#pragma unroll
                for (int v = 0; v < n; ++v) {
                    const float gval = gw[-u * p.GS + po[v]];
#pragma unroll
                    for (int c = 0; c < CI; ++c) acc[c][u * n + v] = fmaf(xin[c], gval, acc[c][u * n + v]);
                }
            ir += p.step_i;
            j += p.step_j;
            if (j >= p.N0) { j -= p.N0; ++ir; }
        }
    }

    // ---- the workgroup's sums -----------------------------------------------------------------
#pragma unroll
    for (int c = 0; c < CI; ++c)
#pragma unroll
        for (int t = 0; t < NN; ++t) {
            float v = acc[c][t];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
            if (lane == 0) red[wave][c * NN + t] = v;
        }
    __syncthreads();
    for (int i = tid; i < S; i += BI_THREADS) {
        const int c = i / NN, t = i - c * NN;
        const float sum = (red[0][i] + red[1][i]) + (red[2][i] + red[3][i]);
        dst[(size_t)w * p.Cout * p.Cin * NN + ((size_t)co * p.Cin + c) * NN + t] = sum;
    }
}

// Input gradient of the same layers with one output channel:
//
//   din[b][ci][i][j] = sum over u, v of g[b][0][2 i + P - u][2 j + P - v] * w[0][ci][u][v]
//
// The same strips and the same staged rows of g (the next strip's on their way while this one is
// multiplied); a lane computes its positions for all input channels from one window of g and
// stores them along the rows of din.  The kernels of all input channels sit in vector registers,
// read once from LDS (as scalar values they would not fit beside the bookkeeping).
template <int n, int CI, typename T>
__global__ void __launch_bounds__(BI_THREADS) backward_input_image_kernel(const float *__restrict__ g,
                                                                           const T *__restrict__ w, float *__restrict__ din,
                                                                           ImageGradParams p)
{
    constexpr int NN = n * n;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int grows = 2 * p.RB + n - 1;
    float *gs = lds;                                // [grows][GS]
    __shared__ float wl[CI * NN];
    const int tid = threadIdx.x;
    const size_t in_plane = (size_t)p.N0 * p.N0;

    for (int e = tid; e < grows * p.GS; e += BI_THREADS) gs[e] = 0.0f;
    for (int e = tid; e < CI * NN; e += BI_THREADS) wl[e] = to_f32(w[e]);       // w[0][ci][u][v]
    __syncthreads();
    float wk[CI][NN];
#pragma unroll
    for (int c = 0; c < CI; ++c)
#pragma unroll
        for (int t = 0; t < NN; ++t) wk[c][t] = wl[c * NN + t];

    const int i0 = tid / p.N0, j0 = tid - i0 * p.N0;
    // Column c0 - v + 2 j of a g row, for tap column v: cell po[v] + j.
    int po[n];
#pragma unroll
    for (int v = 0; v < n; ++v) po[v] = g_cell(p, p.padc + p.P - v);
    const int strips = p.B * p.strips_per_item;
    const int w0 = blockIdx.x;
    float gv[bi_rows_per_wave<n>()][BI_XK];
    if (w0 < strips) g_rows_fetch<n>(p, g, strip_of<n>(p, w0), 0, tid, gv);
    for (int strip = w0; strip < strips; strip += p.wgs) {
        const Strip st = strip_of<n>(p, strip);
        __syncthreads();                                        // the strip before is done with LDS
        g_rows_land<n>(p, gs, st, tid, gv);
        __syncthreads();
        if (strip + p.wgs < strips) g_rows_fetch<n>(p, g, strip_of<n>(p, strip + p.wgs), 0, tid, gv);
        float *dp = din + (size_t)st.b * p.Cin * in_plane + (size_t)st.i_lo * p.N0;
        int ir = i0, j = j0;
        while (ir < st.rows) {
            float acc[CI];
#pragma unroll
            for (int c = 0; c < CI; ++c) acc[c] = 0.0f;
            const float *gw = gs + (2 * ir + (n - 1)) * p.GS + j;
#pragma unroll
            for (int u = 0; u < n; ++u)
#pragma unroll
                for (int v = 0; v < n; ++v) {
                    const float gval = gw[-u * p.GS + po[v]];
#pragma unroll
                    for (int c = 0; c < CI; ++c) acc[c] = fmaf(gval, wk[c][u * n + v], acc[c]);
                }
#pragma unroll
            for (int c = 0; c < CI; ++c) dp[c * in_plane + (size_t)ir * p.N0 + j] = acc[c];
            ir += p.step_i;
            j += p.step_j;
            if (j >= p.N0) { j -= p.N0; ++ir; }
        }
    }
}

bool image_plan(const Shape &s, ImageGradParams &p, size_t &lds)
{
    const int N0 = s.N - 2 * s.frame;
    if (s.n < 1 || s.n > 7 || s.Cin > 4 || s.Cin * s.n * s.n > 100 || s.Cout > 8) return false;
    if (N0 < 64 || (N0 & 3) != 0) return false;
    if ((long long)s.B * N0 * N0 < (1 << 18)) return false;     // small layers stay with the register kernel
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.N0 = N0; p.M = s.M; p.n = s.n;
    p.P = 2 * s.frame;
    p.padc = s.n - 1 - p.P > 0 ? s.n - 1 - p.P : 0;
    p.GS = (p.M + 2 * p.padc + 1) & ~1;
    p.RB = 0;
    // (Shorter strips for small batches, so that every workgroup has a second strip to fetch while it
    // multiplies, were measured and change nothing: 16 images 21 and 35 us either way.)
    for (int rb = 8; rb >= 2; rb >>= 1) {
        lds = ((((size_t)(2 * rb + s.n - 1) * p.GS + 3) & ~(size_t)3) + (size_t)s.Cin * rb * N0) * sizeof(float);
        if (lds <= 78 * 1024) { p.RB = rb; break; }             // two workgroups per CU
    }
    if (p.RB == 0) return false;
    p.strips_per_item = (N0 + p.RB - 1) / p.RB;
    const long long strips = (long long)s.B * p.strips_per_item;
    p.wgs = (int)(strips < 512 / s.Cout ? strips : 512 / s.Cout);
    if (p.wgs < 1) p.wgs = 1;
    p.pre = p.M <= 64 * BI_XK && p.RB * N0 <= BI_XE * BI_THREADS;
    p.step_i = BI_THREADS / N0;
    p.step_j = BI_THREADS - p.step_i * N0;
    return true;
}

template <int n, int CI, typename T, bool PRE>
hipError_t launch_pre(const T *in, const float *g, float *dst, const ImageGradParams &p, size_t lds, hipStream_t stream)
{
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&backward_weight_image_kernel<n, CI, T, PRE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((backward_weight_image_kernel<n, CI, T, PRE>), dim3((unsigned)(p.wgs * p.Cout)), dim3(BI_THREADS), lds,
                       stream, in, g, dst, p);
    return hipGetLastError();
}

template <int n, int CI, typename T>
hipError_t launch_ci(const T *in, const float *g, float *dst, const ImageGradParams &p, size_t lds, hipStream_t stream)
{
    if (p.pre) return launch_pre<n, CI, T, true>(in, g, dst, p, lds, stream);
    return launch_pre<n, CI, T, false>(in, g, dst, p, lds, stream);
}

template <int n, typename T>
hipError_t launch_n(const T *in, const float *g, float *dst, const ImageGradParams &p, size_t lds, hipStream_t stream)
{
    switch (p.Cin) {
        case 1: return launch_ci<n, 1, T>(in, g, dst, p, lds, stream);
        case 2: return launch_ci<n, 2, T>(in, g, dst, p, lds, stream);
        case 3:
            if constexpr (3 * n * n <= 100) return launch_ci<n, 3, T>(in, g, dst, p, lds, stream);
            break;
        case 4:
            if constexpr (4 * n * n <= 100) return launch_ci<n, 4, T>(in, g, dst, p, lds, stream);
            break;
    }
    return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_t(const T *in, const float *g, float *dst, const ImageGradParams &p, size_t lds, hipStream_t stream)
{
    switch (p.n) {
        case 1: return launch_n<1, T>(in, g, dst, p, lds, stream);
        case 2: return launch_n<2, T>(in, g, dst, p, lds, stream);
        case 3: return launch_n<3, T>(in, g, dst, p, lds, stream);
        case 4: return launch_n<4, T>(in, g, dst, p, lds, stream);
        case 5: return launch_n<5, T>(in, g, dst, p, lds, stream);
        case 6: return launch_n<6, T>(in, g, dst, p, lds, stream);
        case 7: return launch_n<7, T>(in, g, dst, p, lds, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int n, int CI, typename T>
hipError_t launch_din_ci(const float *g, const T *w, float *din, const ImageGradParams &p, hipStream_t stream)
{
    const size_t lds = (size_t)(2 * p.RB + n - 1) * p.GS * sizeof(float);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&backward_input_image_kernel<n, CI, T>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((backward_input_image_kernel<n, CI, T>), dim3((unsigned)p.wgs), dim3(BI_THREADS), lds, stream, g, w, din, p);
    return hipGetLastError();
}

template <int n, typename T>
hipError_t launch_din_n(const float *g, const T *w, float *din, const ImageGradParams &p, hipStream_t stream)
{
    switch (p.Cin) {
        case 1: return launch_din_ci<n, 1, T>(g, w, din, p, stream);
        case 2: return launch_din_ci<n, 2, T>(g, w, din, p, stream);
        case 3:
            if constexpr (3 * n * n <= 100) return launch_din_ci<n, 3, T>(g, w, din, p, stream);
            break;
        case 4:
            if constexpr (4 * n * n <= 100) return launch_din_ci<n, 4, T>(g, w, din, p, stream);
            break;
    }
    return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_din_t(const float *g, const T *w, float *din, const ImageGradParams &p, hipStream_t stream)
{
    switch (p.n) {
        case 1: return launch_din_n<1, T>(g, w, din, p, stream);
        case 2: return launch_din_n<2, T>(g, w, din, p, stream);
        case 3: return launch_din_n<3, T>(g, w, din, p, stream);
        case 4: return launch_din_n<4, T>(g, w, din, p, stream);
        case 5: return launch_din_n<5, T>(g, w, din, p, stream);
        case 6: return launch_din_n<6, T>(g, w, din, p, stream);
        case 7: return launch_din_n<7, T>(g, w, din, p, stream);
        default: return hipErrorInvalidValue;
    }
}

// The input gradient's kernel: one output channel, and a map whose rows of g fit a lane's registers.
bool din_plan(const Shape &s, ImageGradParams &p)
{
    size_t lds;
    return s.Cout == 1 && image_plan(s, p, lds) && p.pre;
}

}  // namespace

bool backward_weight_image_apply(const Shape &s)
{
    ImageGradParams p;
    size_t lds;
    return image_plan(s, p, lds);
}

int backward_weight_image_slices(const Shape &s)
{
    ImageGradParams p;
    size_t lds;
    return image_plan(s, p, lds) ? p.wgs : 0;
}

hipError_t launch_backward_weight_image(const void *in, const float *g, float *dst, const Shape &s, kst_dtype dt,
                                        hipStream_t stream)
{
    ImageGradParams p;
    size_t lds;
    if (!image_plan(s, p, lds)) return hipErrorInvalidValue;
    if (dt == KST_BF16) return launch_t<uint16_t>((const uint16_t *)in, g, dst, p, lds, stream);
    if (dt == KST_F16) return launch_t<half_bits>((const half_bits *)in, g, dst, p, lds, stream);
    return launch_t<float>((const float *)in, g, dst, p, lds, stream);
}

bool backward_input_image_apply(const Shape &s)
{
    ImageGradParams p;
    return din_plan(s, p);
}

hipError_t launch_backward_input_image(const float *g, const void *w, float *din, const Shape &s, kst_dtype dt,
                                       hipStream_t stream)
{
    ImageGradParams p;
    if (!din_plan(s, p)) return hipErrorInvalidValue;
    if (dt == KST_BF16) return launch_din_t<uint16_t>(g, (const uint16_t *)w, din, p, stream);
    if (dt == KST_F16) return launch_din_t<half_bits>(g, (const half_bits *)w, din, p, stream);
    return launch_din_t<float>(g, (const float *)w, din, p, stream);
}

}  // namespace kst
