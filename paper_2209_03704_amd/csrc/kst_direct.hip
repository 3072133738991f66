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
#include "kst_direct_flat.h"
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
    Epilogue epi;
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
    if (epi_on(p.epi)) {                                     // uniform
        const float bias = epi_bias(p.epi, co);
#pragma unroll
        for (int q = 0; q < D_RPT; ++q)
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) acc[q][r][s2] = epi_apply(acc[q][r][s2], bias, p.epi.act);
    }
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

// ---------------------------------------------------------------------------
// Row-strip variant: the fast path whenever a strip of full input rows fits in LDS.
//
// On this chip a store that is not 16-byte aligned costs about a third of the
// write bandwidth, and with an odd M every other output row starts misaligned,
// so the per-quad stores of the tile kernel cannot reach the HBM roofline.
// Here the roles are turned round: a lane owns one 16-byte ALIGNED group of
// four consecutive outputs of one row.  Within a row the parity pattern of the
// group (s = 0,1,0,1 or 1,0,1,0) and the row parity r are the same for every
// lane, so the four sub-kernels still apply with wave-uniform control flow:
// the group needs Ta(r) input rows x (fl + 2) columns of the original input and
// produces two outputs of each column parity (Eqs. 7-10, two quad halves at a
// time).  Only the first and last group of a row can be partial; those use
// masked scalar stores.  A workgroup owns R consecutive output rows of one
// plane; their R/2 + fl input rows are one contiguous run of the input and are
// staged in LDS (with 4 floats of slack on both sides of each row so that
// partial groups read inside the buffer).  Accumulators stay in registers
// across input channels.
// ---------------------------------------------------------------------------
struct RowsParams {
    int B, Cin, Cout, N, M;
    int R;                    // output rows per workgroup (even)
    int chunks_per_plane;     // ceil(M / R)
    unsigned nchunks;         // planes * chunks_per_plane
    unsigned xcd_slots;       // ceil(nchunks / 8)
    int xcd_remap;
    int prefetch;             // single-channel kernel: next strip's loads fly during compute
    int xs_buf;               // floats per LDS input buffer
    int xs_stride;            // floats per staged row: N rounded up to 4, plus 8
    unsigned off[4];
    Epilogue epi;
};

constexpr int R_PAD = 4;      // slack floats left of each staged row (and at least as many right)

// One aligned group of row parity r whose first output has column parity `par`.
// rowp: staged input row i + r of this output row, at column 0.  cbase: first window column.
template <int n, int r, int par>
__device__ __forceinline__ void rows_group(float4 &acc, const float *__restrict__ rowp, int xs_stride, int cbase,
                                           const float (&wk)[2][2][((n + 1) / 2) * ((n + 1) / 2)])
{
    constexpr int fl = n / 2;
    constexpr int Ta = r ? n / 2 : (n + 1) / 2;
    constexpr int Tb0 = (n + 1) / 2, Tb1 = n / 2;
    float win[Ta > 0 ? Ta : 1][fl + 2];
#pragma unroll
    for (int a = 0; a < Ta; ++a)
#pragma unroll
        for (int c = 0; c < fl + 2; ++c) win[a][c] = rowp[a * xs_stride + cbase + c];
    // Output k of the group has column parity s_k and starts its taps at window column c_k.
    constexpr int s_k[4] = {par, 1 - par, par, 1 - par};
    constexpr int c_k[4] = {0, par ? 0 : 1, 1, par ? 1 : 2};
    float o[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int Tb = s_k[k] ? Tb1 : Tb0;
#pragma unroll
        for (int a = 0; a < Ta; ++a)
#pragma unroll
            for (int bq = 0; bq < Tb; ++bq) o[k] = fmaf(win[a][c_k[k] + bq], wk[r][s_k[k]][a * Tb + bq], o[k]);
    }
    acc = make_float4(o[0], o[1], o[2], o[3]);
}

// Shared prologue of the two row-strip kernels: strip geometry and input staging.
struct RowsGeom {
    int plane, b, co, y0, i0, rows_out, rows_in;
    size_t plane_base;
};

__device__ __forceinline__ void rows_geometry(const RowsParams &p, int fl, unsigned logical, RowsGeom &g)
{
    g.plane = (int)(logical / (unsigned)p.chunks_per_plane);
    const int chunk = (int)(logical - (unsigned)g.plane * p.chunks_per_plane);
    g.b = g.plane / p.Cout;
    g.co = g.plane - g.b * p.Cout;
    g.y0 = chunk * p.R;
    g.i0 = g.y0 >> 1;
    g.rows_out = min(p.R, p.M - g.y0);
    g.rows_in = min(p.R / 2 + fl, p.N - g.i0);
    g.plane_base = (size_t)g.plane * p.M * p.M;
}

// Stage input rows i0 .. i0+rows_in-1 of (b, ci): one contiguous run of the input.
template <typename T>
__device__ __forceinline__ void rows_stage(float *__restrict__ Xs, const T *__restrict__ in, const RowsParams &p,
                                           const RowsGeom &g, int ci)
{
    const int tid = threadIdx.x;
    const T *src = in + (((size_t)g.b * p.Cin + ci) * p.N + g.i0) * p.N;
    if (sizeof(T) == 4 && (p.N & 3) == 0 && (reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
        // All loads of a batch are issued before the first LDS write waits for any of them.
        const float4 *s4 = reinterpret_cast<const float4 *>(src);
        const int n4 = p.N >> 2, count4 = g.rows_in * n4;
        for (int base = 0; base < count4; base += 4 * 256) {
            float4 tmp[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                tmp[k] = s4[min(base + k * 256 + tid, count4 - 1)];   // clamped: always a valid load
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int v = base + k * 256 + tid;
                if (v < count4) {
                    const int rr = v / n4, x4 = v - rr * n4;
                    *reinterpret_cast<float4 *>(Xs + rr * p.xs_stride + R_PAD + 4 * x4) = tmp[k];
                }
            }
        }
    } else {
        const int count = g.rows_in * p.N;
        for (int base = 0; base < count; base += 4 * 256) {
            T tmp[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                tmp[k] = src[min(base + k * 256 + tid, count - 1)];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int e = base + k * 256 + tid;
                if (e < count) {
                    const int rr = e / p.N, x = e - rr * p.N;
                    Xs[rr * p.xs_stride + R_PAD + x] = to_f32(tmp[k]);
                }
            }
        }
    }
}

template <int n, typename T>
__device__ __forceinline__ void rows_weights(float (&wk)[2][2][((n + 1) / 2) * ((n + 1) / 2)],
                                             const T *__restrict__ w_seg, const RowsParams &p, int ci, int co)
{
    constexpr int Ta0 = (n + 1) / 2, Ta1 = n / 2;
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int Ta = r ? Ta1 : Ta0, Tb = s ? Ta1 : Ta0;
#pragma unroll
            for (int t = 0; t < Ta * Tb; ++t)
                wk[r][s][t] = to_f32(w_seg[wseg_index<T>(p.off[2 * r + s], Ta * Tb, p.Cout, ci, t, co)]);
        }
}

__device__ __forceinline__ void rows_store(float *__restrict__ o, const float4 &v4, int x0, int M)
{
    if (x0 >= 0 && x0 + 3 < M) {
        store_streaming4(o, v4.x, v4.y, v4.z, v4.w);            // 16-byte aligned by construction
    } else {
        const float v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (x0 + k >= 0 && x0 + k < M) o[k] = v[k];
    }
}

// One output row of parity r for a single input channel: compute and store at once.
template <int n, int r>
__device__ __forceinline__ void rows_emit(float *__restrict__ out, const float *__restrict__ Xs, const RowsParams &p,
                                          const RowsGeom &g, int row, int shift,
                                          const float (&wk)[2][2][((n + 1) / 2) * ((n + 1) / 2)])
{
    const int y = g.y0 + row;
    const float *rowp = Xs + ((row >> 1) + r) * p.xs_stride + R_PAD;
    float *orow = out + g.plane_base + (size_t)y * p.M;
    const bool epi = epi_on(p.epi);                          // uniform
    const float bias = epi ? epi_bias(p.epi, g.co) : 0.0f;
    for (int t = threadIdx.x; 4 * t - shift < p.M; t += 256) {
        const int x0 = 4 * t - shift;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (shift & 1) rows_group<n, r, 1>(acc, rowp, p.xs_stride, ((x0 - 1) >> 1) + 1, wk);
        else rows_group<n, r, 0>(acc, rowp, p.xs_stride, x0 >> 1, wk);
        if (epi) epi_apply4(acc.x, acc.y, acc.z, acc.w, bias, p.epi.act);
        rows_store(orow + x0, acc, x0, p.M);
    }
}

// Single input channel (the bandwidth-bound case).  Nothing has to be accumulated, so
// each row is computed and stored straight away and a lane keeps almost no state.
// The kernel is persistent: a workgroup walks over many strips, and while it computes
// and stores strip k from one LDS buffer the 16-byte loads of strip k+1 are already in
// flight into registers (written to the other buffer afterwards, one barrier per
// strip).  Without that overlap all workgroups of a launch load, compute and store in
// lock-step and the read and write phases of the whole chip add up instead of overlapping.
constexpr int R_NLD = 4;      // float4 loads in flight per lane (pre0..pre3): strips of at most 256 * 4 * 4 floats

template <int n, typename T>
__global__ void __launch_bounds__(256) direct_rows1_kernel(const T *__restrict__ in, const T *__restrict__ w_seg,
                                                             float *__restrict__ out, RowsParams p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];   // 2 x [R/2 + fl][xs_stride]
    const int tid = threadIdx.x;
    // Strip schedule: with xcd_remap, XCD x owns strips [x * xcd_slots, (x+1) * xcd_slots) and
    // its workgroups interleave over them; otherwise all workgroups interleave over everything.
    unsigned c, c_end, stride;
    if (p.xcd_remap) {
        const unsigned xcd = blockIdx.x & 7u;
        c = xcd * p.xcd_slots + (blockIdx.x >> 3);
        c_end = min((xcd + 1) * p.xcd_slots, p.nchunks);
        stride = gridDim.x >> 3;
    } else {
        c = blockIdx.x;
        c_end = p.nchunks;
        stride = gridDim.x;
    }
    if (c >= c_end) return;

    RowsGeom g;
    rows_geometry(p, n / 2, c, g);
    const int n4 = p.N >> 2;
    rows_stage<T>(lds, in, p, g, 0);                      // first strip: plain staging
    __syncthreads();

    float wk[2][2][((n + 1) / 2) * ((n + 1) / 2)];
    int cur_co = -1;
    const int mstep = p.M & 3;
    int buf = 0;
    while (true) {
        const unsigned cn = c + stride;
        const bool more = cn < c_end;
        // Geometry of the next strip (of this one again after the last: the loads below are
        // then redundant but still valid, which keeps them unconditional and in registers).
        RowsGeom gn;
        rows_geometry(p, n / 2, more ? cn : c, gn);
        float4 pre0, pre1, pre2, pre3;
        const int count4 = gn.rows_in * n4;
        if (p.prefetch) {
            const float4 *s4 = reinterpret_cast<const float4 *>(in + (((size_t)gn.b * p.Cin) * p.N + gn.i0) * p.N);
            pre0 = s4[min(tid, count4 - 1)];
            pre1 = s4[min(256 + tid, count4 - 1)];
            pre2 = s4[min(512 + tid, count4 - 1)];
            pre3 = s4[min(768 + tid, count4 - 1)];
        }
        if (g.co != cur_co) {
            rows_weights<n, T>(wk, w_seg, p, 0, g.co);
            cur_co = g.co;
        }
        const float *Xs = lds + buf * p.xs_buf;
        int shift = (int)((g.plane_base + (size_t)g.y0 * p.M) & 3);
#pragma unroll 1
        for (int row = 0; row < g.rows_out; row += 2) {
            rows_emit<n, 0>(out, Xs, p, g, row, shift, wk);
            shift = (shift + mstep) & 3;
            if (row + 1 < g.rows_out) rows_emit<n, 1>(out, Xs, p, g, row + 1, shift, wk);
            shift = (shift + mstep) & 3;
        }
        if (!more) break;
        float *Xn = lds + (buf ^ 1) * p.xs_buf;
        if (p.prefetch) {
            const float4 pre[4] = {pre0, pre1, pre2, pre3};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int v = k * 256 + tid;
                if (v < count4) {
                    const int rr = v / n4, x4 = v - rr * n4;
                    *reinterpret_cast<float4 *>(Xn + rr * p.xs_stride + R_PAD + 4 * x4) = pre[k];
                }
            }
        } else {
            rows_stage<T>(Xn, in, p, gn, 0);
        }
        __syncthreads();
        g = gn;
        c = cn;
        buf ^= 1;
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
            if (epi_on(p.epi)) a = epi_apply(a, epi_bias(p.epi, co), p.epi.act);
            out[((size_t)plane * p.M + y) * p.M + x] = a;
        }
}

template <int n, typename T>
static void launch_tiled(const T *in, const T *w_seg, float *out, const DirectParams &p, unsigned blocks,
                         hipStream_t stream)
{
    hipLaunchKernelGGL((direct_kernel<n, T>), dim3(blocks), dim3(256), 0, stream, in, w_seg, out, p);
}

constexpr size_t kRowsLdsLimit = 64 * 1024;

// Strip plan of the single-channel rows kernel (several input channels are the multi-channel
// kernel's job): R output rows per strip.
template <int n, typename T>
static bool try_rows(const T *in, const T *w_seg, float *out, const Shape &s, kst_dtype dt, hipStream_t stream)
{
    if (s.Cin != 1) return false;
    RowsParams p;
    p.xs_stride = ((s.N + 3) & ~3) + 2 * R_PAD;
    // Tallest strip (up to 16 rows) whose input fits the prefetch registers and 20 KB of LDS.
    int R = 8;
    const bool vec = sizeof(T) == 4 && (s.N & 3) == 0;
    while (R > 2 && ((size_t)(R / 2 + s.fl) * p.xs_stride * sizeof(float) > 20 * 1024 ||
                     (vec && (size_t)(R / 2 + s.fl) * s.N > (size_t)256 * R_NLD * 4)))
        R -= 2;
    p.R = R;
    p.xs_buf = (R / 2 + s.fl) * p.xs_stride;
    p.prefetch = vec && (size_t)(R / 2 + s.fl) * s.N <= (size_t)256 * R_NLD * 4;
    const size_t lds = (size_t)2 * p.xs_buf * sizeof(float);
    if (lds > kRowsLdsLimit) return false;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.N = s.N; p.M = s.M;
    p.chunks_per_plane = (s.M + p.R - 1) / p.R;
    const size_t nchunks = (size_t)s.B * s.Cout * p.chunks_per_plane;
    if (nchunks >= 0x7ffffff0u) return false;
    p.nchunks = (unsigned)nchunks;
    p.xcd_slots = (p.nchunks + 7) / 8;
    // Plain interleaving measured faster than XCD-contiguous ranges (one stream over the chip
    // keeps HBM pages hot).
    p.xcd_remap = 0;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, dt);
    p.epi = s.epi;
    // Persistent: a few workgroups per CU, each walking over its share of the strips.
    unsigned grid = 1024;
    if (grid > p.xcd_slots * 8) grid = p.xcd_slots * 8;
    grid = grid < 8 ? 8 : (grid & ~7u);                        // whole multiples of the 8 XCDs
    hipLaunchKernelGGL((direct_rows1_kernel<n, T>), dim3(grid), dim3(256), lds, stream, in, w_seg, out, p);
    return true;
}

template <typename T>
static bool run_rows(const T *in, const T *w_seg, float *out, const Shape &s, kst_dtype dt, hipStream_t stream)
{
    switch (s.n) {
        case 1: return try_rows<1, T>(in, w_seg, out, s, dt, stream);
        case 2: return try_rows<2, T>(in, w_seg, out, s, dt, stream);
        case 3: return try_rows<3, T>(in, w_seg, out, s, dt, stream);
        case 4: return try_rows<4, T>(in, w_seg, out, s, dt, stream);
        case 5: return try_rows<5, T>(in, w_seg, out, s, dt, stream);
        case 6: return try_rows<6, T>(in, w_seg, out, s, dt, stream);
        case 7: return try_rows<7, T>(in, w_seg, out, s, dt, stream);
        default: return false;
    }
}

template <typename T>
static hipError_t run(const T *in, const T *w_seg, float *out, const Shape &s, kst_dtype dt, hipStream_t stream)
{
    if (run_rows<T>(in, w_seg, out, s, dt, stream)) return hipGetLastError();
    DirectParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.N = s.N; p.M = s.M; p.E = s.E;
    p.tiles_x = (s.E + D_TJ - 1) / D_TJ;
    p.tiles_y = (s.E + D_TI - 1) / D_TI;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, dt);
    p.epi = s.epi;
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

bool direct_takes_virtual_frame(const Shape &s, int q, int crop, kst_dtype dt)
{
    FlatParams fp;
    unsigned grid;
    size_t lds;
    Shape framed = s;
    framed.frame = q;
    framed.crop = crop;
    if (direct_flat_plan(framed, dt, fp, grid, lds)) return true;       // the flat kernel keeps the frame in LDS
    Shape dense = s;
    dense.frame = 0;
    return !direct_flat_plan(dense, dt, fp, grid, lds) && direct_multi_supported(dense);
}

hipError_t launch_direct(const void *in, const void *w_seg, float *out, const Shape &s, kst_dtype dt,
                         hipStream_t stream)
{
    FlatParams fp;
    unsigned grid;
    size_t lds;
    if (s.frame != 0) {
        if (direct_flat_plan(s, dt, fp, grid, lds))
            return launch_direct_flat((const float *)in, (const float *)w_seg, out, s, fp, grid, lds, stream);
        if (!direct_takes_virtual_frame(s, s.frame, s.crop, dt)) return hipErrorInvalidValue;
        return launch_direct_multi(in, w_seg, out, s, dt, stream);
    }
    if (direct_flat_plan(s, dt, fp, grid, lds))
        return launch_direct_flat((const float *)in, (const float *)w_seg, out, s, fp, grid, lds, stream);
    if (direct_multi_supported(s)) return launch_direct_multi(in, w_seg, out, s, dt, stream);
    if (dt == KST_BF16) return run<uint16_t>((const uint16_t *)in, (const uint16_t *)w_seg, out, s, dt, stream);
    if (dt == KST_F16) return run<half_bits>((const half_bits *)in, (const half_bits *)w_seg, out, s, dt, stream);
    return run<float>((const float *)in, (const float *)w_seg, out, s, dt, stream);
}

}  // namespace kst
