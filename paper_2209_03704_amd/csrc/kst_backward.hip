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

// Kernel sizes up to 7, any channel counts: the same sums with register blocking.
//
// Kernel gradient: a workgroup owns CI input channels, CO output channels (n*n*CO <= 64; more than
// one input channel only with CO = 1, n*n*CI <= 100) and a slice of the positions; a lane keeps
// all n*n*CO*CI partial sums in registers, so an input value is loaded once for n*n*CO products, a
// value of g once for CI, and nothing is re-read per kernel element.  The partial sums are added
// across the lanes with wave shuffles, across the four waves through LDS.
template <int n, int CO, int CI, typename T>
__global__ void __launch_bounds__(256) backward_weight_regs_kernel(const T *__restrict__ in, const float *__restrict__ g,
                                                                    float *__restrict__ dst, int B, int Cin, int Cout,
                                                                    int N, int M, int q, int per_slice)
{
    // N: edge of `in` as it lies in memory; q: zero frame the forward put around it (its products
    // are zeros and are skipped): position (a, c) meets g rows 2 (a + q) - u.
    constexpr int NN = n * n;
    constexpr int S = NN * CO * CI;                               // sums per lane
    __shared__ float red[4][S];
    const int groups = Cout / CO;                                 // CO divides Cout
    const int cigs = (Cin + CI - 1) / CI;
    unsigned id = blockIdx.x;
    const int ci0 = (int)(id % (unsigned)cigs) * CI;
    id /= (unsigned)cigs;
    const int co0 = (int)(id % (unsigned)groups) * CO;
    const int slice = (int)(id / (unsigned)groups);
    const int tid = threadIdx.x;
    const int per_item = N * N;
    const int total = B * per_item;
    const int e_begin = slice * per_slice, e_end = min(total, e_begin + per_slice);

    float acc[CI][CO][NN];
#pragma unroll
    for (int q = 0; q < CI; ++q)
#pragma unroll
        for (int k = 0; k < CO; ++k)
#pragma unroll
            for (int t = 0; t < NN; ++t) acc[q][k][t] = 0.0f;

    for (int e = e_begin + tid; e < e_end; e += 256) {
        const int b = e / per_item, rem = e - b * per_item;
        const int a = rem / N, c = rem - a * N;
        float xin[CI];
#pragma unroll
        for (int q = 0; q < CI; ++q)
            xin[q] = ci0 + q < Cin ? to_f32(in[(((size_t)b * Cin + ci0 + q) * N + a) * N + c]) : 0.0f;
        const float *gp = g + ((size_t)b * Cout + co0) * M * M;
#pragma unroll
        for (int u = 0; u < n; ++u) {
            const int y = 2 * (a + q) - u;
            if (y < 0 || y >= M) continue;
#pragma unroll
            for (int v = 0; v < n; ++v) {
                const int x = 2 * (c + q) - v;
                if (x < 0 || x >= M) continue;
#pragma unroll
                for (int k = 0; k < CO; ++k) {
                    const float gv = gp[((size_t)k * M + y) * M + x];
#pragma unroll
                    for (int q = 0; q < CI; ++q) acc[q][k][u * n + v] = fmaf(xin[q], gv, acc[q][k][u * n + v]);
                }
            }
        }
    }

    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int q = 0; q < CI; ++q)
#pragma unroll
        for (int k = 0; k < CO; ++k)
#pragma unroll
            for (int t = 0; t < NN; ++t) {
                float v = acc[q][k][t];
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
                if (lane == 0) red[wave][(q * CO + k) * NN + t] = v;
            }
    __syncthreads();
    for (int i = tid; i < S; i += 256) {
        const int q = i / (CO * NN), r = i - q * (CO * NN);
        const int k = r / NN, t = r - k * NN;
        const float sum = (red[0][i] + red[1][i]) + (red[2][i] + red[3][i]);
        if (ci0 + q < Cin) dst[(size_t)slice * Cout * Cin * NN + ((size_t)(co0 + k) * Cin + ci0 + q) * NN + t] = sum;
    }
}

// Kernel gradient for layers with many input channels (and any, typically few, output channels):
// a workgroup is one wave whose lanes are 64 input channels; it walks a slice of the positions.
// At a position every lane loads its channel's input value, and the n*n*CO values of g the
// position meets are loaded once by the first n*n*CO lanes (one predicated load, bounds per lane)
// and handed to all lanes with lane reads, so a product costs no load of its own and g is not
// fetched again for every input channel.  Positions are taken eight at a time so that their
// loads are in flight together.  A lane ends with the n*n*CO sums of its own channel: no
// reduction across lanes; every wave writes one partial result, added up by a second pass.
constexpr int L_BATCH = 8;

template <int n, int CO, typename T>
__global__ void __launch_bounds__(64) backward_weight_lanes_kernel(const T *__restrict__ in, const float *__restrict__ g,
                                                                    float *__restrict__ dst, int B, int Cin, int Cout,
                                                                    int N, int M, int q, int per_slice)
{
    // (N, q: as in the kernel above)
    constexpr int NN = n * n;
    constexpr int W = NN * CO;                                    // window values per position (<= 64)
    const int cgroups = (Cin + 63) / 64, groups = Cout / CO;      // CO divides Cout
    unsigned id = blockIdx.x;
    const int cg = (int)(id % (unsigned)cgroups);
    id /= (unsigned)cgroups;
    const int co0 = (int)(id % (unsigned)groups) * CO;
    const int slice = (int)(id / (unsigned)groups);
    const int lane = threadIdx.x;
    const int ci = cg * 64 + lane;
    const bool ci_ok = ci < Cin;
    const int per_item = N * N;
    const int total = B * per_item;
    const int e_begin = slice * per_slice, e_end = min(total, e_begin + per_slice);
    // this lane's window element: output channel k, kernel element (u, v)
    const int wk = lane / NN, wuv = lane - wk * NN;
    const int wu = wuv / n, wv = wuv - wu * n;
    const bool w_ok = lane < W;

    float acc[W];
#pragma unroll
    for (int t = 0; t < W; ++t) acc[t] = 0.0f;

    for (int e0 = e_begin; e0 < e_end; e0 += L_BATCH) {
        float xin[L_BATCH], gv[L_BATCH];
#pragma unroll
        for (int j = 0; j < L_BATCH; ++j) {
            const int e = e0 + j;                                 // wave-uniform
            xin[j] = 0.0f;
            gv[j] = 0.0f;
            if (e < e_end) {
                const int b = e / per_item, rem = e - b * per_item;
                const int a = rem / N, c = rem - a * N;
                if (ci_ok) xin[j] = to_f32(in[(((size_t)b * Cin + ci) * N + a) * N + c]);
                const int y = 2 * (a + q) - wu, x = 2 * (c + q) - wv;
                if (w_ok && y >= 0 && y < M && x >= 0 && x < M)
                    gv[j] = g[(((size_t)b * Cout + co0 + wk) * M + y) * M + x];
            }
        }
#pragma unroll
        for (int j = 0; j < L_BATCH; ++j)
#pragma unroll
            for (int t = 0; t < W; ++t)
                acc[t] = fmaf(xin[j], __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, gv[j]), t)),
                              acc[t]);
    }
    if (!ci_ok) return;
    float *o = dst + (size_t)slice * Cout * Cin * NN;
#pragma unroll
    for (int t = 0; t < W; ++t) {
        const int k = t / NN, uv = t - k * NN;
        o[((size_t)(co0 + k) * Cin + ci) * NN + uv] = acc[t];
    }
}

// Input gradient: a lane owns one position (a, c) of one batch item for a group of Q input
// channels.  Per pass over CG output channels (n*n*CG <= 64) it loads the n x n window of g it
// needs once into registers and multiplies it with the kernels of its Q channels, which the
// workgroup has staged in LDS (the same values for every lane: 16-byte reads at one address).
// CG: output channels per pass; Q: input channels per workgroup (8, or 4 for layers with at most 4).
// N: edge of din as it lies in memory; q: zero frame the forward put around the input (its
// gradient is not wanted): position (a, c) meets g rows 2 (a + q) - u.
template <int n, int CG, int Q, typename T>
__global__ void __launch_bounds__(256) backward_input_regs_kernel(const float *__restrict__ g, const T *__restrict__ w,
                                                                   float *__restrict__ din, int B, int Cin, int Cout,
                                                                   int N, int M, int q)
{
    constexpr int NN = n * n;
    constexpr int WPC = (NN * CG + 3) & ~3;                       // staged weights per input channel, padded
    __shared__ __attribute__((aligned(16))) float Wl[Q * WPC];
    const int tiles = (N * N + 255) / 256;
    const int cigs = (Cin + Q - 1) / Q;
    unsigned id = blockIdx.x;
    const int tile = (int)(id % (unsigned)tiles);
    id /= (unsigned)tiles;
    const int ci0 = (int)(id % (unsigned)cigs) * Q;
    const int b = (int)(id / (unsigned)cigs);
    const int tid = threadIdx.x;
    const int pos = tile * 256 + tid;
    const bool live = pos < N * N;
    const int a = live ? pos / N : 0, c = live ? pos - (pos / N) * N : 0;

    float acc[Q];
#pragma unroll
    for (int j = 0; j < Q; ++j) acc[j] = 0.0f;

    for (int co0 = 0; co0 < Cout; co0 += CG) {
        // This pass's kernels -> LDS: [channel of the group][output channel of the pass][u][v].
        __syncthreads();                                          // the previous pass has read its weights
        for (int e = tid; e < Q * WPC; e += 256) {
            const int j = e / WPC, rem = e - j * WPC;
            const int k = rem / NN, t = rem - k * NN;
            float v = 0.0f;
            if (k < CG && co0 + k < Cout && ci0 + j < Cin) v = to_f32(w[((size_t)(co0 + k) * Cin + ci0 + j) * NN + t]);
            Wl[e] = v;
        }
        // The window of g this position meets (zero outside the map and past the last channel).
        float gw[CG][NN];
#pragma unroll
        for (int k = 0; k < CG; ++k) {
            const bool k_ok = live && co0 + k < Cout;
            const float *gp = g + ((size_t)b * Cout + min(co0 + k, Cout - 1)) * M * M;
#pragma unroll
            for (int u = 0; u < n; ++u)
#pragma unroll
                for (int v = 0; v < n; ++v) {
                    const int y = 2 * (a + q) - u, x = 2 * (c + q) - v;
                    const bool ok = k_ok && y >= 0 && y < M && x >= 0 && x < M;
                    gw[k][u * n + v] = ok ? gp[(size_t)y * M + x] : 0.0f;
                }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            float wv[WPC];
#pragma unroll
            for (int g4 = 0; g4 < WPC / 4; ++g4) {
                const float4 v = *reinterpret_cast<const float4 *>(&Wl[j * WPC + 4 * g4]);
                wv[4 * g4] = v.x;
                wv[4 * g4 + 1] = v.y;
                wv[4 * g4 + 2] = v.z;
                wv[4 * g4 + 3] = v.w;
            }
#pragma unroll
            for (int k = 0; k < CG; ++k)
#pragma unroll
                for (int t = 0; t < NN; ++t) acc[j] = fmaf(gw[k][t], wv[k * NN + t], acc[j]);
        }
    }
    if (!live) return;
#pragma unroll
    for (int j = 0; j < Q; ++j)
        if (ci0 + j < Cin) din[(((size_t)b * Cin + ci0 + j) * N + a) * N + c] = acc[j];
}

// Output channels per workgroup (kernel gradient) or per pass (input gradient): the largest of
// 4, 3, 2, 1 with n*n*k <= 64 (and, for the kernel gradient, dividing Cout).
constexpr int regs_fit(int n) { return 64 / (n * n) < 4 ? 64 / (n * n) : 4; }

inline int weight_co(int n, int Cout)
{
    for (int k = regs_fit(n); k > 1; --k)
        if (Cout % k == 0) return k;
    return 1;
}

// Input channels per workgroup of that kernel: more than one only with a single output channel.
inline int weight_ci(int n, int co, int Cin)
{
    if (co != 1) return 1;
    int k = Cin < 4 ? Cin : 4;
    while (k > 1 && k * n * n > 100) --k;
    return k;
}

template <int n, int CO, int CI, typename T>
void launch_weight_regs_ci(const T *in, const float *g, float *dst, const Shape &s, int slices, int per_slice,
                           hipStream_t stream)
{
    const unsigned blocks = (unsigned)((s.Cin + CI - 1) / CI) * (unsigned)(s.Cout / CO) * (unsigned)slices;
    hipLaunchKernelGGL((backward_weight_regs_kernel<n, CO, CI, T>), dim3(blocks), dim3(256), 0, stream, in, g, dst, s.B,
                       s.Cin, s.Cout, s.N - 2 * s.frame, s.M, s.frame, per_slice);
}

template <int n, int CO, typename T>
void launch_weight_regs_co(const T *in, const float *g, float *dst, const Shape &s, int slices, int per_slice,
                           hipStream_t stream)
{
    if constexpr (CO == 1) {
        const int ci = weight_ci(n, 1, s.Cin);
        if constexpr (4 * n * n <= 100)
            if (ci == 4) return launch_weight_regs_ci<n, 1, 4, T>(in, g, dst, s, slices, per_slice, stream);
        if constexpr (3 * n * n <= 100)
            if (ci == 3) return launch_weight_regs_ci<n, 1, 3, T>(in, g, dst, s, slices, per_slice, stream);
        if constexpr (2 * n * n <= 100)
            if (ci == 2) return launch_weight_regs_ci<n, 1, 2, T>(in, g, dst, s, slices, per_slice, stream);
    }
    launch_weight_regs_ci<n, CO, 1, T>(in, g, dst, s, slices, per_slice, stream);
}

template <int n, typename T>
void launch_weight_regs_n(const T *in, const float *g, float *dst, const Shape &s, int slices, int per_slice,
                          hipStream_t stream)
{
    const int co = weight_co(n, s.Cout);
    if constexpr (regs_fit(n) >= 4)
        if (co == 4) return launch_weight_regs_co<n, 4, T>(in, g, dst, s, slices, per_slice, stream);
    if constexpr (regs_fit(n) >= 3)
        if (co == 3) return launch_weight_regs_co<n, 3, T>(in, g, dst, s, slices, per_slice, stream);
    if constexpr (regs_fit(n) >= 2)
        if (co == 2) return launch_weight_regs_co<n, 2, T>(in, g, dst, s, slices, per_slice, stream);
    launch_weight_regs_co<n, 1, T>(in, g, dst, s, slices, per_slice, stream);
}

template <typename T>
bool launch_weight_regs(const T *in, const float *g, float *dst, const Shape &s, int slices, int per_slice,
                        hipStream_t stream)
{
    switch (s.n) {
        case 1: launch_weight_regs_n<1, T>(in, g, dst, s, slices, per_slice, stream); return true;
        case 2: launch_weight_regs_n<2, T>(in, g, dst, s, slices, per_slice, stream); return true;
        case 3: launch_weight_regs_n<3, T>(in, g, dst, s, slices, per_slice, stream); return true;
        case 4: launch_weight_regs_n<4, T>(in, g, dst, s, slices, per_slice, stream); return true;
        case 5: launch_weight_regs_n<5, T>(in, g, dst, s, slices, per_slice, stream); return true;
        case 6: launch_weight_regs_n<6, T>(in, g, dst, s, slices, per_slice, stream); return true;
        case 7: launch_weight_regs_n<7, T>(in, g, dst, s, slices, per_slice, stream); return true;
        default: return false;
    }
}

// Edge of the maps as they lie in memory: the shape's edge less its virtual frame.
inline int unframed_edge(const Shape &s) { return s.N - 2 * s.frame; }

template <int n, int CG, int Q, typename T>
void launch_input_regs_q(const float *g, const T *w, float *din, const Shape &s, hipStream_t stream)
{
    const int N0 = unframed_edge(s);
    const unsigned tiles = (unsigned)((N0 * N0 + 255) / 256), cigs = (unsigned)((s.Cin + Q - 1) / Q);
    hipLaunchKernelGGL((backward_input_regs_kernel<n, CG, Q, T>), dim3(tiles * cigs * (unsigned)s.B), dim3(256), 0,
                       stream, g, w, din, s.B, s.Cin, s.Cout, N0, s.M, s.frame);
}

// Output channels per pass: as many as fit the registers, or one for a single-channel output;
// input channels per workgroup: 8, or 4 for layers with at most 4.
template <int n, typename T>
void launch_input_regs_n(const float *g, const T *w, float *din, const Shape &s, hipStream_t stream)
{
    constexpr int CG = regs_fit(n);
    if (s.Cout == 1 && CG > 1) {
        if (s.Cin <= 4) return launch_input_regs_q<n, 1, 4, T>(g, w, din, s, stream);
        return launch_input_regs_q<n, 1, 8, T>(g, w, din, s, stream);
    }
    if (s.Cin <= 4) return launch_input_regs_q<n, CG, 4, T>(g, w, din, s, stream);
    launch_input_regs_q<n, CG, 8, T>(g, w, din, s, stream);
}

template <typename T>
bool launch_input_regs(const float *g, const T *w, float *din, const Shape &s, hipStream_t stream)
{
    const int N0 = unframed_edge(s);
    const size_t blocks = (size_t)((N0 * N0 + 255) / 256) * ((s.Cin + 3) / 4) * s.B;
    if (blocks >= 0x7fffffffu) return false;
    switch (s.n) {
        case 1: launch_input_regs_n<1, T>(g, w, din, s, stream); return true;
        case 2: launch_input_regs_n<2, T>(g, w, din, s, stream); return true;
        case 3: launch_input_regs_n<3, T>(g, w, din, s, stream); return true;
        case 4: launch_input_regs_n<4, T>(g, w, din, s, stream); return true;
        case 5: launch_input_regs_n<5, T>(g, w, din, s, stream); return true;
        case 6: launch_input_regs_n<6, T>(g, w, din, s, stream); return true;
        case 7: launch_input_regs_n<7, T>(g, w, din, s, stream); return true;
        default: return false;
    }
}

template <int n, int CO, typename T>
void launch_weight_lanes_co(const T *in, const float *g, float *dst, const Shape &s, int slices, int per_slice,
                            hipStream_t stream)
{
    const unsigned blocks = (unsigned)((s.Cin + 63) / 64) * (unsigned)(s.Cout / CO) * (unsigned)slices;
    hipLaunchKernelGGL((backward_weight_lanes_kernel<n, CO, T>), dim3(blocks), dim3(64), 0, stream, in, g, dst, s.B,
                       s.Cin, s.Cout, unframed_edge(s), s.M, s.frame, per_slice);
}

template <int n, typename T>
void launch_weight_lanes_n(const T *in, const float *g, float *dst, const Shape &s, int slices, int per_slice,
                           hipStream_t stream)
{
    const int co = weight_co(n, s.Cout);
    if constexpr (regs_fit(n) >= 4)
        if (co == 4) return launch_weight_lanes_co<n, 4, T>(in, g, dst, s, slices, per_slice, stream);
    if constexpr (regs_fit(n) >= 3)
        if (co == 3) return launch_weight_lanes_co<n, 3, T>(in, g, dst, s, slices, per_slice, stream);
    if constexpr (regs_fit(n) >= 2)
        if (co == 2) return launch_weight_lanes_co<n, 2, T>(in, g, dst, s, slices, per_slice, stream);
    launch_weight_lanes_co<n, 1, T>(in, g, dst, s, slices, per_slice, stream);
}

template <typename T>
void launch_weight_lanes(const T *in, const float *g, float *dst, const Shape &s, int slices, int per_slice,
                         hipStream_t stream)
{
    switch (s.n) {
        case 1: return launch_weight_lanes_n<1, T>(in, g, dst, s, slices, per_slice, stream);
        case 2: return launch_weight_lanes_n<2, T>(in, g, dst, s, slices, per_slice, stream);
        case 3: return launch_weight_lanes_n<3, T>(in, g, dst, s, slices, per_slice, stream);
        case 4: return launch_weight_lanes_n<4, T>(in, g, dst, s, slices, per_slice, stream);
        case 5: return launch_weight_lanes_n<5, T>(in, g, dst, s, slices, per_slice, stream);
        case 6: return launch_weight_lanes_n<6, T>(in, g, dst, s, slices, per_slice, stream);
        default: return launch_weight_lanes_n<7, T>(in, g, dst, s, slices, per_slice, stream);
    }
}

// Lanes over input channels pay once a wave's lanes are mostly busy.
bool weight_lanes_apply(const Shape &s) { return s.n <= 7 && s.Cin >= 48; }

// Slices of the position range for that kernel: about 2048 waves, at least 64 positions each.
int weight_lane_slices(const Shape &s)
{
    const long long waves_per_slice = (long long)((s.Cin + 63) / 64) * (s.Cout / weight_co(s.n, s.Cout));
    const long long total = (long long)s.B * (s.N - 2 * s.frame) * (s.N - 2 * s.frame);
    long long slices = (2048 + waves_per_slice - 1) / waves_per_slice;
    if (slices > (total + 63) / 64) slices = (total + 63) / 64;
    return slices < 1 ? 1 : (int)slices;
}

// Slices of the position range: few (co, ci) pairs alone cannot fill the chip.  About 1024
// workgroups, at least 1024 positions per slice.
int weight_slices(const Shape &s)
{
    if (backward_weight_image_apply(s)) return backward_weight_image_slices(s);
    if (weight_lanes_apply(s)) return weight_lane_slices(s);
    long long wgs = (long long)s.Cout * s.Cin;                     // workgroups per slice
    if (s.n <= 7) {
        const int co = weight_co(s.n, s.Cout), ci = weight_ci(s.n, co, s.Cin);
        wgs = (long long)(s.Cout / co) * ((s.Cin + ci - 1) / ci);
    }
    const long long total = (long long)s.B * (s.N - 2 * s.frame) * (s.N - 2 * s.frame);
    long long slices = (1024 + wgs - 1) / wgs;
    if (slices > (total + 1023) / 1024) slices = (total + 1023) / 1024;
    return slices < 1 ? 1 : (int)slices;
}

}  // namespace

// The register-blocked kernels (n <= 7) skip a virtual frame (Shape::frame); the plain ones take
// the framed problem as it is.
bool backward_generic_takes_frame(const Shape &s)
{
    const int N0 = s.N - 2 * s.frame;
    return s.n <= 7 && (size_t)((N0 * N0 + 255) / 256) * ((s.Cin + 3) / 4) * s.B < 0x7fffffffu;
}

hipError_t launch_backward_input_generic(const float *g, const void *w, float *din, const Shape &s, kst_dtype dt,
                                         hipStream_t stream)
{
    if (backward_input_image_apply(s)) return launch_backward_input_image(g, w, din, s, dt, stream);
    if (dt == KST_BF16   ? launch_input_regs<uint16_t>(g, (const uint16_t *)w, din, s, stream)
        : dt == KST_F16 ? launch_input_regs<half_bits>(g, (const half_bits *)w, din, s, stream)
                        : launch_input_regs<float>(g, (const float *)w, din, s, stream))
        return hipGetLastError();
    if (s.frame) return hipErrorInvalidValue;                    // the plain kernel knows no virtual frame
    const size_t total = (size_t)s.B * s.Cin * s.N * s.N;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dt == KST_BF16)
        hipLaunchKernelGGL(backward_input_generic_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream, g,
                           (const uint16_t *)w, din, s.B, s.Cin, s.Cout, s.N, s.M, s.n);
    else if (dt == KST_F16)
        hipLaunchKernelGGL(backward_input_generic_kernel<half_bits>, dim3(blocks), dim3(256), 0, stream, g,
                           (const half_bits *)w, din, s.B, s.Cin, s.Cout, s.N, s.M, s.n);
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
    const int total = s.B * (s.N - 2 * s.frame) * (s.N - 2 * s.frame);
    const int per_slice = (total + slices - 1) / slices;
    const unsigned blocks = (unsigned)s.Cout * (unsigned)s.Cin * (unsigned)slices;
    float *dst = slices > 1 ? (float *)ws : dw;
    bool regs = false;
    if (backward_weight_image_apply(s)) {
        hipError_t e = launch_backward_weight_image(in, g, dst, s, dt, stream);
        if (e != hipSuccess || slices == 1) return e;
        return launch_splitk_reduce((const float *)ws, dw, (size_t)s.Cout * s.Cin * s.n * s.n, slices, stream);
    }
    if (weight_lanes_apply(s)) {
        if (dt == KST_BF16) launch_weight_lanes<uint16_t>((const uint16_t *)in, g, dst, s, slices, per_slice, stream);
        else if (dt == KST_F16) launch_weight_lanes<half_bits>((const half_bits *)in, g, dst, s, slices, per_slice, stream);
        else launch_weight_lanes<float>((const float *)in, g, dst, s, slices, per_slice, stream);
        regs = true;
    } else {
        regs = dt == KST_BF16   ? launch_weight_regs<uint16_t>((const uint16_t *)in, g, dst, s, slices, per_slice, stream)
               : dt == KST_F16 ? launch_weight_regs<half_bits>((const half_bits *)in, g, dst, s, slices, per_slice, stream)
                               : launch_weight_regs<float>((const float *)in, g, dst, s, slices, per_slice, stream);
    }
    if (regs) {
        // the register-blocked kernel has run
    } else if (s.frame) {
        return hipErrorInvalidValue;                             // the plain kernel knows no virtual frame
    } else if (dt == KST_BF16) {
        hipLaunchKernelGGL(backward_weight_generic_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream,
                           (const uint16_t *)in, g, dst, s.B, s.Cin, s.Cout, s.N, s.M, s.n, per_slice);
    } else if (dt == KST_F16) {
        hipLaunchKernelGGL(backward_weight_generic_kernel<half_bits>, dim3(blocks), dim3(256), 0, stream,
                           (const half_bits *)in, g, dst, s.B, s.Cin, s.Cout, s.N, s.M, s.n, per_slice);
    } else {
        hipLaunchKernelGGL(backward_weight_generic_kernel<float>, dim3(blocks), dim3(256), 0, stream, (const float *)in, g,
                           dst, s.B, s.Cin, s.Cout, s.N, s.M, s.n, per_slice);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || slices == 1) return e;
    return launch_splitk_reduce((const float *)ws, dw, (size_t)s.Cout * s.Cin * s.n * s.n, slices, stream);
}

}  // namespace kst
