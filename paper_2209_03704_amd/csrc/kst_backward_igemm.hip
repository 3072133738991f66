// Gradients of the transpose convolution on the matrix cores (fp32): input gradient first,
// kernel gradient below.
//
// End of Section 3.3: the segregated method also serves back-propagation.  With
// g = d(loss)/d(out) and no padding factor,
//
//   din[b][ci][a][c] = sum_co sum_u sum_v g[b][co][2a-u][2c-v] * w[co][ci][u][v]
//
// over the (u, v) whose g index lies inside the M x M map: the forward's products read
// backwards, one for every original input pixel and kernel element, none for an embedded
// zero.  As a GEMM: rows = input channels ci, columns = positions (b, a, c), reduction over
// (co, u, v); the B operand is gathered from g at stride 2.
//
// Tile: 128 positions x 128 input channels per 512-thread workgroup, 8 waves of 64 channels
// x 32 positions (v_mfma_f32_32x32x2f32, 32 accumulators per lane); the reduction walks the
// output channels in chunks of 4.  Per chunk the workgroup stages
//   * the rows of g the tile's positions touch, into a zero-framed LDS image: "virtual"
//     row VR = b * Hv + (y + n - 1), Hv = 2N + n - 2, and column x + n - 1, so that every tap
//     of every position reads inside the image and finds a zero where g has no element;
//   * the chunk's weights w[co][ci][u][v], read as they lie in memory (ci-major runs of n * n
//     floats) and written to LDS as [co][u v][ci] with an odd row stride.
// Both are loaded into registers one chunk ahead of the MFMAs that consume the previous
// chunk from LDS.  Few tiles: the reduction is split over launches' z-range into a workspace
// and summed by the forward path's reduction pass (fixed order).
#include "kst_igemm_common.h"

namespace kst {

namespace {

constexpr int B_TM = 128;        // positions per workgroup
constexpr int B_TCI = 128;       // input channels per workgroup
constexpr int B_THREADS = 512;
constexpr int B_KC = 4;          // output channels per chunk (two MFMA reduction steps)
constexpr int B_WST = B_TCI + 1; // LDS row stride of the staged weights (odd: the transposing writes spread over the banks)
constexpr int B_PX = 16;         // g elements a lane stages per chunk at most

struct BwdParams {
    int B, Cin, Cout, M, n;
    int N, q;              // positions per row and column; zero frame of the input map around them (its
                           // gradient is not wanted): position (a, c) meets g rows 2 (a + q) - u
    int Hv, Wl;            // virtual rows per batch item, LDS columns per row
    int lrows;             // virtual rows staged per channel
    int Mtot;              // B * N * N positions
    int tiles_m, tiles_ci, splits, co_per_split;
    size_t out_elems;
};

template <int n>
__global__ void __launch_bounds__(B_THREADS) backward_input_f32_kernel(const float *__restrict__ g,
                                                                        const float *__restrict__ w,
                                                                        float *__restrict__ dst, BwdParams p)
{
    constexpr int NN = n * n;
    constexpr int WE = B_KC * NN * B_TCI;                        // weight floats per chunk
    constexpr int NWE = WE / B_THREADS;                          // ... per lane
    static_assert(WE % B_THREADS == 0, "whole number of weight elements per lane");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int xplane = p.lrows * p.Wl;                           // floats per staged channel
    float *Xs = lds;                                             // [B_KC][lrows][Wl]
    float *Ws = lds + B_KC * xplane;                             // [B_KC][NN][B_WST]

    unsigned id = blockIdx.x;
    const int tile_m = (int)(id % (unsigned)p.tiles_m);
    id /= (unsigned)p.tiles_m;
    const int tile_ci = (int)(id % (unsigned)p.tiles_ci);
    const int split = (int)(id / (unsigned)p.tiles_ci);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kk = lane >> 5;
    const int wci = wave & 1, wpos = wave >> 1;

    const int NNp = p.N * p.N;
    const int m0 = tile_m * B_TM;
    const int ci0 = tile_ci * B_TCI;
    // first virtual row the tile can touch: position m0's taps u = n - 1 .. 0 read rows 2a .. 2a + n - 1
    const int b0 = m0 / NNp;
    const int a0 = (m0 - b0 * NNp) / p.N;
    const int VR0 = b0 * p.Hv + 2 * (a0 + p.q);

    int m = m0 + wpos * 32 + l32;
    const bool m_valid = m < p.Mtot;
    if (!m_valid) m = p.Mtot - 1;
    const int mb = m / NNp;
    const int mrem = m - mb * NNp;
    const int ma = mrem / p.N, mc = mrem - ma * p.N;
    // LDS offset of this lane's tap (u, v) = (0, 0): row 2a + n - 1, column 2c + n - 1
    const int xbase = (mb * p.Hv + 2 * (ma + p.q) + (n - 1) - VR0) * p.Wl + 2 * (mc + p.q) + (n - 1) + kk * xplane;
    const int wbase = kk * (NN * B_WST) + wci * 64 + l32;

    const int co_begin = split * p.co_per_split;
    const int co_end = min(p.Cout, co_begin + p.co_per_split);

    // ---- staging plan -------------------------------------------------------------------------
    // weights: element e of the chunk = (c, ci, uv) as it lies in memory for a fixed output
    // channel: w[co][ci0 + ci][uv], uv fastest
    unsigned w_off[NWE];
    int w_lds[NWE], w_c[NWE];                      // LDS float index; channel within the chunk, or 1 << 20 when unused
#pragma unroll
    for (int k = 0; k < NWE; ++k) {
        const int e = tid + k * B_THREADS;
        const int c = e / (NN * B_TCI);
        const int rem = e - c * (NN * B_TCI);
        const int ci = rem / NN, uv = rem - ci * NN;
        const bool ok = ci0 + ci < p.Cin;
        w_off[k] = (((unsigned)(co_begin + c) * p.Cin + ci0 + (ok ? ci : 0)) * NN) + uv;
        w_lds[k] = (c * NN + uv) * B_WST + ci;
        w_c[k] = ok ? c : (1 << 20);
    }
    const unsigned w_inc = (unsigned)B_KC * p.Cin * NN;
    // g: element e of the chunk = (c, virtual row, LDS column)
    unsigned x_off[B_PX];
    int x_c[B_PX];
#pragma unroll
    for (int k = 0; k < B_PX; ++k) {
        const int e = tid + k * B_THREADS;
        const int c = e / xplane;
        const int rem = e - c * xplane;
        const int lr = rem / p.Wl, lc = rem - lr * p.Wl;
        const int VR = VR0 + lr;
        const int bb = VR / p.Hv;
        const int y = VR - bb * p.Hv - (n - 1), x = lc - (n - 1);
        const bool ok = e < B_KC * xplane && bb < p.B && y >= 0 && y < p.M && x >= 0 && x < p.M;
        x_off[k] = ok ? ((((unsigned)bb * p.Cout + co_begin + c) * p.M + y) * p.M + x) : 0u;
        x_c[k] = ok ? c : (1 << 20);
    }
    const unsigned x_inc = (unsigned)B_KC * p.M * p.M;

    floatx16 acc[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[h][v] = 0.0f;

    float w_reg[NWE], x_reg[B_PX];
    auto load_chunk = [&](int co_first) {
#pragma unroll
        for (int k = 0; k < NWE; ++k) w_reg[k] = co_first + w_c[k] < co_end ? w[w_off[k]] : 0.0f;
#pragma unroll
        for (int k = 0; k < B_PX; ++k) x_reg[k] = co_first + x_c[k] < co_end ? g[x_off[k]] : 0.0f;
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int k = 0; k < NWE; ++k) Ws[w_lds[k]] = w_reg[k];
#pragma unroll
        for (int k = 0; k < B_PX; ++k)
            if (tid + k * B_THREADS < B_KC * xplane) Xs[tid + k * B_THREADS] = x_reg[k];
    };

    load_chunk(co_begin);
    store_chunk();
    __syncthreads();

    for (int co0 = co_begin; co0 < co_end; co0 += B_KC) {
        // Next chunk's loads (all-zero past the end of this split's channels).
        const int cn = co0 + B_KC;
#pragma unroll
        for (int k = 0; k < NWE; ++k) w_off[k] += w_inc;
#pragma unroll
        for (int k = 0; k < B_PX; ++k) x_off[k] += x_c[k] < B_KC ? x_inc : 0u;
        load_chunk(cn);

#pragma unroll
        for (int c2 = 0; c2 < B_KC; c2 += 2) {
#pragma unroll
            for (int u = 0; u < n; ++u)
#pragma unroll
                for (int v = 0; v < n; ++v) {
                    const float xf = Xs[c2 * xplane + xbase - u * p.Wl - v];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const float wf = Ws[(c2 * NN + u * n + v) * B_WST + wbase + h * 32];
                        acc[h] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf, xf, acc[h], 0, 0, 0);
                    }
                }
        }
        if (cn >= co_end) break;
        __syncthreads();                                         // every wave is done reading this chunk
        store_chunk();
        __syncthreads();
    }

    if (!m_valid) return;
    // acc[h][v]: input channel ci0 + 64 wci + 32 h + 8 (v / 4) + 4 kk + v % 4 at this lane's position
    float *o = dst + (size_t)split * p.out_elems;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int ci = ci0 + wci * 64 + h * 32 + 8 * (v >> 2) + 4 * kk + (v & 3);
            if (ci < p.Cin) o[(((size_t)mb * p.Cin + ci) * p.N + ma) * p.N + mc] = acc[h][v];
        }
}

// The same tile with 16-byte staging, for layers whose rows of g and runs of w are whole float4
// (M, Cin and Cout multiples of 4).  The chunk's weights are copied as they lie in memory
// ([co][ci][u v], one run of 128 n*n floats per output channel) and read back at stride n*n
// (for n = 4 the four float4 of a channel are rotated by ci / 4 so that the 32 channels of an
// MFMA operand do not fall into four banks); the image of g has a frame of 4 columns on the left
// (>= n - 1) and rows of whole float4, so a float4 of g goes to LDS as it is.  All loads are
// free of branches: a lane's list of float4 is fixed, a float4 outside the tensors re-reads
// element 0 and is written as zeros (g) or feeds channels that are never stored (w).
constexpr int V_XF = 4;          // columns of zeros left of the image of g

template <int n>
__global__ void __launch_bounds__(B_THREADS) backward_input_vec_kernel(const float *__restrict__ g,
                                                                        const float *__restrict__ w,
                                                                        float *__restrict__ dst, BwdParams p)
{
    constexpr int NN = n * n;
    constexpr int WSZ = B_TCI * NN;                               // floats per staged output channel
    constexpr int WV = B_KC * WSZ / 4;                            // weight float4 per chunk
    constexpr int NWV = (WV + B_THREADS - 1) / B_THREADS;         // ... per lane
    constexpr int NXV = B_PX / 4;                                 // g float4 per lane per chunk at most
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int xplane = p.lrows * p.Wl;                            // floats per staged channel (Wl a multiple of 4)
    float *Xs = lds;                                              // [B_KC][lrows][Wl]
    float *Ws = lds + B_KC * xplane;                              // [B_KC][B_TCI * NN]

    unsigned id = blockIdx.x;
    const int tile_m = (int)(id % (unsigned)p.tiles_m);
    id /= (unsigned)p.tiles_m;
    const int tile_ci = (int)(id % (unsigned)p.tiles_ci);
    const int split = (int)(id / (unsigned)p.tiles_ci);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kk = lane >> 5;
    const int wci = wave & 1, wpos = wave >> 1;

    const int NNp = p.N * p.N;
    const int m0 = tile_m * B_TM;
    const int ci0 = tile_ci * B_TCI;
    const int b0 = m0 / NNp;
    const int a0 = (m0 - b0 * NNp) / p.N;
    const int VR0 = b0 * p.Hv + 2 * (a0 + p.q);

    int m = m0 + wpos * 32 + l32;
    const bool m_valid = m < p.Mtot;
    if (!m_valid) m = p.Mtot - 1;
    const int mb = m / NNp;
    const int mrem = m - mb * NNp;
    const int ma = mrem / p.N, mc = mrem - ma * p.N;
    // LDS offset of this lane's tap (u, v) = (0, 0): row 2a + n - 1, column 2c + V_XF
    const int xbase = (mb * p.Hv + 2 * (ma + p.q) + (n - 1) - VR0) * p.Wl + 2 * (mc + p.q) + V_XF + kk * xplane;
    // weights of this lane's two channels (h = 0, 1): float offset of element (ci, u v = 0) of
    // output channel kk of a channel pair; for n = 4, one offset per float4 of the channel
    int wrow[2][n == 4 ? 4 : 1];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int ci = wci * 64 + h * 32 + l32;
        if constexpr (n == 4) {
#pragma unroll
            for (int q = 0; q < 4; ++q) wrow[h][q] = kk * WSZ + ci * NN + 4 * ((q + (ci >> 2)) & 3);
        } else {
            wrow[h][0] = kk * WSZ + ci * NN;
        }
    }

    const int co_begin = split * p.co_per_split;
    const int co_end = min(p.Cout, co_begin + p.co_per_split);

    // ---- staging plan -------------------------------------------------------------------------
    unsigned w_off[NWV], w_step[NWV];
    int w_lds[NWV];                                 // float index in Ws, or -1
    const int w_valid4 = (min(B_TCI, p.Cin - ci0) * NN) / 4;     // float4 of one output channel's run inside the tensor
#pragma unroll
    for (int k = 0; k < NWV; ++k) {
        const int e4 = tid + k * B_THREADS;
        const int c = e4 / (WSZ / 4), r = e4 - c * (WSZ / 4);
        const bool in_list = e4 < WV;
        const bool ok = in_list && r < w_valid4;
        w_off[k] = ok ? (((unsigned)(co_begin + c) * p.Cin + ci0) * NN + 4 * r) : 0u;
        w_step[k] = ok ? (unsigned)B_KC * p.Cin * NN : 0u;
        int cell = 4 * r;
        if constexpr (n == 4) {
            const int ci = r >> 2, q = r & 3;
            cell = ci * NN + 4 * ((q + (ci >> 2)) & 3);
        }
        w_lds[k] = in_list ? c * WSZ + cell : -1;
    }
    unsigned x_off[NXV];
    int x_ok[NXV];                                  // 1: inside g, 0: a zero cell of the image, -1: past the image
    const int wl4 = p.Wl >> 2, xp4 = xplane >> 2;
#pragma unroll
    for (int k = 0; k < NXV; ++k) {
        const int e4 = tid + k * B_THREADS;
        const int c = e4 / xp4;
        const int rem = e4 - c * xp4;
        const int lr = rem / wl4, x4 = rem - lr * wl4;
        const int VR = VR0 + lr;
        const int bb = VR / p.Hv;
        const int y = VR - bb * p.Hv - (n - 1), x = 4 * x4 - V_XF;
        const bool in_list = e4 < B_KC * xp4;
        const bool ok = in_list && bb < p.B && y >= 0 && y < p.M && x >= 0 && x < p.M;
        x_off[k] = ok ? ((((unsigned)bb * p.Cout + co_begin + c) * p.M + y) * p.M + x) : 0u;
        x_ok[k] = ok ? 1 : in_list ? 0 : -1;
    }
    const unsigned x_inc = (unsigned)B_KC * p.M * p.M;

    floatx16 acc[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[h][v] = 0.0f;

    float4 w_reg[NWV], x_reg[NXV];
    // Registers <- the chunk at output channel co_first (whole chunks: Cout is a multiple of 4; a
    // chunk past the end re-reads element 0 and is never multiplied); offsets move on afterwards.
    auto load_chunk = [&](int co_first) {
        const bool live = co_first < co_end;                      // wave-uniform
#pragma unroll
        for (int k = 0; k < NWV; ++k) {
            w_reg[k] = *reinterpret_cast<const float4 *>(w + (live ? w_off[k] : 0u));
            w_off[k] += w_step[k];
        }
#pragma unroll
        for (int k = 0; k < NXV; ++k) {
            const float4 v = *reinterpret_cast<const float4 *>(g + (live ? x_off[k] : 0u));
            x_reg[k] = x_ok[k] == 1 ? v : make_float4(0.f, 0.f, 0.f, 0.f);
            x_off[k] += x_ok[k] == 1 ? x_inc : 0u;
        }
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int k = 0; k < NWV; ++k) {
            const float4 v = make_float4(w_reg[k].x, w_reg[k].y, w_reg[k].z, w_reg[k].w);
            if (w_lds[k] >= 0) *reinterpret_cast<float4 *>(Ws + w_lds[k]) = v;
        }
#pragma unroll
        for (int k = 0; k < NXV; ++k) {
            const float4 v = make_float4(x_reg[k].x, x_reg[k].y, x_reg[k].z, x_reg[k].w);
            if (x_ok[k] >= 0) reinterpret_cast<float4 *>(Xs)[tid + k * B_THREADS] = v;
        }
    };

    load_chunk(co_begin);
    store_chunk();
    __syncthreads();

    for (int co0 = co_begin; co0 < co_end; co0 += B_KC) {
        const int cn = co0 + B_KC;
        load_chunk(cn);
#pragma unroll
        for (int c2 = 0; c2 < B_KC; c2 += 2) {
#pragma unroll
            for (int u = 0; u < n; ++u)
#pragma unroll
                for (int v = 0; v < n; ++v) {
                    const float xf = Xs[c2 * xplane + xbase - u * p.Wl - v];
                    const int uv = u * n + v;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        float wf;
                        if constexpr (n == 4) wf = Ws[c2 * WSZ + wrow[h][uv >> 2] + (uv & 3)];
                        else wf = Ws[c2 * WSZ + wrow[h][0] + uv];
                        acc[h] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf, xf, acc[h], 0, 0, 0);
                    }
                }
        }
        if (cn >= co_end) break;
        __syncthreads();                                         // every wave is done reading this chunk
        store_chunk();
        __syncthreads();
    }

    if (!m_valid) return;
    float *o = dst + (size_t)split * p.out_elems;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int ci = ci0 + wci * 64 + h * 32 + 8 * (v >> 2) + 4 * kk + (v & 3);
            if (ci < p.Cin) o[(((size_t)mb * p.Cin + ci) * p.N + ma) * p.N + mc] = acc[h][v];
        }
}

BwdParams plan(const Shape &s)
{
    BwdParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.M = s.M; p.n = s.n;
    p.q = s.frame;
    p.N = s.N - 2 * s.frame;
    p.Hv = 2 * s.N + s.n - 2;
    p.Wl = 2 * s.N + s.n - 2;
    p.Mtot = s.B * p.N * p.N;
    p.tiles_m = (p.Mtot + B_TM - 1) / B_TM;
    // Virtual rows the positions of one tile can touch: from the first position's top tap row to
    // the last position's bottom one; the largest over the tiles.
    p.lrows = 0;
    for (int t = 0; t < p.tiles_m; ++t) {
        const int m0 = t * B_TM, m1 = (m0 + B_TM < p.Mtot ? m0 + B_TM : p.Mtot) - 1;
        const int b0 = m0 / (p.N * p.N), a0 = (m0 - b0 * p.N * p.N) / p.N;
        const int b1 = m1 / (p.N * p.N), a1 = (m1 - b1 * p.N * p.N) / p.N;
        const int rows = (b1 * p.Hv + 2 * (a1 + p.q) + s.n - 1) - (b0 * p.Hv + 2 * (a0 + p.q)) + 1;
        if (rows > p.lrows) p.lrows = rows;
    }
    p.tiles_ci = (s.Cin + B_TCI - 1) / B_TCI;
    const int tiles = p.tiles_m * p.tiles_ci;
    const int chunks = (s.Cout + B_KC - 1) / B_KC;
    p.out_elems = (size_t)s.B * s.Cin * p.N * p.N;
    // Split count: launch rounds on 256 CUs times a tile's share of the reduction, plus the
    // summing pass; a split has to beat the unsplit launch by a tenth to be worth its workspace.
    int splits = 1;
    {
        const double tile_s = (double)B_TM * B_TCI * s.Cout * s.n * s.n / 2.0e11;
        const double out_b = (double)p.out_elems * 4.0;
        double best = (double)((tiles + 255) / 256) * tile_s;
        const double unsplit = best;
        for (int c = 2; c <= 16 && c <= chunks; ++c) {
            const double t = (double)(((size_t)tiles * c + 255) / 256) * tile_s / c + (c + 1) * out_b / 4.0e12;
            if (t < best && t < 0.9 * unsplit) { best = t; splits = c; }
        }
    }
    const int cps = (chunks + splits - 1) / splits;
    p.co_per_split = cps * B_KC;
    p.splits = (chunks + cps - 1) / cps;
    return p;
}

// Geometry of the 16-byte variant: the image of g has V_XF columns of frame on the left and rows
// of whole float4 (largest column read: 2 (N - 1) + V_XF).
BwdParams plan_vec(const Shape &s)
{
    BwdParams p = plan(s);
    p.Wl = (2 * s.N + V_XF - 1 + 3) & ~3;
    return p;
}

size_t lds_bytes_vec(const BwdParams &p)
{
    return ((size_t)B_KC * p.lrows * p.Wl + (size_t)B_KC * B_TCI * p.n * p.n) * sizeof(float);
}

bool vec_applies(const Shape &s)
{
    if ((s.M & 3) || (s.Cin & 3) || (s.Cout & 3)) return false;
    const BwdParams p = plan_vec(s);
    if ((size_t)B_KC * p.lrows * p.Wl / 4 > (size_t)B_THREADS * (B_PX / 4)) return false;
    if (lds_bytes_vec(p) > 160 * 1024) return false;
    return (size_t)s.B * p.Hv < 0x7fffffffu / (size_t)p.Wl;
}

size_t lds_bytes(const BwdParams &p)
{
    return ((size_t)B_KC * p.lrows * p.Wl + (size_t)B_KC * p.n * p.n * B_WST) * sizeof(float);
}

template <int n>
hipError_t launch_n(const float *g, const float *w, float *dst, const BwdParams &p, hipStream_t stream)
{
    const size_t lds = lds_bytes(p);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&backward_input_f32_kernel<n>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)p.tiles_m * p.tiles_ci * p.splits;
    hipLaunchKernelGGL(backward_input_f32_kernel<n>, dim3(blocks), dim3(B_THREADS), lds, stream, g, w, dst, p);
    return hipGetLastError();
}

template <int n>
hipError_t launch_vec_n(const float *g, const float *w, float *dst, const BwdParams &p, hipStream_t stream)
{
    const size_t lds = lds_bytes_vec(p);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&backward_input_vec_kernel<n>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)p.tiles_m * p.tiles_ci * p.splits;
    hipLaunchKernelGGL(backward_input_vec_kernel<n>, dim3(blocks), dim3(B_THREADS), lds, stream, g, w, dst, p);
    return hipGetLastError();
}

}  // namespace

// fp32 weights, kernels up to 5 x 5, a chunk of g that 16 elements per lane can stage, all
// element counts inside 32 bits (the boundary checks the tensors; the virtual image is larger).
bool backward_input_igemm_supported(const Shape &s, kst_dtype dt)
{
    if (dt != KST_F32 || s.n < 1 || s.n > 5) return false;
    // at least 8 channels on either side, or a wide input with a few output channels (a
    // generator's last layer: the reduction is short, the tile of 128 input channels is full)
    if (s.Cin < 8 || (s.Cout < 8 && !(s.Cin >= 64 && s.Cout >= 2))) return false;
    const BwdParams p = plan(s);
    if ((size_t)B_KC * p.lrows * p.Wl > (size_t)B_THREADS * B_PX) return false;
    if (lds_bytes(p) > 160 * 1024) return false;
    if ((size_t)s.B * p.Hv >= 0x7fffffffu / (size_t)p.Wl) return false;
    if ((size_t)p.tiles_m * p.tiles_ci * p.splits >= 0x7fffffffu) return false;
    return true;
}

size_t backward_input_igemm_workspace_bytes(const Shape &s)
{
    const BwdParams p = plan(s);
    return p.splits > 1 ? (((size_t)p.splits * p.out_elems * sizeof(float) + 255) & ~(size_t)255) : 0;
}

hipError_t launch_backward_input_igemm(const float *g, const float *w, float *din, void *ws, const Shape &s,
                                       hipStream_t stream)
{
    if (!backward_input_igemm_supported(s, KST_F32)) return hipErrorInvalidValue;
    const bool vec = vec_applies(s);
    const BwdParams p = vec ? plan_vec(s) : plan(s);
    float *dst = p.splits > 1 ? (float *)ws : din;
    hipError_t e;
    if (vec) {
        switch (s.n) {
            case 1: e = launch_vec_n<1>(g, w, dst, p, stream); break;
            case 2: e = launch_vec_n<2>(g, w, dst, p, stream); break;
            case 3: e = launch_vec_n<3>(g, w, dst, p, stream); break;
            case 4: e = launch_vec_n<4>(g, w, dst, p, stream); break;
            case 5: e = launch_vec_n<5>(g, w, dst, p, stream); break;
            default: return hipErrorInvalidValue;
        }
    } else {
        switch (s.n) {
            case 1: e = launch_n<1>(g, w, dst, p, stream); break;
            case 2: e = launch_n<2>(g, w, dst, p, stream); break;
            case 3: e = launch_n<3>(g, w, dst, p, stream); break;
            case 4: e = launch_n<4>(g, w, dst, p, stream); break;
            case 5: e = launch_n<5>(g, w, dst, p, stream); break;
            default: return hipErrorInvalidValue;
        }
    }
    if (e != hipSuccess) return e;
    if (p.splits > 1) e = launch_splitk_reduce((const float *)ws, din, p.out_elems, p.splits, stream);
    return e;
}

// ---------------------------------------------------------------------------------------------
// Kernel gradient on the matrix cores (fp32):
//
//   dw[co][ci][u][v] = sum_b sum_a sum_c in[b][ci][a][c] * g[b][co][2a-u][2c-v]
//
// over the terms whose g index lies inside the map.  As n * n GEMMs that share their B
// operand: rows = output channels co (A gathered from g at stride 2, shifted by the tap),
// columns = input channels ci, reduction over the positions (b, a, c).
//
// The kernel reads g from a copy framed by n - 1 zeros on every side (made by the caller of the
// launch function), so every tap of every position reads inside that copy and no g load needs a
// bounds check.
//
// Tile: 32 co x 32 or 64 ci x all n * n taps per workgroup of four or eight waves; the taps are
// dealt over four waves (tap t goes to wave t % 4), so a wave holds at most ceil(n * n / 4)
// accumulators per block of 32 input channels.
// The reduction walks chunks: up to 16 consecutive positions of 1, 2, 3, 4 or 6 consecutive input
// rows of one batch item; per chunk the workgroup stages those inputs for its input channels and
// the rows and columns of g the chunk's taps touch for its 32 output channels.  Staging is
// branch-free (every lane has a fixed list of elements: byte offset from the chunk's base address
// and LDS cell) and runs two chunks ahead through registers into the LDS stage that is not being
// multiplied; one barrier per chunk.
// The position range is split over workgroups; the partial sums are added by the forward path's
// reduction pass (fixed order).
namespace {

constexpr int W_T = 32;          // output channels per workgroup; input channels: W_T per block, 1 or 2 blocks
constexpr int W_CW = 16;         // positions per chunk at most
constexpr int W_DUMP = 32;       // floats at the end of an LDS stage that nothing reads
constexpr int W_FOLD_CO = 8;     // output channels at most where (channel, kernel element) pairs are the GEMM's rows

struct BwdWParams {
    int B, Cin, Cout, M, n;
    int N, q;              // edge of `in` as it lies in memory; zero frame the forward put around it
                           // (its products are zeros and are skipped): position (a, c) meets g rows 2 (a + q) - u
    int Mf, Mfs;           // framed copy of g: rows M + 2 (n - 1), elements between its rows (>= Mf)
    int cw;                // positions per chunk and row (even), column chunks per row, rows per chunk
    int ccs, rows;
    int is, gl, gs;        // LDS: floats per staged input channel, columns and floats per staged g channel
    int nchunks, chunks_per_split, splits;
    int tiles_co, tiles_ci;
    int cb;                // blocks of 32 input channels per workgroup
    int halves;            // wave quartets per workgroup
    int co_fast;           // the output-channel tile index runs faster than the input-channel one
    int fold, gc;          // rows are (channel, kernel element) pairs; channels of g staged per chunk
    int slices;            // partial results written (1: the result itself)
    size_t out_elems;
};

// KS: half the positions a chunk takes of one input row (an MFMA takes two); R: consecutive input
// rows of one batch item per chunk (they share all but two of their n rows of g each, and a chunk
// of several rows has that many more MFMAs per barrier: what small maps need).  All chunk
// geometry is a constant expression.
// CB: blocks of 32 input channels per workgroup.  With two, every staged value of g and every A
// fragment read from LDS feeds two MFMAs (4 -> 8 generator layer of 4 x 4 kernels, batch 64:
// 318 -> 252 us; 16 -> 32: 269 -> 240 us), for twice the accumulators and so fewer waves per CU.
// (A tile of 128 input channels on eight waves was measured slower than one of 32: 502 against
// 393 us on the 8 -> 16 generator layer, one workgroup per CU.)
// H: wave quartets per workgroup.  With two, each takes half of a chunk's R rows for all taps
// (two waves per SIMD: one multiplies while the other stages or waits), and the second quartet's
// sums are added to the first's through LDS at the end.
// FOLD: layers with few output channels (Cout * n * n <= 128).  The GEMM's rows are the pairs
// (output channel, kernel element) instead of the output channels with one GEMM per kernel
// element: row block w (32 rows) belongs to wave w, a lane's A operand comes from its own channel
// and tap of the staged g, W_FOLD_CO channels of g are staged, every quartet writes a partial
// result of its own (slot split * H + quartet), straight from the registers (dw is small).
template <int n, int KS, int R, int CB, int H, bool FOLD>
__global__ void __launch_bounds__(256 * H) backward_weight_f32_kernel(const float *__restrict__ in,
                                                                  const float *__restrict__ gf,
                                                                  float *__restrict__ dst, BwdWParams p)
{
    constexpr int NN = n * n;
    // With two channel blocks and a tap count that four waves cannot share evenly (n odd), a wave
    // takes one channel block and every second tap instead of both blocks and every fourth tap:
    // 3 x 3 kernels then keep the waves busy 5 : 5 : 4 : 4 instead of 6 : 4 : 4 : 4.
    constexpr bool PAIR = CB == 2 && !FOLD && NN % 4 != 0;
    constexpr int TSTEP = PAIR ? 2 : 4;                          // taps tw0, tw0 + TSTEP, ... belong to a wave
    constexpr int CBW = PAIR ? 1 : CB;                           // channel blocks a wave multiplies
    constexpr int TW = FOLD ? 1 : PAIR ? (NN + 1) / 2 : (NN + 3) / 4;   // taps (row blocks) per wave at most
    constexpr int GC = FOLD ? W_FOLD_CO : W_T;                   // channels of g staged per chunk
    constexpr int THREADS = 256 * H;
    constexpr int RH = R / H;                                    // rows per quartet
    static_assert(R % H == 0, "rows split evenly");
    constexpr int CW = 2 * KS;                                   // positions per chunk and row
    constexpr int IS = R * CW + 1;                               // odd strides: lanes of different channels hit different banks
    constexpr int GR = n + 2 * (R - 1);                          // rows of g a chunk meets
    constexpr int GL = 2 * CW + n - 2;
    constexpr int GS = GR * GL + ((GR * GL) % 2 == 0 ? 1 : 0);
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int CI_T = W_T * CB;                               // input channels per workgroup
    constexpr int stage = CI_T * IS + GC * GS + W_DUMP;          // floats per stage: [CI_T][R][CW], [GC][GR][GL], dump cells

    // Consecutive workgroups go to consecutive XCDs, each with an L2 of its own.  The split index
    // runs fastest (different splits read different positions of both operands), then the tile
    // index of the larger operand: what one XCD reads of it, the others do not.
    unsigned id = blockIdx.x;
    const int split = (int)(id % (unsigned)p.splits);
    id /= (unsigned)p.splits;
    const unsigned fast = p.co_fast ? p.tiles_co : p.tiles_ci;
    const int t_fast = (int)(id % fast), t_slow = (int)(id / fast);
    const int tile_co = p.co_fast ? t_fast : t_slow, tile_ci = p.co_fast ? t_slow : t_fast;
    const int co0 = tile_co * W_T, ci0 = tile_ci * CI_T;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6) & 3;      // owner of taps wave, wave + 4, ... (or see PAIR)
    const int half = __builtin_amdgcn_readfirstlane(tid >> 8);         // quartet
    const int l32 = lane & 31, kk = lane >> 5;

    // ---- staging plan, the same for every chunk ----------------------------------------------------
    // Input element (ci, r, cc): offset ci * N * N + r * N + cc from the chunk's first input
    // position; it is dropped (zero) when column c0 + cc is past the row.  g element (co, lr, lc):
    // row 2 a0 + lr and column 2 c0 + lc of the framed copy.  A lane past the lists, or a channel
    // past the tensor, repeats channel 0: what it stages is read by no stored output.
    constexpr int n_in = CI_T * R * CW, n_g = GC * GR * GL;
    constexpr int NI = (n_in + THREADS - 1) / THREADS, NG = (n_g + THREADS - 1) / THREADS;
    constexpr int ITEMS = NI + NG;
    unsigned i_off[NI], g_off[NG];                               // byte offsets
    int i_lds[NI], i_cc[NI], g_lds[NG];
    const int dump = stage - W_DUMP + (tid & (W_DUMP - 1));      // where a lane past the lists writes
#pragma unroll
    for (int k = 0; k < NI; ++k) {
        const int e = tid + k * THREADS;
        const int ci = e / (R * CW), rem = e - ci * (R * CW);
        const int r = rem / CW, cc = rem - r * CW;
        const bool ok = e < n_in;
        i_off[k] = 4u * ((ok && ci0 + ci < p.Cin ? (unsigned)(ci0 + ci) * p.N * p.N : 0u) + (ok ? r * p.N + cc : 0));
        i_cc[k] = ok ? cc : (1 << 20);
        i_lds[k] = ok ? ci * IS + rem : dump;
    }
#pragma unroll
    for (int k = 0; k < NG; ++k) {
        const int e = tid + k * THREADS;
        const int co = e / (GR * GL);
        const int rem = e - co * (GR * GL);
        const int lr = rem / GL, lc = rem - lr * GL;
        const bool ok = e < n_g;
        g_off[k] = ok ? 4u * ((co0 + co < p.Cout ? (unsigned)(co0 + co) * p.Mf * p.Mfs : 0u) + (unsigned)lr * p.Mfs + lc) : 0u;
        g_lds[k] = ok ? CI_T * IS + co * GS + rem : dump;
    }

    const int tw0 = PAIR ? wave >> 1 : wave;                     // this wave's first tap
    const int cw0 = PAIR ? wave & 1 : 0;                         // ... and first channel block
    floatx16 acc[TW][CBW];
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int c = 0; c < CBW; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][c][v] = 0.0f;

    const int chunk_begin = split * p.chunks_per_split;
    const int chunk_end = min(p.nchunks, chunk_begin + p.chunks_per_split);
    // B operand: input channel l32 of block 0, this quartet's first row, position 2 k + kk
    const int ibase = l32 * IS + kk + half * RH * CW + cw0 * W_T * IS;
    // A operand: output channel l32, row 0, position 2 k + kk, tap t of this wave (tw0 + TSTEP t): its cell at k = 0
    int abase[TW];
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        if constexpr (FOLD) {
            const int j = min(32 * wave + l32, p.Cout * NN - 1);  // (a row past the last repeats it and is not stored)
            const int co = j / NN, uv = j - co * NN;
            const int u = uv / n, v = uv - u * n;
            abase[t] = CI_T * IS + co * GS + 2 * kk + (n - 1) + (n - 1 - u) * GL - v + 2 * half * RH * GL;
        } else {
            const int uv = min(tw0 + TSTEP * t, NN - 1);         // (a tap past the last is not multiplied)
            const int u = uv / n, v = uv - u * n;
            abase[t] = CI_T * IS + l32 * GS + 2 * kk + (n - 1) + (n - 1 - u) * GL - v + 2 * half * RH * GL;
        }
    }

    // Staging runs through registers, two chunks ahead: while chunk ch is multiplied the registers
    // hold chunk ch + 1; item j of the lists writes its register to the stage that is not being
    // read and reloads it with chunk ch + 2.  The cursor below names the chunk being loaded (past
    // the last chunk it stays on the last one: valid addresses, unused data).
    float i_reg[NI], g_reg[NG];
    const int groups = p.N / R;                                  // row groups per batch item (R divides N)
    int f_ch = min(chunk_begin, p.nchunks - 1);
    int f_cc, f_g, f_b;
    {
        const int rg = f_ch / p.ccs;
        f_cc = f_ch - rg * p.ccs;
        f_b = rg / groups;
        f_g = rg - f_b * groups;
    }
    auto advance = [&]() {
        if (f_ch + 1 < p.nchunks) {
            ++f_ch;
            if (++f_cc == p.ccs) {
                f_cc = 0;
                if (++f_g == groups) { f_g = 0; ++f_b; }
            }
        }
    };
    const char *ip, *gp;
    int f_c0, h_c0 = 0;                                           // first column of the chunk being loaded / held in registers
    auto aim = [&]() {
        const int a0 = f_g * R;
        f_c0 = f_cc * CW;
        ip = reinterpret_cast<const char *>(in + (((size_t)f_b * p.Cin * p.N + a0) * p.N + f_c0));
        gp = reinterpret_cast<const char *>(gf + ((size_t)f_b * p.Cout * p.Mf * p.Mfs + (size_t)(2 * (a0 + p.q)) * p.Mfs +
                                                  2 * (f_c0 + p.q)));
    };
    // An input position past its row is staged as zero (the chunk's last columns may be).
    auto put = [&](int j, int at) {
        if (j < NI)
            lds[at + i_lds[j]] = h_c0 + i_cc[j] < p.N ? i_reg[j] : 0.0f;
        else
            lds[at + g_lds[j - NI]] = g_reg[j - NI];
    };
    auto get = [&](int j) {
        if (j < NI)
            i_reg[j] = *reinterpret_cast<const float *>(ip + (f_c0 + i_cc[j] < p.N ? i_off[j] : 0u));
        else
            g_reg[j - NI] = *reinterpret_cast<const float *>(gp + g_off[j - NI]);
    };

    if (chunk_begin < chunk_end) {
        aim();
        static_for<ITEMS>([&](auto jc) { get(decltype(jc)::value); });
        h_c0 = f_c0;
        advance();
        aim();
        static_for<ITEMS>([&](auto jc) { put(decltype(jc)::value, 0); get(decltype(jc)::value); });
        h_c0 = f_c0;
        advance();
    }
    __syncthreads();

    // The wave issues in order, so whatever stands between two MFMAs delays the second one by all
    // it takes beyond the first one's run time: the items are dealt out over the MFMAs of the taps
    // every wave has (the last tap may belong to fewer waves).  1 x 1 kernels have no such tap
    // (one wave multiplies): there the items go in one block.  (Folded rows: over all MFMA slots.)
    constexpr int TS = FOLD ? 0 : PAIR ? NN / 2 : NN % 4 == 0 ? TW : TW - 1;
    constexpr int SLOTS = TS > 0 ? RH * TS * KS * CBW : 1;
    int cur = 0;
    for (int ch = chunk_begin; ch < chunk_end; ++ch) {
        const float *S = lds + cur;
        const int other = stage - cur;
        aim();
        __builtin_amdgcn_sched_barrier(0);
        float bf[CB][KS], af[2][KS];               // the A values of tap t + 1 are read before tap t is multiplied
        constexpr int CBL = FOLD ? CB : CBW;       // channel blocks whose B values this wave reads
        static_for<RH * TW>([&](auto qc) {
            constexpr int r = decltype(qc)::value / TW, t = decltype(qc)::value % TW;
            if constexpr (t == 0) {
#pragma unroll
                for (int c = 0; c < CBL; ++c)
#pragma unroll
                    for (int k = 0; k < KS; ++k) bf[c][k] = S[ibase + c * W_T * IS + r * CW + 2 * k];
#pragma unroll
                for (int k = 0; k < KS; ++k) af[0][k] = S[abase[0] + 2 * r * GL + 4 * k];
            }
            if constexpr (t + 1 < TW) {
#pragma unroll
                for (int k = 0; k < KS; ++k) af[(t + 1) & 1][k] = S[abase[t + 1] + 2 * r * GL + 4 * k];
            }
            if constexpr (!FOLD && TS == 0 && r == RH / 2 && t == 0)
                static_for<ITEMS>([&](auto jc) { put(decltype(jc)::value, other); get(decltype(jc)::value); });
            if constexpr (FOLD) {
                // a wave without a row block skips the MFMAs, not its share of the staging
                const bool mine = 32 * wave < p.Cout * NN;
                static_for<KS * CB>([&](auto mc) {
                    constexpr int k = decltype(mc)::value / CB, c = decltype(mc)::value % CB;
                    if (mine) acc[0][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[0][k], bf[c][k], acc[0][c], 0, 0, 0);
                    constexpr int slot = (r * KS + k) * CB + c;
                    constexpr int j0 = slot * ITEMS / (RH * KS * CB), j1 = (slot + 1) * ITEMS / (RH * KS * CB);
                    static_for<j1 - j0>([&](auto jc) { put(j0 + decltype(jc)::value, other); get(j0 + decltype(jc)::value); });
                    __builtin_amdgcn_sched_barrier(0);
                });
            }
            // every wave has its taps 0 .. TS - 1; the last one only while it lies inside the kernel
            if (!FOLD && (t < TS || tw0 + TSTEP * t < NN)) {
                static_for<KS * CBW>([&](auto mc) {
                    constexpr int k = decltype(mc)::value / CBW, c = decltype(mc)::value % CBW;
                    acc[t][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t & 1][k], bf[c][k], acc[t][c], 0, 0, 0);
                    if constexpr (t < TS) {
                        constexpr int slot = ((r * TS + t) * KS + k) * CBW + c;
                        constexpr int j0 = slot * ITEMS / SLOTS, j1 = (slot + 1) * ITEMS / SLOTS;
                        static_for<j1 - j0>([&](auto jc) { put(j0 + decltype(jc)::value, other); get(j0 + decltype(jc)::value); });
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            }
        });
        h_c0 = f_c0;
        advance();
        __syncthreads();
        cur = other;
    }

    // ---- epilogue -------------------------------------------------------------------------------
    // acc[t][c][v]: output channel co0 + 8 (v / 4) + 4 kk + v % 4, input channel ci0 + 32 c + l32,
    // tap tw0 + TSTEP t (channel block cw0 + c).  In dw the taps of one (co, ci) lie side by side and the input channels of
    // one co follow each other, so a tile's part of one output channel is ONE run of
    // (channels of the tile) * n * n floats.  Eight output channels at a time go through LDS
    // (the loop's last barrier has passed: nobody reads a stage any more) and leave as whole
    // runs, consecutive lanes writing consecutive floats.  (Straight from the registers a lane's
    // stores lie n * n floats apart: 35-45 us of the 4 x 4 generator layers' 210-220 us.)
    // With two quartets the second one writes its sums first and the first adds its own.
    if constexpr (FOLD) {
        // acc[0][c][v]: row 32 wave + 8 (v / 4) + 4 kk + v % 4 = (co, kernel element), input channel ci0 + 32 c + l32
        float *of = dst + (size_t)(split * H + half) * p.out_elems;
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            const int ci = ci0 + c * W_T + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int j = 32 * wave + 8 * (v >> 2) + 4 * kk + (v & 3);
                const int co = j / NN, uv = j - co * NN;
                if (j < p.Cout * NN && ci < p.Cin) of[((size_t)co * p.Cin + ci) * NN + uv] = acc[0][c][v];
            }
        }
        return;
    }
    constexpr int NP = NN | 1;                                   // odd stride between a channel's taps in LDS
    float *o = dst + (size_t)split * p.out_elems;
    const int run = min(CI_T, p.Cin - ci0) * NN;                 // floats of one output channel's run
    static_for<4>([&](auto vqc) {
        constexpr int vq = decltype(vqc)::value;
        auto cell = [&](int t, int c, int j) { return ((4 * kk + j) * CI_T + (cw0 + c) * W_T + l32) * NP + tw0 + TSTEP * t; };
        if (H == 1 || half == 1) {
            static_for<TW * CBW * 4>([&](auto ec) {
                constexpr int t = decltype(ec)::value / (CBW * 4), c = (decltype(ec)::value / 4) % CBW, j = decltype(ec)::value % 4;
                if (tw0 + TSTEP * t < NN) lds[cell(t, c, j)] = acc[t][c][4 * vq + j];
            });
        }
        __syncthreads();
        if constexpr (H == 2) {
            if (half == 0) {
                static_for<TW * CBW * 4>([&](auto ec) {
                    constexpr int t = decltype(ec)::value / (CBW * 4), c = (decltype(ec)::value / 4) % CBW, j = decltype(ec)::value % 4;
                    if (tw0 + TSTEP * t < NN) lds[cell(t, c, j)] += acc[t][c][4 * vq + j];
                });
            }
            __syncthreads();
        }
        for (int i = tid; i < 8 * CI_T * NN; i += THREADS) {
            const int co8 = i / (CI_T * NN), e = i - co8 * (CI_T * NN);
            const int ci_l = e / NN, uv = e - ci_l * NN;
            const int co = co0 + 8 * vq + co8;
            if (co < p.Cout && e < run) o[((size_t)co * p.Cin + ci0) * NN + e] = lds[(co8 * CI_T + ci_l) * NP + uv];
        }
        if constexpr (vq < 3) __syncthreads();
    });
}

constexpr size_t W_LDS_MAX = 96 * 1024;     // LDS a workgroup of two quartets may take (one runs per CU)

// Few output channels, many input channels (a generator's last layer).
bool weight_folds(const Shape &s) { return s.Cout < 8 && s.Cout * s.n * s.n <= 128 && s.Cin >= 64; }

// Rows per chunk.  One quartet: the largest of 6, 3, 2, 1 that divides N and keeps a chunk within
// 18 MFMA steps per tap (kernels of 3 x 3 and larger with at most 10 positions per row; else one
// row).  Two quartets: 4 or 2 rows (an even number, at most 8 steps per tap and quartet), or 0
// when N is odd (then one quartet does the work).
int weight_rows(int n, int N, int cw, int cb, int halves, int gc)
{
    if (halves == 1 && (n < 3 || cw > 10)) return 1;
    const int cands[4] = {6, 4, 3, 2};
    for (int c : cands) {
        // (6 rows on two quartets would need rows of at most 4 positions, which 6 does not divide)
        if (c % halves != 0 || (c == 4 && halves == 1) || (c == 6 && halves == 2)) continue;
        const int gr = n + 2 * (c - 1), gl = 2 * cw + n - 2;
        const size_t lds = 2 * ((size_t)W_T * cb * (c * cw + 1) + (size_t)gc * (gr * gl + 1) + W_DUMP) * sizeof(float);
        if (N % c == 0 && (c / halves) * (cw / 2) <= (halves == 2 ? 8 : 18) && lds <= (halves == 2 ? W_LDS_MAX : 64 * 1024))
            return c;
    }
    return halves == 2 ? 0 : 1;
}

BwdWParams plan_w(const Shape &s)
{
    BwdWParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.M = s.M; p.n = s.n;
    p.q = s.frame;
    p.N = s.N - 2 * s.frame;
    p.Mf = s.M + 2 * (s.n - 1);
    // Equal chunks of an even number of positions, 16 at most: a row of 18 is cut 10 + 8, not 16 + 2.
    p.ccs = (p.N + W_CW - 1) / W_CW;
    p.cw = (((p.N + p.ccs - 1) / p.ccs) + 1) & ~1;
    // The last chunk of a row may run past it: the input values of those positions are dropped,
    // and the g columns they would meet (up to 2 ccs cw + 2 q + n - 3) are zeros of the framed
    // copy's wider rows.
    p.Mfs = p.Mf > 2 * p.ccs * p.cw + 2 * p.q + s.n - 2 ? p.Mf : 2 * p.ccs * p.cw + 2 * p.q + s.n - 2;
    p.cb = s.Cin > W_T ? 2 : 1;
    // Two quartets where the tile has two channel blocks, an even number of rows fits a chunk and
    // two waves' accumulators fit a SIMD's registers (kernels up to 4 x 4: 128 of 256 each).
    p.halves = p.cb == 2 && s.n >= 2 && s.n <= 4 ? 2 : 1;
    p.fold = weight_folds(s) ? 1 : 0;
    p.gc = p.fold ? W_FOLD_CO : W_T;
    p.rows = weight_rows(s.n, p.N, p.cw, p.cb, p.halves, p.gc);
    if (p.rows == 0) {
        p.halves = 1;
        p.rows = p.fold ? 1 : weight_rows(s.n, p.N, p.cw, p.cb, 1, p.gc);
    } else if (p.fold && p.halves == 1) {
        p.rows = 1;
    }
    const int gr = s.n + 2 * (p.rows - 1);
    p.is = p.rows * p.cw + 1;                          // (the kernel derives the same LDS geometry from cw and rows)
    p.gl = 2 * p.cw + s.n - 2;
    p.gs = gr * p.gl + ((gr * p.gl) % 2 == 0 ? 1 : 0);
    p.nchunks = s.B * (p.N / p.rows) * p.ccs;
    p.tiles_co = p.fold ? 1 : (s.Cout + W_T - 1) / W_T;
    p.tiles_ci = (s.Cin + W_T * p.cb - 1) / (W_T * p.cb);
    p.out_elems = (size_t)s.Cout * s.Cin * s.n * s.n;
    p.co_fast = (double)s.Cout * p.Mf * p.Mfs >= (double)s.Cin * p.N * p.N ? 1 : 0;
    // Split count: the workgroups a CU holds at a time (by their registers) times 256 run together;
    // cost = rounds x chunks per split x the time of a chunk, plus the traffic of the partial sums.
    const int tiles = p.tiles_co * p.tiles_ci;
    // (two-block tiles: counted as one per CU, the setting that measured best)
    const int per_cu = p.cb == 2 ? 1 : s.n <= 3 ? 4 : s.n == 4 ? 3 : 2;
    // MFMA groups a wave runs per row and reduction step (see PAIR in the kernel)
    const int nn = s.n * s.n;
    const int groups_per_wave = p.fold ? p.cb : (p.cb == 2 && nn % 4 != 0) ? (nn + 1) / 2 : (nn + 3) / 4 * p.cb;
    const double chunk_s = (double)per_cu * p.rows * (p.cw / 2) * groups_per_wave * 64.0 / 2.1e9 / 0.45;
    const double out_b = (double)p.out_elems * 4.0;
    int splits = 1;
    double best = 1e30;
    for (int c = 1; c <= (p.fold ? 1024 : 64) && c <= (p.nchunks + 3) / 4; ++c) {
        const double rounds = (double)(((size_t)tiles * c + 256 * per_cu - 1) / (256 * per_cu));
        const double t = rounds * ((p.nchunks + c - 1) / c) * chunk_s + (c > 1 ? (c + 1) * out_b / 4.0e12 : 0.0);
        if (t < best) { best = t; splits = c; }
    }
    p.chunks_per_split = (p.nchunks + splits - 1) / splits;
    p.splits = (p.nchunks + p.chunks_per_split - 1) / p.chunks_per_split;
    p.slices = p.splits * (p.fold ? p.halves : 1);
    return p;
}

size_t lds_bytes_w(const BwdWParams &p)
{
    const size_t stages = 2 * ((size_t)W_T * p.cb * p.is + (size_t)p.gc * p.gs + W_DUMP) * sizeof(float);
    const size_t epilogue = p.fold ? 0 : (size_t)8 * W_T * p.cb * ((p.n * p.n) | 1) * sizeof(float);      // eight output channels of the tile
    return stages > epilogue ? stages : epilogue;
}

template <int n, int KS, int R, int CB, int H, bool FOLD = false>
hipError_t launch_w_k(const float *in, const float *g, float *dst, const BwdWParams &p, hipStream_t stream)
{
    const unsigned blocks = (unsigned)p.tiles_ci * p.tiles_co * p.splits;
    const size_t lds = lds_bytes_w(p);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&backward_weight_f32_kernel<n, KS, R, CB, H, FOLD>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((backward_weight_f32_kernel<n, KS, R, CB, H, FOLD>), dim3(blocks), dim3(256 * H), lds, stream, in, g,
                       dst, p);
    return hipGetLastError();
}

// The instantiations weight_rows can ask for: one quartet with 1, 2, 3 or 6 rows (several rows
// only for 3 x 3 and larger kernels with at most 10 positions per row), two quartets (two channel
// blocks) with 2 or 4 rows.
template <int n, int KS>
hipError_t launch_w_ks(const float *in, const float *g, float *dst, const BwdWParams &p, hipStream_t stream)
{
    if (p.fold) {                                    // two channel blocks; two quartets (2 or 4 rows), or one with one row
        if (p.cb != 2) return hipErrorInvalidValue;
        if (p.halves == 2) {
            if constexpr (n >= 2 && n <= 4) {
                if constexpr (2 * KS <= 8)
                    if (p.rows == 4) return launch_w_k<n, KS, 4, 2, 2, true>(in, g, dst, p, stream);
                if (p.rows == 2) return launch_w_k<n, KS, 2, 2, 2, true>(in, g, dst, p, stream);
            }
            return hipErrorInvalidValue;
        }
        if (p.rows != 1) return hipErrorInvalidValue;
        return launch_w_k<n, KS, 1, 2, 1, true>(in, g, dst, p, stream);
    }
    if (p.halves == 2) {
        if constexpr (n >= 2 && n <= 4) {
            if (p.cb != 2) return hipErrorInvalidValue;
            if constexpr (2 * KS <= 8)
                if (p.rows == 4) return launch_w_k<n, KS, 4, 2, 2>(in, g, dst, p, stream);
            if (p.rows == 2) return launch_w_k<n, KS, 2, 2, 2>(in, g, dst, p, stream);
        }
        return hipErrorInvalidValue;
    }
    if constexpr (n >= 3 && KS <= 5) {
        if constexpr (6 * KS <= 18)
            if (p.rows == 6)
                return p.cb == 2 ? launch_w_k<n, KS, 6, 2, 1>(in, g, dst, p, stream) : launch_w_k<n, KS, 6, 1, 1>(in, g, dst, p, stream);
        if (p.rows == 3)
            return p.cb == 2 ? launch_w_k<n, KS, 3, 2, 1>(in, g, dst, p, stream) : launch_w_k<n, KS, 3, 1, 1>(in, g, dst, p, stream);
        if (p.rows == 2)
            return p.cb == 2 ? launch_w_k<n, KS, 2, 2, 1>(in, g, dst, p, stream) : launch_w_k<n, KS, 2, 1, 1>(in, g, dst, p, stream);
    }
    if (p.rows != 1) return hipErrorInvalidValue;
    return p.cb == 2 ? launch_w_k<n, KS, 1, 2, 1>(in, g, dst, p, stream) : launch_w_k<n, KS, 1, 1, 1>(in, g, dst, p, stream);
}

template <int n>
hipError_t launch_w(const float *in, const float *g, float *dst, const BwdWParams &p, hipStream_t stream)
{
    switch (p.cw / 2) {
        case 1: return launch_w_ks<n, 1>(in, g, dst, p, stream);
        case 2: return launch_w_ks<n, 2>(in, g, dst, p, stream);
        case 3: return launch_w_ks<n, 3>(in, g, dst, p, stream);
        case 4: return launch_w_ks<n, 4>(in, g, dst, p, stream);
        case 5: return launch_w_ks<n, 5>(in, g, dst, p, stream);
        case 6: return launch_w_ks<n, 6>(in, g, dst, p, stream);
        case 7: return launch_w_ks<n, 7>(in, g, dst, p, stream);
        case 8: return launch_w_ks<n, 8>(in, g, dst, p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// fp32 operands, kernels up to 5 x 5, at least 8 channels on either side; element counts
// inside 32 bits are the boundary's business.
bool backward_weight_igemm_supported(const Shape &s, kst_dtype dt)
{
    if (dt != KST_F32 || s.n < 1 || s.n > 5) return false;
    if ((s.Cin < 8 || s.Cout < 8) && !weight_folds(s)) return false;
    const BwdWParams p = plan_w(s);
    // (the staging lists hold byte offsets inside one batch item in 32 bits)
    if ((size_t)s.Cout * p.Mf * p.Mfs * sizeof(float) >= 0xffffffffu) return false;
    if ((size_t)s.Cin * s.N * s.N * sizeof(float) >= 0xffffffffu) return false;
    if (lds_bytes_w(p) > W_LDS_MAX) return false;
    if ((size_t)p.tiles_ci * p.tiles_co * p.splits >= 0x7fffffffu) return false;
    return true;
}

void backward_weight_igemm_g_copy(const Shape &s, int *frame, int *row_stride)
{
    const BwdWParams p = plan_w(s);
    *frame = s.n - 1;
    *row_stride = p.Mfs;
}

size_t backward_weight_igemm_workspace_bytes(const Shape &s)
{
    const BwdWParams p = plan_w(s);
    return p.slices > 1 ? (((size_t)p.slices * p.out_elems * sizeof(float) + 255) & ~(size_t)255) : 0;
}

hipError_t launch_backward_weight_igemm(const float *in, const float *g_framed, float *dw, void *ws, const Shape &s,
                                        hipStream_t stream)
{
    const float *g = g_framed;
    if (!backward_weight_igemm_supported(s, KST_F32)) return hipErrorInvalidValue;
    const BwdWParams p = plan_w(s);
    float *dst = p.slices > 1 ? (float *)ws : dw;
    hipError_t e;
    switch (s.n) {
        case 1: e = launch_w<1>(in, g, dst, p, stream); break;
        case 2: e = launch_w<2>(in, g, dst, p, stream); break;
        case 3: e = launch_w<3>(in, g, dst, p, stream); break;
        case 4: e = launch_w<4>(in, g, dst, p, stream); break;
        case 5: e = launch_w<5>(in, g, dst, p, stream); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    if (p.slices > 1) e = launch_splitk_reduce((const float *)ws, dw, p.out_elems, p.slices, stream);
    return e;
}

}  // namespace kst
