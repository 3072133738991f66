// Layers with many input channels and very few output channels (the output layer of the
// generators of Table 3: 128 -> 3 with a 4 x 4 kernel) on the matrix cores, batched.
//
// Eqs. 7-10 give every output its own few taps, so with the output channels down the MFMA rows
// such a layer fills 3 rows of 16 or 32.  The same multiply-adds, summed in another order, fill
// them: for one input position (i, j) and every tap (u, v) of every sub-kernel
//
//     Y[(u, v, co)][(i, j)] = sum over ci of w[co][ci][u][v] * in[ci][i][j]
//
// is a matrix product with n * n * Cout rows (48 here), the input channels as the reduction and
// the input positions as columns, and an output element is the sum of the Y entries of its
// sub-kernel's taps (Section 3.2: output (y, x) takes tap (u, v) of the input position with
// 2 i + P - u = y, 2 j + P - v = x, where that is a position of the map; u and v run over one
// parity each, which is what selects the sub-kernel).  No product with an inserted or padded
// zero is formed, as in every other kernel here; the padding factor P is only an offset in that
// index relation, so the tensor is read as it lies in memory, whatever P.
//
// A workgroup (8 waves) owns YB output rows of all channels of one batch item.  The input rows
// that reach them (YB / 2 + a halo of (n - 1) / 2) times the map's width are at most 320
// positions = 20 column blocks of 16, two or three per wave.  The weights, regrouped as rows of
// Y, stay in LDS for the whole tile, and a wave's A operand is shared by its column blocks; the
// B operands come straight from memory, 32 channels at a time, the next 32 on their way while
// these are multiplied, with no barrier inside the reduction.  The Y tile then goes to LDS, and
// the waves gather every output's taps from it and store whole output rows.
#include "kst_internal.h"

namespace kst {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int TM_THREADS = 512;
constexpr int TM_WAVES = 8;                     // two per SIMD: one's LDS and index work runs under the other's MFMAs
constexpr int TM_POS = 320;                     // positions per workgroup at most: 20 column blocks of 16
constexpr int TM_CT = (TM_POS / 16 + TM_WAVES - 1) / TM_WAVES;   // column blocks per wave: 3
constexpr int TM_KC = 32;                       // input channels per block of the reduction

struct TapMajorParams {
    int B, Cin, Cout, N0, M, n, P;   // N0: edge of the tensor in memory; M: edge of the planes written; P: padding factor
    int YB;                          // output rows per workgroup
    int XS;                          // floats per row of Y in LDS
    int row_blocks;                  // ceil(M / YB)
    unsigned off[4];                 // element offset of W_p in the segregated weights
    Epilogue epi;
};

// RT: blocks of 16 rows of Y (n * n * Cout <= 16 RT); NK: the kernel edge n.
template <int RT, int NK>
__global__ void __launch_bounds__(TM_THREADS) tapmajor_f32_kernel(const float *__restrict__ in,
                                                                    const float *__restrict__ w_seg,
                                                                    float *__restrict__ out, TapMajorParams p)
{
    constexpr int R16 = 16 * RT;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *Wl = lds;                                // [Cin][R16]
    float *Ys = lds + p.Cin * R16;                  // Y: [R16][p.XS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kgrp = lane >> 4;
    const int b = blockIdx.x / p.row_blocks, rb = blockIdx.x - b * p.row_blocks;
    const int y0 = rb * p.YB;
    const int y1 = min(p.M, y0 + p.YB);             // rows y0 .. y1 - 1
    const int R = p.n * p.n * p.Cout;

    // Input rows that reach these output rows: 2 i + P - u = y for some tap row u.
    const int i_lo = max(0, (y0 - p.P + 1) >> 1);
    const int i_hi = min(p.N0 - 1, (y1 - 1 - p.P + p.n - 1) >> 1);
    const int rows = max(0, i_hi - i_lo + 1);
    const int npos = rows * p.N0;                   // <= TM_POS by the plan; a multiple of 4
    const int ntiles = (npos + 15) >> 4;
    const size_t plane = (size_t)p.N0 * p.N0;
    // (a block of rows that only the zero padding reaches has no input rows: npos = 0, and the loads
    // that are issued regardless read the last row)
    const float *src = in + (size_t)b * p.Cin * plane + (size_t)min(i_lo, p.N0 - 1) * p.N0;

    // ---- B operands straight from memory: lane (channel kgrp of a step, position col of a column block) ------
    // A lane's element of step kk of a block of 32 channels, column block t, is in[ci0 + 4 kk + kgrp][position]:
    // sixteen lanes read 64 consecutive bytes.  A column past the last position re-reads position 0 (its
    // products only reach columns of Y that nobody gathers).  The loads of the next block of channels are in
    // flight while this one is multiplied, and the waves of a workgroup are not held together by barriers
    // in between, so the memory system sees a steady stream.
    int b_off[TM_CT];
#pragma unroll
    for (int t = 0; t < TM_CT; ++t) {
        const int pos = 16 * (wave + TM_WAVES * t) + col;
        b_off[t] = kgrp * (int)plane + (pos < npos ? pos : 0);
    }
    constexpr int KB = TM_KC / 4;                   // steps per block of channels
    float cur[TM_CT][KB], nxt[TM_CT][KB];
    auto load_block = [&](float (&dst)[TM_CT][KB], int ci0) {
#pragma unroll
        for (int kk = 0; kk < KB; ++kk)
#pragma unroll
            for (int t = 0; t < TM_CT; ++t) dst[t][kk] = src[(size_t)(ci0 + 4 * kk) * plane + b_off[t]];
    };
    load_block(cur, 0);

    // ---- the weights as rows of Y: row (u n + v) Cout + co, zero beyond R ------------------
    // Where row rho of channel ci lies in the segregated buffer: first[rho] + ci * stride[rho], worked
    // out once per row (the divisions), then sixteen values per lane in flight.
    {
        int *first = reinterpret_cast<int *>(Ys);   // [R16], then stride[R16]: the place of Y is still free
        int *stride = first + R16;
        if (tid < R16) {
            int fo = -1, st = 0;
            if (tid < R) {
                const int tap = tid / p.Cout, co = tid - tap * p.Cout;
                const int u = tap / p.n, v = tap - u * p.n;
                const int cls = 2 * (u & 1) + (v & 1);
                const int Tb = taps_for_parity(p.n, v & 1);
                const int Tp = taps_for_parity(p.n, u & 1) * Tb;
                fo = (int)p.off[cls] + ((u >> 1) * Tb + (v >> 1)) * p.Cout + co;
                st = Tp * p.Cout;
            }
            first[tid] = fo;
            stride[tid] = st;
        }
        __syncthreads();
        const int W = p.Cin * R16;
        for (int e0 = 0; e0 < W; e0 += 16 * TM_THREADS) {
            float val[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int e = e0 + k * TM_THREADS + tid;
                const int ci = e / R16, rho = e - ci * R16;     // (a constant divisor)
                const int fo = e < W ? first[rho] : -1;
                val[k] = fo >= 0 ? w_seg[fo + ci * stride[rho]] : 0.0f;
            }
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int e = e0 + k * TM_THREADS + tid;
                if (e < W) Wl[e] = val[k];
            }
        }
        __syncthreads();                            // the weights are in place
    }

    floatx4 acc[TM_CT][RT];
#pragma unroll
    for (int c = 0; c < TM_CT; ++c)
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[c][r] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (int ci0 = 0; ci0 < p.Cin; ci0 += TM_KC) {
        if (ci0 + TM_KC < p.Cin) load_block(nxt, ci0 + TM_KC);      // uniform
        // A: lane (row col of a row block, channel kgrp of a step).
#pragma unroll
        for (int kk = 0; kk < KB; ++kk) {
            float a[RT];
#pragma unroll
            for (int r = 0; r < RT; ++r) a[r] = Wl[(ci0 + 4 * kk + kgrp) * R16 + 16 * r + col];
#pragma unroll
            for (int t = 0; t < TM_CT; ++t) {
                if (wave + TM_WAVES * t < ntiles) {               // uniform over the wave
#pragma unroll
                    for (int r = 0; r < RT; ++r)
                        acc[t][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r], cur[t][kk], acc[t][r], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < TM_CT; ++t)
#pragma unroll
            for (int kk = 0; kk < KB; ++kk) cur[t][kk] = nxt[t][kk];
    }

    // ---- Y -> LDS: lane holds rows 16 r + 4 kgrp + v of position col of its column blocks -----
#pragma unroll
    for (int t = 0; t < TM_CT; ++t) {
        const int tile = wave + TM_WAVES * t;
        if (tile < ntiles) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int v = 0; v < 4; ++v) Ys[(16 * r + 4 * kgrp + v) * p.XS + 16 * tile + col] = acc[t][r][v];
        }
    }
    __syncthreads();

    // ---- every output gathers the taps of its sub-kernel -------------------------------------
    // A wave takes whole output rows (of one channel), its lanes run along the row.
    const bool epi = epi_on(p.epi);
    const int yrows = y1 - y0;
    for (int rr = wave; rr < p.Cout * yrows; rr += TM_WAVES) {
        const int co = rr / yrows, y = y0 + rr - co * yrows;    // uniform over the wave
        const float bias = epi ? epi_bias(p.epi, co) : 0.0f;
        float *orow = out + (((size_t)b * p.Cout + co) * p.M + y) * p.M;
        // The row's tap rows: u = u0, u0 + 2, ... (2 i = y - P + u), at most (n + 1) / 2 of them.
        const int u0 = (y - p.P) & 1;
        for (int x = lane; x < p.M; x += 64) {
            const int v0 = (x - p.P) & 1;
            float sum = 0.0f;
            // All loads of an output are issued together: a tap that does not exist, or whose input position lies
            // outside the map, reads a valid cell and adds zero.
#pragma unroll
            for (int a = 0; a < (NK + 1) / 2; ++a) {
                const int u = u0 + 2 * a, i = (y - p.P + u) >> 1;
                const bool u_ok = u < NK && i >= 0 && i < p.N0;          // uniform over the wave
                const float *yr = Ys + ((u_ok ? u : 0) * NK * p.Cout + co) * p.XS + (u_ok ? i - i_lo : 0) * p.N0;
#pragma unroll
                for (int bq = 0; bq < (NK + 1) / 2; ++bq) {
                    const int v = v0 + 2 * bq, j = (x - p.P + v) >> 1;
                    const bool ok = u_ok && v < NK && j >= 0 && j < p.N0;
                    const float val = yr[(v < NK ? v : 0) * p.Cout * p.XS + (ok ? j : 0)];
                    sum += ok ? val : 0.0f;
                }
            }
            if (epi) sum = epi_apply(sum, bias, p.epi.act);
            orow[x] = sum;
        }
    }
}

bool tapmajor_plan(const Shape &s, TapMajorParams &p, size_t &lds)
{
    const int R = s.n * s.n * s.Cout;
    if (s.n < 2 || s.n > 7 || s.Cout > 4 || R > 64 || s.Ns != s.N) return false;
    if (s.Cin % TM_KC != 0 || s.Cin < 2 * TM_KC) return false;
    // (None of the conditions depends on Shape::crop: the launch is planned before it is known.)
    const int N0 = s.N - 2 * s.frame;
    if (N0 < 4 || (N0 & 3) != 0) return false;
    const int rt = (R + 15) / 16;
    // Output rows per workgroup: as many (even, at most 32) as keep the input rows that reach them within TM_POS positions.
    int YB = 0;
    for (int yb = 32; yb >= 2; yb -= 2)
        if (((yb + s.n) / 2) * N0 <= TM_POS) { YB = yb; break; }
    if (YB == 0) return false;
    if ((long long)s.B * ((s.M + YB - 1) / YB) < 128) return false;      // too few workgroups for the chip
    p.XS = ((YB + s.n) / 2) * N0 + 16;
    lds = ((size_t)s.Cin * 16 * rt + (size_t)16 * rt * p.XS) * sizeof(float);
    if (lds > 150 * 1024) return false;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.n = s.n;
    p.N0 = N0;
    p.M = s.M - 2 * s.crop;
    p.P = 2 * s.frame - s.crop;
    if (p.M < 1 || p.P < 0) return false;
    p.YB = YB;
    p.row_blocks = (p.M + YB - 1) / YB;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, KST_F32);
    p.epi = s.epi;
    return true;
}

template <int RT, int NK>
hipError_t launch_rt(const float *in, const float *w_seg, float *out, const TapMajorParams &p, size_t lds, hipStream_t stream)
{
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tapmajor_f32_kernel<RT, NK>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((tapmajor_f32_kernel<RT, NK>), dim3((unsigned)(p.B * p.row_blocks)), dim3(TM_THREADS), lds, stream, in,
                       w_seg, out, p);
    return hipGetLastError();
}

// The row blocks a kernel edge can need with one to four output channels: ceil(n * n * Cout / 16) <= 4.
template <int NK>
hipError_t launch_n(const float *in, const float *w_seg, float *out, const TapMajorParams &p, size_t lds, hipStream_t stream)
{
    const int rt = (NK * NK * p.Cout + 15) / 16;
    if constexpr (NK * NK <= 16)
        if (rt == 1) return launch_rt<1, NK>(in, w_seg, out, p, lds, stream);
    if constexpr (NK * NK <= 32 && NK * NK * 4 > 16)
        if (rt == 2) return launch_rt<2, NK>(in, w_seg, out, p, lds, stream);
    if constexpr (NK * NK <= 48 && NK * NK * 4 > 32)
        if (rt == 3) return launch_rt<3, NK>(in, w_seg, out, p, lds, stream);
    if constexpr (NK * NK * 4 > 48)
        if (rt == 4) return launch_rt<4, NK>(in, w_seg, out, p, lds, stream);
    return hipErrorInvalidValue;
}

}  // namespace

bool tapmajor_f32_supported(const Shape &s)
{
    TapMajorParams p;
    size_t lds;
    return tapmajor_plan(s, p, lds);
}

hipError_t launch_tapmajor_f32(const float *in, const float *w_seg, float *out, const Shape &s, hipStream_t stream)
{
    TapMajorParams p;
    size_t lds;
    if (!tapmajor_plan(s, p, lds)) return hipErrorInvalidValue;
    switch (s.n) {
        case 2: return launch_n<2>(in, w_seg, out, p, lds, stream);
        case 3: return launch_n<3>(in, w_seg, out, p, lds, stream);
        case 4: return launch_n<4>(in, w_seg, out, p, lds, stream);
        case 5: return launch_n<5>(in, w_seg, out, p, lds, stream);
        case 6: return launch_n<6>(in, w_seg, out, p, lds, stream);
        case 7: return launch_n<7>(in, w_seg, out, p, lds, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace kst
