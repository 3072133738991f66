// Matrix-core (MFMA) segregated forward pass, fp32 operands and arithmetic.
//
// Section 3.3, Eqs. 7-10, as four implicit GEMMs that share one input tile:
// for parity class p = (r, s)
//     C_p[co][m] = sum_k  W_p[co][k] * X_p[k][m],   k = (ci, a, b'),  m = (b, i, j)
// with X_p[k][m] = in[b][ci][i + r + a][j + s + b'] gathered on the fly from an
// LDS copy of the input rows the tile touches (never materialised), and the
// four C_p interleaved into out[b][co][2i + r][2j + s] on the way out.
//
// Output channels run down the MFMA rows and quad positions run across its
// columns, so that for one accumulator register the 32 lanes of a half-wave
// hold 32 consecutive quads of one output row: the s = 0 / s = 1 accumulators
// pair up into 8-byte stores that tile a contiguous row segment.
//
// Positions are numbered m = (b*E + i)*E + j over the E x E quad grid
// (E = ceil(M/2)); a workgroup owns TM consecutive positions for TCO output
// channels and all four classes.  Odd M: the phantom last row/column members
// are computed (their reads stay inside the map) and not stored.
#include "kst_igemm_common.h"

namespace kst {

constexpr int G_KC = 4;          // input channels staged per step (even)

template <int n>
__global__ void __launch_bounds__(G_THREADS) igemm_f32_kernel(const float *__restrict__ in,
                                                                const float *__restrict__ w_seg,
                                                                float *__restrict__ dst, IgemmParams p)
{
    constexpr int fl = n / 2;
    constexpr int NN = n * n;
    extern __shared__ float lds[];
    const int xplane = p.lrows * p.N;            // floats per staged channel
    float *Xs = lds;                             // [G_KC][lrows*N]
    float *Ws = lds + G_KC * xplane;             // [G_KC][NN][G_TCO]

    unsigned id = blockIdx.x;
    const int tile_m = (int)(id % (unsigned)p.tiles_m);
    id /= (unsigned)p.tiles_m;
    const int tile_co = (int)(id % (unsigned)p.tiles_co);
    const int split = (int)(id / (unsigned)p.tiles_co);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kk = lane >> 5;
    const int wco = wave & 1, wpos = wave >> 1;

    const int m0 = tile_m * G_TM;
    const int co0 = tile_co * G_TCO;
    const int b0 = m0 / p.EE;
    const int i0 = (m0 - b0 * p.EE) / p.E;
    const int R0 = b0 * p.N + i0;                // first stacked input row of the tile

    // This lane's quad position (clamped so that every LDS read stays inside the tile).
    int m = m0 + wpos * 32 + l32;
    const bool m_valid = m < p.Mtot;
    if (!m_valid) m = p.Mtot - 1;
    const int mb = m / p.EE;
    const int mrem = m - mb * p.EE;
    const int mi = mrem / p.E, mj = mrem - mi * p.E;
    const int xbase = ((mb * p.N + mi) - R0) * p.N + mj + kk * xplane;
    const int wbase = kk * (NN * G_TCO) + wco * 64 + l32;

    floatx16 acc[4][2];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][h][v] = 0.0f;

    const int ci_begin = split * p.ci_per_split;
    const int ci_end = min(p.Cin, ci_begin + p.ci_per_split);

    for (int ci0 = ci_begin; ci0 < ci_end; ci0 += G_KC) {
        if (ci0 != ci_begin) __syncthreads();
        // Stage the input rows [R0, R0 + lrows) of channels ci0 .. ci0+KC-1.
        for (int e = tid; e < G_KC * xplane; e += G_THREADS) {
            const int c = e / xplane;
            const int rem = e - c * xplane;
            const int lr = rem / p.N, x = rem - lr * p.N;
            const int R = R0 + lr;
            const int bb = R / p.N, y = R - bb * p.N;
            float v = 0.0f;
            if (bb < p.B && ci0 + c < ci_end)
                v = in[(((size_t)bb * p.Cin + ci0 + c) * p.N + y) * p.N + x];
            Xs[e] = v;
        }
        // Stage the weights of those channels: all taps of all classes, TCO channels.
        for (int e = tid; e < G_KC * NN * G_TCO; e += G_THREADS) {
            const int tco = e % G_TCO;
            const int rest = e / G_TCO;
            const int T = rest % NN, c = rest / NN;
            int cls = 0;
#pragma unroll
            for (int q = 1; q < 4; ++q)
                if (T >= class_tap_base(n, q)) cls = q;
            const int Tp = class_taps(n, cls);
            const int t = T - class_tap_base(n, cls);
            float v = 0.0f;
            if (co0 + tco < p.Cout && ci0 + c < ci_end)
                v = w_seg[p.off[cls] + ((size_t)(ci0 + c) * Tp + t) * p.Cout + co0 + tco];
            Ws[e] = v;
        }
        __syncthreads();

#pragma unroll
        for (int c2 = 0; c2 < G_KC; c2 += 2) {
            // Input fragments for every window offset (dy, dx): shared by all classes.
            float xf[fl + 1][fl + 1];
#pragma unroll
            for (int dy = 0; dy <= fl; ++dy)
#pragma unroll
                for (int dx = 0; dx <= fl; ++dx)
                    xf[dy][dx] = Xs[c2 * xplane + xbase + dy * p.N + dx];
#pragma unroll
            for (int cls = 0; cls < 4; ++cls) {
                const int r = cls >> 1, s = cls & 1;
                const int Ta = taps_for_parity(n, r), Tb = taps_for_parity(n, s);
#pragma unroll
                for (int a = 0; a < Ta; ++a)
#pragma unroll
                    for (int bq = 0; bq < Tb; ++bq) {
                        const int T = class_tap_base(n, cls) + a * Tb + bq;
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const float wf = Ws[(c2 * NN + T) * G_TCO + wbase + h * 32];
                            acc[cls][h] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf, xf[r + a][s + bq], acc[cls][h], 0, 0, 0);
                        }
                    }
            }
        }
    }

    // Epilogue: interleave the four classes; lanes l32 = consecutive quads of a row.
    if (!m_valid) return;
    igemm_store(dst + (size_t)split * p.out_elems, acc, p, co0 + wco * 64, kk, mb, mi, mj);
}

// ---------------------------------------------------------------------------
// Pipelined variant (N and Cout multiples of 4): the same tile and MFMA loop,
// but operands are staged with 16-byte loads whose addresses are worked out
// once per lane before the channel loop, and the loads of chunk k+1 are in
// flight (into registers) while chunk k is multiplied out of LDS.
// ---------------------------------------------------------------------------
constexpr int P_NX4 = 2;         // input float4 per lane per chunk at most

// What a lane needs to know about its column of the tile when the accumulators are stored.
struct PipeLane {
    int mb, mi, mj;      // batch item and quad of this lane's position
    bool m_valid;        // false for lanes past the last position (they computed a clamped copy)
};

// Geometry of lane `tid` in position tile `tile_m` (no memory access).
__device__ __forceinline__ PipeLane pipe_lane(const IgemmParams &p, int tile_m, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    int m = tile_m * G_TM + (wave >> 1) * 32 + (lane & 31);
    PipeLane L;
    L.m_valid = m < p.Mtot;
    if (!L.m_valid) m = p.Mtot - 1;
    L.mb = m / p.EE;
    const int mrem = m - L.mb * p.EE;
    L.mi = mrem / p.E;
    L.mj = mrem - L.mi * p.E;
    return L;
}

// acc = the tile's sums over input channels [ci_begin, ci_end).  Every thread of the workgroup
// calls it; LDS is free to be overwritten once all of them have passed a barrier afterwards.
template <int n>
__device__ __forceinline__ void pipe_accumulate(const float *__restrict__ in, const float *__restrict__ w_seg,
                                                const IgemmParams &p, float *lds, int tile_m, int tile_co,
                                                int ci_begin, int ci_end, const PipeLane &L, int tid,
                                                floatx16 (&acc)[4][2])
{
    constexpr int fl = n / 2;
    constexpr int NN = n * n;
    constexpr int W4 = G_KC * NN * (G_TCO / 4);                  // weight float4 per chunk
    constexpr int NW4 = (W4 + G_THREADS - 1) / G_THREADS;        // ... per lane
    const int xplane = p.lrows * p.Ns;                           // floats per staged channel (multiple of 4)
    float *Xs = lds;                                             // [G_KC][xplane]
    float *Ws = lds + G_KC * xplane;                             // [G_KC][NN][G_TCO]

    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kk = lane >> 5;
    const int wco = wave & 1;

    const int m0 = tile_m * G_TM;
    const int co0 = tile_co * G_TCO;
    const int b0 = m0 / p.EE;
    const int i0 = (m0 - b0 * p.EE) / p.E;
    const int R0 = b0 * p.N + i0;

    const int xbase = ((L.mb * p.N + L.mi) - R0) * p.Ns + L.mj + kk * xplane;
    const int wbase = kk * (NN * G_TCO) + wco * 64 + l32;

    // ---- staging plan: where each of this lane's float4 comes from and goes to -------------
    unsigned w_off[NW4], w_inc[NW4];
    int w_c[NW4];                                   // channel within the chunk, or 1 << 20 when unused
#pragma unroll
    for (int k = 0; k < NW4; ++k) {
        const int e4 = tid + k * G_THREADS;
        const int tco4 = e4 & (G_TCO / 4 - 1);
        const int rest = e4 / (G_TCO / 4);
        const int T = rest % NN, c = rest / NN;
        int cls = 0;
#pragma unroll
        for (int q = 1; q < 4; ++q)
            if (T >= class_tap_base(n, q)) cls = q;
        const int Tp = cls == 0 ? class_taps(n, 0) : cls == 1 ? class_taps(n, 1) : cls == 2 ? class_taps(n, 2) : class_taps(n, 3);
        const int tb = cls == 0 ? 0 : cls == 1 ? class_tap_base(n, 1) : cls == 2 ? class_tap_base(n, 2) : class_tap_base(n, 3);
        const bool ok = e4 < W4 && co0 + 4 * tco4 < p.Cout;
        w_off[k] = p.off[cls] + ((unsigned)(ci_begin + c) * Tp + (T - tb)) * p.Cout + co0 + 4 * tco4;
        w_inc[k] = (unsigned)G_KC * Tp * p.Cout;
        w_c[k] = ok ? c : (1 << 20);
    }
    const int xp4 = xplane >> 2, n4 = p.Ns >> 2;
    unsigned x_off[P_NX4];
    int x_c[P_NX4];
#pragma unroll
    for (int k = 0; k < P_NX4; ++k) {
        const int e4 = tid + k * G_THREADS;
        const int c = e4 / xp4;
        const int rem = e4 - c * xp4;
        const int lr = rem / n4, x4 = rem - lr * n4;
        const int R = R0 + lr;
        const int bb = R / p.N, y = R - bb * p.N;
        const bool ok = e4 < G_KC * xp4 && bb < p.B;
        x_off[k] = (((unsigned)bb * p.Cin + ci_begin + c) * p.N + y) * p.Ns + 4 * x4;
        x_c[k] = ok ? c : (1 << 20);
    }
    const unsigned x_inc = (unsigned)G_KC * p.N * p.Ns;

#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][h][v] = 0.0f;

    float4 w_reg[NW4], x_reg[P_NX4];
    // Chunk at ci_begin -> registers -> LDS.
#pragma unroll
    for (int k = 0; k < NW4; ++k)
    {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ci_begin + w_c[k] < ci_end) v = *reinterpret_cast<const float4 *>(w_seg + w_off[k]);
        w_reg[k] = v;
    }
#pragma unroll
    for (int k = 0; k < P_NX4; ++k)
    {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ci_begin + x_c[k] < ci_end) v = *reinterpret_cast<const float4 *>(in + x_off[k]);
        x_reg[k] = v;
    }
#pragma unroll
    for (int k = 0; k < NW4; ++k)
        if (tid + k * G_THREADS < W4) reinterpret_cast<float4 *>(Ws)[tid + k * G_THREADS] = w_reg[k];
#pragma unroll
    for (int k = 0; k < P_NX4; ++k)
        if (tid + k * G_THREADS < G_KC * xp4) reinterpret_cast<float4 *>(Xs)[tid + k * G_THREADS] = x_reg[k];
    __syncthreads();

    for (int ci0 = ci_begin; ci0 < ci_end; ci0 += G_KC) {
        // Next chunk's loads (all-zero past the end of this range of channels).
        const int cn = ci0 + G_KC;
#pragma unroll
        for (int k = 0; k < NW4; ++k) {
            w_off[k] += w_inc[k];
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (cn + w_c[k] < ci_end) v = *reinterpret_cast<const float4 *>(w_seg + w_off[k]);
            w_reg[k] = v;
        }
#pragma unroll
        for (int k = 0; k < P_NX4; ++k) {
            x_off[k] += x_inc;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (cn + x_c[k] < ci_end) v = *reinterpret_cast<const float4 *>(in + x_off[k]);
            x_reg[k] = v;
        }

#pragma unroll
        for (int c2 = 0; c2 < G_KC; c2 += 2) {
            float xf[fl + 1][fl + 1];
#pragma unroll
            for (int dy = 0; dy <= fl; ++dy)
#pragma unroll
                for (int dx = 0; dx <= fl; ++dx)
                    xf[dy][dx] = Xs[c2 * xplane + xbase + dy * p.Ns + dx];
#pragma unroll
            for (int cls = 0; cls < 4; ++cls) {
                const int r = cls >> 1, s = cls & 1;
                const int Ta = taps_for_parity(n, r), Tb = taps_for_parity(n, s);
#pragma unroll
                for (int a = 0; a < Ta; ++a)
#pragma unroll
                    for (int bq = 0; bq < Tb; ++bq) {
                        const int T = class_tap_base(n, cls) + a * Tb + bq;
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const float wf = Ws[(c2 * NN + T) * G_TCO + wbase + h * 32];
                            acc[cls][h] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf, xf[r + a][s + bq], acc[cls][h], 0, 0, 0);
                        }
                    }
            }
        }
        if (cn >= ci_end) break;
        __syncthreads();                                         // every wave is done reading this chunk
#pragma unroll
        for (int k = 0; k < NW4; ++k)
            if (tid + k * G_THREADS < W4) reinterpret_cast<float4 *>(Ws)[tid + k * G_THREADS] = w_reg[k];
#pragma unroll
        for (int k = 0; k < P_NX4; ++k)
            if (tid + k * G_THREADS < G_KC * xp4) reinterpret_cast<float4 *>(Xs)[tid + k * G_THREADS] = x_reg[k];
        __syncthreads();
    }
}

template <int n>
__global__ void __launch_bounds__(G_THREADS) igemm_f32_pipe_kernel(const float *__restrict__ in,
                                                                     const float *__restrict__ w_seg,
                                                                     float *__restrict__ dst, IgemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    unsigned id = blockIdx.x;
    const int tile_m = (int)(id % (unsigned)p.tiles_m);
    id /= (unsigned)p.tiles_m;
    const int tile_co = (int)(id % (unsigned)p.tiles_co);
    const int split = (int)(id / (unsigned)p.tiles_co);
    const int ci_begin = split * p.ci_per_split;
    const int ci_end = min(p.Cin, ci_begin + p.ci_per_split);

    const PipeLane L = pipe_lane(p, tile_m, threadIdx.x);
    floatx16 acc[4][2];
    pipe_accumulate<n>(in, w_seg, p, lds, tile_m, tile_co, ci_begin, ci_end, L, (int)threadIdx.x, acc);
    if (!L.m_valid) return;
    const int wave = threadIdx.x >> 6, kk = (threadIdx.x & 63) >> 5;
    igemm_store(dst + (size_t)split * p.out_elems, acc, p, tile_co * G_TCO + (wave & 1) * 64, kk, L.mb, L.mi, L.mj);
}

// ---------------------------------------------------------------------------
// Even shares ("stream-K"): the (tile, channel chunk) pairs of the whole layer, tile-major, are
// one list cut into SK_GRID equal ranges, one per persistent workgroup (one workgroup fits a
// CU), so every CU multiplies for the same time whatever the tile count.  A range is a run of
// pieces, each a span of chunks of one tile.  A piece that covers its tile's whole reduction is
// stored straight to the output; any other is written raw (the accumulator registers, lane by
// lane) to one of the workgroup's two slots: slot 2g for the first piece of workgroup g's range,
// 2g + 1 for a later one (only the last can be partial then).  A second kernel adds the slots of
// every tile that has more than one contributor in workgroup order (deterministic) and stores.
// ---------------------------------------------------------------------------
constexpr int SK_GRID = 256;                                  // CUs of the chip
constexpr size_t SK_SLOT_FLOATS = (size_t)G_TM * G_TCO * 4;   // one tile's accumulators

struct StreamK {
    int chunks;                // channel chunks per tile
    int grid;                  // workgroups (<= SK_GRID, <= units)
    unsigned long long units;  // tiles * chunks
};

__device__ __forceinline__ unsigned long long sk_begin(const StreamK &k, int g)
{
    return (unsigned long long)g * k.units / (unsigned)k.grid;
}

template <int n>
__global__ void __launch_bounds__(G_THREADS) igemm_f32_streamk_kernel(const float *__restrict__ in,
                                                                        const float *__restrict__ w_seg,
                                                                        float *__restrict__ out, float *__restrict__ ws,
                                                                        IgemmParams p, StreamK k)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int g = blockIdx.x;
    const int tid = threadIdx.x;
    unsigned long long u = sk_begin(k, g);
    const unsigned long long u_end = sk_begin(k, g + 1);
    bool first = true;
    while (u < u_end) {
        const int tile = (int)(u / (unsigned)k.chunks);
        const int c0 = (int)(u - (unsigned long long)tile * k.chunks);
        const unsigned long long left = u_end - u;
        const int c1 = left < (unsigned long long)(k.chunks - c0) ? c0 + (int)left : k.chunks;
        const int tile_m = tile % p.tiles_m, tile_co = tile / p.tiles_m;
        if (!first) __syncthreads();                 // the previous piece's last LDS reads are done
        // A fresh copy of the lane number the compiler cannot see through: the staging plan is then
        // worked out anew for every piece instead of being kept in registers across the pieces.
        int tid_p = tid;
        asm volatile("" : "+v"(tid_p));
        const PipeLane L = pipe_lane(p, tile_m, tid_p);
        floatx16 acc[4][2];
        pipe_accumulate<n>(in, w_seg, p, lds, tile_m, tile_co, c0 * G_KC, min(p.Cin, c1 * G_KC), L, tid_p, acc);
        if (c0 == 0 && c1 == k.chunks) {
            if (L.m_valid) {
                const int wave = tid >> 6, kk = (tid & 63) >> 5;
                igemm_store(out, acc, p, tile_co * G_TCO + (wave & 1) * 64, kk, L.mb, L.mi, L.mj);
            }
        } else {
            float4 *d = reinterpret_cast<float4 *>(ws + (size_t)(2 * g + (first ? 0 : 1)) * SK_SLOT_FLOATS);
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        d[((c * 2 + h) * 4 + q) * G_THREADS + tid] =
                            make_float4(acc[c][h][4 * q], acc[c][h][4 * q + 1], acc[c][h][4 * q + 2], acc[c][h][4 * q + 3]);
        }
        first = false;
        u += (unsigned)(c1 - c0);
    }
}

// One workgroup per tile: nothing to do when a single workgroup produced it; otherwise the sum of
// its contributors' slots, in workgroup order, goes to the output.
__global__ void __launch_bounds__(G_THREADS) igemm_f32_streamk_sum_kernel(const float *__restrict__ ws,
                                                                            float *__restrict__ out, IgemmParams p, StreamK k)
{
    const int tile = blockIdx.x, tid = threadIdx.x;
    const unsigned long long u0 = (unsigned long long)tile * k.chunks, u1 = u0 + k.chunks - 1;
    auto owner = [&](unsigned long long unit) {
        int g = (int)(unit * (unsigned)k.grid / k.units);
        while (g + 1 < k.grid && sk_begin(k, g + 1) <= unit) ++g;
        while (g > 0 && sk_begin(k, g) > unit) --g;
        return g;
    };
    const int g0 = owner(u0), g1 = owner(u1);
    if (g0 == g1) return;
    floatx16 acc[4][2];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][h][v] = 0.0f;
    for (int g = g0; g <= g1; ++g) {
        const int slot = 2 * g + (sk_begin(k, g) < u0 ? 1 : 0);
        const float4 *d = reinterpret_cast<const float4 *>(ws + (size_t)slot * SK_SLOT_FLOATS);
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 v = d[((c * 2 + h) * 4 + q) * G_THREADS + tid];
                    acc[c][h][4 * q] += v.x;
                    acc[c][h][4 * q + 1] += v.y;
                    acc[c][h][4 * q + 2] += v.z;
                    acc[c][h][4 * q + 3] += v.w;
                }
    }
    const int tile_m = tile % p.tiles_m, tile_co = tile / p.tiles_m;
    const PipeLane L = pipe_lane(p, tile_m, tid);
    if (!L.m_valid) return;
    const int wave = tid >> 6, kk = (tid & 63) >> 5;
    igemm_store(out, acc, p, tile_co * G_TCO + (wave & 1) * 64, kk, L.mb, L.mi, L.mj);
}

// Sum the per-split partial outputs (fixed order: deterministic).
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float *__restrict__ ws, float *__restrict__ out,
                                                              size_t elems, int splits)
{
    const size_t e = (size_t)blockIdx.x * 256u + threadIdx.x;
    if (e >= elems) return;
    float a = ws[e];
    for (int s = 1; s < splits; ++s) a += ws[(size_t)s * elems + e];
    out[e] = a;
}

static IgemmParams plan(const Shape &s) { return igemm_plan(s, KST_F32, G_KC); }

// The pipelined kernel wants 16-byte rows and fits its input chunk in P_NX4 loads per lane.
static bool pipe_ok(const IgemmParams &p)
{
    return (p.Ns & 3) == 0 && (p.Cout & 3) == 0 && (size_t)G_KC * p.lrows * p.Ns / 4 <= (size_t)P_NX4 * G_THREADS;
}

static size_t lds_bytes(const IgemmParams &p, int n)
{
    return (size_t)G_KC * ((size_t)p.lrows * p.Ns + (size_t)n * n * G_TCO) * sizeof(float);
}

bool igemm_f32_supported(const Shape &s)
{
    if (s.n > 7) return false;
    return lds_bytes(plan(s), s.n) <= 160 * 1024;
}

bool igemm_f32_takes_row_stride(const Shape &s)
{
    return igemm_f32_supported(s) && pipe_ok(plan(s));
}

// Even shares or whole tiles?  Even shares when the pipelined kernel applies and the model says
// they beat the best launch of whole (or split) tiles by 7 %: the longest range's multiply time
// plus writing and reading every partial slot.
struct SkPlan {
    bool use;
    StreamK k;
};

static SkPlan streamk_plan(const Shape &s, const IgemmParams &p)
{
    SkPlan r;
    r.use = false;
    r.k.chunks = (s.Cin + G_KC - 1) / G_KC;
    const unsigned long long tiles = (unsigned long long)p.tiles_m * p.tiles_co;
    r.k.units = tiles * (unsigned)r.k.chunks;
    r.k.grid = r.k.units < (unsigned long long)SK_GRID ? (int)r.k.units : SK_GRID;
    // Beyond 16 rounds of whole tiles the last, part-filled round costs less than the threshold.
    if (!pipe_ok(p) || tiles % SK_GRID == 0 || tiles > 16u * SK_GRID) return r;
    unsigned long long partial = 0;                       // pieces that go through a slot
    for (int g = 0; g < r.k.grid; ++g) {
        unsigned long long u = (unsigned long long)g * r.k.units / (unsigned)r.k.grid;
        const unsigned long long u_end = (unsigned long long)(g + 1) * r.k.units / (unsigned)r.k.grid;
        while (u < u_end) {                               // the pieces, as the kernel walks them
            const unsigned long long c0 = u % (unsigned)r.k.chunks;
            const unsigned long long room = (unsigned)r.k.chunks - c0, left = u_end - u;
            const unsigned long long len = left < room ? left : room;
            if (len != (unsigned)r.k.chunks) ++partial;
            u += len;
        }
    }
    const double tile_s = (double)G_TM * G_TCO * s.Cin * s.n * s.n / 2.0e11;
    const double longest = (double)((r.k.units + r.k.grid - 1) / r.k.grid);
    const double t = longest * tile_s / r.k.chunks + (double)partial * SK_SLOT_FLOATS * 4.0 * 2.0 / 4.0e12 + 5.0e-6;
    r.use = t < 0.93 * p.est_s;
    return r;
}

size_t igemm_f32_workspace_bytes(const Shape &s)
{
    const IgemmParams p = plan(s);
    const SkPlan sk = streamk_plan(s, p);
    if (sk.use) return (size_t)2 * sk.k.grid * SK_SLOT_FLOATS * sizeof(float);
    return p.splits > 1 ? (size_t)p.splits * p.out_elems * sizeof(float) : 0;
}

template <int n>
static hipError_t launch_streamk_n(const float *in, const float *w_seg, float *out, float *ws, const IgemmParams &p,
                                   const StreamK &k, hipStream_t stream)
{
    const size_t lds = lds_bytes(p, n);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_f32_streamk_kernel<n>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(igemm_f32_streamk_kernel<n>, dim3((unsigned)k.grid), dim3(G_THREADS), lds, stream, in, w_seg,
                       out, ws, p, k);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(igemm_f32_streamk_sum_kernel, dim3((unsigned)(p.tiles_m * p.tiles_co)), dim3(G_THREADS), 0,
                       stream, ws, out, p, k);
    return hipGetLastError();
}

template <int n>
static hipError_t launch_n(const float *in, const float *w_seg, float *dst, const IgemmParams &p, hipStream_t stream)
{
    const size_t lds = lds_bytes(p, n);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_f32_kernel<n>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)p.tiles_m * p.tiles_co * p.splits;
    const bool pipe = pipe_ok(p);
    if (!pipe && p.Ns != p.N) return hipErrorInvalidValue;
    if (pipe) {
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_f32_pipe_kernel<n>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(igemm_f32_pipe_kernel<n>, dim3(blocks), dim3(G_THREADS), lds, stream, in, w_seg, dst, p);
    } else {
        hipLaunchKernelGGL(igemm_f32_kernel<n>, dim3(blocks), dim3(G_THREADS), lds, stream, in, w_seg, dst, p);
    }
    return hipGetLastError();
}

hipError_t launch_igemm_f32(const float *in, const float *w_seg, float *out, void *ws, const Shape &s,
                            hipStream_t stream)
{
    const IgemmParams p = plan(s);
    const SkPlan sk = streamk_plan(s, p);
    if (sk.use) {
        float *slots = (float *)ws;
        switch (s.n) {
            case 1: return launch_streamk_n<1>(in, w_seg, out, slots, p, sk.k, stream);
            case 2: return launch_streamk_n<2>(in, w_seg, out, slots, p, sk.k, stream);
            case 3: return launch_streamk_n<3>(in, w_seg, out, slots, p, sk.k, stream);
            case 4: return launch_streamk_n<4>(in, w_seg, out, slots, p, sk.k, stream);
            case 5: return launch_streamk_n<5>(in, w_seg, out, slots, p, sk.k, stream);
            case 6: return launch_streamk_n<6>(in, w_seg, out, slots, p, sk.k, stream);
            case 7: return launch_streamk_n<7>(in, w_seg, out, slots, p, sk.k, stream);
            default: return hipErrorInvalidValue;
        }
    }
    float *dst = p.splits > 1 ? (float *)ws : out;
    hipError_t e;
    switch (s.n) {
        case 1: e = launch_n<1>(in, w_seg, dst, p, stream); break;
        case 2: e = launch_n<2>(in, w_seg, dst, p, stream); break;
        case 3: e = launch_n<3>(in, w_seg, dst, p, stream); break;
        case 4: e = launch_n<4>(in, w_seg, dst, p, stream); break;
        case 5: e = launch_n<5>(in, w_seg, dst, p, stream); break;
        case 6: e = launch_n<6>(in, w_seg, dst, p, stream); break;
        case 7: e = launch_n<7>(in, w_seg, dst, p, stream); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    if (p.splits > 1) e = launch_splitk_reduce((const float *)ws, out, p.out_elems, p.splits, stream);
    return e;
}

hipError_t launch_splitk_reduce(const float *ws, float *out, size_t elems, int splits, hipStream_t stream)
{
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, stream,
                       ws, out, elems, splits);
    return hipGetLastError();
}

}  // namespace kst
