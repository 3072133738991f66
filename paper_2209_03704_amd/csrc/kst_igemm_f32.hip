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

#include <utility>

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
    igemm_store(dst + (size_t)split * p.out_elems, acc, p, co0 + wco * 64, kk, mb, mi, mj, p.splits == 1);
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
// H: 32-channel blocks per wave (the workgroup's tile is TCO = 64 H output channels wide).
template <int n, bool DB, int H>
__device__ __forceinline__ void pipe_accumulate(const float *__restrict__ in, const float *__restrict__ w_seg,
                                                const IgemmParams &p, float *lds, int tile_m, int tile_co,
                                                int ci_begin, int ci_end, const PipeLane &L, int tid,
                                                floatx16 (&acc)[4][H])
{
    constexpr int fl = n / 2;
    constexpr int NN = n * n;
    constexpr int TCO = 64 * H;
    constexpr int W4 = G_KC * NN * (TCO / 4);                  // weight float4 per chunk
    constexpr int NW4 = (W4 + G_THREADS - 1) / G_THREADS;        // ... per lane
    const int xplane = p.lrows * p.Ns;                           // floats per staged channel (multiple of 4)
    float *Xs = lds;                                             // [G_KC][xplane]
    float *Ws = lds + G_KC * xplane;                             // [G_KC][NN][TCO]

    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kk = lane >> 5;
    const int wco = wave & 1;

    const int m0 = tile_m * G_TM;
    const int co0 = tile_co * TCO;
    const int b0 = m0 / p.EE;
    const int i0 = (m0 - b0 * p.EE) / p.E;
    const int R0 = b0 * p.N + i0;

    const int xbase = ((L.mb * p.N + L.mi) - R0) * p.Ns + p.pad + L.mj + kk * xplane;
    const int wbase = kk * (NN * TCO) + wco * (32 * H) + l32;

    // ---- staging plan: where each of this lane's float4 comes from and goes to -------------
    // Cin is a multiple of G_KC here, so a chunk is either whole or past the end.  A lane with
    // nothing to stage (past the chunk, past Cout, past the last batch item) loads the first
    // element of the tensor over and over: whatever it brings only reaches output channels or
    // positions that are never stored (an MFMA row depends on its own weight row only, a column
    // on its own input column only).
    unsigned w_off[NW4], w_inc[NW4];
#pragma unroll
    for (int k = 0; k < NW4; ++k) {
        const int e4 = tid + k * G_THREADS;
        const int tco4 = e4 & (TCO / 4 - 1);
        const int rest = e4 / (TCO / 4);
        const int T = rest % NN, c = rest / NN;
        int cls = 0;
#pragma unroll
        for (int q = 1; q < 4; ++q)
            if (T >= class_tap_base(n, q)) cls = q;
        const int Tp = cls == 0 ? class_taps(n, 0) : cls == 1 ? class_taps(n, 1) : cls == 2 ? class_taps(n, 2) : class_taps(n, 3);
        const int tb = cls == 0 ? 0 : cls == 1 ? class_tap_base(n, 1) : cls == 2 ? class_tap_base(n, 2) : class_tap_base(n, 3);
        const bool ok = e4 < W4 && co0 + 4 * tco4 < p.Cout;
        w_off[k] = ok ? p.off[cls] + ((unsigned)(ci_begin + c) * Tp + (T - tb)) * p.Cout + co0 + 4 * tco4 : 0u;
        w_inc[k] = ok ? (unsigned)G_KC * Tp * p.Cout : 0u;
    }
    // With a frame supplied here (p.q > 0) the staged rows are rows of the framed map, the tensor
    // in memory is the dense unframed one, and an item is either 16 bytes of a row that exists or
    // four cells of the frame (or of the slack beside it): those are cleared once, below, and
    // never written again, in either stage.
    const int xp4 = xplane >> 2, n4 = p.Ns >> 2;
    const int g_first = (p.pad + p.q) >> 2, g_count = p.N0 >> 2;   // 16-byte groups of a staged row that hold tensor data
    unsigned x_off[P_NX4], x_inc[P_NX4];
    bool x_keep[P_NX4];                                           // (frame only) the item's cells keep their zeros
#pragma unroll
    for (int k = 0; k < P_NX4; ++k) {
        const int e4 = tid + k * G_THREADS;
        const int c = e4 / xp4;
        const int rem = e4 - c * xp4;
        const int lr = rem / n4, x4 = rem - lr * n4;
        const int R = R0 + lr;
        const int bb = R / p.N, y = R - bb * p.N;
        bool ok = e4 < G_KC * xp4 && bb < p.B;
        x_keep[k] = false;
        if (p.q > 0) {                                            // uniform
            const bool real = y >= p.q && y < p.N - p.q && x4 >= g_first && x4 < g_first + g_count;
            x_keep[k] = e4 < G_KC * xp4 && !real;
            ok = ok && real;
            x_off[k] = ok ? (((unsigned)bb * p.Cin + ci_begin + c) * p.N0 + (y - p.q)) * p.N0 + 4 * (x4 - g_first) : 0u;
            x_inc[k] = ok ? (unsigned)G_KC * p.N0 * p.N0 : 0u;
        } else {
            x_off[k] = ok ? (((unsigned)bb * p.Cin + ci_begin + c) * p.N + y) * p.Ns + 4 * x4 : 0u;
            x_inc[k] = ok ? (unsigned)G_KC * p.N * p.Ns : 0u;
        }
    }

#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int h = 0; h < H; ++h)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][h][v] = 0.0f;

    // With two LDS stages (DB) chunk k + 1 is written into the other stage while chunk k is
    // multiplied, and one barrier per chunk is enough; with one stage the writes wait between
    // two barriers at the end of the chunk.
    const int stage_floats = DB ? G_KC * (xplane + NN * TCO) : 0;
    int cur = 0;                                    // float offset of the stage being multiplied
    // A lane stages NW4 + P_NX4 float4 per chunk ("items": weights first, then input), each
    // through a register of its own: item -> LDS at float offset `at`, and item <- global memory
    // for the chunk at channel c0 (all-zero past the end of this range of channels; the item's
    // offset moves on by one chunk afterwards).
    constexpr int ITEMS = NW4 + P_NX4;
    float4 w_reg[NW4], x_reg[P_NX4];
    // Loads carry no branch (a chunk past the end re-reads the first element): straight-line code
    // lets the compiler count how many newer loads may be in flight when an item is needed,
    // instead of waiting for all of them.
    auto write_item = [&](auto jc, int at) {
        constexpr int j = decltype(jc)::value;
        // (copied member by member: a whole-struct copy from the register array into LDS makes
        // the compiler keep the array in scratch memory)
        if constexpr (j < NW4) {
            const float4 v = make_float4(w_reg[j].x, w_reg[j].y, w_reg[j].z, w_reg[j].w);
            if ((j + 1) * G_THREADS <= W4 || tid + j * G_THREADS < W4)
                reinterpret_cast<float4 *>(Ws + at)[tid + j * G_THREADS] = v;
        } else {
            constexpr int k = j - NW4;
            const float4 v = make_float4(x_reg[k].x, x_reg[k].y, x_reg[k].z, x_reg[k].w);
            if (tid + k * G_THREADS < G_KC * xp4 && !x_keep[k]) reinterpret_cast<float4 *>(Xs + at)[tid + k * G_THREADS] = v;
        }
    };
    auto fetch_item = [&](auto jc, int c0) {
        constexpr int j = decltype(jc)::value;
        const bool live = c0 < ci_end;                  // wave-uniform
        if constexpr (j < NW4) {
            w_reg[j] = *reinterpret_cast<const float4 *>(w_seg + (live ? w_off[j] : 0u));
            w_off[j] += w_inc[j];
        } else {
            constexpr int k = j - NW4;
            x_reg[k] = *reinterpret_cast<const float4 *>(in + (live ? x_off[k] : 0u));
            x_off[k] += x_inc[k];
        }
    };
    // First chunk -> LDS; the second is on its way into the registers while the first is
    // multiplied.  From then on an item is written to LDS late in a chunk and its register
    // refilled at once with the chunk after the next, so a load has a whole chunk's MFMAs to arrive.
    static_for<ITEMS>([&](auto jc) { fetch_item(jc, ci_begin); });
    if (p.q > 0) {                                                // uniform: the frame's cells, in every stage
#pragma unroll
        for (int k = 0; k < P_NX4; ++k)
            if (x_keep[k]) {
                reinterpret_cast<float4 *>(Xs)[tid + k * G_THREADS] = make_float4(0.f, 0.f, 0.f, 0.f);
                if constexpr (DB)
                    reinterpret_cast<float4 *>(Xs + stage_floats)[tid + k * G_THREADS] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
    }
    static_for<ITEMS>([&](auto jc) {
        write_item(jc, 0);
        fetch_item(jc, ci_begin + G_KC);
    });
    __syncthreads();

    constexpr int STEPS = G_KC / 2;                 // channel pairs per chunk (an MFMA takes two channels)
    // DB: item j goes to LDS (and is refilled) behind tap Q_WRITE + j, so that the staging
    // instructions are spread over the MFMAs instead of holding them up in one block.
    constexpr int Q_WRITE = STEPS * NN > ITEMS + 1 ? STEPS * NN - ITEMS - 1 : 0;
    float xf[2][fl + 1][fl + 1], wf[2][H];
    auto read_x = [&](auto stc) {
        constexpr int st = decltype(stc)::value;
#pragma unroll
        for (int dy = 0; dy <= fl; ++dy)
#pragma unroll
            for (int dx = 0; dx <= fl; ++dx)
                xf[st & 1][dy][dx] = Xs[cur + 2 * st * xplane + xbase + dy * p.Ns + dx];
    };
    auto read_w = [&](auto qc) {                    // the two weight values of tap q of the chunk
        constexpr int q = decltype(qc)::value;
#pragma unroll
        for (int h = 0; h < H; ++h) wf[q & 1][h] = Ws[cur + (2 * (q / NN) * NN + q % NN) * TCO + wbase + 32 * h];
    };

    for (int ci0 = ci_begin; ci0 < ci_end; ci0 += G_KC) {
        const int cn = ci0 + G_KC;
        // The MFMAs of this chunk, one tap after the other (class-major order); the two weight
        // values of tap q + 1 are read from LDS before the MFMAs of tap q are issued, and the
        // window of the next channel pair half-way through the current one, so that no MFMA waits
        // for an LDS read issued right in front of it.
        read_x(std::integral_constant<int, 0>{});
        read_w(std::integral_constant<int, 0>{});
        static_for<STEPS * NN>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            constexpr int st = q / NN, T = q % NN;
            if constexpr (q + 1 < STEPS * NN) read_w(std::integral_constant<int, q + 1>{});
            if constexpr (T == NN / 2 && st + 1 < STEPS) read_x(std::integral_constant<int, st + 1>{});
            constexpr int cls = tap_class(n, T);
            constexpr int r = cls >> 1, sp = cls & 1;
            constexpr int local = T - class_tap_base(n, cls);
            constexpr int Tb = taps_for_parity(n, sp);
            constexpr int a = local / Tb, bq = local - a * Tb;
#pragma unroll
            for (int h = 0; h < H; ++h)
                acc[cls][h] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[q & 1][h], xf[st & 1][r + a][sp + bq],
                                                                   acc[cls][h], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (DB && q >= Q_WRITE) {
                static_for<ITEMS>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    if constexpr (q - Q_WRITE == j || (q == STEPS * NN - 1 && j > q - Q_WRITE)) {
                        write_item(jc, stage_floats - cur);             // past the end: nobody reads it
                        fetch_item(jc, cn + G_KC);
                    }
                });
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        if (cn >= ci_end) break;
        __syncthreads();                            // every wave is done reading this chunk
        if constexpr (DB) {
            cur = stage_floats - cur;
        } else {
            static_for<ITEMS>([&](auto jc) {
                write_item(jc, 0);
                fetch_item(jc, cn + G_KC);
            });
            __syncthreads();
        }
    }
}

template <int n, bool DB, int H>
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
    floatx16 acc[4][H];
    pipe_accumulate<n, DB, H>(in, w_seg, p, lds, tile_m, tile_co, ci_begin, ci_end, L, (int)threadIdx.x, acc);
    if (!L.m_valid) return;
    const int wave = threadIdx.x >> 6, kk = (threadIdx.x & 63) >> 5;
    igemm_store<H>(dst + (size_t)split * p.out_elems, acc, p, (tile_co * 2 + (wave & 1)) * (32 * H), kk, L.mb, L.mi, L.mj,
                   p.splits == 1);
}

// ---------------------------------------------------------------------------
// Even shares ("stream-K"): every persistent workgroup (one fits a CU) first does whole tiles,
// one per round of SK_GRID, as long as full rounds last; the (tile, channel chunk) pairs of the
// remaining tiles, tile-major, are one list cut into SK_GRID equal ranges, one per workgroup,
// so every CU multiplies for the same time whatever the tile count.  A range is a run of
// pieces, each a span of chunks of one tile.  A piece that covers its tile's whole reduction is
// stored straight to the output; any other is written raw (the accumulator registers, lane by
// lane) to one of the workgroup's two slots: slot 2g for the first piece of workgroup g's range,
// 2g + 1 for a later one (only the last can be partial then).  A second kernel adds the slots of
// every tile that has more than one contributor in workgroup order (deterministic) and stores.
// ---------------------------------------------------------------------------
constexpr int SK_GRID = 256;                                  // CUs of the chip
// One tile's accumulators.
__host__ __device__ constexpr size_t sk_slot_floats(int tco) { return (size_t)G_TM * (size_t)tco * 4; }

struct StreamK {
    int chunks;                // channel chunks per tile
    int grid;                  // workgroups (<= SK_GRID)
    int whole;                 // tiles 0 .. whole - 1 (a multiple of grid) are done whole, one workgroup each
    unsigned long long units;  // (tiles - whole) * chunks: the list that is cut into grid ranges
};

__device__ __forceinline__ unsigned long long sk_begin(const StreamK &k, int g)
{
    return (unsigned long long)g * k.units / (unsigned)k.grid;
}

template <int n, bool DB, int H>
__global__ void __launch_bounds__(G_THREADS) igemm_f32_streamk_kernel(const float *__restrict__ in,
                                                                        const float *__restrict__ w_seg,
                                                                        float *__restrict__ out, float *__restrict__ ws,
                                                                        IgemmParams p, StreamK k)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int g = blockIdx.x;
    const int tid = threadIdx.x;
    // The pieces of this workgroup: whole tiles g, g + grid, ... below k.whole, then its range of
    // the shared list (unit u of it is chunk u % chunks of tile k.whole + u / chunks).
    int whole_tile = g;
    unsigned long long u = sk_begin(k, g);
    const unsigned long long u_end = sk_begin(k, g + 1);
    bool first = true, started = false;              // first: first piece of the shared range
    while (whole_tile < k.whole || u < u_end) {
        int tile, c0, c1;
        const bool is_whole = whole_tile < k.whole;
        if (is_whole) {
            tile = whole_tile;
            c0 = 0;
            c1 = k.chunks;
            whole_tile += k.grid;
        } else {
            const int rel = (int)(u / (unsigned)k.chunks);
            tile = k.whole + rel;
            c0 = (int)(u - (unsigned long long)rel * k.chunks);
            const unsigned long long left = u_end - u;
            c1 = left < (unsigned long long)(k.chunks - c0) ? c0 + (int)left : k.chunks;
        }
        const int tile_m = tile % p.tiles_m, tile_co = tile / p.tiles_m;
        if (started) __syncthreads();                // the previous piece's last LDS reads are done
        started = true;
        // A fresh copy of the lane number the compiler cannot see through: the staging plan is then
        // worked out anew for every piece instead of being kept in registers across the pieces.
        int tid_p = tid;
        asm volatile("" : "+v"(tid_p));
        const PipeLane L = pipe_lane(p, tile_m, tid_p);
        floatx16 acc[4][H];
        pipe_accumulate<n, DB, H>(in, w_seg, p, lds, tile_m, tile_co, c0 * G_KC, min(p.Cin, c1 * G_KC), L, tid_p, acc);
        if (c0 == 0 && c1 == k.chunks) {
            if (L.m_valid) {
                const int wave = tid >> 6, kk = (tid & 63) >> 5;
                igemm_store<H>(out, acc, p, (tile_co * 2 + (wave & 1)) * (32 * H), kk, L.mb, L.mi, L.mj);
            }
        } else {
            float4 *d = reinterpret_cast<float4 *>(ws + (size_t)(2 * g + (first ? 0 : 1)) * sk_slot_floats(64 * H));
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int h = 0; h < H; ++h)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        d[((c * H + h) * 4 + q) * G_THREADS + tid] =
                            make_float4(acc[c][h][4 * q], acc[c][h][4 * q + 1], acc[c][h][4 * q + 2], acc[c][h][4 * q + 3]);
        }
        if (!is_whole) {
            first = false;
            u += (unsigned)(c1 - c0);
        }
    }
}

// H workgroups per tile of the shared list (one per 32-channel block of every wave's share, H = tile width / 64):
// nothing to do when a single workgroup produced the tile; otherwise the sum of its contributors' slots, in workgroup
// order, goes to the output.
__global__ void __launch_bounds__(G_THREADS) igemm_f32_streamk_sum_kernel(const float *__restrict__ ws,
                                                                            float *__restrict__ out, IgemmParams p, StreamK k)
{
    const int H = p.tco >> 6;
    const int rel = blockIdx.x / H, h = blockIdx.x - rel * H, tid = threadIdx.x;   // tile k.whole + rel of the shared list
    const int tile = k.whole + rel;
    const unsigned long long u0 = (unsigned long long)rel * k.chunks, u1 = u0 + k.chunks - 1;
    auto owner = [&](unsigned long long unit) {
        int g = (int)(unit * (unsigned)k.grid / k.units);
        while (g + 1 < k.grid && sk_begin(k, g + 1) <= unit) ++g;
        while (g > 0 && sk_begin(k, g) > unit) --g;
        return g;
    };
    const int g0 = owner(u0), g1 = owner(u1);
    if (g0 == g1) return;
    float4 a[4][4];                                   // [class][four registers each]
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int q = 0; q < 4; ++q) a[c][q] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int g = g0; g <= g1; ++g) {
        if (sk_begin(k, g) == sk_begin(k, g + 1)) continue;      // an empty range (fewer units than workgroups)
        const int slot = 2 * g + (sk_begin(k, g) < u0 ? 1 : 0);
        const float4 *d = reinterpret_cast<const float4 *>(ws + (size_t)slot * sk_slot_floats(p.tco));
        float4 v[4][4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int q = 0; q < 4; ++q) v[c][q] = d[((c * H + h) * 4 + q) * G_THREADS + tid];
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                a[c][q].x += v[c][q].x;
                a[c][q].y += v[c][q].y;
                a[c][q].z += v[c][q].z;
                a[c][q].w += v[c][q].w;
            }
    }
    const int tile_m = tile % p.tiles_m, tile_co = tile / p.tiles_m;
    const PipeLane L = pipe_lane(p, tile_m, tid);
    if (!L.m_valid) return;
    floatx16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            acc[c][4 * q] = a[c][q].x;
            acc[c][4 * q + 1] = a[c][q].y;
            acc[c][4 * q + 2] = a[c][q].z;
            acc[c][4 * q + 3] = a[c][q].w;
        }
    const int wave = tid >> 6, kk = (tid & 63) >> 5;
    igemm_store_block(out, acc[0], acc[1], acc[2], acc[3], p, (tile_co * 2 + (wave & 1)) * (32 * H) + h * 32, kk,
                      L.mb, L.mi, L.mj);
}

// Sum the per-split partial outputs (fixed order: deterministic).
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float *__restrict__ ws, float *__restrict__ out,
                                                              size_t elems, int splits, Epilogue epi, size_t plane_elems,
                                                              int Cout)
{
    const size_t e = (size_t)blockIdx.x * 256u + threadIdx.x;
    if (e >= elems) return;
    float a = ws[e];
    for (int s = 1; s < splits; ++s) a += ws[(size_t)s * elems + e];
    if (epi_on(epi)) a = epi_apply(a, epi_bias(epi, (int)((e / plane_elems) % (size_t)Cout)), epi.act);
    out[e] = a;
}

static IgemmParams plan(const Shape &s, bool force_even = false);

// The pipelined kernels want 16-byte rows, whole channel chunks, and an input chunk that fits
// P_NX4 loads per lane.
static bool pipe_ok(const IgemmParams &p)
{
    if (p.q > 0 && ((p.N0 & 3) != 0 || p.N0 < 4)) return false;     // a frame supplied by the kernel: whole 16-byte groups of tensor rows
    return (p.Ns & 3) == 0 && (p.Cout & 3) == 0 && p.Cin % G_KC == 0 &&
           (size_t)G_KC * p.lrows * p.Ns / 4 <= (size_t)P_NX4 * G_THREADS;
}

static size_t lds_bytes(const IgemmParams &p, int n)
{
    return (size_t)G_KC * ((size_t)p.lrows * p.Ns + (size_t)n * n * p.tco) * sizeof(float);
}

// The pipelined kernels keep two stages in LDS when they fit (n <= 5: the larger kernels have no
// registers to spare for it).
static bool two_stages(const IgemmParams &p, int n)
{
    return n <= 5 && 2 * lds_bytes(p, n) <= 160 * 1024;
}

// The kernels for ordinary layers (tiles of 128 positions); layers with very few positions have a kernel of their own.
static bool tiles_fit(const IgemmParams &p, int n)
{
    return n <= 7 && lds_bytes(p, n) <= 160 * 1024;
}

static bool tiles_supported(const Shape &s)
{
    return tiles_fit(plan(s), s.n);
}

bool igemm_f32_supported(const Shape &s)
{
    return igemm_f32_small_supported(s) || tapmajor_f32_supported(s) || tiles_supported(s);
}

bool igemm_f32_takes_row_stride(const Shape &s)
{
    return tiles_supported(s) && pipe_ok(plan(s));
}

bool igemm_f32_takes_virtual_frame(const Shape &s)
{
    if (s.frame <= 0 || s.Ns != s.N) return false;
    return igemm_f32_small_supported(s) || tapmajor_f32_supported(s) || (tiles_supported(s) && pipe_ok(plan(s)));
}

// Even shares or whole tiles?  Even shares when the pipelined kernel applies and the model says
// they beat the best launch of whole (or split) tiles: the longest range's multiply time plus the
// traffic of the partial slots.
struct SkPlan {
    bool use;
    StreamK k;
    double t;          // the model's time for even shares (seconds), where it was worked out
};

static SkPlan streamk_plan(const Shape &s, const IgemmParams &p, bool force)
{
    SkPlan r;
    r.use = false;
    r.t = 0.0;
    r.k.chunks = (s.Cin + G_KC - 1) / G_KC;
    const unsigned long long tiles = (unsigned long long)p.tiles_m * p.tiles_co;
    const unsigned long long all_units = tiles * (unsigned)r.k.chunks;
    r.k.grid = all_units < (unsigned long long)SK_GRID ? (int)all_units : SK_GRID;
    r.k.whole = (int)(tiles / SK_GRID) * SK_GRID;             // (0 unless grid == SK_GRID)
    r.k.units = (tiles - r.k.whole) * (unsigned)r.k.chunks;
    if (!tiles_fit(p, s.n) || !pipe_ok(p) || tiles > (1u << 22)) return r;
    if (force) {
        r.use = true;
        return r;
    }
    // Beyond 16 rounds of whole tiles the last, part-filled round costs less than the threshold.
    if (tiles % SK_GRID == 0 || tiles > 16u * SK_GRID) return r;
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
    // The slots are written while other workgroups still multiply; what shows is about half of
    // their traffic (measured on 64 x 1024 x 512 x 8 x 8, n = 5: 483 us against 514 us for seven splits).
    const double tile_s = (double)G_TM * p.tco * s.Cin * s.n * s.n / 2.0e11;
    const double longest = (double)(r.k.whole / r.k.grid) * r.k.chunks + (double)((r.k.units + r.k.grid - 1) / r.k.grid);
    // The summing pass walks a tile's contributors one after the other (about 2.5 us each, measured
    // on one-sample layers with 64 and 128 contributors per tile); up to four hide in its launch.
    const unsigned long long shared_tiles = tiles - (unsigned)r.k.whole;
    const double per_tile = shared_tiles ? (double)partial / (double)shared_tiles : 0.0;
    const double serial_sum = per_tile > 4.0 ? (per_tile - 4.0) * 2.5e-6 : 0.0;
    const double t = longest * tile_s / r.k.chunks + (double)partial * sk_slot_floats(p.tco) * 4.0 * 2.0 / 8.0e12 + 5.0e-6 +
                     serial_sum;
    r.t = t;
    r.use = t < 0.99 * p.est_s;
    return r;
}

// Tiles of 128 or of 64 output channels (pipelined kernels only).  Half-width tiles are twice as many, which
// saves a split of the reduction, or half the work where a layer has 64 output channels; a wave then
// multiplies every window value it reads into one 32-channel block instead of two.
static IgemmParams plan(const Shape &s, bool force_even)
{
    const IgemmParams wide = igemm_plan(s, KST_F32, G_KC);
    if (!pipe_ok(wide) || !tiles_fit(wide, s.n)) return wide;
    const IgemmParams narrow = igemm_plan(s, KST_F32, G_KC, 64);
    if (s.Cout <= 64) return narrow;
    if (force_even) return wide;                     // a forced launch does not depend on the cost model
    // Measured: with tiles to spare the half-width tile costs 5 % (cfg3 844 -> 885 us); where the wide tiles
    // are fewer than the CUs it wins by halving the split of the reduction (64 x 256 x 128 x 16 x 16, n = 4:
    // 163 -> 145 us; 64 x 512 x 256 x 8 x 8: 163 -> 156 us).
    const SkPlan a = streamk_plan(s, wide, false), b = streamk_plan(s, narrow, false);
    const double ta = a.use ? a.t : wide.est_s, tb = b.use ? b.t : narrow.est_s;
    const double handicap = wide.tiles_m * wide.tiles_co < SK_GRID ? 1.0 : 1.05;
    return handicap * tb <= ta ? narrow : wide;
}

bool igemm_f32_even_shares_possible(const Shape &s)
{
    return streamk_plan(s, plan(s, true), true).use;
}

size_t igemm_f32_workspace_bytes(const Shape &s, bool force_even)
{
    if (!force_even && igemm_f32_small_supported(s)) return igemm_f32_small_workspace_bytes(s);
    if (!force_even && tapmajor_f32_supported(s)) return 0;
    const IgemmParams p = plan(s, force_even);
    const SkPlan sk = streamk_plan(s, p, force_even);
    if (sk.use) return (size_t)2 * sk.k.grid * sk_slot_floats(p.tco) * sizeof(float);
    return p.splits > 1 ? (size_t)p.splits * p.out_elems * sizeof(float) : 0;
}

template <int n, bool DB, int H>
static hipError_t launch_streamk_h(const float *in, const float *w_seg, float *out, float *ws, const IgemmParams &p,
                                   const StreamK &k, hipStream_t stream)
{
    const size_t lds = lds_bytes(p, n) * (DB ? 2 : 1);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_f32_streamk_kernel<n, DB, H>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((igemm_f32_streamk_kernel<n, DB, H>), dim3((unsigned)k.grid), dim3(G_THREADS), lds, stream, in,
                       w_seg, out, ws, p, k);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const unsigned shared_tiles = (unsigned)(p.tiles_m * p.tiles_co - k.whole);
    if (shared_tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(igemm_f32_streamk_sum_kernel, dim3((unsigned)H * shared_tiles), dim3(G_THREADS), 0, stream, ws, out, p, k);
    return hipGetLastError();
}

template <int n, bool DB>
static hipError_t launch_streamk_db(const float *in, const float *w_seg, float *out, float *ws, const IgemmParams &p,
                                    const StreamK &k, hipStream_t stream)
{
    if (p.tco == 64) return launch_streamk_h<n, DB, 1>(in, w_seg, out, ws, p, k, stream);
    return launch_streamk_h<n, DB, 2>(in, w_seg, out, ws, p, k, stream);
}

template <int n>
static hipError_t launch_streamk_n(const float *in, const float *w_seg, float *out, float *ws, const IgemmParams &p,
                                   const StreamK &k, hipStream_t stream)
{
    if constexpr (n <= 5)
        if (two_stages(p, n)) return launch_streamk_db<n, true>(in, w_seg, out, ws, p, k, stream);
    return launch_streamk_db<n, false>(in, w_seg, out, ws, p, k, stream);
}

template <int n, bool DB, int H>
static hipError_t launch_pipe_h(const float *in, const float *w_seg, float *dst, const IgemmParams &p, unsigned blocks,
                                hipStream_t stream)
{
    const size_t lds = lds_bytes(p, n) * (DB ? 2 : 1);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_f32_pipe_kernel<n, DB, H>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((igemm_f32_pipe_kernel<n, DB, H>), dim3(blocks), dim3(G_THREADS), lds, stream, in, w_seg, dst, p);
    return hipGetLastError();
}

template <int n, bool DB>
static hipError_t launch_pipe_db(const float *in, const float *w_seg, float *dst, const IgemmParams &p, unsigned blocks,
                                 hipStream_t stream)
{
    if (p.tco == 64) return launch_pipe_h<n, DB, 1>(in, w_seg, dst, p, blocks, stream);
    return launch_pipe_h<n, DB, 2>(in, w_seg, dst, p, blocks, stream);
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
    if (!pipe && (p.Ns != p.N || p.q > 0)) return hipErrorInvalidValue;
    if (pipe) {
        if constexpr (n <= 5)
            if (two_stages(p, n)) return launch_pipe_db<n, true>(in, w_seg, dst, p, blocks, stream);
        return launch_pipe_db<n, false>(in, w_seg, dst, p, blocks, stream);
    } else {
        hipLaunchKernelGGL(igemm_f32_kernel<n>, dim3(blocks), dim3(G_THREADS), lds, stream, in, w_seg, dst, p);
    }
    return hipGetLastError();
}

hipError_t launch_igemm_f32(const float *in, const float *w_seg, float *out, void *ws, const Shape &s,
                            bool force_even, hipStream_t stream)
{
    if (!force_even && igemm_f32_small_supported(s)) return launch_igemm_f32_small(in, w_seg, out, ws, s, stream);
    if (!force_even && tapmajor_f32_supported(s)) return launch_tapmajor_f32(in, w_seg, out, s, stream);
    const IgemmParams p = plan(s, force_even);
    const SkPlan sk = streamk_plan(s, p, force_even);
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
    if (p.splits > 1)
        e = launch_splitk_reduce((const float *)ws, out, p.out_elems, p.splits, stream, p.epi, (size_t)p.M * p.M, p.Cout);
    return e;
}

// The same sum for many partial results of a small tensor: 256 / SH elements x SH strided shares of
// the partial results per workgroup, the shares added through LDS in a fixed order.
template <int SH>
__global__ void __launch_bounds__(256) splitk_reduce_shares_kernel(const float *__restrict__ ws, float *__restrict__ out,
                                                                     size_t elems, int splits, Epilogue epi,
                                                                     size_t plane_elems, int Cout)
{
    constexpr int EL = 256 / SH;
    __shared__ float red[SH][EL + 1];
    const int el = threadIdx.x % EL, share = threadIdx.x / EL;
    const size_t e = (size_t)blockIdx.x * EL + el;
    float a = 0.0f;
    if (e < elems)
        for (int s = share; s < splits; s += SH) a += ws[(size_t)s * elems + e];
    red[share][el] = a;
    __syncthreads();
    if (share == 0 && e < elems) {
        float t = red[0][el];
        for (int k = 1; k < SH; ++k) t += red[k][el];
        if (epi_on(epi)) t = epi_apply(t, epi_bias(epi, (int)((e / plane_elems) % (size_t)Cout)), epi.act);
        out[e] = t;
    }
}

// 64 and more partial results: 16 shares; 512 and more: 64 shares.
hipError_t launch_splitk_reduce(const float *ws, float *out, size_t elems, int splits, hipStream_t stream, Epilogue epi,
                                size_t plane_elems, int Cout)
{
    if (splits >= 512) {
        hipLaunchKernelGGL(splitk_reduce_shares_kernel<64>, dim3((unsigned)((elems + 3) / 4)), dim3(256), 0, stream, ws, out,
                           elems, splits, epi, plane_elems, Cout);
        return hipGetLastError();
    }
    if (splits >= 64) {
        hipLaunchKernelGGL(splitk_reduce_shares_kernel<16>, dim3((unsigned)((elems + 15) / 16)), dim3(256), 0, stream, ws, out,
                           elems, splits, epi, plane_elems, Cout);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, stream,
                       ws, out, elems, splits, epi, plane_elems, Cout);
    return hipGetLastError();
}

}  // namespace kst
