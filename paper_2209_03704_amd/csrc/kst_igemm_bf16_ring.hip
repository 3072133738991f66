// Matrix-core segregated forward pass for bfloat16 operands: LDS ring filled by
// LDS-direct loads, MFMA operands fetched with the transposing LDS read.
//
// Same arithmetic as kst_igemm_bf16.hip (Section 3.3, Eqs. 7-10 as four implicit
// GEMMs on v_mfma_f32_32x32x16_bf16, fp32 accumulation).  What is different is how
// the operands reach the matrix cores:
//   * the input stays in its NCHW order all the way into LDS ([channel][row][x]):
//     a 16-channel chunk of the tile's TI + 1 input rows is copied by 16-byte
//     LDS-direct loads (no registers, no ALU work), and the [position][channel]
//     fragment an MFMA wants is produced by ds_read_b64_tr_b16, which transposes
//     4 x 4 blocks of 16-bit elements across lanes on the way out of LDS;
//   * a transposing read returns four CONSECUTIVE pixels from an 8-byte aligned
//     address, so the window column dx = 1 of Eqs. 7-10 cannot be read the same way;
//     it is the dx = 0 fragment moved down one lane (DPP wave shift), with the two
//     lanes at the block edge patched from the neighbouring block's fragment;
//   * the segregated weights already sit in fragment order in HBM and are copied by
//     LDS-direct loads as well;
//   * three stages form a ring: chunks k+1 and k+2 are in flight while chunk k is
//     multiplied, with one workgroup barrier per chunk.  The compiler would make
//     every LDS read wait for all LDS-direct loads in flight, so inside the
//     reduction loop the LDS reads, the counter waits and the barrier are written
//     as inline assembly and the loop keeps the counts itself.
// Tile: TI quad rows x 64 output channels per 256-thread workgroup, positions in
// blocks of 32 consecutive quad columns of one quad row (the transposing read needs
// consecutive pixels), 4 waves of 32 channels x 64 positions x 4 parity classes,
// two workgroups per CU.  The epilogue is the one of the row-strip kernel: classes
// interleaved in an LDS image, streamed out as 16-byte stores whose lane quads sit
// in one 64-byte segment.
#include "kst_igemm_common.h"

namespace kst {

typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int R_THREADS = 256;
constexpr int R_TCO = 64;
constexpr int R_KC = 16;               // channels per chunk = one MFMA reduction step

template <int n, int N>
struct RingGeom {
    static_assert(n == 2 || n == 3, "window columns 0 and 1 only");
    static_assert(N == 32 || N == 64, "a quad row is one or two 32-column blocks held by one wave");
    static constexpr int fl = n / 2;
    static constexpr int NN = n * n;
    static constexpr int M = 2 * N - n;
    static constexpr int E = (M + 1) / 2;
    static constexpr int CB = (E + 31) / 32;             // 32-column position blocks per quad row
    static constexpr int TI = 4 / CB;                    // quad rows per tile (4 position blocks)
    static constexpr int STRIPS = (E + TI - 1) / TI;
    static constexpr int ROWS = TI + fl;                 // staged input rows
    static constexpr int ROW_B = N * 2;                  // bytes per staged row
    static constexpr int UPR = N / 8;                    // 16-byte units per row
    // Bytes per channel of an image: padded to 64 (mod 128) so that the eight channel rows
    // one transposing read touches spread over the LDS banks.
    static constexpr int CS = (ROWS * ROW_B + 127) / 128 * 128 + 64;
    static constexpr int UPC = CS / 16;                  // units per channel, padding included
    static constexpr int COPY_B = R_KC * CS;             // bytes per image
    static constexpr int W_B = NN * 2 * R_TCO * 16;      // weights per stage: [tap][octet][channel] x 16 bytes
    static constexpr int STAGE_B = W_B + COPY_B;
    static constexpr int STAGES = 3;
    static constexpr int W_SLABS = NN * 2;               // 1 KiB slabs (one wave-wide LDS-direct load each)
    static constexpr int X_SLABS = COPY_B / 1024;
    static_assert(COPY_B % 1024 == 0, "image is a whole number of slabs");
    static constexpr int SLABS = W_SLABS + X_SLABS;
    static constexpr int KMAX = (SLABS + 3) / 4;         // slabs per wave
    static constexpr int LMAX = 2 * TI * M;              // floats per channel run of a tile
    static constexpr int ESTRIDE = (LMAX + 3 + 3) & ~3;  // floats per channel in the epilogue image
    static constexpr int TG = (15 + LMAX - 1) / 4 + 1;   // 16-byte groups per channel run, upper bound
    static constexpr int EPI_B = 32 * ESTRIDE * 4;
    static constexpr int LDS_B = STAGES * STAGE_B > EPI_B ? STAGES * STAGE_B : EPI_B;
};

struct RingParams {
    int B, Cin, Cout, tiles_co;
    unsigned off[4];
    Epilogue epi;
};

// Workgroup barrier that orders LDS traffic only (LDS-direct loads included): global
// stores already issued stay in flight across it.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

#define KST_LDS(T) T __attribute__((address_space(3)))
#define KST_GLB(T) T __attribute__((address_space(1)))

template <int n, int N, bool F16>
__global__ void __launch_bounds__(R_THREADS, 2) igemm_bf16_ring_kernel(const uint16_t *__restrict__ in,
                                                                      const uint16_t *__restrict__ w_seg,
                                                                      float *__restrict__ out, RingParams p)
{
    using G = RingGeom<n, N>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];

    unsigned id = blockIdx.x;
    const int strip = (int)(id % (unsigned)G::STRIPS);
    id /= (unsigned)G::STRIPS;
    const int tile_co = (int)(id % (unsigned)p.tiles_co);
    const int b = (int)(id / (unsigned)p.tiles_co);
    const int co0 = tile_co * R_TCO;
    const int i0 = strip * G::TI;
    const int rows_q = min(G::TI, G::E - i0);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    const int wco = wave & 1, wpos = wave >> 1;

    // This lane's two quad positions (MFMA columns), and the byte offset inside a stage of the
    // 8-byte row it hands to the transposing read: within a block of 16 lanes, lane s supplies
    // channel s / 4 and pixels 4 (s % 4) .. +3, and receives pixel s of four channels.
    int ti[2], tj[2], xrd[2];
    bool pos_ok[2];
    const int s16 = lane & 15, h16 = (lane >> 4) & 1;
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        const int blk = wpos * 2 + pb;
        const int cb = blk % G::CB;
        ti[pb] = blk / G::CB;
        tj[pb] = cb * 32 + l32;
        pos_ok[pb] = ti[pb] < rows_q && tj[pb] < G::E;
        xrd[pb] = G::W_B + (8 * kk + (s16 >> 2)) * G::CS + ti[pb] * G::ROW_B + (32 * cb + 16 * h16 + 4 * (s16 & 3)) * 2;
    }
    const int wrd = (kk * R_TCO + wco * 32 + l32) * 16;

    // ---- LDS-direct plan ----------------------------------------------------------------------
    // Wave w copies slabs w, w + 4, ... of every stage: exactly KMAX loads per wave and chunk
    // (the few slots past the last slab repeat slabs 0, 1, ...: the same bytes to the same
    // place).  A load's address is a wave-uniform base that advances once per chunk plus a
    // per-lane byte offset that never changes.
    const unsigned char *g_base[G::KMAX];
    unsigned g_inc[G::KMAX], g_lane[G::KMAX], g_dst[G::KMAX];
#pragma unroll
    for (int k = 0; k < G::KMAX; ++k) {
        int q = wave + 4 * k;
        if (q >= G::SLABS) q -= G::SLABS;
        g_dst[k] = (unsigned)q * 1024u;
        if (q < G::W_SLABS) {
            const int T = q >> 1, oct = q & 1;
            int cls = 0;
#pragma unroll
            for (int c = 1; c < 4; ++c)
                if (T >= class_tap_base(n, c)) cls = c;
            int Tp = class_taps(n, 0), tb = 0;
#pragma unroll
            for (int c = 1; c < 4; ++c)
                if (cls == c) { Tp = class_taps(n, c); tb = class_tap_base(n, c); }
            g_base[k] = reinterpret_cast<const unsigned char *>(
                w_seg + p.off[cls] + (((size_t)oct * Tp + (T - tb)) * p.Cout + co0) * 8u);
            g_inc[k] = 2u * Tp * p.Cout * 16u;
            g_lane[k] = (unsigned)lane * 16u;
        } else {
            const int u = (q - G::W_SLABS) * 64 + lane;
            const int ci = u / G::UPC;
            int rem = u - ci * G::UPC;
            if (rem >= G::ROWS * G::UPR) rem = 0;                  // padding unit: any valid address
            const int row = rem / G::UPR, x8 = rem - row * G::UPR;
            const int grow = min(i0 + row, N - 1);
            g_base[k] = reinterpret_cast<const unsigned char *>(in + (size_t)b * p.Cin * N * N);
            g_inc[k] = (unsigned)R_KC * N * N * 2u;
            g_lane[k] = (unsigned)(((ci * N + grow) * N + x8 * 8) * 2);
        }
    }

    floatx16 acc[4][2];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][pb][v] = 0.0f;

    auto issue_direct = [&](int stage) {
#pragma unroll
        for (int k = 0; k < G::KMAX; ++k) {
            __builtin_amdgcn_global_load_lds((const KST_GLB(void) *)(g_base[k] + g_lane[k]),
                                             (KST_LDS(void) *)(lds_raw + stage * G::STAGE_B + g_dst[k]), 16, 0, 0);
            g_base[k] += g_inc[k];
        }
    };
    // Wait until at most `allowed` (0 or KMAX) of this wave's vector-memory loads are
    // outstanding (they complete in issue order), then meet the other waves.
    auto wait_loads_and_meet = [&](bool last) {
        if (last)
            asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(G::KMAX) : "memory");
    };
    static_assert(G::KMAX * 4 - G::SLABS < G::W_SLABS && G::KMAX < 64, "repeated slabs are weight slabs");

    // Taps in the order they are multiplied: first those that read window column 0, then those
    // that read column 1 (by then the window registers have been shifted in place).
    struct TapOrder {
        int T[G::NN], cls[G::NN], dy[G::NN], dx[G::NN], n0;
        constexpr TapOrder() : T(), cls(), dy(), dx(), n0(0)
        {
            int m = 0;
            for (int want = 0; want < 2; ++want) {
                for (int c = 0; c < 4; ++c) {
                    const int r = c >> 1, s2 = c & 1;
                    const int Ta = taps_for_parity(n, r), Tb = taps_for_parity(n, s2);
                    for (int a2 = 0; a2 < Ta; ++a2)
                        for (int bq = 0; bq < Tb; ++bq)
                            if (s2 + bq == want) {
                                T[m] = class_tap_base(n, c) + a2 * Tb + bq;
                                cls[m] = c; dy[m] = r + a2; dx[m] = want;
                                ++m;
                            }
                }
                if (want == 0) n0 = m;
            }
        }
    };
    constexpr TapOrder ord;

    const unsigned lds_base = (unsigned)(size_t)(KST_LDS(unsigned char) *)lds_raw;
    // One chunk: the transposing window reads and the first weight fragment in one block that
    // ends with the wait for them; the other weight fragments are ordinary LDS loads issued
    // before the first MFMAs and waited for one by one by the compiler.  The LDS-direct loads
    // of a later chunk are issued behind the first MFMAs, whose execution hides them.
    auto multiply = [&](int stage, bool refill, int refill_stage) {
        const unsigned xa0 = lds_base + stage * G::STAGE_B + xrd[0];
        const unsigned xa1 = lds_base + stage * G::STAGE_B + xrd[1];
        const unsigned wa = lds_base + stage * G::STAGE_B + wrd;
        const unsigned char *sb = lds_raw + stage * G::STAGE_B;
        uintx2 t[2][2][2];                                       // [position block][window row][channel half]
        uintx4 w0;
        bf16x8 wv[G::NN];                                        // in multiplication order
        asm volatile(
            "ds_read_b64_tr_b16 %0, %9\n\t"
            "ds_read_b64_tr_b16 %1, %9 offset:%13\n\t"
            "ds_read_b64_tr_b16 %2, %9 offset:%12\n\t"
            "ds_read_b64_tr_b16 %3, %9 offset:%14\n\t"
            "ds_read_b64_tr_b16 %4, %10\n\t"
            "ds_read_b64_tr_b16 %5, %10 offset:%13\n\t"
            "ds_read_b64_tr_b16 %6, %10 offset:%12\n\t"
            "ds_read_b64_tr_b16 %7, %10 offset:%14\n\t"
            "ds_read_b128 %8, %11 offset:%15\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(t[0][0][0]), "=&v"(t[0][0][1]), "=&v"(t[0][1][0]), "=&v"(t[0][1][1]), "=&v"(t[1][0][0]),
              "=&v"(t[1][0][1]), "=&v"(t[1][1][0]), "=&v"(t[1][1][1]), "=&v"(w0)
            : "v"(xa0), "v"(xa1), "v"(wa), "n"(G::ROW_B), "n"(4 * G::CS), "n"(G::ROW_B + 4 * G::CS), "n"(ord.T[0] * 2048)
            : "memory");
        wv[0] = __builtin_bit_cast(bf16x8, w0);
#pragma unroll
        for (int m = 1; m < G::NN; ++m)
            wv[m] = *reinterpret_cast<const bf16x8 *>(sb + ord.T[m] * (2 * R_TCO * 16) + wrd);
        __builtin_amdgcn_sched_barrier(0);                       // the rest of the weights fly during the first MFMAs

        // Window fragments [block][row]: lanes 0..31 and 32..63 hold the two channel halves of
        // quad columns 0..31 of the block.
        uintx4 x[2][2];
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int dy = 0; dy < 2; ++dy) x[pb][dy] = __builtin_shufflevector(t[pb][dy][0], t[pb][dy][1], 0, 1, 2, 3);
#pragma unroll
        for (int m = 0; m < ord.n0; ++m)
#pragma unroll
            for (int pb = 0; pb < 2; ++pb)
                acc[ord.cls[m]][pb] = mfma16<F16>(
                    wv[m], __builtin_bit_cast(bf16x8, x[pb][ord.dy[m]]), acc[ord.cls[m]][pb]);
        __builtin_amdgcn_sched_barrier(0);
        if (refill) issue_direct(refill_stage);
        // Window column 1 = column 0 of the next quad = the next lane's value.  With both blocks
        // of a quad row in the wave, the halves are regrouped so that one register holds all 64
        // columns of a channel half, shifted down a lane, and regrouped back; a lone block is
        // shifted as it is (its last column lies past the row's last valid quad).
#pragma unroll
        for (int dy = 0; dy < 2; ++dy)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (G::CB == 2) {
                    const auto g = __builtin_amdgcn_permlane32_swap(x[0][dy][i], x[1][dy][i], false, false);
                    const unsigned lo = (unsigned)__builtin_amdgcn_mov_dpp((int)g[0], 0x130, 0xf, 0xf, true);
                    const unsigned hi = (unsigned)__builtin_amdgcn_mov_dpp((int)g[1], 0x130, 0xf, 0xf, true);
                    const auto h = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
                    x[0][dy][i] = h[0];
                    x[1][dy][i] = h[1];
                } else {
                    x[0][dy][i] = (unsigned)__builtin_amdgcn_mov_dpp((int)x[0][dy][i], 0x130, 0xf, 0xf, true);
                    x[1][dy][i] = (unsigned)__builtin_amdgcn_mov_dpp((int)x[1][dy][i], 0x130, 0xf, 0xf, true);
                }
            }
#pragma unroll
        for (int m = ord.n0; m < G::NN; ++m)
#pragma unroll
            for (int pb = 0; pb < 2; ++pb)
                acc[ord.cls[m]][pb] = mfma16<F16>(
                    wv[m], __builtin_bit_cast(bf16x8, x[pb][ord.dy[m]]), acc[ord.cls[m]][pb]);
    };

    // ---- reduction over the input channels ------------------------------------------------------
    // Chunk c lives in stage c % 3.  At the top of iteration c the wave has issued the loads of
    // chunks <= c + 1; it waits for its share of chunk c, meets the others (so chunk c is whole
    // and nobody still reads chunk c - 1), refills the stage of chunk c - 1 with chunk c + 2,
    // and multiplies chunk c.
    const int nchunks = p.Cin / R_KC;
    issue_direct(0);
    if (nchunks > 1) issue_direct(1);
    int cur = 0;
    for (int c = 0; c < nchunks; ++c) {
        wait_loads_and_meet(c + 1 >= nchunks);
        multiply(cur, c + 2 < nchunks, cur == 0 ? 2 : cur - 1);
        cur = cur == 2 ? 0 : cur + 1;
    }

    // ---- epilogue -----------------------------------------------------------------------------
    // Per output channel the tile is one contiguous run of rows_out * M floats.  The four
    // classes are interleaved into that run in LDS, 32 channels per pass, and streamed out
    // with 16-byte stores whose lane quads sit in one 64-byte segment (lane t of a channel
    // owns floats [base64 + 4t, +4), base64 = run start rounded down to 64 bytes); only the
    // groups cut by the ends of a run use scalar stores.
    // Channel cl of a pass keeps its run at Es[cl][(run start & 3) + ...], so that 16-byte
    // groups of the run are 16-byte aligned in LDS too.  M * M is 0 or 1 (mod 4), so among
    // the channels 8q + 4kk + j a lane holds, that shift depends on j alone.
    float *Es = reinterpret_cast<float *>(lds_raw);                 // [32][ESTRIDE]
    const int rows_out = min(2 * rows_q, G::M - 2 * i0);
    const int L = rows_out * G::M;
    constexpr unsigned MM = (unsigned)G::M * G::M;
    const unsigned g_first = (((unsigned)b * p.Cout + co0) * G::M + 2 * i0) * G::M;   // run start of channel co0
#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        lds_barrier();                                               // LDS is free: K loop / previous pass read it
        if (wco == pass) {
#pragma unroll
            for (int pb = 0; pb < 2; ++pb) {
                if (!pos_ok[pb]) continue;
                const bool x1_ok = 2 * tj[pb] + 1 < G::M;
                const bool r1_ok = 2 * ti[pb] + 1 < rows_out;
                float *eq = Es + 4 * kk * G::ESTRIDE + 2 * ti[pb] * G::M + 2 * tj[pb];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float *ej = eq + j * G::ESTRIDE + ((g_first + j * (MM & 3u)) & 3u);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float *e = ej + 8 * q * G::ESTRIDE;
                        const int v = 4 * q + j;
                        e[0] = acc[0][pb][v];
                        if (x1_ok) e[1] = acc[1][pb][v];
                        if (r1_ok) {
                            e[G::M] = acc[2][pb][v];
                            if (x1_ok) e[G::M + 1] = acc[3][pb][v];
                        }
                    }
                }
            }
        }
        lds_barrier();
        // Wave w streams channels w, w + 4, ...; lane t of a channel owns the 16-byte group
        // [base64 + 4t, +4) of the output, base64 = run start rounded down to 64 bytes.
#pragma unroll 2
        for (int cl = wave; cl < 32; cl += R_THREADS / 64) {
            const unsigned g_co = g_first + (unsigned)(pass * 32 + cl) * MM;
            const int a16 = (int)(g_co & 15u);                          // run start inside its 64-byte segment
            const float *erun = Es + cl * G::ESTRIDE - (int)(g_co & 12u);   // group t of the run is at erun + 4t
            float *orun = out + (g_co & ~15u);
            const bool epi = epi_on(p.epi);                             // uniform
            const float bias = epi ? epi_bias(p.epi, co0 + pass * 32 + cl) : 0.0f;
#pragma unroll
            for (int it = 0; it < (G::TG + 63) / 64; ++it) {
                const int t = lane + 64 * it;
                const int rel = 4 * t - a16;                           // first float of the group, relative to the run
                if (rel >= 0 && rel + 3 < L) {
                    float4 v4 = *reinterpret_cast<const float4 *>(erun + 4 * t);
                    if (epi) epi_apply4(v4.x, v4.y, v4.z, v4.w, bias, p.epi.act);
                    store_streaming4(orun + 4 * t, v4.x, v4.y, v4.z, v4.w);
                } else if (rel + 3 >= 0 && rel < L) {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (rel + k >= 0 && rel + k < L)
                            orun[4 * t + k] = epi ? epi_apply(erun[4 * t + k], bias, p.epi.act) : erun[4 * t + k];
                }
            }
        }
    }
}

template <int n, int N, bool F16>
hipError_t launch_ring(const uint16_t *in, const uint16_t *w_seg, float *out, const RingParams &p, hipStream_t stream)
{
    using G = RingGeom<n, N>;
    static_assert(G::LDS_B <= 80 * 1024, "two workgroups per CU");
    if (G::LDS_B > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_bf16_ring_kernel<n, N, F16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_B);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)p.B * p.tiles_co * G::STRIPS;
    hipLaunchKernelGGL((igemm_bf16_ring_kernel<n, N, F16>), dim3(blocks), dim3(R_THREADS), G::LDS_B, stream, in, w_seg, out, p);
    return hipGetLastError();
}

}  // namespace

bool igemm_bf16_ring_supported(const Shape &s)
{
    if (s.n != 2 && s.n != 3) return false;
    if (s.N != 32 && s.N != 64) return false;
    if (s.Cin % R_KC != 0 || s.Cout % R_TCO != 0) return false;
    const size_t strips = (size_t)(s.E + (4 / ((s.E + 31) / 32)) - 1) / (4 / ((s.E + 31) / 32));
    return (size_t)s.B * (s.Cout / R_TCO) * strips < 0x7fffffffu;
}

hipError_t launch_igemm_bf16_ring(const void *in, const void *w_seg, float *out, const Shape &s, bool f16,
                                  hipStream_t stream)
{
    if (!igemm_bf16_ring_supported(s)) return hipErrorInvalidValue;
    RingParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.tiles_co = s.Cout / R_TCO;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, KST_BF16);
    p.epi = s.epi;
    const uint16_t *i16 = (const uint16_t *)in, *w16 = (const uint16_t *)w_seg;
    switch (s.n * 1000 + s.N) {
        case 2032: return f16 ? launch_ring<2, 32, true>(i16, w16, out, p, stream) : launch_ring<2, 32, false>(i16, w16, out, p, stream);
        case 2064: return f16 ? launch_ring<2, 64, true>(i16, w16, out, p, stream) : launch_ring<2, 64, false>(i16, w16, out, p, stream);
        case 3032: return f16 ? launch_ring<3, 32, true>(i16, w16, out, p, stream) : launch_ring<3, 32, false>(i16, w16, out, p, stream);
        case 3064: return f16 ? launch_ring<3, 64, true>(i16, w16, out, p, stream) : launch_ring<3, 64, false>(i16, w16, out, p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace kst
