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

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
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

template <int n, int N>
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

    // ---- LDS-direct plan: wave w copies slabs w, w + 4, ... of every stage -------------------
    unsigned g_off[G::KMAX], g_inc[G::KMAX];
#pragma unroll
    for (int k = 0; k < G::KMAX; ++k) {
        const int q = wave + 4 * k;
        g_off[k] = 0;
        g_inc[k] = 0;
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
            g_off[k] = p.off[cls] + (((unsigned)oct * Tp + (T - tb)) * p.Cout + co0 + lane) * 8u;
            g_inc[k] = 2u * Tp * p.Cout * 8u;
        } else if (q < G::SLABS) {
            const int u = (q - G::W_SLABS) * 64 + lane;
            const int ci = u / G::UPC;
            int rem = u - ci * G::UPC;
            if (rem >= G::ROWS * G::UPR) rem = 0;                  // padding unit: any valid address
            const int row = rem / G::UPR, x8 = rem - row * G::UPR;
            const int grow = min(i0 + row, N - 1);
            g_off[k] = (((unsigned)b * p.Cin + ci) * N + grow) * N + x8 * 8;
            g_inc[k] = (unsigned)R_KC * N * N;
        }
    }
    int my_slabs = 0;                                           // LDS-direct loads this wave issues per chunk
#pragma unroll
    for (int k = 0; k < G::KMAX; ++k)
        if (wave + 4 * k < G::SLABS) ++my_slabs;

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
            const int q = wave + 4 * k;
            if (q < G::SLABS) {
                const uint16_t *src = (q < G::W_SLABS ? w_seg : in) + g_off[k];
                __builtin_amdgcn_global_load_lds((const KST_GLB(void) *)src,
                                                 (KST_LDS(void) *)(lds_raw + stage * G::STAGE_B + q * 1024), 16, 0, 0);
                g_off[k] += g_inc[k];
            }
        }
    };
    // Wait until at most `allowed` of this wave's vector-memory loads are outstanding (they
    // complete in issue order), then meet the other waves.  allowed is 0 or my_slabs.
    auto wait_loads_and_meet = [&](int allowed) {
        if (allowed == 0)
            asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        else if (allowed == G::KMAX)
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(G::KMAX) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(G::KMAX - 1) : "memory");
    };
    static_assert(G::KMAX * 4 - G::SLABS < 4 && G::KMAX >= 2 && G::KMAX < 64, "a wave issues KMAX or KMAX - 1 loads per chunk");

    const unsigned lds_base = (unsigned)(size_t)(KST_LDS(unsigned char) *)lds_raw;
    // One chunk: every LDS read of the wave in one block that ends with the wait for them,
    // window column 1 by lane shift, then the MFMAs.
    auto multiply = [&](int stage) {
        const unsigned xa0 = lds_base + stage * G::STAGE_B + xrd[0];
        const unsigned xa1 = lds_base + stage * G::STAGE_B + xrd[1];
        const unsigned wa = lds_base + stage * G::STAGE_B + wrd;
        uintx2 t[2][2][2];                                       // [position block][window row][channel half]
        uintx4 wv[G::NN];
        if constexpr (n == 3) {
            asm volatile(
                "ds_read_b64_tr_b16 %0, %17\n\t"
                "ds_read_b64_tr_b16 %1, %17 offset:%21\n\t"
                "ds_read_b64_tr_b16 %2, %17 offset:%20\n\t"
                "ds_read_b64_tr_b16 %3, %17 offset:%22\n\t"
                "ds_read_b64_tr_b16 %4, %18\n\t"
                "ds_read_b64_tr_b16 %5, %18 offset:%21\n\t"
                "ds_read_b64_tr_b16 %6, %18 offset:%20\n\t"
                "ds_read_b64_tr_b16 %7, %18 offset:%22\n\t"
                "ds_read_b128 %8, %19\n\t"
                "ds_read_b128 %9, %19 offset:2048\n\t"
                "ds_read_b128 %10, %19 offset:4096\n\t"
                "ds_read_b128 %11, %19 offset:6144\n\t"
                "ds_read_b128 %12, %19 offset:8192\n\t"
                "ds_read_b128 %13, %19 offset:10240\n\t"
                "ds_read_b128 %14, %19 offset:12288\n\t"
                "ds_read_b128 %15, %19 offset:14336\n\t"
                "ds_read_b128 %16, %19 offset:16384\n\t"
                "s_waitcnt lgkmcnt(0)"
                : "=&v"(t[0][0][0]), "=&v"(t[0][0][1]), "=&v"(t[0][1][0]), "=&v"(t[0][1][1]), "=&v"(t[1][0][0]),
                  "=&v"(t[1][0][1]), "=&v"(t[1][1][0]), "=&v"(t[1][1][1]), "=&v"(wv[0]), "=&v"(wv[1]), "=&v"(wv[2]),
                  "=&v"(wv[3]), "=&v"(wv[4]), "=&v"(wv[5]), "=&v"(wv[6]), "=&v"(wv[7]), "=&v"(wv[8])
                : "v"(xa0), "v"(xa1), "v"(wa), "n"(G::ROW_B), "n"(4 * G::CS), "n"(G::ROW_B + 4 * G::CS)
                : "memory");
        } else {
            asm volatile(
                "ds_read_b64_tr_b16 %0, %12\n\t"
                "ds_read_b64_tr_b16 %1, %12 offset:%16\n\t"
                "ds_read_b64_tr_b16 %2, %12 offset:%15\n\t"
                "ds_read_b64_tr_b16 %3, %12 offset:%17\n\t"
                "ds_read_b64_tr_b16 %4, %13\n\t"
                "ds_read_b64_tr_b16 %5, %13 offset:%16\n\t"
                "ds_read_b64_tr_b16 %6, %13 offset:%15\n\t"
                "ds_read_b64_tr_b16 %7, %13 offset:%17\n\t"
                "ds_read_b128 %8, %14\n\t"
                "ds_read_b128 %9, %14 offset:2048\n\t"
                "ds_read_b128 %10, %14 offset:4096\n\t"
                "ds_read_b128 %11, %14 offset:6144\n\t"
                "s_waitcnt lgkmcnt(0)"
                : "=&v"(t[0][0][0]), "=&v"(t[0][0][1]), "=&v"(t[0][1][0]), "=&v"(t[0][1][1]), "=&v"(t[1][0][0]),
                  "=&v"(t[1][0][1]), "=&v"(t[1][1][0]), "=&v"(t[1][1][1]), "=&v"(wv[0]), "=&v"(wv[1]), "=&v"(wv[2]),
                  "=&v"(wv[3])
                : "v"(xa0), "v"(xa1), "v"(wa), "n"(G::ROW_B), "n"(4 * G::CS), "n"(G::ROW_B + 4 * G::CS)
                : "memory");
        }
        // Window fragments [block][row][column]: column 0 as read; column 1 = column 0 of the
        // next quad, i.e. the next lane's value (lanes 0..31 and 32..63 hold the two channel
        // halves of columns 0..31).  Lanes 31 and 63 take theirs from the block to the right
        // when the wave holds it; otherwise they belong to a quad column past the row's last
        // valid one and may hold anything.
        bf16x8 xf[2][2][2];
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int dy = 0; dy < 2; ++dy) {
                const uintx4 x0 = __builtin_shufflevector(t[pb][dy][0], t[pb][dy][1], 0, 1, 2, 3);
                uintx4 x1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    unsigned v = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x0[i], 0x130, 0xf, 0xf, false);   // lane l <- lane l + 1
                    if (G::CB == 2 && pb == 0) {
                        const unsigned nb = i < 2 ? t[1][dy][0][i] : t[1][dy][1][i - 2];
                        const unsigned e0 = (unsigned)__builtin_amdgcn_readlane((int)nb, 0);
                        const unsigned e1 = (unsigned)__builtin_amdgcn_readlane((int)nb, 32);
                        v = lane == 31 ? e0 : v;
                        v = lane == 63 ? e1 : v;
                    }
                    x1[i] = v;
                }
                xf[pb][dy][0] = __builtin_bit_cast(bf16x8, x0);
                xf[pb][dy][1] = __builtin_bit_cast(bf16x8, x1);
            }
#pragma unroll
        for (int cls = 0; cls < 4; ++cls) {
            const int r = cls >> 1, s = cls & 1;
            const int Ta = taps_for_parity(n, r), Tb = taps_for_parity(n, s);
#pragma unroll
            for (int a = 0; a < Ta; ++a)
#pragma unroll
                for (int bq = 0; bq < Tb; ++bq) {
                    const int T = class_tap_base(n, cls) + a * Tb + bq;
                    const bf16x8 wf = __builtin_bit_cast(bf16x8, wv[T]);
#pragma unroll
                    for (int pb = 0; pb < 2; ++pb)
                        acc[cls][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[pb][r + a][s + bq],
                                                                                acc[cls][pb], 0, 0, 0);
                }
        }
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
        wait_loads_and_meet(c + 1 < nchunks ? my_slabs : 0);
        if (c + 2 < nchunks) issue_direct(cur == 0 ? 2 : cur - 1);
        multiply(cur);
        cur = cur == 2 ? 0 : cur + 1;
    }

    // ---- epilogue -----------------------------------------------------------------------------
    // Per output channel the tile is one contiguous run of rows_out * M floats.  The four
    // classes are interleaved into that run in LDS, 32 channels per pass, and streamed out
    // with 16-byte stores whose lane quads sit in one 64-byte segment (lane t of a channel
    // owns floats [base64 + 4t, +4), base64 = run start rounded down to 64 bytes); only the
    // groups cut by the ends of a run use scalar stores.
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
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int cl = 8 * (v >> 2) + 4 * kk + (v & 3);
                    const unsigned g_co = g_first + (unsigned)(pass * 32 + cl) * MM;
                    float *e = Es + cl * G::ESTRIDE + (g_co & 3u) + 2 * ti[pb] * G::M + 2 * tj[pb];
#pragma unroll
                    for (int r = 0; r < 2; ++r) {
                        if (2 * ti[pb] + r >= rows_out) continue;
                        e[r * G::M] = acc[2 * r][pb][v];
                        if (x1_ok) e[r * G::M + 1] = acc[2 * r + 1][pb][v];
                    }
                }
            }
        }
        lds_barrier();
        // Wave w streams channels w, w + 4, ...; its lanes walk the channel's 16-byte groups.
        for (int cl = wave; cl < 32; cl += R_THREADS / 64) {
            const unsigned g_co = g_first + (unsigned)(pass * 32 + cl) * MM;
            const unsigned base64 = g_co & ~15u;
            const float *erow = Es + cl * G::ESTRIDE + (int)(g_co & 3u);
            for (int t = lane; t < G::TG; t += 64) {
                const unsigned f0 = base64 + 4u * t;
                const int rel = (int)(f0 - g_co);
                if (rel + 3 < 0 || rel >= L) continue;
                const float *src = erow + rel;                       // 16-byte aligned
                float *dst = out + f0;
                if (rel >= 0 && rel + 3 < L) {
                    *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src);
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (rel + k >= 0 && rel + k < L) dst[k] = src[k];
                }
            }
        }
    }
}

template <int n, int N>
hipError_t launch_ring(const uint16_t *in, const uint16_t *w_seg, float *out, const RingParams &p, hipStream_t stream)
{
    using G = RingGeom<n, N>;
    static_assert(G::LDS_B <= 80 * 1024, "two workgroups per CU");
    if (G::LDS_B > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_bf16_ring_kernel<n, N>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_B);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)p.B * p.tiles_co * G::STRIPS;
    hipLaunchKernelGGL((igemm_bf16_ring_kernel<n, N>), dim3(blocks), dim3(R_THREADS), G::LDS_B, stream, in, w_seg, out, p);
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

hipError_t launch_igemm_bf16_ring(const void *in, const void *w_seg, float *out, const Shape &s, hipStream_t stream)
{
    if (!igemm_bf16_ring_supported(s)) return hipErrorInvalidValue;
    RingParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.tiles_co = s.Cout / R_TCO;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, KST_BF16);
    const uint16_t *i16 = (const uint16_t *)in, *w16 = (const uint16_t *)w_seg;
    switch (s.n * 1000 + s.N) {
        case 2032: return launch_ring<2, 32>(i16, w16, out, p, stream);
        case 2064: return launch_ring<2, 64>(i16, w16, out, p, stream);
        case 3032: return launch_ring<3, 32>(i16, w16, out, p, stream);
        case 3064: return launch_ring<3, 64>(i16, w16, out, p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace kst
