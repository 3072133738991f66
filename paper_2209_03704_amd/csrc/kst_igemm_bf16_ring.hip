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
//     address, so the window column dx = 1 of Eqs. 7-10 cannot be read from the same
//     image; a second image shifted left by one pixel is staged through registers
//     (one 16-byte load + one 4-byte load, four funnel shifts, one LDS write);
//   * the segregated weights already sit in fragment order in HBM and are copied by
//     LDS-direct loads as well;
//   * two stages form a ring: chunk k+1 lands in one stage while chunk k is
//     multiplied out of the other, with one workgroup barrier per chunk.
// Tile: TI quad rows x 64 output channels per 256-thread workgroup, positions in
// blocks of 32 consecutive quad columns of one quad row (the transposing read needs
// consecutive pixels), 4 waves of 32 channels x 64 positions x 4 parity classes,
// two workgroups per CU.  The epilogue is the one of the row-strip kernel: classes
// interleaved in an LDS image, streamed out as 16-byte stores whose lane quads sit
// in one 64-byte segment.
#include "kst_igemm_common.h"

namespace kst {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int R_THREADS = 256;
constexpr int R_TCO = 64;
constexpr int R_KC = 16;               // channels per chunk = one MFMA reduction step

template <int n, int N>
struct RingGeom {
    static_assert(n == 2 || n == 3, "window columns 0 and 1 only");
    static_assert(N == 32 || N == 64 || N == 128, "row of whole 32-column blocks");
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
    static constexpr int STAGE_B = W_B + 2 * COPY_B;
    static constexpr int W_SLABS = NN * 2;               // 1 KiB slabs (one wave-wide LDS-direct load each)
    static constexpr int X_SLABS = COPY_B / 1024;
    static_assert(COPY_B % 1024 == 0, "image is a whole number of slabs");
    static constexpr int SLABS = W_SLABS + X_SLABS;
    static constexpr int KMAX = (SLABS + 3) / 4;         // slabs per wave
    static constexpr int RU = R_KC * ROWS * UPR;         // real units of the shifted image
    static constexpr int NU = (RU + R_THREADS - 1) / R_THREADS;
    static constexpr int LMAX = 2 * TI * M;              // floats per channel run of a tile
    static constexpr int ESTRIDE = (LMAX + 3 + 3) & ~3;  // floats per channel in the epilogue image
    static constexpr int TG = (15 + LMAX - 1) / 4 + 1;   // 16-byte groups per channel run, upper bound
    static constexpr int EPI_B = 32 * ESTRIDE * 4;
    static constexpr int LDS_B = 2 * STAGE_B > EPI_B ? 2 * STAGE_B : EPI_B;
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
    // ---- shifted image: unit -> (channel, row, 8 pixels), through registers -------------------
    unsigned b_off[G::NU], b_xoff[G::NU];
    int b_dst[G::NU];
    bool b_ok[G::NU];
#pragma unroll
    for (int j = 0; j < G::NU; ++j) {
        const int u = tid + j * R_THREADS;
        b_ok[j] = u < G::RU;
        const int uu = b_ok[j] ? u : 0;
        const int ci = uu / (G::ROWS * G::UPR);
        const int rem = uu - ci * (G::ROWS * G::UPR);
        const int row = rem / G::UPR, x8 = rem - row * G::UPR;
        const int grow = min(i0 + row, N - 1);
        b_off[j] = (((unsigned)b * p.Cin + ci) * N + grow) * N + x8 * 8;
        // The pixel after the unit; for the last unit of a row it only feeds a column no
        // valid position reads, so that lane re-reads its own first word.
        b_xoff[j] = x8 + 1 < G::UPR ? b_off[j] + 8 : b_off[j];
        b_dst[j] = G::W_B + G::COPY_B + ci * G::CS + row * G::ROW_B + x8 * 16;
    }

    floatx16 acc[4][2];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][pb][v] = 0.0f;

    uint4 b_reg[G::NU];
    unsigned b_ext[G::NU];

    auto load_shifted = [&]() {
#pragma unroll
        for (int j = 0; j < G::NU; ++j) {
            if (b_ok[j]) {
                b_reg[j] = *reinterpret_cast<const uint4 *>(in + b_off[j]);
                b_ext[j] = *reinterpret_cast<const unsigned *>(in + b_xoff[j]);
            }
            b_off[j] += (unsigned)R_KC * N * N;
            b_xoff[j] += (unsigned)R_KC * N * N;
        }
    };
    auto store_shifted = [&](int stage) {
#pragma unroll
        for (int j = 0; j < G::NU; ++j) {
            if (b_ok[j]) {
                const uint4 d = b_reg[j];
                const uint4 o = make_uint4(__builtin_amdgcn_alignbit(d.y, d.x, 16), __builtin_amdgcn_alignbit(d.z, d.y, 16),
                                           __builtin_amdgcn_alignbit(d.w, d.z, 16), __builtin_amdgcn_alignbit(b_ext[j], d.w, 16));
                *reinterpret_cast<uint4 *>(lds_raw + stage * G::STAGE_B + b_dst[j]) = o;
            }
        }
    };
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
    // The window fragments of a chunk: (position block, window row, window column) -> eight
    // channels of one pixel per lane.  They are fetched before the next chunk's LDS-direct
    // loads are issued: the compiler makes a transposing read wait for every LDS-direct load
    // in flight, and at that point there is none.
    bf16x8 xf[2][2][2];
    auto fetch_windows = [&](int stage) {
        const unsigned char *sb = lds_raw + stage * G::STAGE_B;
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int dy = 0; dy < 2; ++dy)
#pragma unroll
                for (int dx = 0; dx < 2; ++dx) {
                    const unsigned char *a = sb + xrd[pb] + dx * G::COPY_B + dy * G::ROW_B;
                    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((KST_LDS(shortx4) *)a);
                    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((KST_LDS(shortx4) *)(a + 4 * G::CS));
                    const shortx8 t = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    xf[pb][dy][dx] = __builtin_bit_cast(bf16x8, t);
                }
    };
    auto multiply = [&](int stage) {
        const unsigned char *sb = lds_raw + stage * G::STAGE_B;
#pragma unroll
        for (int cls = 0; cls < 4; ++cls) {
            const int r = cls >> 1, s = cls & 1;
            const int Ta = taps_for_parity(n, r), Tb = taps_for_parity(n, s);
#pragma unroll
            for (int a = 0; a < Ta; ++a)
#pragma unroll
                for (int bq = 0; bq < Tb; ++bq) {
                    const int T = class_tap_base(n, cls) + a * Tb + bq;
                    const bf16x8 wf = *reinterpret_cast<const bf16x8 *>(sb + T * (2 * R_TCO * 16) + wrd);
#pragma unroll
                    for (int pb = 0; pb < 2; ++pb)
                        acc[cls][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[pb][r + a][s + bq],
                                                                                acc[cls][pb], 0, 0, 0);
                }
        }
    };

    // ---- reduction over the input channels ------------------------------------------------------
    const int nchunks = p.Cin / R_KC;
    load_shifted();
    issue_direct(0);
    store_shifted(0);
    for (int c = 0; c < nchunks; ++c) {
        lds_barrier();                       // stage c & 1 is complete; the other stage is free
        const int cur = c & 1;
        const bool more = c + 1 < nchunks;   // uniform
        fetch_windows(cur);
        if (more) {
            load_shifted();
            issue_direct(cur ^ 1);
        }
        multiply(cur);
        if (more) store_shifted(cur ^ 1);
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
    if (s.N != 32 && s.N != 64 && s.N != 128) return false;
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
        case 2128: return launch_ring<2, 128>(i16, w16, out, p, stream);
        case 3032: return launch_ring<3, 32>(i16, w16, out, p, stream);
        case 3064: return launch_ring<3, 64>(i16, w16, out, p, stream);
        case 3128: return launch_ring<3, 128>(i16, w16, out, p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace kst
