// Matrix-core segregated forward pass for bfloat16 operands, row-strip tiling.
//
// Same arithmetic as kst_igemm_bf16.hip (Section 3.3, Eqs. 7-10 as four implicit
// GEMMs on v_mfma_f32_32x32x16_bf16, fp32 accumulation), organised for maps whose
// quad rows are at most 128 quads wide:
//   * a workgroup owns TI whole quad rows of one batch item (TI * E <= 128 quad
//     positions) for 64 output channels, so its input is TI + fl full rows (one
//     contiguous run per channel) and its output is 2*TI full rows per channel;
//   * 4 waves, each 32 channels x 64 positions x 4 parity classes (128 fp32
//     accumulators): one weight fragment feeds two position blocks, which keeps
//     the LDS read traffic per MFMA low enough for the bf16 MFMA rate; two such
//     workgroups share a CU, so one's epilogue overlaps the other's MFMA loop;
//   * operands of chunk k+1 travel from HBM into registers while chunk k is
//     multiplied out of LDS; the input is transposed from NCHW to [pixel][ci]
//     on the way (eight 4-byte loads of one pixel pair, eight channels -> two
//     16-byte LDS writes).
#include "kst_igemm_common.h"

namespace kst {


namespace {

constexpr int S_THREADS = 256;
constexpr int S_TCO = 64;
constexpr int S_KC = 16;               // channels per chunk = one MFMA reduction step
constexpr int S_XS = S_KC + 8;         // LDS pixel stride in bf16 (48 bytes)
constexpr int S_NXU = 2;               // (pixel pair, channel octet) units per lane per chunk at most

struct StripParams {
    int B, Cin, Cout, N, M, E;
    int TI, strips, tiles_co;
    int lrows, npix;
    int cin_oct;
    int estride;            // floats per channel in the epilogue's LDS image (multiple of 4)
    int tg;                 // 16-byte groups per channel run, upper bound
    unsigned off[4];
    Epilogue epi;
};

template <int n, bool F16>
__global__ void __launch_bounds__(S_THREADS, 2) igemm_bf16_strip_kernel(const uint16_t *__restrict__ in,
                                                                       const uint16_t *__restrict__ w_seg,
                                                                       float *__restrict__ out, StripParams p)
{
    constexpr int fl = n / 2;
    constexpr int NN = n * n;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint16_t *Xs = reinterpret_cast<uint16_t *>(lds_raw);                                // [npix][S_XS]
    uint4 *Ws = reinterpret_cast<uint4 *>(lds_raw + (size_t)p.npix * S_XS * 2);         // [NN][2][S_TCO]

    unsigned id = blockIdx.x;
    const int strip = (int)(id % (unsigned)p.strips);
    id /= (unsigned)p.strips;
    const int tile_co = (int)(id % (unsigned)p.tiles_co);
    const int b = (int)(id / (unsigned)p.tiles_co);
    const int co0 = tile_co * S_TCO;
    const int i0 = strip * p.TI;
    const int rows_q = min(p.TI, p.E - i0);
    const int npos = rows_q * p.E;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kk = lane >> 5;
    const int wco = wave & 1, wpos = wave >> 1;

    // This lane's two quad positions (clamped: every LDS read stays inside the staged rows).
    int ti[2], tj[2], xbase[2];
    bool pos_ok[2];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
        int m = (wpos * 2 + pb) * 32 + l32;
        pos_ok[pb] = m < npos;
        if (!pos_ok[pb]) m = npos - 1;
        ti[pb] = m / p.E;
        tj[pb] = m - ti[pb] * p.E;
        xbase[pb] = (ti[pb] * p.N + tj[pb]) * S_XS + kk * 8;
    }
    const int wbase = kk * S_TCO + wco * 32 + l32;

    // ---- staging plan ------------------------------------------------------------------------
    // Weights: lane -> (tap parity, octet, channel), unit k -> tap 2k + (tid >> 7): one 16-byte group each.
    constexpr int NWU = (NN + 1) / 2;
    const int w_oc = (tid >> 6) & 1, w_co = tid & 63;
    unsigned w_off[NWU], w_inc[NWU];
    bool w_ok[NWU];
#pragma unroll
    for (int k = 0; k < NWU; ++k) {
        const int T = 2 * k + (tid >> 7);
        int cls = 0;
#pragma unroll
        for (int q = 1; q < 4; ++q)
            if (T >= class_tap_base(n, q)) cls = q;
        const int Tp = class_taps(n, cls), t = T - class_tap_base(n, cls);
        w_ok[k] = T < NN && co0 + w_co < p.Cout;
        w_off[k] = w_ok[k] ? p.off[cls] + (((unsigned)w_oc * Tp + t) * p.Cout + co0 + w_co) * 8u : 0u;
        w_inc[k] = w_ok[k] ? 2u * Tp * p.Cout * 8u : 0u;
    }
    // Input: unit -> (pixel pair, octet); eight channels of the pair are loaded as 4-byte words.
    const int npairs = p.npix >> 1;
    unsigned x_off[S_NXU], x_incv[S_NXU];
    int x_dst[S_NXU], x_oc[S_NXU];
    bool x_ok[S_NXU];
#pragma unroll
    for (int k = 0; k < S_NXU; ++k) {
        const int e = tid + k * S_THREADS;
        const int oc = e / npairs, pp = e - oc * npairs;
        const int pix = 2 * pp;
        const int lr = pix / p.N, x = pix - lr * p.N;
        x_ok[k] = e < 2 * npairs && i0 + lr < p.N;
        x_oc[k] = oc;
        x_off[k] = x_ok[k] ? ((((unsigned)b * p.Cin + oc * 8) * p.N + i0 + lr) * p.N + x) : 0u;
        x_incv[k] = x_ok[k] ? (unsigned)S_KC * p.N * p.N : 0u;
        x_dst[k] = pix * S_XS + oc * 8;
    }
    const unsigned plane = (unsigned)p.N * p.N;

    floatx16 acc[4][2];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][pb][v] = 0.0f;

    uint4 w_reg[NWU];
    unsigned x_reg[S_NXU][8];

    auto load_chunk = [&](int ci0) {
        const int oct0 = ci0 >> 3;
#pragma unroll
        for (int k = 0; k < NWU; ++k) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (w_ok[k] && oct0 + w_oc < p.cin_oct) v = *reinterpret_cast<const uint4 *>(w_seg + w_off[k]);
            w_reg[k] = v;
            w_off[k] += w_inc[k];
        }
#pragma unroll
        for (int k = 0; k < S_NXU; ++k) {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                unsigned v = 0;
                if (x_ok[k] && ci0 + x_oc[k] * 8 + c < p.Cin)
                    v = *reinterpret_cast<const unsigned *>(in + x_off[k] + c * plane);
                x_reg[k][c] = v;
            }
            x_off[k] += x_incv[k];
        }
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int k = 0; k < NWU; ++k)
            if (2 * k + (tid >> 7) < NN) Ws[k * S_THREADS + tid] = w_reg[k];
#pragma unroll
        for (int k = 0; k < S_NXU; ++k) {
            if (tid + k * S_THREADS < 2 * npairs) {
                const unsigned *v = x_reg[k];
                const uint4 lo = make_uint4((v[0] & 0xffffu) | (v[1] << 16), (v[2] & 0xffffu) | (v[3] << 16),
                                            (v[4] & 0xffffu) | (v[5] << 16), (v[6] & 0xffffu) | (v[7] << 16));
                const uint4 hi = make_uint4((v[0] >> 16) | (v[1] & 0xffff0000u), (v[2] >> 16) | (v[3] & 0xffff0000u),
                                            (v[4] >> 16) | (v[5] & 0xffff0000u), (v[6] >> 16) | (v[7] & 0xffff0000u));
                *reinterpret_cast<uint4 *>(Xs + x_dst[k]) = lo;              // first pixel of the pair
                *reinterpret_cast<uint4 *>(Xs + x_dst[k] + S_XS) = hi;       // second pixel
            }
        }
    };

    load_chunk(0);
    store_chunk();
    __syncthreads();

    for (int ci0 = 0; ci0 < p.Cin; ci0 += S_KC) {
        const int cn = ci0 + S_KC;
        if (cn < p.Cin) load_chunk(cn);

        bf16x8 xf[2][fl + 1][fl + 1];
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int dy = 0; dy <= fl; ++dy)
#pragma unroll
                for (int dx = 0; dx <= fl; ++dx)
                    xf[pb][dy][dx] = *reinterpret_cast<const bf16x8 *>(Xs + xbase[pb] + (dy * p.N + dx) * S_XS);
#pragma unroll
        for (int cls = 0; cls < 4; ++cls) {
            const int r = cls >> 1, s = cls & 1;
            const int Ta = taps_for_parity(n, r), Tb = taps_for_parity(n, s);
#pragma unroll
            for (int a = 0; a < Ta; ++a)
#pragma unroll
                for (int bq = 0; bq < Tb; ++bq) {
                    const int T = class_tap_base(n, cls) + a * Tb + bq;
                    const bf16x8 wf = *reinterpret_cast<const bf16x8 *>(&Ws[T * 2 * S_TCO + wbase]);
#pragma unroll
                    for (int pb = 0; pb < 2; ++pb)
                        acc[cls][pb] = mfma16<F16>(wf, xf[pb][r + a][s + bq],
                                                                                acc[cls][pb]);
                }
        }
        if (cn >= p.Cin) break;
        __syncthreads();
        store_chunk();
        __syncthreads();
    }

    // ---- epilogue -----------------------------------------------------------------------------
    // Per output channel the strip is one contiguous run of rows_out * M floats.  The four
    // classes are interleaved into that run in LDS, 32 channels per pass, and streamed out
    // with 16-byte stores whose lane quads sit in one 64-byte segment (lane t of a channel
    // owns floats [base64 + 4t, +4), base64 = run start rounded down to 64 bytes); only the
    // groups cut by the ends of a run use scalar stores.
    float *Es = reinterpret_cast<float *>(lds_raw);                 // [32][estride]
    const int rows_out = min(2 * rows_q, p.M - 2 * i0);
    const int L = rows_out * p.M;
    const unsigned MM = (unsigned)p.M * p.M;
    const unsigned g_first = (((unsigned)b * p.Cout + co0) * p.M + 2 * i0) * p.M;   // run start of channel co0
    for (int pass = 0; pass < 2; ++pass) {
        __syncthreads();                                             // LDS is free: K loop / previous pass read it
        const int nco = min(32, p.Cout - (co0 + pass * 32));
        if (nco <= 0) break;                                         // uniform
        if (wco == pass) {
#pragma unroll
            for (int pb = 0; pb < 2; ++pb) {
                if (!pos_ok[pb]) continue;
                const bool x1_ok = 2 * tj[pb] + 1 < p.M;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int cl = 8 * (v >> 2) + 4 * kk + (v & 3);
                    if (cl >= nco) continue;
                    const unsigned g_co = g_first + (unsigned)(pass * 32 + cl) * MM;
                    float *e = Es + cl * p.estride + (g_co & 3u) + 2 * ti[pb] * p.M + 2 * tj[pb];
#pragma unroll
                    for (int r = 0; r < 2; ++r) {
                        if (2 * ti[pb] + r >= rows_out) continue;
                        e[r * p.M] = acc[2 * r][pb][v];
                        if (x1_ok) e[r * p.M + 1] = acc[2 * r + 1][pb][v];
                    }
                }
            }
        }
        __syncthreads();
        // Wave w streams channels w, w + 4, ...; its lanes walk the channel's 16-byte groups.
        for (int cl = wave; cl < nco; cl += S_THREADS / 64) {
            const unsigned g_co = g_first + (unsigned)(pass * 32 + cl) * MM;
            const unsigned base64 = g_co & ~15u;
            const float *erow = Es + cl * p.estride + (int)(g_co & 3u);
            const bool epi = epi_on(p.epi);                             // uniform
            const float bias = epi ? epi_bias(p.epi, co0 + pass * 32 + cl) : 0.0f;
            for (int t = lane; t < p.tg; t += 64) {
                const unsigned f0 = base64 + 4u * t;
                const int rel = (int)(f0 - g_co);
                if (rel + 3 < 0 || rel >= L) continue;
                const float *src = erow + rel;                       // 16-byte aligned
                float *dst = out + f0;
                if (rel >= 0 && rel + 3 < L) {
                    float4 v4 = *reinterpret_cast<const float4 *>(src);
                    if (epi) epi_apply4(v4.x, v4.y, v4.z, v4.w, bias, p.epi.act);
                    store_streaming4(dst, v4.x, v4.y, v4.z, v4.w);
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (rel + k >= 0 && rel + k < L) dst[k] = epi ? epi_apply(src[k], bias, p.epi.act) : src[k];
                }
            }
        }
    }
}

bool strip_plan(const Shape &s, StripParams &p, size_t &lds)
{
    if (s.n > 4 || (s.N & 1) || s.E > 128 || s.E < 16) return false;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.N = s.N; p.M = s.M; p.E = s.E;
    p.TI = 128 / s.E;
    p.strips = (s.E + p.TI - 1) / p.TI;
    p.tiles_co = (s.Cout + S_TCO - 1) / S_TCO;
    p.lrows = p.TI + s.fl;
    p.npix = p.lrows * s.N;
    if (p.npix > S_NXU * S_THREADS) return false;             // (npix / 2 pairs) * 2 octets units
    p.cin_oct = (s.Cin + 7) / 8;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, KST_BF16);
    p.epi = s.epi;
    const int Lmax = 2 * p.TI * s.M;
    p.estride = (Lmax + 3 + 3) & ~3;
    p.tg = (15 + Lmax - 1) / 4 + 1;
    lds = (size_t)p.npix * S_XS * 2 + (size_t)s.n * s.n * 2 * S_TCO * 16;
    const size_t lds_epi = (size_t)32 * p.estride * sizeof(float);
    if (lds_epi > lds) lds = lds_epi;
    return lds <= 160 * 1024 && (size_t)s.B * p.tiles_co * p.strips < 0x7fffffffu;
}

template <int n, bool F16>
hipError_t launch_n(const uint16_t *in, const uint16_t *w_seg, float *out, const StripParams &p, size_t lds,
                    hipStream_t stream)
{
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_bf16_strip_kernel<n, F16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)p.B * p.tiles_co * p.strips;
    hipLaunchKernelGGL((igemm_bf16_strip_kernel<n, F16>), dim3(blocks), dim3(S_THREADS), lds, stream, in, w_seg, out, p);
    return hipGetLastError();
}

}  // namespace

bool igemm_bf16_strip_supported(const Shape &s)
{
    StripParams p;
    size_t lds;
    return strip_plan(s, p, lds);
}

hipError_t launch_igemm_bf16_strip(const void *in, const void *w_seg, float *out, const Shape &s, bool f16,
                                   hipStream_t stream)
{
    StripParams p;
    size_t lds;
    if (!strip_plan(s, p, lds)) return hipErrorInvalidValue;
    const uint16_t *i16 = (const uint16_t *)in, *w16 = (const uint16_t *)w_seg;
    switch (s.n) {
        case 1: return f16 ? launch_n<1, true>(i16, w16, out, p, lds, stream) : launch_n<1, false>(i16, w16, out, p, lds, stream);
        case 2: return f16 ? launch_n<2, true>(i16, w16, out, p, lds, stream) : launch_n<2, false>(i16, w16, out, p, lds, stream);
        case 3: return f16 ? launch_n<3, true>(i16, w16, out, p, lds, stream) : launch_n<3, false>(i16, w16, out, p, lds, stream);
        case 4: return f16 ? launch_n<4, true>(i16, w16, out, p, lds, stream) : launch_n<4, false>(i16, w16, out, p, lds, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace kst
