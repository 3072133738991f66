// Matrix-core (MFMA) segregated forward pass, bfloat16 operands, fp32
// accumulation and output.  Same decomposition as the fp32 kernel (Section
// 3.3, Eqs. 7-10 as four implicit GEMMs over one shared input tile, output
// channels down the MFMA rows, quad positions across its columns); what
// differs is the operand feed.  v_mfma_f32_32x32x16_bf16 takes, per lane, eight
// consecutive reduction indices of one row/column, so the reduction index is
// ordered (tap, ci) with ci fastest and both LDS images keep eight channels
// contiguous: weights as [tap][ci/8][co][8] (the segregated layout as it
// is), the input transposed on the way in from NCHW to [pixel][ci].
#include "kst_igemm_common.h"

namespace kst {


constexpr int H_KC = 16;               // input channels staged per step = one MFMA reduction step
constexpr int H_XS = H_KC + 8;         // LDS pixel stride in bf16: 48 bytes, conflict-free 16-byte reads

template <int n, bool F16>
__global__ void __launch_bounds__(G_THREADS) igemm_bf16_kernel(const uint16_t *__restrict__ in,
                                                                 const uint16_t *__restrict__ w_seg,
                                                                 float *__restrict__ dst, IgemmParams p)
{
    constexpr int fl = n / 2;
    constexpr int NN = n * n;
    constexpr int OCT = H_KC / 8;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int npix = p.lrows * p.N;
    uint16_t *Xs = reinterpret_cast<uint16_t *>(lds_raw);                      // [npix][H_XS]
    uint4 *Ws = reinterpret_cast<uint4 *>(lds_raw + (((size_t)npix * H_XS * 2 + 15) & ~(size_t)15));  // [NN][OCT][G_TCO]

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
    const int R0 = b0 * p.N + i0;

    int m = m0 + wpos * 32 + l32;
    const bool m_valid = m < p.Mtot;
    if (!m_valid) m = p.Mtot - 1;
    const int mb = m / p.EE;
    const int mrem = m - mb * p.EE;
    const int mi = mrem / p.E, mj = mrem - mi * p.E;
    const int xbase = (((mb * p.N + mi) - R0) * p.N + mj) * H_XS + kk * 8;   // in bf16 elements
    const int wbase = kk * G_TCO + wco * 64 + l32;                              // in 16-byte units

    floatx16 acc[4][2];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][h][v] = 0.0f;

    const int ci_begin = split * p.ci_per_split;
    const int ci_end = min(p.Cin, ci_begin + p.ci_per_split);
    const int cin_oct = (p.Cin + 7) / 8;

    for (int ci0 = ci_begin; ci0 < ci_end; ci0 += H_KC) {
        if (ci0 != ci_begin) __syncthreads();
        // Input rows [R0, R0 + lrows) of channels ci0 .. ci0+15, transposed to [pixel][ci].
        for (int e = tid; e < H_KC * npix; e += G_THREADS) {
            const int c = e / npix;
            const int pix = e - c * npix;
            const int lr = pix / p.N, x = pix - lr * p.N;
            const int R = R0 + lr;
            const int bb = R / p.N, y = R - bb * p.N;
            uint16_t v = 0;
            if (bb < p.B && ci0 + c < ci_end)
                v = in[(((size_t)bb * p.Cin + ci0 + c) * p.N + y) * p.N + x];
            Xs[pix * H_XS + c] = v;
        }
        // Weights: 16-byte groups of eight channels, all taps, TCO output channels.
        for (int e = tid; e < NN * OCT * G_TCO; e += G_THREADS) {
            const int tco = e % G_TCO;
            const int rest = e / G_TCO;
            const int oc = rest % OCT, T = rest / OCT;
            int cls = 0;
#pragma unroll
            for (int q = 1; q < 4; ++q)
                if (T >= class_tap_base(n, q)) cls = q;
            const int Tp = class_taps(n, cls);
            const int t = T - class_tap_base(n, cls);
            const int oct = ci0 / 8 + oc;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (co0 + tco < p.Cout && oct < cin_oct && oct * 8 < ci_end)
                v = *reinterpret_cast<const uint4 *>(w_seg + p.off[cls] +
                                                     (((size_t)oct * Tp + t) * p.Cout + co0 + tco) * 8);
            Ws[e] = v;
        }
        __syncthreads();

        bf16x8 xf[fl + 1][fl + 1];
#pragma unroll
        for (int dy = 0; dy <= fl; ++dy)
#pragma unroll
            for (int dx = 0; dx <= fl; ++dx)
                xf[dy][dx] = *reinterpret_cast<const bf16x8 *>(Xs + xbase + (dy * p.N + dx) * H_XS);
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
                        const bf16x8 wf = *reinterpret_cast<const bf16x8 *>(&Ws[T * OCT * G_TCO + wbase + h * 32]);
                        acc[cls][h] = mfma16<F16>(wf, xf[r + a][s + bq], acc[cls][h]);
                    }
                }
        }
    }

    if (!m_valid) return;
    igemm_store(dst + (size_t)split * p.out_elems, acc, p, co0 + wco * 64, kk, mb, mi, mj, p.splits == 1);
}

static IgemmParams plan(const Shape &s) { return igemm_plan(s, KST_BF16, H_KC); }

static size_t lds_bytes(const IgemmParams &p, int n)
{
    const size_t x = (((size_t)p.lrows * p.N * H_XS * 2) + 15) & ~(size_t)15;
    return x + (size_t)n * n * (H_KC / 8) * G_TCO * 16;
}

bool igemm_bf16_supported(const Shape &s)
{
    if (igemm_bf16_ring_supported(s) || igemm_bf16_strip_supported(s)) return true;
    if (s.n > 7) return false;
    return lds_bytes(plan(s), s.n) <= 160 * 1024;
}

size_t igemm_bf16_workspace_bytes(const Shape &s)
{
    if (igemm_bf16_ring_supported(s) || igemm_bf16_strip_supported(s)) return 0;
    const IgemmParams p = plan(s);
    return p.splits > 1 ? (size_t)p.splits * p.out_elems * sizeof(float) : 0;
}

template <int n, bool F16>
static hipError_t launch_n(const uint16_t *in, const uint16_t *w_seg, float *dst, const IgemmParams &p,
                           hipStream_t stream)
{
    const size_t lds = lds_bytes(p, n);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_bf16_kernel<n, F16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)p.tiles_m * p.tiles_co * p.splits;
    hipLaunchKernelGGL((igemm_bf16_kernel<n, F16>), dim3(blocks), dim3(G_THREADS), lds, stream, in, w_seg, dst, p);
    return hipGetLastError();
}

template <bool F16>
static hipError_t launch_plain(const void *in_v, const void *w_seg_v, float *out, void *ws, const Shape &s,
                               hipStream_t stream)
{
    const uint16_t *in = (const uint16_t *)in_v, *w_seg = (const uint16_t *)w_seg_v;
    const IgemmParams p = plan(s);
    float *dst = p.splits > 1 ? (float *)ws : out;
    hipError_t e;
    switch (s.n) {
        case 1: e = launch_n<1, F16>(in, w_seg, dst, p, stream); break;
        case 2: e = launch_n<2, F16>(in, w_seg, dst, p, stream); break;
        case 3: e = launch_n<3, F16>(in, w_seg, dst, p, stream); break;
        case 4: e = launch_n<4, F16>(in, w_seg, dst, p, stream); break;
        case 5: e = launch_n<5, F16>(in, w_seg, dst, p, stream); break;
        case 6: e = launch_n<6, F16>(in, w_seg, dst, p, stream); break;
        case 7: e = launch_n<7, F16>(in, w_seg, dst, p, stream); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    if (p.splits > 1)
        e = launch_splitk_reduce((const float *)ws, out, p.out_elems, p.splits, stream, p.epi, (size_t)p.M * p.M, p.Cout);
    return e;
}

// f16: half-precision operands (else bfloat16).
hipError_t launch_igemm_bf16(const void *in_v, const void *w_seg_v, float *out, void *ws, const Shape &s, bool f16,
                             hipStream_t stream)
{
    if (igemm_bf16_wide_supported(s)) return launch_igemm_bf16_wide(in_v, w_seg_v, out, s, f16, stream);
    if (igemm_bf16_ring_supported(s)) return launch_igemm_bf16_ring(in_v, w_seg_v, out, s, f16, stream);
    if (igemm_bf16_strip_supported(s)) return launch_igemm_bf16_strip(in_v, w_seg_v, out, s, f16, stream);
    return f16 ? launch_plain<true>(in_v, w_seg_v, out, ws, s, stream) : launch_plain<false>(in_v, w_seg_v, out, ws, s, stream);
}

}  // namespace kst
