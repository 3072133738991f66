// Matrix-core segregated forward pass for fp32 layers with very few positions: one sample (or a
// few) of a small map -- the way Table 3 times the generator layers -- where a layer is a stream
// of weights over 16 or 64 quad positions (Section 3.3, Eqs. 7-10 as four implicit GEMMs).
//
// The kernel for ordinary layers multiplies tiles of 128 positions: with 16 positions seven
// eighths of its matrix-core work and of its partial sums are padding.  Here the position block
// is the 16 columns of v_mfma_f32_16x16x4f32, so nothing is padded beyond the last block:
//   * a wave owns 16 positions x 64 output channels (four MFMA row blocks) x the four parity
//     classes: 64 accumulator registers; a workgroup is one such wave, or four that share out
//     the workgroup's part of a long reduction and add their sums through LDS before storing;
//   * the reduction over input channels is cut into `splits` ranges, one workgroup each, so that
//     the layer's weights -- each read exactly once, straight from memory into the A operands, 16
//     bytes per lane and 256 consecutive bytes per 16 lanes: a lane's four values are its row of
//     the four row blocks, so row i of block j is output channel 4 i + j of the wave's 64 -- are
//     pulled by a few waves on every SIMD of the chip; the partial outputs are added by the
//     strided-share pass (fixed order: reproducible);
//   * the B operand is the lane's own position and channel: its (fl+1) x (fl+1) window is loaded
//     from the input tensor as it lies in memory, the zero frame of a padded layer by predicate
//     (no framed copy), once per chunk of four channels for all taps;
//   * the loads of chunk c + 1 are issued before the MFMAs of chunk c.
#include "kst_igemm_common.h"

namespace kst {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int SM_TCO = 64;            // output channels per wave: four row blocks of 16
constexpr int SM_POS = 16;            // positions per wave: the MFMA's columns
constexpr int SM_KC = 4;              // input channels per MFMA

struct SmallParams {
    int B, Cin, Cout, N0, q, E, EE, Mtot;
    int M, crop;                      // edge of the planes that are written; 1: quad members land one row / column earlier
    int pos_blocks, co_blocks, splits, chunks_per_split, chunks;
    int waves;                        // waves per workgroup (1 or 4): a workgroup's range of chunks is shared out among them
    unsigned off[4];                  // element offset of W_p in the segregated weights
    size_t out_elems;
    Epilogue epi;
};

// V4: Cout is a multiple of 4 and the weights are read as 16-byte groups; otherwise (the 128 -> 3
// output layer of a generator) one value at a time, rows past Cout reading the last channel again.
// WV: waves per workgroup.  With four, each takes a quarter of the workgroup's chunks and their sums are
// added through LDS in wave order before anything is stored: a quarter of the partial outputs for
// the same number of waves pulling weights (one sample of a 1024 -> 512 layer writes 16.7 MB of
// partial outputs beside its 33.5 MB of weights with one wave per workgroup).
template <int n, bool V4, int WV>
__global__ void __launch_bounds__(64 * WV) igemm_f32_small_kernel(const float *__restrict__ in, const float *__restrict__ w_seg,
                                                               float *__restrict__ dst, SmallParams p)
{
    constexpr int fl = n / 2;
    constexpr int NN = n * n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, k = lane >> 4;          // column / row-in-block of the operands; channel of the chunk
    unsigned id = blockIdx.x;
    const int co_block = (int)(id % (unsigned)p.co_blocks);
    id /= (unsigned)p.co_blocks;
    const int pos_block = (int)(id % (unsigned)p.pos_blocks);
    const int split = (int)(id / (unsigned)p.pos_blocks);
    const int co0 = co_block * SM_TCO;

    // This lane's position (B operand column m): batch item and quad, clamped past the end.
    int pos = pos_block * SM_POS + m;
    const bool pos_valid = pos < p.Mtot;
    if (!pos_valid) pos = p.Mtot - 1;
    const int mb = pos / p.EE;
    const int prem = pos - mb * p.EE;
    const int mi = prem / p.E, mj = prem - mi * p.E;

    // Window of the position in the tensor as it lies in memory: rows mi - q .. mi - q + fl, the
    // same for columns; cells outside the tensor belong to the zero frame.
    unsigned x_off[fl + 1][fl + 1];
    bool x_ok[fl + 1][fl + 1];
#pragma unroll
    for (int dy = 0; dy <= fl; ++dy)
#pragma unroll
        for (int dx = 0; dx <= fl; ++dx) {
            const int y = mi + dy - p.q, x = mj + dx - p.q;
            x_ok[dy][dx] = y >= 0 && y < p.N0 && x >= 0 && x < p.N0;
            x_off[dy][dx] = x_ok[dy][dx] ? (((unsigned)mb * p.Cin + k) * p.N0 + y) * p.N0 + x : 0u;
        }
    const unsigned x_step = (unsigned)SM_KC * p.N0 * p.N0;

    // A operands: lane (m, k) loads the weights of output channels co0 + 4 m .. + 3, input channel
    // ci0 + k, as one 16-byte group; value j is its row (m) of row block j.  Groups past Cout (the
    // last block of a ragged layer; Cout is a multiple of 4) read the last group again: their
    // accumulator rows are never stored.
    const unsigned w_col = V4 ? (unsigned)min(co0 + 4 * m, p.Cout - 4) : 0u;
    unsigned w_cols[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w_cols[j] = (unsigned)min(co0 + 4 * m + j, p.Cout - 1);

    const int wg_begin = split * p.chunks_per_split;
    const int wg_end = min(p.chunks, wg_begin + p.chunks_per_split);
    const int per_wave = (wg_end - wg_begin + WV - 1) / WV;
    const int c_begin = wg_begin + wave * per_wave;
    const int c_end = min(wg_end, c_begin + per_wave);

    floatx4 acc[4][4];                               // [class][row block]
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) acc[c][blk] = floatx4{0.f, 0.f, 0.f, 0.f};

    float xf[2][fl + 1][fl + 1];
    float4 wf[2][NN];
    auto fetch = [&](auto bufc, int chunk) {
        constexpr int buf = decltype(bufc)::value;
        const unsigned ci = (unsigned)(chunk * SM_KC + k);
#pragma unroll
        for (int dy = 0; dy <= fl; ++dy)
#pragma unroll
            for (int dx = 0; dx <= fl; ++dx) {
                const float v = in[x_off[dy][dx] + (unsigned)chunk * x_step];   // (frame cells read element 0 of the channel block: valid, unused)
                xf[buf][dy][dx] = x_ok[dy][dx] ? v : 0.0f;
            }
#pragma unroll
        for (int T = 0; T < NN; ++T) {
            constexpr int dummy = 0;
            (void)dummy;
            const int cls = tap_class(n, T);
            const unsigned Tp = (unsigned)class_taps(n, cls);
            const unsigned t = (unsigned)(T - class_tap_base(n, cls));
            const unsigned row = p.off[cls] + (ci * Tp + t) * (unsigned)p.Cout;
            if constexpr (V4)
                wf[buf][T] = *reinterpret_cast<const float4 *>(w_seg + row + w_col);     // 16-byte aligned: offsets are multiples of 4
            else
                wf[buf][T] = make_float4(w_seg[row + w_cols[0]], w_seg[row + w_cols[1]], w_seg[row + w_cols[2]],
                                         w_seg[row + w_cols[3]]);
        }
    };
    auto multiply = [&](auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        static_for<NN>([&](auto Tc) {
            constexpr int T = decltype(Tc)::value;
            constexpr int cls = tap_class(n, T);
            constexpr int r = cls >> 1, sp = cls & 1;
            constexpr int local = T - class_tap_base(n, cls);
            constexpr int Tb = taps_for_parity(n, sp);
            constexpr int a = local / Tb, bq = local - a * Tb;
            const float x = xf[buf][r + a][sp + bq];
            acc[cls][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[buf][T].x, x, acc[cls][0], 0, 0, 0);
            acc[cls][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[buf][T].y, x, acc[cls][1], 0, 0, 0);
            acc[cls][2] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[buf][T].z, x, acc[cls][2], 0, 0, 0);
            acc[cls][3] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[buf][T].w, x, acc[cls][3], 0, 0, 0);
        });
    };

    if (c_begin < c_end) {
        fetch(std::integral_constant<int, 0>{}, c_begin);
        int c = c_begin;
        while (true) {
            if (c + 1 < c_end) fetch(std::integral_constant<int, 1>{}, c + 1);
            multiply(std::integral_constant<int, 0>{});
            if (++c >= c_end) break;
            if (c + 1 < c_end) fetch(std::integral_constant<int, 0>{}, c + 1);
            multiply(std::integral_constant<int, 1>{});
            if (++c >= c_end) break;
        }
    }

    // D layout: lane (m, k) holds rows 4 k + v (v = 0..3) of column m; row i of block blk is output
    // channel co0 + 4 i + blk, at this lane's position.  Stored from there a lane's 64 values
    // would go to 64 different planes, 64 scattered 4-byte writes per instruction (measured: most of
    // the kernel's time).  They go through an LDS image [channel][position][class] instead, and
    // leave one channel per instruction with the lanes running along the output rows: lane
    // (r, position, s) writes member (r, s) of its quad, so neighbouring lanes write neighbouring
    // columns.
    __shared__ float buf[(WV > 1 ? (WV - 1) * 64 : 64) * 64];    // the other waves' sums [wave - 1][register][lane]; then the image (64 x 64 floats)
    float *img = buf;                                            // [SM_TCO][SM_POS][4]
    if constexpr (WV > 1) {
        if (wave > 0) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int blk = 0; blk < 4; ++blk)
#pragma unroll
                    for (int v = 0; v < 4; ++v) buf[((wave - 1) * 64 + (c * 4 + blk) * 4 + v) * 64 + lane] = acc[c][blk][v];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int w = 1; w < WV; ++w)
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[c][blk][v] += buf[((w - 1) * 64 + (c * 4 + blk) * 4 + v) * 64 + lane];
        }
        __syncthreads();                                         // every lane of wave 0 has read the sums: the image may overwrite them
    }
    if (wave == 0) {
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int col = 4 * (4 * k + v) + blk;           // channel of the workgroup's 64
                *reinterpret_cast<float4 *>(&img[(col * SM_POS + m) * 4]) =
                    make_float4(acc[0][blk][v], acc[1][blk][v], acc[2][blk][v], acc[3][blk][v]);
            }
    }
    __syncthreads();
    const int r2 = lane >> 5, m2 = (lane >> 1) & 15, s2 = lane & 1;
    const int pos2 = pos_block * SM_POS + m2;
    if (pos2 >= p.Mtot) return;
    const int mb2 = pos2 / p.EE;
    const int prem2 = pos2 - mb2 * p.EE;
    const int mi2 = prem2 / p.E, mj2 = prem2 - mi2 * p.E;
    const int y = 2 * mi2 + r2 - p.crop, x = 2 * mj2 + s2 - p.crop;
    if (y < 0 || y >= p.M || x < 0 || x >= p.M) return;
    const bool final = p.splits == 1;
    const bool epi = final && epi_on(p.epi);
    float *o = dst + (size_t)split * p.out_elems + ((size_t)mb2 * p.Cout + co0) * p.M * p.M + (size_t)y * p.M + x;
    const size_t plane = (size_t)p.M * p.M;
    const int ncol = min(SM_TCO, p.Cout - co0);
    for (int col = wave; col < ncol; col += WV) {                // the waves share out the channels
        float val = img[(col * SM_POS + m2) * 4 + 2 * r2 + s2];
        if (epi) val = epi_apply(val, epi_bias(p.epi, co0 + col), p.epi.act);
        o[(size_t)col * plane] = val;
    }
}

bool small_plan(const Shape &s, SmallParams &p)
{
    if (s.n < 1 || s.n > 5 || s.Ns != s.N) return false;
    if (s.Cin % SM_KC != 0 || s.Cin < 64) return false;
    const long long Mtot = (long long)s.B * s.E * s.E;
    // Every block of 16 positions streams the layer's weights once (through L2): worth it while the
    // positions are few, or the weights small.  Beyond that the tiles of 128 positions x 128 (or 64)
    // channels, which stage a weight once for all their positions, are the better kernel
    // (measured on one sample of Table 3's generators: no layer loses with a limit of 128 MB of
    // weight reads, and the widest maps gain: 64 x 64 channels on 128 x 128 positions 52.8 -> 40.8 us,
    // 128 x 64 channels on 64 x 64 positions 37.8 -> 34.3 us).
    const double w_bytes = (double)s.Cin * s.Cout * s.n * s.n * 4.0;
    const double budget = 128.0e6;
    if (Mtot > (1 << 20) || (Mtot > 256 && (double)((Mtot + 15) / 16) * w_bytes > budget)) return false;
    // Fewer than 16 output channels leave most of a 64-row block empty: only where the padded
    // multiply-adds are still next to nothing for the chip (about 5 us of matrix-core work).
    if (s.Cout < 16 && (double)((Mtot + 15) / 16) * 16.0 * 64.0 * s.Cin * s.n * s.n > 4.0e8) return false;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout;
    p.q = s.frame;
    p.N0 = s.N - 2 * s.frame;
    if (p.N0 < 1) return false;
    p.E = s.E; p.EE = s.E * s.E; p.Mtot = (int)Mtot;
    p.crop = s.crop;
    p.M = s.M - 2 * s.crop;
    if (p.M < 1) return false;
    p.pos_blocks = (p.Mtot + SM_POS - 1) / SM_POS;
    p.co_blocks = (s.Cout + SM_TCO - 1) / SM_TCO;
    p.chunks = s.Cin / SM_KC;
    // About two waves per SIMD over the chip, but at least four chunks per workgroup (so that the
    // partial outputs stay well below the weights in bytes); with a long reduction (64 chunks and
    // more) four waves per workgroup, two chunks each at least -- except where a single position
    // block would then leave the weights to fewer than 512 workgroups (measured on one sample of
    // Table 3's layers: 512 -> 256 on 4 x 4 positions 13.1 us with one wave, 15.3 with four;
    // 1024 -> 512: 20.2 and 21.0; 2048 -> 1024: 46.4 and 42.1; with 64 and 256 positions four waves
    // win throughout, 19.9 -> 16.1, 24.6 -> 14.3, 37.8 -> 31.2 us).
    p.waves = p.chunks >= 64 && (p.pos_blocks > 1 || p.co_blocks * (p.chunks / 8) >= 512) ? 4 : 1;
    const int wgs = 2048 / p.waves;
    const int want = (wgs + p.pos_blocks * p.co_blocks - 1) / (p.pos_blocks * p.co_blocks);
    const int most = p.chunks / (2 * p.waves);
    int splits = most < want ? most : want;
    if (splits < 1) splits = 1;
    p.chunks_per_split = (p.chunks + splits - 1) / splits;
    p.splits = (p.chunks + p.chunks_per_split - 1) / p.chunks_per_split;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, KST_F32);
    p.out_elems = (size_t)s.B * s.Cout * p.M * p.M;
    p.epi = s.epi;
    return (size_t)p.pos_blocks * p.co_blocks * p.splits < 0x7fffffffu;
}

template <int n>
hipError_t launch_small_n(const float *in, const float *w_seg, float *dst, const SmallParams &p, hipStream_t stream)
{
    const unsigned blocks = (unsigned)(p.pos_blocks * p.co_blocks * p.splits);
    const bool v4 = (p.Cout & 3) == 0;
    if (p.waves == 4) {
        if (v4)
            hipLaunchKernelGGL((igemm_f32_small_kernel<n, true, 4>), dim3(blocks), dim3(256), 0, stream, in, w_seg, dst, p);
        else
            hipLaunchKernelGGL((igemm_f32_small_kernel<n, false, 4>), dim3(blocks), dim3(256), 0, stream, in, w_seg, dst, p);
    } else {
        if (v4)
            hipLaunchKernelGGL((igemm_f32_small_kernel<n, true, 1>), dim3(blocks), dim3(64), 0, stream, in, w_seg, dst, p);
        else
            hipLaunchKernelGGL((igemm_f32_small_kernel<n, false, 1>), dim3(blocks), dim3(64), 0, stream, in, w_seg, dst, p);
    }
    return hipGetLastError();
}

}  // namespace

bool igemm_f32_small_supported(const Shape &s)
{
    SmallParams p;
    return small_plan(s, p);
}

size_t igemm_f32_small_workspace_bytes(const Shape &s)
{
    SmallParams p;
    if (!small_plan(s, p)) return 0;
    return p.splits > 1 ? (size_t)p.splits * p.out_elems * sizeof(float) : 0;
}

hipError_t launch_igemm_f32_small(const float *in, const float *w_seg, float *out, void *ws, const Shape &s,
                                  hipStream_t stream)
{
    SmallParams p;
    if (!small_plan(s, p)) return hipErrorInvalidValue;
    float *dst = p.splits > 1 ? (float *)ws : out;
    hipError_t e;
    switch (s.n) {
        case 1: e = launch_small_n<1>(in, w_seg, dst, p, stream); break;
        case 2: e = launch_small_n<2>(in, w_seg, dst, p, stream); break;
        case 3: e = launch_small_n<3>(in, w_seg, dst, p, stream); break;
        case 4: e = launch_small_n<4>(in, w_seg, dst, p, stream); break;
        case 5: e = launch_small_n<5>(in, w_seg, dst, p, stream); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    if (p.splits > 1)
        e = launch_splitk_reduce((const float *)ws, out, p.out_elems, p.splits, stream, p.epi, (size_t)p.M * p.M, p.Cout);
    return e;
}

}  // namespace kst
