// Pieces shared by the fp32 and bf16 matrix-core kernels: the tile plan, the
// class-interleaving epilogue and the split-reduction pass.
#pragma once
#include "kst_internal.h"

#include <utility>

namespace kst {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

// One 32x32x16 MFMA on eight 16-bit values per lane and operand: bfloat16, or half precision
// (the operands travel through the kernels as bit patterns; only the multiply tells them apart).
template <bool F16>
__device__ __forceinline__ floatx16 mfma16(bf16x8 a, bf16x8 b, floatx16 c)
{
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a
// constant expression inside the body, so register arrays are only ever indexed by constants.
template <class F, int... I>
__device__ __forceinline__ void static_for_each(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_each(f, std::make_integer_sequence<int, N>{});
}


constexpr int G_TM = 128;        // positions per workgroup (4 MFMA column blocks)
constexpr int G_TCO = 128;       // output channels per workgroup (4 MFMA row blocks)
constexpr int G_THREADS = 512;   // 8 waves: 2 (channel halves) x 4 (position blocks)

struct IgemmParams {
    int B, Cin, Cout, N, M, E, EE;
    int Ns;                // row stride of the input in elements (>= N); with a frame supplied by the kernel
                           // (q > 0): row stride of the staged, framed rows in LDS
    int q, N0, pad;        // zero frame the kernel supplies; edge of the tensor in memory (N - 2q); LDS column
                           // of the framed map's column 0 (pad + q is a multiple of 4)
    int Mtot;              // B * E * E
    int tco;               // output channels per workgroup tile: G_TCO, or half of it in the fp32 pipelined kernels
    int tiles_m, tiles_co, splits;
    int ci_per_split;      // multiple of the kernel's channel step
    int lrows;             // input rows (stacked over batch items) held per channel
    unsigned off[4];       // element offset of W_p
    size_t out_elems;
    double est_s;          // the cost model's time for the launch chosen here (seconds)
    Epilogue epi;          // applied by the stores that write final values (not by those of partial sums)
    int crop;              // 1: quad members land one row and one column earlier (odd padding factor)
};

// kc: input channels staged per step; tco: output channels per workgroup tile.
inline IgemmParams igemm_plan(const Shape &s, kst_dtype dt, int kc, int tco = G_TCO)
{
    IgemmParams p;
    p.tco = tco;
    // M: edge of the planes that are written -- with Shape::crop the interior of the map only, whose
    // element (y, x) is the map's (y + 1, x + 1); positions and tiles are those of the whole map.
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.N = s.N; p.M = s.M - 2 * s.crop; p.E = s.E;
    p.crop = s.crop;
    p.q = s.frame;
    p.N0 = s.N - 2 * s.frame;
    p.pad = (4 - (s.frame & 3)) & 3;
    p.Ns = s.frame > 0 ? (p.pad + s.N + 3) & ~3 : s.Ns;
    p.EE = s.E * s.E;
    p.Mtot = s.B * p.EE;
    p.tiles_m = (p.Mtot + G_TM - 1) / G_TM;
    p.tiles_co = (s.Cout + tco - 1) / tco;
    // Rows of one channel that G_TM consecutive positions can touch: the quad rows
    // spanned, the rows skipped at each batch-item boundary, and the window halo.
    const int dg = (G_TM - 2) / s.E + 1;
    const int crossings = (dg + s.E - 1) / s.E;
    p.lrows = dg + crossings * (s.N - s.E) + s.fl + 1;
    // Split the channel reduction when the tile grid alone cannot fill the chip.
    const int tiles = p.tiles_m * p.tiles_co;
    const int chunks = (s.Cin + kc - 1) / kc;
    // Candidates: split counts up to 16.  Cost of one: launch rounds on 256 CUs times the time
    // of a tile's share of the reduction, plus the pass that sums the partial outputs (it reads
    // `splits` copies and writes one).  A split has to beat the unsplit launch by a tenth to be
    // worth its workspace.
    int splits = 1;
    double est;
    {
        const double tile_s = (double)G_TM * tco * s.Cin * s.n * s.n / (dt != KST_F32 ? 1.0e12 : 2.0e11);
        const double out_b = (double)s.B * s.Cout * p.M * p.M * 4.0;
        double best = (double)((tiles + 255) / 256) * tile_s;
        const double unsplit = best;
        // A layer with very few tiles (one sample of a small map) may split further, up to one
        // workgroup per CU: its reduction is a stream of weights that only many CUs can pull.
        const int c_max = tiles * 16 < 256 ? 256 / tiles : 16;
        for (int c = 2; c <= c_max && c <= chunks; ++c) {
            const double t = (double)(((size_t)tiles * c + 255) / 256) * tile_s / c + (c + 1) * out_b / 4.0e12;
            if (t < best && t < 0.9 * unsplit) { best = t; splits = c; }
        }
        est = best;
    }
    p.est_s = est;
    const int cps = (chunks + splits - 1) / splits;
    p.ci_per_split = cps * kc;
    p.splits = (chunks + cps - 1) / cps;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, dt);
    p.out_elems = (size_t)s.B * s.Cout * p.M * p.M;
    p.epi = s.epi;
    return p;
}

// Store 32 output channels of one wave's accumulators.  acc[cls] is the 32 x 32 block of class
// cls (rows: output channels co_base + 8(v/4) + 4kk + v%4; column: this lane's quad).  The
// s = 0 / s = 1 classes of a row parity sit side by side in memory.
// final: these are the element's final values (the epilogue applies), not partial sums.
__device__ __forceinline__ void igemm_store_block(float *__restrict__ o, const floatx16 &a0, const floatx16 &a1,
                                                  const floatx16 &a2, const floatx16 &a3, const IgemmParams &p,
                                                  int co_base, int kk, int mb, int mi, int mj, bool final = true)
{
    const bool x1_ok = 2 * mj + 1 < p.M;
    const bool epi = final && epi_on(p.epi);            // uniform
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int co = co_base + 8 * (v >> 2) + 4 * kk + (v & 3);
        if (co >= p.Cout) continue;
        const float bias = epi ? epi_bias(p.epi, co) : 0.0f;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            float v0 = r ? a2[v] : a0[v], v1 = r ? a3[v] : a1[v];
            if (epi) {
                v0 = epi_apply(v0, bias, p.epi.act);
                v1 = epi_apply(v1, bias, p.epi.act);
            }
            if (p.crop) {                               // uniform: members at (2 mi + r - 1, 2 mj + s - 1)
                const int yc = 2 * mi + r - 1, xc = 2 * mj - 1;
                if (yc < 0 || yc >= p.M) continue;
                float *qc = o + (((size_t)mb * p.Cout + co) * p.M + yc) * p.M + xc;
                if (xc >= 0 && xc < p.M) qc[0] = v0;
                if (xc + 1 < p.M) qc[1] = v1;
                continue;
            }
            const int y = 2 * mi + r;
            if (y >= p.M) continue;
            float *q = o + (((size_t)mb * p.Cout + co) * p.M + y) * p.M + 2 * mj;
            if (x1_ok) {
                if ((reinterpret_cast<uintptr_t>(q) & 7u) == 0) {
                    *reinterpret_cast<float2 *>(q) = make_float2(v0, v1);
                } else {
                    q[0] = v0;
                    q[1] = v1;
                }
            } else {
                q[0] = v0;
            }
        }
    }
}

// Store one wave's accumulators: acc[cls][h] covers output channels co_base + 32h .. + 31.
template <int H>
__device__ __forceinline__ void igemm_store(float *__restrict__ o, const floatx16 (&acc)[4][H], const IgemmParams &p,
                                            int co_base, int kk, int mb, int mi, int mj, bool final = true)
{
#pragma unroll
    for (int h = 0; h < H; ++h)
        igemm_store_block(o, acc[0][h], acc[1][h], acc[2][h], acc[3][h], p, co_base + h * 32, kk, mb, mi, mj, final);
}

// out[e] = sum over splits of ws[split][e], in split order (deterministic), then the epilogue if
// one is active (element e belongs to output channel (e / plane_elems) % Cout).
hipError_t launch_splitk_reduce(const float *ws, float *out, size_t elems, int splits, hipStream_t stream,
                                Epilogue epi = {nullptr, KST_ACT_NONE}, size_t plane_elems = 1, int Cout = 1);

}  // namespace kst
