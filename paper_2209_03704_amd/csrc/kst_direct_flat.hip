// Single-channel, bandwidth-bound segregated forward pass (Section 3.3, Eqs. 7-10):
// the kernel that the roofline of the headline layer is measured on.
//
// What decides the speed here is the shape of the stores, not the arithmetic
// (2.5 flop per byte).  On this chip a wave's 1 KB store reaches full write
// bandwidth only if every four lanes fall into one 64-byte segment; with an
// odd M no per-row lane assignment can guarantee that.  So the output tensor
// is treated as one flat array: a workgroup owns an aligned block of CH
// floats, a lane owns the 16-byte aligned group of four consecutive floats
// f0 = 4q .. 4q+3, whatever rows they fall in.
//
// Arithmetic for a group: within output row y the group starting at column x0
// has row parity r = y & 1 and column parities par, 1-par, par, 1-par with
// par = x0 & 1, so it is two quad halves of Eqs. 7-10: Ta(r) input rows by
// fl + 2 input columns feed all four outputs, with the sub-kernels K1..K4
// held in scalar registers.  (r, par) is uniform over a wave except in the
// wave that contains a row end, which runs two variants under its lane mask.
// A group that straddles a row end is computed twice, once as the tail of row
// y and once as the head of row y + 1 (x0 - M < 0), and the two halves are
// merged before its single aligned store.  Elements outside the block's part
// of the plane (plane ends are not 16-byte aligned) are masked out and
// written by scalar stores.
//
// The kernel is persistent and software-pipelined: while a workgroup computes
// and stores one piece from one LDS buffer, the 16-byte loads of the next
// piece's input rows are in flight into registers; they are written to the
// other buffer afterwards, one barrier per piece.  Without this all
// workgroups of a launch load, compute and store in lock-step and the read
// and write phases of the whole chip add up instead of overlapping.
//
// Measured on this chip the kernel is bound by instruction issue (about one
// instruction per SIMD every four cycles, scalar ones included), so all
// bookkeeping is incremental: block, row and column positions advance by
// host-computed steps with carries instead of divisions, and a wave whose 256
// floats lie in one row, or cross exactly one row end, runs code specialised
// by scalar (r, par) with LDS addresses of the form scalar base + 2 * lane.
#include "kst_direct_flat.h"

namespace kst {

namespace {

// 16-byte aligned streaming store of four outputs.
__device__ __forceinline__ void store_streaming(float *dst, const float (&o)[4]) { store_streaming4(dst, o[0], o[1], o[2], o[3]); }
// on: whether an epilogue is active (uniform over the workgroup).
__device__ __forceinline__ void flat_epilogue(float (&o)[4], bool on, float bias, int act)
{
    if (on) epi_apply4(o[0], o[1], o[2], o[3], bias, act);
}

constexpr int F_PAD = 4;      // slack floats left and right of each staged input row
constexpr int F_THREADS = 512;
constexpr int F_NPRE = 1024 / F_THREADS;      // float4 loads in flight per lane (1024 per piece at most)
constexpr int F_STEP = 4 * F_THREADS;         // floats the workgroup covers per iteration
constexpr int F_STEP_LOG2 = F_THREADS == 512 ? 11 : 10;
static_assert(F_THREADS == 256 || F_THREADS == 512, "two or four float4 per lane");

// Flat output indices fit 32 bits: the ABI keeps every tensor below 2^31 elements.
struct Piece {
    unsigned j;               // block the piece belongs to
    unsigned fa, fb;          // flat output range of this piece, inside one plane
    unsigned p0;              // flat index of the plane's first element
    int plane;
    int ya, xa;               // row / column of fa inside the plane
    int yb;                   // last output row touched
    int ia;                   // first input row staged
    int rows_in;              // input rows staged
    int full;                 // covers its whole block: fa = j*CH, fb = fa + CH
    const float *src;         // in + first staged row
};

// Position (plane, row, column) of the first float of block j.
struct BlockPos {
    unsigned j;
    int plane, y, x;
};

__device__ __forceinline__ void finish_piece(const FlatParams &p, const float *__restrict__ in, Piece &pc)
{
    const unsigned block_end = min((pc.j + 1) * p.CH, p.total);
    pc.p0 = pc.fa - (unsigned)(pc.ya * p.M + pc.xa);
    pc.fb = min(block_end, pc.p0 + p.MM);
    pc.full = pc.fa == pc.j * p.CH && pc.fb - pc.fa == p.CH;
    if (pc.full) {
        pc.yb = pc.ya + p.c_y + (pc.xa + p.c_x >= p.M ? 1 : 0);
    } else {
        pc.yb = (int)((pc.fb - 1 - pc.p0) / (unsigned)p.M);          // rare: blocks at a plane end
    }
    pc.ia = pc.ya >> 1;
    const int ib = min(p.N - 1, (pc.yb >> 1) + p.fl);
    pc.rows_in = ib - pc.ia + 1;
    // Cin == 1: plane -> batch item.  32-bit offsets: the input has fewer than 2^31 elements.
    const unsigned b = p.Cout == 1 ? (unsigned)pc.plane : (unsigned)pc.plane / (unsigned)p.Cout;
    pc.src = in + (b * (unsigned)p.N + (unsigned)pc.ia) * (unsigned)p.N;
}

__device__ __forceinline__ void first_piece(const FlatParams &p, const float *__restrict__ in, const BlockPos &bp, Piece &pc)
{
    pc.j = bp.j;
    pc.fa = bp.j * p.CH;
    pc.plane = bp.plane;
    pc.ya = bp.y;
    pc.xa = bp.x;
    finish_piece(p, in, pc);
}

// One aligned group in output row parity r whose first column has parity par.
template <int n, int r, int par>
__device__ __forceinline__ void flat_group(float (&o)[4], const float *__restrict__ rowp, int xs_stride, int cbase,
                                           const float (&wk)[2][2][((n + 1) / 2) * ((n + 1) / 2)])
{
    constexpr int fl = n / 2;
    constexpr int Ta = r ? n / 2 : (n + 1) / 2;
    constexpr int Tb0 = (n + 1) / 2, Tb1 = n / 2;
    float win[Ta > 0 ? Ta : 1][fl + 2];
#pragma unroll
    for (int a = 0; a < Ta; ++a)
#pragma unroll
        for (int c = 0; c < fl + 2; ++c) win[a][c] = rowp[a * xs_stride + cbase + c];
    constexpr int s_k[4] = {par, 1 - par, par, 1 - par};       // column parity of output k
    constexpr int c_k[4] = {0, par ? 0 : 1, 1, par ? 1 : 2};  // window column where its taps start
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int Tb = s_k[k] ? Tb1 : Tb0;
        float acc = 0.0f;
#pragma unroll
        for (int a = 0; a < Ta; ++a)
#pragma unroll
            for (int bq = 0; bq < Tb; ++bq) acc = fmaf(win[a][c_k[k] + bq], wk[r][s_k[k]][a * Tb + bq], acc);
        o[k] = acc;
    }
}

// Outputs of the group at (row y, first column x0), x0 in [-3, M).
template <int n>
__device__ __forceinline__ void flat_row_group(float (&o)[4], const float *__restrict__ Xs, const FlatParams &p, int ia,
                                               int y, int x0,
                                               const float (&wk)[2][2][((n + 1) / 2) * ((n + 1) / 2)])
{
    const int r = y & 1;
    const float *rowp = Xs + ((y >> 1) - ia + r) * p.xs_stride + F_PAD;
    if (x0 & 1) {
        const int cbase = ((x0 - 1) >> 1) + 1;
        if (r) flat_group<n, 1, 1>(o, rowp, p.xs_stride, cbase, wk);
        else flat_group<n, 0, 1>(o, rowp, p.xs_stride, cbase, wk);
    } else {
        const int cbase = x0 >> 1;
        if (r) flat_group<n, 1, 0>(o, rowp, p.xs_stride, cbase, wk);
        else flat_group<n, 0, 0>(o, rowp, p.xs_stride, cbase, wk);
    }
}

// Segment = the 256 consecutive floats one wave covers in one iteration; it starts at
// (row y, column xs) and crosses exactly one row end.  Lanes left of the row end compute
// their group in row y, lanes right of it in row y + 1, the lane on it both.
template <int n>
__device__ __forceinline__ void cross_segment(float (&o)[4], const float *__restrict__ Xs, const FlatParams &p, int ia,
                                              int y, int xs, int lane,
                                              const float (&wk)[2][2][((n + 1) / 2) * ((n + 1) / 2)])
{
    const int x0 = xs + 4 * lane;
    float oa[4] = {0.f, 0.f, 0.f, 0.f}, ob[4] = {0.f, 0.f, 0.f, 0.f};
    if (x0 < p.M) {
        const int r = y & 1;
        const float *rowp = Xs + ((y >> 1) - ia + r) * p.xs_stride + F_PAD + 2 * lane;
        if (xs & 1) {
            const int cbase = ((xs - 1) >> 1) + 1;
            if (r) flat_group<n, 1, 1>(oa, rowp, p.xs_stride, cbase, wk);
            else flat_group<n, 0, 1>(oa, rowp, p.xs_stride, cbase, wk);
        } else {
            const int cbase = xs >> 1;
            if (r) flat_group<n, 1, 0>(oa, rowp, p.xs_stride, cbase, wk);
            else flat_group<n, 0, 0>(oa, rowp, p.xs_stride, cbase, wk);
        }
    }
    if (x0 + 3 >= p.M) {
        const int y1 = y + 1, xs1 = xs - p.M;                        // negative column: head of the next row
        const int r = y1 & 1;
        const float *rowp = Xs + ((y1 >> 1) - ia + r) * p.xs_stride + F_PAD + 2 * lane;
        if (xs1 & 1) {
            const int cbase = ((xs1 - 1) >> 1) + 1;
            if (r) flat_group<n, 1, 1>(ob, rowp, p.xs_stride, cbase, wk);
            else flat_group<n, 0, 1>(ob, rowp, p.xs_stride, cbase, wk);
        } else {
            const int cbase = xs1 >> 1;
            if (r) flat_group<n, 1, 0>(ob, rowp, p.xs_stride, cbase, wk);
            else flat_group<n, 0, 0>(ob, rowp, p.xs_stride, cbase, wk);
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) o[k] = x0 + k < p.M ? oa[k] : ob[k];
}

template <int n>
__global__ void __launch_bounds__(F_THREADS) direct_flat_kernel(const float *__restrict__ in,
                                                                  const float *__restrict__ w_seg,
                                                                  float *__restrict__ out, FlatParams p)
{
    constexpr int Ta0 = (n + 1) / 2, Ta1 = n / 2;
    extern __shared__ __attribute__((aligned(16))) float lds[];   // 2 x [max_rows][xs_stride]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n4 = p.N >> 2;

    // This workgroup's blocks: blockIdx.x, + gridDim.x, ...  The position of the first one costs
    // the only divisions of the common path; later ones are reached by adding the grid step.
    // Workgroups are dealt round-robin to the 8 XCDs: runs of `run` consecutive blocks go to the
    // same XCD, so that neighbouring blocks find their shared input rows in that XCD's L2, while
    // the chip as a whole still sweeps the tensor front to back.  (The grid is a multiple of
    // 8 * run, which keeps a workgroup's stride at gridDim.x blocks.)
    BlockPos bp;
    bp.j = blockIdx.x;
    if (p.run > 1) {
        const unsigned xcd = blockIdx.x & 7u, w = blockIdx.x >> 3;
        bp.j = ((w / p.run) * 8u + xcd) * p.run + (w % p.run);
    }
    if (bp.j >= p.nblocks) return;
    {
        const unsigned f = bp.j * p.CH;
        const unsigned plane = f / p.MM;
        const unsigned rel = f - plane * p.MM;
        bp.plane = (int)plane;
        bp.y = (int)(rel / (unsigned)p.M);
        bp.x = (int)(rel - (unsigned)bp.y * (unsigned)p.M);
    }
    // Row / column offset of this wave's 256 floats inside an iteration.
    const int w_y = (wave * 256) / p.M, w_x = wave * 256 - w_y * p.M;

    // Where float4 number k * threads + tid of a staged run lands in an LDS buffer (same for every piece).
    int lds_off[F_NPRE];
#pragma unroll
    for (int k = 0; k < F_NPRE; ++k) {
        const int e = k * F_THREADS + tid;
        const int rr = e / n4, x4 = e - rr * n4;
        lds_off[k] = rr * p.xs_stride + F_PAD + 4 * x4;
    }

    Piece pc;
    first_piece(p, in, bp, pc);
    // First piece: plain staging (all loads issued before the first LDS write).
    {
        const float4 *s4 = reinterpret_cast<const float4 *>(pc.src);
        const int count4 = pc.rows_in * n4;
        const float4 t0 = s4[min(tid, count4 - 1)];
        const float4 t1 = s4[min(F_THREADS + tid, count4 - 1)];
        const float4 t2 = F_NPRE > 2 ? s4[min(2 * F_THREADS + tid, count4 - 1)] : t0;
        const float4 t3 = F_NPRE > 2 ? s4[min(3 * F_THREADS + tid, count4 - 1)] : t0;
        const float4 t[4] = {t0, t1, t2, t3};
#pragma unroll
        for (int k = 0; k < F_NPRE; ++k)
            if (k * F_THREADS + tid < count4) *reinterpret_cast<float4 *>(lds + lds_off[k]) = t[k];
    }
    __syncthreads();

    float wk[2][2][Ta0 * Ta0];
    int cur_co = -1;
    const bool epi = epi_on(p.epi);
    float bias = 0.0f;
    int buf = 0;
    while (true) {
        // ---- the next piece and its loads --------------------------------------------------------
        // (After the last piece the loads below simply fetch this piece's rows again: valid, unused.)
        Piece pn = pc;
        bool more = true;
        if (pc.fb < min((pc.j + 1) * p.CH, p.total)) {           // the plane ended inside the block
            pn.fa = pc.fb;
            pn.plane = pc.plane + 1;
            pn.ya = 0;
            pn.xa = 0;
            finish_piece(p, in, pn);
        } else {
            bp.j += gridDim.x;
            bp.plane += p.g_plane;
            bp.y += p.g_y;
            bp.x += p.g_x;
            if (bp.x >= p.M) { bp.x -= p.M; ++bp.y; }
            if (bp.y >= p.M) { bp.y -= p.M; ++bp.plane; }
            if (bp.j < p.nblocks) first_piece(p, in, bp, pn);
            else more = false;
        }
        const int count4n = pn.rows_in * n4;
        const float4 *s4 = reinterpret_cast<const float4 *>(pn.src);
        const float4 pre0 = s4[min(tid, count4n - 1)];
        const float4 pre1 = s4[min(F_THREADS + tid, count4n - 1)];
        const float4 pre2 = F_NPRE > 2 ? s4[min(2 * F_THREADS + tid, count4n - 1)] : pre0;
        const float4 pre3 = F_NPRE > 2 ? s4[min(3 * F_THREADS + tid, count4n - 1)] : pre0;

        // ---- weights of this plane's output channel (scalar registers) ----------------------
        const int co = p.Cout == 1 ? 0 : (int)((unsigned)pc.plane % (unsigned)p.Cout);
        if (co != cur_co) {
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int Ta = r ? Ta1 : Ta0, Tb = s ? Ta1 : Ta0;
#pragma unroll
                    for (int t = 0; t < Ta * Tb; ++t)
                        wk[r][s][t] = w_seg[p.off[2 * r + s] + (unsigned)(t * p.Cout + co)];   // Cin == 1
                }
            if (epi) bias = epi_bias(p.epi, co);
            cur_co = co;
        }

        // ---- compute and store this piece -------------------------------------------------------
        const float *Xs = lds + buf * p.xs_buf;
        if (pc.full && p.fast) {
            // Every wave segment lies inside the piece and the plane.  (y, xs): row and column of
            // the wave's first float, advanced by one workgroup iteration at a time.
            int y = pc.ya + w_y, xs = pc.xa + w_x;
            if (xs >= p.M) { xs -= p.M; ++y; }
            unsigned fw = pc.fa + 256u * (unsigned)wave;
#pragma unroll 1
            for (int it = 0; it < (int)(p.CH / F_STEP); ++it) {
                float o[4];
                if (xs + 255 < p.M) {
                    const int r = y & 1;
                    const float *rowp = Xs + ((y >> 1) - pc.ia + r) * p.xs_stride + F_PAD + 2 * lane;
                    if (xs & 1) {
                        const int cbase = ((xs - 1) >> 1) + 1;
                        if (r) flat_group<n, 1, 1>(o, rowp, p.xs_stride, cbase, wk);
                        else flat_group<n, 0, 1>(o, rowp, p.xs_stride, cbase, wk);
                    } else {
                        const int cbase = xs >> 1;
                        if (r) flat_group<n, 1, 0>(o, rowp, p.xs_stride, cbase, wk);
                        else flat_group<n, 0, 0>(o, rowp, p.xs_stride, cbase, wk);
                    }
                } else {
                    cross_segment<n>(o, Xs, p, pc.ia, y, xs, lane, wk);
                }
                flat_epilogue(o, epi, bias, p.epi.act);
                store_streaming(out + fw + 4 * lane, o);
                fw += F_STEP;
                xs += p.s_x;
                y += p.s_y;
                if (xs >= p.M) { xs -= p.M; ++y; }
            }
        } else {
            // General path: pieces cut by a plane end, and maps narrower than a wave segment.
            const unsigned block_start = pc.j * p.CH;
            const int it0 = (int)((pc.fa - block_start) >> F_STEP_LOG2);
            const int it1 = (int)((pc.fb - 1 - block_start) >> F_STEP_LOG2);
            unsigned f0 = block_start + ((unsigned)it0 << F_STEP_LOG2) + 4 * tid;
            int y, x0;                                           // floor-division form, y may start negative
            {
                const int K = p.s_y + 1;                         // K * M > F_STEP > distance to the plane start
                const unsigned relp = (unsigned)((int)(f0 - pc.p0) + K * p.M);
                const unsigned q = relp / (unsigned)p.M;
                y = (int)q - K;
                x0 = (int)(relp - q * (unsigned)p.M);
            }
            for (int it = it0; it <= it1; ++it) {
                if (f0 + 3 >= pc.fa && f0 < pc.fb) {
                    // A group hanging over the start of the plane is the head of row 0 (negative column).
                    const int yy = y < 0 ? 0 : y, xx = y < 0 ? x0 - p.M : x0;
                    float o[4];
                    flat_row_group<n>(o, Xs, p, pc.ia, yy, xx, wk);
                    if (xx + 3 >= p.M && yy + 1 <= pc.yb) {      // straddles a row end: head of the next row
                        float o2[4];
                        flat_row_group<n>(o2, Xs, p, pc.ia, yy + 1, xx - p.M, wk);
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (xx + k >= p.M) o[k] = o2[k];
                    }
                    float *dst = out + f0;                       // 16-byte aligned
                    flat_epilogue(o, epi, bias, p.epi.act);
                    if (f0 >= pc.fa && f0 + 3 < pc.fb) {
                        store_streaming(dst, o);
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (f0 + k >= pc.fa && f0 + k < pc.fb) dst[k] = o[k];
                    }
                }
                f0 += F_STEP;
                x0 += p.s_x;
                y += p.s_y;
                if (x0 >= p.M) { x0 -= p.M; ++y; }
            }
        }
        if (!more) break;

        // ---- land the prefetched rows in the other buffer -----------------------------------
        float *Xn = lds + (buf ^ 1) * p.xs_buf;
        const float4 pre[4] = {pre0, pre1, pre2, pre3};
#pragma unroll
        for (int k = 0; k < F_NPRE; ++k)
            if (k * F_THREADS + tid < count4n) *reinterpret_cast<float4 *>(Xn + lds_off[k]) = pre[k];
        __syncthreads();
        pc = pn;
        buf ^= 1;
    }
}

template <int n>
hipError_t launch_n(const float *in, const float *w_seg, float *out, const FlatParams &p, unsigned grid, size_t lds,
                    hipStream_t stream)
{
    hipLaunchKernelGGL(direct_flat_kernel<n>, dim3(grid), dim3(F_THREADS), lds, stream, in, w_seg, out, p);
    return hipGetLastError();
}

}  // namespace

bool direct_flat_plan(const Shape &s, kst_dtype dt, FlatParams &p, unsigned &grid, size_t &lds)
{
    if (dt != KST_F32 || s.Cin != 1 || s.n > 7 || (s.N & 3) != 0) return false;
    const unsigned CH = 8192;
    const long long MM = (long long)s.M * s.M;
    if (MM < CH || s.M < 8) return false;                       // a block may touch at most two planes
    p.Cout = s.Cout; p.N = s.N; p.M = s.M; p.fl = s.fl;
    p.CH = CH;
    p.MM = (unsigned)MM;
    p.total = (unsigned)((long long)s.B * s.Cout * MM);
    p.nblocks = (p.total + CH - 1) / CH;
    p.fast = s.M >= 256;
    // Input rows one piece can need: the rows its output span maps to, plus halo.
    const int span = (int)((CH - 1 + s.M - 1) / s.M);           // yb - ya at most
    p.max_rows = span / 2 + 1 + s.fl + 1;
    if (p.max_rows > s.N) p.max_rows = s.N;
    if ((size_t)p.max_rows * s.N > (size_t)F_THREADS * F_NPRE * 4) return false;   // prefetch registers
    p.xs_stride = s.N + 2 * F_PAD;
    p.xs_buf = p.max_rows * p.xs_stride;
    lds = (size_t)2 * p.xs_buf * sizeof(float);
    if (lds > 64 * 1024) return false;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(1, s.Cout, s.n, c, KST_F32);
    p.epi = s.epi;
    // One resident round: three 512-lane workgroups per CU on 256 CUs.
    const int wgs = 768;
    grid = (unsigned)wgs;
    if (grid > p.nblocks) grid = p.nblocks;
    p.run = grid % 64 == 0 ? 8 : 1;                             // 1: plain blockIdx order
    const unsigned long long gstep = (unsigned long long)grid * CH;
    p.g_plane = (int)(gstep / (unsigned long long)MM);
    const unsigned grem = (unsigned)(gstep % (unsigned long long)MM);
    p.g_y = (int)(grem / (unsigned)s.M);
    p.g_x = (int)(grem % (unsigned)s.M);
    p.s_y = F_STEP / s.M;
    p.s_x = F_STEP % s.M;
    p.c_y = (int)((CH - 1) / (unsigned)s.M);
    p.c_x = (int)((CH - 1) % (unsigned)s.M);
    return true;
}

hipError_t launch_direct_flat(const float *in, const float *w_seg, float *out, const Shape &s, const FlatParams &p,
                              unsigned grid, size_t lds, hipStream_t stream)
{
    switch (s.n) {
        case 1: return launch_n<1>(in, w_seg, out, p, grid, lds, stream);
        case 2: return launch_n<2>(in, w_seg, out, p, grid, lds, stream);
        case 3: return launch_n<3>(in, w_seg, out, p, grid, lds, stream);
        case 4: return launch_n<4>(in, w_seg, out, p, grid, lds, stream);
        case 5: return launch_n<5>(in, w_seg, out, p, grid, lds, stream);
        case 6: return launch_n<6>(in, w_seg, out, p, grid, lds, stream);
        case 7: return launch_n<7>(in, w_seg, out, p, grid, lds, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace kst
