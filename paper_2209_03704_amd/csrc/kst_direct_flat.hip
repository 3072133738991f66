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
#include <cstdlib>

#include "kst_direct_flat.h"

namespace kst {

namespace {

constexpr int F_PAD = 4;      // slack floats left and right of each staged input row
#ifndef KST_FLAT_THREADS
#define KST_FLAT_THREADS 512
#endif
constexpr int F_THREADS = KST_FLAT_THREADS;
constexpr int F_NPRE = 1024 / F_THREADS;      // float4 loads in flight per lane (1024 per piece at most)
constexpr int F_STEP = 4 * F_THREADS;         // floats the workgroup covers per iteration
constexpr int F_STEP_LOG2 = F_THREADS == 512 ? 11 : 10;
static_assert(F_THREADS == 256 || F_THREADS == 512, "two or four float4 per lane");

// Flat output indices fit 32 bits: the ABI keeps every tensor below 2^31 elements.
struct Piece {
    unsigned fa, fb;          // flat output range of this piece, inside one plane
    unsigned p0;              // flat index of the plane's first element
    int co;                   // output channel of the plane
    int ya, yb;               // first / last output row touched
    int ia;                   // first input row staged
    int rows_in;              // input rows staged
    const float *src;         // in + first staged row
};

// Work-unit walk: block j covers flat [j*CH, (j+1)*CH) and is cut at plane ends.
struct Cursor {
    unsigned j;               // block
    unsigned f;               // next flat index to process within block j
};

__device__ __forceinline__ void piece_at(const FlatParams &p, const float *__restrict__ in, const Cursor &c, Piece &pc)
{
    const unsigned block_end = min((c.j + 1) * p.CH, p.total);
    const unsigned plane = c.f / p.MM;
    pc.p0 = plane * p.MM;
    pc.fa = c.f;
    pc.fb = min(block_end, pc.p0 + p.MM);
    const int b = (int)(plane / (unsigned)p.Cout);
    pc.co = (int)(plane - (unsigned)b * p.Cout);
    pc.ya = (int)((pc.fa - pc.p0) / (unsigned)p.M);
    pc.yb = (int)((pc.fb - 1 - pc.p0) / (unsigned)p.M);
    pc.ia = pc.ya >> 1;
    const int ib = min(p.N - 1, (pc.yb >> 1) + p.fl);
    pc.rows_in = ib - pc.ia + 1;
    pc.src = in + ((size_t)b * p.N + pc.ia) * p.N;          // Cin == 1
}

// Block schedule.  Workgroups are dealt round-robin to the 8 XCDs; runs of `run`
// consecutive blocks go to the same XCD so that neighbouring blocks find their
// shared input rows in that XCD's L2, while the chip as a whole still sweeps the
// tensor front to back.
__device__ __forceinline__ unsigned block_of(const FlatParams &p, unsigned v)
{
    const unsigned xcd = v & 7u, w = v >> 3;
    return ((w / p.run) * 8u + xcd) * p.run + (w % p.run);
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

    // This workgroup's blocks: v, v + gridDim.x, ... mapped through block_of().
    unsigned v = blockIdx.x;
    const unsigned v_end = p.vblocks;
    Cursor cur;
    // Skip virtual slots that map past the last block (the run layout rounds up).
    while (v < v_end && block_of(p, v) >= p.nblocks) v += gridDim.x;
    if (v >= v_end) return;
    cur.j = block_of(p, v);
    cur.f = cur.j * p.CH;

    // Where float4 number k*256 + tid of a staged run lands in an LDS buffer (the same for every piece).
    int lds_off[F_NPRE];
#pragma unroll
    for (int k = 0; k < F_NPRE; ++k) {
        const int e = k * F_THREADS + tid;
        const int rr = e / n4, x4 = e - rr * n4;
        lds_off[k] = rr * p.xs_stride + F_PAD + 4 * x4;
    }

    Piece pc;
    piece_at(p, in, cur, pc);
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
    int buf = 0;
    while (true) {
        // ---- where the next piece is, and its loads ------------------------------------------
        Cursor nxt = cur;
        {
            const unsigned block_end = min((cur.j + 1) * p.CH, p.total);
            if (pc.fb < block_end) {
                nxt.f = pc.fb;
            } else {
                v += gridDim.x;
                while (v < v_end && block_of(p, v) >= p.nblocks) v += gridDim.x;
                nxt.j = v < v_end ? block_of(p, v) : 0xffffffffu;
                nxt.f = nxt.j * p.CH;
            }
        }
        const bool more = nxt.j != 0xffffffffu;
        Piece pn;
        piece_at(p, in, more ? nxt : cur, pn);      // after the last piece: reload it (valid, unused)
        const int count4n = pn.rows_in * n4;
        const float4 *s4 = reinterpret_cast<const float4 *>(pn.src);
        const float4 pre0 = s4[min(tid, count4n - 1)];
        const float4 pre1 = s4[min(F_THREADS + tid, count4n - 1)];
        const float4 pre2 = F_NPRE > 2 ? s4[min(2 * F_THREADS + tid, count4n - 1)] : pre0;
        const float4 pre3 = F_NPRE > 2 ? s4[min(3 * F_THREADS + tid, count4n - 1)] : pre0;

        // ---- weights of this plane's output channel (scalar registers) ----------------------
        if (pc.co != cur_co) {
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int Ta = r ? Ta1 : Ta0, Tb = s ? Ta1 : Ta0;
#pragma unroll
                    for (int t = 0; t < Ta * Tb; ++t)
                        wk[r][s][t] = w_seg[p.off[2 * r + s] + (size_t)t * p.Cout + pc.co];   // Cin == 1
                }
            cur_co = pc.co;
        }

        // ---- compute and store this piece -------------------------------------------------------
        // Wave-level bookkeeping lives in scalar registers: fw is the flat index of the wave's
        // first float this iteration and (ys, xs) its row and column in floor-division form
        // (ys < 0 while the wave still starts before the plane).
        const float *Xs = lds + buf * p.xs_buf;
        const unsigned block_start = cur.j * p.CH;
        const int it0 = (int)((pc.fa - block_start) >> F_STEP_LOG2), it1 = (int)((pc.fb - 1 - block_start) >> F_STEP_LOG2);
        unsigned fw = block_start + ((unsigned)it0 << F_STEP_LOG2) + 256u * (unsigned)wave;
        int ys, xs;
        {
            const int K = p.dy + 1;                             // K * M > F_STEP > distance to the plane start
            const unsigned relp = (unsigned)((int)(fw - pc.p0) + K * p.M);
            const unsigned q = relp / (unsigned)p.M;
            ys = (int)q - K;
            xs = (int)(relp - q * (unsigned)p.M);
        }
        for (int it = it0; it <= it1; ++it) {
            if (fw >= pc.fa && fw + 255 < pc.fb && ys >= 0 && xs + 255 < p.M) {
                // The whole wave lies in one row and inside the piece: (r, par) are uniform, the
                // LDS window is a scalar base plus 2 * lane, the store is one full aligned float4.
                const int r = ys & 1;
                const float *rowp = Xs + ((ys >> 1) - pc.ia + r) * p.xs_stride + F_PAD + 2 * lane;
                float o[4];
                if (xs & 1) {
                    const int cbase = ((xs - 1) >> 1) + 1;
                    if (r) flat_group<n, 1, 1>(o, rowp, p.xs_stride, cbase, wk);
                    else flat_group<n, 0, 1>(o, rowp, p.xs_stride, cbase, wk);
                } else {
                    const int cbase = xs >> 1;
                    if (r) flat_group<n, 1, 0>(o, rowp, p.xs_stride, cbase, wk);
                    else flat_group<n, 0, 0>(o, rowp, p.xs_stride, cbase, wk);
                }
                *reinterpret_cast<float4 *>(out + fw + 4 * lane) = make_float4(o[0], o[1], o[2], o[3]);
            } else if (fw + 255 >= pc.fa && fw < pc.fb) {
                // General path: the wave meets a row end, a plane end or a block edge.
                const unsigned f0 = fw + 4 * lane;
                if (f0 + 3 >= pc.fa && f0 < pc.fb) {
                    int y = ys, x0 = xs + 4 * lane;
                    if (x0 >= p.M) {
                        const int qq = x0 / p.M;
                        y += qq;
                        x0 -= qq * p.M;
                    }
                    // A group hanging over the start of the plane is the head of row 0 (negative column).
                    const int yy = y < 0 ? 0 : y, xx = y < 0 ? x0 - p.M : x0;
                    float o[4];
                    flat_row_group<n>(o, Xs, p, pc.ia, yy, xx, wk);
                    if (xx + 3 >= p.M && yy + 1 <= pc.yb) {     // straddles a row end: head of the next row
                        float o2[4];
                        flat_row_group<n>(o2, Xs, p, pc.ia, yy + 1, xx - p.M, wk);
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (xx + k >= p.M) o[k] = o2[k];
                    }
                    float *dst = out + f0;                      // 16-byte aligned
                    if (f0 >= pc.fa && f0 + 3 < pc.fb) {
                        *reinterpret_cast<float4 *>(dst) = make_float4(o[0], o[1], o[2], o[3]);
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (f0 + k >= pc.fa && f0 + k < pc.fb) dst[k] = o[k];
                    }
                }
            }
            fw += F_STEP;
            xs += p.dx;
            ys += p.dy;
            if (xs >= p.M) { xs -= p.M; ++ys; }
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
        cur = nxt;
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
    p.run = 8;
    p.vblocks = ((p.nblocks + 8 * p.run - 1) / (8 * p.run)) * (8 * p.run);
    p.dy = F_STEP / s.M;
    p.dx = F_STEP % s.M;
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
    static const int wgs = getenv("KST_WGS") ? atoi(getenv("KST_WGS")) : 768;
    grid = (unsigned)wgs;
    static const int md = getenv("KST_MODE") ? atoi(getenv("KST_MODE")) : 0;
    p.mode = md;
    static const int rn = getenv("KST_RUN") ? atoi(getenv("KST_RUN")) : 8;
    p.run = rn;
    p.vblocks = ((p.nblocks + 8 * p.run - 1) / (8 * p.run)) * (8 * p.run);
    if (grid > p.vblocks) grid = p.vblocks;
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
