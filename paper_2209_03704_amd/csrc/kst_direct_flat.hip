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
//
// The same kernel serves the three-channel image layers of Tables 1-2 (CI = 3 input channels, one
// output channel or a few) and padded layers (FRAME): a piece then stages its rows of every
// input channel, a lane adds the channels' contributions to its four outputs, and the zero
// frame of a padded layer exists in LDS only -- frame columns are cells that are cleared once
// and never written, frame rows are cleared when a piece at the top or bottom of a plane needs
// them -- so no framed copy of the input is made.
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
// float4 loads in flight per lane: a piece's input is at most 1024 float4 with one input channel,
// 3072 with several.
__host__ __device__ constexpr int flat_npre(int CI) { return CI == 1 ? 2 : 6; }
constexpr int F_STEP = 4 * F_THREADS;         // floats the workgroup covers per iteration
constexpr int F_STEP_LOG2 = 11;

// Flat output indices fit 32 bits: the ABI keeps every tensor below 2^31 elements.
struct Piece {
    unsigned j;               // block the piece belongs to
    unsigned fa, fb;          // flat output range of this piece, inside one plane
    unsigned p0;              // flat index of the plane's first element
    int plane;
    int ya, xa;               // row / column of fa inside the plane
    int yb;                   // last output row touched
    int ia;                   // first input row staged (a row of the framed map, if there is a frame)
    int rows_in;              // input rows staged
    int top;                  // of those, frame rows above the first row that exists in memory
    int rows_real;            // rows that exist in memory
    int full;                 // covers its whole block: fa = j*CH, fb = fa + CH
    const float *src;         // channel 0 of the batch item, first staged row that exists in memory
};

// Position (plane, row, column) of the first float of block j.
struct BlockPos {
    unsigned j;
    int plane, y, x;
};

template <bool FRAME>
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
    // (sh: with an odd padding factor output row y is row y + 1 of the map one ring wider that the
    // framed input defines; the same for columns)
    const int sh = FRAME ? p.sh : 0;
    pc.ia = (pc.ya + sh) >> 1;
    const int ib = min(p.N - 1, ((pc.yb + sh) >> 1) + p.fl);
    pc.rows_in = ib - pc.ia + 1;
    // plane -> batch item.  32-bit offsets: the input has fewer than 2^31 elements.
    const unsigned b = p.Cout == 1 ? (unsigned)pc.plane : (unsigned)pc.plane / (unsigned)p.Cout;
    if constexpr (FRAME) {
        // The staged rows in the coordinates of the tensor in memory: lo .. hi, of which only
        // those inside 0 .. N0 - 1 exist (possibly none, for a piece inside the frame).
        const int lo = pc.ia - p.q, hi = ib - p.q;
        const int first = max(lo, 0), last = min(hi, p.N0 - 1);
        pc.top = min(pc.rows_in, max(-lo, 0));
        pc.rows_real = max(last - first + 1, 0);
        const int ra = min(first, p.N0 - 1);                     // a row that exists, whatever the piece
        pc.src = in + (b * (unsigned)p.Cin * (unsigned)p.N0 + (unsigned)ra) * (unsigned)p.N0;
    } else {
        pc.top = 0;
        pc.rows_real = pc.rows_in;
        pc.src = in + (b * (unsigned)p.Cin * (unsigned)p.N + (unsigned)pc.ia) * (unsigned)p.N;
    }
}

template <bool FRAME>
__device__ __forceinline__ void first_piece(const FlatParams &p, const float *__restrict__ in, const BlockPos &bp, Piece &pc)
{
    pc.j = bp.j;
    pc.fa = bp.j * p.CH;
    pc.plane = bp.plane;
    pc.ya = bp.y;
    pc.xa = bp.x;
    finish_piece<FRAME>(p, in, pc);
}

// One aligned group in output row parity r whose first column has parity par.
// ADD: add to o instead of setting it (the second and further input channels).
template <int n, int r, int par, bool ADD = false>
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
        float acc = ADD ? o[k] : 0.0f;
#pragma unroll
        for (int a = 0; a < Ta; ++a)
#pragma unroll
            for (int bq = 0; bq < Tb; ++bq) acc = fmaf(win[a][c_k[k] + bq], wk[r][s_k[k]][a * Tb + bq], acc);
        o[k] = acc;
    }
}

// Sub-kernel (r, s) of input channel c and output channel co, from the segregated weights [class][Cin][tap][Cout].
template <int n, int r, int s>
__device__ __forceinline__ void flat_load_class(float (&w)[((n + 1) / 2) * ((n + 1) / 2)], const float *__restrict__ w_seg,
                                                unsigned off, int c, int co, int Cout)
{
    constexpr int T = (r ? n / 2 : (n + 1) / 2) * (s ? n / 2 : (n + 1) / 2);
    const float *base = w_seg + off;
#pragma unroll
    for (int t = 0; t < T; ++t) w[t] = base[(c * T + t) * Cout + co];
}

// Where the sub-kernels of all input channels do not fit the scalar registers (three channels of a
// 5 x 5 kernel are 75 values; kept resident they spill into vector-register lanes, and every
// multiply-add then pays a lane read first), a group fetches the two sub-kernels of its row parity
// from memory when it needs them: scalar loads that the scalar cache serves.  One output channel only
// (then a channel's taps are consecutive in the segregated layout and load as wide scalar loads).
struct WeightSource {
    const float *w_seg;
    unsigned off[4];
};

// The same group summed over the CI staged input channels (chan: floats between two channels' rows in LDS).
template <int n, int r, int par, int CI, bool WMEM>
__device__ __forceinline__ void flat_group_ci(float (&o)[4], const float *__restrict__ rowp, int xs_stride, int chan,
                                              int cbase, const float (&wk)[CI][2][2][((n + 1) / 2) * ((n + 1) / 2)],
                                              const WeightSource &ws)
{
    if constexpr (WMEM) {
#pragma unroll
        for (int c = 0; c < CI; ++c) {
            float w[2][2][((n + 1) / 2) * ((n + 1) / 2)];
            flat_load_class<n, r, 0>(w[r][0], ws.w_seg, ws.off[2 * r], c, 0, 1);
            flat_load_class<n, r, 1>(w[r][1], ws.w_seg, ws.off[2 * r + 1], c, 0, 1);
            if (c == 0) flat_group<n, r, par, false>(o, rowp, xs_stride, cbase, w);
            else flat_group<n, r, par, true>(o, rowp + c * chan, xs_stride, cbase, w);
        }
    } else {
        flat_group<n, r, par, false>(o, rowp, xs_stride, cbase, wk[0]);
#pragma unroll
        for (int c = 1; c < CI; ++c) flat_group<n, r, par, true>(o, rowp + c * chan, xs_stride, cbase, wk[c]);
    }
}

// (r, par) selected at run time; rowp points at the group's first tap row, column 0 of the map.
template <int n, int CI, bool WMEM>
__device__ __forceinline__ void flat_group_rp(float (&o)[4], const float *__restrict__ rowp, const FlatParams &p, int r,
                                              int x0, const float (&wk)[CI][2][2][((n + 1) / 2) * ((n + 1) / 2)],
                                              const WeightSource &ws)
{
    if (x0 & 1) {
        const int cbase = ((x0 - 1) >> 1) + 1;
        if (r) flat_group_ci<n, 1, 1, CI, WMEM>(o, rowp, p.xs_stride, p.chan_lds, cbase, wk, ws);
        else flat_group_ci<n, 0, 1, CI, WMEM>(o, rowp, p.xs_stride, p.chan_lds, cbase, wk, ws);
    } else {
        const int cbase = x0 >> 1;
        if (r) flat_group_ci<n, 1, 0, CI, WMEM>(o, rowp, p.xs_stride, p.chan_lds, cbase, wk, ws);
        else flat_group_ci<n, 0, 0, CI, WMEM>(o, rowp, p.xs_stride, p.chan_lds, cbase, wk, ws);
    }
}

// Outputs of the group at (row y, first column x0), x0 in [-3, M).  pad0: LDS column of the map's column 0.
template <int n, int CI, bool WMEM>
__device__ __forceinline__ void flat_row_group(float (&o)[4], const float *__restrict__ Xs, const FlatParams &p, int pad0,
                                               int ia, int y, int x0,
                                               const float (&wk)[CI][2][2][((n + 1) / 2) * ((n + 1) / 2)],
                                               const WeightSource &ws, int sh = 0)
{
    y += sh;
    const int r = y & 1;
    flat_group_rp<n, CI, WMEM>(o, Xs + ((y >> 1) - ia + r) * p.xs_stride + pad0, p, r, x0 + sh, wk, ws);
}

// Segment = the 256 consecutive floats one wave covers in one iteration; it starts at
// (row y, column xs) and crosses exactly one row end.  Lanes left of the row end compute
// their group in row y, lanes right of it in row y + 1, the lane on it both.
template <int n, int CI, bool WMEM>
__device__ __forceinline__ void cross_segment(float (&o)[4], const float *__restrict__ Xs, const FlatParams &p, int pad0,
                                              int ia, int y, int xs, int lane,
                                              const float (&wk)[CI][2][2][((n + 1) / 2) * ((n + 1) / 2)],
                                              const WeightSource &ws, int sh = 0)
{
    const int x0 = xs + 4 * lane;
    float oa[4] = {0.f, 0.f, 0.f, 0.f}, ob[4] = {0.f, 0.f, 0.f, 0.f};
    if (x0 < p.M) {
        const int ys = y + sh, r = ys & 1;
        flat_group_rp<n, CI, WMEM>(oa, Xs + ((ys >> 1) - ia + r) * p.xs_stride + pad0 + 2 * lane, p, r, xs + sh, wk, ws);
    }
    if (x0 + 3 >= p.M) {
        const int y1 = y + 1 + sh, xs1 = xs - p.M + sh;              // negative column: head of the next row
        const int r = y1 & 1;
        flat_group_rp<n, CI, WMEM>(ob, Xs + ((y1 >> 1) - ia + r) * p.xs_stride + pad0 + 2 * lane, p, r, xs1, wk, ws);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) o[k] = x0 + k < p.M ? oa[k] : ob[k];
}

// Rows of the zero frame above or below the rows a piece finds in memory (pieces at the top and
// bottom of a plane only): cleared over the map's width in every channel.
template <int CI>
__device__ __forceinline__ void clear_frame_rows(float *X, const FlatParams &p, int pad0, int tid, int top, int rows_real,
                                                 int rows_in)
{
    const int nz = rows_in - rows_real;                          // top + below
    if (nz == 0) return;                                         // uniform
    for (int e = tid; e < CI * nz * p.N; e += F_THREADS) {
        const int rc = e / p.N, col = e - rc * p.N;
        const int c = rc / nz, z = rc - c * nz;
        const int row = z < top ? z : rows_real + z;             // below the real rows: top + rows_real + (z - top)
        X[c * p.chan_lds + row * p.xs_stride + pad0 + col] = 0.0f;
    }
}

template <int n, int CI, bool FRAME, bool WMEM, int NPRE>
__global__ void __launch_bounds__(F_THREADS) direct_flat_kernel(const float *__restrict__ in,
                                                                  const float *__restrict__ w_seg,
                                                                  float *__restrict__ out, FlatParams p)
{
    constexpr int Ta0 = (n + 1) / 2;
    extern __shared__ __attribute__((aligned(16))) float lds[];   // 2 x [CI][max_rows][xs_stride]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n4 = (FRAME ? p.N0 : p.N) >> 2;                     // float4 per row of the tensor in memory
    const int pad0 = FRAME ? p.pad0 : F_PAD;                      // LDS column of the (framed) map's column 0
    const int sh = FRAME ? p.sh : 0;                              // odd padding factor: output (y, x) is (y + 1, x + 1) of the framed input's map

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

    // float4 number e = k * threads + tid of a staged piece is (row rr, channel c, group x4) with
    // e = (rr * CI + c) * n4 + x4, the same for every piece: where it comes from, relative to the
    // piece's first row of channel 0, and where it lands in an LDS buffer.
    int lds_off[NPRE], src_off[NPRE], row_of[NPRE];
#pragma unroll
    for (int k = 0; k < NPRE; ++k) {
        const int e = k * F_THREADS + tid;
        const int rc = e / n4, x4 = e - rc * n4;
        const int rr = rc / CI, c = rc - rr * CI;
        row_of[k] = rr;
        lds_off[k] = c * p.chan_lds + rr * p.xs_stride + pad0 + (FRAME ? p.q : 0) + 4 * x4;
        src_off[k] = c * (int)p.chan_in + rr * (FRAME ? p.N0 : p.N) + 4 * x4;
    }

    if constexpr (FRAME) {
        // The frame columns and the slack of every staged row are cells nobody writes: clear them
        // (and everything else) once.
        for (int e = tid; e < 2 * p.xs_buf; e += F_THREADS) lds[e] = 0.0f;
        __syncthreads();
    }

    Piece pc;
    first_piece<FRAME>(p, in, bp, pc);
    // First piece: plain staging (all loads issued before the first LDS write).
    {
        // (named values, gathered into an array only where they are consumed: an array that lives
        // across the loads is kept in memory by the compiler)
        auto fetch = [&](int k) {                                // k < NPRE, constant after inlining
            return *reinterpret_cast<const float4 *>(pc.src + (row_of[k] < pc.rows_real ? src_off[k] : 0));
        };
        const float4 t0 = fetch(0), t1 = fetch(1);
        const float4 t2 = NPRE > 2 ? fetch(NPRE > 2 ? 2 : 0) : t0, t3 = NPRE > 3 ? fetch(NPRE > 3 ? 3 : 0) : t0;
        const float4 t4 = NPRE > 4 ? fetch(NPRE > 4 ? 4 : 0) : t0, t5 = NPRE > 5 ? fetch(NPRE > 5 ? 5 : 0) : t0;
        const float4 t[6] = {t0, t1, t2, t3, t4, t5};
        if constexpr (FRAME) clear_frame_rows<CI>(lds, p, pad0, tid, pc.top, pc.rows_real, pc.rows_in);
#pragma unroll
        for (int k = 0; k < NPRE; ++k)
            if (row_of[k] < pc.rows_real) {
                float *d = lds + lds_off[k] + (FRAME ? pc.top * p.xs_stride : 0);
                *reinterpret_cast<float4 *>(d) = t[k];          // pad0 + q is a multiple of 4: 16-byte aligned
            }
    }
    __syncthreads();

    float wk[CI][2][2][Ta0 * Ta0];                           // WMEM: unused
    WeightSource ws = {w_seg, {p.off[0], p.off[1], p.off[2], p.off[3]}};
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
            finish_piece<FRAME>(p, in, pn);
        } else {
            bp.j += gridDim.x;
            bp.plane += p.g_plane;
            bp.y += p.g_y;
            bp.x += p.g_x;
            if (bp.x >= p.M) { bp.x -= p.M; ++bp.y; }
            if (bp.y >= p.M) { bp.y -= p.M; ++bp.plane; }
            if (bp.j < p.nblocks) first_piece<FRAME>(p, in, bp, pn);
            else more = false;
        }
        auto fetch = [&](int k) {                                // k < NPRE, constant after inlining
            return *reinterpret_cast<const float4 *>(pn.src + (row_of[k] < pn.rows_real ? src_off[k] : 0));
        };
        const float4 pre0 = fetch(0), pre1 = fetch(1);
        const float4 pre2 = NPRE > 2 ? fetch(NPRE > 2 ? 2 : 0) : pre0, pre3 = NPRE > 3 ? fetch(NPRE > 3 ? 3 : 0) : pre0;
        const float4 pre4 = NPRE > 4 ? fetch(NPRE > 4 ? 4 : 0) : pre0, pre5 = NPRE > 5 ? fetch(NPRE > 5 ? 5 : 0) : pre0;

        // ---- weights of this plane's output channel (scalar registers) ----------------------
        const int co = p.Cout == 1 ? 0 : (int)((unsigned)pc.plane % (unsigned)p.Cout);
        if (co != cur_co) {
#pragma unroll
            for (int c = 0; c < (WMEM ? 0 : CI); ++c) {
                flat_load_class<n, 0, 0>(wk[c][0][0], w_seg, p.off[0], c, co, p.Cout);
                flat_load_class<n, 0, 1>(wk[c][0][1], w_seg, p.off[1], c, co, p.Cout);
                flat_load_class<n, 1, 0>(wk[c][1][0], w_seg, p.off[2], c, co, p.Cout);
                flat_load_class<n, 1, 1>(wk[c][1][1], w_seg, p.off[3], c, co, p.Cout);
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
                // (the offsets pass through an empty statement the compiler cannot see through, or it
                // would move the weight loads out of the loop and keep every value resident again)
                if constexpr (WMEM) asm volatile("" : "+s"(ws.off[0]), "+s"(ws.off[1]), "+s"(ws.off[2]), "+s"(ws.off[3]));
                if (xs + 255 < p.M) {
                    const int ys = y + sh, r = ys & 1;
                    flat_group_rp<n, CI, WMEM>(o, Xs + ((ys >> 1) - pc.ia + r) * p.xs_stride + pad0 + 2 * lane, p, r, xs + sh, wk, ws);
                } else {
                    cross_segment<n, CI, WMEM>(o, Xs, p, pad0, pc.ia, y, xs, lane, wk, ws, sh);
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
                if constexpr (WMEM) asm volatile("" : "+s"(ws.off[0]), "+s"(ws.off[1]), "+s"(ws.off[2]), "+s"(ws.off[3]));
                if (f0 + 3 >= pc.fa && f0 < pc.fb) {
                    // A group hanging over the start of the plane is the head of row 0 (negative column).
                    const int yy = y < 0 ? 0 : y, xx = y < 0 ? x0 - p.M : x0;
                    float o[4];
                    flat_row_group<n, CI, WMEM>(o, Xs, p, pad0, pc.ia, yy, xx, wk, ws, sh);
                    if (xx + 3 >= p.M && yy + 1 <= pc.yb) {      // straddles a row end: head of the next row
                        float o2[4];
                        flat_row_group<n, CI, WMEM>(o2, Xs, p, pad0, pc.ia, yy + 1, xx - p.M, wk, ws, sh);
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
        if constexpr (FRAME) clear_frame_rows<CI>(Xn, p, pad0, tid, pn.top, pn.rows_real, pn.rows_in);
        const float4 pre[6] = {pre0, pre1, pre2, pre3, pre4, pre5};
#pragma unroll
        for (int k = 0; k < NPRE; ++k)
            if (row_of[k] < pn.rows_real) {
                float *d = Xn + lds_off[k] + (FRAME ? pn.top * p.xs_stride : 0);
                *reinterpret_cast<float4 *>(d) = pre[k];
            }
        __syncthreads();
        pc = pn;
        buf ^= 1;
    }
}

template <int n, int CI, bool FRAME, bool WMEM, int NPRE>
hipError_t launch_variant(const float *in, const float *w_seg, float *out, const FlatParams &p, unsigned grid, size_t lds,
                          hipStream_t stream)
{
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&direct_flat_kernel<n, CI, FRAME, WMEM, NPRE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((direct_flat_kernel<n, CI, FRAME, WMEM, NPRE>), dim3(grid), dim3(F_THREADS), lds, stream, in, w_seg, out, p);
    return hipGetLastError();
}

template <int n, int CI, bool FRAME, int NPRE>
hipError_t launch_npre(const float *in, const float *w_seg, float *out, const FlatParams &p, unsigned grid, size_t lds,
                       hipStream_t stream)
{
    // More sub-kernel values than the scalar registers hold beside the kernel's bookkeeping: fetched per group.
    if constexpr (CI * n * n > 40)
        if (p.Cout == 1) return launch_variant<n, CI, FRAME, true, NPRE>(in, w_seg, out, p, grid, lds, stream);
    return launch_variant<n, CI, FRAME, false, NPRE>(in, w_seg, out, p, grid, lds, stream);
}

template <int n, int CI, bool FRAME>
hipError_t launch_kernel(const float *in, const float *w_seg, float *out, const FlatParams &p, unsigned grid, size_t lds,
                         hipStream_t stream)
{
    if constexpr (CI == 1) {
        return launch_npre<n, CI, FRAME, 2>(in, w_seg, out, p, grid, lds, stream);
    } else {
        if (p.npre == 3) return launch_npre<n, CI, FRAME, 3>(in, w_seg, out, p, grid, lds, stream);
        return launch_npre<n, CI, FRAME, 6>(in, w_seg, out, p, grid, lds, stream);
    }
}

// One input channel with or without a frame, three (the image layers of Tables 1-2) likewise.
template <int n>
hipError_t launch_n(const float *in, const float *w_seg, float *out, const FlatParams &p, unsigned grid, size_t lds,
                    hipStream_t stream)
{
    if (p.q == 0) {
        if (p.Cin == 1) return launch_kernel<n, 1, false>(in, w_seg, out, p, grid, lds, stream);
        if (p.Cin == 3) return launch_kernel<n, 3, false>(in, w_seg, out, p, grid, lds, stream);
    } else if constexpr (n >= 2) {
        if (p.Cin == 1) return launch_kernel<n, 1, true>(in, w_seg, out, p, grid, lds, stream);
        if (p.Cin == 3) return launch_kernel<n, 3, true>(in, w_seg, out, p, grid, lds, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

// s.N is the edge of the map the kernel sees (with the frame, if s.frame > 0); s.frame > 0 means
// the tensor in memory is the dense unframed one and the kernel supplies the frame.
bool direct_flat_plan(const Shape &s, kst_dtype dt, FlatParams &p, unsigned &grid, size_t &lds)
{
    const int q = s.frame, N0 = s.N - 2 * q;
    if (dt != KST_F32 || (s.Cin != 1 && s.Cin != 3) || s.n > 7 || N0 < 4 || (N0 & 3) != 0 || s.Ns != s.N) return false;
    if (q < 0 || q > 4 || (q > 0 && s.n < 2)) return false;
    if (s.crop != 0 && (s.crop != 1 || q == 0)) return false;
    int npre = flat_npre(s.Cin);
    const int M = s.M - 2 * s.crop;                             // edge of the planes that are written
    if (M < 1) return false;
    const long long MM = (long long)M * M;
    // One input channel: blocks of 8192 outputs, three workgroups per CU.  Three channels: blocks of
    // 4096 where their rows fit three prefetch loads per lane and a third of the LDS, again three
    // workgroups per CU (measured against blocks of 8192 at two per CU, whose prefetch registers
    // leave room for four waves per SIMD only: Table 1's 5 x 5 kernel at a batch of 256 119 -> 107 us,
    // the 3 x 3 kernel unchanged; the narrow blocks re-read more halo rows, from L2); otherwise
    // 8192 at two per CU, or 4096 at two per CU where the rows for 8192 fit neither.
    unsigned CH = 8192;
    int per_cu = s.Cin == 1 ? 3 : 2;
    if (s.Cin > 1) {
        const size_t stride = (size_t)((8 + s.N + F_PAD + 3) & ~3);
        const int rows = (int)((CH - 1 + M - 1) / M) / 2 + 1 + s.fl + 1;
        const int rows_half = (int)((CH / 2 - 1 + M - 1) / M) / 2 + 1 + s.fl + 1;
        if ((size_t)s.Cin * rows_half * N0 <= (size_t)F_THREADS * 3 * 4 &&
            3 * 2 * s.Cin * rows_half * stride * sizeof(float) <= 160 * 1024) {
            CH = 4096; npre = 3; per_cu = 3;
        } else if ((size_t)s.Cin * rows * N0 > (size_t)F_THREADS * npre * 4 ||
                   2 * 2 * s.Cin * rows * stride * sizeof(float) > 160 * 1024) {
            CH = 4096;
        }
    }
    if (MM < CH || M < 8) return false;                       // a block may touch at most two planes
    p.Cin = s.Cin; p.Cout = s.Cout; p.N = s.N; p.M = M; p.fl = s.fl;
    p.sh = s.crop;
    p.q = q; p.N0 = N0;
    p.pad0 = q > 0 ? 8 - q : F_PAD;                             // the tensor's column 0 lands on LDS column 8 (or 4)
    p.CH = CH;
    p.npre = npre;
    p.MM = (unsigned)MM;
    p.total = (unsigned)((long long)s.B * s.Cout * MM);
    p.nblocks = (p.total + CH - 1) / CH;
    // Three channels: only where every workgroup walks over several blocks.  Below that the many small
    // workgroups of the multi-channel kernel finish sooner (16 images of 224 x 224: 10 us against 12).
    if (s.Cin > 1 && p.total / 8192 < 1024) return false;
    p.fast = M >= 256;
    // Input rows one piece can need: the rows its output span maps to, plus halo.
    const int span = (int)((CH - 1 + M - 1) / M);           // yb - ya at most
    p.max_rows = span / 2 + 1 + s.fl + 1;
    if (p.max_rows > s.N) p.max_rows = s.N;
    if ((size_t)s.Cin * p.max_rows * N0 > (size_t)F_THREADS * npre * 4) return false;   // prefetch registers
    p.xs_stride = (p.pad0 + s.N + F_PAD + 3) & ~3;
    p.chan_lds = p.max_rows * p.xs_stride;
    p.chan_in = (unsigned)N0 * (unsigned)N0;
    p.xs_buf = s.Cin * p.chan_lds;
    lds = (size_t)2 * p.xs_buf * sizeof(float);
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, KST_F32);
    p.epi = s.epi;
    // One resident round on 256 CUs.
    if (lds * per_cu > 160 * 1024) return false;
    const int wgs = 256 * per_cu;
    grid = (unsigned)wgs;
    if (grid > p.nblocks) grid = p.nblocks;
    p.run = grid % 64 == 0 ? 8 : 1;                             // 1: plain blockIdx order
    const unsigned long long gstep = (unsigned long long)grid * CH;
    p.g_plane = (int)(gstep / (unsigned long long)MM);
    const unsigned grem = (unsigned)(gstep % (unsigned long long)MM);
    p.g_y = (int)(grem / (unsigned)M);
    p.g_x = (int)(grem % (unsigned)M);
    p.s_y = F_STEP / M;
    p.s_x = F_STEP % M;
    p.c_y = (int)((CH - 1) / (unsigned)M);
    p.c_x = (int)((CH - 1) % (unsigned)M);
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
