// Matrix-core segregated forward pass for bfloat16 operands, persistent wide-tile variant.
//
// Same arithmetic as kst_igemm_bf16_ring.hip (Section 3.3, Eqs. 7-10 as four implicit
// GEMMs on v_mfma_f32_32x32x16_bf16, fp32 accumulation) and the same way of feeding
// the matrix cores (LDS-direct loads into a ring of stages, transposing LDS reads,
// window column 1 by a lane shift).  What differs is the shape of the work:
//   * a wave owns 32 channels x 4 position blocks (two quad rows of a 64-column map,
//     four of a 32-column map) x 4 parity classes = 256 fp32 accumulators, the whole
//     accumulator file, so there is ONE wave per SIMD.  A weight fragment read from
//     LDS feeds four MFMAs instead of two and neighbouring quad rows share their
//     window rows: 21 LDS reads per 36 MFMAs instead of 17 per 18;
//   * with one wave per SIMD nothing hides a wave's own latencies or issue slots, so
//     the reduction loop is software pipelined by hand.  There is one set of fragment
//     registers, re-read for chunk c + 1 while the MFMAs of chunk c run (each register
//     right after its last use); the chunk is laid out as a sequence of slots, one MFMA
//     each, over which the lane shifts, the LDS reads, the LDS-direct loads (three
//     instructions apiece) and the one barrier are dealt; the ring is three stages deep
//     (two chunks of global latency in flight; deeper rings measured slower);
//   * one workgroup per CU (4 waves, tile = 64 channels x 8 / CB quad rows, CB = 32-column
//     blocks per quad row) walks over tiles: tile t + grid follows tile t.
// The epilogue interleaves the classes into an LDS image of 32 channels per pass (all
// four waves write, 16 channels of each channel half) and streams it out as
// 64-byte-segment aligned 16-byte stores; its barriers wait for LDS traffic only, so
// the stores of a pass drain behind the next pass and behind the next tile's loads.
#include <type_traits>

#include "kst_igemm_common.h"

namespace kst {

typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int W_THREADS = 256;
constexpr int W_TCO = 64;
constexpr int W_KC = 16;               // channels per chunk = one MFMA reduction step

template <int n, int N>
struct WideGeom {
    static_assert(n == 2 || n == 3, "window columns 0 and 1 only");
    static_assert(N == 32 || N == 64, "a quad row is one or two 32-column blocks");
    static constexpr int fl = n / 2;
    static constexpr int NN = n * n;
    static constexpr int M = 2 * N - n;
    static constexpr int E = (M + 1) / 2;
    static constexpr int CB = (E + 31) / 32;             // 32-column position blocks per quad row
    static constexpr int QH = 1;                         // workgroups per CU
    static constexpr int QW = 4 / CB / QH;               // quad rows per wave
    static constexpr int TI = 2 * QW;                    // quad rows per tile
    static constexpr int XR = QW + fl;                   // input rows a wave reads
    static constexpr int STRIPS = (E + TI - 1) / TI;
    static constexpr int ROWS = TI + fl;                 // staged input rows
    static constexpr int ROW_B = N * 2;                  // bytes per staged row
    static constexpr int UPR = N / 8;                    // 16-byte units per row
    // Bytes per channel of an image: padded to 64 (mod 128) so that the eight channel rows
    // one transposing read touches spread over the LDS banks.
    static constexpr int CS = (ROWS * ROW_B + 127) / 128 * 128 + 64;
    static constexpr int UPC = CS / 16;                  // units per channel, padding included
    static constexpr int COPY_B = W_KC * CS;             // bytes per image
    static constexpr int W_B = NN * 2 * W_TCO * 16;      // weights per stage: [tap][octet][channel] x 16 bytes
    static constexpr int STAGE_B = W_B + COPY_B;
    static constexpr int STAGES = 3;
    static constexpr int W_SLABS = NN * 2;               // 1 KiB slabs (one wave-wide LDS-direct load each)
    static constexpr int X_SLABS = COPY_B / 1024;
    static_assert(COPY_B % 1024 == 0, "image is a whole number of slabs");
    static constexpr int SLABS = W_SLABS + X_SLABS;
    static constexpr int KW = (W_SLABS + 3) / 4;         // weight slabs per wave
    static constexpr int KX = (X_SLABS + 3) / 4;         // image slabs per wave
    static constexpr int KMAX = KW + KX;                 // LDS-direct loads per wave and chunk
    static_assert(KW * 4 - W_SLABS < 4 && KX * 4 - X_SLABS < 4 && W_SLABS >= 4 && X_SLABS >= 4, "at most one repeated slab per wave");
    static constexpr int LMAX = 2 * TI * M;              // floats per channel run of a tile
    static constexpr int ESTRIDE = (LMAX + 3 + 3) & ~3;  // floats per channel in the epilogue image
    static constexpr int TG = (15 + LMAX - 1) / 4 + 1;   // 16-byte groups per channel run, upper bound
    static constexpr int ITS = (TG + 63) / 64;           // 64-lane sweeps over the groups of a channel run
    // The image starts 64 bytes in; the last channel's sweeps may read past its run.
    static constexpr int EPI_B = (16 + 31 * ESTRIDE + 4 * 64 * ITS) * 4;
    static constexpr int LDS_B = STAGES * STAGE_B > EPI_B ? STAGES * STAGE_B : EPI_B;
    static_assert(LDS_B <= 160 * 1024 / QH, "workgroups per CU");
    static_assert(STAGES * KMAX < 64, "the vector-memory counter holds the whole ring");
};

struct WideParams {
    int B, Cin, Cout, tiles_co, ntiles;
    unsigned off[4];
    Epilogue epi;
};

#define KST_LDS(T) T __attribute__((address_space(3)))

// Workgroup barrier behind this wave's LDS traffic.  Vector-memory operations (global
// stores of an earlier pass, LDS-direct loads the caller has accounted for) stay in flight.
__device__ __forceinline__ void lds_meet() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// One LDS-direct load of 16 bytes per lane, in two statements: M0 <- LDS byte address of
// lane 0's 16 bytes (lane l lands 16 l bytes further), then the load of base + lane_off.
// An instruction must sit between the two (M0 needs a wait state before the load reads
// it): the callers put an MFMA there.  The compiler keeps nothing in M0 across statements
// (it loads it right in front of each use of its own).  Written as assembly so that the
// waits on these loads are the kernel's own: the compiler would put a wait for ALL
// vector-memory operations, global stores included, in front of every LDS access it sees
// while such a load may be in flight.
__device__ __forceinline__ void lds_direct_aim(unsigned stage_addr, unsigned dst)
{
    asm volatile("s_add_u32 m0, %0, %1" :: "s"(stage_addr), "s"(dst) : "scc", "memory");
}
__device__ __forceinline__ void lds_direct_load(const unsigned char *base, unsigned lane_off)
{
    asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(lane_off), "s"(base) : "memory");
}

// Wait until at most `chunks` chunks (KMAX loads each) of this wave's LDS-direct loads are
// outstanding (vector-memory operations complete in issue order), then meet the other waves.
template <int KMAX>
__device__ __forceinline__ void wait_loads_and_meet(int chunks)
{
    switch (chunks) {
        case 0: asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory"); break;
        case 1: asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(KMAX) : "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * KMAX) : "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(3 * KMAX) : "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(4 * KMAX) : "memory"); break;
    }
}

// Taps in the order they are multiplied: first those that read window column 0, then those
// that read column 1.
template <int n>
struct TapOrder {
    int T[n * n], cls[n * n], dy[n * n], dx[n * n], n0;
    bool first[n * n];            // no earlier tap in this order belongs to the same class
    constexpr TapOrder() : T(), cls(), dy(), dx(), n0(0), first()
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
        for (int a = 0; a < n * n; ++a) {
            first[a] = true;
            for (int b = 0; b < a; ++b)
                if (cls[b] == cls[a]) first[a] = false;
        }
    }
};

// EPI: an instantiation of its own for layers with an epilogue (bias, activation), so that the
// store loop of the bare layer stays exactly as it is scheduled without one.
template <int n, int N, bool F16, bool EPI>
__global__ void __launch_bounds__(W_THREADS, (WideGeom<n, N>::QH)) igemm_bf16_wide_kernel(const uint16_t *__restrict__ in,
                                                                      const uint16_t *__restrict__ w_seg,
                                                                      float *__restrict__ out, WideParams p)
{
    using G = WideGeom<n, N>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    constexpr TapOrder<n> ord;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    const int wco = wave & 1, wrow = wave >> 1;

    // Byte offset inside a stage of the 8-byte row piece this lane hands to the transposing
    // read of block cb, first row of the wave: within a block of 16 lanes, lane s supplies
    // channel s / 4 and pixels 4 (s % 4) .. +3, and receives pixel s of four channels.
    const int s16 = lane & 15, h16 = (lane >> 4) & 1;
    unsigned xrd[G::CB];
#pragma unroll
    for (int cb = 0; cb < G::CB; ++cb)
        xrd[cb] = (unsigned)(G::W_B + (8 * kk + (s16 >> 2)) * G::CS + wrow * G::QW * G::ROW_B +
                             (32 * cb + 16 * h16 + 4 * (s16 & 3)) * 2);
    const unsigned wrd = (unsigned)((kk * W_TCO + wco * 32 + l32) * 16);
    const unsigned lds_base = (unsigned)(size_t)(KST_LDS(unsigned char) *)lds_raw;

    // ---- LDS-direct plan, the part that does not depend on the tile --------------------------
    // A stage is W_SLABS weight slabs followed by X_SLABS image slabs of 1 KiB (one wave-wide
    // 16-byte-per-lane load each).  Wave w copies weight slabs w, w + 4, ... in its first KW
    // slots and image slabs w, w + 4, ... in its last KX slots: exactly KMAX loads per wave
    // and chunk (a slot past the last slab repeats slab 0, 1, ...: the same bytes to the same
    // place).  A load's address is a wave-uniform base that advances once per chunk plus a
    // per-lane byte offset.
    unsigned g_dst[G::KMAX], g_inc[G::KW], w_fix[G::KW], x_fix[G::KX];
    int x_row[G::KX];                    // staged row of this lane's image unit
#pragma unroll
    for (int k = 0; k < G::KW; ++k) {
        int q = wave + 4 * k;
        if (q >= G::W_SLABS) q -= G::W_SLABS;
        g_dst[k] = (unsigned)q * 1024u;
        const int T = q >> 1, oct = q & 1;
        int cls = 0;
#pragma unroll
        for (int c = 1; c < 4; ++c)
            if (T >= class_tap_base(n, c)) cls = c;
        int Tp = class_taps(n, 0), tb = 0;
#pragma unroll
        for (int c = 1; c < 4; ++c)
            if (cls == c) { Tp = class_taps(n, c); tb = class_tap_base(n, c); }
        // byte offset of (class, octet, tap, channel 0) inside w_seg
        w_fix[k] = (p.off[cls] + (unsigned)((oct * Tp + (T - tb)) * p.Cout) * 8u) * 2u;
        g_inc[k] = 2u * Tp * p.Cout * 16u;
    }
#pragma unroll
    for (int k = 0; k < G::KX; ++k) {
        int q = wave + 4 * k;
        if (q >= G::X_SLABS) q -= G::X_SLABS;
        g_dst[G::KW + k] = (unsigned)(G::W_SLABS + q) * 1024u;
        const int u = q * 64 + lane;
        const int ci = u / G::UPC;
        int rem = u - ci * G::UPC;
        if (rem >= G::ROWS * G::UPR) rem = 0;                      // padding unit: any valid address
        const int row = rem / G::UPR, x8 = rem - row * G::UPR;
        x_fix[k] = (unsigned)((ci * N * N + x8 * 8) * 2);
        x_row[k] = row;
    }
    constexpr unsigned x_inc = (unsigned)W_KC * N * N * 2u;

    const int nchunks = p.Cin / W_KC;
    const int ring = nchunks < G::STAGES ? nchunks : G::STAGES;

#pragma unroll 1
    for (int tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
        unsigned id = (unsigned)tile;
        const int strip = (int)(id % (unsigned)G::STRIPS);
        id /= (unsigned)G::STRIPS;
        const int tile_co = (int)(id % (unsigned)p.tiles_co);
        const int b = (int)(id / (unsigned)p.tiles_co);
        const int co0 = tile_co * W_TCO;
        const int i0 = strip * G::TI;
        const int rows_q = min(G::TI, G::E - i0);

        // Two wave-uniform bases for the whole tile; the per-lane byte offsets move on by one
        // chunk each time their load is issued.
        const unsigned char *w_base = reinterpret_cast<const unsigned char *>(w_seg) + (size_t)co0 * 16u;
        const unsigned char *x_base = reinterpret_cast<const unsigned char *>(in + (size_t)b * p.Cin * N * N);
        unsigned g_off[G::KMAX];
#pragma unroll
        for (int k = 0; k < G::KW; ++k) g_off[k] = w_fix[k] + (unsigned)lane * 16u;
#pragma unroll
        for (int k = 0; k < G::KX; ++k) g_off[G::KW + k] = x_fix[k] + (unsigned)(min(i0 + x_row[k], N - 1) * N * 2);

        // Load k of the next chunk to be issued, in two halves with an instruction between them.
        auto aim_one = [&](int k, unsigned stage_addr) {
            lds_direct_aim(stage_addr, g_dst[k]);
        };
        auto load_one = [&](int k) {
            lds_direct_load(k < G::KW ? w_base : x_base, g_off[k]);
            g_off[k] += k < G::KW ? g_inc[k < G::KW ? k : 0] : x_inc;
        };

        // Fragment registers: ONE set, refreshed in place.  t[r][cb][h] is a window-row
        // fragment as the transposing read returns it, w[m] the weight fragment of tap m (in
        // multiplication order).  The reads of a chunk are issued, always in the same order
        // (ending with w[NN - 1]), while the previous chunk is multiplied: each register is
        // re-read after its last use.  LDS returns data in issue order, so a counter wait that
        // allows k reads in flight covers all but the k newest.
        uintx2 t[G::XR][G::CB][2];
        uintx4 w[G::NN];
        auto read_w = [&](unsigned sb, int m) {
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(w[m]) : "v"(sb + wrd), "n"(ord.T[m] * 2048) : "memory");
        };
        auto read_t = [&](unsigned sb, int r, int cb) {
            asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\t"
                         "ds_read_b64_tr_b16 %1, %2 offset:%4"
                         : "=&v"(t[r][cb][0]), "=&v"(t[r][cb][1])
                         : "v"(sb + xrd[cb]), "n"(r * G::ROW_B), "n"(r * G::ROW_B + 4 * G::CS)
                         : "memory");
        };
        // Nothing may look at a fragment register before a wait that names it.  The reads of a
        // chunk are issued in this order: w[0 .. n0) behind the column-0 taps, then the window
        // reads in the first slots of the column-1 taps, with w[m] behind tap m.  LATE = the
        // weight reads issued after the last window read: at the top of a chunk they may still
        // be in flight (wait_early), the wave waits for them behind the first tap (wait_late).
        constexpr int TAP_MFMA_ = G::QW * G::CB;
        constexpr int NT_ = G::XR * G::CB;                     // window reads (pairs), one per slot
        constexpr int LATE = G::NN - ord.n0 - NT_ / TAP_MFMA_;   // taps whose first slot comes after slot NT_, plus w[NN - 1]
        static_assert(LATE >= 1 && LATE <= G::NN - ord.n0 && LATE < 15, "late weight reads");
        auto wait_early = [&]() {
#pragma unroll
            for (int r = 0; r < G::XR; ++r) {
                if constexpr (G::CB == 2)
                    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(t[r][0][0]), "+v"(t[r][0][1]), "+v"(t[r][1][0]), "+v"(t[r][1][1]) : "n"(LATE) : "memory");
                else
                    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(t[r][0][0]), "+v"(t[r][0][1]) : "n"(LATE) : "memory");
            }
#pragma unroll
            for (int m = 0; m < G::NN - LATE; ++m) asm volatile("" : "+v"(w[m]));
        };
        auto wait_late = [&]() {
#pragma unroll
            for (int m = G::NN - LATE; m < G::NN; ++m) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w[m]) :: "memory");
        };

        // The accumulators are not cleared: in a tile's first chunk the first tap of every class
        // multiplies into zeros (the MFMA's addend is the constant 0).
        floatx16 acc[G::QW][4][G::CB];
        constexpr floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

        // Chunk c, multiplied out of the stage at LDS address `cur`, while chunk c + 1 is read
        // from the stage at `nxt`.  The wave is alone on its SIMD and issues in order, so
        // whatever stands between two MFMAs must fit in the time the first one runs: the body
        // is a sequence of slots, one MFMA each, and the other instructions of the chunk are
        // dealt out over them.
        //   column-0 taps: the lane shifts that make the column-1 fragments, a window row per
        //     tap, interleaved with the tap's MFMAs by the compiler;
        //   behind the first tap: the wave waits for its share of chunk c + 1 and meets the
        //     others (every wave then holds ALL of chunk c in registers, so the stage of chunk c
        //     may be refilled with chunk c + STAGES, and chunk c + 1 is whole);
        //   column-1 taps: the window reads of chunk c + 1 (the unshifted fragments are dead by
        //     then), then the LDS-direct loads of chunk c + STAGES, M0 written in front of a
        //     slot's MFMA and the load issued behind it;
        //   at the first MFMA of each tap: the weight fragment of the tap before, for chunk c + 1.
        // more: a chunk follows; issue: chunk c + STAGES exists.
        auto chunk = [&](int c, unsigned cur, unsigned nxt, auto more_tag, auto issue_tag, auto first_tag) {
            constexpr bool more = decltype(more_tag)::value;
            constexpr bool issue = decltype(issue_tag)::value;
            constexpr bool first_chunk = decltype(first_tag)::value;
            constexpr int TAP_MFMA = G::QW * G::CB;
            constexpr int S1 = (G::NN - ord.n0) * TAP_MFMA;
            constexpr int NT = G::XR * G::CB;                  // window reads (pairs)
            constexpr int RPT = (G::XR + ord.n0 - 1) / ord.n0; // window rows shifted per column-0 tap
            constexpr int ROW_OPS = G::CB == 2 ? 16 : 4;       // vector instructions of one row's shift
            static_assert(NT + 1 < S1, "window reads and loads fit the column-1 slots");
            wait_early();
            uintx4 x[G::XR][G::CB], xs[G::XR][G::CB];
#pragma unroll
            for (int r = 0; r < G::XR; ++r)
#pragma unroll
                for (int cb = 0; cb < G::CB; ++cb)
                    x[r][cb] = __builtin_shufflevector(t[r][cb][0], t[r][cb][1], 0, 1, 2, 3);
            // Window column 1 = column 0 of the next quad = the next lane's value.  With both
            // blocks of a quad row in the wave, the halves are regrouped so that one register
            // holds all 64 columns of a channel half, shifted down a lane, and regrouped back; a
            // lone block is shifted as it is (its last column lies past the row's last valid quad).
            auto shift_row = [&](int r) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (G::CB == 2) {
                        const auto g = __builtin_amdgcn_permlane32_swap(x[r][0][i], x[r][1][i], false, false);
                        const unsigned lo = (unsigned)__builtin_amdgcn_mov_dpp((int)g[0], 0x130, 0xf, 0xf, true);
                        const unsigned hi = (unsigned)__builtin_amdgcn_mov_dpp((int)g[1], 0x130, 0xf, 0xf, true);
                        const auto h = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
                        xs[r][0][i] = h[0];
                        xs[r][1][i] = h[1];
                    } else {
                        xs[r][0][i] = (unsigned)__builtin_amdgcn_mov_dpp((int)x[r][0][i], 0x130, 0xf, 0xf, true);
                    }
                }
            };
#pragma unroll
            for (int m = 0; m < ord.n0; ++m) {
                // a register is re-read one MFMA after the last MFMA that reads it has been issued
                if constexpr (more)
                    if (m > 0) read_w(nxt, m - 1);
#pragma unroll
                for (int q = 0; q < G::QW; ++q)
#pragma unroll
                    for (int cb = 0; cb < G::CB; ++cb)
                        acc[q][ord.cls[m]][cb] = mfma16<F16>(
                            __builtin_bit_cast(bf16x8, w[m]), __builtin_bit_cast(bf16x8, x[q + ord.dy[m]][cb]),
                            first_chunk && ord.first[m] ? zero16 : acc[q][ord.cls[m]][cb]);
#pragma unroll
                for (int r = m * RPT; r < (m + 1) * RPT && r < G::XR; ++r) shift_row(r);
#pragma unroll
                for (int i = 0; i < TAP_MFMA; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, (RPT * ROW_OPS + TAP_MFMA - 1) / TAP_MFMA, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (m == 0) {
                    wait_late();
                    if constexpr (more) {
                        if constexpr (issue)
                            wait_loads_and_meet<G::KMAX>(G::STAGES - 2);            // chunks c + 2 .. stay in flight
                        else
                            wait_loads_and_meet<G::KMAX>(min(G::STAGES - 1, nchunks - 1 - c) - 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            int slot = 0;
#pragma unroll
            for (int m = ord.n0; m < G::NN; ++m) {
#pragma unroll
                for (int q = 0; q < G::QW; ++q)
#pragma unroll
                    for (int cb = 0; cb < G::CB; ++cb) {
                        // loads: slots NT + 1 .. , spread evenly; the load of slot s is aimed in front of its MFMA
                        constexpr int SL = S1 - NT - 1;
                        const int s2 = slot - NT - 1;
                        const int k0 = s2 >= 0 ? s2 * G::KMAX / SL : 0, k1 = s2 >= 0 ? (s2 + 1) * G::KMAX / SL : 0;
                        if constexpr (issue)
                            if (k1 > k0) { aim_one(k0, cur); __builtin_amdgcn_sched_barrier(0); }
                        acc[q][ord.cls[m]][cb] = mfma16<F16>(
                            __builtin_bit_cast(bf16x8, w[m]), __builtin_bit_cast(bf16x8, xs[q + ord.dy[m]][cb]),
                            first_chunk && ord.first[m] ? zero16 : acc[q][ord.cls[m]][cb]);
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (more) {
                            if (q == 0 && cb == 0) read_w(nxt, m - 1);
                            if (slot >= 1 && slot <= NT) read_t(nxt, (slot - 1) / G::CB, (slot - 1) % G::CB);
                            if constexpr (issue) {
#pragma unroll
                                for (int k = k0; k < k1; ++k) {
                                    if (k > k0) { aim_one(k, cur); asm volatile("s_nop 0"); }
                                    load_one(k);
                                }
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        ++slot;
                    }
            }
            if constexpr (more) read_w(nxt, G::NN - 1);
            __builtin_amdgcn_sched_barrier(0);
        };

        // ---- reduction over the input channels -------------------------------------------------
        for (int c = 0; c < ring; ++c) {
#pragma unroll
            for (int k = 0; k < G::KMAX; ++k) {
                aim_one(k, lds_base + (unsigned)c * G::STAGE_B);
                asm volatile("s_nop 0");
                load_one(k);
            }
        }
        wait_loads_and_meet<G::KMAX>(ring - 1);
        // the first chunk's fragments, in the order every later chunk's are read
#pragma unroll
        for (int m = 0; m + 1 < ord.n0; ++m) read_w(lds_base, m);
        {
            int slot = 0;
#pragma unroll
            for (int m = ord.n0; m < G::NN; ++m) {
#pragma unroll
                for (int i = 0; i < TAP_MFMA_; ++i, ++slot) {
                    if (i == 0) read_w(lds_base, m - 1);
                    if (slot >= 1 && slot <= NT_) read_t(lds_base, (slot - 1) / G::CB, (slot - 1) % G::CB);
                }
            }
            read_w(lds_base, G::NN - 1);
        }
        {
            constexpr unsigned RING_B = (unsigned)G::STAGES * G::STAGE_B;
            unsigned cur = lds_base;                               // stage of chunk c
            auto next_of = [&](unsigned a) { return a + G::STAGE_B == lds_base + RING_B ? lds_base : a + G::STAGE_B; };
            // (the launcher takes layers with more than STAGES chunks only: the first chunk always
            // has a successor and a chunk to issue loads for)
            {
                const unsigned nxt = next_of(cur);
                chunk(0, cur, nxt, std::true_type{}, std::true_type{}, std::true_type{});
                cur = nxt;
            }
            int c = 1;
#pragma unroll 1
            for (; c + G::STAGES < nchunks; ++c) {
                const unsigned nxt = next_of(cur);
                chunk(c, cur, nxt, std::true_type{}, std::true_type{}, std::false_type{});
                cur = nxt;
            }
#pragma unroll 1
            for (; c + 1 < nchunks; ++c) {
                const unsigned nxt = next_of(cur);
                chunk(c, cur, nxt, std::true_type{}, std::false_type{}, std::false_type{});
                cur = nxt;
            }
            chunk(c, cur, cur, std::false_type{}, std::false_type{}, std::false_type{});
        }

        // ---- epilogue ----------------------------------------------------------------------------
        // Per output channel the tile is one contiguous run of rows_out * M floats.  The four
        // classes are interleaved into that run in LDS, 32 channels per pass, and streamed out
        // with 16-byte stores whose lane quads sit in one 64-byte segment (lane t of a channel
        // owns floats [base64 + 4t, +4), base64 = run start rounded down to 64 bytes); only the
        // groups cut by the ends of a run use scalar stores.
        // Channel cl of a pass keeps its run at Es[cl][(run start & 3) + ...], so that 16-byte
        // groups of the run are 16-byte aligned in LDS too.  M * M is 0 or 1 (mod 4), so among
        // the channels 8q + 4kk + j a lane holds, that shift depends on j alone.
        // The image starts 64 bytes into LDS: a channel's first group may begin up to 12 floats
        // ahead of its run.  The barriers wait for LDS traffic only: the global stores of a pass
        // stay in flight across them.
        float *Es = reinterpret_cast<float *>(lds_raw) + 16;            // [32][ESTRIDE]
        // The lane's place is re-read behind an opaque statement: the epilogue's per-lane
        // addresses would otherwise be computed once, ahead of the tile loop, and sit in
        // registers the reduction loop needs.
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        const int l32e = lane_e & 31, kke = lane_e >> 5;
        const int rows_out = min(2 * rows_q, G::M - 2 * i0);
        const int L = rows_out * G::M;
        constexpr unsigned MM = (unsigned)G::M * G::M;
        const unsigned g_first = (((unsigned)b * p.Cout + co0) * G::M + 2 * i0) * G::M;   // run start of channel co0
#pragma unroll 1
        for (int pass = 0; pass < 2; ++pass) {
            lds_meet();                                                  // LDS is free: K loop / previous pass read it
            // Every wave writes the half of its accumulators that holds channels 16 pass .. +15 of
            // its 32: image slot 16 wco + (channel - 16 pass) <-> channel co0 + 32 wco + 16 pass + ...
            auto write_half = [&](auto half_tag) {
                constexpr int H = decltype(half_tag)::value;
#pragma unroll
                for (int qr = 0; qr < G::QW; ++qr)
#pragma unroll
                    for (int cb = 0; cb < G::CB; ++cb) {
                        const int ti = wrow * G::QW + qr, tj = cb * 32 + l32e;
                        if (ti >= rows_q || tj >= G::E) continue;
                        const bool x1_ok = 2 * tj + 1 < G::M;
                        const bool r1_ok = 2 * ti + 1 < rows_out;
                        float *eq = Es + (16 * wco + 4 * kke) * G::ESTRIDE + 2 * ti * G::M + 2 * tj;
                        // One predicate per class, set once around its stores.
#pragma unroll
                        for (int cls = 0; cls < 4; ++cls) {
                            if ((cls & 1) && !x1_ok) continue;
                            if ((cls & 2) && !r1_ok) continue;
                            float *ec = eq + (cls & 1) + (cls >> 1) * G::M;
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                float *ej = ec + j * G::ESTRIDE + ((g_first + j * (MM & 3u)) & 3u);
                                ej[0] = acc[qr][cls][cb][8 * H + j];
                                ej[8 * G::ESTRIDE] = acc[qr][cls][cb][8 * H + 4 + j];
                            }
                        }
                    }
            };
            if (pass == 0) write_half(std::integral_constant<int, 0>{});
            else write_half(std::integral_constant<int, 1>{});
            lds_meet();
            // Wave w streams image slots w, w + 4, ...; lane t of a channel owns the 16-byte group
            // [base64 + 4t, +4) of the output, base64 = run start rounded down to 64 bytes.  All
            // groups of a channel are read from LDS first (those outside the run are read too and
            // dropped: they lie inside the LDS allocation), then stored.
            constexpr int ITS = G::ITS;
            static_assert(16 + 31 * G::ESTRIDE + 4 * 64 * ITS <= G::LDS_B / 4, "group reads stay inside LDS");
#pragma unroll 2
            for (int cl = wave; cl < 32; cl += W_THREADS / 64) {
                const int ch = 32 * (cl >> 4) + 16 * pass + (cl & 15);      // channel of the tile in image slot cl
                const unsigned g_co = g_first + (unsigned)ch * MM;
                const int a16 = (int)(g_co & 15u);                          // run start inside its 64-byte segment
                const float *erun = Es + cl * G::ESTRIDE - (int)(g_co & 12u);   // group t of the run is at erun + 4t
                float *orun = out + (g_co & ~15u);
                float4 v[ITS];
#pragma unroll
                for (int it = 0; it < ITS; ++it) v[it] = *reinterpret_cast<const float4 *>(erun + 4 * (lane_e + 64 * it));
                if constexpr (EPI) {
                    const float bias = epi_bias(p.epi, co0 + ch);
#pragma unroll
                    for (int it = 0; it < ITS; ++it) epi_apply4(v[it].x, v[it].y, v[it].z, v[it].w, bias, p.epi.act);
                }
#pragma unroll
                for (int it = 0; it < ITS; ++it) {
                    const int tt = lane_e + 64 * it;
                    const int rel = 4 * tt - a16;                          // first float of the group, relative to the run
                    if (rel >= 0 && rel + 3 < L) {
                        // streaming store: the line is written back soon instead of sitting in L2
                        // until the whole chip's next burst of stores pushes it out
                        store_streaming4(orun + 4 * tt, v[it].x, v[it].y, v[it].z, v[it].w);
                    } else if (rel + 3 >= 0 && rel < L) {
                        const float f[4] = {v[it].x, v[it].y, v[it].z, v[it].w};
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (rel + k >= 0 && rel + k < L) orun[4 * tt + k] = f[k];
                    }
                }
            }
        }
        lds_meet();                                                      // the image has been read: the ring may refill
    }
}

template <int n, int N, bool F16, bool EPI>
hipError_t launch_wide_epi(const uint16_t *in, const uint16_t *w_seg, float *out, const WideParams &p, hipStream_t stream)
{
    using G = WideGeom<n, N>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_bf16_wide_kernel<n, N, F16, EPI>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_B);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    const unsigned blocks = (unsigned)min(p.ntiles, (cus > 0 ? cus : 256) * G::QH);
    hipLaunchKernelGGL((igemm_bf16_wide_kernel<n, N, F16, EPI>), dim3(blocks), dim3(W_THREADS), G::LDS_B, stream, in, w_seg, out, p);
    return hipGetLastError();
}

template <int n, int N, bool F16>
hipError_t launch_wide(const uint16_t *in, const uint16_t *w_seg, float *out, const WideParams &p, hipStream_t stream)
{
    if (epi_on(p.epi)) return launch_wide_epi<n, N, F16, true>(in, w_seg, out, p, stream);
    return launch_wide_epi<n, N, F16, false>(in, w_seg, out, p, stream);
}

template <int n, int N>
constexpr int wide_strips() { return WideGeom<n, N>::STRIPS; }

int strips_of(const Shape &s)
{
    switch (s.n * 1000 + s.N) {
        case 2032: return wide_strips<2, 32>();
        case 2064: return wide_strips<2, 64>();
        case 3032: return wide_strips<3, 32>();
        case 3064: return wide_strips<3, 64>();
        default: return 0;
    }
}

}  // namespace

// The wide tiles pay off once there is at least one of them per CU.
bool igemm_bf16_wide_supported(const Shape &s)
{
    if (s.n != 2 && s.n != 3) return false;
    if (s.N != 32 && s.N != 64) return false;
    if (s.Cin % W_KC != 0 || s.Cout % W_TCO != 0) return false;
    if (s.Cin / W_KC <= 3) return false;            // more chunks than ring stages (3 for every geometry)
    const size_t tiles = (size_t)s.B * (s.Cout / W_TCO) * strips_of(s);
    return tiles >= 224 && tiles < 0x7fffffffu;
}

hipError_t launch_igemm_bf16_wide(const void *in, const void *w_seg, float *out, const Shape &s, bool f16,
                                  hipStream_t stream)
{
    if (!igemm_bf16_wide_supported(s)) return hipErrorInvalidValue;
    WideParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.tiles_co = s.Cout / W_TCO;
    p.ntiles = s.B * p.tiles_co * strips_of(s);
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, KST_BF16);
    p.epi = s.epi;
    const uint16_t *i16 = (const uint16_t *)in, *w16 = (const uint16_t *)w_seg;
    switch (s.n * 1000 + s.N) {
        case 2032: return f16 ? launch_wide<2, 32, true>(i16, w16, out, p, stream) : launch_wide<2, 32, false>(i16, w16, out, p, stream);
        case 2064: return f16 ? launch_wide<2, 64, true>(i16, w16, out, p, stream) : launch_wide<2, 64, false>(i16, w16, out, p, stream);
        case 3032: return f16 ? launch_wide<3, 32, true>(i16, w16, out, p, stream) : launch_wide<3, 32, false>(i16, w16, out, p, stream);
        case 3064: return f16 ? launch_wide<3, 64, true>(i16, w16, out, p, stream) : launch_wide<3, 64, false>(i16, w16, out, p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace kst
