// Matrix-core segregated forward pass for 16-bit operands on 64 x 64 maps with 3 x 3 kernels,
// "row-parity passes": the variant whose output leaves the chip WHILE the matrix cores work.
//
// Section 3.3, Eqs. 7-10 give the four members of an output quad from the four sub-kernels.
// The two members on an even output row need K1 and K2 (kernel rows 0 and 2), the two on an odd
// row K3 and K4 (kernel row 1).  A tile (64 output channels x 4 quad rows of one batch item) is
// therefore worked in two passes over the input channels: pass A accumulates its even output
// rows, pass B its odd ones.  Each pass owns its own accumulator registers, so while one pass
// multiplies, the finished rows of the pass before it are drained, a few values per chunk of the
// reduction, through a small per-wave LDS image to global memory.  The stores of a tile are thus
// spread evenly over the next pass instead of leaving as one burst of the whole chip during which
// no matrix core has work.
//
// Window column 1 of Eqs. 7-10 (input pixel j + 1 for the quad at column j) is the column-0
// fragment moved down one lane, as in the other 16-bit ring kernels; here the fragments of chunk
// c + 1 are read and shifted while chunk c is multiplied (two sets of fragment registers).
//
// One workgroup of 4 waves per CU, one wave per SIMD: 2 x 128 accumulators per lane (the whole
// accumulation register file).  A wave owns 32 channels x 2 quad rows x 64 columns.  Operands
// reach LDS by LDS-direct loads into a ring of four stages (weights already in fragment order,
// input rows in NCHW order) and leave it through ds_read_b128 / the transposing
// ds_read_b64_tr_b16.  The reduction is fully unrolled (16 chunks of 16 channels), so every
// register index, ring stage and memory-counter value is a constant, and everything a chunk has to
// do besides multiplying is dealt out over its multiplications in a fixed order.
#include <type_traits>

#include "kst_igemm_common.h"

namespace kst {

namespace {

typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

#define KST_LDS(T) T __attribute__((address_space(3)))

struct PP {
    static constexpr int N = 64, M = 125, E = 63;          // map edge, output edge 2N - 3, quad rows
    static constexpr unsigned MM = (unsigned)M * M;
    static constexpr int THREADS = 256, TCO = 64, KC = 16;
    static constexpr int CHUNKS = 16;                      // Cin / KC: the unrolled reduction
    static constexpr int TI = 4, STRIPS = (E + TI - 1) / TI;
    // The last strip of a pass is moved up so that it ends on the pass's last quad row (62 has an
    // even output row, 61 the last odd one): a few rows are computed twice, to the same values,
    // and no wave ever has a row without output.
    static constexpr int I0A_MAX = E - TI, I0B_MAX = E - 1 - TI;
    static constexpr int ROWS = TI + 1, ROW_B = N * 2, UPR = N / 8;
    static constexpr int CS = (ROWS * ROW_B + 127) / 128 * 128 + 64;   // bytes per channel of a staged image
    static constexpr int UPC = CS / 16;
    static constexpr int X_B = KC * CS, X_SLABS = X_B / 1024;
    static constexpr int WA_SLOTS = 6, WB_SLOTS = 3;       // weight fragments per chunk: pass A, pass B
    static constexpr int W_B = WA_SLOTS * 2048;
    static constexpr int STAGE_B = W_B + X_B;
    static constexpr int STAGES = 4;                       // CHUNKS % STAGES == 0: a chunk's stage is a constant
    static constexpr int RING_B = STAGES * STAGE_B;
    static constexpr int RS = 132;                         // floats per row of a drain image
    static constexpr int IMG_ROW_B = RS * 4, IMG_BUF_B = 4 * IMG_ROW_B, IMG_WAVE_B = 2 * IMG_BUF_B;
    static constexpr int LDS_B = RING_B + 4 * IMG_WAVE_B;
    static constexpr int KL_A = 6, KL_B = 5;               // LDS-direct loads per wave and chunk
    static constexpr int ST = 5;                           // global stores per wave and chunk
    static_assert(X_B % 1024 == 0 && CHUNKS % STAGES == 0 && LDS_B <= 160 * 1024, "geometry");
    static_assert(X_SLABS == 11 && 4 * 3 >= X_SLABS && 4 * 3 == WA_SLOTS * 2, "slab shares");
};

struct PPParams {
    int B, Cin, Cout, tiles_co, ntiles;
    unsigned off[4];
};

// Weight slots of a chunk, in the order they are multiplied: first the taps that read window
// column 0, then those that read column 1.  Pass A (even output rows): K1 taps (a', b') = 2a' + b'
// and K2 taps a' (kernel rows 0 and 2); pass B (odd rows): K3 taps b' and K4 (kernel row 1).
//   pass A: K1(0,0) K1(1,0) | K1(0,1) K1(1,1) K2(0) K2(1)        pass B: K3(0) | K3(1) K4
__device__ constexpr int pp_slot_cls(bool passB, int s) { return passB ? (s < 2 ? 2 : 3) : (s < 4 ? 0 : 1); }
__device__ constexpr int pp_slot_tap(bool passB, int s)
{
    return passB ? (s < 2 ? s : 0) : (s == 0 ? 0 : s == 1 ? 2 : s == 2 ? 1 : s == 3 ? 3 : s - 4);
}
__device__ constexpr int pp_slot_row(bool passB, int s) { return passB ? 0 : (s == 0 || s == 2 || s == 4 ? 0 : 1); }   // a'
__device__ constexpr int pp_slot_dx(bool passB, int s) { return passB ? (s >= 1 ? 1 : 0) : (s >= 2 ? 1 : 0); }
__device__ constexpr bool pp_slot_first(bool passB, int s) { return passB ? (s == 0 || s == 2) : (s == 0 || s == 4); }
__device__ constexpr int pp_cls_taps(int cls) { return cls == 0 ? 4 : cls == 3 ? 1 : 2; }

// Vector-memory operations a wave issues in chunk j of a pass (j < 0: the last chunks of the pass
// before it), LDS-direct loads first, then the drain's stores.  The loads of chunk j fill the
// ring four chunks ahead: from chunk 12 on they belong to the next pass.
__device__ constexpr int pp_kl(bool passB, int j)
{
    const bool own = j < PP::CHUNKS - PP::STAGES;          // j < 0: the pass before loads for this one
    return (own ? passB : !passB) ? PP::KL_B : PP::KL_A;
}
// At the top of chunk c the loads issued three chunks earlier must have landed.  Vector-memory
// operations retire in issue order, so that holds once no more operations are outstanding than
// were issued after them.
__device__ constexpr int pp_allowed(bool passB, int c)
{
    return PP::ST + pp_kl(passB, c - 2) + PP::ST + pp_kl(passB, c - 1) + PP::ST;
}

template <int N_>
__device__ __forceinline__ void wait_loads_and_meet()
{
    static_assert(N_ >= 0 && N_ < 64, "vmcnt field");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N_) : "memory");
}

// One LDS-direct load of 16 bytes per lane: M0 <- LDS byte address of lane 0's 16 bytes, one wait
// state, the load of base + lane_off.  Assembly, so that the waits on these loads are this file's
// own (the compiler does not see them and leaves the LDS reads alone).
__device__ __forceinline__ void lds_direct(unsigned lds_dst, const unsigned char *base, unsigned lane_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_dst), "v"(lane_off), "s"(base)
                 : "memory");
}

// The five streaming stores of one drain step: four rows of 8-byte pairs under the lane mask of
// their alignment, then the four partnerless elements by lanes 0..3.  One statement, so that the
// lane mask is written three times per step and nothing else runs under it (the wave runs with all
// lanes on; a write to the mask waits for the vector instructions in flight).
template <int OFF0, int OFF1, int OFFS>
__device__ __forceinline__ void store_step(unsigned long long mask, unsigned lane_off, const uintx2 (&row)[4], unsigned single_off,
                                           unsigned single, const unsigned char *b0, const unsigned char *b1)
{
    asm volatile("s_mov_b64 exec, %0\n\t"
                 "global_store_dwordx2 %1, %2, %6 offset:%8 nt\n\t"
                 "global_store_dwordx2 %1, %3, %6 offset:%9 nt\n\t"
                 "global_store_dwordx2 %1, %4, %7 offset:%8 nt\n\t"
                 "global_store_dwordx2 %1, %5, %7 offset:%9 nt\n\t"
                 "s_mov_b64 exec, 15\n\t"
                 "global_store_dword %10, %11, %6 offset:%12 nt\n\t"
                 "s_mov_b64 exec, -1" ::"s"(mask),
                 "v"(lane_off), "v"(row[0]), "v"(row[1]), "v"(row[2]), "v"(row[3]), "s"(b0), "s"(b1), "n"(OFF0), "n"(OFF1),
                 "v"(single_off), "v"(single), "n"(OFFS)
                 : "memory");
}

template <bool F16>
__global__ void __launch_bounds__(PP::THREADS, 1) igemm_bf16_pp_kernel(const uint16_t *__restrict__ in,
                                                                         const uint16_t *__restrict__ w_seg,
                                                                         float *__restrict__ out, PPParams p)
{
    using G = PP;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    KST_LDS(unsigned char) *L = (KST_LDS(unsigned char) *)lds_raw;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kk = lane >> 5;
    const int wco = wave & 1, wr = wave >> 1;
    const int s16 = lane & 15, h16 = (lane >> 4) & 1;
    const unsigned lds_base = (unsigned)(size_t)L;

    // ---- per-lane LDS addresses (byte offsets from the start of LDS) ---------------------------
    // weight fragment of slot s in stage t: + t * STAGE_B + s * 2048
    const unsigned wrd = (unsigned)((kk * G::TCO + wco * 32 + l32) * 16);
    // transposing read of block cb, row j of the wave, stage t: + t * STAGE_B + j * ROW_B (+ 4 CS: channels + 4).
    // Within a block of 16 lanes, lane s supplies channel s / 4, pixels 4 (s % 4) .. +3, and receives
    // pixel s of four channels.
    unsigned xrd[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
        xrd[cb] = (unsigned)(G::W_B + (8 * kk + (s16 >> 2)) * G::CS + 2 * wr * G::ROW_B + (32 * cb + 16 * h16 + 4 * (s16 & 3)) * 2);
    // drain image of this wave: two buffers of four rows (2 kk + q) of RS floats.  Output column x
    // of a row sits at float 2 + par + x, par = parity of the row's first element in `out`: an
    // 8-byte pair of the image is then an 8-byte aligned pair of `out`.
    const unsigned img = (unsigned)(G::RING_B + wave * G::IMG_WAVE_B);
    const unsigned iw = img + (unsigned)((2 * kk * G::RS + 2 * l32) * 4);      // this lane's column 2 X of row 2 kk
    const unsigned ir = img + (unsigned)lane * 8u;                               // pair `lane` of row 0
    const unsigned is = img + (unsigned)((lane & 3) * G::IMG_ROW_B);             // row `lane & 3`
    const unsigned lane8 = (unsigned)lane * 8u;
    // lanes 0..3 store the one element of rows 0..3 that has no partner: byte offset of row r = 2 kk + q
    const unsigned gsingle = (unsigned)(((lane >> 1) & 1) * 4 * (int)G::MM * 4 + (lane & 1) * 2 * G::M * 4);
    const unsigned long long mask_even = 0x7ffffffffffffffeull;   // row starts on an even element: pairs 1..62
    const unsigned long long mask_odd = 0xfffffffffffffffcull;    // odd: pairs 2..63

    // ---- LDS-direct plan -----------------------------------------------------------------------
    // A stage is WA_SLOTS x 2 weight slabs followed by X_SLABS image slabs of 1 KiB (one wave-wide
    // 16-byte-per-lane load each).  Wave w copies slabs w, w + 4, ... of either kind; a share that
    // runs past the last slab repeats an earlier one (the same bytes to the same place).
    const unsigned lane16 = (unsigned)lane * 16u;
    unsigned wdstA[3], wdstB[2], xdst[3];          // LDS byte address of the slab inside stage 0
    unsigned wfixA[3], wincA[3], wfixB[2], wincB[2];   // byte offset in w_seg of the slab for tile channel 0, chunk 0; per chunk
    unsigned xfix[3];                              // per lane: byte offset of its 16 bytes in a batch item, row 0, chunk 0
    int xrow[3];                                   // per lane: staged row of that unit
    auto weight_slab = [&](bool passB, int q, unsigned &dst, unsigned &fix, unsigned &inc) {
        const int s = q >> 1, oct = q & 1;
        const int cls = pp_slot_cls(passB, s), tap = pp_slot_tap(passB, s), Tp = pp_cls_taps(cls);
        const unsigned off = cls == 0 ? p.off[0] : cls == 1 ? p.off[1] : cls == 2 ? p.off[2] : p.off[3];
        dst = lds_base + (unsigned)q * 1024u;
        fix = (off + (unsigned)((oct * Tp + tap) * p.Cout) * 8u) * 2u;      // [octet][tap][channel][8] inside the class
        inc = 2u * Tp * p.Cout * 16u;                                       // a chunk is two octets
    };
#pragma unroll
    for (int k = 0; k < 3; ++k) weight_slab(false, wave + 4 * k, wdstA[k], wfixA[k], wincA[k]);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        int q = wave + 4 * k;
        if (q >= 2 * G::WB_SLOTS) q -= 2 * G::WB_SLOTS;
        weight_slab(true, q, wdstB[k], wfixB[k], wincB[k]);
    }
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        int q = wave + 4 * k;
        if (q >= G::X_SLABS) q -= G::X_SLABS;
        xdst[k] = lds_base + (unsigned)(G::W_B + q * 1024);
        const int u = q * 64 + lane;
        const int ci = u / G::UPC;
        int rem = u - ci * G::UPC;
        if (rem >= G::ROWS * G::UPR) rem = 0;                      // padding unit: any valid address
        const int row = rem / G::UPR, x8 = rem - row * G::UPR;
        xfix[k] = (unsigned)((ci * G::N * G::N + x8 * 8) * 2);
        xrow[k] = row;
    }
    constexpr unsigned x_inc = (unsigned)G::KC * G::N * G::N * 2u;

    // ---- tiles of this workgroup -----------------------------------------------------------------
    struct Tile {
        int b, co0, strip;
    };
    auto tile_of = [&](int t) {
        unsigned id = (unsigned)t;
        Tile r;
        r.strip = (int)(id % (unsigned)G::STRIPS);
        id /= (unsigned)G::STRIPS;
        r.co0 = (int)(id % (unsigned)p.tiles_co) * G::TCO;
        r.b = (int)(id / (unsigned)p.tiles_co);
        return r;
    };
    auto first_row = [&](const Tile &t, bool passB) { return min(t.strip * G::TI, passB ? G::I0B_MAX : G::I0A_MAX); };
    // Address of out[b][co0 + 32 wco][y0][0], y0 = the wave's first output row of the pass.
    auto drain_base = [&](const Tile &t, bool passB) {
        const int y0 = 2 * (first_row(t, passB) + 2 * wr) + (passB ? 1 : 0);
        const size_t e = ((size_t)(t.b * p.Cout + t.co0 + 32 * wco) * G::M + y0) * G::M;
        return reinterpret_cast<const unsigned char *>(out + e);
    };

    // Load cursors: where the next chunk of a pass is fetched from.
    struct Cursor {
        const unsigned char *wb[3];      // per weight slab of the wave: address for lane 0, current chunk
        unsigned xo[3];                  // per image slab: this lane's byte offset from xb, current chunk
        const unsigned char *xb;
    };
    auto cursor_for = [&](const Tile &t, bool passB) {
        Cursor c;
        const unsigned char *w0 = reinterpret_cast<const unsigned char *>(w_seg) + (size_t)t.co0 * 16u;
        c.wb[0] = w0 + (passB ? wfixB[0] : wfixA[0]);
        c.wb[1] = w0 + (passB ? wfixB[1] : wfixA[1]);
        c.wb[2] = w0 + wfixA[2];
        c.xb = reinterpret_cast<const unsigned char *>(in + (size_t)t.b * p.Cin * G::N * G::N);
        const int i0 = first_row(t, passB);
#pragma unroll
        for (int k = 0; k < 3; ++k) c.xo[k] = xfix[k] + (unsigned)(min(i0 + xrow[k], G::N - 1) * G::N * 2);
        return c;
    };
    // Load k of one chunk into stage `stage` (weight slabs first); the cursor moves on by one chunk.
    auto issue_load = [&](Cursor &c, auto passB_tag, auto k_tag, int stage) {
        constexpr bool passB = decltype(passB_tag)::value;
        constexpr int k = decltype(k_tag)::value, nw = passB ? 2 : 3;
        const unsigned so = (unsigned)stage * G::STAGE_B;
        if constexpr (k < nw) {
            lds_direct((passB ? wdstB[k < 2 ? k : 0] : wdstA[k]) + so, c.wb[k], lane16);
            c.wb[k] += passB ? wincB[k < 2 ? k : 0] : wincA[k];
        } else {
            lds_direct(xdst[k - nw] + so, c.xb, c.xo[k - nw]);
            c.xo[k - nw] += x_inc;
        }
    };
    auto issue_loads = [&](Cursor &c, auto passB_tag, int stage) {
        static_for<(decltype(passB_tag)::value ? G::KL_B : G::KL_A)>([&](auto k) { issue_load(c, passB_tag, k, stage); });
    };

    // ---- registers -------------------------------------------------------------------------------
    // acc?[class][q][cb]: class 0 = output column 2j (K1 / K3), 1 = column 2j + 1 (K2 / K4); q = quad
    // row of the wave; cb = 32-column block.  Rows of a block: output channels 8 (v / 4) + 4 kk + v % 4.
    floatx16 accA[2][2][2], accB[2][2][2];
    constexpr floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) accB[s2][q][cb] = zero16;
    // Fragments.  Input rows: two buffers, chunk c multiplies out of buffer c % 2 while chunk c + 1 is
    // read into the other.  Weights: the slots used early in a chunk have ONE register set, re-read
    // for the next chunk right behind their last multiplication; only the slots used last (pass A:
    // 4 and 5, pass B: 2) have two.
    uintx4 ws[4], wd[2][2];
    uintx4 xf[2][3][2];                  // [buffer][row j of the wave][cb]; pass B uses rows 0, 1 (= staged rows 1, 2)
    uintx4 xs[2][3][2];                  // the same moved down one lane: window column 1
    // Window column 1 = column 0 of the next quad = the next lane's value.  The two blocks of a row are
    // regrouped so that one register holds all 64 columns of a channel half, shifted down a lane, and
    // regrouped back (the last column of the row gets no valid value: its quad does not exist).
    // One call moves register i of row j, both blocks: four instructions.
    auto shift_x = [&](auto buf_tag, auto j_tag, auto i_tag) {
        constexpr int bf = decltype(buf_tag)::value, j = decltype(j_tag)::value, i = decltype(i_tag)::value;
        const auto g = __builtin_amdgcn_permlane32_swap(xf[bf][j][0][i], xf[bf][j][1][i], false, false);
        const unsigned lo = (unsigned)__builtin_amdgcn_mov_dpp((int)g[0], 0x130, 0xf, 0xf, true);
        const unsigned hi = (unsigned)__builtin_amdgcn_mov_dpp((int)g[1], 0x130, 0xf, 0xf, true);
        const auto h = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
        xs[bf][j][0][i] = h[0];
        xs[bf][j][1][i] = h[1];
    };
    auto read_w = [&](auto passB_tag, auto buf_tag, auto slot_tag, int stage) {
        constexpr bool passB = decltype(passB_tag)::value;
        constexpr int bf = decltype(buf_tag)::value, sl = decltype(slot_tag)::value, single = passB ? 2 : 4;
        const uintx4 v = *(KST_LDS(uintx4) *)(L + (wrd + (unsigned)(stage * G::STAGE_B + sl * 2048)));
        if constexpr (sl < single) ws[sl] = v; else wd[bf][sl - single] = v;
    };
    auto read_x = [&](auto passB_tag, auto buf_tag, auto frag_tag, int stage) {
        constexpr bool passB = decltype(passB_tag)::value;
        constexpr int bf = decltype(buf_tag)::value, j = decltype(frag_tag)::value / 2, cb = decltype(frag_tag)::value % 2;
        const unsigned a = xrd[cb] + (unsigned)(stage * G::STAGE_B + (j + (passB ? 1 : 0)) * G::ROW_B);
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((KST_LDS(shortx4) *)(L + a));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((KST_LDS(shortx4) *)(L + (a + 4u * G::CS)));
        const uintx2 l2 = __builtin_bit_cast(uintx2, lo), h2 = __builtin_bit_cast(uintx2, hi);
        xf[bf][j][cb] = uintx4{l2[0], l2[1], h2[0], h2[1]};
    };
    auto read_frags = [&](auto passB_tag, auto buf_tag, int stage) {
        constexpr bool passB = decltype(passB_tag)::value;
        static_for<(passB ? G::WB_SLOTS : G::WA_SLOTS)>([&](auto sl) { read_w(passB_tag, buf_tag, sl, stage); });
        static_for<(passB ? 4 : 6)>([&](auto fr) { read_x(passB_tag, buf_tag, fr, stage); });
        static_for<(passB ? 8 : 12)>([&](auto g) {
            shift_x(buf_tag, std::integral_constant<int, decltype(g)::value / 4>{}, std::integral_constant<int, decltype(g)::value % 4>{});
        });
    };

    // ---- the drain ---------------------------------------------------------------------------------
    // Step v (0..15) moves accumulator element v of every block of one pass: channels 8 (v / 4) + v % 4
    // (lanes kk = 0) and + 4 (kk = 1), the wave's two rows q: four image rows.  Piece 0..3 = (q, cb):
    // the lane's two neighbouring output columns 2X, 2X + 1.
    auto drain_write = [&](const floatx16 (&acc)[2][2][2], auto v_tag, auto par_tag, auto piece_tag) {
        constexpr int v = decltype(v_tag)::value, par = decltype(par_tag)::value, bufo = (v & 1) * G::IMG_BUF_B;
        constexpr int q = decltype(piece_tag)::value / 2, cb = decltype(piece_tag)::value % 2;
        KST_LDS(float) *e = (KST_LDS(float) *)(L + (iw + (unsigned)(bufo + q * G::IMG_ROW_B + (2 + par + 64 * cb) * 4)));
        e[0] = acc[0][q][cb][v];
        e[1] = acc[1][q][cb][v];
    };
    // read back step v's four rows as 8-byte pairs (lane = pair) and the four partnerless elements
    struct Drained {
        uintx2 row[4];
        unsigned single;
    };
    auto drain_read = [&](auto v_tag, auto par_tag) {
        constexpr int v = decltype(v_tag)::value, par = decltype(par_tag)::value, bufo = (v & 1) * G::IMG_BUF_B;
        Drained d;
#pragma unroll
        for (int r = 0; r < 4; ++r) d.row[r] = *(KST_LDS(uintx2) *)(L + (ir + (unsigned)(bufo + r * G::IMG_ROW_B)));
        // even start: output column 124 (float 126) is alone; odd start: column 0 (float 3)
        d.single = *(KST_LDS(unsigned) *)(L + (is + (unsigned)(bufo + (par ? 3 : 126) * 4)));
        return d;
    };
    // rows r = 2 kk + q of step v start at base + ((8 (v / 4) + v % 4 + 4 kk) M M + 2 q M) floats
    auto drain_store = [&](const Drained &d, const unsigned char *base, auto v_tag, auto par_tag) {
        constexpr int v = decltype(v_tag)::value, par = decltype(par_tag)::value;
        const unsigned char *b0 = base + (size_t)((8 * (v / 4) + v % 4) * G::MM) * 4u;
        const unsigned char *b1 = b0 + (size_t)(4 * G::MM) * 4u;
        constexpr int back = -(par + 2) * 4;                 // image float 0 of a row is `par + 2` elements before its start
        store_step<back, back + 2 * G::M * 4, (par ? 0 : 124) * 4>(par ? mask_odd : mask_even, lane8, d.row, gsingle, d.single, b0, b1);
    };

    // ---- one pass ----------------------------------------------------------------------------------
    // passB_tag: which rows are accumulated (false: even rows into accA, true: odd rows into accB).
    // The other pass's sets are drained to drain_to meanwhile; own / next are the load cursors of
    // this pass (chunks 4..15 still to fetch) and of the pass after it (its chunks 0..3).
    // drain_prev: where the rows of the pass before this one's drain go (its last step is read back
    // and stored in this pass's first chunk; they are rows of the parity this pass accumulates).
    auto run_pass = [&](auto passB_tag, Cursor &own, Cursor &next, const unsigned char *drain_to, const unsigned char *drain_prev) {
        constexpr bool passB = decltype(passB_tag)::value;
        constexpr int NM = passB ? 12 : 24;                               // multiplications per chunk
        constexpr int WSINGLE = passB ? 2 : 4;
        static_for<G::CHUNKS>([&](auto c_tag) {
            constexpr int c = decltype(c_tag)::value;
            constexpr int cur = c & 1, nxt = cur ^ 1;
            using nxt_t = std::integral_constant<int, nxt>;
            constexpr int vprev = (c + 15) & 15;                         // drain step read back in this chunk
            // parity of the first element of the drained rows: they belong to the OTHER pass (pass A
            // drains odd rows), except the step read back in chunk 0, which the pass before wrote.
            // Element ((b Cout + ch) M + y) M with M odd and b Cout even: parity of ch + y.
            constexpr int par_w = ((c & 3) + (passB ? 0 : 1)) & 1;
            constexpr int par_r = c == 0 ? ((vprev & 3) + (passB ? 1 : 0)) & 1 : ((vprev & 3) + (passB ? 0 : 1)) & 1;
            using vprev_t = std::integral_constant<int, vprev>;
            using par_w_t = std::integral_constant<int, par_w>;
            using par_r_t = std::integral_constant<int, par_r>;
            // the chunk after this one: its pass, its stage
            constexpr bool nB = c + 1 < G::CHUNKS ? passB : !passB;
            using nB_t = std::integral_constant<bool, nB>;
            constexpr int nstage = (c + 1) % G::STAGES;
            constexpr int NWn = nB ? G::WB_SLOTS : G::WA_SLOTS, WSINGLEn = nB ? 2 : 4, NXFn = nB ? 4 : 6;
            constexpr int NKL = c + G::STAGES < G::CHUNKS ? (passB ? G::KL_B : G::KL_A) : (passB ? G::KL_A : G::KL_B);
            // Where things go among the multiplications 0 .. NM - 1 (behind the one named):
            //   input fragments of the next chunk      0 .. NXFn - 1, one each
            //   LDS-direct loads                       0 .. NKL - 1, one each
            //   weights of the next chunk              single slots behind their last use; the others at WD
            //   drain: read back                       RB
            //   lane shifts of the next chunk          SH0 .., SHPER groups of four instructions each
            //   drain: image writes (4 pieces)         DW0 .., one each
            //   drain: stores (5)                      ST0
            constexpr int WD = passB ? 4 : 6, RB = passB ? 4 : 6;
            constexpr int NSH = NXFn * 2;                                  // shift groups: rows x 4 registers
            constexpr int SH0 = passB ? 4 : 7, SHPER = passB ? (NSH + 7) / 8 : 1;
            constexpr int DW0 = passB ? 5 : 19;
            constexpr int ST0 = passB ? 9 : 21;
            static_assert(NXFn <= NM && NKL <= NM && SH0 + (NSH + SHPER - 1) / SHPER <= NM && DW0 + 4 <= NM && ST0 < NM, "schedule");
            const unsigned char *dst = c == 0 ? drain_prev : drain_to;
            Drained d;

            wait_loads_and_meet<pp_allowed(passB, c)>();
            __builtin_amdgcn_sched_barrier(0);
            // One group per multiplication; the compiler may not move anything from one group to another.
            static_for<NM>([&](auto m_tag) {
                constexpr int m = decltype(m_tag)::value;
                constexpr int slot = m / 4, q = (m / 2) & 1, cb = m & 1;
                constexpr int a2 = pp_slot_row(passB, slot), dx = pp_slot_dx(passB, slot), cls = pp_slot_cls(passB, slot) & 1;
                const uintx4 &wfrag = slot < WSINGLE ? ws[slot < WSINGLE ? slot : 0] : wd[cur][slot < WSINGLE ? 0 : slot - WSINGLE];
                const uintx4 &xfrag = dx ? xs[cur][q + a2][cb] : xf[cur][q + a2][cb];
                floatx16 &acc = passB ? accB[cls][q][cb] : accA[cls][q][cb];
                acc = mfma16<F16>(__builtin_bit_cast(bf16x8, wfrag), __builtin_bit_cast(bf16x8, xfrag),
                                  c == 0 && pp_slot_first(passB, slot) ? zero16 : acc);
                if constexpr (m < NXFn) read_x(nB_t{}, nxt_t{}, m_tag, nstage);
                if constexpr (m < NKL) {
                    if constexpr (c + G::STAGES < G::CHUNKS) issue_load(own, passB_tag, m_tag, c % G::STAGES);
                    else issue_load(next, std::integral_constant<bool, !passB>{}, m_tag, c % G::STAGES);
                }
                // a single-buffered weight slot is re-read behind its last multiplication (slots the
                // next chunk does not have are skipped; slots it has beyond this pass's are read at WD)
                if constexpr ((m & 3) == 3 && slot < WSINGLE && slot < NWn) read_w(nB_t{}, nxt_t{}, std::integral_constant<int, slot>{}, nstage);
                if constexpr (m == WD) {
                    static_for<NWn>([&](auto sl) {
                        if constexpr (decltype(sl)::value >= WSINGLEn || decltype(sl)::value >= WSINGLE) read_w(nB_t{}, nxt_t{}, sl, nstage);
                    });
                }
                if constexpr (m == RB) d = drain_read(vprev_t{}, par_r_t{});
                if constexpr (m >= SH0) {
                    static_for<SHPER>([&](auto k) {
                        constexpr int g = (m - SH0) * SHPER + decltype(k)::value;
                        if constexpr (g < NSH) shift_x(nxt_t{}, std::integral_constant<int, g / 4>{}, std::integral_constant<int, g % 4>{});
                    });
                }
                if constexpr (m >= DW0 && m < DW0 + 4) {
                    using piece = std::integral_constant<int, m - DW0>;
                    if constexpr (passB) drain_write(accA, c_tag, par_w_t{}, piece{});
                    else drain_write(accB, c_tag, par_w_t{}, piece{});
                }
                if constexpr (m == ST0) drain_store(d, dst, vprev_t{}, par_r_t{});
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    };

    // ---- the workgroup's walk over its tiles -------------------------------------------------------
    int tile = blockIdx.x;
    Tile t = tile_of(tile);
    Cursor curA = cursor_for(t, false), curB = cursor_for(t, true);
#pragma unroll
    for (int c = 0; c < G::STAGES; ++c) issue_loads(curA, std::false_type{}, c);
    wait_loads_and_meet<0>();
    read_frags(std::false_type{}, std::integral_constant<int, 0>{}, 0);
    // Before the first tile there is nothing to drain: the zeros in accB and in the image buffer read
    // back first go to this workgroup's first tile, where the same wave stores the results later
    // (same wave, same addresses, in order).
#pragma unroll
    for (int r = 0; r < 4; ++r) *(KST_LDS(uintx2) *)(L + (ir + (unsigned)(G::IMG_BUF_B + r * G::IMG_ROW_B))) = uintx2{0u, 0u};
    const unsigned char *dA = drain_base(t, false);         // even rows of the tile whose accA is live or leaving
    const unsigned char *dB = drain_base(t, true);          // odd rows, accB
#pragma unroll 1
    for (;;) {
        const int tile_next = tile + (int)gridDim.x;
        const bool last = tile_next >= p.ntiles;
        const unsigned char *dA_t = drain_base(t, false), *dB_t = drain_base(t, true);
        run_pass(std::false_type{}, curA, curB, dB, dA);      // even rows of t; accB (tile before) leaves
        dA = dA_t;
        // a workgroup's last pass fetches its own tile once more instead of a tile that does not exist
        const Tile tn = last ? t : tile_of(tile_next);
        curA = cursor_for(tn, false);
        run_pass(std::true_type{}, curB, curA, dA, dB);       // odd rows of t; accA leaves
        dB = dB_t;
        if (last) break;
        tile = tile_next;
        t = tn;
        curB = cursor_for(t, true);
    }
    // ---- what is still in registers and in the image ------------------------------------------------
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");     // the ring's last (unused) loads have landed
    {
        using v15 = std::integral_constant<int, 15>;
        using par1 = std::integral_constant<int, 1>;
        const Drained d = drain_read(v15{}, par1{});
        drain_store(d, dA, v15{}, par1{});
    }
    static_for<16>([&](auto v_tag) {
        constexpr int v = decltype(v_tag)::value;
        using par = std::integral_constant<int, ((v & 3) + 1) & 1>;
        static_for<4>([&](auto piece) { drain_write(accB, v_tag, par{}, piece); });
        const Drained d = drain_read(v_tag, par{});
        drain_store(d, dB, v_tag, par{});
    });
}

template <bool F16>
hipError_t launch_pp(const uint16_t *in, const uint16_t *w_seg, float *out, const PPParams &p, hipStream_t stream)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_bf16_pp_kernel<F16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PP::LDS_B);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    const unsigned blocks = (unsigned)min(p.ntiles, cus > 0 ? cus : 256);
    hipLaunchKernelGGL((igemm_bf16_pp_kernel<F16>), dim3(blocks), dim3(PP::THREADS), PP::LDS_B, stream, in, w_seg, out, p);
    return hipGetLastError();
}

}  // namespace

// 3 x 3 kernels on 64 x 64 maps with exactly 16 chunks of 16 input channels (the reduction is
// unrolled), whole channel tiles, and at least about one tile per CU.
bool igemm_bf16_pp_supported(const Shape &s)
{
    if (s.n != 3 || s.N != PP::N || s.Ns != s.N || s.frame != 0) return false;
    if (s.Cin != PP::CHUNKS * PP::KC || s.Cout % PP::TCO != 0) return false;
    const size_t tiles = (size_t)s.B * (s.Cout / PP::TCO) * PP::STRIPS;
    return tiles >= 224 && tiles < 0x7fffffffu;
}

hipError_t launch_igemm_bf16_pp(const void *in, const void *w_seg, float *out, const Shape &s, bool f16, hipStream_t stream)
{
    if (!igemm_bf16_pp_supported(s)) return hipErrorInvalidValue;
    PPParams p;
    p.B = s.B; p.Cin = s.Cin; p.Cout = s.Cout; p.tiles_co = s.Cout / PP::TCO;
    p.ntiles = s.B * p.tiles_co * PP::STRIPS;
    for (int c = 0; c < 4; ++c) p.off[c] = (unsigned)seg_offset(s.Cin, s.Cout, s.n, c, KST_BF16);
    const uint16_t *i16 = (const uint16_t *)in, *w16 = (const uint16_t *)w_seg;
    return f16 ? launch_pp<true>(i16, w16, out, p, stream) : launch_pp<false>(i16, w16, out, p, stream);
}

}  // namespace kst
