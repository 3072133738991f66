// Plan and launcher of the flat, persistent single-channel direct kernel.
#pragma once
#include "kst_internal.h"

namespace kst {

struct FlatParams {
    int Cin, Cout, N, M, fl;   // N: edge of the map the kernel sees (frame included)
    int q, N0;              // zero frame the kernel supplies, edge of the tensor in memory (N - 2q)
    int pad0;               // LDS column of the map's column 0
    int sh;                 // 1: output (y, x) is element (y + 1, x + 1) of the map the framed input defines (odd padding factor)
    int chan_lds;           // floats per input channel in an LDS buffer
    unsigned chan_in;       // floats per input channel in memory
    unsigned CH;            // floats per block: workgroups own 1 KB-aligned blocks of the flat output
    unsigned MM;            // M * M
    unsigned total;         // B * Cout * M * M (below 2^31)
    unsigned nblocks;       // ceil(total / CH)
    // How (plane, row, column) move when the flat index advances by ...
    int g_plane, g_y, g_x;  // ... gridDim.x * CH floats (a workgroup's next block)
    int s_y, s_x;           // ... one workgroup iteration (4 * threads floats)
    int c_y, c_x;           // ... CH - 1 floats (first to last float of a full block)
    unsigned run;           // consecutive blocks handed to one XCD (1: plain blockIdx order)
    int fast;               // M >= 256: a wave's 256 floats cross at most one row end
    int max_rows;           // input rows one piece can need
    int npre;               // 16-byte loads a lane keeps in flight for the next piece
    int xs_stride, xs_buf;  // floats per staged row / per LDS buffer
    unsigned off[4];        // element offset of W_p in the segregated weights
    Epilogue epi;
};

// False when the shape is outside what the kernel covers (then the caller uses another path).
bool direct_flat_plan(const Shape &s, kst_dtype dt, FlatParams &p, unsigned &grid, size_t &lds);
hipError_t launch_direct_flat(const float *in, const float *w_seg, float *out, const Shape &s, const FlatParams &p,
                              unsigned grid, size_t lds, hipStream_t stream);

}  // namespace kst
