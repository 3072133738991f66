// Plan and launcher of the flat, persistent single-channel direct kernel.
#pragma once
#include "kst_internal.h"

namespace kst {

struct FlatParams {
    int Cout, N, M, fl;
    unsigned CH;            // floats per block: workgroups own 1 KB-aligned blocks of the flat output
    unsigned MM;            // M * M
    unsigned total;         // B * Cout * M * M (below 2^31)
    unsigned nblocks;       // ceil(total / CH)
    unsigned vblocks;       // nblocks rounded up to whole XCD runs
    unsigned run;           // consecutive blocks handed to one XCD
    int dx, dy;             // step = dy * M + dx: how (row, column) move per workgroup iteration
    int max_rows;           // input rows one piece can need
    int xs_stride, xs_buf;  // floats per staged row / per LDS buffer
    unsigned off[4];        // element offset of W_p in the segregated weights
    int mode;               // TEMP ablation
};

// False when the shape is outside what the kernel covers (then the caller uses another path).
bool direct_flat_plan(const Shape &s, kst_dtype dt, FlatParams &p, unsigned &grid, size_t &lds);
hipError_t launch_direct_flat(const float *in, const float *w_seg, float *out, const Shape &s, const FlatParams &p,
                              unsigned grid, size_t lds, hipStream_t stream);

}  // namespace kst
