/*
 * kst -- kernel-segregated transpose convolution (arxiv 2209.03704) for
 * AMD MI355X (gfx950).  C ABI of libkst.so.
 *
 * The operation (Section 1 and Eq. 1 of Section 2 of the paper): an N x N map
 * is up-sampled to (2N-1) x (2N-1) by embedding a zero after every row and
 * column, then correlated (no kernel flip, stride 1) with an n x n kernel,
 * summed over input channels, giving an M x M map with M = 2N - n.  The
 * library never builds the up-sampled map: it splits each kernel into four
 * sub-kernels by (row, column) parity (Section 3.2) and applies them to the
 * original input, four outputs per step (Section 3.3, Eqs. 7-10).
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer to memory the caller owns
 *     (hipMalloc or a PyTorch tensor).  The library keeps none of them.
 *   - Dense row-major layouts: in[B][Cin][N][N], w[Cout][Cin][n][n],
 *     out[B][Cout][M][M].  out is always fp32 and is completely overwritten
 *     (no bias, no activation, no accumulation).  Buffers must not alias.
 *   - dtype describes in and w: KST_F32 (fp32 operands, fp32 arithmetic),
 *     KST_BF16 (bfloat16 operands, fp32 accumulation, fp32 out) or KST_F16 (IEEE
 *     half-precision operands, fp32 accumulation, fp32 out; not in the paper:
 *     the same kernels as KST_BF16 with the other 16-bit multiply).
 *   - Work is enqueued on `stream` and the call returns without waiting for
 *     it.  Arguments are validated on the host before anything is launched;
 *     errors come back as a kst_status, nothing throws or aborts.
 *   - Every data pointer must be 16-byte aligned.
 *   - Legal shapes: B, Cin, Cout, N, n >= 1 and 2N - n >= 1, with every tensor
 *     below 2^31 elements.
 *   - Calls on different streams may run concurrently.
 */
#ifndef KST_H
#define KST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Same definition as the HIP runtime's, so that no HIP header is needed here. */
typedef struct ihipStream_t *hipStream_t;

typedef enum {
    KST_F32 = 0,
    KST_BF16 = 1,
    KST_F16 = 2
} kst_dtype;

typedef enum {
    KST_OK = 0,
    KST_ERR_NULL = 1,       /* a required pointer is NULL                              */
    KST_ERR_SHAPE = 2,      /* a size < 1, 2N - n < 1, or a tensor of 2^31+ elements   */
    KST_ERR_DTYPE = 3,      /* dtype is none of KST_F32, KST_BF16, KST_F16             */
    KST_ERR_WORKSPACE = 4,  /* workspace missing or smaller than kst_workspace_bytes  */
    KST_ERR_HIP = 5,        /* the HIP runtime refused an allocation or a launch      */
    KST_ERR_PATH = 6,       /* unknown kst_path, or a path that cannot run this shape */
    KST_ERR_ALIGN = 7,      /* a data pointer is not 16-byte aligned                  */
    KST_ERR_ACT = 8         /* activation is none of KST_ACT_NONE, _RELU, _TANH       */
} kst_status;

/* Which kernel family kst_forward_seg uses.  AUTO picks DIRECT for small
 * channel counts (bandwidth-bound) and IGEMM (matrix cores) otherwise; of
 * the layers with fewer than 16 output channels it also gives IGEMM those
 * with many input channels that the matrix cores can take with the
 * sub-kernels' taps as rows (a batch of them) or with the reduction split
 * over the chip (one sample).
 * IGEMM_EVEN (for tests and tuning) is IGEMM with one of its launch forms
 * forced: the (tile, channel chunk) list of the layer cut into equal ranges
 * over persistent workgroups, which IGEMM itself takes only where its cost
 * model says it pays.  It exists for KST_F32 layers with Cin, Cout and the
 * input row stride multiples of 4 whose tile fits the kernel; any other
 * layer gets KST_ERR_PATH.  Its workspace differs from IGEMM's: ask
 * kst_workspace_bytes with the same path.
 * IGEMM_PASSES (for tests and measurement) forces a second 16-bit matrix-core
 * kernel: a tile's even and odd output rows in two passes, one pass's rows
 * leaving for memory while the other multiplies.  It exists for 3 x 3 kernels
 * on 64 x 64 maps with 256 input channels, output channels a multiple of 64 and
 * at least 224 tiles of 64 channels x 4 quad rows; any other layer gets
 * KST_ERR_PATH.  AUTO and IGEMM never take it (it measures slower than the
 * kernel they take).  No workspace. */
typedef enum {
    KST_PATH_AUTO = 0,
    KST_PATH_DIRECT = 1,
    KST_PATH_IGEMM = 2,
    KST_PATH_IGEMM_EVEN = 3,
    KST_PATH_IGEMM_PASSES = 4
} kst_path;

/* What kst_forward_seg_epilogue applies to every output element after the bias. */
typedef enum {
    KST_ACT_NONE = 0,       /* v            */
    KST_ACT_RELU = 1,       /* max(v, 0)    */
    KST_ACT_TANH = 2        /* tanh(v)      */
} kst_activation;

int kst_version(void);
const char *kst_status_string(int status);

/* M = 2N - n, the output edge (Section 1).  May be < 1 for illegal shapes. */
int kst_out_size(int N, int n);

/*
 * Shape of sub-kernel p of an n x n kernel (Section 3.2).  p = 2r + s selects
 * the rows of parity r and the columns of parity s: p = 0..3 are the paper's
 * K1 (K00), K2 (K01), K3 (K10), K4 (K11).  Writes Ta = ceil((n-r)/2) rows and
 * Tb = ceil((n-s)/2) columns (either may be 0 for n = 1).  Returns KST_OK, or
 * KST_ERR_SHAPE for n < 1 or p outside 0..3.  Host pointers.
 */
kst_status kst_subkernel_shape(int n, int p, int *Ta, int *Tb);

/*
 * Segregated-weight buffer (the output of kst_segregate_weights).
 *
 * The buffer is the four per-parity tensors W_0..W_3, each contiguous, one
 * after the other; W_p starts kst_segregated_offset(...) elements into it.
 * With t = a*Tb + b the tap index inside sub-kernel p, and
 * W_p(co, ci, a, b) = w[co][ci][2a + r][2b + s]:
 *
 *   KST_F32 :  W_p laid out as [Cin][Ta*Tb][Cout]            (co fastest)
 *   KST_BF16, KST_F16:  W_p laid out as [ceil(Cin/8)][Ta*Tb][Cout][8] (ci mod 8 fastest),
 *              input channels padded with zeros to a multiple of 8.
 *
 * Both put the reduction index next to the output channel the way the matrix
 * cores read it.  kst_segregated_elems is the total element count (of 4 or 2
 * bytes); for KST_F32 it equals Cout*Cin*n*n: segregation is a permutation.
 * Both return 0 for illegal arguments.
 */
size_t kst_segregated_elems(int Cin, int Cout, int n, kst_dtype dtype);
size_t kst_segregated_offset(int Cin, int Cout, int n, int p, kst_dtype dtype);

/*
 * Weight pre-segregation (Section 3.2, the sub-kernel matrices K00..K11).
 * Reads w[Cout][Cin][n][n], writes every element of w_seg in the layout above.
 * Done once per weight tensor.  One kernel launch on `stream`.
 */
kst_status kst_segregate_weights(const void *w, void *w_seg, int Cin, int Cout, int n,
                                 kst_dtype dtype, hipStream_t stream);

/*
 * Bytes of scratch kst_forward_seg needs for this shape and path (0 when it
 * needs none).  The matrix-core path uses it for partial sums when it splits
 * the input-channel reduction across workgroups.
 */
size_t kst_workspace_bytes(int B, int Cin, int Cout, int N, int n, kst_dtype dtype, kst_path path);

/*
 * Segregated forward pass (Section 3.3, Eqs. 7-10), weights already
 * segregated:
 *   out[b][co][2i+r][2j+s] = sum_ci sum_a sum_b' in[b][ci][i+r+a][j+s+b'] * W_p(co,ci,a,b')
 * for every (i, j, r, s) with 2i+r < M and 2j+s < M; the extra row and column
 * the quad sweep would produce for odd M are never written.  ws/ws_bytes:
 * scratch of at least kst_workspace_bytes(...) bytes, 16-byte aligned (may
 * be NULL/0 when that is 0).  Its contents are undefined afterwards.
 */
kst_status kst_forward_seg(const void *in, const void *w_seg, void *out, void *ws, size_t ws_bytes,
                           int B, int Cin, int Cout, int N, int n, kst_dtype dtype, kst_path path,
                           hipStream_t stream);

/*
 * For callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, serving loops with a fixed memory plan, harnesses that forbid hipMalloc.
 * kst_forward_seg with the same kernels, results and statuses, its workspace taken from an
 * array of KST_STATIC_SCRATCH_BYTES that is part of the library's device code (each GPU the
 * library runs on holds one until the process ends) instead of from the caller.  It calls no
 * hipMalloc, hipFree or other allocating routine; the first call on a device looks the array's
 * address up (hipGetSymbolAddress), later calls only launch.  A layer whose path needs more
 * workspace than the array holds gets KST_ERR_WORKSPACE and nothing is launched
 * (kst_workspace_bytes tells beforehand).  All calls on one GPU share that GPU's array: calls
 * that overlap in time on one GPU (different streams, different threads) race on it; calls on
 * one stream are ordered and safe.  The array's contents are undefined between calls.
 */
#define KST_STATIC_SCRATCH_BYTES (64u << 20)
kst_status kst_forward_seg_static(const void *in, const void *w_seg, void *out,
                                  int B, int Cin, int Cout, int N, int n, kst_dtype dtype, kst_path path,
                                  hipStream_t stream);

/*
 * Whole path from un-segregated weights: segregates w into scratch, then runs
 * the segregated forward pass with path AUTO.  Same result as
 * kst_segregate_weights + kst_forward_seg.  The scratch (segregated weights
 * and workspace) is taken from and returned to a stream-ordered memory pool
 * that the library keeps per device (hipMallocFromPoolAsync / hipFreeAsync on
 * `stream`): no host synchronisation, but not usable under stream capture.
 * The pool keeps freed blocks for the next call (at most the largest scratch
 * any call has needed, up to about 0.2 GB) until the process ends.
 */
kst_status kst_forward(const void *in, const void *w, void *out,
                       int B, int Cin, int Cout, int N, int n, kst_dtype dtype, hipStream_t stream);

/*
 * Padding factor P (Section 3.3, Figs. 5-7): the up-sampled (2N-1) x (2N-1)
 * map is framed by P >= 0 zeros on every side before the n x n correlation, so
 * the output edge is kst_out_size_padded(N, n, P) = 2N + 2P - n (it must be
 * >= 1; P = 0 is the unframed operation above).  The segregated method moves the
 * frame to the ORIGINAL input with the reduced factor floor(P / 2); for odd P the
 * four sub-kernels swap roles (K4, K3, K2, K1).  Here the frame is ceil(P / 2)
 * zeros.  The direct kernels supply it themselves (in LDS, or by predicated
 * loads) and for odd P write output (y, x) as element (y + 1, x + 1) of the
 * map the framed input defines, which is that swap of roles: no workspace.
 * The fp32 matrix-core kernel for channel counts that are multiples of 4
 * supplies the frame while it stages its input; the other matrix-core kernels
 * run on a framed copy of the input made in the workspace.  They shift their
 * stores in the same way for odd P, except three
 * 16-bit kernels (maps of 16 to 128 quads a row), which for odd P run into a
 * second workspace buffer one pixel wider on every side, whose interior is
 * then copied to `out` (one extra pass over the output).  Layouts, dtypes, alignment, stream and error behaviour are
 * those of kst_forward_seg / kst_forward; `out` is [B][Cout][2N+2P-n][2N+2P-n]
 * fp32.  kst_workspace_bytes_padded returns 0 for an illegal shape or
 * unsupported path, and for layers whose kernel needs neither copy (the direct
 * path, frames of up to 4 with one or three input channels, any frame with
 * several): then ws may be NULL.
 */
int kst_out_size_padded(int N, int n, int P);
size_t kst_workspace_bytes_padded(int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, kst_path path);
kst_status kst_forward_seg_padded(const void *in, const void *w_seg, void *out, void *ws, size_t ws_bytes,
                                  int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, kst_path path,
                                  hipStream_t stream);
kst_status kst_forward_padded(const void *in, const void *w, void *out,
                              int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, hipStream_t stream);

/*
 * The layer as a generator uses it (not part of the paper's method, whose
 * layers are timed bare; the generators of its Table 3 follow each of them
 * with a bias and a ReLU or, on the last layer, a tanh):
 *     out[b][co][y][x] = act( T[b][co][y][x] + bias[co] )
 * with T the result of kst_forward_seg_padded on the same arguments.  The bias
 * and the activation are applied in fp32 where a kernel stores the final value
 * of an element (for split reductions: in the pass that sums the partial
 * results), so the layer costs no extra pass over `out`.  bias: Cout fp32
 * values in device memory, 4-byte aligned, or NULL for none.  act: see
 * kst_activation (KST_ERR_ACT for anything else).  Everything else -- layouts,
 * P, workspace (kst_workspace_bytes_padded), paths, stream, statuses -- is as
 * for kst_forward_seg_padded; KST_PATH_IGEMM_PASSES takes no epilogue
 * (KST_ERR_PATH).  With bias = NULL and KST_ACT_NONE the call is
 * kst_forward_seg_padded.
 */
kst_status kst_forward_seg_epilogue(const void *in, const void *w_seg, const float *bias, void *out, void *ws,
                                    size_t ws_bytes, int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype,
                                    kst_activation act, kst_path path, hipStream_t stream);

/*
 * Gradients (end of Section 3.3: the segregated method also gives the input and
 * kernel gradients of back-propagation).  g = d(loss)/d(out) is fp32,
 * [B][Cout][M][M] with M = kst_out_size_padded(N, n, P); the results are fp32:
 *   din[b][ci][a][c]  = sum_co sum_u sum_v g[b][co][P+2a-u][P+2c-v] * w[co][ci][u][v]
 *   dw[co][ci][u][v]  = sum_b sum_a sum_c in[b][ci][a][c] * g[b][co][P+2a-u][P+2c-v]
 * over the terms whose g index lies inside the map: exactly the products of the
 * forward pass that involve an original input pixel.  w (un-segregated,
 * [Cout][Cin][n][n]) and in are of type `dtype`.  din [B][Cin][N][N] and dw
 * [Cout][Cin][n][n] are fully overwritten.  ws / ws_bytes: scratch of at least
 * kst_backward_*_workspace_bytes(...): for framed copies as in
 * kst_forward_seg_padded (kernels up to 7 x 7 need none of `in` and no framed
 * result: they visit the unframed positions only; odd P frames g by one pixel),
 * for the zero-framed copy of g the matrix-core kernel-gradient kernel reads,
 * for the partial sums of split reductions (the matrix-core kernels: n <= 5,
 * at least 8 channels on either side, or at least 64 input channels with a few
 * output channels; the other kernel-gradient kernels when they slice the
 * positions), and for the fp32 copy of w or in that the matrix-core kernels
 * read when the operands are 16-bit (widening is exact); it
 * may be 0 (then ws may be NULL).  The byte count depends
 * on the shape only, never on the pointers, as in
 * kst_forward_seg_padded.  Pointers, alignment, stream and statuses as above.
 */
size_t kst_backward_input_workspace_bytes(int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype);
size_t kst_backward_weight_workspace_bytes(int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype);
kst_status kst_backward_input(const void *g, const void *w, void *din, void *ws, size_t ws_bytes,
                              int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, hipStream_t stream);
kst_status kst_backward_weight(const void *in, const void *g, void *dw, void *ws, size_t ws_bytes,
                               int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, hipStream_t stream);

/*
 * The conventional method the paper compares against (Section 1; Eq. 1 on the
 * up-sampled map), kept as the speed-up reference and never tuned: one kernel
 * writes U[B][Cin][2N-1][2N-1] (same dtype as in) including all its zeros,
 * a second computes every output with the full n x n x Cin loop over U.
 * U must hold B*Cin*(2N-1)^2 elements.
 */
kst_status kst_forward_zero_insert(const void *in, const void *w, void *U, void *out,
                                   int B, int Cin, int Cout, int N, int n, kst_dtype dtype,
                                   hipStream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* KST_H */
