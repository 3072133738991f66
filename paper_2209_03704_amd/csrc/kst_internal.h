// Internal declarations shared by the translation units of libkst.so.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stddef.h>
#include <stdint.h>

#include "kst.h"

namespace kst {

// Sub-kernel geometry of Section 3.2: parity r keeps rows r, r+2, ... of an n-row kernel.
__host__ __device__ constexpr int taps_for_parity(int n, int r) { return (n - r + 1) / 2; }
__host__ __device__ constexpr int class_taps(int n, int p)
{
    return taps_for_parity(n, p >> 1) * taps_for_parity(n, p & 1);
}
// Taps of all classes before class p (class-major tap numbering 0..n*n-1).
__host__ __device__ constexpr int class_tap_base(int n, int p)
{
    int s = 0;
    for (int q = 0; q < p; ++q) s += class_taps(n, q);
    return s;
}

// Class of tap T in that numbering.
__host__ __device__ constexpr int tap_class(int n, int T)
{
    int c = 0;
    for (int q = 1; q < 4; ++q)
        if (T >= class_tap_base(n, q) && class_taps(n, q) > 0) c = q;
    return c;
}

// Operand element -> fp32.  bfloat16 operands travel as raw 16-bit patterns (uint16_t), half
// precision ones as half_bits.
struct half_bits {
    uint16_t v;
    half_bits() = default;
    __host__ __device__ explicit half_bits(int bits) : v((uint16_t)bits) {}
};
__device__ inline float to_f32(float v) { return v; }
__device__ inline float to_f32(uint16_t v) { return __uint_as_float((unsigned)v << 16); }
__device__ inline float to_f32(half_bits h) { return (float)__builtin_bit_cast(_Float16, h.v); }

// The two 16-bit operand types share layouts, sizes and kernels.
inline bool is16(kst_dtype dt) { return dt == KST_BF16 || dt == KST_F16; }

// 16-byte aligned streaming store: output lines are written once and never read back by
// the kernel that writes them, so they need not stay in L2 (measured: a map-sized output
// drains at about 6 TB/s this way against 4.5 with plain stores).
typedef float kst_floatx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_streaming4(float *dst, float a, float b, float c, float d)
{
    const kst_floatx4 v = {a, b, c, d};
    __builtin_nontemporal_store(v, reinterpret_cast<kst_floatx4 *>(dst));
}

// Optional epilogue on the store path (not part of the paper's method; the layers of the GAN
// generators its Table 3 lists are followed by a bias and a ReLU or tanh):
// out = act(out + bias[co]).  bias: Cout fp32 values in device memory, or nullptr for none.
struct Epilogue {
    const float *bias;
    int act;             // kst_activation
};
__host__ __device__ inline bool epi_on(const Epilogue &e) { return e.bias != nullptr || e.act != KST_ACT_NONE; }
__device__ __forceinline__ float epi_bias(const Epilogue &e, int co) { return e.bias ? e.bias[co] : 0.0f; }
// One uniform branch (tanh or not); identity and ReLU share a branch-free form: max(v + b, floor)
// with floor = 0 or -infinity.
__device__ __forceinline__ float epi_floor(int act) { return act == KST_ACT_RELU ? 0.0f : -__builtin_inff(); }
__device__ __forceinline__ float epi_apply(float v, float b, int act)
{
    if (act == KST_ACT_TANH) return tanhf(v + b);
    return fmaxf(v + b, epi_floor(act));
}
__device__ __forceinline__ void epi_apply4(float &a, float &b, float &c, float &d, float bias, int act)
{
    if (act == KST_ACT_TANH) {
        a = tanhf(a + bias);
        b = tanhf(b + bias);
        c = tanhf(c + bias);
        d = tanhf(d + bias);
    } else {
        const float lo = epi_floor(act);
        a = fmaxf(a + bias, lo);
        b = fmaxf(b + bias, lo);
        c = fmaxf(c + bias, lo);
        d = fmaxf(d + bias, lo);
    }
}

struct Shape {
    int B, Cin, Cout, N, n;
    int M;    // output edge 2N - n
    int E;    // quad rows/columns: ceil(M / 2)
    int fl;   // floor(n / 2): halo of the input window of one quad
    int Ns;   // elements between consecutive rows of `in` (N unless the caller framed it with a wider stride)
    int frame; // > 0: `in` is the dense [B][Cin][N - 2 frame][N - 2 frame] tensor and the kernel supplies the
               // zero frame of that width itself (only kernels for which *_takes_virtual_frame says so)
    int crop;  // 1: only the interior of the M x M map is wanted -- `out` is the dense [B][Cout][M - 2][M - 2] tensor
               // whose element (y, x) is element (y + 1, x + 1) of the map (an odd padding factor; only kernels for
               // which *_takes_virtual_frame says so)
    Epilogue epi;  // applied where the final value of an element is stored (every forward kernel but the
                   // row-parity-passes one, which must be given an inactive one)
};

inline Shape make_shape(int B, int Cin, int Cout, int N, int n)
{
    Shape s{B, Cin, Cout, N, n, 2 * N - n, (2 * N - n + 1) / 2, n / 2, N, 0, 0, {nullptr, KST_ACT_NONE}};
    return s;
}

// Element offset of W_p inside the segregated buffer, and the total size.
inline size_t seg_cin_padded(int Cin, kst_dtype dt) { return dt != KST_F32 ? (size_t)((Cin + 7) / 8) * 8 : (size_t)Cin; }
inline size_t seg_offset(int Cin, int Cout, int n, int p, kst_dtype dt)
{
    return seg_cin_padded(Cin, dt) * (size_t)Cout * (size_t)class_tap_base(n, p);
}
inline size_t seg_elems(int Cin, int Cout, int n, kst_dtype dt)
{
    return seg_cin_padded(Cin, dt) * (size_t)Cout * (size_t)n * (size_t)n;
}

// Launchers (each enqueues on `stream` and returns the launch status).
hipError_t launch_segregate(const void *w, void *w_seg, int Cin, int Cout, int n, kst_dtype dt,
                            hipStream_t stream);
hipError_t launch_zero_insert(const void *in, const void *w, void *U, float *out, const Shape &s,
                              kst_dtype dt, hipStream_t stream);
// Measurement yardsticks: a loop of matrix-core instructions only, and a streaming copy.
size_t yardstick_mfma_sink_elems();
double yardstick_mfma_flops(kst_dtype dt, int iters);
hipError_t launch_yardstick_mfma(kst_dtype dt, int iters, float *sink, hipStream_t stream);
hipError_t launch_yardstick_copy(const void *src, void *dst, size_t bytes, hipStream_t stream);
// Frame the input by q zeros on every side / drop the outermost rows and columns of an output.
hipError_t launch_frame_input(const void *in, void *in_framed, int B, int Cin, int N, int q, int Ns, kst_dtype dt,
                              hipStream_t stream);
hipError_t launch_crop(const float *wide, float *out, int planes_b, int planes_c, int M, int q, hipStream_t stream);
// dst (fp32) = src (16-bit operands of type dt), element by element.
hipError_t launch_widen(const void *src, float *dst, size_t elems, kst_dtype dt, hipStream_t stream);
// Gradients, P = 0, any shape (plain ALU kernels).  g, din and dw are fp32; w and in are of type dt.
bool backward_generic_takes_frame(const Shape &s);     // these two skip Shape::frame themselves (else: frame must be 0)
hipError_t launch_backward_input_generic(const float *g, const void *w, float *din, const Shape &s, kst_dtype dt,
                                         hipStream_t stream);
size_t backward_weight_generic_workspace_bytes(const Shape &s);    // partial sums when the positions are sliced
hipError_t launch_backward_weight_generic(const void *in, const float *g, float *dw, void *ws, const Shape &s,
                                          kst_dtype dt, hipStream_t stream);
// Input and kernel gradient on the matrix cores (fp32 operands, kernels up to 5 x 5): whether
// they take the shape, the scratch of their split reductions, launch.
bool backward_input_igemm_supported(const Shape &s, kst_dtype dt);
size_t backward_input_igemm_workspace_bytes(const Shape &s);
hipError_t launch_backward_input_igemm(const float *g, const float *w, float *din, void *ws, const Shape &s,
                                       hipStream_t stream);
bool backward_weight_igemm_supported(const Shape &s, kst_dtype dt);
size_t backward_weight_igemm_workspace_bytes(const Shape &s);
// The copy of g that launch_backward_weight_igemm reads: g (edge s.M) framed by *frame zeros on
// every side, its rows *row_stride elements apart (zeros past the frame).
void backward_weight_igemm_g_copy(const Shape &s, int *frame, int *row_stride);
hipError_t launch_backward_weight_igemm(const float *in, const float *g, float *dw, void *ws, const Shape &s,
                                        hipStream_t stream);
// Direct path: any shape.
// Direct kernel for several input channels (one lane per quad and output channel, input staged
// in LDS by channel chunks); dense rows only.
bool direct_multi_supported(const Shape &s);
// True when the direct path reads a padded layer's input in place: s is the framed problem (s.N
// includes the frame of q zeros per side), the kernel is then given Shape::frame = q and the dense tensor.
// crop = 1: and writes only the interior of the map, straight into the caller's tensor (Shape::crop).
bool direct_takes_virtual_frame(const Shape &s, int q, int crop, kst_dtype dt);
hipError_t launch_direct_multi(const void *in, const void *w_seg, float *out, const Shape &s, kst_dtype dt,
                               hipStream_t stream);
hipError_t launch_direct(const void *in, const void *w_seg, float *out, const Shape &s, kst_dtype dt,
                         hipStream_t stream);
// Matrix-core path: whether the kernels can run the shape, scratch they need, launch.
bool igemm_f32_supported(const Shape &s);
bool igemm_f32_takes_row_stride(const Shape &s);   // s.Ns != s.N is only read by the pipelined fp32 kernel
bool igemm_f32_takes_virtual_frame(const Shape &s); // s.frame > 0: that kernel supplies the zero frame while it stages (dense unframed tensor)
bool igemm_bf16_supported(const Shape &s);
bool igemm_bf16_strip_supported(const Shape &s);   // row-strip variant (quad rows of at most 128 quads)
hipError_t launch_igemm_bf16_strip(const void *in, const void *w_seg, float *out, const Shape &s, bool f16,
                                   hipStream_t stream);   // f16: half-precision operands (else bfloat16), here and below
bool igemm_bf16_ring_supported(const Shape &s);    // LDS-ring variant (n = 2, 3; N = 32, 64; whole channel tiles)
hipError_t launch_igemm_bf16_ring(const void *in, const void *w_seg, float *out, const Shape &s, bool f16,
                                  hipStream_t stream);
bool igemm_bf16_wide_supported(const Shape &s);    // persistent wide-tile variant (same shapes, at least ~one tile per CU)
hipError_t launch_igemm_bf16_wide(const void *in, const void *w_seg, float *out, const Shape &s, bool f16,
                                  hipStream_t stream);
bool igemm_bf16_pp_supported(const Shape &s);      // row-parity passes: 3 x 3 kernels, 64 x 64 maps, 256 input channels
hipError_t launch_igemm_bf16_pp(const void *in, const void *w_seg, float *out, const Shape &s, bool f16,
                                hipStream_t stream);
// Layers with at most 64 quad positions in all (one sample of a small map): position blocks of 16.
// Kernel gradient of layers with at most four input channels on large maps (rows of `in` and `g` staged through LDS,
// one partial result per workgroup): whether it applies, how many partial results it writes, the launch.
bool backward_weight_image_apply(const Shape &s);
int backward_weight_image_slices(const Shape &s);
hipError_t launch_backward_weight_image(const void *in, const float *g, float *dst, const Shape &s, kst_dtype dt,
                                        hipStream_t stream);
// ... and the input gradient of such layers with one output channel (din is the unframed tensor).
bool backward_input_image_apply(const Shape &s);
hipError_t launch_backward_input_image(const float *g, const void *w, float *din, const Shape &s, kst_dtype dt,
                                       hipStream_t stream);
// fp32 layers of many input and at most four output channels, batched: the taps of all sub-kernels as the rows of
// one matrix product over the input channels (s.frame, s.crop as for the other kernels that take a virtual frame).
bool tapmajor_f32_supported(const Shape &s);
hipError_t launch_tapmajor_f32(const float *in, const float *w_seg, float *out, const Shape &s, hipStream_t stream);
bool igemm_f32_small_supported(const Shape &s);
size_t igemm_f32_small_workspace_bytes(const Shape &s);
hipError_t launch_igemm_f32_small(const float *in, const float *w_seg, float *out, void *ws, const Shape &s,
                                  hipStream_t stream);
// force_even: take the even-share launch whenever igemm_f32_even_shares_possible, whatever the cost model says.
bool igemm_f32_even_shares_possible(const Shape &s);
size_t igemm_f32_workspace_bytes(const Shape &s, bool force_even = false);
size_t igemm_bf16_workspace_bytes(const Shape &s);
hipError_t launch_igemm_f32(const float *in, const float *w_seg, float *out, void *ws, const Shape &s,
                            bool force_even, hipStream_t stream);
hipError_t launch_igemm_bf16(const void *in, const void *w_seg, float *out, void *ws, const Shape &s, bool f16,
                             hipStream_t stream);

}  // namespace kst
