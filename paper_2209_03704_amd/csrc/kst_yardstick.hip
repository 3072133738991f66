// Yardsticks for the roofline figures: what this chip sustains with nothing in the way.
//
//  * mfma_rate_kernel: a loop of nothing but matrix-core instructions of the shape the
//    matrix-core paths use (v_mfma_f32_32x32x2f32, v_mfma_f32_32x32x16_bf16), four independent
//    accumulator sets per wave so that consecutive instructions never wait on each other,
//    two waves per SIMD on every CU.
//  * stream_copy_kernel: 16-byte loads and streaming 16-byte stores over a flat buffer.
//
// Neither takes part in the method; bench.py prints their rates next to the published peaks.
#include "kst_internal.h"

namespace kst {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int Y_THREADS = 256;      // four waves: one per SIMD
constexpr int Y_WG_PER_CU = 2;
constexpr int Y_SETS = 4;           // independent accumulator sets per wave
constexpr int Y_CUS = 256;

template <bool BF16>
__global__ __launch_bounds__(Y_THREADS) void mfma_rate_kernel(float *sink, int iters) {
    const int lane = threadIdx.x & 63;
    f32x16 acc[Y_SETS];
    for (int k = 0; k < Y_SETS; ++k)
        for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;
    // Operands of ordinary magnitude and mixed sign (all-zero operands would draw less power
    // than real data and flatter the clock).
    const float av = 0.001f * static_cast<float>((lane % 13) - 6);
    const float bv = (lane & 1) ? -0.75f : 0.5f;
    if constexpr (BF16) {
        bf16x8 a, b;
        for (int e = 0; e < 8; ++e) {
            a[e] = static_cast<__bf16>(av * static_cast<float>(e + 1));
            b[e] = static_cast<__bf16>(bv);
        }
        for (int it = 0; it < iters; ++it)
            for (int k = 0; k < Y_SETS; ++k)
                acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
    } else {
        for (int it = 0; it < iters; ++it)
            for (int k = 0; k < Y_SETS; ++k)
                acc[k] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[k], 0, 0, 0);
    }
    float total = 0.f;
    for (int k = 0; k < Y_SETS; ++k)
        for (int e = 0; e < 16; ++e) total += acc[k][e];
    sink[static_cast<size_t>(blockIdx.x) * Y_THREADS + threadIdx.x] = total;
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const f32x4 *__restrict__ src,
                                                          f32x4 *__restrict__ dst, size_t n4) {
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n4; i += stride)
        __builtin_nontemporal_store(src[i], dst + i);
}

}  // namespace

size_t yardstick_mfma_sink_elems() { return static_cast<size_t>(Y_CUS) * Y_WG_PER_CU * Y_THREADS; }

double yardstick_mfma_flops(kst_dtype dt, int iters) {
    const double per_mfma = dt == KST_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    const double waves = static_cast<double>(Y_CUS) * Y_WG_PER_CU * (Y_THREADS / 64);
    return per_mfma * Y_SETS * static_cast<double>(iters) * waves;
}

hipError_t launch_yardstick_mfma(kst_dtype dt, int iters, float *sink, hipStream_t s) {
    const dim3 grid(Y_CUS * Y_WG_PER_CU), block(Y_THREADS);
    if (dt == KST_BF16)
        mfma_rate_kernel<true><<<grid, block, 0, s>>>(sink, iters);
    else
        mfma_rate_kernel<false><<<grid, block, 0, s>>>(sink, iters);
    return hipGetLastError();
}

hipError_t launch_yardstick_copy(const void *src, void *dst, size_t bytes, hipStream_t s) {
    const size_t n4 = bytes / 16;
    if (n4 == 0) return hipSuccess;
    const size_t want = (n4 + 255) / 256;
    const unsigned grid = static_cast<unsigned>(want < 256u * 16u ? want : 256u * 16u);
    stream_copy_kernel<<<dim3(grid), dim3(256), 0, s>>>(static_cast<const f32x4 *>(src),
                                                        static_cast<f32x4 *>(dst), n4);
    return hipGetLastError();
}

}  // namespace kst
