// C ABI of libkst.so: argument validation, path choice, launches.
#include "kst_internal.h"
#include "kst_yardstick.h"

#include <mutex>

using namespace kst;

namespace {

constexpr size_t kMaxElems = (size_t)1 << 31;

bool dtype_ok(int dt) { return dt == KST_F32 || dt == KST_BF16 || dt == KST_F16; }
size_t elt_bytes(kst_dtype dt) { return is16(dt) ? 2 : 4; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

kst_status check_weight_shape(int Cin, int Cout, int n)
{
    if (Cin < 1 || Cout < 1 || n < 1) return KST_ERR_SHAPE;
    const size_t pad = ((size_t)Cin + 7) / 8 * 8;
    if (n > 46340 || pad * (size_t)Cout >= kMaxElems / ((size_t)n * n)) return KST_ERR_SHAPE;
    return KST_OK;
}

kst_status check_shape(int B, int Cin, int Cout, int N, int n)
{
    if (B < 1 || N < 1) return KST_ERR_SHAPE;
    kst_status st = check_weight_shape(Cin, Cout, n);
    if (st != KST_OK) return st;
    if (N > 32768) return KST_ERR_SHAPE;
    const long long M = 2LL * N - n;
    if (M < 1) return KST_ERR_SHAPE;
    const size_t S = 2 * (size_t)N - 1;
    if ((size_t)B * Cin >= kMaxElems / (S * S)) return KST_ERR_SHAPE;            // up-sampled map (and in)
    if ((size_t)B * Cout >= kMaxElems / ((size_t)(M + 1) * (M + 1))) return KST_ERR_SHAPE;   // out, quad grid
    return KST_OK;
}

// AUTO: the matrix cores pay off once both channel counts can fill MFMA blocks.
kst_path choose_path(const Shape &s, kst_dtype dt)
{
    const bool ok = is16(dt) ? igemm_bf16_supported(s) : igemm_f32_supported(s);
    if (ok && s.Cout >= 16 && s.Cin >= 8) return KST_PATH_IGEMM;
    // One sample of a generator's output layer (many input channels, three output channels): the
    // position-block kernel splits its reduction over the chip, the direct kernel has four tiles.
    if (dt == KST_F32 && s.Cout < 16 && igemm_f32_small_supported(s)) return KST_PATH_IGEMM;
    // ... and a batch of them: the taps of all sub-kernels as the rows of one matrix product.
    if (dt == KST_F32 && tapmajor_f32_supported(s)) return KST_PATH_IGEMM;
    return KST_PATH_DIRECT;
}

kst_status resolve_path(const Shape &s, kst_dtype dt, int path, kst_path *out)
{
    if (path == KST_PATH_AUTO) { *out = choose_path(s, dt); return KST_OK; }
    if (path == KST_PATH_DIRECT) { *out = KST_PATH_DIRECT; return KST_OK; }
    if (path == KST_PATH_IGEMM) {
        const bool ok = is16(dt) ? igemm_bf16_supported(s) : igemm_f32_supported(s);
        if (!ok) return KST_ERR_PATH;
        *out = KST_PATH_IGEMM;
        return KST_OK;
    }
    if (path == KST_PATH_IGEMM_PASSES) {
        if (!is16(dt) || !igemm_bf16_pp_supported(s)) return KST_ERR_PATH;
        *out = KST_PATH_IGEMM_PASSES;
        return KST_OK;
    }
    if (path == KST_PATH_IGEMM_EVEN) {
        if (dt != KST_F32 || !igemm_f32_supported(s) || !igemm_f32_even_shares_possible(s)) return KST_ERR_PATH;
        *out = KST_PATH_IGEMM_EVEN;
        return KST_OK;
    }
    return KST_ERR_PATH;
}

bool on_matrix_cores(kst_path path)
{
    return path == KST_PATH_IGEMM || path == KST_PATH_IGEMM_EVEN || path == KST_PATH_IGEMM_PASSES;
}

size_t workspace_for(const Shape &s, kst_dtype dt, kst_path path)
{
    if (!on_matrix_cores(path) || path == KST_PATH_IGEMM_PASSES) return 0;
    return is16(dt) ? igemm_bf16_workspace_bytes(s) : igemm_f32_workspace_bytes(s, path == KST_PATH_IGEMM_EVEN);
}

// The segregated forward pass on a validated shape (s.Ns may exceed s.N only where
// igemm_f32_takes_row_stride says the kernel that will run reads it).
kst_status run_forward_seg(const void *in, const void *w_seg, void *out, void *ws, size_t ws_bytes, const Shape &s,
                           kst_dtype dtype, int path, hipStream_t stream)
{
    kst_path chosen;
    kst_status st = resolve_path(s, dtype, path, &chosen);
    if (st != KST_OK) return st;
    if (!aligned16(in) || !aligned16(w_seg) || !aligned16(out)) return KST_ERR_ALIGN;
    const size_t need = workspace_for(s, dtype, chosen);
    if (need > 0) {
        if (!ws || ws_bytes < need) return KST_ERR_WORKSPACE;
        if (!aligned16(ws)) return KST_ERR_ALIGN;
    }
    if (s.Ns != s.N && !(on_matrix_cores(chosen) && dtype == KST_F32 && igemm_f32_takes_row_stride(s)))
        return KST_ERR_SHAPE;
    if (chosen == KST_PATH_IGEMM_PASSES && epi_on(s.epi)) return KST_ERR_PATH;    // that kernel stores bare sums only
    hipError_t e;
    if (chosen == KST_PATH_DIRECT)
        e = launch_direct(in, w_seg, (float *)out, s, dtype, stream);
    else if (chosen == KST_PATH_IGEMM_PASSES)
        e = launch_igemm_bf16_pp(in, w_seg, (float *)out, s, dtype == KST_F16, stream);
    else if (is16(dtype))
        e = launch_igemm_bf16(in, w_seg, (float *)out, ws, s, dtype == KST_F16, stream);
    else
        e = launch_igemm_f32((const float *)in, (const float *)w_seg, (float *)out, ws, s,
                             chosen == KST_PATH_IGEMM_EVEN, stream);
    return e == hipSuccess ? KST_OK : KST_ERR_HIP;
}

// Scratch of the entry points that take un-segregated weights (kst_forward, kst_forward_padded):
// a stream-ordered memory pool of the library's own per device, which keeps what is freed
// (release threshold: never) so that call after call re-uses one block instead of mapping and
// unmapping it every time -- with the runtime's default pool a 128 MiB workspace cost about
// 100 us per call.  The pool holds at most the largest scratch any call has asked for.
constexpr int kMaxPoolDevices = 64;
std::mutex pool_mutex;
hipMemPool_t pools[kMaxPoolDevices];
bool pool_tried[kMaxPoolDevices];

hipError_t scratch_alloc(void **ptr, size_t bytes, hipStream_t stream)
{
    int dev = -1;
    hipMemPool_t pool = nullptr;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxPoolDevices) {
        std::lock_guard<std::mutex> lock(pool_mutex);
        if (!pool_tried[dev]) {
            pool_tried[dev] = true;
            hipMemPoolProps props = {};
            props.allocType = hipMemAllocationTypePinned;
            props.handleTypes = hipMemHandleTypeNone;
            props.location.type = hipMemLocationTypeDevice;
            props.location.id = dev;
            hipMemPool_t made = nullptr;
            if (hipMemPoolCreate(&made, &props) == hipSuccess) {
                uint64_t keep = UINT64_MAX;
                if (hipMemPoolSetAttribute(made, hipMemPoolAttrReleaseThreshold, &keep) == hipSuccess)
                    pools[dev] = made;
                else
                    (void)hipMemPoolDestroy(made);
            }
            (void)hipGetLastError();       // a refused pool is no error of the call: the default pool serves
        }
        pool = pools[dev];
    }
    if (pool) return hipMallocFromPoolAsync(ptr, bytes, pool, stream);
    return hipMallocAsync(ptr, bytes, stream);
}

}  // namespace

extern "C" {

int kst_version(void) { return 103; }

const char *kst_status_string(int status)
{
    switch (status) {
        case KST_OK: return "ok";
        case KST_ERR_NULL: return "null pointer";
        case KST_ERR_SHAPE: return "illegal shape";
        case KST_ERR_DTYPE: return "unknown dtype";
        case KST_ERR_WORKSPACE: return "workspace missing or too small";
        case KST_ERR_HIP: return "HIP runtime error";
        case KST_ERR_PATH: return "unknown or unsupported path";
        case KST_ERR_ALIGN: return "pointer not 16-byte aligned";
        case KST_ERR_ACT: return "unknown activation";
        default: return "unknown status";
    }
}

int kst_out_size(int N, int n) { return 2 * N - n; }

kst_status kst_subkernel_shape(int n, int p, int *Ta, int *Tb)
{
    if (!Ta || !Tb) return KST_ERR_NULL;
    if (n < 1 || p < 0 || p > 3) return KST_ERR_SHAPE;
    *Ta = taps_for_parity(n, p >> 1);
    *Tb = taps_for_parity(n, p & 1);
    return KST_OK;
}

size_t kst_segregated_elems(int Cin, int Cout, int n, kst_dtype dtype)
{
    if (!dtype_ok(dtype) || check_weight_shape(Cin, Cout, n) != KST_OK) return 0;
    return seg_elems(Cin, Cout, n, dtype);
}

size_t kst_segregated_offset(int Cin, int Cout, int n, int p, kst_dtype dtype)
{
    if (!dtype_ok(dtype) || check_weight_shape(Cin, Cout, n) != KST_OK || p < 0 || p > 3) return 0;
    return seg_offset(Cin, Cout, n, p, dtype);
}

kst_status kst_segregate_weights(const void *w, void *w_seg, int Cin, int Cout, int n, kst_dtype dtype,
                                 hipStream_t stream)
{
    if (!w || !w_seg) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    kst_status st = check_weight_shape(Cin, Cout, n);
    if (st != KST_OK) return st;
    if (!aligned16(w) || !aligned16(w_seg)) return KST_ERR_ALIGN;
    return launch_segregate(w, w_seg, Cin, Cout, n, dtype, stream) == hipSuccess ? KST_OK : KST_ERR_HIP;
}

size_t kst_workspace_bytes(int B, int Cin, int Cout, int N, int n, kst_dtype dtype, kst_path path)
{
    if (!dtype_ok(dtype) || check_shape(B, Cin, Cout, N, n) != KST_OK) return 0;
    const Shape s = make_shape(B, Cin, Cout, N, n);
    kst_path chosen;
    if (resolve_path(s, dtype, path, &chosen) != KST_OK) return 0;
    return workspace_for(s, dtype, chosen);
}

kst_status kst_forward_seg(const void *in, const void *w_seg, void *out, void *ws, size_t ws_bytes,
                           int B, int Cin, int Cout, int N, int n, kst_dtype dtype, kst_path path,
                           hipStream_t stream)
{
    if (!in || !w_seg || !out) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    kst_status st = check_shape(B, Cin, Cout, N, n);
    if (st != KST_OK) return st;
    return run_forward_seg(in, w_seg, out, ws, ws_bytes, make_shape(B, Cin, Cout, N, n), dtype, path, stream);
}

// ---- the entry point that allocates nothing --------------------------------------------------
}  // extern "C"

// Workspace of kst_forward_seg_static: one array per GPU, part of the loaded code object, held
// until the process ends.  In host code `scratch` is only a handle for hipGetSymbolAddress; the
// kernels get the device address that call returns.
static __device__ __align__(256) unsigned char scratch[KST_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, looked up once

// The current device's copy of `scratch`, or nullptr (with *st set) when it cannot be had.
void *static_scratch(kst_status *st)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        *st = KST_ERR_HIP;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            *st = KST_ERR_HIP;
            return nullptr;
        }
        scratch_ptr[dev] = ptr;
    }
    return scratch_ptr[dev];
}

}  // namespace

extern "C" {

kst_status kst_forward_seg_static(const void *in, const void *w_seg, void *out, int B, int Cin, int Cout, int N, int n,
                                  kst_dtype dtype, kst_path path, hipStream_t stream)
{
    if (!in || !w_seg || !out) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    kst_status st = check_shape(B, Cin, Cout, N, n);
    if (st != KST_OK) return st;
    const Shape s = make_shape(B, Cin, Cout, N, n);
    kst_path chosen;
    st = resolve_path(s, dtype, path, &chosen);
    if (st != KST_OK) return st;
    const size_t need = workspace_for(s, dtype, chosen);
    if (need > (size_t)KST_STATIC_SCRATCH_BYTES) return KST_ERR_WORKSPACE;     // larger than the array: refuse
    void *ws = nullptr;
    if (need) {
        ws = static_scratch(&st);
        if (!ws) return st;
    }
    // The kernels write every workspace word before they read it: nothing has to be cleared
    // between calls, whatever the previous call left there.
    return run_forward_seg(in, w_seg, out, ws, need, s, dtype, chosen, stream);
}

kst_status kst_forward(const void *in, const void *w, void *out, int B, int Cin, int Cout, int N, int n,
                       kst_dtype dtype, hipStream_t stream)
{
    if (!in || !w || !out) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    kst_status st = check_shape(B, Cin, Cout, N, n);
    if (st != KST_OK) return st;
    if (!aligned16(in) || !aligned16(w) || !aligned16(out)) return KST_ERR_ALIGN;
    const Shape s = make_shape(B, Cin, Cout, N, n);
    const kst_path chosen = choose_path(s, dtype);
    const size_t seg_bytes = (seg_elems(Cin, Cout, n, dtype) * elt_bytes(dtype) + 255) & ~(size_t)255;
    const size_t ws_bytes = workspace_for(s, dtype, chosen);
    void *scratch = nullptr;
    if (scratch_alloc(&scratch, seg_bytes + ws_bytes, stream) != hipSuccess) return KST_ERR_HIP;
    void *ws = ws_bytes ? (void *)((char *)scratch + seg_bytes) : nullptr;
    st = kst_segregate_weights(w, scratch, Cin, Cout, n, dtype, stream);
    if (st == KST_OK)
        st = kst_forward_seg(in, scratch, out, ws, ws_bytes, B, Cin, Cout, N, n, dtype, chosen, stream);
    if (hipFreeAsync(scratch, stream) != hipSuccess && st == KST_OK) st = KST_ERR_HIP;
    return st;
}

// ---- padding factor P -------------------------------------------------------------------------
namespace {

struct Framed {
    int q, Nq, M, Mq;                 // frame on the input, framed input edge, output edge, inner output edge
    Shape s;                          // the inner, unframed problem (s.Ns: row stride of the framed copy)
    kst_path chosen;
    size_t in_bytes, wide_bytes;      // workspace parts before the inner kernels' own scratch (256-byte multiples)
};

kst_status framed_plan(int B, int Cin, int Cout, int N, int n, int P, kst_dtype dt, int path, Framed *f)
{
    if (P < 0 || P > 32768 || B < 1 || N < 1 || N > 32768) return KST_ERR_SHAPE;
    f->q = (P + 1) / 2;
    f->Nq = N + 2 * f->q;
    kst_status st = check_shape(B, Cin, Cout, f->Nq, n);        // also bounds the element counts
    if (st != KST_OK) return st;
    f->M = 2 * N + 2 * P - n;
    f->Mq = 2 * f->Nq - n;
    if (f->M < 1) return KST_ERR_SHAPE;
    f->s = make_shape(B, Cin, Cout, f->Nq, n);
    // The pipelined fp32 matrix-core kernel supplies the frame itself while it stages its input
    // rows (tensor rows of whole 16-byte groups): no framed copy.
    Shape in_place = f->s;
    in_place.frame = f->q;
    const bool frame_in_kernel = dt == KST_F32 && igemm_f32_takes_virtual_frame(in_place);
    if (path == KST_PATH_IGEMM_EVEN) {
        if (frame_in_kernel) f->s = in_place;
        else f->s.Ns = (f->Nq + 3) & ~3;                            // the stride that launch form wants of a copy
    }
    st = resolve_path(f->s, dt, path, &f->chosen);
    if (st != KST_OK) return st;
    // (the tap-major kernel of few-output-channel layers reads the tensor as it lies in memory and is
    // planned on its edge, which only the in-place view carries)
    if (path == KST_PATH_AUTO && dt == KST_F32 && f->chosen == KST_PATH_DIRECT && tapmajor_f32_supported(in_place))
        f->chosen = KST_PATH_IGEMM;
    if (on_matrix_cores(f->chosen) && dt == KST_F32) {
        if (frame_in_kernel) {
            f->s = in_place;
        } else if ((f->Nq & 3) != 0) {
            // Otherwise that kernel wants rows of whole 16-byte groups: give the framed copy a row
            // stride rounded up to 4 elements when that is the kernel that will run.
            Shape wide = f->s;
            wide.Ns = (f->Nq + 3) & ~3;
            if (igemm_f32_takes_row_stride(wide)) f->s = wide;
        }
    }
    f->in_bytes = f->s.frame > 0 ? 0 : ((size_t)B * Cin * f->Nq * f->s.Ns * elt_bytes(dt) + 255) & ~(size_t)255;
    f->wide_bytes = (P & 1) ? (((size_t)B * Cout * f->Mq * f->Mq * sizeof(float) + 255) & ~(size_t)255) : 0;
    // The direct kernels supply the zero frame themselves: no framed copy at all; and for an odd
    // padding factor the flat-output kernel writes the interior of the wider map straight to
    // `out` (output row y is row y + 1 of that map: the row parities, hence the sub-kernels,
    // swap roles as in Fig. 7): no wider buffer and no copy of its interior either.
    // The matrix-core kernels whose accumulators go straight to memory (all fp32 ones, the first
    // 16-bit one) store the interior of the wider map directly as well; those that leave through
    // an LDS image of whole rows keep the wider buffer and the copy.
    if ((P & 1) && on_matrix_cores(f->chosen) && f->chosen != KST_PATH_IGEMM_PASSES &&
        (!is16(dt) || !(igemm_bf16_wide_supported(f->s) || igemm_bf16_ring_supported(f->s) ||
                        igemm_bf16_strip_supported(f->s)))) {
        f->s.crop = 1;
        f->wide_bytes = 0;
    }
    if (f->chosen == KST_PATH_DIRECT) {
        if ((P & 1) && direct_takes_virtual_frame(f->s, f->q, 1, dt)) {
            f->s.frame = f->q;
            f->s.crop = 1;
            f->in_bytes = 0;
            f->wide_bytes = 0;
        } else if (direct_takes_virtual_frame(f->s, f->q, 0, dt)) {
            f->s.frame = f->q;
            f->in_bytes = 0;
        }
    }
    return KST_OK;
}

}  // namespace

int kst_out_size_padded(int N, int n, int P) { return 2 * N + 2 * P - n; }

size_t kst_workspace_bytes_padded(int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, kst_path path)
{
    if (!dtype_ok(dtype)) return 0;
    if (P == 0) return kst_workspace_bytes(B, Cin, Cout, N, n, dtype, path);
    Framed f;
    if (framed_plan(B, Cin, Cout, N, n, P, dtype, path, &f) != KST_OK) return 0;
    return f.in_bytes + f.wide_bytes + workspace_for(f.s, dtype, f.chosen);
}

}  // extern "C"

namespace {

// The segregated forward pass for any padding factor, with an optional epilogue at the stores
// that write final values (the copy that crops an odd padding factor's wider map moves them on unchanged).
kst_status forward_seg_padded_impl(const void *in, const void *w_seg, void *out, void *ws, size_t ws_bytes, int B, int Cin,
                                   int Cout, int N, int n, int P, kst_dtype dtype, int path, const Epilogue &epi,
                                   hipStream_t stream)
{
    if (!in || !w_seg || !out) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    if (P == 0) {
        kst_status st0 = check_shape(B, Cin, Cout, N, n);
        if (st0 != KST_OK) return st0;
        Shape s0 = make_shape(B, Cin, Cout, N, n);
        s0.epi = epi;
        return run_forward_seg(in, w_seg, out, ws, ws_bytes, s0, dtype, path, stream);
    }
    Framed f;
    kst_status st = framed_plan(B, Cin, Cout, N, n, P, dtype, path, &f);
    if (st != KST_OK) return st;
    f.s.epi = epi;
    if (!aligned16(in) || !aligned16(w_seg) || !aligned16(out)) return KST_ERR_ALIGN;
    const size_t inner = workspace_for(f.s, dtype, f.chosen);
    const size_t need = f.in_bytes + f.wide_bytes + inner;
    if (need > 0) {
        if (!ws || ws_bytes < need) return KST_ERR_WORKSPACE;
        if (!aligned16(ws)) return KST_ERR_ALIGN;
    }
    char *base = (char *)ws;
    void *in_framed = base;
    float *wide = f.wide_bytes ? (float *)(base + f.in_bytes) : nullptr;
    void *inner_ws = inner ? (void *)(base + f.in_bytes + f.wide_bytes) : nullptr;
    if (f.s.frame == 0) {
        if (launch_frame_input(in, in_framed, B, Cin, N, f.q, f.s.Ns, dtype, stream) != hipSuccess) return KST_ERR_HIP;
    } else {
        in_framed = const_cast<void *>(in);
    }
    st = run_forward_seg(in_framed, w_seg, wide ? (void *)wide : out, inner_ws, inner, f.s, dtype, f.chosen, stream);
    if (st != KST_OK) return st;
    if (wide && launch_crop(wide, (float *)out, B, Cout, f.M, 1, stream) != hipSuccess) return KST_ERR_HIP;
    return KST_OK;
}

}  // namespace

extern "C" {

kst_status kst_forward_seg_padded(const void *in, const void *w_seg, void *out, void *ws, size_t ws_bytes,
                                  int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, kst_path path,
                                  hipStream_t stream)
{
    const Epilogue none = {nullptr, KST_ACT_NONE};
    return forward_seg_padded_impl(in, w_seg, out, ws, ws_bytes, B, Cin, Cout, N, n, P, dtype, path, none, stream);
}

kst_status kst_forward_seg_epilogue(const void *in, const void *w_seg, const float *bias, void *out, void *ws,
                                    size_t ws_bytes, int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype,
                                    kst_activation act, kst_path path, hipStream_t stream)
{
    if (act != KST_ACT_NONE && act != KST_ACT_RELU && act != KST_ACT_TANH) return KST_ERR_ACT;
    if (bias && (reinterpret_cast<uintptr_t>(bias) & 3u) != 0) return KST_ERR_ALIGN;
    const Epilogue epi = {bias, (int)act};
    return forward_seg_padded_impl(in, w_seg, out, ws, ws_bytes, B, Cin, Cout, N, n, P, dtype, path, epi, stream);
}

kst_status kst_forward_padded(const void *in, const void *w, void *out, int B, int Cin, int Cout, int N, int n, int P,
                              kst_dtype dtype, hipStream_t stream)
{
    if (P == 0) return kst_forward(in, w, out, B, Cin, Cout, N, n, dtype, stream);
    if (!in || !w || !out) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    Framed f;
    kst_status st = framed_plan(B, Cin, Cout, N, n, P, dtype, KST_PATH_AUTO, &f);
    if (st != KST_OK) return st;
    if (!aligned16(in) || !aligned16(w) || !aligned16(out)) return KST_ERR_ALIGN;
    const size_t seg_bytes = (seg_elems(Cin, Cout, n, dtype) * elt_bytes(dtype) + 255) & ~(size_t)255;
    const size_t ws_bytes = f.in_bytes + f.wide_bytes + workspace_for(f.s, dtype, f.chosen);   // may be 0
    void *scratch = nullptr;
    if (scratch_alloc(&scratch, seg_bytes + ws_bytes, stream) != hipSuccess) return KST_ERR_HIP;
    st = kst_segregate_weights(w, scratch, Cin, Cout, n, dtype, stream);
    if (st == KST_OK)
        st = kst_forward_seg_padded(in, scratch, out, ws_bytes ? (char *)scratch + seg_bytes : nullptr, ws_bytes, B, Cin,
                                    Cout, N, n, P, dtype, KST_PATH_AUTO, stream);
    if (hipFreeAsync(scratch, stream) != hipSuccess && st == KST_OK) st = KST_ERR_HIP;
    return st;
}

// ---- gradients --------------------------------------------------------------------------------
namespace {

// Workspace of the gradient entry points: for P > 0 the unframed kernels run on framed copies.
//   input gradient:  [g framed by one zero (odd P)] [din of the framed input] [partial sums of the
//                    matrix-core kernel's split reduction]
//   kernel gradient: [input framed by q] [g framed by one zero (odd P)] [partial sums, as above]
struct GradPlan {
    int q, Nq, M, Mq;
    Shape s;                          // the problem on the framed input map (what the plain kernels see)
    Shape si;                         // the same with frame = q: the matrix-core kernels work on the unframed
                                      // positions only (din without the frame; in read as it lies in memory)
    size_t g_bytes, din_bytes, in_bytes;
    size_t split_bytes, wsplit_bytes; // input / kernel gradient on the matrix cores: partial sums
    size_t gw_bytes;                  // kernel gradient on the matrix cores: its framed copy of g (replaces g_bytes)
    int gw_frame, gw_stride;          // frame on the caller's g and row stride of that copy
    bool plain_unframed;              // the other kernels work on the unframed positions too (kernels up to 7 x 7)
    bool din_cores, dw_cores;         // the gradient runs on the matrix cores (fp32 kernels; 16-bit operands are
                                      // widened to fp32 first, which is exact)
    size_t wconv_bytes, xconv_bytes;  // fp32 copies of w (input gradient) and of in (kernel gradient) for that
};

kst_status grad_plan(int B, int Cin, int Cout, int N, int n, int P, kst_dtype dt, GradPlan *f)
{
    if (P < 0 || P > 32768 || B < 1 || N < 1 || N > 32768) return KST_ERR_SHAPE;
    f->q = (P + 1) / 2;
    f->Nq = N + 2 * f->q;
    kst_status st = check_shape(B, Cin, Cout, f->Nq, n);
    if (st != KST_OK) return st;
    f->M = 2 * N + 2 * P - n;
    f->Mq = 2 * f->Nq - n;
    if (f->M < 1) return KST_ERR_SHAPE;
    f->s = make_shape(B, Cin, Cout, f->Nq, n);
    f->g_bytes = (P & 1) ? (((size_t)B * Cout * f->Mq * f->Mq * sizeof(float) + 255) & ~(size_t)255) : 0;
    f->din_bytes = P ? (((size_t)B * Cin * f->Nq * f->Nq * sizeof(float) + 255) & ~(size_t)255) : 0;
    f->in_bytes = P ? (((size_t)B * Cin * f->Nq * f->Nq * elt_bytes(dt) + 255) & ~(size_t)255) : 0;
    f->si = f->s;
    f->si.frame = f->q;
    f->split_bytes = 0;
    f->plain_unframed = backward_generic_takes_frame(f->si);
    f->din_cores = backward_input_igemm_supported(f->si, KST_F32);
    f->dw_cores = backward_weight_igemm_supported(f->si, KST_F32);
    f->wconv_bytes = is16(dt) && f->din_cores ? (((size_t)Cout * Cin * n * n * sizeof(float) + 255) & ~(size_t)255) : 0;
    f->xconv_bytes = is16(dt) && f->dw_cores ? (((size_t)B * Cin * N * N * sizeof(float) + 255) & ~(size_t)255) : 0;
    if (f->din_cores) {
        f->split_bytes = backward_input_igemm_workspace_bytes(f->si);
        f->din_bytes = 0;                              // written in place, frame never computed
    } else if (f->plain_unframed) {
        f->din_bytes = 0;
    }
    if (f->plain_unframed) f->in_bytes = 0;            // `in` read as it lies in memory
    f->wsplit_bytes = f->dw_cores
                          ? backward_weight_igemm_workspace_bytes(f->si)
                          : backward_weight_generic_workspace_bytes(f->plain_unframed ? f->si : f->s);
    f->gw_bytes = 0;
    f->gw_frame = f->gw_stride = 0;
    if (f->dw_cores) {
        int frame, stride;
        backward_weight_igemm_g_copy(f->si, &frame, &stride);
        f->gw_frame = frame + (P & 1);                 // on top of the odd padding factor's one-pixel frame
        f->gw_stride = stride;
        const size_t rows = (size_t)f->M + 2 * (size_t)f->gw_frame;
        f->gw_bytes = ((size_t)B * Cout * rows * stride * sizeof(float) + 255) & ~(size_t)255;
    }
    return KST_OK;
}

}  // namespace

size_t kst_backward_input_workspace_bytes(int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype)
{
    GradPlan f;
    if (!dtype_ok(dtype) || grad_plan(B, Cin, Cout, N, n, P, dtype, &f) != KST_OK) return 0;
    return f.g_bytes + f.din_bytes + f.split_bytes + f.wconv_bytes;
}

size_t kst_backward_weight_workspace_bytes(int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype)
{
    GradPlan f;
    if (!dtype_ok(dtype) || grad_plan(B, Cin, Cout, N, n, P, dtype, &f) != KST_OK) return 0;
    return f.dw_cores ? f.gw_bytes + f.wsplit_bytes + f.xconv_bytes : f.in_bytes + f.g_bytes + f.wsplit_bytes;
}

kst_status kst_backward_input(const void *g, const void *w, void *din, void *ws, size_t ws_bytes,
                              int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, hipStream_t stream)
{
    if (!g || !w || !din) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    GradPlan f;
    kst_status st = grad_plan(B, Cin, Cout, N, n, P, dtype, &f);
    if (st != KST_OK) return st;
    if (!aligned16(g) || !aligned16(w) || !aligned16(din)) return KST_ERR_ALIGN;
    const size_t need = f.g_bytes + f.din_bytes + f.split_bytes + f.wconv_bytes;
    if (need) {
        if (!ws || ws_bytes < need) return KST_ERR_WORKSPACE;
        if (!aligned16(ws)) return KST_ERR_ALIGN;
    }
    const float *g_in = (const float *)g;
    float *d_out = (float *)din;
    if (f.g_bytes) {          // odd P: the forward dropped the outermost ring of the wider output
        if (launch_frame_input(g, ws, B, Cout, f.M, 1, f.Mq, KST_F32, stream) != hipSuccess) return KST_ERR_HIP;
        g_in = (const float *)ws;
    }
    if (f.din_cores) {
        // the matrix-core kernels compute the unframed positions only, straight into din
        void *split_ws = f.split_bytes ? (char *)ws + f.g_bytes : nullptr;
        const float *w32 = (const float *)w;
        if (f.wconv_bytes) {
            float *wc = (float *)((char *)ws + f.g_bytes + f.split_bytes);
            if (launch_widen(w, wc, (size_t)Cout * Cin * n * n, dtype, stream) != hipSuccess) return KST_ERR_HIP;
            w32 = wc;
        }
        return launch_backward_input_igemm(g_in, w32, (float *)din, split_ws, f.si, stream) == hipSuccess
                   ? KST_OK
                   : KST_ERR_HIP;
    }
    if (f.plain_unframed)
        return launch_backward_input_generic(g_in, w, d_out, f.si, dtype, stream) == hipSuccess ? KST_OK : KST_ERR_HIP;
    if (P) d_out = (float *)((char *)ws + f.g_bytes);
    if (launch_backward_input_generic(g_in, w, d_out, f.s, dtype, stream) != hipSuccess) return KST_ERR_HIP;
    if (P && launch_crop(d_out, (float *)din, B, Cin, N, f.q, stream) != hipSuccess) return KST_ERR_HIP;
    return KST_OK;
}

kst_status kst_backward_weight(const void *in, const void *g, void *dw, void *ws, size_t ws_bytes,
                               int B, int Cin, int Cout, int N, int n, int P, kst_dtype dtype, hipStream_t stream)
{
    if (!in || !g || !dw) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    GradPlan f;
    kst_status st = grad_plan(B, Cin, Cout, N, n, P, dtype, &f);
    if (st != KST_OK) return st;
    if (!aligned16(in) || !aligned16(g) || !aligned16(dw)) return KST_ERR_ALIGN;
    const bool cores = f.dw_cores;
    const size_t g_copy = cores ? f.gw_bytes : f.g_bytes;
    const size_t in_copy = cores ? 0 : f.in_bytes;     // the matrix-core kernel reads `in` as it lies in memory
    const size_t need = in_copy + g_copy + f.wsplit_bytes + (cores ? f.xconv_bytes : 0);
    if (need) {
        if (!ws || ws_bytes < need) return KST_ERR_WORKSPACE;
        if (!aligned16(ws)) return KST_ERR_ALIGN;
    }
    const void *x_in = in;
    const float *g_in = (const float *)g;
    if (P && !cores && !f.plain_unframed) {
        if (launch_frame_input(in, ws, B, Cin, N, f.q, f.Nq, dtype, stream) != hipSuccess) return KST_ERR_HIP;
        x_in = ws;
    }
    void *gw = (char *)ws + in_copy;
    void *partial_ws = f.wsplit_bytes ? (char *)ws + in_copy + g_copy : nullptr;
    if (cores) {
        if (f.xconv_bytes) {
            float *xc = (float *)((char *)ws + in_copy + g_copy + f.wsplit_bytes);
            if (launch_widen(in, xc, (size_t)B * Cin * N * N, dtype, stream) != hipSuccess) return KST_ERR_HIP;
            x_in = xc;
        }
        // g framed once for the odd padding factor and for the kernel's own bounds-free reads
        if (launch_frame_input(g, gw, B, Cout, f.M, f.gw_frame, f.gw_stride, KST_F32, stream) != hipSuccess)
            return KST_ERR_HIP;
        return launch_backward_weight_igemm((const float *)x_in, (const float *)gw, (float *)dw, partial_ws, f.si, stream) ==
                       hipSuccess
                   ? KST_OK
                   : KST_ERR_HIP;
    }
    if (f.g_bytes) {
        if (launch_frame_input(g, gw, B, Cout, f.M, 1, f.Mq, KST_F32, stream) != hipSuccess) return KST_ERR_HIP;
        g_in = (const float *)gw;
    }
    return launch_backward_weight_generic(x_in, g_in, (float *)dw, partial_ws, f.plain_unframed ? f.si : f.s, dtype,
                                          stream) == hipSuccess
               ? KST_OK
               : KST_ERR_HIP;
}

kst_status kst_forward_zero_insert(const void *in, const void *w, void *U, void *out, int B, int Cin, int Cout,
                                   int N, int n, kst_dtype dtype, hipStream_t stream)
{
    if (!in || !w || !U || !out) return KST_ERR_NULL;
    if (!dtype_ok(dtype)) return KST_ERR_DTYPE;
    kst_status st = check_shape(B, Cin, Cout, N, n);
    if (st != KST_OK) return st;
    if (!aligned16(in) || !aligned16(w) || !aligned16(U) || !aligned16(out)) return KST_ERR_ALIGN;
    const Shape s = make_shape(B, Cin, Cout, N, n);
    return launch_zero_insert(in, w, U, (float *)out, s, dtype, stream) == hipSuccess ? KST_OK : KST_ERR_HIP;
}

size_t kst_yardstick_mfma_sink_elems(void) { return yardstick_mfma_sink_elems(); }

double kst_yardstick_mfma_flops(kst_dtype dtype, int iters)
{
    if ((dtype != KST_F32 && dtype != KST_BF16) || iters < 1) return 0.0;
    return yardstick_mfma_flops(dtype, iters);
}

kst_status kst_yardstick_mfma(kst_dtype dtype, int iters, float *sink, size_t sink_elems, hipStream_t stream)
{
    if (!sink) return KST_ERR_NULL;
    if (dtype != KST_F32 && dtype != KST_BF16) return KST_ERR_DTYPE;
    if (iters < 1 || iters > (1 << 22)) return KST_ERR_SHAPE;
    if (sink_elems < yardstick_mfma_sink_elems()) return KST_ERR_WORKSPACE;
    return launch_yardstick_mfma(dtype, iters, sink, stream) == hipSuccess ? KST_OK : KST_ERR_HIP;
}

kst_status kst_yardstick_copy(const void *src, void *dst, size_t bytes, hipStream_t stream)
{
    if (!src || !dst) return KST_ERR_NULL;
    if (bytes % 16 != 0) return KST_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return KST_ERR_ALIGN;
    return launch_yardstick_copy(src, dst, bytes, stream) == hipSuccess ? KST_OK : KST_ERR_HIP;
}

}  // extern "C"
