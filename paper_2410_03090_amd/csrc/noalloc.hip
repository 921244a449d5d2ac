// uncomp_head_entropy_noalloc: the truncated matrix entropy for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels as
// uncomp_head_entropy; the partial second-moment sums that call keeps in the context's workspace live here in
// a fixed array inside the library's code object.
#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "common.h"

namespace {

// Partial sums of at most 512 (matrix, token chunk) pairs: 512 * (128*128 + 128) floats.  Every GPU the
// library runs on holds its own copy of this array from the moment the code object is loaded until the
// process ends.
constexpr size_t kScratchBytes = (size_t)512 * (uncomp::kD * uncomp::kD + uncomp::kD) * sizeof(float) + 4096;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
struct DeviceState {
    bool ready = false;
    char* ptr = nullptr;         // device address of `scratch` on this device (the array's name is no address on the host)
};
DeviceState g_state[kMaxDevices];
std::mutex g_mutex;
thread_local char g_err[256] = "";

uncomp_status fail(uncomp_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

}  // namespace

namespace uncomp {
const char* noalloc_last_error() { return g_err[0] != 0 ? g_err : "null context"; }
}  // namespace uncomp

extern "C" uncomp_status uncomp_head_entropy_noalloc(const void* X, uncomp_dtype dtype, int n_mat, int N, int D,
                                                     int64_t mat_stride, int64_t ldx, int k_trunc, unsigned flags,
                                                     float* entropy_out, float* eig_out, void* stream) {
    using namespace uncomp;
    if (X == nullptr || entropy_out == nullptr) return fail(UNCOMP_ERR_INVALID_ARG, "head_entropy_noalloc: null pointer");
    if (n_mat <= 0 || N <= 0) return fail(UNCOMP_ERR_INVALID_ARG, "head_entropy_noalloc: n_mat and N must be positive");
    if (dtype != UNCOMP_BF16 && dtype != UNCOMP_F32) return fail(UNCOMP_ERR_UNSUPPORTED, "head_entropy_noalloc: dtype");
    if (D != kD) return fail(UNCOMP_ERR_UNSUPPORTED, "head_entropy_noalloc: D must be 128");
    if (k_trunc < 1) return fail(UNCOMP_ERR_UNSUPPORTED, "head_entropy_noalloc: k_trunc must be >= 1");
    if (flags & ~(UNCOMP_CENTER | UNCOMP_TRUNC_RENORM | UNCOMP_LAYER_DELTA_INCREASE))
        return fail(UNCOMP_ERR_UNSUPPORTED, "head_entropy_noalloc: unknown flag bits");
    if (ldx < D || (ldx & 7) || (mat_stride & 7) || mat_stride < 0 || (reinterpret_cast<uintptr_t>(X) & 15u))
        return fail(UNCOMP_ERR_INVALID_ARG,
                    "head_entropy_noalloc: strides must be multiples of 8 elements, ldx >= D, X 16-byte aligned");
    // the partial sums must fit the fixed array: fewer, longer token chunks if need be, at most 512 matrices
    const EntropyPlan p = plan_entropy(n_mat, N, kScratchBytes);
    if (p.bytes > kScratchBytes)
        return fail(UNCOMP_ERR_WORKSPACE,
                    "head_entropy_noalloc: %d matrices need %zu bytes of partial sums, the fixed array holds %zu "
                    "(at most 512 matrices per call)", n_mat, p.bytes, kScratchBytes);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(UNCOMP_ERR_HIP, "head_entropy_noalloc: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(UNCOMP_ERR_UNSUPPORTED, "head_entropy_noalloc: device index %d", dev);
    char* ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState& st = g_state[dev];
        if (!st.ready) {
            // once per device, with that device current: where this device keeps its copy of the array, and
            // the LDS limit of the Gram kernel
            void* sym = nullptr;
            e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
            if (e != hipSuccess || sym == nullptr)
                return fail(UNCOMP_ERR_HIP, "head_entropy_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
            e = init_gram_kernels();
            if (e != hipSuccess) return fail(UNCOMP_ERR_HIP, "head_entropy_noalloc: kernel set-up: %s", hipGetErrorString(e));
            st.ptr = static_cast<char*>(sym);
            st.ready = true;
        }
        ws = st.ptr;
    }
    const Env env{static_cast<hipStream_t>(stream), nullptr, false};
    e = launch_gram(X, dtype, n_mat, N, mat_stride, ldx, p, ws, env);
    if (e != hipSuccess) return fail(UNCOMP_ERR_HIP, "head_entropy_noalloc: gram launch: %s", hipGetErrorString(e));
    e = launch_tridiag_entropy(n_mat, N, k_trunc, flags, p, ws, entropy_out, eig_out, env);
    if (e != hipSuccess) return fail(UNCOMP_ERR_HIP, "head_entropy_noalloc: eigen launch: %s", hipGetErrorString(e));
    return UNCOMP_OK;
}
