// C interface of libuncomp: argument checks, workspace carving and kernel launches.
// Every entry point validates on the host, launches on the caller's stream and returns a
// status; nothing here synchronises or allocates after uncomp_create.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "common.h"

using namespace uncomp;

namespace {

uncomp_status fail(uncomp_ctx* ctx, uncomp_status st, const char* fmt, ...) {
    if (ctx != nullptr) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return st;
}

uncomp_status hip_fail(uncomp_ctx* ctx, hipError_t e, const char* what) {
    return fail(ctx, UNCOMP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr size_t kDefaultWorkspace = 64ull << 20;
constexpr size_t kBudgetScratch = 4096 * sizeof(double);

}  // namespace

extern "C" {

uncomp_status uncomp_create(uncomp_ctx** ctx_out, int device, size_t workspace_bytes) {
    if (ctx_out == nullptr) return UNCOMP_ERR_INVALID_ARG;
    *ctx_out = nullptr;
    int n_dev = 0;
    hipError_t e = hipGetDeviceCount(&n_dev);
    if (e != hipSuccess || device < 0 || device >= n_dev) return UNCOMP_ERR_INVALID_ARG;
    uncomp_ctx* ctx = new (std::nothrow) uncomp_ctx();
    if (ctx == nullptr) return UNCOMP_ERR_HIP;
    ctx->device = device;
    ctx->err[0] = 0;
    ctx->ws = nullptr;
    ctx->ws_bytes = workspace_bytes == 0 ? kDefaultWorkspace : align_up(workspace_bytes, 256);
    if (ctx->ws_bytes < kBudgetScratch) ctx->ws_bytes = kBudgetScratch;
    int prev = 0;
    (void)hipGetDevice(&prev);
    e = hipSetDevice(device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
    if (e == hipSuccess) {
        ctx->num_cu = prop.multiProcessorCount;
        e = hipMalloc(reinterpret_cast<void**>(&ctx->ws), ctx->ws_bytes);
    }
    // kernels with more than 64 KiB of dynamic LDS get their limit raised here, not in the hot calls
    if (e == hipSuccess) e = init_gram_kernels();
    if (e == hipSuccess) e = init_score_kernels();
    if (e == hipSuccess) e = init_select_kernels();
    if (e == hipSuccess) e = init_jacobi_kernels();
    if (e == hipSuccess) e = init_decode_kernels();
    if (e == hipSuccess) e = init_subspace_kernels();
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming);
    (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
        if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
        if (ctx->side) (void)hipStreamDestroy(ctx->side);
        if (ctx->ws) (void)hipFree(ctx->ws);
        delete ctx;
        return UNCOMP_ERR_HIP;
    }
    *ctx_out = ctx;
    return UNCOMP_OK;
}

uncomp_status uncomp_destroy(uncomp_ctx* ctx) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    hipError_t e = hipSuccess;
    if (ctx->side != nullptr) {
        (void)hipStreamSynchronize(ctx->side);
        (void)hipStreamDestroy(ctx->side);
    }
    if (ctx->ev_fork != nullptr) (void)hipEventDestroy(ctx->ev_fork);
    if (ctx->ev_join != nullptr) (void)hipEventDestroy(ctx->ev_join);
    if (ctx->ws != nullptr) e = hipFree(ctx->ws);
    for (int i = 0; i < ctx->prof.n_events; ++i) {
        (void)hipEventDestroy(ctx->prof.start[i]);
        (void)hipEventDestroy(ctx->prof.stop[i]);
    }
    delete ctx;
    return e == hipSuccess ? UNCOMP_OK : UNCOMP_ERR_HIP;
}

size_t uncomp_workspace_bytes(int n_mat, int N, int D, int B, int H, int G, int w) {
    (void)D;
    // three regions that may be live at once in overlap mode: budgets | entropy | score
    size_t need = kBudgetScratch;
    if (n_mat > 0 && N > 0) need += plan_entropy(n_mat, N).bytes;
    if (B > 0 && H > 0 && G > 0 && N > 0 && w > 0 && w < N) need += plan_score(B, H, G, N, w).bytes;
    return need;
}

uncomp_status uncomp_profile(uncomp_ctx* ctx, int on) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (on != 0 && ctx->prof.n_events < Profiler::kMax) {
        // every event pair a profiled region may use is created here, outside any timed call
        int prev = 0;
        (void)hipGetDevice(&prev);
        hipError_t e = hipSetDevice(ctx->device);
        while (e == hipSuccess && ctx->prof.n_events < Profiler::kMax) {
            const int i = ctx->prof.n_events;
            e = hipEventCreate(&ctx->prof.start[i]);
            if (e == hipSuccess) {
                e = hipEventCreate(&ctx->prof.stop[i]);
                if (e != hipSuccess) (void)hipEventDestroy(ctx->prof.start[i]);
            }
            if (e == hipSuccess) ctx->prof.n_events = i + 1;
        }
        (void)hipSetDevice(prev);
        if (e != hipSuccess) return hip_fail(ctx, e, "profile: hipEventCreate");
    }
    ctx->prof.on = on != 0;
    ctx->prof.n = 0;
    return UNCOMP_OK;
}

uncomp_status uncomp_set_overlap(uncomp_ctx* ctx, int on) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    ctx->overlap = on != 0;
    return UNCOMP_OK;
}

uncomp_status uncomp_join(uncomp_ctx* ctx, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (!ctx->side_pending) return UNCOMP_OK;
    hipError_t e = hipEventRecord(ctx->ev_join, ctx->side);
    if (e == hipSuccess) e = hipStreamWaitEvent(static_cast<hipStream_t>(stream), ctx->ev_join, 0);
    if (e != hipSuccess) return hip_fail(ctx, e, "join");
    ctx->side_pending = false;
    return UNCOMP_OK;
}

uncomp_status uncomp_set_kernel_path(uncomp_ctx* ctx, int plain_alu) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    ctx->force_alu = plain_alu != 0;
    return UNCOMP_OK;
}

int uncomp_profile_read(uncomp_ctx* ctx, int max_records, const char** names, float* ms) {
    if (ctx == nullptr || max_records < 0) return UNCOMP_ERR_INVALID_ARG;
    int n = ctx->prof.n < max_records ? ctx->prof.n : max_records;
    for (int i = 0; i < n; ++i) {
        float t = 0.f;
        hipError_t e = hipEventElapsedTime(&t, ctx->prof.start[i], ctx->prof.stop[i]);
        if (e != hipSuccess) return hip_fail(ctx, e, "profile_read: hipEventElapsedTime");
        if (names != nullptr) names[i] = ctx->prof.name[i];
        if (ms != nullptr) ms[i] = t;
    }
    ctx->prof.n = 0;
    return n;
}

uncomp_status uncomp_measure_peaks(uncomp_ctx* ctx, const void* buf, size_t bytes, double* read_GBps,
                                   double* mfma_TFLOPs_live, double* mfma_TFLOPs_zero, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (buf == nullptr || read_GBps == nullptr || mfma_TFLOPs_live == nullptr || mfma_TFLOPs_zero == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "measure_peaks: null pointer");
    if (bytes < (64u << 20) || !aligned16(buf))
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "measure_peaks: need at least 64 MiB of 16-byte aligned device memory");
    uncomp_status js = uncomp_join(ctx, stream);                 // the sink word is the start of the workspace
    if (js != UNCOMP_OK) return js;
    double out[3] = {0.0, 0.0, 0.0};
    hipError_t e = measure_peaks(buf, bytes / 16, ctx->num_cu, reinterpret_cast<uint32_t*>(ctx->ws),
                                 static_cast<hipStream_t>(stream), out);
    if (e != hipSuccess) return hip_fail(ctx, e, "measure_peaks");
    *read_GBps = out[0];
    *mfma_TFLOPs_live = out[1];
    *mfma_TFLOPs_zero = out[2];
    return UNCOMP_OK;
}

const char* uncomp_last_error(const uncomp_ctx* ctx) { return ctx != nullptr ? ctx->err : noalloc_last_error(); }

uncomp_status uncomp_head_entropy(uncomp_ctx* ctx, const void* X, uncomp_dtype dtype, int n_mat,
                                  int N, int D, int64_t mat_stride, int64_t ldx, int k_trunc,
                                  unsigned flags, float* entropy_out, float* eig_out, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (X == nullptr || entropy_out == nullptr) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "head_entropy: null pointer");
    if (n_mat <= 0 || N <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "head_entropy: n_mat and N must be positive");
    if (dtype != UNCOMP_BF16 && dtype != UNCOMP_F32) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "head_entropy: dtype");
    if (D != kD && D != 64) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "head_entropy: D must be 64 or 128");
    if (k_trunc < 1) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "head_entropy: k_trunc must be >= 1");
    if (flags & ~(UNCOMP_CENTER | UNCOMP_TRUNC_RENORM | UNCOMP_LAYER_DELTA_INCREASE))
        return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "head_entropy: unknown flag bits");
    if (ldx < D || (ldx & 7) || (mat_stride & 7) || mat_stride < 0 || !aligned16(X))
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "head_entropy: strides must be multiples of 8 elements, ldx >= D, X 16-byte aligned");
    if ((int64_t)n_mat * 64 > 0x7fffffffLL) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "head_entropy: too many matrices");
    EntropyPlan p = plan_entropy(n_mat, N);
    if (kBudgetScratch + p.bytes > ctx->ws_bytes)
        return fail(ctx, UNCOMP_ERR_WORKSPACE, "head_entropy: needs %zu workspace bytes, context has %zu",
                    kBudgetScratch + p.bytes, ctx->ws_bytes);
    ctx->key_range.ptr = nullptr;
    // an eigen stage of an earlier call may still be reading the Gram partials on the side stream
    uncomp_status js = uncomp_join(ctx, stream);
    if (js != UNCOMP_OK) return js;
    char* ws = ctx->ws + kBudgetScratch;
    ctx->score_ws_off = kBudgetScratch + p.bytes;
    Env env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu};
    hipError_t e = launch_gram(X, dtype, n_mat, N, mat_stride, ldx, p, ws, env, D);
    if (e != hipSuccess) return hip_fail(ctx, e, "head_entropy: gram launch");
    if (ctx->overlap) {
        // the eigen stage moves to the side stream, ordered after the Gram kernel
        e = hipEventRecord(ctx->ev_fork, env.s);
        if (e == hipSuccess) e = hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0);
        if (e != hipSuccess) return hip_fail(ctx, e, "head_entropy: fork");
        env.s = ctx->side;
        ctx->side_pending = true;
    }
    // the plain-ALU switch also selects the fp32 Jacobi eigen stage (an independent cross-check)
    e = ctx->force_alu ? launch_jacobi_entropy(n_mat, N, k_trunc, flags, p, ws, entropy_out, eig_out, env, D)
                       : launch_tridiag_entropy(n_mat, N, k_trunc, flags, p, ws, entropy_out, eig_out, env, nullptr, D);
    if (e != hipSuccess) return hip_fail(ctx, e, "head_entropy: eigen launch");
    return UNCOMP_OK;
}

uncomp_status uncomp_assign_budgets(uncomp_ctx* ctx, const float* entropy, int n_layer, int n_batch,
                                    int H, int M, int n_max, int step, int N, int w, float eps,
                                    int delta_n, unsigned flags, int32_t* head_budget,
                                    int32_t* head_group, int32_t* layer_group, int32_t* layer_tokens,
                                    void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (entropy == nullptr) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "assign_budgets: null entropy");
    if ((head_budget == nullptr) != (head_group == nullptr) || (layer_group == nullptr) != (layer_tokens == nullptr))
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "assign_budgets: outputs come in pairs");
    if (head_budget == nullptr && layer_group == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "assign_budgets: no output requested");
    if (n_layer <= 0 || n_batch <= 0 || H <= 0 || N <= 0)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "assign_budgets: sizes must be positive");
    if (H > 1024 || n_layer > 4096) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "assign_budgets: H <= 1024, n_layer <= 4096");
    if (M < 1 || H % M != 0) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "assign_budgets: M must divide H");
    if (w <= 0 || w >= N) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "assign_budgets: need 0 < w < N");
    if (step < 0 || delta_n < 0 || n_max < 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "assign_budgets: negative n_max, step or delta_n");
    if ((int64_t)n_layer * n_batch * H > 0x7fffffffLL) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "assign_budgets: too many heads");
    if (!(eps == eps)) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "assign_budgets: eps is NaN");
    // in overlap mode the entropies are being produced on the side stream: follow them there
    hipStream_t bs = (ctx->overlap && ctx->side_pending) ? ctx->side : static_cast<hipStream_t>(stream);
    hipError_t e = launch_budgets(entropy, n_layer, n_batch, H, M, n_max, step, N, w, eps, delta_n, flags,
                                  head_budget, head_group, layer_group, layer_tokens, ctx->ws,
                                  Env{bs, &ctx->prof, ctx->force_alu});
    if (e != hipSuccess) return hip_fail(ctx, e, "assign_budgets: launch");
    return UNCOMP_OK;
}

uncomp_status uncomp_window_score(uncomp_ctx* ctx, const void* Qwin, const void* K, uncomp_dtype dtype,
                                  int B, int H, int G, int N, int D, int w, int pool,
                                  const int64_t k_strides[3], const float* lse_opt, float* score_out,
                                  void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (Qwin == nullptr || K == nullptr || score_out == nullptr || k_strides == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "window_score: null pointer");
    if (B <= 0 || H <= 0 || G <= 0 || N <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "window_score: sizes must be positive");
    if (dtype != UNCOMP_BF16 && dtype != UNCOMP_F32) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "window_score: dtype");
    if (D != kD && D != 64) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "window_score: D must be 64 or 128");
    if (w <= 0 || w >= N) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "window_score: need 0 < w < N");
    if (pool < 1 || pool > 15 || (pool & 1) == 0) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "window_score: pool must be odd in [1,15]");
    if ((int64_t)G * w > 512) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "window_score: G*w must be <= 512");
    if (k_strides[2] < D || (k_strides[0] & 7) || (k_strides[1] & 7) || (k_strides[2] & 7) || k_strides[0] < 0 ||
        k_strides[1] < 0 || !aligned16(K) || !aligned16(Qwin))
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "window_score: strides must be multiples of 8 elements, token stride >= D, 16-byte aligned pointers");
    if ((int64_t)B * H * ((N + 255) / 256) > 0x7fffffffLL) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "window_score: problem too large");
    ScorePlan p = plan_score(B, H, G, N, w);
    // keep clear of the entropy region while side-stream work may still read it
    const size_t off = ctx->side_pending ? ctx->score_ws_off : kBudgetScratch;
    if (off + p.bytes > ctx->ws_bytes)
        return fail(ctx, UNCOMP_ERR_WORKSPACE, "window_score: needs %zu workspace bytes, context has %zu",
                    off + p.bytes, ctx->ws_bytes);
    ctx->key_range.ptr = nullptr;
    hipError_t e = launch_window_score(Qwin, K, dtype, B, H, G, N, w, pool, k_strides, p, ctx->ws + off, score_out,
                                       Env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu}, lse_opt, D);
    if (e != hipSuccess) return hip_fail(ctx, e, "window_score: launch");
    ctx->key_range.ptr = reinterpret_cast<const uint32_t*>(ctx->ws + off + p.range_off);
    ctx->key_range.score = score_out;
    ctx->key_range.groups = B * H;
    ctx->key_range.P = N - w;
    ctx->key_range.n_tiles = p.n_range_tiles;
    return UNCOMP_OK;
}

uncomp_status uncomp_select_gather(uncomp_ctx* ctx, const float* score, const int32_t* budget, const void* K,
                                   const void* V, uncomp_dtype dtype, int B, int H, int N, int D, int w,
                                   const int64_t kv_strides[3], int cap, void* K_out, void* V_out,
                                   int32_t* idx_out, int32_t* len_out, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (score == nullptr || budget == nullptr || idx_out == nullptr || len_out == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "select_gather: null pointer");
    const bool any_kv = K != nullptr || V != nullptr || K_out != nullptr || V_out != nullptr;
    const bool all_kv = K != nullptr && V != nullptr && K_out != nullptr && V_out != nullptr;
    if (any_kv && !all_kv) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "select_gather: K, V, K_out, V_out must be given together");
    if (B <= 0 || H <= 0 || N <= 0 || cap <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "select_gather: sizes must be positive");
    if (dtype != UNCOMP_BF16 && dtype != UNCOMP_F32) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "select_gather: dtype");
    if (D != kD && D != 64) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "select_gather: D must be 64 or 128");
    if (w <= 0 || w >= N) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "select_gather: need 0 < w < N");
    if (cap < w) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "select_gather: cap must be >= w");
    if (!aligned16(score)) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "select_gather: score must be 16-byte aligned");
    if (all_kv) {
        if (kv_strides == nullptr) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "select_gather: null strides");
        if (kv_strides[2] < D || (kv_strides[0] & 7) || (kv_strides[1] & 7) || (kv_strides[2] & 7) ||
            kv_strides[0] < 0 || kv_strides[1] < 0 || !aligned16(K) || !aligned16(V) || !aligned16(K_out) ||
            !aligned16(V_out))
            return fail(ctx, UNCOMP_ERR_INVALID_ARG, "select_gather: strides must be multiples of 8 elements, token stride >= D, 16-byte aligned pointers");
    }
    if ((int64_t)B * H * ((cap + 7) / 8) > 0x7fffffffLL) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "select_gather: problem too large");
    static const int64_t zero_strides[3] = {0, 0, 0};
    uncomp_status js = uncomp_join(ctx, stream);
    if (js != UNCOMP_OK) return js;
    // key ranges of these very scores, if uncomp_window_score has just left them in the workspace
    const bool ranged = ctx->key_range.ptr != nullptr && ctx->key_range.score == score &&
                        ctx->key_range.groups == B * H && ctx->key_range.P == N - w;
    // A layer's worth of heads with long rows (the call as a layer-by-layer prefill makes it) would leave most of
    // the chip idle with one workgroup per head: split every row over many workgroups.  Their scratch takes the
    // front of the workspace, which is free on this stream after the join; the key ranges there are not needed.
    const SelectWidePlan sw = plan_select_wide(B * H, N, w);
    const bool wide = !ctx->force_alu && B * H <= kWideSelectRows && N - w >= kWideSelectScores &&
                      kBudgetScratch + sw.bytes <= ctx->ws_bytes;
    if (wide) ctx->key_range.ptr = nullptr;
    hipError_t e = launch_select_gather(score, budget, all_kv ? K : nullptr, V, dtype, B, H, N, w,
                                        all_kv ? kv_strides : zero_strides, cap, K_out, V_out, idx_out, len_out,
                                        Env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu},
                                        ranged && !wide ? ctx->key_range.ptr : nullptr,
                                        ranged && !wide ? ctx->key_range.n_tiles : 0, D, wide ? &sw : nullptr,
                                        ctx->ws + kBudgetScratch);
    if (e != hipSuccess) return hip_fail(ctx, e, "select_gather: launch");
    return UNCOMP_OK;
}

namespace {
struct HiddenPlan {
    ScorePlan sp;
    LastTokenPlan lt;            // the bf16 path's regions start where the general path's scoring region does
    SelectWidePlan sw;
    bool wide_select;            // few rows, long ones: the selection is split over many workgroups
    size_t score_off, sum_off, sw_off, bytes;
};
HiddenPlan plan_hidden(int B, int H, int G, int N, int w) {
    HiddenPlan p;
    p.sp = plan_score(B, H, G, N, 1);
    p.lt = plan_last_token(B, H, G, N);
    const size_t scoring = p.sp.bytes > p.lt.bytes ? p.sp.bytes : p.lt.bytes;
    p.score_off = align_up(kBudgetScratch + scoring, 256);
    p.sum_off = align_up(p.score_off + (size_t)B * H * (N - 1) * sizeof(float), 256);
    p.sw_off = align_up(p.sum_off + (size_t)B * (N - w) * sizeof(float), 256);
    p.sw = plan_select_wide(B, N, w);
    p.wide_select = B <= kWideSelectRows && N - w >= kWideSelectScores;
    p.bytes = p.sw_off + (p.wide_select ? p.sw.bytes : 0);
    return p;
}
}  // namespace

size_t uncomp_matrix_workspace_bytes(int N, int D) {
    if (N <= 0 || D <= 0 || D % kD != 0) return 0;
    return kBudgetScratch + plan_matrix(N, D).bytes;
}

uncomp_status uncomp_matrix_entropy(uncomp_ctx* ctx, const void* X, uncomp_dtype dtype, int n_mat, int N, int D,
                                    int64_t mat_stride, int64_t ldx, int k_trunc, unsigned flags, int n_iter,
                                    float* entropy_out, float* eig_out, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (X == nullptr || entropy_out == nullptr) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "matrix_entropy: null pointer");
    if (n_mat <= 0 || N <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "matrix_entropy: n_mat and N must be positive");
    if (dtype != UNCOMP_BF16 && dtype != UNCOMP_F32) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "matrix_entropy: dtype");
    if (D < 2 * kD || D > 16384 || D % kD != 0)
        return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "matrix_entropy: D must be a multiple of 128 in [256, 16384]");
    if (k_trunc < 1 || k_trunc > kD) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "matrix_entropy: need 1 <= k_trunc <= 128");
    if (n_iter < 1 || n_iter > 1000) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "matrix_entropy: need 1 <= n_iter <= 1000");
    if (flags & ~(UNCOMP_CENTER | UNCOMP_TRUNC_RENORM | UNCOMP_LAYER_DELTA_INCREASE))
        return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "matrix_entropy: unknown flag bits");
    if (ldx < D || (ldx & 7) || (mat_stride & 7) || mat_stride < 0 || !aligned16(X))
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "matrix_entropy: strides must be multiples of 8 elements, ldx >= D, X 16-byte aligned");
    const MatrixPlan p = plan_matrix(N, D);
    if (kBudgetScratch + p.bytes > ctx->ws_bytes)
        return fail(ctx, UNCOMP_ERR_WORKSPACE, "matrix_entropy: needs %zu workspace bytes, context has %zu",
                    kBudgetScratch + p.bytes, ctx->ws_bytes);
    ctx->key_range.ptr = nullptr;
    uncomp_status js = uncomp_join(ctx, stream);
    if (js != UNCOMP_OK) return js;
    hipError_t e = launch_matrix_entropy(X, dtype, n_mat, N, D, mat_stride, ldx, k_trunc, flags, n_iter, p,
                                         ctx->ws + kBudgetScratch, entropy_out, eig_out,
                                         Env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu});
    if (e != hipSuccess) return hip_fail(ctx, e, "matrix_entropy: launch");
    return UNCOMP_OK;
}

size_t uncomp_hidden_workspace_bytes(int B, int H, int G, int N, int w) {
    if (B <= 0 || H <= 0 || G <= 0 || N < 2 || w < 1 || w >= N) return 0;
    return plan_hidden(B, H, G, N, w).bytes;
}

uncomp_status uncomp_hidden_evict(uncomp_ctx* ctx, const void* q_last, const void* K, uncomp_dtype dtype, int B,
                                  int H, int G, int N, int D, const int64_t k_strides[3], const int32_t* n_keep,
                                  int w, const void* Hs, const int64_t hs_strides[2], int Dm, int cap,
                                  void* Hs_out, int32_t* idx_out, int32_t* len_out, float* score_out,
                                  void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (q_last == nullptr || K == nullptr || k_strides == nullptr || n_keep == nullptr || idx_out == nullptr ||
        len_out == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "hidden_evict: null pointer");
    if ((Hs == nullptr) != (Hs_out == nullptr) || (Hs != nullptr && hs_strides == nullptr))
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "hidden_evict: Hs, hs_strides and Hs_out must be given together");
    if (B <= 0 || H <= 0 || G <= 0 || N <= 0 || cap <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "hidden_evict: sizes must be positive");
    if (dtype != UNCOMP_BF16 && dtype != UNCOMP_F32) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "hidden_evict: dtype");
    if (D != kD) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "hidden_evict: D must be 128");
    if (w < 1 || w >= N) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "hidden_evict: need 1 <= w < N");
    if (cap < w) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "hidden_evict: cap must be >= w");
    if (G > 512) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "hidden_evict: G must be <= 512");
    if (k_strides[2] < D || (k_strides[0] & 7) || (k_strides[1] & 7) || (k_strides[2] & 7) || k_strides[0] < 0 ||
        k_strides[1] < 0 || !aligned16(K) || !aligned16(q_last))
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "hidden_evict: key strides must be multiples of 8 elements, token stride >= D, 16-byte aligned pointers");
    const int esz = dtype == UNCOMP_BF16 ? 2 : 4;
    if (Hs != nullptr) {
        if (Dm <= 0 || ((int64_t)Dm * esz) % 16 != 0 || hs_strides[1] < Dm || (hs_strides[0] * esz) % 16 != 0 ||
            (hs_strides[1] * esz) % 16 != 0 || hs_strides[0] < 0 || !aligned16(Hs) || !aligned16(Hs_out))
            return fail(ctx, UNCOMP_ERR_INVALID_ARG, "hidden_evict: hidden rows must be whole 16-byte units with 16-byte aligned strides and pointers");
    }
    if ((int64_t)B * H * ((N + 255) / 256) > 0x7fffffffLL || (int64_t)B * ((cap + 3) / 4) > 0x7fffffffLL)
        return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "hidden_evict: problem too large");
    const HiddenPlan p = plan_hidden(B, H, G, N, w);
    if (p.bytes > ctx->ws_bytes)
        return fail(ctx, UNCOMP_ERR_WORKSPACE, "hidden_evict: needs %zu workspace bytes, context has %zu", p.bytes,
                    ctx->ws_bytes);
    ctx->key_range.ptr = nullptr;
    uncomp_status js = uncomp_join(ctx, stream);          // the whole workspace is used: wait for side-stream work
    if (js != UNCOMP_OK) return js;
    const Env env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu};
    float* score = reinterpret_cast<float*>(ctx->ws + p.score_off);
    float* sum = score_out != nullptr ? score_out : reinterpret_cast<float*>(ctx->ws + p.sum_off);
    hipError_t e;
    if (dtype == UNCOMP_BF16 && !ctx->force_alu && G <= 16) {
        // bf16: one streamed MFMA pass over the keys and a merge
        e = launch_last_token_score(q_last, K, B, H, G, N, k_strides, N - w, p.lt, ctx->ws + kBudgetScratch, sum, env);
    } else {
        // the last token's attention = window score with a one-token window and no pooling
        e = launch_window_score(q_last, K, dtype, B, H, G, N, 1, 1, k_strides, p.sp, ctx->ws + kBudgetScratch, score,
                                env);
        if (e == hipSuccess) e = launch_head_sum(score, B, H, N - 1, N - w, sum, env);
    }
    if (e == hipSuccess) {
        if (p.wide_select)
            e = launch_select_rows_wide(sum, n_keep, 0, B, N, w, cap, p.sw, ctx->ws + p.sw_off, idx_out, len_out, env);
        else
            e = launch_select_rows(sum, n_keep, 0, B, N, w, cap, idx_out, len_out, env);
    }
    if (e == hipSuccess && Hs != nullptr)
        e = launch_gather_rows(Hs, idx_out, len_out, B, cap, N, Dm * esz, hs_strides[0] * esz, hs_strides[1] * esz,
                               Hs_out, env);
    if (e != hipSuccess) return hip_fail(ctx, e, "hidden_evict: launch");
    return UNCOMP_OK;
}

namespace {
uncomp_status check_prepare_dims(uncomp_ctx* ctx, const char* who, int L, int H, int M) {
    if (L <= 0 || H <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "%s: sizes must be positive", who);
    if (H > 1024 || L > 4096) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "%s: H <= 1024, n_layer <= 4096", who);
    if (M < 1 || H % M != 0) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "%s: M must divide H", who);
    return UNCOMP_OK;
}
}  // namespace

uncomp_status uncomp_prepare_reset(uncomp_ctx* ctx, int n_layer, int H, int M, double* erank_sum, int32_t* votes,
                                   int32_t* count, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (erank_sum == nullptr || votes == nullptr || count == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "prepare_reset: null pointer");
    uncomp_status st = check_prepare_dims(ctx, "prepare_reset", n_layer, H, M);
    if (st != UNCOMP_OK) return st;
    hipError_t e = launch_prepare_reset(n_layer, H, M, erank_sum, votes, count,
                                        Env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu});
    if (e != hipSuccess) return hip_fail(ctx, e, "prepare_reset: launch");
    return UNCOMP_OK;
}

uncomp_status uncomp_prepare_accumulate(uncomp_ctx* ctx, const float* entropy, int n_layer, int n_batch, int H, int M,
                                        double* erank_sum, int32_t* votes, int32_t* count, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (entropy == nullptr || erank_sum == nullptr || votes == nullptr || count == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "prepare_accumulate: null pointer");
    if (n_batch <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "prepare_accumulate: sizes must be positive");
    uncomp_status st = check_prepare_dims(ctx, "prepare_accumulate", n_layer, H, M);
    if (st != UNCOMP_OK) return st;
    // in overlap mode the entropies may still be under way on the side stream
    st = uncomp_join(ctx, stream);
    if (st != UNCOMP_OK) return st;
    hipError_t e = launch_prepare_accumulate(entropy, n_layer, n_batch, H, M, erank_sum, votes, count,
                                             Env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu});
    if (e != hipSuccess) return hip_fail(ctx, e, "prepare_accumulate: launch");
    return UNCOMP_OK;
}

uncomp_status uncomp_prepare_finish(uncomp_ctx* ctx, int n_layer, int H, int M, const double* erank_sum,
                                    const int32_t* votes, const int32_t* count, int32_t* labels_mean,
                                    int32_t* labels_vote, float* mean_erank_out, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (erank_sum == nullptr || votes == nullptr || count == nullptr || labels_mean == nullptr ||
        labels_vote == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "prepare_finish: null pointer");
    uncomp_status st = check_prepare_dims(ctx, "prepare_finish", n_layer, H, M);
    if (st != UNCOMP_OK) return st;
    hipError_t e = launch_prepare_finish(n_layer, H, M, erank_sum, votes, count, labels_mean, labels_vote,
                                         mean_erank_out, Env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu});
    if (e != hipSuccess) return hip_fail(ctx, e, "prepare_finish: launch");
    return UNCOMP_OK;
}

uncomp_status uncomp_budgets_from_labels(uncomp_ctx* ctx, const int32_t* labels, int n_layer, int n_batch, int H,
                                         int n_max, int step, int N, int w, int32_t* head_budget, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (labels == nullptr || head_budget == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "budgets_from_labels: null pointer");
    if (n_layer <= 0 || n_batch <= 0 || H <= 0 || N <= 0)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "budgets_from_labels: sizes must be positive");
    if (w <= 0 || w >= N) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "budgets_from_labels: need 0 < w < N");
    if (step < 0 || n_max < 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "budgets_from_labels: negative n_max or step");
    hipError_t e = launch_labels_to_budget(labels, n_layer, n_batch, H, n_max, step, N, w, head_budget,
                                           Env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu});
    if (e != hipSuccess) return hip_fail(ctx, e, "budgets_from_labels: launch");
    return UNCOMP_OK;
}

size_t uncomp_decode_workspace_bytes(int n_heads, int G, int cap) {
    if (n_heads <= 0 || G <= 0 || cap <= 0) return 0;
    return plan_decode(n_heads, G, cap).bytes;
}

uncomp_status uncomp_decode_init(uncomp_ctx* ctx, const float* score, const int32_t* idx, const int32_t* len,
                                 int n_heads, int N, int w, int cap, float* cum_out, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (score == nullptr || idx == nullptr || len == nullptr || cum_out == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "decode_init: null pointer");
    if (n_heads <= 0 || N <= 0 || cap <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "decode_init: sizes must be positive");
    if (w <= 0 || w >= N) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "decode_init: need 0 < w < N");
    hipError_t e = launch_decode_init(score, idx, len, n_heads, N, w, cap, cum_out,
                                      Env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu});
    if (e != hipSuccess) return hip_fail(ctx, e, "decode_init: launch");
    return UNCOMP_OK;
}

uncomp_status uncomp_decode_step(uncomp_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                                 uncomp_dtype dtype, int n_heads, int G, int D, const int32_t* pos,
                                 const int32_t* budget, int w, int cap, void* K_c, void* V_c, int32_t* idx,
                                 float* cum, int32_t* len, float* out, int32_t* evicted, void* stream) {
    if (ctx == nullptr) return UNCOMP_ERR_INVALID_ARG;
    if (q == nullptr || k_new == nullptr || v_new == nullptr || pos == nullptr || budget == nullptr ||
        K_c == nullptr || V_c == nullptr || idx == nullptr || cum == nullptr || len == nullptr)
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "decode_step: null pointer");
    if (n_heads <= 0 || cap <= 0) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "decode_step: sizes must be positive");
    if (dtype != UNCOMP_BF16 && dtype != UNCOMP_F32) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "decode_step: dtype");
    if (D != kD) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "decode_step: D must be 128");
    if (G < 1 || G > 16) return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "decode_step: need 1 <= G <= 16");
    if (w < 1 || w > cap) return fail(ctx, UNCOMP_ERR_INVALID_ARG, "decode_step: need 1 <= w <= cap");
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(K_c) || !aligned16(V_c))
        return fail(ctx, UNCOMP_ERR_INVALID_ARG, "decode_step: 16-byte aligned pointers required");
    if ((int64_t)n_heads * (((int64_t)cap + 128) / 128) > 0x7fffffffLL)
        return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "decode_step: problem too large");
    const DecodePlan p = plan_decode(n_heads, G, cap);
    const bool wave_path = dtype == UNCOMP_BF16 && !ctx->force_alu;
    if (!wave_path && (int64_t)G * ((int64_t)cap + 1) > 36864)
        return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "decode_step: fp32 caches need G*(cap+1) <= 36864");
    if (wave_path && decode_update_lds_bytes(p) > kLdsDefaultLimit)
        return fail(ctx, UNCOMP_ERR_UNSUPPORTED, "decode_step: cap %d at G %d needs %zu bytes of LDS per head, limit %zu",
                    cap, G, decode_update_lds_bytes(p), kLdsDefaultLimit);
    const size_t need = wave_path ? p.bytes : (out == nullptr ? p.p_off : 0);
    if (need > ctx->ws_bytes)
        return fail(ctx, UNCOMP_ERR_WORKSPACE, "decode_step: needs %zu workspace bytes, context has %zu", need,
                    ctx->ws_bytes);
    // the workspace starts at offset 0: side-stream work of an earlier entropy call may still use it
    ctx->key_range.ptr = nullptr;
    uncomp_status js = uncomp_join(ctx, stream);
    if (js != UNCOMP_OK) return js;
    // the kernels always form the output; without a destination it lands in the workspace
    float* out_p = out != nullptr ? out : reinterpret_cast<float*>(ctx->ws + p.out_off);
    const Env env{static_cast<hipStream_t>(stream), &ctx->prof, ctx->force_alu};
    hipError_t e = wave_path ? launch_decode_wave(q, k_new, v_new, n_heads, G, pos, budget, w, cap, K_c, V_c, idx, cum,
                                                  len, out_p, evicted, p, ctx->ws, env)
                             : launch_decode_step(q, k_new, v_new, dtype, n_heads, G, pos, budget, w, cap, K_c, V_c,
                                                  idx, cum, len, out_p, evicted, env);
    if (e != hipSuccess) return hip_fail(ctx, e, "decode_step: launch");
    return UNCOMP_OK;
}

}  // extern "C"
