// Shared host-side declarations of libuncomp: the context, the workspace planner and the
// launchers implemented by the kernel files.  Not part of the public interface.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/uncomp.h"

namespace uncomp {
// Optional per-kernel timing: when switched on, each kernel launch of a hot call is put
// between two HIP events recorded on the caller's stream.
struct Profiler {
    static constexpr int kMax = 1024;
    bool on = false;
    int n = 0;                       // records used since the last reset
    int n_events = 0;                // event pairs created so far
    const char* name[kMax];
    hipEvent_t start[kMax], stop[kMax];
};
}  // namespace uncomp

struct uncomp_ctx {
    int device;
    int num_cu;
    char* ws;            // device workspace
    size_t ws_bytes;
    char err[256];
    uncomp::Profiler prof;
    bool force_alu = false;
    // overlap mode: the eigen stage and the budget kernels run on `side`, beside the scoring
    // kernels of the caller's stream, and are joined before the selection kernels
    bool overlap = false;
    bool side_pending = false;       // work enqueued on `side` that the caller's stream has not waited for
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    size_t score_ws_off = 0;         // where the scoring workspace starts (after the entropy region)
    // Key ranges left in the workspace by the last uncomp_window_score, for the selection that follows it.
    // Cleared by every call that may overwrite that part of the workspace; the selection kernel checks the
    // range against every score anyway, so a range that does not belong to the scores costs time, not results.
    struct {
        const uint32_t* ptr = nullptr;
        const float* score = nullptr;
        int groups = 0, P = 0, n_tiles = 0;
    } key_range;
};

namespace uncomp {

constexpr int kD = 128;                 // head dimension all kernels are written for
constexpr int kGramTile = 128;          // tokens a Gram workgroup folds per inner step
constexpr int kJacobiLd = kD + 4;       // padded column stride of the LDS matrix (floats)
constexpr int kMaxSweeps = 30;          // hard stop of the Jacobi iteration

// ---- workspace planning (host) -------------------------------------------------------
struct EntropyPlan {
    int n_chunks;        // token chunks per matrix (split of the Gram sum)
    int chunk;           // tokens per chunk (multiple of kGramTile)
    size_t gram_off;     // float [n_mat][n_chunks][D*D]
    size_t sum_off;      // float [n_mat][n_chunks][D]
    size_t bytes;
};
EntropyPlan plan_entropy(int n_mat, int N, size_t max_bytes = 0);

struct ScorePlan {
    int R;               // query rows per KV head = G*w
    int n_chunks;        // token chunks per head for the softmax-statistics pass
    int chunk;           // tokens per chunk
    size_t stats_off;    // float2 [BH][n_chunks][R]   (running max, running sum)
    size_t lse_off;      // float  [BH][R]
    size_t vote_off;     // float  [BH][G][P]
    size_t range_off;    // uint32 [BH][n_range_tiles][2]: smallest / largest selection key of every 1024 scores
    int n_range_tiles;
    size_t bytes;
};
ScorePlan plan_score(int B, int H, int G, int N, int w);

// Stream plus optional profiler, handed to every launcher.
struct Env {
    hipStream_t s;
    Profiler* prof;
    bool force_alu = false;          // use the plain-ALU kernels even where an MFMA kernel exists
    // Marks the start / end of one kernel launch (no-ops unless profiling is on).
    void begin(const char* kernel_name) const {
        if (prof == nullptr || !prof->on || prof->n >= Profiler::kMax) return;
        int i = prof->n;
        if (i >= prof->n_events) return;             // events are created by uncomp_profile, never here
        prof->name[i] = kernel_name;
        (void)hipEventRecord(prof->start[i], s);
    }
    void end() const {
        if (prof == nullptr || !prof->on || prof->n >= Profiler::kMax || prof->n >= prof->n_events) return;
        (void)hipEventRecord(prof->stop[prof->n], s);
        prof->n += 1;
    }
};

// ---- launchers (each returns the hipError_t of its launches) ---------------------------
// D: features per token, 128, or 64 (then the plain-ALU kernel runs and features 64..127 of the 128-wide
// partial sums are zero, which leaves the non-zero eigenvalues and the entropy as they are).
hipError_t launch_gram(const void* X, uncomp_dtype dt, int n_mat, int N, int64_t mat_stride,
                       int64_t ldx, const EntropyPlan& p, char* ws, const Env& env, int D = kD);
hipError_t launch_jacobi_entropy(int n_mat, int N, int k_trunc, unsigned flags,
                                 const EntropyPlan& p, char* ws, float* entropy_out,
                                 float* eig_out, const Env& env, int eig_ld = kD);
// trace_total: optional DEVICE pointer to two doubles, the raw (unnormalised) centred and
// uncentred traces of the larger matrix that the one handed in is a projection of: Eq. 5 without
// renormalisation divides by the one that applies, and a larger matrix without spread gives 0.
hipError_t launch_tridiag_entropy(int n_mat, int N, int k_trunc, unsigned flags,
                                  const EntropyPlan& p, char* ws, float* entropy_out,
                                  float* eig_out, const Env& env, const double* trace_total = nullptr,
                                  int eig_ld = kD);
hipError_t launch_budgets(const float* entropy, int L, int B, int H, int M, int n_max, int step,
                          int N, int w, float eps, int delta_n, unsigned flags,
                          int32_t* head_budget, int32_t* head_group, int32_t* layer_group,
                          int32_t* layer_tokens, char* ws, const Env& env);
// lse_nat: optional DEVICE [B*H*G*w] natural-log normalisers of the window rows; when given the
// softmax-statistics pass is skipped.
hipError_t launch_window_score(const void* Q, const void* K, uncomp_dtype dt, int B, int H, int G,
                               int N, int w, int pool, const int64_t ks[3], const ScorePlan& p,
                               char* ws, float* score_out, const Env& env, const float* lse_nat = nullptr,
                               int D = kD);
hipError_t launch_select_gather(const float* score, const int32_t* budget, const void* K,
                                const void* V, uncomp_dtype dt, int B, int H, int N, int w,
                                const int64_t ks[3], int cap, void* K_out, void* V_out,
                                int32_t* idx_out, int32_t* len_out, const Env& env,
                                const uint32_t* tile_range = nullptr, int n_range_tiles = 0, int D = kD,
                                const struct SelectWidePlan* wide = nullptr, char* wide_ws = nullptr);
// The same selection for a few long rows, each split over n_wg workgroups (select_wide.hip); ws: p.bytes.
struct SelectWidePlan {
    int n_wg;            // workgroups (chunks of 2048 positions) per row
    size_t bytes;
};
// few rows (at most kWideSelectRows), long ones (at least kWideSelectScores scores): worth splitting
constexpr int kWideSelectRows = 32, kWideSelectScores = 32768;
SelectWidePlan plan_select_wide(int n_groups, int N, int w);
hipError_t launch_select_rows_wide(const float* score, const int32_t* budget, int budget_stride, int n_groups, int N,
                                   int w, int cap, const SelectWidePlan& p, char* ws, int32_t* idx_out, int32_t* len_out,
                                   const Env& env);
hipError_t launch_select_rows(const float* score, const int32_t* budget, int budget_stride, int n_groups,
                              int N, int w, int cap, int32_t* idx_out, int32_t* len_out, const Env& env);
hipError_t launch_gather_rows(const void* src, const int32_t* idx, const int32_t* len, int n_groups, int cap,
                              int n_src_rows, int row_bytes, int64_t group_stride_bytes, int64_t row_stride_bytes,
                              void* dst, const Env& env);
// Workspace of the bf16 last-token attention of the hidden-state eviction.
struct LastTokenPlan {
    int GT, wave_rows, s_rows, np;
    size_t p_off, ml_off, head_off, bytes;
};
LastTokenPlan plan_last_token(int B, int H, int G, int N);
hipError_t launch_last_token_score(const void* q, const void* K, int B, int H, int G, int N, const int64_t ks[3],
                                   int P_out, const LastTokenPlan& p, char* ws, float* out, const Env& env);
hipError_t launch_head_sum(const float* score, int B, int H, int P_in, int P_out, float* out, const Env& env);
hipError_t launch_prepare_reset(int L, int H, int M, double* erank_sum, int32_t* votes, int32_t* count,
                                const Env& env);
hipError_t launch_prepare_accumulate(const float* entropy, int L, int B, int H, int M, double* erank_sum,
                                     int32_t* votes, int32_t* count, const Env& env);
hipError_t launch_prepare_finish(int L, int H, int M, const double* erank_sum, const int32_t* votes,
                                 const int32_t* count, int32_t* labels_mean, int32_t* labels_vote, float* mean_out,
                                 const Env& env);
hipError_t launch_labels_to_budget(const int32_t* labels, int L, int B, int H, int n_max, int step, int N, int w,
                                   int32_t* head_budget, const Env& env);
// Workspace of the wide-matrix entropy (one matrix at a time).
struct MatrixPlan {
    int stat_chunks, stat_chunk;     // token chunks of the column statistics
    int w_chunks, w_chunk;           // token chunks of W = X^T Z
    int gram_slices, gram_rows;      // row slices of the fp64 Gram of W
    int zgram_slices, zgram_rows;    // token slices of the fp64 Gram of the projected tokens
    int z_splits;                    // split of the sum over d in the MFMA version of Z = X Q
    int t_chunks, t_chunk;           // token chunks of the MFMA version of W = X^T Z
    size_t qt_off, zpart_off, zsplit_off;
    EntropyPlan ep;                  // the 128-wide entropy path on the projected tokens
    size_t ep_off, statpart_off, s_off, trace_off, zsum_off, q_off, w_off, wpart_off, z_off, gpart_off, spart_off, rinv_off;
    size_t bytes;
};
MatrixPlan plan_matrix(int N, int D);
hipError_t launch_xtz_mfma(const uint16_t* X, int64_t ldx, const float* Z, int N, int D, uint16_t* Zt, int t_chunk,
                           int n_tchunks, float* Wpart, hipStream_t s, bool zt_ready);
hipError_t launch_xq_mfma(const uint16_t* X, int64_t ldx, int N, int D, const uint16_t* Qt_hi, const uint16_t* Qt_lo,
                          int n_split, float* Zpart, float* Z, hipStream_t s, bool precise, bool want_zt, uint16_t* Zt,
                          bool* zt_written);
hipError_t launch_gram_f32_mfma(const float* X, int n_mat, int N, int64_t mat_stride, int64_t ldx, int n_chunks, int chunk,
                                float* gram_part, float* sum_part, hipStream_t s);
hipError_t launch_matrix_entropy(const void* X, uncomp_dtype dt, int n_mat, int N, int D, int64_t mat_stride,
                                 int64_t ldx, int k_trunc, unsigned flags, int n_iter, const MatrixPlan& p, char* ws,
                                 float* entropy_out, float* eig_out, const Env& env);
// Workspace of the bf16 decode path (two kernels per step).
struct DecodePlan {
    int GT;              // query heads per KV head rounded up to 4, 8 or 16
    int wave_rows;       // rows of one head that one wave owns (128 or 256)
    int s_rows;          // rows per head in the probability table (cap + 1 rounded up to whole waves)
    int np_max;          // waves (128-row parts) per head
    size_t out_off;      // float [n_heads][G][D]: attention output when the caller wants none
    size_t p_off;        // float [n_heads][s_rows][GT]
    size_t ml_off;       // float [n_heads][np_max][GT][2]
    size_t acc_off;      // float [n_heads][np_max][GT][D]
    size_t bytes;
};
DecodePlan plan_decode(int n_heads, int G, int cap);
hipError_t launch_decode_wave(const void* q, const void* k_new, const void* v_new, int n_heads, int G,
                              const int32_t* pos, const int32_t* budget, int w, int cap, void* Kc, void* Vc,
                              int32_t* idx, float* cum, int32_t* len, float* out, int32_t* evicted,
                              const DecodePlan& p, char* ws, const Env& env);
hipError_t launch_decode_init(const float* score, const int32_t* idx, const int32_t* len, int n_heads,
                              int N, int w, int cap, float* cum, const Env& env);
size_t decode_step_lds_bytes(int G, int cap);
hipError_t launch_decode_step(const void* q, const void* k_new, const void* v_new, uncomp_dtype dt,
                              int n_heads, int G, const int32_t* pos, const int32_t* budget, int w, int cap,
                              void* Kc, void* Vc, int32_t* idx, float* cum, int32_t* len, float* out,
                              int32_t* evicted, const Env& env);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// LDS a workgroup may use on gfx950 (160 KiB) and what a kernel gets without asking (64 KiB).
constexpr size_t kLdsPerWorkgroup = 160 * 1024;
constexpr size_t kLdsDefaultLimit = 64 * 1024;

// Kernels that take more than 64 KiB of dynamic LDS have their limit raised here, once per context
// at creation (device current), so that no hot call changes function attributes.
inline hipError_t allow_dynamic_lds(const void* kernel, size_t bytes) {
    return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}
hipError_t measure_peaks(const void* buf, size_t n16, int num_cu, uint32_t* sink, hipStream_t s, double out[3]);
const char* noalloc_last_error();
hipError_t init_gram_kernels();
hipError_t init_select_kernels();
hipError_t init_score_kernels();
hipError_t init_jacobi_kernels();
hipError_t init_decode_kernels();
hipError_t init_subspace_kernels();
// Largest dynamic LDS request of the bf16 decode update kernel (three tables of [np_max][GT] floats).
size_t decode_update_lds_bytes(const DecodePlan& p);

}  // namespace uncomp
