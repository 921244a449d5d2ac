// Offline preparation (Sec. 3.3.1 "Preparation Stage", Eq. 7: a head's grouping metric is its
// erank averaged over the sampled prompts; App. Alg. 1: per sample every head gets one of M
// labels from its entropy and the final label is the majority's), and Eq. 11 budgets from the
// stored labels.  The entropies come from uncomp_head_entropy; what is left is a few hundred
// comparisons per layer: one thread per (layer, head), samples visited in order, so every sum
// has a fixed order and nothing needs an atomic.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

__global__ __launch_bounds__(256) void prepare_reset_kernel(double* __restrict__ erank_sum,
                                                            int32_t* __restrict__ votes,
                                                            int32_t* __restrict__ count, int LH, int M) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e < LH) {
        erank_sum[e] = 0.0;
        for (int g = 0; g < M; ++g) votes[(int64_t)e * M + g] = 0;
    }
    if (e == 0) *count = 0;
}

// One workgroup per layer, thread h < H.  Label of a head in a sample: rank by entropy inside the
// layer (larger first, equal values by lower index) / (H / M).
__global__ __launch_bounds__(1024) void prepare_accumulate_kernel(const float* __restrict__ entropy, int B, int H,
                                                                  int M, double* __restrict__ erank_sum,
                                                                  int32_t* __restrict__ votes,
                                                                  int32_t* __restrict__ count) {
    const int l = blockIdx.x, h = threadIdx.x;
    if (h < H) {
        const int per = H / M;
        double acc = erank_sum[(int64_t)l * H + h];
        int32_t* my_votes = votes + ((int64_t)l * H + h) * M;
        for (int b = 0; b < B; ++b) {
            const float* row = entropy + ((int64_t)l * B + b) * H;
            const float mine = row[h];
            int rank = 0;
            for (int o = 0; o < H; ++o) {
                const float v = row[o];
                rank += (v > mine || (v == mine && o < h)) ? 1 : 0;
            }
            my_votes[rank / per] += 1;
            acc += exp((double)mine);
        }
        erank_sum[(int64_t)l * H + h] = acc;
    }
    if (l == 0 && h == 0) *count += B;
}

__global__ __launch_bounds__(1024) void prepare_finish_kernel(const double* __restrict__ erank_sum,
                                                              const int32_t* __restrict__ votes,
                                                              const int32_t* __restrict__ count, int H, int M,
                                                              int32_t* __restrict__ labels_mean,
                                                              int32_t* __restrict__ labels_vote,
                                                              float* __restrict__ mean_out) {
    __shared__ double mean[1024];
    const int l = blockIdx.x, h = threadIdx.x;
    const int n = *count > 0 ? *count : 1;
    if (h < H) mean[h] = erank_sum[(int64_t)l * H + h] / (double)n;
    __syncthreads();
    if (h >= H) return;
    const double mine = mean[h];
    int rank = 0;
    for (int o = 0; o < H; ++o) rank += (mean[o] > mine || (mean[o] == mine && o < h)) ? 1 : 0;
    labels_mean[(int64_t)l * H + h] = rank / (H / M);
    const int32_t* my_votes = votes + ((int64_t)l * H + h) * M;
    int best = 0;
    for (int g = 1; g < M; ++g)
        if (my_votes[g] > my_votes[best]) best = g;
    labels_vote[(int64_t)l * H + h] = best;
    if (mean_out != nullptr) mean_out[(int64_t)l * H + h] = (float)mine;
}

__global__ __launch_bounds__(256) void labels_to_budget_kernel(const int32_t* __restrict__ labels, int L, int B,
                                                               int H, int n_max, int step, int N, int w,
                                                               int32_t* __restrict__ head_budget) {
    const int64_t total = (int64_t)L * B * H;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int h = (int)(e % H);
        const int l = (int)(e / ((int64_t)B * H));
        long long b = (long long)n_max - (long long)labels[(int64_t)l * H + h] * step;
        const int lo = w < N ? w : N;
        b = b < lo ? lo : b;
        b = b > N ? N : b;
        head_budget[e] = (int32_t)b;
    }
}

hipError_t launch_prepare_reset(int L, int H, int M, double* erank_sum, int32_t* votes, int32_t* count,
                                const Env& env) {
    env.begin("prepare_reset");
    prepare_reset_kernel<<<dim3((unsigned)((L * H + 255) / 256)), dim3(256), 0, env.s>>>(erank_sum, votes, count, L * H,
                                                                                       M);
    env.end();
    return hipGetLastError();
}

hipError_t launch_prepare_accumulate(const float* entropy, int L, int B, int H, int M, double* erank_sum,
                                     int32_t* votes, int32_t* count, const Env& env) {
    env.begin("prepare_accumulate");
    prepare_accumulate_kernel<<<dim3((unsigned)L), dim3((unsigned)((H + 63) / 64 * 64)), 0, env.s>>>(
        entropy, B, H, M, erank_sum, votes, count);
    env.end();
    return hipGetLastError();
}

hipError_t launch_prepare_finish(int L, int H, int M, const double* erank_sum, const int32_t* votes,
                                 const int32_t* count, int32_t* labels_mean, int32_t* labels_vote, float* mean_out,
                                 const Env& env) {
    env.begin("prepare_finish");
    prepare_finish_kernel<<<dim3((unsigned)L), dim3((unsigned)((H + 63) / 64 * 64)), 0, env.s>>>(
        erank_sum, votes, count, H, M, labels_mean, labels_vote, mean_out);
    env.end();
    return hipGetLastError();
}

hipError_t launch_labels_to_budget(const int32_t* labels, int L, int B, int H, int n_max, int step, int N, int w,
                                   int32_t* head_budget, const Env& env) {
    const int64_t total = (int64_t)L * B * H;
    const unsigned blocks = (unsigned)((total + 255) / 256 > 1024 ? 1024 : (total + 255) / 256);
    env.begin("labels_to_budget");
    labels_to_budget_kernel<<<dim3(blocks), dim3(256), 0, env.s>>>(labels, L, B, H, n_max, step, N, w, head_budget);
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
