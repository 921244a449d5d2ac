// Budgets from entropies (Sec. 3.3.3 "Design" and Eq. 11 for the head groups; Sec. 3.3.2
// Eq. 8-10 for the layer stages).  The work is a few hundred comparisons: one small kernel
// ranks the heads of every (layer, batch) by counting, a second one walks the layers.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

__global__ __launch_bounds__(256) void head_budget_kernel(const float* __restrict__ entropy, int n_lb,
                                                          int H, int M, int n_max, int step, int N, int w,
                                                          int32_t* __restrict__ head_budget,
                                                          int32_t* __restrict__ head_group) {
    const int total = n_lb * H;
    const int per = H / M;
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < total; e += gridDim.x * blockDim.x) {
        const int lb = e / H, h = e - lb * H;
        const float* row = entropy + (int64_t)lb * H;
        const float mine = row[h];
        int rank = 0;                         // heads that come before h: larger entropy, or equal and lower index
        for (int o = 0; o < H; ++o) {
            float v = row[o];
            rank += (v > mine || (v == mine && o < h)) ? 1 : 0;
        }
        const int g = rank / per;
        long long b = (long long)n_max - (long long)g * step;      // g*step may exceed 32 bits
        const long long lo = w < N ? w : N;
        b = b < lo ? lo : b;
        b = b > N ? N : b;
        head_budget[e] = (int32_t)b;
        head_group[e] = g;
    }
}

// One workgroup.  Thread l averages exp(entropy) of layer l in fp64 in index order; thread 0
// then counts stage boundaries front to back.
__global__ __launch_bounds__(256) void layer_stage_kernel(const float* __restrict__ entropy, int L, int BH,
                                                          int N, int w, float eps, int delta_n,
                                                          int increase, double* __restrict__ layer_mean,
                                                          int32_t* __restrict__ layer_group,
                                                          int32_t* __restrict__ layer_tokens) {
    for (int l = threadIdx.x; l < L; l += blockDim.x) {
        double acc = 0.0;
        for (int i = 0; i < BH; ++i) acc += exp((double)entropy[(int64_t)l * BH + i]);
        layer_mean[l] = acc / (double)BH;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int c = 0;
        for (int l = 0; l < L; ++l) {
            if (l > 0) {
                double d = layer_mean[l - 1] - layer_mean[l];
                if (increase) d = -d;
                if (d > (double)eps) ++c;
            }
            layer_group[l] = c;
            long long t = (long long)N - (long long)c * delta_n;
            layer_tokens[l] = t > w ? (int32_t)t : w;
        }
    }
}

hipError_t launch_budgets(const float* entropy, int L, int B, int H, int M, int n_max, int step,
                          int N, int w, float eps, int delta_n, unsigned flags,
                          int32_t* head_budget, int32_t* head_group, int32_t* layer_group,
                          int32_t* layer_tokens, char* ws, const Env& env) {
    hipStream_t s = env.s;
    if (head_budget != nullptr) {
        int total = L * B * H;
        int blocks = (total + 255) / 256;
        if (blocks > 1024) blocks = 1024;
        env.begin("head_budget");
        head_budget_kernel<<<blocks, 256, 0, s>>>(entropy, L * B, H, M, n_max, step, N, w,
                                                  head_budget, head_group);
        env.end();
    }
    if (layer_group != nullptr) {
        env.begin("layer_stage");
        layer_stage_kernel<<<1, 256, 0, s>>>(entropy, L, B * H, N, w, eps, delta_n,
                                             (flags & UNCOMP_LAYER_DELTA_INCREASE) ? 1 : 0,
                                             reinterpret_cast<double*>(ws), layer_group, layer_tokens);
        env.end();
    }
    return hipGetLastError();
}

}  // namespace uncomp
