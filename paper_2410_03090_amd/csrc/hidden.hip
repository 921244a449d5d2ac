// Stage-1 hidden-state eviction (Sec. 3.3.2 "Hidden State Eviction": the tokens that enter the
// next layer group are those that receive the most attention from the last token of the current
// layer; their number comes from Eq. 10).  The last token's attention is the observation-window
// score with a one-token window and no pooling, so the scoring kernels are reused; this file adds
// the sum over the KV heads.  Selection and the row copy are the kernels of the per-head
// compaction, run with one group per batch entry and rows of the model width.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

// out[b][j] = sum_h score[b][h][j] for j < P_out; score rows have P_in >= P_out entries.
__global__ __launch_bounds__(256) void head_sum_kernel(const float* __restrict__ score, int H, int P_in,
                                                       int P_out, float* __restrict__ out) {
    const int b = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= P_out) return;
    const float* s = score + (int64_t)b * H * P_in + j;
    float acc = 0.f;
    for (int h = 0; h < H; ++h) acc += s[(int64_t)h * P_in];
    out[(int64_t)b * P_out + j] = acc;
}

hipError_t launch_head_sum(const float* score, int B, int H, int P_in, int P_out, float* out, const Env& env) {
    env.begin("head_sum");
    head_sum_kernel<<<dim3((unsigned)((P_out + 255) / 256), (unsigned)B), dim3(256), 0, env.s>>>(score, H, P_in,
                                                                                               P_out, out);
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
