// Observation-window score (Sec. 3.3.3 "Dynamic KV Cache Eviction"): attention of the last
// w queries over all keys, summed per prefix token, max-pooled along the token axis and
// summed over the G query heads of a KV head.
//
// The softmax needs each query row's normaliser before any probability can be summed, so
// the keys are streamed twice:
//   pass 1  running (max, sum of exp) of every query row over token chunks   -> stats
//   merge   per row: log-sum-exp over the chunks (base 2)                     -> lse
//   pass 2  p_ij = exp2(logit_ij - lse_i), summed over the w rows of a head   -> vote[g][j]
//   pool    max over the +-pool/2 neighbours per query head, sum over heads   -> score
// Logits are kept in base 2 (q.k * log2(e)/sqrt(D)) so that a single v_exp_f32 gives the
// exponential.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kStatTile = 32;     // tokens staged per step in pass 1 (plain-ALU kernel)
constexpr int kVoteRows = 32;     // query rows staged per step in pass 2 (plain-ALU kernel)
}

// ---------------------------------------------------------------------------------------
// pass 1, plain ALU: one thread per query row (row = g*w + i of the KV head), the row's
// query in registers, keys broadcast from LDS.  Row i of a head sits at position P+i and
// sees tokens j <= P+i.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(512) void score_stats_alu_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, int H, int G, int N, int w, int64_t ks_b,
    int64_t ks_h, int64_t ks_t, int n_chunks, int chunk, float2* __restrict__ stats) {
    __shared__ float kt[kStatTile][kD];
    const int bh = blockIdx.x / n_chunks, c = blockIdx.x % n_chunks;
    const int b = bh / H, h = bh % H;
    const int R = G * w, P = N - w;
    const int row = threadIdx.x;
    const bool live = row < R;
    const int i = live ? row % w : 0;
    const T* Kh = K + b * ks_b + h * ks_h;
    const float scale2 = kLog2e * rsqrtf((float)kD);

    float q[kD];
    if (live) {
        const T* qp = Q + ((int64_t)bh * R + row) * kD;
#pragma unroll
        for (int d = 0; d < kD; d += 8) load8(qp + d, q + d);
    } else {
#pragma unroll
        for (int d = 0; d < kD; ++d) q[d] = 0.f;
    }

    float mx = -INFINITY, sum = 0.f;
    const int t_begin = c * chunk, t_end = min(N, t_begin + chunk);
    const int last = P + i;                       // last token this row may see
    for (int t0 = t_begin; t0 < t_end; t0 += kStatTile) {
        for (int g8 = threadIdx.x; g8 < kStatTile * (kD / 8); g8 += blockDim.x) {
            int tt = g8 >> 4, f8 = (g8 & 15) * 8;
            float v[8];
            if (t0 + tt < t_end) {
                load8(Kh + (int64_t)(t0 + tt) * ks_t + f8, v);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = 0.f;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) kt[tt][f8 + e] = v[e];
        }
        __syncthreads();
        if (live) {
            const int n_here = min(kStatTile, min(t_end, last + 1) - t0);
            for (int tt = 0; tt < n_here; ++tt) {
                float acc = 0.f;
#pragma unroll
                for (int d = 0; d < kD; ++d) acc = fmaf(q[d], kt[tt][d], acc);
                const float s = acc * scale2;
                if (s > mx) {
                    sum = sum * exp2f(mx - s) + 1.f;
                    mx = s;
                } else {
                    sum += exp2f(s - mx);
                }
            }
        }
        __syncthreads();
    }
    if (live) stats[((int64_t)bh * n_chunks + c) * R + row] = make_float2(mx, sum);
}

// merge: one thread per (head, row)
__global__ __launch_bounds__(256) void score_lse_kernel(const float2* __restrict__ stats, int n_rows_total,
                                                        int R, int n_chunks, float* __restrict__ lse) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_rows_total) return;
    const int bh = e / R, row = e % R;
    const float2* st = stats + (int64_t)bh * n_chunks * R + row;
    float mx = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) mx = fmaxf(mx, st[(int64_t)c * R].x);
    float sum = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        float2 v = st[(int64_t)c * R];
        if (v.y > 0.f) sum += v.y * exp2f(v.x - mx);
    }
    lse[e] = mx + log2f(sum);
}

// ---------------------------------------------------------------------------------------
// pass 2, plain ALU: one thread per prefix token, the token's key in registers, query rows
// and their normalisers broadcast from LDS, one query head at a time.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void score_vote_alu_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const float* __restrict__ lse, int H, int G,
    int N, int w, int64_t ks_b, int64_t ks_h, int64_t ks_t, int n_tiles, float* __restrict__ vote) {
    __shared__ float qs[kVoteRows][kD];
    __shared__ float ls[kVoteRows];
    const int bh = blockIdx.x / n_tiles, tile = blockIdx.x % n_tiles;
    const int b = bh / H, h = bh % H;
    const int R = G * w, P = N - w;
    const int j = tile * 256 + threadIdx.x;
    const bool live = j < P;
    const float scale2 = kLog2e * rsqrtf((float)kD);

    float k[kD];
    if (live) {
        const T* kp = K + b * ks_b + h * ks_h + (int64_t)j * ks_t;
#pragma unroll
        for (int d = 0; d < kD; d += 8) load8(kp + d, k + d);
    } else {
#pragma unroll
        for (int d = 0; d < kD; ++d) k[d] = 0.f;
    }

    for (int g = 0; g < G; ++g) {
        float v = 0.f;
        for (int r0 = 0; r0 < w; r0 += kVoteRows) {
            const int nr = min(kVoteRows, w - r0);
            for (int g8 = threadIdx.x; g8 < nr * (kD / 8); g8 += 256) {
                int rr = g8 >> 4, f8 = (g8 & 15) * 8;
                float tmp[8];
                load8(Q + ((int64_t)bh * R + g * w + r0 + rr) * kD + f8, tmp);
#pragma unroll
                for (int e = 0; e < 8; ++e) qs[rr][f8 + e] = tmp[e];
            }
            if (threadIdx.x < nr) ls[threadIdx.x] = lse[(int64_t)bh * R + g * w + r0 + threadIdx.x];
            __syncthreads();
            for (int rr = 0; rr < nr; ++rr) {
                float acc = 0.f;
#pragma unroll
                for (int d = 0; d < kD; ++d) acc = fmaf(k[d], qs[rr][d], acc);
                v += exp2f(acc * scale2 - ls[rr]);
            }
            __syncthreads();
        }
        if (live) vote[((int64_t)bh * G + g) * P + j] = v;
    }
}

// pool + group sum: one thread per prefix token
__global__ __launch_bounds__(256) void score_pool_kernel(const float* __restrict__ vote, int G, int P,
                                                         int half, int n_tiles, float* __restrict__ score) {
    const int bh = blockIdx.x / n_tiles, tile = blockIdx.x % n_tiles;
    const int j = tile * 256 + threadIdx.x;
    if (j >= P) return;
    const int lo = max(0, j - half), hi = min(P - 1, j + half);
    float total = 0.f;
    for (int g = 0; g < G; ++g) {
        const float* vg = vote + ((int64_t)bh * G + g) * P;
        float mx = vg[lo];
        for (int jj = lo + 1; jj <= hi; ++jj) mx = fmaxf(mx, vg[jj]);
        total += mx;
    }
    score[(int64_t)bh * P + j] = total;
}

ScorePlan plan_score(int B, int H, int G, int N, int w) {
    ScorePlan p;
    const int BH = B * H;
    p.R = G * w;
    int max_chunks = N / 2048 > 0 ? N / 2048 : 1;
    int want = (2048 + BH - 1) / (BH > 0 ? BH : 1);
    int nc = want < 1 ? 1 : want;
    if (nc > max_chunks) nc = max_chunks;
    int chunk = (N + nc - 1) / nc;
    chunk = (chunk + 255) / 256 * 256;
    nc = (N + chunk - 1) / chunk;
    p.n_chunks = nc;
    p.chunk = chunk;
    const size_t P = (size_t)(N - w);
    p.stats_off = 0;
    p.lse_off = align_up((size_t)BH * nc * p.R * sizeof(float2), 256);
    p.vote_off = p.lse_off + align_up((size_t)BH * p.R * sizeof(float), 256);
    p.bytes = p.vote_off + align_up((size_t)BH * G * P * sizeof(float), 256);
    return p;
}

template <typename T>
static hipError_t run_score(const T* Q, const T* K, int B, int H, int G, int N, int w, int pool,
                            const int64_t ks[3], const ScorePlan& p, char* ws, float* score_out,
                            const Env& env) {
    hipStream_t s = env.s;
    const int BH = B * H, P = N - w;
    float2* stats = reinterpret_cast<float2*>(ws + p.stats_off);
    float* lse = reinterpret_cast<float*>(ws + p.lse_off);
    float* vote = reinterpret_cast<float*>(ws + p.vote_off);
    const int threads1 = (p.R + 63) / 64 * 64;
    env.begin("score_stats_alu");
    score_stats_alu_kernel<T><<<dim3((unsigned)(BH * p.n_chunks)), dim3(threads1), 0, s>>>(
        Q, K, H, G, N, w, ks[0], ks[1], ks[2], p.n_chunks, p.chunk, stats);
    env.end();
    const int rows = BH * p.R;
    env.begin("score_lse");
    score_lse_kernel<<<dim3((rows + 255) / 256), dim3(256), 0, s>>>(stats, rows, p.R, p.n_chunks, lse);
    env.end();
    const int n_tiles = (P + 255) / 256;
    env.begin("score_vote_alu");
    score_vote_alu_kernel<T><<<dim3((unsigned)(BH * n_tiles)), dim3(256), 0, s>>>(
        Q, K, lse, H, G, N, w, ks[0], ks[1], ks[2], n_tiles, vote);
    env.end();
    env.begin("score_pool");
    score_pool_kernel<<<dim3((unsigned)(BH * n_tiles)), dim3(256), 0, s>>>(vote, G, P, pool / 2, n_tiles,
                                                                          score_out);
    env.end();
    return hipGetLastError();
}

hipError_t launch_window_score(const void* Q, const void* K, uncomp_dtype dt, int B, int H, int G,
                               int N, int w, int pool, const int64_t ks[3], const ScorePlan& p,
                               char* ws, float* score_out, const Env& env) {
    if (dt == UNCOMP_BF16)
        return run_score<bf16_bits>(static_cast<const bf16_bits*>(Q), static_cast<const bf16_bits*>(K), B, H,
                                    G, N, w, pool, ks, p, ws, score_out, env);
    return run_score<float>(static_cast<const float*>(Q), static_cast<const float*>(K), B, H, G, N, w,
                            pool, ks, p, ws, score_out, env);
}

}  // namespace uncomp
