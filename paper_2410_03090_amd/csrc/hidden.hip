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


// ---- bf16: the last token's attention on the matrix cores -----------------------------------
// Every wave owns WR consecutive positions of one KV head and runs on its own: keys stream into MFMA
// operand layout, the G queries of the last position are the other operand, the wave takes its own
// maximum and sum per query head and leaves the unnormalised probabilities (rows of GT floats, via
// LDS so that the stores are whole rows) and (maximum, sum) in the workspace.
template <int GT, int WR>
__global__ __launch_bounds__(256) void lasttoken_attend_wave_kernel(
    const bf16_bits* __restrict__ q, const bf16_bits* __restrict__ K, int BH, int H, int G, int N, int64_t ks_b,
    int64_t ks_h, int64_t ks_t, int np, int s_rows, float* __restrict__ ws_p, float2* __restrict__ ws_ml) {
    constexpr int kTiles = WR / 16;
    extern __shared__ __align__(16) float pl_all[];                 // [4 waves][WR][GT]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int c16 = lane & 15, j = lane >> 4;
    const int wid = blockIdx.x * 4 + wv;
    const int bh = wid / np, part = wid - bh * np;
    if (bh >= BH) return;
    const int row0 = part * WR;
    if (row0 >= N) return;                                          // waves run on their own: no barrier below
    const int n_t = min(kTiles, (N - row0 + 15) >> 4);
    float* pl = pl_all + wv * WR * GT;
    const bf16_bits* Kh = K + (bh / H) * ks_b + (bh % H) * ks_h;
    bf16x8_t qb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (c16 < G) v = *reinterpret_cast<const uint4*>(q + ((int64_t)bh * G + c16) * kD + 32 * ks + 8 * j);
        qb[ks] = __builtin_bit_cast(bf16x8_t, v);
    }
    auto load_k = [&](uint4 dst[4], int t) {                        // clamped, never predicated
        const int r = min(row0 + 16 * t + c16, N - 1);
        const bf16_bits* src = Kh + (int64_t)r * ks_t + 8 * j;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dst[ks] = *reinterpret_cast<const uint4*>(src + 32 * ks);
    };
    f32x4_t s[kTiles];
    uint4 ka[4], kb[4];
    auto dots = [&](const uint4 kt[4], int t) {
        f32x4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kt[ks]), qb[ks], c, 0, 0, 0);
        s[t] = c;
    };
    load_k(ka, 0);
#pragma unroll
    for (int t = 0; t < kTiles; t += 2) {
        if (t < n_t) {
            load_k(kb, t + 1);
            dots(ka, t);
        }
        if (t + 1 < n_t) {
            load_k(ka, t + 2);
            dots(kb, t + 1);
        }
    }
    const float qs = 0.08838834764831845f * 1.4426950408889634f;    // 1/sqrt(128) * log2(e)
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
        if (t < n_t) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool live = row0 + 16 * t + 4 * j + v < N;
                s[t][v] = live ? s[t][v] * qs : -INFINITY;
                mx = fmaxf(mx, s[t][v]);
            }
        }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));                         // row0 < N: at least one live row
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
        if (t < n_t) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float e = exp2f(s[t][v] - mx);
                sum += e;
                if (c16 < GT) pl[(16 * t + 4 * j + v) * GT + c16] = e;
            }
        }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    if (j == 0 && c16 < G) ws_ml[((int64_t)bh * np + part) * GT + c16] = make_float2(mx, sum);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float* dst = ws_p + ((int64_t)bh * s_rows + row0) * GT;
    const int n_f4 = n_t * 16 * GT / 4;
    for (int i = lane; i < n_f4; i += 64) reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(pl)[i];
}

// One wave per (head, query head): the head's maximum M and 1 / sum over the parts -> head[bh][g] = (M, 1/L).
__global__ __launch_bounds__(256) void lasttoken_head_kernel(const float2* __restrict__ ws_ml, int BH, int G, int GT,
                                                             int np, float2* __restrict__ head) {
    const int wid = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (wid >= BH * G) return;
    const int bh = wid / G, g = wid - bh * G;
    const float2* ml = ws_ml + (int64_t)bh * np * GT + g;
    float m = -INFINITY;
    for (int p = lane; p < np; p += 64) m = fmaxf(m, ml[(int64_t)p * GT].x);
    m = wave_max(m);
    float l = 0.f;
    for (int p = lane; p < np; p += 64) {
        const float2 v = ml[(int64_t)p * GT];
        l += v.y * exp2f(v.x - m);
    }
    l = wave_sum(l);
    if (lane == 0) head[(int64_t)bh * GT + g] = make_float2(m, 1.0f / l);
}

// out[b][j] = sum over the KV heads h and their query heads g of p[bh][j][g] * 2^(m_part - M) / L, j < P_out.
template <int GT>
__global__ __launch_bounds__(256) void lasttoken_merge_kernel(const float* __restrict__ ws_p,
                                                              const float2* __restrict__ ws_ml,
                                                              const float2* __restrict__ head, int H, int G, int np,
                                                              int wave_rows, int s_rows, int P_out,
                                                              float* __restrict__ out) {
    const int b = blockIdx.y;
    const int jpos = blockIdx.x * 256 + threadIdx.x;
    if (jpos >= P_out) return;
    const int part = jpos / wave_rows;
    float acc = 0.f;
    for (int h = 0; h < H; ++h) {
        const int bh = b * H + h;
        const float* pr = ws_p + ((int64_t)bh * s_rows + jpos) * GT;
        const float2* ml = ws_ml + ((int64_t)bh * np + part) * GT;
        const float2* hd = head + (int64_t)bh * GT;
        float a = 0.f;
#pragma unroll
        for (int g = 0; g < GT; ++g)
            if (g < G) a += pr[g] * (exp2f(ml[g].x - hd[g].x) * hd[g].y);
        acc += a;
    }
    out[(int64_t)b * P_out + jpos] = acc;
}

LastTokenPlan plan_last_token(int B, int H, int G, int N) {
    LastTokenPlan p;
    p.GT = G <= 4 ? 4 : (G <= 8 ? 8 : 16);
    const int64_t waves256 = (int64_t)B * H * ((N + 255) / 256);
    p.wave_rows = (p.GT <= 8 && waves256 >= 2048) ? 256 : 128;
    p.s_rows = (N + p.wave_rows - 1) / p.wave_rows * p.wave_rows;
    p.np = p.s_rows / p.wave_rows;
    size_t off = 0;
    p.p_off = off;
    off = align_up(off + (size_t)B * H * p.s_rows * p.GT * sizeof(float), 256);
    p.ml_off = off;
    off = align_up(off + (size_t)B * H * p.np * p.GT * sizeof(float2), 256);
    p.head_off = off;
    off = align_up(off + (size_t)B * H * p.GT * sizeof(float2), 256);
    p.bytes = off;
    return p;
}

template <int GT, int WR>
static hipError_t last_token_score_t(const bf16_bits* q, const bf16_bits* K, int B, int H, int G, int N,
                                     const int64_t ks[3], int P_out, const LastTokenPlan& p, char* ws, float* out,
                                     const Env& env) {
    float* ws_p = reinterpret_cast<float*>(ws + p.p_off);
    float2* ws_ml = reinterpret_cast<float2*>(ws + p.ml_off);
    float2* head = reinterpret_cast<float2*>(ws + p.head_off);
    const int BH = B * H;
    const int64_t waves = (int64_t)BH * p.np;
    env.begin("lasttoken_attend_wave");
    lasttoken_attend_wave_kernel<GT, WR><<<dim3((unsigned)((waves + 3) / 4)), dim3(256), (size_t)4 * WR * GT * sizeof(float),
                                          env.s>>>(q, K, BH, H, G, N, ks[0], ks[1], ks[2], p.np, p.s_rows, ws_p, ws_ml);
    env.end();
    env.begin("lasttoken_merge");
    lasttoken_head_kernel<<<dim3((unsigned)((BH * G + 3) / 4)), dim3(256), 0, env.s>>>(ws_ml, BH, G, GT, p.np, head);
    lasttoken_merge_kernel<GT><<<dim3((unsigned)((P_out + 255) / 256), (unsigned)B), dim3(256), 0, env.s>>>(
        ws_p, ws_ml, head, H, G, p.np, WR, p.s_rows, P_out, out);
    env.end();
    return hipGetLastError();
}

// score[b][j], j < P_out, of the last position's queries q [B][H*G][128] over the N keys of each head (bf16).
hipError_t launch_last_token_score(const void* q, const void* K, int B, int H, int G, int N, const int64_t ks[3],
                                   int P_out, const LastTokenPlan& p, char* ws, float* out, const Env& env) {
    const bf16_bits* qq = static_cast<const bf16_bits*>(q);
    const bf16_bits* kk = static_cast<const bf16_bits*>(K);
#define UNCOMP_LT_CASE(GT, WR) return last_token_score_t<GT, WR>(qq, kk, B, H, G, N, ks, P_out, p, ws, out, env)
    if (p.wave_rows == 256) {
        if (p.GT == 4) UNCOMP_LT_CASE(4, 256);
        UNCOMP_LT_CASE(8, 256);
    }
    if (p.GT == 4) UNCOMP_LT_CASE(4, 128);
    if (p.GT == 8) UNCOMP_LT_CASE(8, 128);
    UNCOMP_LT_CASE(16, 128);
#undef UNCOMP_LT_CASE
}

hipError_t launch_head_sum(const float* score, int B, int H, int P_in, int P_out, float* out, const Env& env) {
    env.begin("head_sum");
    head_sum_kernel<<<dim3((unsigned)((P_out + 255) / 256), (unsigned)B), dim3(256), 0, env.s>>>(score, H, P_in,
                                                                                               P_out, out);
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
