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
#include "score_stats_body.h"

namespace uncomp {

namespace {
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
    const T* __restrict__ Q, const T* __restrict__ K, int H, int G, int N, int D, int w, int64_t ks_b,
    int64_t ks_h, int64_t ks_t, int n_chunks, int chunk, float2* __restrict__ stats) {
    __shared__ float kt[kStatTile][kD];
    const int bh = blockIdx.x / n_chunks, c = blockIdx.x % n_chunks;
    const int b = bh / H, h = bh % H;
    const int R = G * w, P = N - w;
    const int row = threadIdx.x;
    const bool live = row < R;
    const int i = live ? row % w : 0;
    const T* Kh = K + b * ks_b + h * ks_h;
    const float scale2 = kLog2e * rsqrtf((float)D);

    float q[kD];                                 // features beyond D (a 64-wide head) are zeros on both sides
#pragma unroll
    for (int d = 0; d < kD; ++d) q[d] = 0.f;
    if (live) {
        const T* qp = Q + ((int64_t)bh * R + row) * D;
#pragma unroll
        for (int d = 0; d < kD; d += 8)
            if (d < D) load8(qp + d, q + d);
    }

    float mx = -INFINITY, sum = 0.f;
    const int t_begin = c * chunk, t_end = min(N, t_begin + chunk);
    const int last = P + i;                       // last token this row may see
    for (int t0 = t_begin; t0 < t_end; t0 += kStatTile) {
        for (int g8 = threadIdx.x; g8 < kStatTile * (kD / 8); g8 += blockDim.x) {
            int tt = g8 >> 4, f8 = (g8 & 15) * 8;
            float v[8];
            if (t0 + tt < t_end && f8 < D) {
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

// ---------------------------------------------------------------------------------------
// Pass 1 for a one-token window (w = 1: the last token's attention, R = G rows per head).  The
// kernel above gives a thread to every query row, which leaves most of the machine idle when
// there are only G of them; here the tokens are spread over the threads instead: 16 lanes read
// one key row (8 features each), the G queries sit in registers, dot products are closed with
// DPP row rotations and every group of 16 lanes keeps running (maximum, sum) pairs that are
// merged at the end.  Same output layout as the kernel above.
// ---------------------------------------------------------------------------------------
template <typename T, int GT>
__global__ __launch_bounds__(256) void score_stats_lastrow_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, int H, int G, int N, int D, int64_t ks_b, int64_t ks_h,
    int64_t ks_t, int n_chunks, int chunk, float2* __restrict__ stats) {
    __shared__ float2 part[16][GT];
    const int bh = blockIdx.x / n_chunks, c = blockIdx.x % n_chunks;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, sub = tid & 15, rg = tid >> 4;
    const T* Kh = K + b * ks_b + h * ks_h;
    const float scale2 = kLog2e * rsqrtf((float)D);
    const bool has = 8 * sub < D;                 // lanes whose eight features lie beyond D hold zeros
    float qf[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        if (g < G && has) {
            load8(Q + ((int64_t)bh * G + g) * D + 8 * sub, qf[g]);
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[g][e] *= scale2;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[g][e] = 0.f;
        }
    }
    float mx[GT], sum[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        mx[g] = -INFINITY;
        sum[g] = 0.f;
    }
    const int t_begin = c * chunk, t_end = min(N, t_begin + chunk);
    constexpr int U = 4;
    for (int t0 = t_begin; t0 < t_end; t0 += 16 * U) {
        float kv[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = min(t0 + 16 * u + rg, t_end - 1);          // clamped, never predicated
            load8(Kh + (int64_t)t * ks_t + (has ? 8 * sub : 0), kv[u]);   // lanes beyond D re-read the first piece; their queries are zero
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool live = t0 + 16 * u + rg < t_end;
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d = fmaf(qf[g][e], kv[u][e], d);
                d += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(d), 0x128, 0xF, 0xF, false));
                d += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(d), 0x124, 0xF, 0xF, false));
                d += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(d), 0x122, 0xF, 0xF, false));
                d += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(d), 0x121, 0xF, 0xF, false));
                if (live) {
                    const float m_new = fmaxf(mx[g], d);
                    sum[g] = sum[g] * exp2f(mx[g] - m_new) + exp2f(d - m_new);
                    mx[g] = m_new;
                }
            }
        }
    }
    if (sub == 0) {
#pragma unroll
        for (int g = 0; g < GT; ++g) part[rg][g] = make_float2(mx[g], sum[g]);
    }
    __syncthreads();
    if (tid < G) {
        float m = -INFINITY;
        for (int r = 0; r < 16; ++r) m = fmaxf(m, part[r][tid].x);
        float l = 0.f;
        for (int r = 0; r < 16; ++r) {
            const float2 pr = part[r][tid];
            if (pr.y > 0.f) l += pr.y * exp2f(pr.x - m);               // groups that saw no token hold (-inf, 0)
        }
        stats[((int64_t)bh * n_chunks + c) * G + tid] = make_float2(m, l);
    }
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernels.  Logits S = Q K^T contract over the 128 features, which are contiguous
// in memory, so both operands of v_mfma_f32_16x16x32_bf16 load straight from rows.  Both
// passes use the same barrier-free streaming scheme: the query rows of the KV head sit in
// LDS for the whole kernel (rows padded by 16 bytes so that eight consecutive lanes of a
// 128-bit read hit distinct banks) and are re-read per 64-token tile; every wave streams its
// own key tiles straight from global memory in operand layout (lane = token lane%16 of a
// 16-token sub-tile, features 32ks + 8*(lane/16)..), double-buffered in registers.  Key loads
// are clamped to the last valid token instead of predicated: straight-line loads let the
// compiler keep exact counts of the loads in flight (a predicated load makes it wait for all
// of them), and whatever a token past the end contributes is masked or never stored.
// ---------------------------------------------------------------------------------------

// pass 1 without barriers: same streaming scheme as the vote kernel below (queries in LDS, every
// wave streams its own key tiles), with the MFMA operands swapped so that an accumulator lane
// holds ONE query row (lane%16 of the block) and 16 tokens of the tile: a row's running
// (reference, sum of exp2) is then a single pair of registers per block, updated once per tile.
// Every wave writes its own partial statistics (4 per chunk); the merge kernel combines them.
template <int NRB>     // 16-row blocks the LDS and the per-lane state are sized for
__global__ __launch_bounds__(256, 2) void score_stats_wave_kernel(
    const bf16_bits* __restrict__ Q, const bf16_bits* __restrict__ K, int H, int R, int N, int w,
    int64_t ks_b, int64_t ks_h, int64_t ks_t, int n_chunks, int chunk, float2* __restrict__ stats) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* qs = smem;                                             // [16*NRB][kRowBytes]
    const int bh = blockIdx.x / n_chunks, c = blockIdx.x % n_chunks;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const bf16_bits* Qh = Q + (int64_t)bh * R * kD;
    for (int idx = tid; idx < 16 * NRB * 16; idx += 256) {
        const int row = idx >> 4, piece = idx & 15;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row < R) v = *reinterpret_cast<const uint4*>(Qh + (int64_t)row * kD + piece * 8);
        *reinterpret_cast<uint4*>(qs + row * kRowBytes + piece * 16) = v;
    }
    __syncthreads();
    const int t_begin = c * chunk, t_end = min(N, t_begin + chunk);
    score_stats_wave_body<NRB>(qs, K + b * ks_b + h * ks_h, ks_t, t_begin, t_end, N - w, w, R, wv, lane,
                               stats + ((int64_t)bh * (n_chunks * 4) + c * 4 + wv) * R);
}
template <int NRB, bool W8 = false>     // LDS is sized for 16*NRB query rows; W8: the window is 8 positions
__global__ __launch_bounds__(256) void score_vote_wave_kernel(
    const bf16_bits* __restrict__ Q, const bf16_bits* __restrict__ K, const float* __restrict__ lse, int H,
    int G, int N, int w, int64_t ks_b, int64_t ks_h, int64_t ks_t, int n_chunks, int chunk,
    float* __restrict__ vote) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* qs = smem;                                             // [16*NRB][kRowBytes]
    float* nls = reinterpret_cast<float*>(smem + 16 * NRB * kRowBytes);   // [16*NRB] minus lse (base 2)
    const int bh = blockIdx.x / n_chunks, c = blockIdx.x % n_chunks;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int R = G * w, P = N - w;
    const int n_rb = R >> 4, bph = w >> 4;          // 16-row blocks per KV head / per query head
    const bf16_bits* Kh = K + b * ks_b + h * ks_h;
    const float scale2 = kLog2e * rsqrtf((float)kD);
    const int t_begin = c * chunk, t_end = min(P, t_begin + chunk);
    if (t_begin >= t_end) return;
    const int n_tiles = (t_end - t_begin + kTile - 1) / kTile;

    const bf16_bits* Qh = Q + (int64_t)bh * R * kD;
    for (int idx = tid; idx < 16 * NRB * 16; idx += 256) {
        const int row = idx >> 4, piece = idx & 15;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row < R) v = *reinterpret_cast<const uint4*>(Qh + (int64_t)row * kD + piece * 8);
        *reinterpret_cast<uint4*>(qs + row * kRowBytes + piece * 16) = v;
    }
    for (int r = tid; r < 16 * NRB; r += 256) nls[r] = r < R ? -lse[(int64_t)bh * R + r] : 0.f;
    __syncthreads();

    float* vote_h = vote + (int64_t)bh * G * P;
    uint4 ka[4][4], kb[4][4];                        // [sub-tile][k-step] B operands of two tiles
    auto load_tile = [&](uint4 dst[4][4], int tile) {            // clamped, never predicated
        const int t0 = t_begin + tile * kTile;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const int tok = min(t0 + 16 * st + m, t_end - 1);
            const bf16_bits* src = Kh + (int64_t)tok * ks_t + 8 * g;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) dst[st][ks] = *reinterpret_cast<const uint4*>(src + 32 * ks);
        }
    };
    struct RowBlock { bf16x8_t a[4]; float4 nl; };     // A operands and normalisers of one 16-row block
    auto read_block = [&](RowBlock& rbk, int rb) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            rbk.a[ks] = __builtin_bit_cast(
                bf16x8_t, *reinterpret_cast<const uint4*>(qs + (16 * rb + m) * kRowBytes + 64 * ks + 16 * g));
        rbk.nl = *reinterpret_cast<const float4*>(nls + 16 * rb + 4 * g);
    };
    auto process = [&](const uint4 cur[4][4], uint4 nxt[4][4], int tile) {
        load_tile(nxt, tile + 4);
        const int t0 = t_begin + tile * kTile;
        float pq[4] = {0.f, 0.f, 0.f, 0.f};          // per sub-tile: this lane's rows of the current query head
        int in_head = 0, qh = 0;
        auto step = [&](const RowBlock& rbk) {
            f32x4_t acc[4];
#pragma unroll
            for (int st = 0; st < 4; ++st) acc[st] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            __builtin_amdgcn_s_setprio(1);                        // matrix work first: the partner wave fills the gaps
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int st = 0; st < 4; ++st)
                    acc[st] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        rbk.a[ks], __builtin_bit_cast(bf16x8_t, cur[st][ks]), acc[st], 0, 0, 0);
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int st = 0; st < 4; ++st)
                pq[st] += (__builtin_amdgcn_exp2f(fmaf(acc[st][0], scale2, rbk.nl.x)) +
                           __builtin_amdgcn_exp2f(fmaf(acc[st][1], scale2, rbk.nl.y))) +
                          (__builtin_amdgcn_exp2f(fmaf(acc[st][2], scale2, rbk.nl.z)) +
                           __builtin_amdgcn_exp2f(fmaf(acc[st][3], scale2, rbk.nl.w)));
            if constexpr (W8) {
                // two query heads per row block (rows 0-7 and 8-15, i.e. lane rows 0,1 and 2,3): one
                // v_permlane16_swap per pair of sub-tiles adds the lane rows pairwise; lane row g then holds
                // head 2 rb + g / 2, sub-tile g % 2 (first pair) resp. 2 + g % 2 (second pair)
                auto s01 = __builtin_amdgcn_permlane16_swap(__float_as_uint(pq[0]), __float_as_uint(pq[1]), false, false);
                auto s23 = __builtin_amdgcn_permlane16_swap(__float_as_uint(pq[2]), __float_as_uint(pq[3]), false, false);
                const float t01 = __uint_as_float(s01[0]) + __uint_as_float(s01[1]);
                const float t23 = __uint_as_float(s23[0]) + __uint_as_float(s23[1]);
                const int head = 2 * qh + (g >> 1);
                const int j01 = t0 + 16 * (g & 1) + m, j23 = j01 + 32;
                if (j01 < t_end) vote_h[(int64_t)head * P + j01] = t01;
                if (j23 < t_end) vote_h[(int64_t)head * P + j23] = t23;
                pq[0] = pq[1] = pq[2] = pq[3] = 0.f;
                ++qh;                                 // counts row blocks here
            } else if (++in_head == bph) {
                // lane group g now receives the total of sub-tile {0,2,1,3}[g]
                const float tot = reduce4_over_rows(pq[0], pq[1], pq[2], pq[3]);
                const int j = t0 + 16 * (((g & 1) << 1) | (g >> 1)) + m;
                if (j < t_end) vote_h[(int64_t)qh * P + j] = tot;
                pq[0] = pq[1] = pq[2] = pq[3] = 0.f;
                in_head = 0;
                ++qh;
            }
        };
        // fully unrolled over the row blocks, so that the scheduler can run the MFMAs of one
        // block under the exp2 work of the previous one
        RowBlock blk;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            if (rb < n_rb) {
                read_block(blk, rb);
                step(blk);
            }
        }
    };
    load_tile(ka, wv);
    for (int tile = wv; tile < n_tiles; tile += 8) {
        process(ka, kb, tile);
        if (tile + 4 < n_tiles) process(kb, ka, tile + 4);
    }
}

// normalisers handed in by the caller (natural log) -> the base-2 ones the vote pass reads
__global__ __launch_bounds__(256) void score_lse_import_kernel(const float* __restrict__ lse_nat, int n,
                                                               float* __restrict__ lse) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) lse[e] = lse_nat[e] * kLog2e;
}

// merge of the partial (maximum, sum) pairs of every query row: a workgroup takes 64 rows, four threads per row
// each fold every fourth partial (four loads in flight; with a layer's few heads there are hundreds of partials
// per row and one thread walking them all was 114 us of latency), then the four are folded in order.
__device__ __forceinline__ void lse_fold(float& m, float& sum, float2 v) {
    if (v.y > 0.f) {
        const float M = fmaxf(m, v.x);
        sum = sum * exp2f(m - M) + v.y * exp2f(v.x - M);         // m = -inf, sum = 0 at the start: 0 * 0 + ...
        m = M;
    }
}
__global__ __launch_bounds__(256) void score_lse_kernel(const float2* __restrict__ stats, int n_rows_total,
                                                        int R, int n_chunks, float* __restrict__ lse) {
    __shared__ float2 part[3][64];
    const int i = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + i;
    float m = -INFINITY, sum = 0.f;
    if (e < n_rows_total) {
        const int bh = e / R, row = e % R;
        const float2* st = stats + (int64_t)bh * n_chunks * R + row;
        int c = q;
        for (; c + 12 < n_chunks; c += 16) {
            const float2 v0 = st[(int64_t)c * R], v1 = st[(int64_t)(c + 4) * R];
            const float2 v2 = st[(int64_t)(c + 8) * R], v3 = st[(int64_t)(c + 12) * R];
            lse_fold(m, sum, v0);
            lse_fold(m, sum, v1);
            lse_fold(m, sum, v2);
            lse_fold(m, sum, v3);
        }
        for (; c < n_chunks; c += 4) lse_fold(m, sum, st[(int64_t)c * R]);
    }
    if (q > 0) part[q - 1][i] = make_float2(m, sum);
    __syncthreads();
    if (q == 0 && e < n_rows_total) {
#pragma unroll
        for (int x = 0; x < 3; ++x) lse_fold(m, sum, part[x][i]);
        lse[e] = m + log2f(sum);
    }
}

// ---------------------------------------------------------------------------------------
// pass 2, plain ALU: one thread per prefix token, the token's key in registers, query rows
// and their normalisers broadcast from LDS, one query head at a time.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void score_vote_alu_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const float* __restrict__ lse, int H, int G,
    int N, int D, int w, int64_t ks_b, int64_t ks_h, int64_t ks_t, int n_tiles, float* __restrict__ vote) {
    __shared__ float qs[kVoteRows][kD];
    __shared__ float ls[kVoteRows];
    const int bh = blockIdx.x / n_tiles, tile = blockIdx.x % n_tiles;
    const int b = bh / H, h = bh % H;
    const int R = G * w, P = N - w;
    const int j = tile * 256 + threadIdx.x;
    const bool live = j < P;
    const float scale2 = kLog2e * rsqrtf((float)D);

    float k[kD];                                 // features beyond D (a 64-wide head) are zeros on both sides
#pragma unroll
    for (int d = 0; d < kD; ++d) k[d] = 0.f;
    if (live) {
        const T* kp = K + b * ks_b + h * ks_h + (int64_t)j * ks_t;
#pragma unroll
        for (int d = 0; d < kD; d += 8)
            if (d < D) load8(kp + d, k + d);
    }

    for (int g = 0; g < G; ++g) {
        float v = 0.f;
        for (int r0 = 0; r0 < w; r0 += kVoteRows) {
            const int nr = min(kVoteRows, w - r0);
            for (int g8 = threadIdx.x; g8 < nr * (kD / 8); g8 += 256) {
                int rr = g8 >> 4, f8 = (g8 & 15) * 8;
                float tmp[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                if (f8 < D) load8(Q + ((int64_t)bh * R + g * w + r0 + rr) * D + f8, tmp);
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

// pool + group sum.  A workgroup takes 1024 consecutive tokens of one KV head; the votes of up
// to four query heads at a time (plus HALF tokens either side, -inf outside [0, P)) are staged
// in LDS (one 16-byte load per thread where the row allows it), each thread forms the running
// maxima of four consecutive tokens from 4 + 2*HALF staged values per query head and adds them.
constexpr int kPoolTile = 1024;

template <int HALF>
__global__ __launch_bounds__(256) void score_pool_kernel(const float* __restrict__ vote, int G, int P,
                                                         int n_tiles, float* __restrict__ score,
                                                         uint32_t* __restrict__ tile_range) {
    __shared__ float sh[4][kPoolTile + 2 * HALF + 4];
    __shared__ uint32_t wave_range[4][2];
    const int bh = blockIdx.x / n_tiles, tile = blockIdx.x % n_tiles;
    const int tile0 = tile * kPoolTile;
    const int tid = threadIdx.x;
    const bool vec = (P & 3) == 0;               // rows start 16-byte aligned
    float total[4] = {0.f, 0.f, 0.f, 0.f};
    for (int g0 = 0; g0 < G; g0 += 4) {
        const int ng = min(4, G - g0);
        for (int gi = 0; gi < ng; ++gi) {
            const float* vg = vote + ((int64_t)bh * G + g0 + gi) * P;
            const int j = tile0 + 4 * tid;
            float4 v = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (vec && j + 3 < P) {
                v = *reinterpret_cast<const float4*>(vg + j);
            } else {
                if (j < P) v.x = vg[j];
                if (j + 1 < P) v.y = vg[j + 1];
                if (j + 2 < P) v.z = vg[j + 2];
                if (j + 3 < P) v.w = vg[j + 3];
            }
            float* dst = &sh[gi][HALF + 4 * tid];
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
            if (tid < 2 * HALF) {                 // HALF tokens before and after the tile
                const int idx = tid < HALF ? tid : kPoolTile + tid;
                const int jh = tile0 - HALF + idx;
                sh[gi][idx] = (jh >= 0 && jh < P) ? vg[jh] : -INFINITY;
            }
        }
        __syncthreads();
        for (int gi = 0; gi < ng; ++gi) {
            float v[4 + 2 * HALF];
#pragma unroll
            for (int k = 0; k < 4 + 2 * HALF; ++k) v[k] = sh[gi][4 * tid + k];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float mx = v[e];
#pragma unroll
                for (int d = 1; d <= 2 * HALF; ++d) mx = fmaxf(mx, v[e + d]);
                total[e] += mx;
            }
        }
        __syncthreads();
    }
    // the tile's smallest and largest selection key ride along: the top-k kernel starts from them instead of
    // reading every score once more to find their range
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int j = tile0 + 4 * tid + e;
        if (j < P) {
            score[(int64_t)bh * P + j] = total[e];
            const uint32_t key = order_key(total[e]);
            kmin = key < kmin ? key : kmin;
            kmax = key > kmax ? key : kmax;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t a = __shfl_xor(kmin, o, 64), c = __shfl_xor(kmax, o, 64);
        kmin = a < kmin ? a : kmin;
        kmax = c > kmax ? c : kmax;
    }
    if ((tid & 63) == 0) {
        wave_range[tid >> 6][0] = kmin;
        wave_range[tid >> 6][1] = kmax;
    }
    __syncthreads();
    if (tid == 0) {
        for (int i = 1; i < 4; ++i) {
            kmin = wave_range[i][0] < kmin ? wave_range[i][0] : kmin;
            kmax = wave_range[i][1] > kmax ? wave_range[i][1] : kmax;
        }
        tile_range[((int64_t)bh * n_tiles + tile) * 2] = kmin;
        tile_range[((int64_t)bh * n_tiles + tile) * 2 + 1] = kmax;
    }
}

// staged query rows of the MFMA kernels: up to 128 / 256 rows per KV head
constexpr int kScoreLds8 = 16 * 8 * kRowBytes, kScoreLds16 = 16 * 16 * kRowBytes;

hipError_t init_score_kernels() {
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(score_stats_wave_kernel<8>), kScoreLds8);
    if (e == hipSuccess) e = allow_dynamic_lds(reinterpret_cast<const void*>(score_stats_wave_kernel<16>), kScoreLds16);
    if (e == hipSuccess) e = allow_dynamic_lds(reinterpret_cast<const void*>(score_vote_wave_kernel<8, true>), kScoreLds8 + 16 * 8 * 4);
    if (e == hipSuccess) e = allow_dynamic_lds(reinterpret_cast<const void*>(score_vote_wave_kernel<8, false>), kScoreLds8 + 16 * 8 * 4);
    if (e == hipSuccess) e = allow_dynamic_lds(reinterpret_cast<const void*>(score_vote_wave_kernel<16, true>), kScoreLds16 + 16 * 16 * 4);
    if (e == hipSuccess) e = allow_dynamic_lds(reinterpret_cast<const void*>(score_vote_wave_kernel<16, false>), kScoreLds16 + 16 * 16 * 4);
    return e;
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
    chunk = (chunk + 255) / 256 * 256;             // whole 64-token tiles
    nc = (N + chunk - 1) / chunk;
    p.n_chunks = nc;
    p.chunk = chunk;
    const size_t P = (size_t)(N - w);
    p.stats_off = 0;
    p.lse_off = align_up((size_t)BH * nc * 4 * p.R * sizeof(float2), 256);   // up to 4 partials per chunk
    p.vote_off = p.lse_off + align_up((size_t)BH * p.R * sizeof(float), 256);
    p.range_off = p.vote_off + align_up((size_t)BH * G * P * sizeof(float), 256);
    p.n_range_tiles = (int)((P + kPoolTile - 1) / kPoolTile);
    p.bytes = p.range_off + align_up((size_t)BH * p.n_range_tiles * 2 * sizeof(uint32_t), 256);
    return p;
}

template <typename T>
static hipError_t run_score(const T* Q, const T* K, int B, int H, int G, int N, int w, int pool,
                            const int64_t ks[3], const ScorePlan& p, char* ws, float* score_out,
                            const Env& env, bool mfma, const float* lse_nat, int D) {
    hipStream_t s = env.s;
    const int BH = B * H, P = N - w;
    float2* stats = reinterpret_cast<float2*>(ws + p.stats_off);
    float* lse = reinterpret_cast<float*>(ws + p.lse_off);
    float* vote = reinterpret_cast<float*>(ws + p.vote_off);
    uint32_t* tile_range = reinterpret_cast<uint32_t*>(ws + p.range_off);
    const dim3 grid1((unsigned)(BH * p.n_chunks));
    int n_parts = p.n_chunks;            // partial statistics per query row
    const int rows = BH * p.R;
    const bool own_stats = lse_nat == nullptr;
    if (!own_stats) {
        env.begin("score_lse_import");
        score_lse_import_kernel<<<dim3((rows + 255) / 256), dim3(256), 0, s>>>(lse_nat, rows, lse);
        env.end();
    }
    if constexpr (sizeof(T) == 2) {
        if (mfma && own_stats) {
            env.begin("score_stats_wave");
            if (p.R <= 128) {
                constexpr int lds_bytes = kScoreLds8;
                score_stats_wave_kernel<8><<<grid1, dim3(256), lds_bytes, s>>>(Q, K, H, p.R, N, w, ks[0], ks[1], ks[2],
                                                                               p.n_chunks, p.chunk, stats);
            } else {
                constexpr int lds_bytes = kScoreLds16;
                score_stats_wave_kernel<16><<<grid1, dim3(256), lds_bytes, s>>>(Q, K, H, p.R, N, w, ks[0], ks[1], ks[2],
                                                                                p.n_chunks, p.chunk, stats);
            }
            env.end();
            n_parts = p.n_chunks * 4;
        }
    }
    if (!own_stats) {
        // normalisers already in place
    } else if (!mfma && w == 1 && G <= 16) {
        env.begin("score_stats_lastrow");
        if (G <= 4)
            score_stats_lastrow_kernel<T, 4><<<grid1, dim3(256), 0, s>>>(Q, K, H, G, N, D, ks[0], ks[1], ks[2], p.n_chunks,
                                                                         p.chunk, stats);
        else if (G <= 8)
            score_stats_lastrow_kernel<T, 8><<<grid1, dim3(256), 0, s>>>(Q, K, H, G, N, D, ks[0], ks[1], ks[2], p.n_chunks,
                                                                         p.chunk, stats);
        else
            score_stats_lastrow_kernel<T, 16><<<grid1, dim3(256), 0, s>>>(Q, K, H, G, N, D, ks[0], ks[1], ks[2], p.n_chunks,
                                                                          p.chunk, stats);
        env.end();
    } else if (!mfma) {
        // This kernel writes one partial per chunk where the wave kernels write four: the statistics region has room
        // for chunks a quarter as long, which is what a short prompt needs to occupy more than a few CUs.
        int nca = 4 * p.n_chunks;
        if (nca > (N + 63) / 64) nca = (N + 63) / 64;
        const int chunk_a = ((N + nca - 1) / nca + kStatTile - 1) / kStatTile * kStatTile;
        nca = (N + chunk_a - 1) / chunk_a;
        const int threads1 = (p.R + 63) / 64 * 64;
        env.begin("score_stats_alu");
        score_stats_alu_kernel<T><<<dim3((unsigned)(BH * nca)), dim3(threads1), 0, s>>>(Q, K, H, G, N, D, w, ks[0], ks[1], ks[2],
                                                                                    nca, chunk_a, stats);
        env.end();
        n_parts = nca;
    }
    if (own_stats) {
        env.begin("score_lse");
        score_lse_kernel<<<dim3((rows + 63) / 64), dim3(256), 0, s>>>(stats, rows, p.R, n_parts, lse);
        env.end();
    }
    const int n_tiles = (P + 255) / 256;
    const int n_pool_tiles = (P + kPoolTile - 1) / kPoolTile;
    if constexpr (sizeof(T) == 2) {
        if (mfma) {
            env.begin("score_vote_wave");
            auto launch_vote = [&](auto kern, int lds_bytes) -> hipError_t {
                kern<<<grid1, dim3(256), lds_bytes, s>>>(Q, K, lse, H, G, N, w, ks[0], ks[1], ks[2], p.n_chunks, p.chunk, vote);
                return hipSuccess;
            };
            constexpr int lds8 = kScoreLds8 + 16 * 8 * 4, lds16 = kScoreLds16 + 16 * 16 * 4;
            hipError_t ve;
            if (w == 8) ve = p.R <= 128 ? launch_vote(score_vote_wave_kernel<8, true>, lds8) : launch_vote(score_vote_wave_kernel<16, true>, lds16);
            else ve = p.R <= 128 ? launch_vote(score_vote_wave_kernel<8, false>, lds8) : launch_vote(score_vote_wave_kernel<16, false>, lds16);
            if (ve != hipSuccess) return ve;
            env.end();
        }
    }
    if (!mfma) {
        env.begin("score_vote_alu");
        score_vote_alu_kernel<T><<<dim3((unsigned)(BH * n_tiles)), dim3(256), 0, s>>>(
            Q, K, lse, H, G, N, D, w, ks[0], ks[1], ks[2], n_tiles, vote);
        env.end();
    }
    env.begin("score_pool");
    {
        const dim3 pg((unsigned)(BH * n_pool_tiles)), pb(256);
        switch (pool / 2) {
            case 0: score_pool_kernel<0><<<pg, pb, 0, s>>>(vote, G, P, n_pool_tiles, score_out, tile_range); break;
            case 1: score_pool_kernel<1><<<pg, pb, 0, s>>>(vote, G, P, n_pool_tiles, score_out, tile_range); break;
            case 2: score_pool_kernel<2><<<pg, pb, 0, s>>>(vote, G, P, n_pool_tiles, score_out, tile_range); break;
            case 3: score_pool_kernel<3><<<pg, pb, 0, s>>>(vote, G, P, n_pool_tiles, score_out, tile_range); break;
            case 4: score_pool_kernel<4><<<pg, pb, 0, s>>>(vote, G, P, n_pool_tiles, score_out, tile_range); break;
            case 5: score_pool_kernel<5><<<pg, pb, 0, s>>>(vote, G, P, n_pool_tiles, score_out, tile_range); break;
            case 6: score_pool_kernel<6><<<pg, pb, 0, s>>>(vote, G, P, n_pool_tiles, score_out, tile_range); break;
            default: score_pool_kernel<7><<<pg, pb, 0, s>>>(vote, G, P, n_pool_tiles, score_out, tile_range); break;
        }
    }
    env.end();
    return hipGetLastError();
}

hipError_t launch_window_score(const void* Q, const void* K, uncomp_dtype dt, int B, int H, int G,
                               int N, int w, int pool, const int64_t ks[3], const ScorePlan& p,
                               char* ws, float* score_out, const Env& env, const float* lse_nat, int D) {
    if (dt == UNCOMP_BF16) {
        // the MFMA kernels need whole 16-row blocks per KV head, a window of 8 (the paper's l) or a multiple of 16,
        // and at most 256 rows per KV head
        const bool mfma = !env.force_alu && D == kD && (w % 16 == 0 || w == 8) && p.R <= 256 && p.R % 16 == 0;
        return run_score<bf16_bits>(static_cast<const bf16_bits*>(Q), static_cast<const bf16_bits*>(K), B, H,
                                    G, N, w, pool, ks, p, ws, score_out, env, mfma, lse_nat, D);
    }
    return run_score<float>(static_cast<const float*>(Q), static_cast<const float*>(K), B, H, G, N, w,
                            pool, ks, p, ws, score_out, env, false, lse_nat, D);
}

}  // namespace uncomp
