// Per-head top-k and compaction (Sec. 3.3.3: each head keeps its N_{i,g} highest-scoring
// tokens; Alg. 2 prefill: compress each head's KV by its group).
//
// select_kernel, one workgroup per (batch, head):
//   - the k-th largest score is found exactly by a most-significant-digit radix select on
//     an order-preserving 32-bit image of the float: digits of up to 11 bits, starting at the
//     highest bit in which the head's keys differ, one LDS histogram per digit;
//   - one more ordered pass writes the kept positions in ascending order: everything above
//     the threshold, and of the scores equal to it the first (k - #above) by position;
//   - the w window positions follow.
// gather_kernel then copies the kept rows of K and V, 16 bytes per lane.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kBins = 2048;
constexpr int kSelLoads = 8;                // 16-byte loads a thread keeps in flight in the range and histogram passes

// float -> uint32 whose unsigned order equals the float order (negative values included)
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f + 0.0f);      // -0.0 and +0.0 compare equal: same key
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t n = __shfl_up(v, o, 64);
        if (lane >= o) v += n;
    }
    return v;
}

struct SelSmem {
    uint32_t hist[kBins];
    uint32_t wsum[kSelWaves];
    uint32_t bcast[4];
};

// Exclusive prefix sum of one value per thread over the workgroup; returns the exclusive
// prefix and stores the grand total in *total.  Ends with a barrier.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, SelSmem& sm, uint32_t* total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    uint32_t inc = wave_incl_scan(v, lane);
    if (lane == 63) sm.wsum[wv] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kSelWaves; ++i) {
        uint32_t s = sm.wsum[i];
        if (i < wv) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

}  // namespace

__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ score,
                                                             const int32_t* __restrict__ budget,
                                                             int budget_stride, int N, int w, int cap,
                                                             int32_t* __restrict__ idx_out,
                                                             int32_t* __restrict__ len_out) {
    __shared__ SelSmem sm;
    const int bh = blockIdx.x;
    const int tid = threadIdx.x;
    const int P = N - w;
    const float* sc = score + (int64_t)bh * P;
    int32_t* idx = idx_out + (int64_t)bh * cap;

    int bud = budget[(int64_t)bh * budget_stride];     // stride 0: one budget for every row of scores
    const int hi = N < cap ? N : cap;
    bud = bud < w ? w : bud;
    bud = bud > hi ? hi : bud;
    const int k = bud - w;                    // prefix positions to keep, 0 <= k <= P

    uint32_t thr = 0;                         // key of the k-th largest score
    uint32_t need_eq = 0;                     // how many keys equal to thr are kept
    if (k > 0 && k < P) {
        // Range of the keys first: the radix digits then start at the highest bit in which
        // any two keys differ.  Scores of one head usually share their exponent and leading
        // mantissa bits; digits taken from the very top would put every key in one counter.
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        // rows of P floats start 16-byte aligned when P is a multiple of 4: 16-byte loads, two
        // per thread in flight; otherwise (and for the tail) plain 4-byte loads
        const int P4 = (P & 3) == 0 ? P >> 2 : 0;
        const float4* sc4 = reinterpret_cast<const float4*>(sc);
        for (int q0 = tid; q0 < P4; q0 += kSelLoads * kSelThreads) {
            float4 v[kSelLoads];                       // kSelLoads 16-byte loads in flight per thread
#pragma unroll
            for (int u = 0; u < kSelLoads; ++u) {
                const int q = q0 + u * kSelThreads;
                v[u] = sc4[q < P4 ? q : q0];           // past the end: this thread's first one again (min/max unchanged)
            }
#pragma unroll
            for (int u = 0; u < kSelLoads; ++u) {
                const float vals[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t key = order_key(vals[e]);
                    kmin = key < kmin ? key : kmin;
                    kmax = key > kmax ? key : kmax;
                }
            }
        }
        for (int j = 4 * P4 + tid; j < P; j += kSelThreads) {
            const uint32_t key = order_key(sc[j]);
            kmin = key < kmin ? key : kmin;
            kmax = key > kmax ? key : kmax;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const uint32_t a = __shfl_xor(kmin, o, 64), c = __shfl_xor(kmax, o, 64);
            kmin = a < kmin ? a : kmin;
            kmax = c > kmax ? c : kmax;
        }
        if ((tid & 63) == 0) {
            sm.wsum[tid >> 6] = kmin;
            sm.hist[tid >> 6] = kmax;
        }
        __syncthreads();
        for (int i = 0; i < kSelWaves; ++i) {
            kmin = sm.wsum[i] < kmin ? sm.wsum[i] : kmin;
            kmax = sm.hist[i] > kmax ? sm.hist[i] : kmax;
        }
        __syncthreads();

        int bits_left = kmin == kmax ? 0 : 32 - __builtin_clz(kmin ^ kmax);   // low bits that can differ
        uint32_t prefix_mask = bits_left >= 32 ? 0u : ~((1u << bits_left) - 1u);
        uint32_t prefix = kmax & prefix_mask;
        uint32_t remaining = (uint32_t)k;     // rank still to be located among matching keys
        while (bits_left > 0) {
            const int width = bits_left < 11 ? bits_left : 11;
            const int shift = bits_left - width;
            const uint32_t nb = 1u << width;
            for (int i = tid; i < kBins; i += kSelThreads) sm.hist[i] = 0;
            __syncthreads();
            auto count = [&](float v) {
                const uint32_t key = order_key(v);
                if ((key & prefix_mask) == prefix) atomicAdd(&sm.hist[(key >> shift) & (nb - 1)], 1u);
            };
            for (int q0 = tid; q0 < P4; q0 += kSelLoads * kSelThreads) {
                float4 v[kSelLoads];
#pragma unroll
                for (int u = 0; u < kSelLoads; ++u) {
                    const int q = q0 + u * kSelThreads;
                    v[u] = sc4[q < P4 ? q : q0];
                }
#pragma unroll
                for (int u = 0; u < kSelLoads; ++u) {
                    if (q0 + u * kSelThreads < P4) {
                        count(v[u].x); count(v[u].y); count(v[u].z); count(v[u].w);
                    }
                }
            }
            for (int j = 4 * P4 + tid; j < P; j += kSelThreads) count(sc[j]);
            __syncthreads();
            // walk the digits from the top: thread t owns digits nb-1-2t and nb-2-2t
            uint32_t c0 = 0, c1 = 0;
            const int d0 = (int)nb - 1 - 2 * tid, d1 = d0 - 1;
            if (d0 >= 0) c0 = sm.hist[d0];
            if (d1 >= 0) c1 = sm.hist[d1];
            uint32_t total;
            uint32_t before = block_excl_scan(c0 + c1, sm, &total);   // keys in higher digits
            if (d0 >= 0 && before < remaining && remaining <= before + c0) {
                sm.bcast[0] = (uint32_t)d0;
                sm.bcast[1] = remaining - before;
            } else if (d1 >= 0 && before + c0 < remaining && remaining <= before + c0 + c1) {
                sm.bcast[0] = (uint32_t)d1;
                sm.bcast[1] = remaining - before - c0;
            }
            __syncthreads();
            prefix |= sm.bcast[0] << shift;
            prefix_mask |= (nb - 1) << shift;
            remaining = sm.bcast[1];
            bits_left = shift;
            __syncthreads();
        }
        thr = prefix;
        need_eq = remaining;
    }

    // ordered compaction, four consecutive positions per thread per step
    if (k > 0) {
        const bool all = (k >= P);
        uint32_t kept_gt = 0, seen_eq = 0;    // running totals over the positions already passed
        float nxt[4];                         // scores of the next step, loaded one step ahead
#pragma unroll
        for (int e = 0; e < 4; ++e) nxt[e] = tid * 4 + e < P ? sc[tid * 4 + e] : 0.f;
        for (int base = 0; base < P; base += kSelThreads * 4) {
            const int j0 = base + tid * 4;
            float cur[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                cur[e] = nxt[e];
                const int jn = j0 + kSelThreads * 4 + e;
                nxt[e] = jn < P ? sc[jn] : 0.f;
            }
            uint32_t gt[4], eq[4], ngt = 0, neq = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                gt[e] = eq[e] = 0;
                if (j0 + e < P) {
                    uint32_t key = order_key(cur[e]);
                    gt[e] = (all || key > thr) ? 1u : 0u;
                    eq[e] = (!all && key == thr) ? 1u : 0u;
                }
                ngt += gt[e];
                neq += eq[e];
            }
            uint32_t total;
            uint32_t ex = block_excl_scan((ngt << 16) | neq, sm, &total);
            uint32_t g_before = kept_gt + (ex >> 16);
            uint32_t e_before = seen_eq + (ex & 0xffffu);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (gt[e]) {
                    uint32_t pos = g_before + (e_before < need_eq ? e_before : need_eq);
                    idx[pos] = j0 + e;
                    ++g_before;
                } else if (eq[e]) {
                    if (e_before < need_eq) idx[g_before + e_before] = j0 + e;
                    ++e_before;
                }
            }
            kept_gt += total >> 16;
            seen_eq += total & 0xffffu;
        }
    }
    for (int i = tid; i < w; i += kSelThreads) idx[k + i] = P + i;
    if (tid == 0) len_out[bh] = bud;
}

// Copies row idx[r] of K and V to row r of the outputs; `lanes` lanes of 16 bytes per row.
__global__ __launch_bounds__(256) void gather_kernel(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                     const int32_t* __restrict__ idx,
                                                     const int32_t* __restrict__ len, int H, int cap,
                                                     int lanes, int64_t sb, int64_t sh, int64_t st,
                                                     int n_row_tiles, uint4* __restrict__ K_out,
                                                     uint4* __restrict__ V_out) {
    const int bh = blockIdx.x / n_row_tiles, tile = blockIdx.x % n_row_tiles;
    const int b = bh / H, h = bh % H;
    const int rows_per_block = 256 / lanes;
    const int r = tile * rows_per_block + threadIdx.x / lanes;
    const int l = threadIdx.x % lanes;
    if (r >= len[bh]) return;
    const int64_t src = b * sb + h * sh + (int64_t)idx[(int64_t)bh * cap + r] * st + l;   // in 16-byte units
    const int64_t dst = ((int64_t)bh * cap + r) * lanes + l;
    K_out[dst] = K[src];
    V_out[dst] = V[src];
}

hipError_t launch_select_gather(const float* score, const int32_t* budget, const void* K,
                                const void* V, uncomp_dtype dt, int B, int H, int N, int w,
                                const int64_t ks[3], int cap, void* K_out, void* V_out,
                                int32_t* idx_out, int32_t* len_out, const Env& env) {
    hipStream_t s = env.s;
    const int BH = B * H;
    env.begin("select");
    select_kernel<<<dim3(BH), dim3(kSelThreads), 0, s>>>(score, budget, 1, N, w, cap, idx_out, len_out);
    env.end();
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || K == nullptr) return e;
    const int esz = dt == UNCOMP_BF16 ? 2 : 4;
    const int per16 = 16 / esz;                       // elements per 16-byte unit
    const int lanes = kD / per16;                     // 16 (bf16) or 32 (fp32)
    const int rows_per_block = 256 / lanes;
    const int n_row_tiles = (cap + rows_per_block - 1) / rows_per_block;
    env.begin("gather");
    gather_kernel<<<dim3((unsigned)(BH * n_row_tiles)), dim3(256), 0, s>>>(
        static_cast<const uint4*>(K), static_cast<const uint4*>(V), idx_out, len_out, H, cap, lanes,
        ks[0] / per16, ks[1] / per16, ks[2] / per16, n_row_tiles, static_cast<uint4*>(K_out),
        static_cast<uint4*>(V_out));
    env.end();
    return hipGetLastError();
}

// Rows of any width: idx[g][r] names the source row of output row r of group g; rows are
// copied in 16-byte units, four rows per workgroup.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ src,
                                                          const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ len, int cap, int units,
                                                          int64_t group_stride, int64_t row_stride,
                                                          int n_row_tiles, uint4* __restrict__ dst) {
    const int g = blockIdx.x / n_row_tiles, tile = blockIdx.x % n_row_tiles;
    const int n = len[g];
    for (int rr = 0; rr < 4; ++rr) {
        const int r = tile * 4 + rr;
        if (r >= n || r >= cap) return;
        const uint4* s = src + g * group_stride + (int64_t)idx[(int64_t)g * cap + r] * row_stride;
        uint4* d = dst + ((int64_t)g * cap + r) * units;
        for (int u = threadIdx.x; u < units; u += 256) d[u] = s[u];
    }
}

hipError_t launch_select_rows(const float* score, const int32_t* budget, int budget_stride, int n_groups,
                              int N, int w, int cap, int32_t* idx_out, int32_t* len_out, const Env& env) {
    env.begin("select");
    select_kernel<<<dim3(n_groups), dim3(kSelThreads), 0, env.s>>>(score, budget, budget_stride, N, w, cap, idx_out,
                                                                  len_out);
    env.end();
    return hipGetLastError();
}

hipError_t launch_gather_rows(const void* src, const int32_t* idx, const int32_t* len, int n_groups, int cap,
                              int row_bytes, int64_t group_stride_bytes, int64_t row_stride_bytes, void* dst,
                              const Env& env) {
    const int n_row_tiles = (cap + 3) / 4;
    env.begin("gather_rows");
    gather_rows_kernel<<<dim3((unsigned)(n_groups * n_row_tiles)), dim3(256), 0, env.s>>>(
        static_cast<const uint4*>(src), idx, len, cap, row_bytes / 16, group_stride_bytes / 16, row_stride_bytes / 16,
        n_row_tiles, static_cast<uint4*>(dst));
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
