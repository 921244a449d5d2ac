// Top-k of a few long rows of scores, split over many workgroups (Sec. 3.3.2: the hidden-state eviction
// keeps the layer's highest-scoring tokens out of one row of N scores per batch entry, far fewer rows than
// the chip has CUs; Sec. 3.3.3 defines the per-row selection).  Same result as select_kernel: the k largest
// scores, ties at the threshold by position, indices ascending, then the w window positions.
//
// A row is cut into chunks of 2048 positions, one workgroup each, and the exact k-th largest key is found
// by a most-significant-digit radix select on the order-preserving 32-bit image of the float with digits of
// 11, 11 and 10 bits at fixed positions.  Workgroups only meet between kernels:
//   zero     clears the three histograms of every row;
//   hist<p>  resolves the histogram of digit p-1 (every workgroup for itself, workgroup 0 records the
//            result), then counts digit p of its chunk's keys that match the digits found so far in LDS
//            and adds the non-empty counters to the row's histogram;
//   count    resolves the last digit: threshold and number of equal keys to take; counts the chunk's keys
//            above / equal to the threshold;
//   write    sums the counts of the chunks before its own and writes its kept positions in order.
// Integer atomics only: the result does not depend on the order in which workgroups run.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kWThreads = 256;
constexpr int kWPer = 8;                         // consecutive positions per thread
constexpr int kWChunk = kWThreads * kWPer;       // positions per workgroup
constexpr int kWBins = 2048;
constexpr int kWStates = 4;                      // state after resolving 0, 1, 2, 3 digits

struct WideState {
    uint32_t prefix;         // digits found so far (in place)
    uint32_t remaining;      // rank of the wanted key among the keys that share the prefix (1 = largest)
    uint32_t pad0, pad1;
};

struct WideSmem {
    uint32_t hist[kWBins];
    uint32_t wsum[kWThreads / 64];
    uint32_t bcast[2];
};

__device__ __forceinline__ int digit_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ uint32_t digit_bins(int pass) { return pass == 2 ? 1024u : 2048u; }
// mask of the digits above digit `pass`
__device__ __forceinline__ uint32_t prefix_mask(int pass) { return pass == 0 ? 0u : (pass == 1 ? 0xffe00000u : 0xfffffc00u); }

__device__ __forceinline__ uint32_t wide_wave_incl_scan(uint32_t v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t n = __shfl_up(v, o, 64);
        if (lane >= o) v += n;
    }
    return v;
}

// exclusive prefix over the workgroup and the total; ends with a barrier
__device__ __forceinline__ uint32_t wide_excl_scan(uint32_t v, WideSmem& sm, uint32_t* total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const uint32_t inc = wide_wave_incl_scan(v, lane);
    if (lane == 63) sm.wsum[wv] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kWThreads / 64; ++i) {
        const uint32_t s = sm.wsum[i];
        if (i < wv) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// the row's budget as the number of prefix positions to keep
__device__ __forceinline__ int prefix_budget(const int32_t* budget, int budget_stride, int g, int N, int w, int cap,
                                             int* bud_out) {
    int bud = budget[(int64_t)g * budget_stride];
    const int hi = N < cap ? N : cap;
    bud = bud < w ? w : bud;
    bud = bud > hi ? hi : bud;
    *bud_out = bud;
    return bud - w;
}

// keys of this thread's kWPer consecutive positions (0 past the end of the row: callers skip those)
__device__ __forceinline__ void load_keys(const float* sc, int P, int j0, uint32_t (&key)[kWPer]) {
    const bool aligned = (P & 3) == 0 && (reinterpret_cast<uintptr_t>(sc) & 15u) == 0;   // every row then starts on 16 bytes
    if (aligned && j0 + kWPer <= P) {
        const float4 a = *reinterpret_cast<const float4*>(sc + j0);
        const float4 b = *reinterpret_cast<const float4*>(sc + j0 + 4);
        key[0] = order_key(a.x); key[1] = order_key(a.y); key[2] = order_key(a.z); key[3] = order_key(a.w);
        key[4] = order_key(b.x); key[5] = order_key(b.y); key[6] = order_key(b.z); key[7] = order_key(b.w);
    } else {
#pragma unroll
        for (int e = 0; e < kWPer; ++e) key[e] = j0 + e < P ? order_key(sc[j0 + e]) : 0u;
    }
}

// Resolves digit `pass` of the row from its finished histogram: the digit that holds the `remaining`-th
// largest key with the prefix found so far.  Every thread returns the new state.  Two barriers inside.
__device__ __forceinline__ WideState resolve_digit(const uint32_t* __restrict__ hist, int pass, WideState st, WideSmem& sm) {
    const int tid = threadIdx.x;
    const uint32_t nb = digit_bins(pass);
    // thread t owns the 8 digits nb-1-8t ... nb-8-8t, highest first
    uint32_t c[8], mine = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int d = (int)nb - 1 - 8 * tid - u;
        c[u] = d >= 0 ? hist[d] : 0u;
        mine += c[u];
    }
    if (tid == 0) {                                                // what a rank beyond the keys counted would leave behind
        sm.bcast[0] = 0u;
        sm.bcast[1] = 1u;
    }
    uint32_t total;
    uint32_t before = wide_excl_scan(mine, sm, &total);          // keys in higher digits
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int d = (int)nb - 1 - 8 * tid - u;
        if (d >= 0 && before < st.remaining && st.remaining <= before + c[u]) {
            sm.bcast[0] = (uint32_t)d;
            sm.bcast[1] = st.remaining - before;
        }
        before += c[u];
    }
    __syncthreads();
    WideState out = st;
    out.prefix = st.prefix | (sm.bcast[0] << digit_shift(pass));
    out.remaining = sm.bcast[1];
    __syncthreads();
    return out;
}

struct WideBufs {
    uint32_t* hist;          // [n_groups][3][kWBins]
    WideState* state;        // [n_groups][kWStates]
    uint32_t* counts;        // [n_groups][n_wg][2]
};

__device__ __forceinline__ WideBufs wide_bufs(char* ws, int n_groups, int n_wg) {
    WideBufs b;
    b.hist = reinterpret_cast<uint32_t*>(ws);
    b.state = reinterpret_cast<WideState*>(ws + (size_t)n_groups * 3 * kWBins * sizeof(uint32_t));
    b.counts = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(b.state) + (size_t)n_groups * kWStates * sizeof(WideState));
    (void)n_wg;
    return b;
}

}  // namespace

__global__ __launch_bounds__(kWThreads) void selw_zero_kernel(uint32_t* __restrict__ hist, int n) {
    const int i = blockIdx.x * kWThreads + threadIdx.x;
    if (i < n) hist[i] = 0u;
}

template <int PASS>
__global__ __launch_bounds__(kWThreads) void selw_hist_kernel(const float* __restrict__ score,
                                                              const int32_t* __restrict__ budget, int budget_stride,
                                                              int N, int w, int cap, int n_groups, char* __restrict__ ws) {
    __shared__ WideSmem sm;
    const int g = blockIdx.y, wg = blockIdx.x, tid = threadIdx.x;
    const int P = N - w;
    const WideBufs b = wide_bufs(ws, n_groups, gridDim.x);
    uint32_t* hist = b.hist + (size_t)g * 3 * kWBins;
    WideState* state = b.state + (size_t)g * kWStates;
    int bud;
    const int k = prefix_budget(budget, budget_stride, g, N, w, cap, &bud);
    if (k <= 0 || k >= P) return;                                  // nothing to search for: the write kernel handles it
    WideState st;
    if (PASS == 0) {
        st.prefix = 0u;
        st.remaining = (uint32_t)k;
        st.pad0 = st.pad1 = 0u;
    } else {
        st = resolve_digit(hist + (PASS - 1) * kWBins, PASS - 1, state[PASS - 1], sm);
    }
    if (wg == 0 && tid == 0) state[PASS] = st;
    for (int i = tid; i < kWBins; i += kWThreads) sm.hist[i] = 0u;
    __syncthreads();
    const float* sc = score + (int64_t)g * P;
    const int j0 = wg * kWChunk + tid * kWPer;
    uint32_t key[kWPer];
    load_keys(sc, P, j0, key);
    const uint32_t pm = prefix_mask(PASS);
    const int shift = digit_shift(PASS);
    const uint32_t nb = digit_bins(PASS);
#pragma unroll
    for (int e = 0; e < kWPer; ++e)
        if (j0 + e < P && (key[e] & pm) == (st.prefix & pm)) atomicAdd(&sm.hist[(key[e] >> shift) & (nb - 1)], 1u);
    __syncthreads();
    for (int i = tid; i < (int)nb; i += kWThreads) {
        const uint32_t c = sm.hist[i];
        if (c != 0u) atomicAdd(&hist[PASS * kWBins + i], c);
    }
}

__global__ __launch_bounds__(kWThreads) void selw_count_kernel(const float* __restrict__ score,
                                                               const int32_t* __restrict__ budget, int budget_stride,
                                                               int N, int w, int cap, int n_groups, char* __restrict__ ws) {
    __shared__ WideSmem sm;
    const int g = blockIdx.y, wg = blockIdx.x, tid = threadIdx.x;
    const int n_wg = gridDim.x;
    const int P = N - w;
    const WideBufs b = wide_bufs(ws, n_groups, n_wg);
    WideState* state = b.state + (size_t)g * kWStates;
    int bud;
    const int k = prefix_budget(budget, budget_stride, g, N, w, cap, &bud);
    if (k <= 0 || k >= P) return;
    const WideState st = resolve_digit(b.hist + ((size_t)g * 3 + 2) * kWBins, 2, state[2], sm);
    if (wg == 0 && tid == 0) state[3] = st;                        // prefix = the threshold key, remaining = equal keys to take
    const float* sc = score + (int64_t)g * P;
    const int j0 = wg * kWChunk + tid * kWPer;
    uint32_t key[kWPer];
    load_keys(sc, P, j0, key);
    uint32_t ngt = 0, neq = 0;
#pragma unroll
    for (int e = 0; e < kWPer; ++e) {
        if (j0 + e < P) {
            ngt += key[e] > st.prefix ? 1u : 0u;
            neq += key[e] == st.prefix ? 1u : 0u;
        }
    }
    uint32_t total;
    wide_excl_scan((ngt << 16) | neq, sm, &total);                 // at most 2048 of either: no carry between the halves
    if (tid == 0) {
        b.counts[((size_t)g * n_wg + wg) * 2] = total >> 16;
        b.counts[((size_t)g * n_wg + wg) * 2 + 1] = total & 0xffffu;
    }
}

__global__ __launch_bounds__(kWThreads) void selw_write_kernel(const float* __restrict__ score,
                                                               const int32_t* __restrict__ budget, int budget_stride,
                                                               int N, int w, int cap, int n_groups, char* __restrict__ ws,
                                                               int32_t* __restrict__ idx_out, int32_t* __restrict__ len_out) {
    __shared__ WideSmem sm;
    const int g = blockIdx.y, wg = blockIdx.x, tid = threadIdx.x;
    const int n_wg = gridDim.x;
    const int P = N - w;
    const WideBufs b = wide_bufs(ws, n_groups, n_wg);
    int32_t* idx = idx_out + (int64_t)g * cap;
    int bud;
    const int k = prefix_budget(budget, budget_stride, g, N, w, cap, &bud);
    if (wg == 0) {
        for (int i = tid; i < w; i += kWThreads) idx[k + i] = P + i;
        if (tid == 0) len_out[g] = bud;
    }
    if (k <= 0) return;
    const int j0 = wg * kWChunk + tid * kWPer;
    if (k >= P) {                                                 // every prefix position is kept
#pragma unroll
        for (int e = 0; e < kWPer; ++e)
            if (j0 + e < P) idx[j0 + e] = j0 + e;
        return;
    }
    const WideState st = b.state[(size_t)g * kWStates + 3];
    const uint32_t thr = st.prefix, need_eq = st.remaining;
    // kept / equal keys in the chunks before this one
    uint32_t gsum = 0, esum = 0;
    for (int i = tid; i < wg; i += kWThreads) {
        gsum += b.counts[((size_t)g * n_wg + i) * 2];
        esum += b.counts[((size_t)g * n_wg + i) * 2 + 1];
    }
    uint32_t g_tot, e_tot;
    wide_excl_scan(gsum, sm, &g_tot);
    wide_excl_scan(esum, sm, &e_tot);
    const float* sc = score + (int64_t)g * P;
    uint32_t key[kWPer];
    load_keys(sc, P, j0, key);
    uint32_t gtm = 0, eqm = 0;
#pragma unroll
    for (int e = 0; e < kWPer; ++e) {
        if (j0 + e < P) {
            if (key[e] > thr) gtm |= 1u << e;
            else if (key[e] == thr) eqm |= 1u << e;
        }
    }
    uint32_t total;
    const uint32_t ex = wide_excl_scan(((uint32_t)__builtin_popcount(gtm) << 16) | (uint32_t)__builtin_popcount(eqm), sm, &total);
    uint32_t g_before = g_tot + (ex >> 16);
    uint32_t e_before = e_tot + (ex & 0xffffu);
    // everything above the threshold and the first need_eq equal keys; writes stay inside the k slots
#pragma unroll
    for (int e = 0; e < kWPer; ++e) {
        if (gtm & (1u << e)) {
            const uint32_t pos = g_before + (e_before < need_eq ? e_before : need_eq);
            if (pos < (uint32_t)k) idx[pos] = j0 + e;
            ++g_before;
        } else if (eqm & (1u << e)) {
            const uint32_t pos = g_before + e_before;
            if (e_before < need_eq && pos < (uint32_t)k) idx[pos] = j0 + e;
            ++e_before;
        }
    }
}

SelectWidePlan plan_select_wide(int n_groups, int N, int w) {
    SelectWidePlan p;
    const int P = N - w > 0 ? N - w : 1;
    p.n_wg = (P + kWChunk - 1) / kWChunk;
    p.bytes = align_up((size_t)n_groups * 3 * kWBins * sizeof(uint32_t) + (size_t)n_groups * kWStates * sizeof(WideState) +
                           (size_t)n_groups * p.n_wg * 2 * sizeof(uint32_t),
                       256);
    return p;
}

hipError_t launch_select_rows_wide(const float* score, const int32_t* budget, int budget_stride, int n_groups, int N,
                                   int w, int cap, const SelectWidePlan& p, char* ws, int32_t* idx_out, int32_t* len_out,
                                   const Env& env) {
    hipStream_t s = env.s;
    const dim3 grid((unsigned)p.n_wg, (unsigned)n_groups), block(kWThreads);
    const int n_hist = n_groups * 3 * kWBins;
    env.begin("select");
    selw_zero_kernel<<<dim3((unsigned)((n_hist + kWThreads - 1) / kWThreads)), block, 0, s>>>(reinterpret_cast<uint32_t*>(ws), n_hist);
    selw_hist_kernel<0><<<grid, block, 0, s>>>(score, budget, budget_stride, N, w, cap, n_groups, ws);
    selw_hist_kernel<1><<<grid, block, 0, s>>>(score, budget, budget_stride, N, w, cap, n_groups, ws);
    selw_hist_kernel<2><<<grid, block, 0, s>>>(score, budget, budget_stride, N, w, cap, n_groups, ws);
    selw_count_kernel<<<grid, block, 0, s>>>(score, budget, budget_stride, N, w, cap, n_groups, ws);
    selw_write_kernel<<<grid, block, 0, s>>>(score, budget, budget_stride, N, w, cap, n_groups, ws, idx_out, len_out);
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
