// Per-head top-k and compaction (Sec. 3.3.3: each head keeps its N_{i,g} highest-scoring
// tokens; Alg. 2 prefill: compress each head's KV by its group).
//
// select_kernel, one workgroup per (batch, head).  The k-th largest score is found exactly by a
// most-significant-digit radix select on an order-preserving 32-bit image of the float, digits of up
// to 11 bits starting at the highest bit in which the head's keys differ.  The scores are read from
// memory twice in the common case:
//   pass A  histogram of the first digit -> the digit d1 that holds the k-th key; keys in higher
//           digits are kept for certain, keys in d1 are candidates, the rest is dropped;
//   pass B  one ordered walk over the positions: certain and candidate positions go, in ascending
//           order, into a list in LDS, the candidates' keys into a second one;
//   then, without touching the scores again: the remaining digits are resolved on the candidate keys,
//   and one ordered walk over the list writes the kept positions (everything above the threshold,
//   and of the scores equal to it the first few by position).
// Heads whose lists would not fit LDS (budgets of many thousands of tokens, or thousands of scores in
// one digit) take more histogram passes over the scores and one ordered pass over all positions.
// The range of the keys either comes from the caller of the kernel (per-tile minima and maxima left
// by the pooling kernel) or is found by a pass of its own; a range handed in is checked against every
// key in pass A and replaced by the true one if any key lies outside it.
// The w window positions follow the kept prefix positions.  gather_kernel then copies the kept rows
// of K and V, 16 bytes per lane.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kBins = 2048;
constexpr int kSelLoads = 4;                // 16-byte loads per thread and round in the range and histogram passes (two rounds in flight)
constexpr int kListCap = 16384;             // positions (certain + candidate) the LDS list holds
constexpr int kCandCap = 8192;              // candidate keys the LDS list holds
constexpr size_t kSelDynLds = (size_t)(kListCap + kCandCap) * sizeof(uint32_t);

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
    uint32_t n_cand;
    uint32_t outside;
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

// sm.hist[0..nb) holds the counts of one digit.  Finds the digit that contains the `remaining`-th key
// counted from the top digit down; returns it, the rank left inside it (*rank_in), its count and the
// number of keys in higher digits.  Every thread gets the same answers.  Ends with a barrier.
__device__ __forceinline__ uint32_t pick_digit(SelSmem& sm, uint32_t nb, uint32_t remaining, uint32_t* rank_in,
                                               uint32_t* count_in, uint32_t* above) {
    const int tid = threadIdx.x;
    uint32_t c0 = 0, c1 = 0;                  // thread t owns digits nb-1-2t and nb-2-2t
    const int d0 = (int)nb - 1 - 2 * tid, d1 = d0 - 1;
    if (d0 >= 0) c0 = sm.hist[d0];
    if (d1 >= 0) c1 = sm.hist[d1];
    uint32_t total;
    const uint32_t before = block_excl_scan(c0 + c1, sm, &total);   // keys in higher digits
    if (d0 >= 0 && before < remaining && remaining <= before + c0) {
        sm.bcast[0] = (uint32_t)d0;
        sm.bcast[1] = remaining - before;
        sm.bcast[2] = c0;
        sm.bcast[3] = before;
    } else if (d1 >= 0 && before + c0 < remaining && remaining <= before + c0 + c1) {
        sm.bcast[0] = (uint32_t)d1;
        sm.bcast[1] = remaining - before - c0;
        sm.bcast[2] = c1;
        sm.bcast[3] = before + c0;
    }
    __syncthreads();
    const uint32_t digit = sm.bcast[0];
    *rank_in = sm.bcast[1];
    *count_in = sm.bcast[2];
    *above = sm.bcast[3];
    __syncthreads();
    return digit;
}

}  // namespace

// tile_range: per group n_range_tiles pairs (smallest key, largest key) that together cover the group's
// scores, or nullptr.
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ score,
                                                             const int32_t* __restrict__ budget,
                                                             int budget_stride, int N, int w, int cap,
                                                             const uint32_t* __restrict__ tile_range,
                                                             int n_range_tiles, int32_t* __restrict__ idx_out,
                                                             int32_t* __restrict__ len_out) {
    __shared__ SelSmem sm;
    extern __shared__ __align__(16) uint32_t sel_dyn[];
    uint32_t* list = sel_dyn;                 // [kListCap] position | candidate flag in bit 31, ascending positions
    uint32_t* cand = sel_dyn + kListCap;      // [kCandCap] candidate keys, any order
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

    // rows of P floats start 16-byte aligned when P is a multiple of 4: 16-byte loads; otherwise (and for
    // the tail) plain 4-byte loads
    const int P4 = (P & 3) == 0 ? P >> 2 : 0;
    const float4* sc4 = reinterpret_cast<const float4*>(sc);

    // applies f(key) to every score of the head; the kSelLoads 16-byte loads of the next round are in flight
    // while the keys of this round are processed
    auto for_all_keys = [&](auto f) {
        float4 cur[kSelLoads], nxt[kSelLoads];
        auto issue = [&](float4 (&dst)[kSelLoads], int q0) {
#pragma unroll
            for (int u = 0; u < kSelLoads; ++u) {
                const int q = q0 + u * kSelThreads;
                dst[u] = sc4[q < P4 ? q : (q0 < P4 ? q0 : 0)];       // past the end: a valid address, value not used
            }
        };
        if (P4 > 0) issue(cur, tid);
        for (int q0 = tid; q0 < P4; q0 += kSelLoads * kSelThreads) {
            issue(nxt, q0 + kSelLoads * kSelThreads);
#pragma unroll
            for (int u = 0; u < kSelLoads; ++u) {
                if (q0 + u * kSelThreads < P4) {
                    f(order_key(cur[u].x)); f(order_key(cur[u].y)); f(order_key(cur[u].z)); f(order_key(cur[u].w));
                }
            }
#pragma unroll
            for (int u = 0; u < kSelLoads; ++u) cur[u] = nxt[u];
        }
        for (int j = 4 * P4 + tid; j < P; j += kSelThreads) f(order_key(sc[j]));
    };
    // Walks the positions in ascending order, kPer consecutive ones per thread and kSelThreads*kPer per step;
    // step(j0, v) gets the thread's first position and its scores (0 past the end).  The next step's loads are
    // in flight during a step, and a step's workgroup-wide prefix sum is shared by sixteen positions per thread.
    constexpr int kPer = 16;
    auto ordered_walk = [&](auto step) {
        float cur[kPer], nxt[kPer];
        auto issue = [&](float (&dst)[kPer], int j0) {
            if (P4 > 0 && j0 + kPer - 1 < P) {
#pragma unroll
                for (int q = 0; q < kPer / 4; ++q) {
                    const float4 t = sc4[(j0 >> 2) + q];
                    dst[4 * q] = t.x; dst[4 * q + 1] = t.y; dst[4 * q + 2] = t.z; dst[4 * q + 3] = t.w;
                }
            } else {
#pragma unroll
                for (int e = 0; e < kPer; ++e) dst[e] = j0 + e < P ? sc[j0 + e] : 0.f;
            }
        };
        issue(cur, tid * kPer);
        for (int base = 0; base < P; base += kSelThreads * kPer) {
            issue(nxt, base + kSelThreads * kPer + tid * kPer);      // the next step's scores travel during this step
            step(base + tid * kPer, cur);
#pragma unroll
            for (int e = 0; e < kPer; ++e) cur[e] = nxt[e];
        }
    };
    // workgroup minimum / maximum of one pair per thread; every thread gets the result
    auto reduce_range = [&](uint32_t& kmin, uint32_t& kmax) {
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
    };
    // Ordered compaction of items [0, n_items): classify(i, &gt, &eq) says whether item i is above the
    // threshold / equal to it, position_of(i) gives the position to write.  Keeps everything above and the
    // first need_eq equal ones; writes stay inside the k slots whatever the counts upstream say.
    auto compact = [&](int n_items, uint32_t need_eq, auto classify, auto position_of) {
        uint32_t kept_gt = 0, seen_eq = 0;    // running totals over the items already passed
        for (int base = 0; base < n_items; base += kSelThreads * 4) {
            const int i0 = base + tid * 4;
            uint32_t gt[4], eq[4], ngt = 0, neq = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                gt[e] = eq[e] = 0;
                if (i0 + e < n_items) classify(i0 + e, gt[e], eq[e]);
                ngt += gt[e];
                neq += eq[e];
            }
            uint32_t total;
            const uint32_t ex = block_excl_scan((ngt << 16) | neq, sm, &total);
            uint32_t g_before = kept_gt + (ex >> 16);
            uint32_t e_before = seen_eq + (ex & 0xffffu);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (gt[e]) {
                    const uint32_t pos = g_before + (e_before < need_eq ? e_before : need_eq);
                    if (pos < (uint32_t)k) idx[pos] = position_of(i0 + e);
                    ++g_before;
                } else if (eq[e]) {
                    const uint32_t pos = g_before + e_before;
                    if (e_before < need_eq && pos < (uint32_t)k) idx[pos] = position_of(i0 + e);
                    ++e_before;
                }
            }
            kept_gt += total >> 16;
            seen_eq += total & 0xffffu;
        }
    };
    // one ordered pass over all scores against a known threshold: everything above it and the first need_eq
    // equal ones are kept; writes stay inside the k slots whatever the counts upstream say
    auto compact_all_scores = [&](uint32_t thr, uint32_t need_eq, bool all) {
        uint32_t kept_gt = 0, seen_eq = 0;
        ordered_walk([&](int j0, const float (&v)[kPer]) {
            uint32_t gtm = 0, eqm = 0;                 // bit e: position j0 + e is above / equal to the threshold
#pragma unroll
            for (int e = 0; e < kPer; ++e) {
                if (j0 + e < P) {
                    const uint32_t key = order_key(v[e]);
                    if (all || key > thr) gtm |= 1u << e;
                    else if (key == thr) eqm |= 1u << e;
                }
            }
            uint32_t total;
            const uint32_t ex = block_excl_scan(((uint32_t)__builtin_popcount(gtm) << 16) | (uint32_t)__builtin_popcount(eqm), sm, &total);
            uint32_t g_before = kept_gt + (ex >> 16);
            uint32_t e_before = seen_eq + (ex & 0xffffu);
#pragma unroll
            for (int e = 0; e < kPer; ++e) {
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
            kept_gt += total >> 16;
            seen_eq += total & 0xffffu;
        });
    };

    if (k >= P && k > 0) {
        compact_all_scores(0u, 0u, true);
    } else if (k > 0) {
        // Range of the keys first: the radix digits then start at the highest bit in which any two keys
        // differ.  Scores of one head usually share their exponent and leading mantissa bits; digits taken
        // from the very top would put every key in one counter.
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        bool range_given = tile_range != nullptr;
        if (range_given) {
            const uint32_t* tr = tile_range + (int64_t)bh * n_range_tiles * 2;
            for (int i = tid; i < n_range_tiles; i += kSelThreads) {
                kmin = tr[2 * i] < kmin ? tr[2 * i] : kmin;
                kmax = tr[2 * i + 1] > kmax ? tr[2 * i + 1] : kmax;
            }
        } else {
            for_all_keys([&](uint32_t key) {
                kmin = key < kmin ? key : kmin;
                kmax = key > kmax ? key : kmax;
            });
        }
        reduce_range(kmin, kmax);

        int bits_left = 0, width = 0, shift = 0;
        uint32_t prefix_mask = 0, prefix = 0, nb = 1;
        uint32_t d1 = 0, rank_in = (uint32_t)k, c1 = 0, above = 0;
        for (;;) {
            bits_left = kmin == kmax ? 0 : 32 - __builtin_clz(kmin ^ kmax);   // low bits that can differ
            prefix_mask = bits_left >= 32 ? 0u : ~((1u << bits_left) - 1u);
            prefix = kmax & prefix_mask;
            if (bits_left == 0) break;
            // pass A: counts of the first digit
            width = bits_left < 11 ? bits_left : 11;
            shift = bits_left - width;
            nb = 1u << width;
            for (int i = tid; i < kBins; i += kSelThreads) sm.hist[i] = 0;
            if (tid == 0) sm.outside = 0;
            __syncthreads();
            bool outside = false;
            for_all_keys([&](uint32_t key) {
                if ((key & prefix_mask) == prefix) atomicAdd(&sm.hist[(key >> shift) & (nb - 1)], 1u);
                else outside = true;
            });
            if (range_given && outside) sm.outside = 1;
            __syncthreads();
            if (!range_given || sm.outside == 0) break;
            // a key lies outside the range that was handed in: find the true one and count again
            __syncthreads();
            range_given = false;
            kmin = 0xffffffffu;
            kmax = 0u;
            for_all_keys([&](uint32_t key) {
                kmin = key < kmin ? key : kmin;
                kmax = key > kmax ? key : kmax;
            });
            reduce_range(kmin, kmax);
        }

        if (bits_left == 0) {
            compact_all_scores(kmax, (uint32_t)k, false);         // every score is the same: the first k positions
        } else {
            d1 = pick_digit(sm, nb, (uint32_t)k, &rank_in, &c1, &above);
            prefix |= d1 << shift;
            prefix_mask |= (nb - 1) << shift;
            bits_left = shift;
            if (bits_left == 0) {
                compact_all_scores(prefix, rank_in, false);       // one digit was the whole key
            } else if (above + c1 <= (uint32_t)kListCap && c1 <= (uint32_t)kCandCap) {
                // pass B: certain and candidate positions, in order, into the LDS list
                if (tid == 0) sm.n_cand = 0;
                __syncthreads();
                uint32_t n_list = 0;
                const uint32_t first_mask = prefix_mask;          // covers the common prefix and the first digit
                ordered_walk([&](int j0, const float (&v)[kPer]) {
                    uint32_t listed = 0, is_cand = 0;             // bit e: position j0 + e goes into the list / is a candidate
#pragma unroll
                    for (int e = 0; e < kPer; ++e) {
                        if (j0 + e < P) {
                            const uint32_t key = order_key(v[e]);
                            const uint32_t top = key & first_mask;
                            if (top > prefix) {
                                listed |= 1u << e;
                            } else if (top == prefix) {
                                listed |= 1u << e;
                                is_cand |= 1u << e;
                                const uint32_t slot = atomicAdd(&sm.n_cand, 1u);
                                if (slot < (uint32_t)kCandCap) cand[slot] = key;
                            }
                        }
                    }
                    uint32_t total;
                    uint32_t at = n_list + block_excl_scan((uint32_t)__builtin_popcount(listed), sm, &total);
#pragma unroll
                    for (int e = 0; e < kPer; ++e)
                        if (listed & (1u << e)) {
                            if (at < (uint32_t)kListCap) list[at] = (uint32_t)(j0 + e) | ((is_cand >> e) << 31);
                            ++at;
                        }
                    n_list += total;
                });
                __syncthreads();
                const uint32_t n_cand = sm.n_cand < (uint32_t)kCandCap ? sm.n_cand : (uint32_t)kCandCap;
                n_list = n_list < (uint32_t)kListCap ? n_list : (uint32_t)kListCap;
                // the remaining digits, on the candidate keys in LDS
                uint32_t remaining = rank_in;
                while (bits_left > 0) {
                    width = bits_left < 11 ? bits_left : 11;
                    shift = bits_left - width;
                    nb = 1u << width;
                    for (int i = tid; i < kBins; i += kSelThreads) sm.hist[i] = 0;
                    __syncthreads();
                    for (uint32_t i = tid; i < n_cand; i += kSelThreads) {
                        const uint32_t key = cand[i];
                        if ((key & prefix_mask) == prefix) atomicAdd(&sm.hist[(key >> shift) & (nb - 1)], 1u);
                    }
                    __syncthreads();
                    uint32_t cnt, abv;
                    const uint32_t d = pick_digit(sm, nb, remaining, &remaining, &cnt, &abv);
                    prefix |= d << shift;
                    prefix_mask |= (nb - 1) << shift;
                    bits_left = shift;
                }
                const uint32_t thr = prefix;
                compact((int)n_list, remaining,
                        [&](int i, uint32_t& gt, uint32_t& eq) {
                            const uint32_t ent = list[i];
                            if (ent & 0x80000000u) {
                                const uint32_t key = order_key(sc[ent & 0x7fffffffu]);
                                gt = key > thr ? 1u : 0u;
                                eq = key == thr ? 1u : 0u;
                            } else {
                                gt = 1u;
                                eq = 0u;
                            }
                        },
                        [&](int i) { return (int32_t)(list[i] & 0x7fffffffu); });
            } else {
                // lists too long for LDS: the remaining digits over the scores themselves
                uint32_t remaining = rank_in;
                while (bits_left > 0) {
                    width = bits_left < 11 ? bits_left : 11;
                    shift = bits_left - width;
                    nb = 1u << width;
                    for (int i = tid; i < kBins; i += kSelThreads) sm.hist[i] = 0;
                    __syncthreads();
                    for_all_keys([&](uint32_t key) {
                        if ((key & prefix_mask) == prefix) atomicAdd(&sm.hist[(key >> shift) & (nb - 1)], 1u);
                    });
                    __syncthreads();
                    uint32_t cnt, abv;
                    const uint32_t d = pick_digit(sm, nb, remaining, &remaining, &cnt, &abv);
                    prefix |= d << shift;
                    prefix_mask |= (nb - 1) << shift;
                    bits_left = shift;
                }
                compact_all_scores(prefix, remaining, false);
            }
        }
    }
    for (int i = tid; i < w; i += kSelThreads) idx[k + i] = P + i;
    if (tid == 0) len_out[bh] = bud;
}

hipError_t init_select_kernels() {
    return allow_dynamic_lds(reinterpret_cast<const void*>(select_kernel), kSelDynLds);
}

// Copies row idx[r] of K and V to row r of the outputs; `lanes` lanes of 16 bytes per row.
__global__ __launch_bounds__(256) void gather_kernel(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                     const int32_t* __restrict__ idx,
                                                     const int32_t* __restrict__ len, int H, int N, int cap,
                                                     int lanes, int64_t sb, int64_t sh, int64_t st,
                                                     int n_row_tiles, uint4* __restrict__ K_out,
                                                     uint4* __restrict__ V_out) {
    const int bh = blockIdx.x / n_row_tiles, tile = blockIdx.x % n_row_tiles;
    const int b = bh / H, h = bh % H;
    const int rows_per_block = 256 / lanes;
    const int r = tile * rows_per_block + threadIdx.x / lanes;
    const int l = threadIdx.x % lanes;
    if (r >= len[bh] || r >= cap) return;
    const int32_t row = idx[(int64_t)bh * cap + r];
    if ((uint32_t)row >= (uint32_t)N) return;          // never follow an index that is no position of the head
    const int64_t src = b * sb + h * sh + (int64_t)row * st + l;   // in 16-byte units
    const int64_t dst = ((int64_t)bh * cap + r) * lanes + l;
    K_out[dst] = K[src];
    V_out[dst] = V[src];
}

hipError_t launch_select_gather(const float* score, const int32_t* budget, const void* K,
                                const void* V, uncomp_dtype dt, int B, int H, int N, int w,
                                const int64_t ks[3], int cap, void* K_out, void* V_out,
                                int32_t* idx_out, int32_t* len_out, const Env& env, const uint32_t* tile_range,
                                int n_range_tiles, int D, const SelectWidePlan* wide, char* wide_ws) {
    hipStream_t s = env.s;
    const int BH = B * H;
    hipError_t e;
    if (wide != nullptr) {
        // a layer's few heads with long rows: many workgroups per row (same indices as select_kernel)
        e = launch_select_rows_wide(score, budget, 1, BH, N, w, cap, *wide, wide_ws, idx_out, len_out, env);
    } else {
        env.begin("select");
        select_kernel<<<dim3(BH), dim3(kSelThreads), kSelDynLds, s>>>(score, budget, 1, N, w, cap, tile_range, n_range_tiles,
                                                                      idx_out, len_out);
        env.end();
        e = hipGetLastError();
    }
    if (e != hipSuccess || K == nullptr) return e;
    const int esz = dt == UNCOMP_BF16 ? 2 : 4;
    const int per16 = 16 / esz;                       // elements per 16-byte unit
    const int lanes = D / per16;                      // 16-byte units per row: 16 (bf16) or 32 (fp32) at D = 128
    const int rows_per_block = 256 / lanes;
    const int n_row_tiles = (cap + rows_per_block - 1) / rows_per_block;
    env.begin("gather");
    gather_kernel<<<dim3((unsigned)(BH * n_row_tiles)), dim3(256), 0, s>>>(
        static_cast<const uint4*>(K), static_cast<const uint4*>(V), idx_out, len_out, H, N, cap, lanes,
        ks[0] / per16, ks[1] / per16, ks[2] / per16, n_row_tiles, static_cast<uint4*>(K_out),
        static_cast<uint4*>(V_out));
    env.end();
    return hipGetLastError();
}

// Rows of any width: idx[g][r] names the source row of output row r of group g; rows are
// copied in 16-byte units, four rows per workgroup.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ src,
                                                          const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ len, int cap, int n_src_rows,
                                                          int units, int64_t group_stride, int64_t row_stride,
                                                          int n_row_tiles, uint4* __restrict__ dst) {
    const int g = blockIdx.x / n_row_tiles, tile = blockIdx.x % n_row_tiles;
    const int n = len[g];
    for (int rr = 0; rr < 4; ++rr) {
        const int r = tile * 4 + rr;
        if (r >= n || r >= cap) return;
        const int32_t row = idx[(int64_t)g * cap + r];
        if ((uint32_t)row >= (uint32_t)n_src_rows) continue;      // never follow an index that is no row of the source
        const uint4* s = src + g * group_stride + (int64_t)row * row_stride;
        uint4* d = dst + ((int64_t)g * cap + r) * units;
        for (int u = threadIdx.x; u < units; u += 256) d[u] = s[u];
    }
}

hipError_t launch_select_rows(const float* score, const int32_t* budget, int budget_stride, int n_groups,
                              int N, int w, int cap, int32_t* idx_out, int32_t* len_out, const Env& env) {
    env.begin("select");
    select_kernel<<<dim3(n_groups), dim3(kSelThreads), kSelDynLds, env.s>>>(score, budget, budget_stride, N, w, cap,
                                                                           nullptr, 0, idx_out, len_out);
    env.end();
    return hipGetLastError();
}

hipError_t launch_gather_rows(const void* src, const int32_t* idx, const int32_t* len, int n_groups, int cap,
                              int n_src_rows, int row_bytes, int64_t group_stride_bytes, int64_t row_stride_bytes,
                              void* dst, const Env& env) {
    const int n_row_tiles = (cap + 3) / 4;
    env.begin("gather_rows");
    gather_rows_kernel<<<dim3((unsigned)(n_groups * n_row_tiles)), dim3(256), 0, env.s>>>(
        static_cast<const uint4*>(src), idx, len, cap, n_src_rows, row_bytes / 16, group_stride_bytes / 16,
        row_stride_bytes / 16,
        n_row_tiles, static_cast<uint4*>(dst));
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
