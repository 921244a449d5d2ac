// Decode-time eviction (Sec. 3.3.3 "Dynamic KV Cache Eviction", last sentence; Alg. 2
// "Decoding").  One generated token per call: the token joins every head's compacted cache,
// the head's G query rows attend to the joined cache, every entry's cumulative score grows
// by the attention it received, and a head that is over its budget gives up its
// lowest-scoring entry outside the recent window.
//
// The evicted entry's slot receives the new token, so nothing is moved: slot order is free,
// idx names each slot.
//
// bf16 caches take two kernels.  decode_attend_wave_kernel: every wave owns 128 consecutive
// rows of one head and runs on its own (no workgroup barrier): keys stream straight into
// MFMA operand layout, the 128 x G logits stay in registers, the wave's softmax (its own
// maximum and sum) goes through LDS to the lanes that stream the value rows, and the wave
// leaves (maximum, sum, unnormalised output, unnormalised probabilities) in the workspace.
// decode_update_kernel: one workgroup per head merges the waves' partials into the output,
// turns the stored probabilities into each row's share, updates the cumulative scores,
// finds the row to give up and places the new token.
//
// fp32 caches (and the plain-ALU switch) take decode_step_kernel: one workgroup per head
// does all of it with the step's probabilities held in LDS, rows read 16 lanes to a row.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kDecodeThreads = 512;
constexpr int kRowsInFlight = 4;

// Sum over the 16 lanes of a DPP row; every lane of the row receives the total.
__device__ __forceinline__ float row16_sum(float v) {
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x128, 0xF, 0xF, false));  // row_ror:8
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x124, 0xF, 0xF, false));  // row_ror:4
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x122, 0xF, 0xF, false));  // row_ror:2
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x121, 0xF, 0xF, false));  // row_ror:1
    return v;
}

// Monotone map of a float onto unsigned integers (smaller float -> smaller key).
__device__ __forceinline__ uint32_t ascending_key(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned long long other = __shfl_xor(v, o, 64);
        v = other < v ? other : v;
    }
    return v;
}

__device__ __forceinline__ void copy8(const bf16_bits* src, bf16_bits* dst) {
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
}
__device__ __forceinline__ void copy8(const float* src, float* dst) {
    reinterpret_cast<uint4*>(dst)[0] = reinterpret_cast<const uint4*>(src)[0];
    reinterpret_cast<uint4*>(dst)[1] = reinterpret_cast<const uint4*>(src)[1];
}

}  // namespace

__global__ __launch_bounds__(256) void decode_init_kernel(const float* __restrict__ score,
                                                          const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ len, int n_heads,
                                                          int P, int cap, float* __restrict__ cum) {
    const int64_t total = (int64_t)n_heads * cap;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int h = (int)(e / cap), r = (int)(e - (int64_t)h * cap);
        float c = 0.f;
        if (r < len[h]) {
            const int j = idx[e];
            if (j >= 0 && j < P) c = score[(int64_t)h * P + j];
        }
        cum[e] = c;
    }
}

// GT: compile-time bound on the query heads per KV head (G <= GT).  S: row stride of the
// probability table in LDS (floats), S >= cap + 1.
template <typename T, int GT>
__global__ __launch_bounds__(kDecodeThreads) void decode_step_kernel(
    const T* __restrict__ q, const T* __restrict__ k_new, const T* __restrict__ v_new, int G,
    const int32_t* __restrict__ pos, const int32_t* __restrict__ budget, int w, int cap, T* Kc, T* Vc,
    int32_t* idx, float* cum, int32_t* len, float* __restrict__ out, int32_t* __restrict__ evicted, int S) {
    constexpr int NT = kDecodeThreads, NW = NT / 64, RPI = NT / 16, U = kRowsInFlight;
    extern __shared__ float dyn[];                  // prob[G][S]; later the per-wave output partials
    __shared__ float red[NW][GT];
    __shared__ unsigned long long wave_best[NW];
    __shared__ int victim_slot;
    __shared__ float new_cum_s;

    const int h = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, sub = lane & 15, rg = tid >> 4;
    int n = len[h];
    n = n < 0 ? 0 : (n > cap ? cap : n);
    const int n1 = n + 1;                           // entries the queries attend to
    T* Kh = Kc + (int64_t)h * cap * kD;
    T* Vh = Vc + (int64_t)h * cap * kD;
    int32_t* idxh = idx + (int64_t)h * cap;
    float* cumh = cum + (int64_t)h * cap;
    const T* kn = k_new + (int64_t)h * kD;
    const T* vn = v_new + (int64_t)h * kD;
    if (tid == 0) victim_slot = -1;

    // ---- logits in the exp2 domain: s_gr = (q_g . k_r) / sqrt(D) * log2(e) -----------------
    {
        float qf[GT][8];
        const float qs = 0.08838834764831845f * 1.4426950408889634f;
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            if (g < G) {
                load8(q + ((int64_t)h * G + g) * kD + 8 * sub, qf[g]);
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[g][e] *= qs;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[g][e] = 0.f;
            }
        }
        for (int r0 = 0; r0 < n1; r0 += RPI * U) {
            float kv[U][8];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * RPI + rg;
                const int rc = r < n ? r : n;       // rows past the end re-read the new token
                const T* src = rc < n ? Kh + (int64_t)rc * kD : kn;
                load8(src + 8 * sub, kv[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * RPI + rg;
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    float d = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) d = fmaf(qf[g][e], kv[u][e], d);
                    d = row16_sum(d);
                    if (sub == 0 && r < n1 && g < G) dyn[g * S + r] = d;
                }
            }
        }
    }
    __syncthreads();

    // ---- softmax over the n1 entries, per query head ---------------------------------------
    float m[GT], inv[GT];
    {
#pragma unroll
        for (int g = 0; g < GT; ++g) m[g] = -INFINITY;
        for (int r = tid; r < n1; r += NT)
#pragma unroll
            for (int g = 0; g < GT; ++g)
                if (g < G) m[g] = fmaxf(m[g], dyn[g * S + r]);
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            float v = wave_max(m[g]);
            if (lane == 0) red[wave][g] = v;
        }
        __syncthreads();
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            float v = red[0][g];
#pragma unroll
            for (int x = 1; x < NW; ++x) v = fmaxf(v, red[x][g]);
            m[g] = v;
        }
        __syncthreads();
        float l[GT];
#pragma unroll
        for (int g = 0; g < GT; ++g) l[g] = 0.f;
        for (int r = tid; r < n1; r += NT)
#pragma unroll
            for (int g = 0; g < GT; ++g)
                if (g < G) {
                    const float e = exp2f(dyn[g * S + r] - m[g]);
                    dyn[g * S + r] = e;
                    l[g] += e;
                }
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            float v = wave_sum(l[g]);
            if (lane == 0) red[wave][g] = v;
        }
        __syncthreads();
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            float v = red[0][g];
#pragma unroll
            for (int x = 1; x < NW; ++x) v += red[x][g];
            inv[g] = 1.0f / v;
        }
    }

    // ---- cumulative scores, candidate for eviction -------------------------------------------
    const int posh = pos[h];
    int b = budget[h];
    b = b < w ? w : b;
    b = b > cap ? cap : b;
    const bool over = n1 > b;
    unsigned long long best = ~0ull;
    for (int r = tid; r < n1; r += NT) {
        float inc = 0.f;
#pragma unroll
        for (int g = 0; g < GT; ++g)
            if (g < G) {
                const float pr = dyn[g * S + r] * inv[g];
                dyn[g * S + r] = pr;
                inc += pr;
            }
        if (r < n) {
            const float c = cumh[r] + inc;
            cumh[r] = c;
            const int id = idxh[r];
            if (id <= posh - w) {
                const unsigned long long key = ((unsigned long long)ascending_key(c) << 32) | (uint32_t)id;
                best = key < best ? key : best;
            }
        } else {
            new_cum_s = inc;
        }
    }
    best = wave_min_u64(best);
    if (lane == 0) wave_best[wave] = best;
    __syncthreads();
    best = wave_best[0];
#pragma unroll
    for (int x = 1; x < NW; ++x) best = wave_best[x] < best ? wave_best[x] : best;
    if (over && best != ~0ull) {
        const int want = (int)(uint32_t)(best & 0xffffffffull);
        for (int r = tid; r < n; r += NT)
            if (idxh[r] == want) victim_slot = r;
    }

    // ---- attention output: out_g = sum_r p_gr v_r ---------------------------------------------
    float acc[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    for (int r0 = 0; r0 < n1; r0 += RPI * U) {
        float vv[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + u * RPI + rg;
            const int rc = r < n ? r : n;
            const T* src = rc < n ? Vh + (int64_t)rc * kD : vn;
            load8(src + 8 * sub, vv[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + u * RPI + rg;
            const int rc = r < n ? r : n;
            const float live = r < n1 ? 1.f : 0.f;
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                if (g < G) {
                    const float pr = dyn[g * S + rc] * live;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(pr, vv[u][e], acc[g][e]);
                }
            }
        }
    }
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[g][e];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            acc[g][e] = v;
        }
    __syncthreads();                                // every wave is done with the probabilities
    if (lane < 16) {
#pragma unroll
        for (int g = 0; g < GT; ++g)
            if (g < G) {
#pragma unroll
                for (int e = 0; e < 8; ++e) dyn[(wave * G + g) * kD + 8 * sub + e] = acc[g][e];
            }
    }
    __syncthreads();
    for (int o = tid; o < G * kD; o += NT) {
        float v = 0.f;
#pragma unroll
        for (int x = 0; x < NW; ++x) v += dyn[x * G * kD + o];
        out[(int64_t)h * G * kD + o] = v;
    }

    // ---- the new token takes the freed slot, or the next free one --------------------------
    int slot = n, ev = -1;
    if (over) {
        slot = victim_slot;
        if (slot >= 0) {
            ev = idxh[slot];
        } else if (n < cap) {
            slot = n;                               // nothing may leave: grow if there is room
        } else {
            ev = -2;                                // no room and nothing may leave: token dropped
        }
    }
    __syncthreads();                                // idxh[slot] read by all before it is replaced
    if (slot >= 0) {
        if (tid < 16) copy8(kn + 8 * tid, Kh + (int64_t)slot * kD + 8 * tid);
        else if (tid < 32) copy8(vn + 8 * (tid - 16), Vh + (int64_t)slot * kD + 8 * (tid - 16));
        else if (tid == 32) {
            idxh[slot] = posh;
            cumh[slot] = new_cum_s;
        }
    }
    if (tid == 0) {
        len[h] = (slot == n) ? n + 1 : n;
        if (evicted != nullptr) evicted[h] = ev;
    }
}


// ---- bf16: wave-per-128-rows attention pass ----------------------------------------------
// A wave owns WR = 128 or 256 consecutive rows of one head: 128 when the launch would
// otherwise have too few waves to fill the chip, 256 when there are plenty (half the
// partial results to write and merge).

// Workspace per head: prob [s_rows][GT] (unnormalised, relative to the owning wave's maximum),
// ml [np_max][GT][2] (maximum in the exp2 domain, sum), acc [np_max][GT][128].
template <int GT, int WR>
__global__ __launch_bounds__(256) void decode_attend_wave_kernel(
    const bf16_bits* __restrict__ q, const bf16_bits* __restrict__ k_new, const bf16_bits* __restrict__ v_new,
    int n_heads, int G, int cap, const bf16_bits* __restrict__ Kc, const bf16_bits* __restrict__ Vc,
    const int32_t* __restrict__ len, int np_max, int s_rows, float* __restrict__ ws_p, float* __restrict__ ws_ml,
    float* __restrict__ ws_acc) {
    constexpr int kTiles = WR / 16;
    extern __shared__ __align__(16) float pl_all[];                 // [4 waves][WR][GT]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int c16 = lane & 15, j = lane >> 4;
    const int wid = blockIdx.x * 4 + wv;
    const int h = wid / np_max, part = wid - h * np_max;
    if (h >= n_heads) return;
    int n = len[h];
    n = n < 0 ? 0 : (n > cap ? cap : n);
    const int n1 = n + 1;
    const int row0 = part * WR;
    if (row0 >= n1) return;                                         // waves run on their own: no barrier below
    const int n_t = min(kTiles, (n1 - row0 + 15) >> 4);
    float* pl = pl_all + wv * WR * GT;
    const bf16_bits* Kh = Kc + (int64_t)h * cap * kD;
    const bf16_bits* Vh = Vc + (int64_t)h * cap * kD;
    const bf16_bits* kn = k_new + (int64_t)h * kD;
    const bf16_bits* vn = v_new + (int64_t)h * kD;

    // queries as the B operand: column c16 = query head, zero beyond G
    bf16x8_t qb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (c16 < G) v = *reinterpret_cast<const uint4*>(q + ((int64_t)h * G + c16) * kD + 32 * ks + 8 * j);
        qb[ks] = __builtin_bit_cast(bf16x8_t, v);
    }
    // rows past the end re-read the new token (clamped, never predicated: straight-line loads
    // keep exact counts of the loads in flight); what they produce is masked below
    auto load_k = [&](uint4 dst[4], int t) {
        const int r = row0 + 16 * t + c16;
        const bf16_bits* src = (r < n ? Kh + (int64_t)r * kD : kn) + 8 * j;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dst[ks] = *reinterpret_cast<const uint4*>(src + 32 * ks);
    };
    auto load_v = [&](uint4 dst[4], int t) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = row0 + 16 * t + 4 * u + j;
            const bf16_bits* src = (r < n ? Vh + (int64_t)r * kD : vn) + 8 * c16;
            dst[u] = *reinterpret_cast<const uint4*>(src);
        }
    };

    // ---- pass 1: logits of the wave's rows; lane holds query head c16, rows 16t + 4j + v ----
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
    uint4 va[4], vb[4];
    load_v(va, 0);                                                  // under way during the softmax arithmetic

    const float qs = 0.08838834764831845f * 1.4426950408889634f;    // 1/sqrt(128) * log2(e)
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
        if (t < n_t) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool live = row0 + 16 * t + 4 * j + v < n1;
                s[t][v] = live ? s[t][v] * qs : -INFINITY;
                mx = fmaxf(mx, s[t][v]);
            }
        }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));                         // row0 < n1: at least one live row
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
    const int64_t hp = (int64_t)h * np_max + part;
    if (j == 0 && c16 < G) {
        ws_ml[(hp * GT + c16) * 2 + 0] = mx;
        ws_ml[(hp * GT + c16) * 2 + 1] = sum;
    }
    // LDS traffic of one wave is processed in issue order; the fences keep the compiler from
    // moving the reads below over the writes above
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // the wave's probabilities go to the workspace as they lie in LDS (rows of GT floats)
    {
        float* dst = ws_p + ((int64_t)h * s_rows + row0) * GT;
        const int n_f4 = n_t * 16 * GT / 4;
        for (int i = lane; i < n_f4; i += 64)
            reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(pl)[i];
    }

    // ---- pass 2: unnormalised output; lane holds features 8*c16.., rows 16t + 4u + j -----------
    float acc[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    auto weigh = [&](const uint4 vt[4], int t) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float vf[8];
            const uint32_t wds[4] = {vt[u].x, vt[u].y, vt[u].z, vt[u].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                vf[2 * i] = __uint_as_float(wds[i] << 16);
                vf[2 * i + 1] = __uint_as_float(wds[i] & 0xffff0000u);
            }
            const float* prow = pl + (16 * t + 4 * u + j) * GT;
#pragma unroll
            for (int g4 = 0; g4 < GT; g4 += 4) {
                const float4 pr = *reinterpret_cast<const float4*>(prow + g4);
                const float prs[4] = {pr.x, pr.y, pr.z, pr.w};
#pragma unroll
                for (int gg = 0; gg < 4; ++gg)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[g4 + gg][e] = fmaf(prs[gg], vf[e], acc[g4 + gg][e]);
            }
        }
    };
#pragma unroll
    for (int t = 0; t < kTiles; t += 2) {
        if (t < n_t) {
            load_v(vb, t + 1);
            weigh(va, t);
        }
        if (t + 1 < n_t) {
            load_v(va, t + 2);
            weigh(vb, t + 1);
        }
    }
    // sum over the four lane rows; lane row j keeps query head g4 + {0,2,1,3}[j]
    const int gsel = ((j & 1) << 1) | (j >> 1);
#pragma unroll
    for (int g4 = 0; g4 < GT; g4 += 4) {
        float tot[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            tot[e] = reduce4_over_rows(acc[g4][e], acc[g4 + 1][e], acc[g4 + 2][e], acc[g4 + 3][e]);
        float* dst = ws_acc + (hp * GT + g4 + gsel) * kD + 8 * c16;
        reinterpret_cast<float4*>(dst)[0] = make_float4(tot[0], tot[1], tot[2], tot[3]);
        reinterpret_cast<float4*>(dst)[1] = make_float4(tot[4], tot[5], tot[6], tot[7]);
    }
}

template <int GT, int NT>
__global__ __launch_bounds__(NT) void decode_update_kernel(
    const bf16_bits* __restrict__ k_new, const bf16_bits* __restrict__ v_new, int G,
    const int32_t* __restrict__ pos, const int32_t* __restrict__ budget, int w, int cap, bf16_bits* Kc,
    bf16_bits* Vc, int32_t* idx, float* cum, int32_t* len, float* __restrict__ out,
    int32_t* __restrict__ evicted, int wave_rows, int np_max, int s_rows, const float* __restrict__ ws_p,
    const float* __restrict__ ws_ml, const float* __restrict__ ws_acc) {
    constexpr int NW = NT / 64;
    extern __shared__ __align__(16) float dynf[];                   // three tables of [np_max][GT]
    float* coef = dynf;                                             // exp2(m_part - m) / sum
    float* pm = dynf + np_max * GT;                                 // the parts' maxima
    float* pl = dynf + 2 * np_max * GT;                             // the parts' sums
    __shared__ float head_m[GT], head_inv[GT];
    __shared__ unsigned long long wave_best[NW];
    __shared__ int victim_slot;
    __shared__ float new_cum_s;
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int n = len[h];
    n = n < 0 ? 0 : (n > cap ? cap : n);
    const int n1 = n + 1;
    const int np = (n1 + wave_rows - 1) / wave_rows;
    bf16_bits* Kh = Kc + (int64_t)h * cap * kD;
    bf16_bits* Vh = Vc + (int64_t)h * cap * kD;
    int32_t* idxh = idx + (int64_t)h * cap;
    float* cumh = cum + (int64_t)h * cap;
    const float2* ml = reinterpret_cast<const float2*>(ws_ml) + (int64_t)h * np_max * GT;
    const int posh = pos[h];
    int b = budget[h];
    b = b < w ? w : b;
    b = b > cap ? cap : b;
    const bool over = n1 > b;
    if (tid == 0) victim_slot = -1;
    for (int i = tid; i < np * GT; i += NT) {
        float2 v = make_float2(0.f, 0.f);
        if ((i % GT) < G) v = ml[i];                                // columns beyond G were never written
        pm[i] = v.x;
        pl[i] = v.y;
    }
    __syncthreads();
    if (tid < GT) {
        float m = -INFINITY, l = 0.f;
        for (int p = 0; p < np; ++p) m = fmaxf(m, pm[p * GT + tid]);
        for (int p = 0; p < np; ++p) l += pl[p * GT + tid] * exp2f(pm[p * GT + tid] - m);
        head_m[tid] = m;
        head_inv[tid] = tid < G ? 1.0f / l : 0.f;
    }
    __syncthreads();
    for (int i = tid; i < np * GT; i += NT) coef[i] = exp2f(pm[i] - head_m[i % GT]) * head_inv[i % GT];
    __syncthreads();
    // attention output: the parts' unnormalised sums, rescaled to the head's maximum
    const float* acch = ws_acc + (int64_t)h * np_max * GT * kD;
    for (int o = tid; o < G * kD; o += NT) {
        const int g = o >> 7, f = o & (kD - 1);
        float v = 0.f;
        for (int p = 0; p < np; ++p) v = fmaf(acch[(p * GT + g) * kD + f], coef[p * GT + g], v);
        out[(int64_t)h * G * kD + o] = v;
    }
    // cumulative scores and the candidate for eviction; two rows per thread in flight
    const float* ph = ws_p + (int64_t)h * s_rows * GT;
    unsigned long long best = ~0ull;
    auto share = [&](int r) {                                       // sum over the query heads of p_gr
        const float* cf = coef + (r / wave_rows) * GT;
        float inc = 0.f;
#pragma unroll
        for (int g4 = 0; g4 < GT; g4 += 4) {
            const float4 pr = *reinterpret_cast<const float4*>(ph + (int64_t)r * GT + g4);
            const float4 cc = *reinterpret_cast<const float4*>(cf + g4);
            inc += pr.x * cc.x;
            inc += pr.y * cc.y;
            inc += pr.z * cc.z;
            inc += pr.w * cc.w;
        }
        return inc;
    };
    for (int r0 = tid; r0 < n1; r0 += 2 * NT) {
        const int r1 = r0 + NT;
        const int ra = r0 < n ? r0 : (n > 0 ? n - 1 : 0), rb = r1 < n ? r1 : ra;   // clamped: loads first
        const float inc0 = share(r0), inc1 = share(r1 < n1 ? r1 : r0);
        const float c0 = n > 0 ? cumh[ra] : 0.f, c1 = n > 0 ? cumh[rb] : 0.f;
        const int id0 = n > 0 ? idxh[ra] : 0, id1 = n > 0 ? idxh[rb] : 0;
        if (r0 < n) {
            const float c = c0 + inc0;
            cumh[r0] = c;
            if (id0 <= posh - w) {
                const unsigned long long key = ((unsigned long long)ascending_key(c) << 32) | (uint32_t)id0;
                best = key < best ? key : best;
            }
        } else {
            new_cum_s = inc0;
        }
        if (r1 < n) {
            const float c = c1 + inc1;
            cumh[r1] = c;
            if (id1 <= posh - w) {
                const unsigned long long key = ((unsigned long long)ascending_key(c) << 32) | (uint32_t)id1;
                best = key < best ? key : best;
            }
        } else if (r1 == n) {
            new_cum_s = inc1;
        }
    }
    best = wave_min_u64(best);
    if (lane == 0) wave_best[wave] = best;
    __syncthreads();
    best = wave_best[0];
#pragma unroll
    for (int x = 1; x < NW; ++x) best = wave_best[x] < best ? wave_best[x] : best;
    if (over && best != ~0ull) {
        const int want = (int)(uint32_t)(best & 0xffffffffull);
        for (int r = tid; r < n; r += NT)
            if (idxh[r] == want) victim_slot = r;
    }
    __syncthreads();
    int slot = n, ev = -1;
    if (over) {
        slot = victim_slot;
        if (slot >= 0) {
            ev = idxh[slot];
        } else if (n < cap) {
            slot = n;
        } else {
            ev = -2;
        }
    }
    __syncthreads();                                                // idxh[slot] read by all before it is replaced
    if (slot >= 0) {
        const bf16_bits* kn = k_new + (int64_t)h * kD;
        const bf16_bits* vn = v_new + (int64_t)h * kD;
        if (tid < 16) copy8(kn + 8 * tid, Kh + (int64_t)slot * kD + 8 * tid);
        else if (tid < 32) copy8(vn + 8 * (tid - 16), Vh + (int64_t)slot * kD + 8 * (tid - 16));
        else if (tid == 32) {
            idxh[slot] = posh;
            cumh[slot] = new_cum_s;
        }
    }
    if (tid == 0) {
        len[h] = (slot == n) ? n + 1 : n;
        if (evicted != nullptr) evicted[h] = ev;
    }
}

DecodePlan plan_decode(int n_heads, int G, int cap) {
    DecodePlan p;
    p.GT = G <= 4 ? 4 : (G <= 8 ? 8 : 16);
    // 256-row waves when that still leaves a few thousand waves to spread over the chip
    const int64_t waves256 = (int64_t)n_heads * ((cap + 1 + 255) / 256);
    p.wave_rows = (p.GT <= 8 && waves256 >= 2048) ? 256 : 128;
    p.s_rows = (cap + 1 + p.wave_rows - 1) / p.wave_rows * p.wave_rows;
    p.np_max = p.s_rows / p.wave_rows;
    size_t off = 0;
    p.out_off = off;
    off = align_up(off + (size_t)n_heads * G * kD * sizeof(float), 256);
    p.p_off = off;
    off = align_up(off + (size_t)n_heads * p.s_rows * p.GT * sizeof(float), 256);
    p.ml_off = off;
    off = align_up(off + (size_t)n_heads * p.np_max * p.GT * 2 * sizeof(float), 256);
    p.acc_off = off;
    off = align_up(off + (size_t)n_heads * p.np_max * p.GT * kD * sizeof(float), 256);
    p.bytes = off;
    return p;
}

template <int GT, int WR>
static hipError_t launch_decode_wave_t(const void* q, const void* k_new, const void* v_new, int n_heads, int G,
                                       const int32_t* pos, const int32_t* budget, int w, int cap, void* Kc,
                                       void* Vc, int32_t* idx, float* cum, int32_t* len, float* out,
                                       int32_t* evicted, const DecodePlan& p, char* ws, const Env& env) {
    float* ws_p = reinterpret_cast<float*>(ws + p.p_off);
    float* ws_ml = reinterpret_cast<float*>(ws + p.ml_off);
    float* ws_acc = reinterpret_cast<float*>(ws + p.acc_off);
    const int64_t waves = (int64_t)n_heads * p.np_max;
    const unsigned grid = (unsigned)((waves + 3) / 4);
    const size_t lds_a = (size_t)4 * WR * GT * sizeof(float);
    env.begin("decode_attend_wave");
    decode_attend_wave_kernel<GT, WR><<<grid, 256, lds_a, env.s>>>(
        static_cast<const bf16_bits*>(q), static_cast<const bf16_bits*>(k_new), static_cast<const bf16_bits*>(v_new),
        n_heads, G, cap, static_cast<const bf16_bits*>(Kc), static_cast<const bf16_bits*>(Vc), len, p.np_max,
        p.s_rows, ws_p, ws_ml, ws_acc);
    env.end();
    const size_t lds_b = (size_t)3 * p.np_max * GT * sizeof(float);
    const bf16_bits* kn = static_cast<const bf16_bits*>(k_new);
    const bf16_bits* vn = static_cast<const bf16_bits*>(v_new);
    bf16_bits* Kp = static_cast<bf16_bits*>(Kc);
    bf16_bits* Vp = static_cast<bf16_bits*>(Vc);
    env.begin("decode_update");
    // few heads: larger workgroups to have more loads in flight; many heads: more workgroups per CU
    if (n_heads < 2048)
        decode_update_kernel<GT, 512><<<n_heads, 512, lds_b, env.s>>>(kn, vn, G, pos, budget, w, cap, Kp, Vp, idx, cum,
                                                                      len, out, evicted, WR, p.np_max, p.s_rows, ws_p,
                                                                      ws_ml, ws_acc);
    else
        decode_update_kernel<GT, 256><<<n_heads, 256, lds_b, env.s>>>(kn, vn, G, pos, budget, w, cap, Kp, Vp, idx, cum,
                                                                      len, out, evicted, WR, p.np_max, p.s_rows, ws_p,
                                                                      ws_ml, ws_acc);
    env.end();
    return hipGetLastError();
}

hipError_t launch_decode_wave(const void* q, const void* k_new, const void* v_new, int n_heads, int G,
                              const int32_t* pos, const int32_t* budget, int w, int cap, void* Kc, void* Vc,
                              int32_t* idx, float* cum, int32_t* len, float* out, int32_t* evicted,
                              const DecodePlan& p, char* ws, const Env& env) {
#define UNCOMP_WAVE_CASE(GT, WR)                                                                                  \
    return launch_decode_wave_t<GT, WR>(q, k_new, v_new, n_heads, G, pos, budget, w, cap, Kc, Vc, idx, cum, len, \
                                        out, evicted, p, ws, env)
    if (p.wave_rows == 256) {
        if (p.GT == 4) UNCOMP_WAVE_CASE(4, 256);
        UNCOMP_WAVE_CASE(8, 256);
    }
    if (p.GT == 4) UNCOMP_WAVE_CASE(4, 128);
    if (p.GT == 8) UNCOMP_WAVE_CASE(8, 128);
    UNCOMP_WAVE_CASE(16, 128);
#undef UNCOMP_WAVE_CASE
}

hipError_t launch_decode_init(const float* score, const int32_t* idx, const int32_t* len, int n_heads,
                              int N, int w, int cap, float* cum, const Env& env) {
    int64_t total = (int64_t)n_heads * cap;
    int blocks = (int)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
    env.begin("decode_init");
    decode_init_kernel<<<blocks, 256, 0, env.s>>>(score, idx, len, n_heads, N - w, cap, cum);
    env.end();
    return hipGetLastError();
}

// dynamic LDS the one-kernel decode path may ask for: G*(cap+1) <= 36864 floats plus rounding of cap
constexpr size_t kDecodeStepLdsMax = (36864 + 64) * sizeof(float);

size_t decode_update_lds_bytes(const DecodePlan& p) { return (size_t)3 * p.np_max * p.GT * sizeof(float); }

size_t decode_step_lds_bytes(int G, int cap) {
    const size_t S = ((size_t)cap + 1 + 3) / 4 * 4;
    size_t prob = (size_t)G * S;
    size_t part = (size_t)(kDecodeThreads / 64) * G * kD;
    return (prob > part ? prob : part) * sizeof(float);
}

template <typename T, int GT>
static hipError_t launch_decode_step_t(const void* q, const void* k_new, const void* v_new, int n_heads, int G,
                                       const int32_t* pos, const int32_t* budget, int w, int cap, void* Kc,
                                       void* Vc, int32_t* idx, float* cum, int32_t* len, float* out,
                                       int32_t* evicted, const Env& env) {
    const int S = (cap + 1 + 3) / 4 * 4;
    const size_t lds = decode_step_lds_bytes(G, cap);
    auto kern = decode_step_kernel<T, GT>;
    if (lds > kDecodeStepLdsMax) return hipErrorInvalidValue;      // the interface checks G*(cap+1) before
    env.begin("decode_step");
    kern<<<n_heads, kDecodeThreads, lds, env.s>>>(static_cast<const T*>(q), static_cast<const T*>(k_new),
                                                  static_cast<const T*>(v_new), G, pos, budget, w, cap,
                                                  static_cast<T*>(Kc), static_cast<T*>(Vc), idx, cum, len, out,
                                                  evicted, S);
    env.end();
    return hipGetLastError();
}

hipError_t launch_decode_step(const void* q, const void* k_new, const void* v_new, uncomp_dtype dt,
                              int n_heads, int G, const int32_t* pos, const int32_t* budget, int w, int cap,
                              void* Kc, void* Vc, int32_t* idx, float* cum, int32_t* len, float* out,
                              int32_t* evicted, const Env& env) {
#define UNCOMP_DECODE_CASE(T, GT)                                                                          \
    return launch_decode_step_t<T, GT>(q, k_new, v_new, n_heads, G, pos, budget, w, cap, Kc, Vc, idx, cum, \
                                       len, out, evicted, env)
    if (dt == UNCOMP_BF16) {
        if (G <= 4) UNCOMP_DECODE_CASE(bf16_bits, 4);
        if (G <= 8) UNCOMP_DECODE_CASE(bf16_bits, 8);
        UNCOMP_DECODE_CASE(bf16_bits, 16);
    }
    if (G <= 4) UNCOMP_DECODE_CASE(float, 4);
    if (G <= 8) UNCOMP_DECODE_CASE(float, 8);
    UNCOMP_DECODE_CASE(float, 16);
#undef UNCOMP_DECODE_CASE
}

template <typename T, int GT>
static hipError_t allow_decode_step() {
    return allow_dynamic_lds(reinterpret_cast<const void*>(decode_step_kernel<T, GT>), kDecodeStepLdsMax);
}

hipError_t init_decode_kernels() {
    hipError_t e = allow_decode_step<bf16_bits, 4>();
    if (e == hipSuccess) e = allow_decode_step<bf16_bits, 8>();
    if (e == hipSuccess) e = allow_decode_step<bf16_bits, 16>();
    if (e == hipSuccess) e = allow_decode_step<float, 4>();
    if (e == hipSuccess) e = allow_decode_step<float, 8>();
    if (e == hipSuccess) e = allow_decode_step<float, 16>();
    return e;
}

}  // namespace uncomp
