// Decode-time eviction (Sec. 3.3.3 "Dynamic KV Cache Eviction", last sentence; Alg. 2
// "Decoding").  One generated token per call: the token joins every head's compacted cache,
// the head's G query rows attend to the joined cache, every entry's cumulative score grows
// by the attention it received, and a head that is over its budget gives up its
// lowest-scoring entry outside the recent window.
//
// One workgroup per KV head; a head's cache is at most a few thousand rows, so the whole
// step (logits, softmax, score update, arg-min, attention output, replacement) stays in one
// kernel with the probabilities of the step held in LDS.  Rows are read 16 lanes to a row
// (16 bytes per lane for bf16), kRowsInFlight rows per lane in flight.  The evicted entry's
// slot receives the new token, so nothing is moved: slot order is free, idx names each slot.
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

hipError_t launch_decode_init(const float* score, const int32_t* idx, const int32_t* len, int n_heads,
                              int N, int w, int cap, float* cum, const Env& env) {
    int64_t total = (int64_t)n_heads * cap;
    int blocks = (int)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
    env.begin("decode_init");
    decode_init_kernel<<<blocks, 256, 0, env.s>>>(score, idx, len, n_heads, N - w, cap, cum);
    env.end();
    return hipGetLastError();
}

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
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
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

}  // namespace uncomp
