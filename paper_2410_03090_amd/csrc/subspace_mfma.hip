// bf16 MFMA versions of the two tall-skinny products of the wide-matrix entropy (Z = X Q and
// W = X^T Z; see subspace.hip).  X is bf16 as it comes; the fp32 factor (Q, resp. Z) is split into
// a high and a low bf16 half, x = hi + lo with |lo| <= 2^-9 |hi|, and both halves go through the
// matrix cores with fp32 accumulation, which keeps the product at ~2^-17 relative error.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kP = 128;
constexpr int kQtRow = 40;               // LDS row of one column of Q^T: 32 elements + 8 of padding (80 bytes:
                                         // 16 consecutive rows then start in 16 different 16-byte bank groups)

// round-to-nearest-even bf16 of a finite float
__device__ __forceinline__ uint32_t bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

}  // namespace

// Qt_hi / Qt_lo [128][D] bf16 from Q [D][128] fp32: the transposed halves that the X Q kernel streams.
__global__ __launch_bounds__(256) void sub_qt_split_kernel(const float* __restrict__ Q, int D, bf16_bits* __restrict__ Qt_hi,
                                                           bf16_bits* __restrict__ Qt_lo) {
    __shared__ float tile[32][33];
    const int d0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;           // 32 x 8
    for (int r = ty; r < 32; r += 8) tile[r][tx] = Q[(int64_t)(d0 + r) * kP + j0 + tx];
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const float v = tile[tx][r];                                  // Q[d0 + tx][j0 + r]
        const uint32_t hi = bf16_rne(v);
        const uint32_t lo = bf16_rne(v - __uint_as_float(hi << 16));
        Qt_hi[(int64_t)(j0 + r) * D + d0 + tx] = (bf16_bits)hi;
        Qt_lo[(int64_t)(j0 + r) * D + d0 + tx] = (bf16_bits)lo;
    }
}

// out[kc][t][j] = sum over the k chunk of X[t][d] (Qt_hi[j][d] + Qt_lo[j][d]).
// Workgroup: 256 rows of X; wave: 64 rows (four 16-row blocks) x 128 columns.  Per step of 32 d the
// X rows come straight from global memory in MFMA A-operand layout (lane = row%16, 16 bytes), the
// step's slice of Q^T (128 x 32, both halves) is staged in LDS by the whole workgroup, double
// buffered, and read as B operands.
// LO: also multiply by the low halves (off in the early rounds of the iteration, whose errors the later rounds remove).
template <bool LO>
__global__ __launch_bounds__(256) void sub_xq_mfma_kernel(const bf16_bits* __restrict__ X, int64_t ldx,
                                                          const bf16_bits* __restrict__ Qt_hi,
                                                          const bf16_bits* __restrict__ Qt_lo, int N, int D,
                                                          int k_chunk, float* __restrict__ out) {
    __shared__ __align__(16) bf16_bits qs[2][2][kP * kQtRow];         // [buffer][half][column][d]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = lane & 15, kq = lane >> 4;
    const int row0 = blockIdx.x * 256 + wv * 64;
    const int kc = blockIdx.y;
    const int k_begin = kc * k_chunk, k_end = min(D, k_begin + k_chunk);
    const int n_steps = (k_end - k_begin) >> 5;
    f32x4_t acc[4][8];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) acc[rb][cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // staging: 128 columns x 4 pieces of 8 d, for both halves: four 16-byte loads per thread
    const int s_col0 = tid >> 2, s_piece = tid & 3;                    // columns s_col0 and s_col0 + 64
    uint4 sh0, sh1, sl0, sl1;                                        // staged pieces of Q^T (named: an array here ends up in scratch)
    uint4 a_cur[4], a_nxt[4];
    auto stage_load = [&](int step) {
        const int k0 = k_begin + 32 * step + 8 * s_piece;
        sh0 = *reinterpret_cast<const uint4*>(Qt_hi + (int64_t)s_col0 * D + k0);
        sh1 = *reinterpret_cast<const uint4*>(Qt_hi + (int64_t)(s_col0 + 64) * D + k0);
        if (LO) {
            sl0 = *reinterpret_cast<const uint4*>(Qt_lo + (int64_t)s_col0 * D + k0);
            sl1 = *reinterpret_cast<const uint4*>(Qt_lo + (int64_t)(s_col0 + 64) * D + k0);
        }
    };
    auto stage_store = [&](int buf) {
        *reinterpret_cast<uint4*>(&qs[buf][0][s_col0 * kQtRow + 8 * s_piece]) = sh0;
        *reinterpret_cast<uint4*>(&qs[buf][0][(s_col0 + 64) * kQtRow + 8 * s_piece]) = sh1;
        if (LO) {
            *reinterpret_cast<uint4*>(&qs[buf][1][s_col0 * kQtRow + 8 * s_piece]) = sl0;
            *reinterpret_cast<uint4*>(&qs[buf][1][(s_col0 + 64) * kQtRow + 8 * s_piece]) = sl1;
        }
    };
    // rows past the end re-read the last row (clamped, never predicated); their results are not stored
    auto load_a_next = [&](int step) {
        const int k0 = k_begin + 32 * step + 8 * kq;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const int r = min(row0 + 16 * rb + n, N - 1);
            a_nxt[rb] = *reinterpret_cast<const uint4*>(X + (int64_t)r * ldx + k0);
        }
    };
    stage_load(0);
    load_a_next(0);
    stage_store(0);
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) a_cur[rb] = a_nxt[rb];
    __syncthreads();
    for (int step = 0; step < n_steps; ++step) {
        const int buf = step & 1;
        const bool more = step + 1 < n_steps;
        if (more) {
            stage_load(step + 1);
            load_a_next(step + 1);
        }
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            const bf16x8_t bh = __builtin_bit_cast(
                bf16x8_t, *reinterpret_cast<const uint4*>(&qs[buf][0][(16 * cb + n) * kQtRow + 8 * kq]));
            bf16x8_t bl = bh;
            if (LO)
                bl = __builtin_bit_cast(
                    bf16x8_t, *reinterpret_cast<const uint4*>(&qs[buf][1][(16 * cb + n) * kQtRow + 8 * kq]));
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const bf16x8_t av = __builtin_bit_cast(bf16x8_t, a_cur[rb]);
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bh, acc[rb][cb], 0, 0, 0);
                if (LO) acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bl, acc[rb][cb], 0, 0, 0);
            }
        }
        if (more) stage_store(buf ^ 1);          // the other buffer: everyone left it at the last barrier
        __syncthreads();
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) a_cur[rb] = a_nxt[rb];
    }
    // accumulator lane: column 16 cb + n, rows 16 rb + 4 kq + v
    float* o = out + (int64_t)kc * N * kP;
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = row0 + 16 * rb + 4 * kq + v;
            if (r < N) {
#pragma unroll
                for (int cb = 0; cb < 8; ++cb) o[(int64_t)r * kP + 16 * cb + n] = acc[rb][cb][v];
            }
        }
}


// Zh / Zl [N][128] bf16 halves of Z [N][128] fp32 (row-major, as the X^T Z kernel streams them).
__global__ __launch_bounds__(256) void sub_z_split_kernel(const float* __restrict__ Z, int64_t total,
                                                          bf16_bits* __restrict__ Zh, bf16_bits* __restrict__ Zl) {
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= total) return;
    const float4 z = *reinterpret_cast<const float4*>(Z + e);
    const float v[4] = {z.x, z.y, z.z, z.w};
    uint32_t h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        h[i] = bf16_rne(v[i]);
        l[i] = bf16_rne(v[i] - __uint_as_float(h[i] << 16));
    }
    *reinterpret_cast<uint2*>(Zh + e) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
    *reinterpret_cast<uint2*>(Zl + e) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
}

// out[tc][d][j] = sum over the token chunk of X[t][d] (Zh[t][j] + Zl[t][j]) for the 128 features d of
// one slab.  The contraction runs over tokens, the slow index of both operands, so operands are
// transposed in registers: a lane loads 8 tokens x 8 features (16 bytes per token) and byte
// permutes turn them into 8 operands "feature 8 i + c over 8 tokens".  The four waves of a
// workgroup share one slab of X: per round of 128 tokens every wave loads and transposes one step
// of 32 tokens and leaves its 8 operands in LDS (double buffered, one barrier per round); then every
// wave multiplies all four steps with its own 32 columns of Z, whose operands (2 columns per lane)
// it builds itself.  Accumulator block (c, b): feature 8 i + c, column 32 w + 2 n + b.
template <bool LO>
__global__ __launch_bounds__(256) void sub_xtz_mfma_kernel(const bf16_bits* __restrict__ X, int64_t ldx,
                                                           const bf16_bits* __restrict__ Zh,
                                                           const bf16_bits* __restrict__ Zl, int N, int D, int t_chunk,
                                                           float* __restrict__ out) {
    __shared__ __align__(16) uint4 xs[2][4][8][64];                   // [buffer][step][operand][lane]: 64 KB
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int slab = blockIdx.x, tc = blockIdx.y;
    const int t_begin = tc * t_chunk, t_end = min(N, t_begin + t_chunk);
    const int n_rounds = (t_end - t_begin + 127) >> 7;
    const bf16_bits* xbase = X + (int64_t)slab * 128 + 8 * m;
    const int col0 = 32 * wv + 2 * m;                                // this lane's two columns of Z
    f32x4_t acc[8][2];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        acc[c][0] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        acc[c][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    uint4 x0, x1, x2, x3, x4, x5, x6, x7;                            // this wave's step of the next round (named: no scratch)
    // tokens past the end contribute nothing: their X rows are taken as zero
    auto row_or_zero = [&](int t) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (t < t_end) v = *reinterpret_cast<const uint4*>(xbase + (int64_t)t * ldx);
        return v;
    };
    auto load_x = [&](int round) {
        const int t0 = t_begin + 128 * round + 32 * wv + 8 * g;
        x0 = row_or_zero(t0);
        x1 = row_or_zero(t0 + 1);
        x2 = row_or_zero(t0 + 2);
        x3 = row_or_zero(t0 + 3);
        x4 = row_or_zero(t0 + 4);
        x5 = row_or_zero(t0 + 5);
        x6 = row_or_zero(t0 + 6);
        x7 = row_or_zero(t0 + 7);
    };
    // operand c, dword j = feature 8m + c of tokens (2j, 2j+1) of this lane's 8 tokens
    auto store_x = [&](int buf) {
        const uint4 raw[8] = {x0, x1, x2, x3, x4, x5, x6, x7};
        uint32_t r[8][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t a[4] = {raw[2 * j].x, raw[2 * j].y, raw[2 * j].z, raw[2 * j].w};
            const uint32_t b[4] = {raw[2 * j + 1].x, raw[2 * j + 1].y, raw[2 * j + 1].z, raw[2 * j + 1].w};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                r[2 * u][j] = __builtin_amdgcn_perm(b[u], a[u], 0x05040100u);       // low halves
                r[2 * u + 1][j] = __builtin_amdgcn_perm(b[u], a[u], 0x07060302u);   // high halves
            }
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) xs[buf][wv][c][lane] = make_uint4(r[c][0], r[c][1], r[c][2], r[c][3]);
    };
    load_x(0);
    store_x(0);
    __syncthreads();
    for (int round = 0; round < n_rounds; ++round) {
        const int buf = round & 1;
        const bool more = round + 1 < n_rounds;
        if (more) load_x(round + 1);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            // Z operands of this step: tokens t0 + e, columns col0, col0 + 1 (one dword per token and half)
            const int t0 = t_begin + 128 * round + 32 * st + 8 * g;
            uint32_t zh[8], zl[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int t = min(t0 + e, N - 1);                    // clamped: X is zero there anyway
                zh[e] = *reinterpret_cast<const uint32_t*>(Zh + (int64_t)t * kP + col0);
                zl[e] = LO ? *reinterpret_cast<const uint32_t*>(Zl + (int64_t)t * kP + col0) : 0u;
            }
            bf16x8_t bh0, bh1, bl0, bl1;
            {
                uint32_t p0[4], p1[4], q0[4], q1[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    p0[j] = __builtin_amdgcn_perm(zh[2 * j + 1], zh[2 * j], 0x05040100u);
                    p1[j] = __builtin_amdgcn_perm(zh[2 * j + 1], zh[2 * j], 0x07060302u);
                    q0[j] = __builtin_amdgcn_perm(zl[2 * j + 1], zl[2 * j], 0x05040100u);
                    q1[j] = __builtin_amdgcn_perm(zl[2 * j + 1], zl[2 * j], 0x07060302u);
                }
                bh0 = __builtin_bit_cast(bf16x8_t, make_uint4(p0[0], p0[1], p0[2], p0[3]));
                bh1 = __builtin_bit_cast(bf16x8_t, make_uint4(p1[0], p1[1], p1[2], p1[3]));
                bl0 = __builtin_bit_cast(bf16x8_t, make_uint4(q0[0], q0[1], q0[2], q0[3]));
                bl1 = __builtin_bit_cast(bf16x8_t, make_uint4(q1[0], q1[1], q1[2], q1[3]));
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const bf16x8_t av = __builtin_bit_cast(bf16x8_t, xs[buf][st][c][lane]);
                acc[c][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bh0, acc[c][0], 0, 0, 0);
                if (LO) acc[c][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bl0, acc[c][0], 0, 0, 0);
                acc[c][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bh1, acc[c][1], 0, 0, 0);
                if (LO) acc[c][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bl1, acc[c][1], 0, 0, 0);
            }
        }
        if (more) store_x(buf ^ 1);
        __syncthreads();
    }
    // accumulator lane: column index n = lane % 16, rows i = 4 (lane / 16) + v
    float* o = out + ((int64_t)tc * D + (int64_t)slab * 128) * kP + 32 * wv;
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int feat = 8 * (4 * g + v) + c;
            *reinterpret_cast<float2*>(o + (int64_t)feat * kP + 2 * m) = make_float2(acc[c][0][v], acc[c][1][v]);
        }
}

// out[e] = sum over the chunks of part[c][e], e < total (fixed order).
__global__ __launch_bounds__(256) void sub_sum_parts_kernel(const float* __restrict__ part, int n_parts, int64_t total,
                                                            float* __restrict__ out) {
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= total) return;
    float4 a = *reinterpret_cast<const float4*>(part + e);
    for (int c = 1; c < n_parts; ++c) {
        const float4 b = *reinterpret_cast<const float4*>(part + (int64_t)c * total + e);
        a.x += b.x;
        a.y += b.y;
        a.z += b.z;
        a.w += b.w;
    }
    *reinterpret_cast<float4*>(out + e) = a;
}

hipError_t launch_xq_mfma(const bf16_bits* X, int64_t ldx, const float* Q, int N, int D, bf16_bits* Qt_hi,
                          bf16_bits* Qt_lo, int n_split, float* Zpart, float* Z, hipStream_t s, bool precise) {
    sub_qt_split_kernel<<<dim3((unsigned)(D / 32), kP / 32), dim3(256), 0, s>>>(Q, D, Qt_hi, Qt_lo);
    const int k_chunk = ((D + n_split - 1) / n_split + 31) / 32 * 32;
    const int splits = (D + k_chunk - 1) / k_chunk;
    float* dst = splits == 1 ? Z : Zpart;
    const dim3 grid((unsigned)((N + 255) / 256), (unsigned)splits);
    if (precise) sub_xq_mfma_kernel<true><<<grid, dim3(256), 0, s>>>(X, ldx, Qt_hi, Qt_lo, N, D, k_chunk, dst);
    else sub_xq_mfma_kernel<false><<<grid, dim3(256), 0, s>>>(X, ldx, Qt_hi, Qt_lo, N, D, k_chunk, dst);
    if (splits > 1) {
        const int64_t total = (int64_t)N * kP;
        sub_sum_parts_kernel<<<dim3((unsigned)((total / 4 + 255) / 256)), dim3(256), 0, s>>>(Zpart, splits, total, Z);
    }
    return hipGetLastError();
}

// Wpart[tc][D][128] = partial X^T Z over token chunks; Zh / Zl are scratch for the two halves of Z.
hipError_t launch_xtz_mfma(const bf16_bits* X, int64_t ldx, const float* Z, int N, int D, bf16_bits* Zh, bf16_bits* Zl,
                           int t_chunk, int n_tchunks, float* Wpart, hipStream_t s, bool precise) {
    const int64_t total = (int64_t)N * kP;
    sub_z_split_kernel<<<dim3((unsigned)((total / 4 + 255) / 256)), dim3(256), 0, s>>>(Z, total, Zh, Zl);
    const dim3 grid((unsigned)(D / 128), (unsigned)n_tchunks);
    if (precise) sub_xtz_mfma_kernel<true><<<grid, dim3(256), 0, s>>>(X, ldx, Zh, Zl, N, D, t_chunk, Wpart);
    else sub_xtz_mfma_kernel<false><<<grid, dim3(256), 0, s>>>(X, ldx, Zh, Zl, N, D, t_chunk, Wpart);
    return hipGetLastError();
}

}  // namespace uncomp
