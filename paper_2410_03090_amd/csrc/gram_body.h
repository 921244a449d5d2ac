// The bf16 Gram pass as device functions, shared by the Gram kernel and by the kernel that runs it
// beside the first scoring pass (Sec. 3.1 Eq. 1: the sums S = sum x x^T and s = sum x that the
// covariance is formed from).
#pragma once

#include "common.h"
#include "device_utils.h"

namespace uncomp {

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernel.  The contraction runs over tokens while memory is feature-contiguous,
// so each operand needs "8 tokens of one feature" per lane.  Because the two operands of
// X^T X are the same data and the order of tokens inside a sum is free, one register
// transpose serves both: lane (m, g) of a wave (m = lane%16, g = lane/16) loads, for the 8
// tokens 8g..8g+7 of a 32-token step, the 16 bytes holding features 8m..8m+7, and eight
// byte-permutes per feature pair turn them into eight operands "feature 8m+c, tokens
// 8g..8g+7" (c = 0..7).  v_mfma_f32_16x16x32_bf16 on operands (cA, cB) then accumulates the
// block G[8i+cA][8j+cB], i,j = 0..15; only cA <= cB is computed (36 of 64 blocks) and
// mirrored on output.  Column sums come from v_dot2 against (1,1) on the same operands.
// The eight waves of a workgroup (two per SIMD) take 32-token steps round-robin with kGramStages
// steps of loads in flight each, and combine their accumulators through LDS at the end of the chunk.
// ---------------------------------------------------------------------------------------
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

constexpr int kGramBlocks = 36;                     // upper-triangular 16x16-output blocks

__device__ __forceinline__ int tri_index(int ca, int cb) { return ca * 8 - ca * (ca - 1) / 2 + (cb - ca); }

struct GramOperands {
    uint32_t r[8][4];     // r[c][j]: feature 8m+c, tokens (2j, 2j+1) of this lane's 8 tokens
};

__device__ __forceinline__ void gram_transpose(const uint4 raw[8], GramOperands& op) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t a[4] = {raw[2 * j].x, raw[2 * j].y, raw[2 * j].z, raw[2 * j].w};
        const uint32_t b[4] = {raw[2 * j + 1].x, raw[2 * j + 1].y, raw[2 * j + 1].z, raw[2 * j + 1].w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            op.r[2 * u][j] = __builtin_amdgcn_perm(b[u], a[u], 0x05040100u);       // low halves
            op.r[2 * u + 1][j] = __builtin_amdgcn_perm(b[u], a[u], 0x07060302u);   // high halves
        }
    }
}

constexpr size_t kGramLdsBytes = (4 * kGramBlocks * 256 + 4 * 64 * 8) * sizeof(float);

// One wave's share of a chunk: steps wv, wv + kWaves, ... of 32 tokens each (wv = 0..kWaves-1).  `base` points at
// this lane's 8 features (8 * (lane % 16) ..) of token 0 of the matrix; g = lane / 16.
template <int kGramStages, int kWaves>   // 32-token steps of loads in flight per wave; waves sharing the chunk
__device__ __forceinline__ void gram_wave_accumulate(const bf16_bits* __restrict__ base, int64_t ldx, int t_begin,
                                                     int t_end, int wv, int g, f32x4_t acc[kGramBlocks],
                                                     float csum[8]) {
    const int n_steps = (t_end - t_begin + 31) / 32;
#pragma unroll
    for (int b = 0; b < kGramBlocks; ++b) acc[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 8; ++i) csum[i] = 0.f;
    uint4 buf[kGramStages][8];
    auto load_step = [&](uint4 dst[8], int step) {
        const int t0 = t_begin + step * 32 + 8 * g;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int t = t0 + e;
            if (step < n_steps && t < t_end) {
                dst[e] = *reinterpret_cast<const uint4*>(base + (int64_t)t * ldx);
            } else {
                dst[e] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
    };
    auto compute_step = [&](const uint4 src[8]) {
        GramOperands op;
        gram_transpose(src, op);
        bf16x8_t v[8];
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
            uint4 packed = make_uint4(op.r[cc][0], op.r[cc][1], op.r[cc][2], op.r[cc][3]);
            v[cc] = __builtin_bit_cast(bf16x8_t, packed);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                csum[cc] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, op.r[cc][j]),
                                                           __builtin_bit_cast(bf16x2_t, 0x3f803f80u), csum[cc], false);
        }
#pragma unroll
        for (int ca = 0; ca < 8; ++ca)
#pragma unroll
            for (int cb = ca; cb < 8; ++cb)
                acc[tri_index(ca, cb)] =
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(v[ca], v[cb], acc[tri_index(ca, cb)], 0, 0, 0);
    };

    // this wave's steps: wv, wv + kWaves, ...; kGramStages of them in flight
#pragma unroll
    for (int st = 0; st < kGramStages; ++st) load_step(buf[st], wv + kWaves * st);
    for (int s0 = wv; s0 < n_steps; s0 += kWaves * kGramStages) {
#pragma unroll
        for (int st = 0; st < kGramStages; ++st) {
            compute_step(buf[st]);
            load_step(buf[st], s0 + kWaves * (st + kGramStages));
        }
    }
}

// Leaves one wave's blocks and column sums in LDS (red: kGramLdsBytes).  A workgroup barrier must follow.
__device__ __forceinline__ void gram_wave_to_lds(float* red, int wv, int lane, const f32x4_t acc[kGramBlocks],
                                                 const float csum[8]) {
    float* my = red + (size_t)wv * (kGramBlocks * 256);
#pragma unroll
    for (int b = 0; b < kGramBlocks; ++b)
        *reinterpret_cast<float4*>(my + b * 256 + lane * 4) = make_float4(acc[b][0], acc[b][1], acc[b][2], acc[b][3]);
    float* sums = red + 4 * kGramBlocks * 256;       // [4][64][8]
#pragma unroll
    for (int i = 0; i < 8; ++i) sums[(wv * 64 + lane) * 8 + i] = csum[i];
}

// Adds the partials that wave `src` left in LDS to this wave's registers (both hold the same blocks and lanes).
__device__ __forceinline__ void gram_wave_add_from_lds(const float* red, int src, int lane, f32x4_t acc[kGramBlocks],
                                                       float csum[8]) {
    const float* other = red + (size_t)src * (kGramBlocks * 256);
#pragma unroll
    for (int b = 0; b < kGramBlocks; ++b) {
        const float4 v = *reinterpret_cast<const float4*>(other + b * 256 + lane * 4);
        acc[b][0] += v.x;
        acc[b][1] += v.y;
        acc[b][2] += v.z;
        acc[b][3] += v.w;
    }
    const float* sums = red + 4 * kGramBlocks * 256;
#pragma unroll
    for (int i = 0; i < 8; ++i) csum[i] += sums[(src * 64 + lane) * 8 + i];
}

// After the barrier: the four waves' partials are added; `nt` threads write the 128x128 sum of the chunk
// and its 128 column sums.
__device__ __forceinline__ void gram_reduce_write(const float* red, int tid, int nt, float* __restrict__ G,
                                                  float* __restrict__ sum_out) {
    const float* sums = red + 4 * kGramBlocks * 256;
    // element (R, C) = (8i+ca, 8j+cb) lives in block (ca, cb) at lane j + 16*(i/4), register i%4
    for (int e = tid; e < kD * kD; e += nt) {
        int R = e >> 7, C = e & 127;
        int i = R >> 3, ca = R & 7, j = C >> 3, cb = C & 7;
        if (ca > cb) {                                // mirrored block: swap roles
            int t = ca; ca = cb; cb = t;
            t = i; i = j; j = t;
        }
        const int off = tri_index(ca, cb) * 256 + (j + 16 * (i >> 2)) * 4 + (i & 3);
        G[e] = (red[off] + red[off + kGramBlocks * 256]) + (red[off + 2 * kGramBlocks * 256] + red[off + 3 * kGramBlocks * 256]);
    }
    if (tid < kD) {
        // feature f = 8m + cc: add the 4 token groups g and the 4 waves
        const int mm = tid >> 3, cc = tid & 7;
        float t = 0.f;
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) t += sums[(w4 * 64 + gg * 16 + mm) * 8 + cc];
        sum_out[tid] = t;
    }
}

}  // namespace uncomp
