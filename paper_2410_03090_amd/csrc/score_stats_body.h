// The first scoring pass of one wave as a device function, shared by the scoring kernel and by the
// kernel that runs the Gram pass beside it (Sec. 3.3.3 "Dynamic KV Cache Eviction": softmax statistics
// of the observation-window queries over a chunk of keys).
#pragma once

#include "common.h"
#include "device_utils.h"

namespace uncomp {

constexpr int kTile = 64;                 // tokens per key tile
constexpr int kRowBytes = 2 * kD + 16;    // padded LDS row of one query
constexpr float kLog2e = 1.4426950408889634f;

// qs: the head's query rows staged in LDS (rows of kRowBytes).  The wave (wv = 0..3 of the four that share a
// chunk) streams key tiles wv, wv + 4, ... of tokens [t_begin, t_end) and writes its partial (reference,
// sum) of every query row to stats_rows[row].  No workgroup barrier inside.
template <int NRB>
__device__ __forceinline__ void score_stats_wave_body(const unsigned char* qs, const bf16_bits* __restrict__ Kh,
                                                      int64_t ks_t, int t_begin, int t_end, int P, int w, int R,
                                                      int wv, int lane, float2* __restrict__ stats_rows) {
    const int m = lane & 15, g = lane >> 4;
    const int n_rb = R >> 4;
    const float scale2 = kLog2e * rsqrtf((float)kD);
    const int n_tiles = t_end > t_begin ? (t_end - t_begin + kTile - 1) / kTile : 0;
    float nref[NRB], sum[NRB];         // of row 16*rb + m: minus the running reference, sum of exp2(logit - reference)
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        nref[rb] = INFINITY;
        sum[rb] = 0.f;
    }
    uint4 ka[4][4], kb[4][4];          // [sub-tile][k-step] key operands of two tiles
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
    auto read_block = [&](bf16x8_t a[4], int rb) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            a[ks] = __builtin_bit_cast(
                bf16x8_t, *reinterpret_cast<const uint4*>(qs + (16 * rb + m) * kRowBytes + 64 * ks + 16 * g));
    };
    auto process = [&](const uint4 cur[4][4], uint4 nxt[4][4], int tile) {
        load_tile(nxt, tile + 4);
        const int t0 = t_begin + tile * kTile;
        const bool edge = t0 + kTile > P || t0 + kTile > t_end;   // causal window or ragged end inside
        // query operands are read one block ahead where registers allow (NRB = 8)
        constexpr bool kAhead = NRB <= 8;
        bf16x8_t qa[kAhead ? 2 : 1][4];
        if (kAhead) read_block(qa[0], 0);
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            if (rb < n_rb) {
                if (kAhead) {
                    if (rb + 1 < NRB) read_block(qa[(rb + 1) & (kAhead ? 1 : 0)], min(rb + 1, n_rb - 1));
                } else {
                    read_block(qa[0], rb);
                }
                // acc[st][v] = logit of token t0 + 16 st + 4 g + v against query row 16 rb + m
                f32x4_t acc[4];
#pragma unroll
                for (int st = 0; st < 4; ++st) acc[st] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                __builtin_amdgcn_s_setprio(1);                    // matrix work first: the partner wave fills the gaps
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int st = 0; st < 4; ++st)
                        acc[st] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8_t, cur[st][ks]), qa[kAhead ? (rb & 1) : 0][ks], acc[st], 0, 0, 0);
                __builtin_amdgcn_s_setprio(0);
                // fast path: all 16 logits against the current reference; a sum outside [0, 2^12]
                // (a logit far above the reference, or no reference yet) takes the slow path
                float t = 0.f;
                bool redo = edge;
                if (!edge) {
                    float t4[4];
#pragma unroll
                    for (int st = 0; st < 4; ++st)
                        t4[st] = (__builtin_amdgcn_exp2f(fmaf(acc[st][0], scale2, nref[rb])) +
                                  __builtin_amdgcn_exp2f(fmaf(acc[st][1], scale2, nref[rb]))) +
                                 (__builtin_amdgcn_exp2f(fmaf(acc[st][2], scale2, nref[rb])) +
                                  __builtin_amdgcn_exp2f(fmaf(acc[st][3], scale2, nref[rb])));
                    t = (t4[0] + t4[1]) + (t4[2] + t4[3]);
                    redo = !(t <= 4096.f);
                }
                if (__builtin_amdgcn_ballot_w64(redo) == 0ull) {
                    sum[rb] += t;
                } else {
                    const int last = P + (16 * rb + m) % w;        // last token this row may see
                    float mx = -INFINITY;
#pragma unroll
                    for (int st = 0; st < 4; ++st)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int j = t0 + 16 * st + 4 * g + v;
                            if (j < t_end && j <= last) mx = fmaxf(mx, acc[st][v] * scale2);
                        }
                    const float r = -nref[rb];                     // -inf before the first token
                    if (mx > r) {
                        sum[rb] *= exp2f(r - mx);                  // exp2(-inf) = 0 on first use
                        nref[rb] = -mx;
                    }
#pragma unroll
                    for (int st = 0; st < 4; ++st)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int j = t0 + 16 * st + 4 * g + v;
                            if (j < t_end && j <= last) sum[rb] += exp2f(fmaf(acc[st][v], scale2, nref[rb]));
                        }
                }
            }
        }
    };
    if (n_tiles > 0) {
        load_tile(ka, wv);
        for (int tile = wv; tile < n_tiles; tile += 8) {
            process(ka, kb, tile);
            if (tile + 4 < n_tiles) process(kb, ka, tile + 4);
        }
    }

    // the four lane groups saw different tokens of the same rows: combine, then one lane per row writes
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        if (rb < n_rb) {
            float r = -nref[rb], sm = sum[rb];
#pragma unroll
            for (int o = 16; o < 64; o <<= 1) {
                const float r2 = __shfl_xor(r, o, 64), s2 = __shfl_xor(sm, o, 64);
                const float nr = fmaxf(r, r2);
                const float a = sm > 0.f ? sm * exp2f(r - nr) : 0.f;
                const float bb = s2 > 0.f ? s2 * exp2f(r2 - nr) : 0.f;
                r = nr;
                sm = a + bb;
            }
            if (g == 0)
                stats_rows[16 * rb + m] = make_float2(r, sm);
        }
    }
}

}  // namespace uncomp
