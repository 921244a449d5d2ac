// bf16 MFMA versions of the two tall-skinny products of the wide-matrix entropy (Z = X Q and
// W = X^T Z; see subspace.hip).  X is bf16 as it comes; the fp32 factor (Q, resp. Z) is split into
// a high and a low bf16 half, x = hi + lo with |lo| <= 2^-9 |hi|, and both halves go through the
// matrix cores with fp32 accumulation, which keeps the product at ~2^-17 relative error.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kP = 128;
constexpr int kQtRow = 72;               // LDS row of one column of Q^T: 64 elements + 8 of padding (144 bytes:
                                         // 16 consecutive rows then start in 16 different 16-byte bank groups)

// round-to-nearest-even bf16 of a finite float
__device__ __forceinline__ uint32_t bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

}  // namespace

// out[kc][t][j] = sum over the k chunk of X[t][d] (Qt_hi[j][d] + Qt_lo[j][d]).
// Workgroup: 256 rows of X; wave: 64 rows (four 16-row blocks) x 128 columns.  Per step of 64 d (one whole
// 128-byte line of every row: with half lines a sixth of X came from HBM twice, the other half having left
// the L2 in between) the X rows come straight from global memory in MFMA A-operand layout (lane = row%16,
// 16 bytes per 32 d), one step ahead; the step's slice of Q^T (128 x 64, both halves) is staged in LDS by
// the whole workgroup, double buffered, and read as B operands.  The step loop is unrolled twice so that
// the two register sets of X rows are addressed by constants and no copy waits for a load in flight.
// Workgroups start at different steps of the sum over d and wrap around, which spreads the rows that are
// read at one time over the HBM channels.
// LO: also multiply by the low halves (off in the early rounds of the iteration, whose errors the later rounds remove).
template <int V>
struct phase_t {
    static constexpr int value = V;
};

constexpr int kQStep = 64;                                           // d per step
template <bool LO>
constexpr size_t xq_lds_bytes() {
    return (size_t)2 * (LO ? 2 : 1) * kP * kQtRow * sizeof(bf16_bits);
}

// ZT: the result goes out as what the X^T Z kernel streams, Z^T rounded to bf16 (Zt [128][n_pad] with zeros for
// the tokens from N to n_pad), instead of as fp32 rows: the rounds of the iteration need nothing else of Z,
// which saves writing it as fp32 and reading it back to round it.
template <bool LO, bool ZT>
__global__ __launch_bounds__(256) void sub_xq_mfma_kernel(const bf16_bits* __restrict__ X, int64_t ldx,
                                                          const bf16_bits* __restrict__ Qt_hi,
                                                          const bf16_bits* __restrict__ Qt_lo, int N, int D,
                                                          int k_chunk, float* __restrict__ out,
                                                          bf16_bits* __restrict__ Zt_hi, int64_t n_pad) {
    extern __shared__ __align__(16) bf16_bits qs_raw[];              // [buffer][half][column][kQtRow]
    constexpr int kHalf = kP * kQtRow, kBuf = (LO ? 2 : 1) * kHalf;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = lane & 15, kq = lane >> 4;
    const int row0 = blockIdx.x * 256 + wv * 64;
    const int kc = blockIdx.y;
    const int k_begin = kc * k_chunk, k_end = min(D, k_begin + k_chunk);
    const int n_steps = (k_end - k_begin) / kQStep;
    f32x4_t acc[4][8];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) acc[rb][cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // staging: 128 columns x 8 pieces of 8 d per half: four 16-byte loads per thread and half
    const int s_col0 = tid >> 3, s_piece = tid & 7;                    // columns s_col0 + 32 i
    uint4 sh0, sh1, sh2, sh3, sl0, sl1, sl2, sl3;                    // (named: an array here ends up in scratch)
    uint4 a[2][2][4];                                                // X rows: [set][32-d half of the step][row block]
    // rows past the end re-read the last row (clamped, never predicated); their results are not stored
    // addresses = a base that is uniform over the workgroup + a 32-bit byte offset per lane (the launcher
    // checks that 256 rows of X and all of Q^T span less than 4 GiB)
    const char* xwg = reinterpret_cast<const char*>(X + (int64_t)blockIdx.x * 256 * ldx + k_begin);
    uint32_t xoff[4];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
        xoff[rb] = (uint32_t)(min(row0 + 16 * rb + n, N - 1) - blockIdx.x * 256) * (uint32_t)(ldx * 2) + 16u * kq;
    const char* qwg = reinterpret_cast<const char*>(Qt_hi + k_begin);
    const int64_t lo_bytes = reinterpret_cast<const char*>(Qt_lo) - reinterpret_cast<const char*>(Qt_hi);
    const uint32_t qoff = ((uint32_t)s_col0 * (uint32_t)D + 8u * s_piece) * 2u;
    const int64_t q32 = (int64_t)32 * D * 2;                         // 32 columns on, in bytes
    const int rot = (int)(((int64_t)blockIdx.x * n_steps) / gridDim.x);
    auto at_step = [&](int step) {
        const int k = step + rot;
        return k >= n_steps ? k - n_steps : k;
    };
    auto stage_load = [&](int step_seq) {
        const char* qs = qwg + 2 * kQStep * at_step(step_seq);
        sh0 = *reinterpret_cast<const uint4*>(qs + qoff);
        sh1 = *reinterpret_cast<const uint4*>(qs + q32 + qoff);
        sh2 = *reinterpret_cast<const uint4*>(qs + 2 * q32 + qoff);
        sh3 = *reinterpret_cast<const uint4*>(qs + 3 * q32 + qoff);
        if (LO) {
            sl0 = *reinterpret_cast<const uint4*>(qs + lo_bytes + qoff);
            sl1 = *reinterpret_cast<const uint4*>(qs + lo_bytes + q32 + qoff);
            sl2 = *reinterpret_cast<const uint4*>(qs + lo_bytes + 2 * q32 + qoff);
            sl3 = *reinterpret_cast<const uint4*>(qs + lo_bytes + 3 * q32 + qoff);
        }
    };
    auto stage_store = [&](int buf) {
        bf16_bits* q = qs_raw + buf * kBuf + s_col0 * kQtRow + 8 * s_piece;
        *reinterpret_cast<uint4*>(q) = sh0;
        *reinterpret_cast<uint4*>(q + 32 * kQtRow) = sh1;
        *reinterpret_cast<uint4*>(q + 64 * kQtRow) = sh2;
        *reinterpret_cast<uint4*>(q + 96 * kQtRow) = sh3;
        if (LO) {
            *reinterpret_cast<uint4*>(q + kHalf) = sl0;
            *reinterpret_cast<uint4*>(q + kHalf + 32 * kQtRow) = sl1;
            *reinterpret_cast<uint4*>(q + kHalf + 64 * kQtRow) = sl2;
            *reinterpret_cast<uint4*>(q + kHalf + 96 * kQtRow) = sl3;
        }
    };
    auto load_a = [&](auto set, int step_seq) {
        constexpr int S = decltype(set)::value;
        const char* xs = xwg + 2 * kQStep * at_step(step_seq);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) a[S][h][rb] = *reinterpret_cast<const uint4*>(xs + 64 * h + xoff[rb]);
    };
    auto body = [&](auto ph, int step) {
        constexpr int PH = decltype(ph)::value;
        if (step >= n_steps) return;                                 // uniform over the workgroup
        const bool more = step + 1 < n_steps;
        if (more) {
            stage_load(step + 1);
            load_a(phase_t<PH ^ 1>{}, step + 1);
        }
        const bf16_bits* qb = qs_raw + PH * kBuf + n * kQtRow + 8 * kq;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) {
                const bf16x8_t bh =
                    __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(qb + 16 * cb * kQtRow + 32 * h));
                bf16x8_t bl = bh;
                if (LO)
                    bl = __builtin_bit_cast(bf16x8_t,
                                            *reinterpret_cast<const uint4*>(qb + kHalf + 16 * cb * kQtRow + 32 * h));
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const bf16x8_t av = __builtin_bit_cast(bf16x8_t, a[PH][h][rb]);
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bh, acc[rb][cb], 0, 0, 0);
                    if (LO) acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bl, acc[rb][cb], 0, 0, 0);
                }
            }
        if (more) stage_store(PH ^ 1);           // the other buffer: everyone left it at the last barrier
        __syncthreads();
    };
    if (n_steps > 0) {
        stage_load(0);
        load_a(phase_t<0>{}, 0);
        stage_store(0);
    }
    __syncthreads();
    for (int s0 = 0; s0 < n_steps; s0 += 2) {
        body(phase_t<0>{}, s0);
        body(phase_t<1>{}, s0 + 1);
    }
    // accumulator lane: column 16 cb + n, rows 16 rb + 4 kq + v
    if constexpr (ZT) {
        // Transposed on the way out through the staging buffers, which are free after the loop's last barrier: a
        // wave packs 64 columns x its 64 tokens, rounded to bf16, into its quarter of them (8 bytes = four tokens
        // of a column per lane and accumulator block), then writes them out as 16-byte pieces, eight lanes to a
        // 128-byte run of one row of Zt (stored straight from the registers the same bytes went out as 32-byte
        // runs, 10 us slower per pass).  Tokens from N to n_pad are zeros; n_pad is a multiple of 128.
        bf16_bits* tile = qs_raw + wv * (64 * kQtRow);                // [64 columns][64 tokens + 8 of padding]
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {                             // columns 64 ch .. + 64
#pragma unroll
            for (int cbh = 0; cbh < 4; ++cbh)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const int r = row0 + 16 * rb + 4 * kq;
                    uint32_t w4[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float z = r + v < N ? acc[rb][4 * ch + cbh][v] : 0.f;
                        w4[v] = bf16_rne(z);
                    }
                    *reinterpret_cast<uint2*>(&tile[(16 * cbh + n) * kQtRow + 16 * rb + 4 * kq]) =
                        make_uint2(w4[0] | (w4[1] << 16), w4[2] | (w4[3] << 16));
                }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = lane + 64 * u, col = idx >> 3, piece = idx & 7;
                const uint4 v = *reinterpret_cast<const uint4*>(&tile[col * kQtRow + 8 * piece]);
                const int t = row0 + 8 * piece;
                if (t < n_pad) *reinterpret_cast<uint4*>(Zt_hi + (int64_t)(64 * ch + col) * n_pad + t) = v;
            }
            __syncthreads();                                         // before the tile is packed again
        }
        return;
    }
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


// Zt [128][n_pad] bf16 from Z [N][128] fp32: Z^T rounded to bf16, as the X^T Z kernel streams it (n_pad = N rounded
// up to 128; the tokens past N are written as zeros).  Tile: 64 tokens x 32 columns.  Only for matrices so short
// that the sum over d of Z = X Q is split over workgroups; otherwise the X Q kernel writes Zt itself.
__global__ __launch_bounds__(256) void sub_z_split_kernel(const float* __restrict__ Z, int N, int64_t n_pad,
                                                          bf16_bits* __restrict__ Zt) {
    __shared__ float tile[64][33];
    const int t0 = blockIdx.x * 64, j0 = blockIdx.y * 32;
    const int tid = threadIdx.x;
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
        const int r = (tid >> 3) + 32 * rep, q = tid & 7;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (t0 + r < N) v = *reinterpret_cast<const float4*>(Z + (int64_t)(t0 + r) * kP + j0 + 4 * q);
        tile[r][4 * q] = v.x;
        tile[r][4 * q + 1] = v.y;
        tile[r][4 * q + 2] = v.z;
        tile[r][4 * q + 3] = v.w;
    }
    __syncthreads();
    const int col = tid >> 3, piece = tid & 7;                        // 8 tokens of one column: 16 bytes
    uint32_t h[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = bf16_rne(tile[8 * piece + i][col]);
    *reinterpret_cast<uint4*>(Zt + (int64_t)(j0 + col) * n_pad + t0 + 8 * piece) =
        make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

// out[tc][d][j] = sum over the token chunk of X[t][d] bf16(Z[t][j]) for the 128 features d of
// one slab.  The contraction runs over tokens, the slow index of X, so X is transposed in registers: a
// lane loads 8 tokens x 8 features (16 bytes per token) and byte permutes turn them into 8 operands
// "feature 8 i + c over 8 tokens".  The four waves of a workgroup share one slab of X: per round of 128
// tokens every wave loads and transposes one step of 32 tokens and leaves its 8 operands in LDS (double
// buffered, one barrier per round); then every wave multiplies all four steps with its own 32 columns of
// Z, which arrive transposed (Zt [128][n_pad]: 16 bytes = 8 tokens of one column = one operand), a whole
// round ahead.  Accumulator block (c, b): feature 8 i + c, column 32 w + 16 b + n.
// Workgroups that share a token chunk are placed on one XCD (the hardware deals consecutive workgroup ids
// round-robin over the 8 XCDs), so each L2 fetches only its own chunks of Z.
__global__ __launch_bounds__(256) void sub_xtz_mfma_kernel(const bf16_bits* __restrict__ X, int64_t ldx,
                                                           const bf16_bits* __restrict__ Zh, int64_t n_pad, int N, int D,
                                                           int n_slabs, int t_chunk, float* __restrict__ out) {
    __shared__ __align__(16) uint4 xs[2][4][8][64];                   // [buffer][step][operand][lane]: 64 KB
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    int vid = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) vid = (vid & 7) * (total >> 3) + (vid >> 3);
    const int slab = vid % n_slabs, tc = vid / n_slabs;
    const int t_begin = tc * t_chunk, t_end = min(N, t_begin + t_chunk);
    const int n_rounds = (t_end - t_begin + 127) >> 7;
    const bf16_bits* xbase = X + (int64_t)slab * 128 + 8 * m;
    const bf16_bits* zh_base = Zh + (int64_t)(32 * wv + m) * n_pad + 8 * g;    // column 32 w + n, then + 16 columns
    f32x4_t acc[8][2];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        acc[c][0] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        acc[c][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    uint4 x0, x1, x2, x3, x4, x5, x6, x7;                            // this wave's step of the next round (named: no scratch)
    uint4 zc[4][2], zn[4][2];                                        // Z operands [step][column block]: this round, the next
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
    // t_begin and the rounds are multiples of 128 and n_pad covers whole rounds: every load stays inside Zt
    auto load_z = [&](uint4 (&zd)[4][2], int round) {
        const int64_t t0 = t_begin + 128 * round;
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int b = 0; b < 2; ++b)
                zd[st][b] = *reinterpret_cast<const uint4*>(zh_base + (int64_t)16 * b * n_pad + t0 + 32 * st);
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
    if (n_rounds > 0) {
        load_x(0);
        load_z(zc, 0);
        store_x(0);
    }
    __syncthreads();
    for (int round = 0; round < n_rounds; ++round) {
        const int buf = round & 1;
        const bool more = round + 1 < n_rounds;
        if (more) {
            load_x(round + 1);
            load_z(zn, round + 1);
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const bf16x8_t bh0 = __builtin_bit_cast(bf16x8_t, zc[st][0]), bh1 = __builtin_bit_cast(bf16x8_t, zc[st][1]);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const bf16x8_t av = __builtin_bit_cast(bf16x8_t, xs[buf][st][c][lane]);
                acc[c][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bh0, acc[c][0], 0, 0, 0);
                acc[c][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bh1, acc[c][1], 0, 0, 0);
            }
        }
        if (more) {
            store_x(buf ^ 1);
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int b = 0; b < 2; ++b) zc[st][b] = zn[st][b];
        }
        __syncthreads();
    }
    // accumulator lane: column index n = lane % 16, rows i = 4 (lane / 16) + v
    float* o = out + ((int64_t)tc * D + (int64_t)slab * 128) * kP + 32 * wv + m;
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int feat = 8 * (4 * g + v) + c;
            o[(int64_t)feat * kP] = acc[c][0][v];
            o[(int64_t)feat * kP + 16] = acc[c][1][v];
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

// Z = X Q, given Q^T as two bf16 halves [128][D] (left by the orthonormalisation); precise: multiply by both.
// want_zt: the caller only needs Z as the operand of launch_xtz_mfma; when the sum over d is not split the kernel
// then writes Zt itself and *zt_written tells launch_xtz_mfma to skip its own rounding pass.
hipError_t launch_xq_mfma(const bf16_bits* X, int64_t ldx, int N, int D, const bf16_bits* Qt_hi, const bf16_bits* Qt_lo,
                          int n_split, float* Zpart, float* Z, hipStream_t s, bool precise, bool want_zt, bf16_bits* Zt,
                          bool* zt_written) {
    const int k_chunk = ((D + n_split - 1) / n_split + kQStep - 1) / kQStep * kQStep;
    const int splits = (D + k_chunk - 1) / k_chunk;
    float* dst = splits == 1 ? Z : Zpart;
    const dim3 grid((unsigned)((N + 255) / 256), (unsigned)splits);
    const int64_t n_pad = ((int64_t)N + 127) / 128 * 128;
    const bool zt = want_zt && splits == 1;
    if (zt_written != nullptr) *zt_written = zt;
    if (zt && precise)
        sub_xq_mfma_kernel<true, true><<<grid, dim3(256), xq_lds_bytes<true>(), s>>>(X, ldx, Qt_hi, Qt_lo, N, D, k_chunk, dst, Zt, n_pad);
    else if (zt)
        sub_xq_mfma_kernel<false, true><<<grid, dim3(256), xq_lds_bytes<false>(), s>>>(X, ldx, Qt_hi, Qt_lo, N, D, k_chunk, dst, Zt, n_pad);
    else if (precise)
        sub_xq_mfma_kernel<true, false><<<grid, dim3(256), xq_lds_bytes<true>(), s>>>(X, ldx, Qt_hi, Qt_lo, N, D, k_chunk, dst, Zt, n_pad);
    else
        sub_xq_mfma_kernel<false, false><<<grid, dim3(256), xq_lds_bytes<false>(), s>>>(X, ldx, Qt_hi, Qt_lo, N, D, k_chunk, dst, Zt, n_pad);
    if (splits > 1) {
        const int64_t total = (int64_t)N * kP;
        sub_sum_parts_kernel<<<dim3((unsigned)((total / 4 + 255) / 256)), dim3(256), 0, s>>>(Zpart, splits, total, Z);
    }
    return hipGetLastError();
}

// Wpart[tc][D][128] = partial X^T bf16(Z) over token chunks (t_chunk a multiple of 128); Zt: Z^T rounded to bf16,
// [128][n_pad] with n_pad = N rounded up to 128, made here from Z unless zt_ready.
hipError_t launch_xtz_mfma(const bf16_bits* X, int64_t ldx, const float* Z, int N, int D, bf16_bits* Zt, int t_chunk,
                           int n_tchunks, float* Wpart, hipStream_t s, bool zt_ready) {
    const int64_t n_pad = ((int64_t)N + 127) / 128 * 128;
    const int n_slabs = D / 128;
    if (!zt_ready) sub_z_split_kernel<<<dim3((unsigned)(n_pad / 64), kP / 32), dim3(256), 0, s>>>(Z, N, n_pad, Zt);
    sub_xtz_mfma_kernel<<<dim3((unsigned)(n_slabs * n_tchunks)), dim3(256), 0, s>>>(X, ldx, Zt, n_pad, N, D, n_slabs, t_chunk, Wpart);
    return hipGetLastError();
}

hipError_t init_subspace_mfma_kernels() {
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(sub_xq_mfma_kernel<true, false>), xq_lds_bytes<true>());
    if (e != hipSuccess) return e;
    return allow_dynamic_lds(reinterpret_cast<const void*>(sub_xq_mfma_kernel<true, true>), xq_lds_bytes<true>());
}

}  // namespace uncomp
