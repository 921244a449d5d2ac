// Gram / covariance stage of the truncated matrix entropy (Sec. 3.1 Eq. 1): for every
// token matrix X (N tokens x 128 features) the second-moment sums S = sum_t x_t x_t^T and
// s = sum_t x_t, split over token chunks.  Each workgroup folds one chunk of one matrix in
// fp32 and writes its partial 128x128 block and 128 column sums; the eigen stage adds the
// partials in fp64 and applies the mean correction there.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

// ---------------------------------------------------------------------------------------
// Plain-ALU kernel (any storage type).  256 threads as a 16x16 grid, each owning an 8x8
// block of the 128x128 output; tokens are staged through LDS 32 at a time.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gram_alu_kernel(const T* __restrict__ X, int N,
                                                       int64_t mat_stride, int64_t ldx,
                                                       int n_chunks, int chunk,
                                                       float* __restrict__ gram_part,
                                                       float* __restrict__ sum_part) {
    constexpr int TT = 32;
    __shared__ float tile[TT][kD];
    const int c = blockIdx.x % n_chunks, m = blockIdx.x / n_chunks;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const T* Xm = X + (int64_t)m * mat_stride;
    const int t_begin = c * chunk;
    const int t_end = min(N, t_begin + chunk);

    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    float colsum = 0.f;

    for (int t0 = t_begin; t0 < t_end; t0 += TT) {
        // 32 tokens x 128 features = 512 groups of 8 elements, two per thread
#pragma unroll
        for (int rep = 0; rep < 2; ++rep) {
            int g = tid + rep * 256;
            int tt = g >> 4, f8 = (g & 15) * 8;
            float v[8];
            if (t0 + tt < t_end) {
                load8(Xm + (int64_t)(t0 + tt) * ldx + f8, v);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) tile[tt][f8 + i] = v[i];
        }
        __syncthreads();
        if (tid < kD) {
#pragma unroll 8
            for (int tt = 0; tt < TT; ++tt) colsum += tile[tt][tid];
        }
#pragma unroll 4
        for (int tt = 0; tt < TT; ++tt) {
            float a[8], b[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) a[i] = tile[tt][ty * 8 + i];
#pragma unroll
            for (int j = 0; j < 8; ++j) b[j] = tile[tt][tx * 8 + j];
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    float* G = gram_part + ((int64_t)m * n_chunks + c) * (kD * kD);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float4* dst = reinterpret_cast<float4*>(G + (ty * 8 + i) * kD + tx * 8);
        dst[0] = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
        dst[1] = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
    }
    if (tid < kD) sum_part[((int64_t)m * n_chunks + c) * kD + tid] = colsum;
}

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
// The four waves of a workgroup take 32-token steps round-robin with three steps of loads
// in flight each, and combine their accumulators through LDS at the end of the chunk.
// ---------------------------------------------------------------------------------------
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kGramBlocks = 36;                     // upper-triangular 16x16-output blocks
constexpr int kGramStages = 3;

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

}  // namespace

__global__ __launch_bounds__(256) void gram_mfma_kernel(const bf16_bits* __restrict__ X, int N,
                                                        int64_t mat_stride, int64_t ldx, int n_chunks,
                                                        int chunk, float* __restrict__ gram_part,
                                                        float* __restrict__ sum_part) {
    extern __shared__ __align__(16) float red[];     // [4 waves][36 blocks][64 lanes][4] + sums [4][64][8]
    const int c = blockIdx.x % n_chunks, m_idx = blockIdx.x / n_chunks;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int t_begin = c * chunk;
    const int t_end = min(N, t_begin + chunk);
    const int n_steps = (t_end - t_begin + 31) / 32;
    const bf16_bits* base = X + (int64_t)m_idx * mat_stride + 8 * m;

    f32x4_t acc[kGramBlocks];
#pragma unroll
    for (int b = 0; b < kGramBlocks; ++b) acc[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float csum[8];
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

    // this wave's steps: wv, wv+4, ...; three in flight
#pragma unroll
    for (int st = 0; st < kGramStages; ++st) load_step(buf[st], wv + 4 * st);
    for (int s0 = wv; s0 < n_steps; s0 += 4 * kGramStages) {
#pragma unroll
        for (int st = 0; st < kGramStages; ++st) {
            compute_step(buf[st]);
            load_step(buf[st], s0 + 4 * (st + kGramStages));
        }
    }

    // ---- combine the four waves --------------------------------------------------------
    float* my = red + (size_t)wv * (kGramBlocks * 256);
#pragma unroll
    for (int b = 0; b < kGramBlocks; ++b)
        *reinterpret_cast<float4*>(my + b * 256 + lane * 4) = make_float4(acc[b][0], acc[b][1], acc[b][2], acc[b][3]);
    float* sums = red + 4 * kGramBlocks * 256;       // [4][64][8]
#pragma unroll
    for (int i = 0; i < 8; ++i) sums[(wv * 64 + lane) * 8 + i] = csum[i];
    __syncthreads();

    // element (R, C) = (8i+ca, 8j+cb) lives in block (ca, cb) at lane j + 16*(i/4), register i%4
    float* G = gram_part + ((int64_t)m_idx * n_chunks + c) * (kD * kD);
    for (int e = tid; e < kD * kD; e += 256) {
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
        sum_part[((int64_t)m_idx * n_chunks + c) * kD + tid] = t;
    }
}

EntropyPlan plan_entropy(int n_mat, int N) {
    EntropyPlan p;
    // Enough workgroups to cover the chip a few times over, but chunks of at least 4096
    // tokens so that the 64 KiB partial a chunk writes stays small next to what it reads.
    int max_chunks = N / 4096 > 0 ? N / 4096 : 1;
    int want = (2048 + n_mat - 1) / (n_mat > 0 ? n_mat : 1);
    int nc = want < 1 ? 1 : want;
    if (nc > max_chunks) nc = max_chunks;
    int chunk = (N + nc - 1) / nc;
    chunk = (chunk + kGramTile - 1) / kGramTile * kGramTile;
    nc = (N + chunk - 1) / chunk;
    if (nc < 1) nc = 1;
    p.n_chunks = nc;
    p.chunk = chunk;
    p.gram_off = 0;
    p.sum_off = align_up((size_t)n_mat * nc * kD * kD * sizeof(float), 256);
    p.bytes = p.sum_off + align_up((size_t)n_mat * nc * kD * sizeof(float), 256);
    return p;
}

hipError_t launch_gram(const void* X, uncomp_dtype dt, int n_mat, int N, int64_t mat_stride,
                       int64_t ldx, const EntropyPlan& p, char* ws, const Env& env) {
    hipStream_t s = env.s;
    const bool force_alu = env.force_alu;
    float* gram = reinterpret_cast<float*>(ws + p.gram_off);
    float* sums = reinterpret_cast<float*>(ws + p.sum_off);
    dim3 grid((unsigned)(p.n_chunks * n_mat)), block(256);
    if (dt == UNCOMP_BF16 && !force_alu) {
        constexpr size_t lds = (4 * kGramBlocks * 256 + 4 * 64 * 8) * sizeof(float);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gram_mfma_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        env.begin("gram_mfma");
        gram_mfma_kernel<<<grid, block, lds, s>>>(static_cast<const bf16_bits*>(X), N, mat_stride, ldx,
                                                  p.n_chunks, p.chunk, gram, sums);
        env.end();
        return hipGetLastError();
    }
    env.begin("gram_alu");
    if (dt == UNCOMP_BF16) {
        gram_alu_kernel<bf16_bits><<<grid, block, 0, s>>>(
            static_cast<const bf16_bits*>(X), N, mat_stride, ldx, p.n_chunks, p.chunk, gram, sums);
    } else {
        gram_alu_kernel<float><<<grid, block, 0, s>>>(
            static_cast<const float*>(X), N, mat_stride, ldx, p.n_chunks, p.chunk, gram, sums);
    }
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
