// Gram / covariance stage of the truncated matrix entropy (Sec. 3.1 Eq. 1): for every
// token matrix X (N tokens x 128 features) the second-moment sums S = sum_t x_t x_t^T and
// s = sum_t x_t, split over token chunks.  Each workgroup folds one chunk of one matrix in
// fp32 and writes its partial 128x128 block and 128 column sums; the eigen stage adds the
// partials in fp64 and applies the mean correction there.
#include "common.h"
#include "device_utils.h"
#include "gram_body.h"

namespace uncomp {

// ---------------------------------------------------------------------------------------
// Plain-ALU kernel (any storage type).  256 threads as a 16x16 grid, each owning an 8x8
// block of the 128x128 output; tokens are staged through LDS 32 at a time.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gram_alu_kernel(const T* __restrict__ X, int N, int D,
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
            if (t0 + tt < t_end && f8 < D) {                 // features beyond D (a 64-wide head) count as zeros
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

// The bf16 MFMA kernel (body in gram_body.h).  Eight waves per workgroup, two per SIMD: one wave's loads and
// byte permutes run under the other's MFMAs (with four waves, one per SIMD, the cache-resident rate was 43 %
// of the MFMA peak instead of 56 %, the streamed rate 5.5 instead of 5.6 TB/s).  One 32-token step of loads
// in flight per wave is what 256 registers leave room for.  Waves 4-7 hand their sums to waves 0-3 through
// LDS, then the four partials are added and written.
__global__ __launch_bounds__(512, 1) void gram_mfma_kernel(const bf16_bits* __restrict__ X, int N, int64_t mat_stride,
                                                            int64_t ldx, int n_chunks, int chunk,
                                                            float* __restrict__ gram_part, float* __restrict__ sum_part) {
    extern __shared__ __align__(16) float red[];
    const int c = blockIdx.x % n_chunks, m_idx = blockIdx.x / n_chunks;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int t_begin = c * chunk;
    const int t_end = min(N, t_begin + chunk);
    f32x4_t acc[kGramBlocks];
    float csum[8];
    gram_wave_accumulate<1, 8>(X + (int64_t)m_idx * mat_stride + 8 * m, ldx, t_begin, t_end, wv, g, acc, csum);
    if (wv >= 4) gram_wave_to_lds(red, wv - 4, lane, acc, csum);
    __syncthreads();
    if (wv < 4) gram_wave_add_from_lds(red, wv, lane, acc, csum);
    __syncthreads();
    if (wv < 4) gram_wave_to_lds(red, wv, lane, acc, csum);
    __syncthreads();
    gram_reduce_write(red, tid, 512, gram_part + ((int64_t)m_idx * n_chunks + c) * (kD * kD),
                      sum_part + ((int64_t)m_idx * n_chunks + c) * kD);
}

EntropyPlan plan_entropy(int n_mat, int N, size_t max_bytes) {
    EntropyPlan p;
    // Two workgroups of eight waves per CU cover the chip; fewer, longer chunks mean fewer 64 KiB
    // partials to write and to add up again (128K workload: 8 chunks per matrix 1.54 ms, 2 chunks
    // 1.46 ms), and chunks stay above 4096 tokens.  A byte limit (max_bytes > 0) lowers the chunk
    // count until the partials fit; p.bytes still exceeds it if even one chunk per matrix does not.
    int max_chunks = N / 4096 > 0 ? N / 4096 : 1;
    int want = (512 + n_mat - 1) / (n_mat > 0 ? n_mat : 1);
    int nc = want < 1 ? 1 : want;
    if (nc > max_chunks) nc = max_chunks;
    for (;;) {
        int chunk = (N + nc - 1) / nc;
        chunk = (chunk + kGramTile - 1) / kGramTile * kGramTile;
        int n = (N + chunk - 1) / chunk;
        if (n < 1) n = 1;
        p.n_chunks = n;
        p.chunk = chunk;
        p.gram_off = 0;
        p.sum_off = align_up((size_t)n_mat * n * kD * kD * sizeof(float), 256);
        p.bytes = p.sum_off + align_up((size_t)n_mat * n * kD * sizeof(float), 256);
        if (max_bytes == 0 || p.bytes <= max_bytes || nc <= 1) break;
        nc = n > 1 ? n - 1 : 1;
    }
    return p;
}

hipError_t launch_gram(const void* X, uncomp_dtype dt, int n_mat, int N, int64_t mat_stride,
                       int64_t ldx, const EntropyPlan& p, char* ws, const Env& env, int D) {
    hipStream_t s = env.s;
    const bool force_alu = env.force_alu || D != kD;       // the MFMA kernel is written for 128 features
    float* gram = reinterpret_cast<float*>(ws + p.gram_off);
    float* sums = reinterpret_cast<float*>(ws + p.sum_off);
    dim3 grid((unsigned)(p.n_chunks * n_mat)), block(256);
    if (dt == UNCOMP_BF16 && !force_alu) {
        constexpr size_t lds = kGramLdsBytes;
        env.begin("gram_mfma");
        gram_mfma_kernel<<<grid, dim3(512), lds, s>>>(static_cast<const bf16_bits*>(X), N, mat_stride, ldx,
                                                      p.n_chunks, p.chunk, gram, sums);
        env.end();
        return hipGetLastError();
    }
    if (dt == UNCOMP_F32 && !force_alu && n_mat <= 65535) {
        // fp32 matrices with 128 features: exact products and fp64 sums on the fp64 matrix cores
        env.begin("gram_f64");
        hipError_t e = launch_gram_f32_mfma(static_cast<const float*>(X), n_mat, N, mat_stride, ldx, p.n_chunks, p.chunk, gram,
                                            sums, s);
        env.end();
        return e;
    }
    env.begin("gram_alu");
    if (dt == UNCOMP_BF16) {
        gram_alu_kernel<bf16_bits><<<grid, block, 0, s>>>(
            static_cast<const bf16_bits*>(X), N, D, mat_stride, ldx, p.n_chunks, p.chunk, gram, sums);
    } else {
        gram_alu_kernel<float><<<grid, block, 0, s>>>(
            static_cast<const float*>(X), N, D, mat_stride, ldx, p.n_chunks, p.chunk, gram, sums);
    }
    env.end();
    return hipGetLastError();
}

hipError_t init_gram_kernels() {
    return allow_dynamic_lds(reinterpret_cast<const void*>(gram_mfma_kernel), kGramLdsBytes);
}

}  // namespace uncomp
