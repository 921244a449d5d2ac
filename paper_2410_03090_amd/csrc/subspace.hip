// Truncated matrix entropy of wide token matrices (Sec. 3.1 Eq. 1, Lemma 2; Sec. 3.2 Eq. 5-6 for
// D = 256 ... 8192, e.g. the hidden states H_m of Sec. 3.3.2) without ever forming the D x D
// covariance: only its k largest eigenvalues enter Eq. 5, and those are the Ritz values of a
// 128-dimensional subspace that block power iteration drives onto the dominant eigenvectors.
//
//   x_bar = mean token, C = sum_t (x_t - x_bar)(x_t - x_bar)^T            (never stored)
//   Q_0   = fixed pseudo-random D x 128 block, orthonormalised
//   repeat:  Z = X Q  (N x 128),  W = C Q = X^T Z - s (s^T Q)/N  (D x 128),  Q = orth(W)
//   end:     Z = X Q;  the centred covariance of the N projected tokens z_t is Q^T C Q, whose
//            eigenvalues (the ordinary 128-wide entropy path) are the Ritz values; Eq. 5 without
//            renormalisation divides them by trace(C), which one pass over X provides.
//
// Every iteration reads X twice (HBM-bound: 2 N D e bytes) and costs 4 N D 128 flops; forming C
// would cost 2 N D^2.  orth() is a Cholesky QR with the 128 x 128 Gram of W accumulated in fp64;
// a pivot that vanishes (rank below 128) retires its column.  Convergence of the k-th value goes
// with (lambda_129 / lambda_k)^(2 iterations): fast when the spectrum falls off before the 129th
// eigenvalue, as it does for the matrices the method looks at (that fall-off is the paper's point).
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kP = 128;                  // width of the iterated block

__device__ __forceinline__ float elem(const bf16_bits* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ float elem(const float* p) { return *p; }

// splitmix-style hash -> value in [-1, 1): the start block must be the same on every run
__device__ __forceinline__ float start_value(uint32_t d, uint32_t j) {
    uint64_t z = ((uint64_t)d << 32 | j) + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (float)((double)(z >> 11) * (2.0 / 9007199254740992.0) - 1.0);
}

}  // namespace

__global__ __launch_bounds__(256) void sub_start_kernel(float* __restrict__ W, int D) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e < D * kP) W[e] = start_value((uint32_t)(e / kP), (uint32_t)(e % kP));
}

// Column sums and sums of squares of X over a chunk of tokens, in fp64: part[chunk][2][D].
// A workgroup covers 512 columns: thread = 8 consecutive columns (read with load8) x one of four row phases,
// eight rows in flight per thread; the four phases are added up in LDS in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void sub_colstats_kernel(const T* __restrict__ X, int N, int D, int64_t ldx,
                                                           int chunk, double* __restrict__ part) {
    __shared__ double red[3][16][64];
    const int cg = threadIdx.x & 63, ph = threadIdx.x >> 6;
    const int d = (blockIdx.x * 64 + cg) * 8;
    const int c = blockIdx.y;
    const bool live = d < D;
    const int t0 = c * chunk, t1 = min(N, t0 + chunk);
    double s[8], q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = q[i] = 0.0;
    if (live) {
        for (int t = t0 + ph; t < t1; t += 32) {
            float v[8][8];
#pragma unroll
            for (int u = 0; u < 8; ++u) load8(X + (int64_t)min(t + 4 * u, t1 - 1) * ldx + d, v[u]);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (t + 4 * u < t1) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const double x = (double)v[u][i];
                        s[i] += x;
                        q[i] = fma(x, x, q[i]);
                    }
                }
            }
        }
    }
    if (ph > 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            red[ph - 1][i][cg] = s[i];
            red[ph - 1][8 + i][cg] = q[i];
        }
    }
    __syncthreads();
    if (ph == 0 && live) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            part[((int64_t)c * 2 + 0) * D + d + i] = ((s[i] + red[0][i][cg]) + red[1][i][cg]) + red[2][i][cg];
            part[((int64_t)c * 2 + 1) * D + d + i] = ((q[i] + red[0][8 + i][cg]) + red[1][8 + i][cg]) + red[2][8 + i][cg];
        }
    }
}

// s[d] = sum over chunks; tpart[wg] = this workgroup's share of (sum_d (q_d - s_d^2 / N), sum_d q_d).
__global__ __launch_bounds__(256) void sub_colstats_finish_kernel(const double* __restrict__ part, int n_chunks, int D,
                                                                  int N, double* __restrict__ s,
                                                                  double* __restrict__ tpart) {
    __shared__ double red[2][4];
    const int d = blockIdx.x * 256 + threadIdx.x;
    double tc = 0.0, tu = 0.0;
    if (d < D) {
        double a = 0.0, q = 0.0;
#pragma unroll 8
        for (int c = 0; c < n_chunks; ++c) {
            a += part[((int64_t)c * 2 + 0) * D + d];
            q += part[((int64_t)c * 2 + 1) * D + d];
        }
        s[d] = a;
        tc = q - a * a / (double)N;
        tu = q;
    }
    tc = wave_sum(tc);
    tu = wave_sum(tu);
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = tc;
        red[1][threadIdx.x >> 6] = tu;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        tpart[2 * blockIdx.x + 0] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        tpart[2 * blockIdx.x + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}
// trace[0] = centred, trace[1] = uncentred trace: the workgroups' shares added in order.
__global__ void sub_trace_kernel(const double* __restrict__ tpart, int n, double* __restrict__ trace) {
    if (threadIdx.x < 2) {
        double t = 0.0;
        for (int i = 0; i < n; ++i) t += tpart[2 * i + threadIdx.x];
        trace[threadIdx.x] = t;
    }
}

// Tall-skinny product with 128 output columns, fp32 accumulation on the plain ALUs.
//   A_KM == false:  out[m][j] = sum_k A[m][k] B[k][j]      (A is M x K, row stride lda)       Z = X Q
//   A_KM == true :  out[m][j] = sum_k A[k][m] B[k][j]      (A is K x M, row stride lda)       W = X^T Z
// blockIdx.x: 64 rows of the output, blockIdx.y: a chunk of k (partial results out[chunk][M][128]).
// B is fp32, K x 128, row stride 128.  A workgroup stages 16 k at a time in LDS; a thread owns
// 4 rows x 8 columns.
template <typename T, bool A_KM>
__global__ __launch_bounds__(256) void sub_gemm_kernel(const T* __restrict__ A, int64_t lda, const float* __restrict__ B,
                                                       int M, int K, int k_chunk, float* __restrict__ out) {
    __shared__ float As[16][64 + 4];
    __shared__ __align__(16) float Bs[16][kP];
    const int m0 = blockIdx.x * 64;
    const int kc = blockIdx.y;
    const int k_begin = kc * k_chunk, k_end = min(K, k_begin + k_chunk);
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    float acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    for (int k0 = k_begin; k0 < k_end; k0 += 16) {
        // stage A: 64 rows x 16 k (four elements per thread)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            int m, k;
            if (A_KM) {
                m = idx & 63;
                k = idx >> 6;
            } else {
                k = idx & 15;
                m = idx >> 4;
            }
            float v = 0.f;
            if (m0 + m < M && k0 + k < k_end)
                v = A_KM ? elem(A + (int64_t)(k0 + k) * lda + m0 + m) : elem(A + (int64_t)(m0 + m) * lda + k0 + k);
            As[k][m] = v;
        }
        // stage B: 16 k x 128 (eight floats per thread)
        {
            const int k = tid >> 4, j = (tid & 15) * 8;
            float4 b0 = make_float4(0.f, 0.f, 0.f, 0.f), b1 = b0;
            if (k0 + k < k_end) {
                b0 = *reinterpret_cast<const float4*>(B + (int64_t)(k0 + k) * kP + j);
                b1 = *reinterpret_cast<const float4*>(B + (int64_t)(k0 + k) * kP + j + 4);
            }
            *reinterpret_cast<float4*>(&Bs[k][j]) = b0;
            *reinterpret_cast<float4*>(&Bs[k][j + 4]) = b1;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][4 * ty + i];
            const float4 b0 = *reinterpret_cast<const float4*>(&Bs[k][8 * tx]);
            const float4 b1 = *reinterpret_cast<const float4*>(&Bs[k][8 * tx + 4]);
            const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    float* o = out + (int64_t)kc * M * kP;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + 4 * ty + i;
        if (m < M) {
            *reinterpret_cast<float4*>(o + (int64_t)m * kP + 8 * tx) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
            *reinterpret_cast<float4*>(o + (int64_t)m * kP + 8 * tx + 4) = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
        }
    }
}

// Q = W Rinv for 32 rows of W per workgroup (fp32 ALUs, a thread owns 2 rows x 8 columns, Rinv staged 16 rows
// at a time), together with what the next round needs of Q besides: its transposed bf16 halves Qt_hi / Qt_lo
// [128][D] (the operand that the MFMA version of Z = X Q streams; skipped when Qt_hi is null) and, when centring
// (s not null), this row block's share of s^T Q in fp64: zpart[block][128].  D is a multiple of 128.
constexpr int kQRows = 32;
__global__ __launch_bounds__(256) void sub_q_kernel(const float* __restrict__ W, const float* __restrict__ Rinv, int D,
                                                    const double* __restrict__ s, float* __restrict__ Q,
                                                    uint16_t* __restrict__ Qt_hi, uint16_t* __restrict__ Qt_lo,
                                                    double* __restrict__ zpart) {
    __shared__ __align__(16) float Ws[kQRows][kP + 4];
    __shared__ __align__(16) float Rs[16][kP];
    __shared__ float Qs[kQRows][kP + 1];
    const int d0 = blockIdx.x * kQRows;
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int idx = tid + 256 * e, r = idx >> 5, q = idx & 31;
        *reinterpret_cast<float4*>(&Ws[r][4 * q]) = *reinterpret_cast<const float4*>(W + (int64_t)(d0 + r) * kP + 4 * q);
    }
    float acc[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < kP; k0 += 16) {
        __syncthreads();                                             // Ws written / the previous 16 rows of Rinv read
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int idx = tid + 256 * e, k = idx >> 5, q = idx & 31;
            *reinterpret_cast<float4*>(&Rs[k][4 * q]) = *reinterpret_cast<const float4*>(Rinv + (int64_t)(k0 + k) * kP + 4 * q);
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const float a0 = Ws[2 * ty][k0 + k], a1 = Ws[2 * ty + 1][k0 + k];
            const float4 b0 = *reinterpret_cast<const float4*>(&Rs[k][8 * tx]);
            const float4 b1 = *reinterpret_cast<const float4*>(&Rs[k][8 * tx + 4]);
            const float bv[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                acc[0][j] = fmaf(a0, bv[j], acc[0][j]);
                acc[1][j] = fmaf(a1, bv[j], acc[1][j]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        float* o = Q + (int64_t)(d0 + 2 * ty + i) * kP + 8 * tx;
        *reinterpret_cast<float4*>(o) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
        *reinterpret_cast<float4*>(o + 4) = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
#pragma unroll
        for (int j = 0; j < 8; ++j) Qs[2 * ty + i][8 * tx + j] = acc[i][j];
    }
    __syncthreads();
    if (Qt_hi != nullptr) {
        // thread = (column, half of the 32 rows): 16 consecutive d of one column = 32 bytes per bf16 half
        const int col = tid >> 1, r0 = 16 * (tid & 1);
        uint32_t h[8], l[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v0 = Qs[r0 + 2 * e][col], v1 = Qs[r0 + 2 * e + 1][col];
            const uint32_t h0 = __float_as_uint(v0), h1 = __float_as_uint(v1);
            const uint32_t hi0 = (h0 + 0x7fffu + ((h0 >> 16) & 1u)) >> 16, hi1 = (h1 + 0x7fffu + ((h1 >> 16) & 1u)) >> 16;   // round to nearest even
            const uint32_t g0 = __float_as_uint(v0 - __uint_as_float(hi0 << 16)), g1 = __float_as_uint(v1 - __uint_as_float(hi1 << 16));
            const uint32_t lo0 = (g0 + 0x7fffu + ((g0 >> 16) & 1u)) >> 16, lo1 = (g1 + 0x7fffu + ((g1 >> 16) & 1u)) >> 16;
            h[e] = hi0 | (hi1 << 16);
            l[e] = lo0 | (lo1 << 16);
        }
        uint4* ph = reinterpret_cast<uint4*>(Qt_hi + (int64_t)col * D + d0 + r0);
        uint4* pl = reinterpret_cast<uint4*>(Qt_lo + (int64_t)col * D + d0 + r0);
        ph[0] = make_uint4(h[0], h[1], h[2], h[3]);
        ph[1] = make_uint4(h[4], h[5], h[6], h[7]);
        pl[0] = make_uint4(l[0], l[1], l[2], l[3]);
        pl[1] = make_uint4(l[4], l[5], l[6], l[7]);
    }
    if (s != nullptr && tid < kP) {
        double t = 0.0;
#pragma unroll 8
        for (int r = 0; r < kQRows; ++r) t += s[d0 + r] * (double)Qs[r][tid];
        zpart[(int64_t)blockIdx.x * kP + tid] = t;
    }
}

// zsum[j] = sum_d s[d] Q[d][j] (= column sums of Z = X Q): the row blocks' shares added in a fixed order
// (eight interleaved partial sums side by side, then those in order).
__global__ __launch_bounds__(1024) void sub_zsum_kernel(const double* __restrict__ zpart, int n_parts, double* __restrict__ zsum) {
    __shared__ double part[8][kP];
    const int j = threadIdx.x & (kP - 1), q = threadIdx.x >> 7;
    double t = 0.0;
    for (int b = q; b < n_parts; b += 8) t += zpart[(int64_t)b * kP + j];
    part[q][j] = t;
    __syncthreads();
    if (q == 0) {
#pragma unroll
        for (int x = 1; x < 8; ++x) t += part[x][j];
        zsum[j] = t;
    }
}

// W[d][j] = sum over chunks of part[c][d][j] - s[d] zsum[j] / N   (the mean correction of C Q)
__global__ __launch_bounds__(256) void sub_reduce_kernel(const float* __restrict__ part, int n_chunks, int D,
                                                         const double* __restrict__ s, const double* __restrict__ zsum,
                                                         double inv_n, float* __restrict__ W) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)D * kP) return;
    double a = 0.0;
    for (int c = 0; c < n_chunks; ++c) a += (double)part[(int64_t)c * D * kP + e];
    if (s != nullptr) a -= s[e / kP] * zsum[e % kP] * inv_n;
    W[e] = (float)a;
}

// Partial Gram of a tall fp32 matrix A (n_rows x 128) in fp64: gpart[slice][128][128] (+ the column sums of
// the slice in spart[slice][128] when asked for) on v_mfma_f64_16x16x4_f64.  Operands: lane l holds row /
// column l%16 at contraction index l/16; result register v of lane l: row 4v + l/16, column l%16.  The rows
// are staged in LDS 64 at a time as fp32 (next tile's loads in flight during the products) and widened on
// the way into the operands (exact).  Only the 36 tiles on and above the diagonal are computed, nine per
// wave (tile rows w and 7 - w); the write-out mirrors them.
constexpr int kGramRows = 64;
constexpr int kGramLd = 144;             // floats per staged row: four consecutive rows start 16 banks apart
constexpr int kGramTiles = 36;           // 16 x 16 tiles on and above the diagonal

typedef double f64x4_t __attribute__((ext_vector_type(4)));

// PACKED (the Gram of the projected tokens, whose partials only feed an fp32 result): the 36 computed tiles go
// out as fp32, tile after tile (fpart[slice][36][16][16], tiles in the order (0,0) (0,1) ... (0,7) (1,1) ...),
// a quarter of the bytes of the mirrored fp64 matrix that the Cholesky step needs.
// MODE 2 (fp32 token matrices of uncomp_head_entropy, 128 features): blockIdx.y is the matrix (mat_stride elements
// apart, rows lda apart), blockIdx.x its token chunk; the chunk's mirrored Gram and column sums go out as fp32 in
// the layout the eigenvalue kernels add up: fpart[(matrix, chunk)][128][128], fsum[(matrix, chunk)][128].
template <int MODE>
__global__ __launch_bounds__(256) void sub_gram64_kernel(const float* __restrict__ A_all, int64_t mat_stride, int64_t lda,
                                                         int n_rows, int rows_per_wg, double* __restrict__ gpart,
                                                         float* __restrict__ fpart, double* __restrict__ spart,
                                                         float* __restrict__ fsum) {
    constexpr bool PACKED = MODE == 1;
    __shared__ __align__(16) float rows[kGramRows][kGramLd];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int c = lane & 15, kk = lane >> 4;
    const float* A = A_all + (int64_t)blockIdx.y * mat_stride;
    const int64_t out_idx = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const int r_begin = blockIdx.x * rows_per_wg;
    const int r_end = min(n_rows, r_begin + rows_per_wg);
    const int I1 = wv, I2 = 7 - wv, n1 = 8 - wv;             // slot s < n1: tile (I1, I1 + s); else (I2, I2 + s - n1)
    f64x4_t acc[9];
#pragma unroll
    for (int sl = 0; sl < 9; ++sl) acc[sl] = f64x4_t{0.0, 0.0, 0.0, 0.0};
    double csum = 0.0;
    float4 pre[8];
    auto fetch = [&](int r0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int e = tid + 256 * i, rr = e >> 5, q = e & 31;
            pre[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r0 + rr < r_end) pre[i] = *reinterpret_cast<const float4*>(A + (int64_t)(r0 + rr) * lda + 4 * q);
        }
    };
    if (r_begin < r_end) fetch(r_begin);
    for (int r0 = r_begin; r0 < r_end; r0 += kGramRows) {
        __syncthreads();                                      // the previous tile has been read
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int e = tid + 256 * i;
            *reinterpret_cast<float4*>(&rows[e >> 5][4 * (e & 31)]) = pre[i];
        }
        __syncthreads();
        if (r0 + kGramRows < r_end) fetch(r0 + kGramRows);
        if ((MODE == 2 || spart != nullptr) && tid < kP) {
#pragma unroll 8
            for (int rr = 0; rr < kGramRows; ++rr) csum += (double)rows[rr][tid];
        }
        for (int k0 = 0; k0 < kGramRows; k0 += 4) {
            const float* row = rows[k0 + kk];
            const double a1 = (double)row[16 * I1 + c], a2 = (double)row[16 * I2 + c];
#pragma unroll
            for (int sl = 0; sl < 9; ++sl) {
                const bool first = sl < n1;
                const int J = first ? I1 + sl : I2 + sl - n1;
                const double bv = (double)row[16 * J + c];
                acc[sl] = __builtin_amdgcn_mfma_f64_16x16x4f64(first ? a1 : a2, bv, acc[sl], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int sl = 0; sl < 9; ++sl) {
        const bool first = sl < n1;
        const int I = first ? I1 : I2, J = first ? I1 + sl : I2 + sl - n1;
        if constexpr (PACKED) {
            float* o = fpart + (out_idx * kGramTiles + (I * 8 - I * (I - 1) / 2 + J - I)) * 256;
#pragma unroll
            for (int v = 0; v < 4; ++v) o[(4 * v + kk) * 16 + c] = (float)acc[sl][v];
        } else if constexpr (MODE == 2) {
            float* o = fpart + out_idx * kP * kP;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = 16 * I + 4 * v + kk, col = 16 * J + c;
                o[r * kP + col] = (float)acc[sl][v];
                if (I != J) o[col * kP + r] = (float)acc[sl][v];
            }
        } else {
            double* o = gpart + out_idx * kP * kP;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = 16 * I + 4 * v + kk, col = 16 * J + c;
                o[r * kP + col] = acc[sl][v];
                if (I != J) o[col * kP + r] = acc[sl][v];
            }
        }
    }
    if (MODE == 2) {
        if (tid < kP) fsum[out_idx * kP + tid] = (float)csum;
    } else if (spart != nullptr && tid < kP) {
        spart[out_idx * kP + tid] = csum;
    }
}

// Gram partials of fp32 token matrices with 128 features for the 128-wide entropy path (see MODE 2 above):
// exact products, fp64 sums inside a chunk, on the fp64 matrix cores instead of the fp32 ALUs.
hipError_t launch_gram_f32_mfma(const float* X, int n_mat, int N, int64_t mat_stride, int64_t ldx, int n_chunks, int chunk,
                                float* gram_part, float* sum_part, hipStream_t s) {
    sub_gram64_kernel<2><<<dim3((unsigned)n_chunks, (unsigned)n_mat), dim3(256), 0, s>>>(X, mat_stride, ldx, N, chunk, nullptr,
                                                                                    gram_part, nullptr, sum_part);
    return hipGetLastError();
}

// gsum = sum of the slices (fixed order); four loads in flight per thread.
__global__ __launch_bounds__(256) void sub_gram64_sum_kernel(const double* __restrict__ gpart, int n_slices,
                                                             double* __restrict__ gsum) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    const double* g = gpart + e;
    double a = 0.0;
    int sl = 0;
    for (; sl + 3 < n_slices; sl += 4) {
        const double v0 = g[(int64_t)sl * kP * kP], v1 = g[(int64_t)(sl + 1) * kP * kP];
        const double v2 = g[(int64_t)(sl + 2) * kP * kP], v3 = g[(int64_t)(sl + 3) * kP * kP];
        a = (((a + v0) + v1) + v2) + v3;
    }
    for (; sl < n_slices; ++sl) a += g[(int64_t)sl * kP * kP];
    gsum[e] = a;
}

// The sums for the Gram of the projected tokens, from the packed fp32 tiles, mirrored into the fp32 single-chunk
// layout that the 128-wide eigenvalue kernel reads: gram[128*128], then the column sums sums[128] (last block of
// the grid).  Slices are added in fp64 in a fixed order.
__global__ __launch_bounds__(256) void sub_zgram_finish_kernel(const float* __restrict__ fpart,
                                                               const double* __restrict__ spart, int n_slices,
                                                               float* __restrict__ gram, float* __restrict__ sums) {
    __shared__ double quarter[3][64];
    if (blockIdx.x == kP * kP / 64) {
        if (threadIdx.x < kP) {
            double a = 0.0;
#pragma unroll 8
            for (int sl = 0; sl < n_slices; ++sl) a += spart[(int64_t)sl * kP + threadIdx.x];
            sums[threadIdx.x] = (float)a;
        }
        return;
    }
    // a workgroup adds 64 entries: four quarters of the slices side by side (sixteen loads in flight per thread:
    // the sum is a chain of memory round trips, not of bytes), then the quarters in order
    const int i = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + i;
    const int r = e >> 7, col = e & (kP - 1);
    const int I = min(r, col) >> 4, J = max(r, col) >> 4;          // the tile that holds (r, col) or its mirror image
    const int ri = r <= col ? r : col, ci = r <= col ? col : r;    // inside an off-diagonal tile: (row of I, column of J)
    int at;
    if (I == J) at = (r & 15) * 16 + (col & 15);                    // diagonal tiles are stored whole
    else at = (ri & 15) * 16 + (ci & 15);
    const float* g = fpart + (int64_t)(I * 8 - I * (I - 1) / 2 + J - I) * 256 + at;
    const int64_t stride = (int64_t)kGramTiles * 256;
    const int per = (n_slices + 3) / 4;
    const int s0 = q * per, s1 = min(n_slices, s0 + per);
    double a = 0.0;
    int sl = s0;
    for (; sl + 15 < s1; sl += 16) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = g[(sl + u) * stride];
#pragma unroll
        for (int u = 0; u < 16; ++u) a += (double)v[u];
    }
    for (; sl < s1; ++sl) a += (double)g[sl * stride];
    if (q > 0) quarter[q - 1][i] = a;
    __syncthreads();
    if (q == 0) gram[e] = (float)(((a + quarter[0][i]) + quarter[1][i]) + quarter[2][i]);
}

// value of x in lane `src` (a compile-time constant after unrolling) as a wave-uniform double
__device__ __forceinline__ double lane_value(double x, int src) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), src);
    return __hiloint2double(hi, lo);
}

// One workgroup: Cholesky G = L L^T in LDS (fp64), then Rinv = L^-T as fp32 so that Q = W Rinv has
// orthonormal columns.  A pivot below 1e-12 of the largest diagonal entry retires its column (its
// row and column of Rinv are zero).  Both halves work on 16-wide blocks, two workgroup barriers
// per block instead of two per column:
//   factor   the 16 x 16 diagonal block in the registers of one wave (lane = row, values of other
//            rows by v_readlane), the rows below it by forward substitution (one thread per row),
//            the trailing triangle by a rank-16 update in 16 x 16 tiles (v_mfma_f64_16x16x4_f64);
//   invert   X = L^-1: the eight 16 x 16 inverses of the diagonal blocks at once (one thread per
//            column), then block row by block row as products of tiles.  X[k][c], k > c, lives at
//            G[c][k] in the unused upper triangle.
// Phase times of one call (100 MHz wall clock, warm input): first diagonal block 3 us, rows below 9,
// trailing tiles with the next diagonal block beside them 22, diagonal inverses 2, block rows of the
// inverse 12: 49 us.  With the tiled parts on the vector ALUs, a substitution per block row and the
// diagonal blocks on their own it was 101.
__global__ __launch_bounds__(256) void sub_chol_kernel(const double* __restrict__ gsum, float* __restrict__ Rinv) {
    extern __shared__ __align__(16) double G[];                // [128][129]
    __shared__ double dinv[kP];
    __shared__ double maxdiag;
    constexpr int LD = kP + 1, B = 16, NB = kP / B;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const double2* g2 = reinterpret_cast<const double2*>(gsum);
    for (int e0 = tid; e0 < kP * kP / 2; e0 += 256 * 16) {         // 32 loads per thread, sixteen in flight
        double2 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = g2[e0 + 256 * u];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int e = e0 + 256 * u, row = e >> 6, col = 2 * (e & 63);
            G[row * LD + col] = v[u].x;
            G[row * LD + col + 1] = v[u].y;
        }
    }
    __syncthreads();
    if (wv == 0) {
        double m = fmax(G[lane * LD + lane], G[(lane + 64) * LD + lane + 64]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m = fmax(m, __shfl_xor(m, o, 64));
        if (lane == 0) maxdiag = m;
    }
    __syncthreads();
    const double tol = maxdiag * 1e-12;
    // diagonal block p, by one wave: lane i (and its copies in the upper lanes) holds row 16 p + i
    auto factor_diagonal = [&](int p) {
        const int j0 = B * p;
        const int i = lane & (B - 1);
        double a[B];
#pragma unroll
        for (int k = 0; k < B; ++k) a[k] = G[(j0 + i) * LD + j0 + k];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const double piv = lane_value(a[j], j);
            const bool live = piv > tol;
            const double di = live ? rsqrt(piv) : 0.0;              // one reciprocal square root instead of a root and a division
            const double d = piv * di;
            a[j] = i == j ? d : a[j] * di;                           // rows i < j: values nobody reads
#pragma unroll
            for (int k = j + 1; k < B; ++k) {
                const double lkj = lane_value(a[j], k);              // L[k][j]
                a[k] = fma(-a[j], lkj, a[k]);                        // G[i][k] -= L[i][j] L[k][j]; only j < k <= i is read later
            }
            if (lane == 0) dinv[j0 + j] = di;
        }
        if (lane < B) {
#pragma unroll
            for (int k = 0; k < B; ++k)
                if (k <= i) G[(j0 + i) * LD + j0 + k] = a[k];
        }
    };
    // Trailing tile t of block p (t = ti (ti + 1) / 2 + tk, tk <= ti: tile (p + 1 + ti, p + 1 + tk)) on the fp64
    // matrix cores: -= L[I][p] L[K][p]^T.  Operand lane (c, kk) holds row c of its factor at column 4 s + kk of the
    // panel; result register v is row 4 v + kk, column c.  Diagonal tiles are computed whole: what lands above
    // the diagonal is not read by the factorisation.
    auto update_tile = [&](int p, int t) {
        const int j0 = B * p;
        const int c = lane & 15, kk = lane >> 4;
        int ti = 0, rem = t;
        while (rem > ti) {
            rem -= ti + 1;
            ++ti;
        }
        const int r0 = B * (p + 1 + ti), c0 = B * (p + 1 + rem);
        f64x4_t acc;
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v] = G[(r0 + 4 * v + kk) * LD + c0 + c];
#pragma unroll
        for (int sx = 0; sx < 4; ++sx) {
            const double av = -G[(r0 + c) * LD + j0 + 4 * sx + kk];
            const double bv = G[(c0 + c) * LD + j0 + 4 * sx + kk];
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) G[(r0 + 4 * v + kk) * LD + c0 + c] = acc[v];
    };
    if (wv == 0) factor_diagonal(0);
    __syncthreads();
    for (int p = 0; p < NB; ++p) {
        const int j0 = B * p;
        {
            // rows below the block: L[r][j0 + j] = (G[r][j0 + j] - sum_{k<j} L[r][j0 + k] L[j0 + j][j0 + k]) / L[j0 + j][j0 + j]
            const int r = j0 + B + tid;
            if (r < kP) {
                // column by column: once l[j] is known, the entries to its right take their updates, which do not
                // depend on one another (the chain through the row is 16 multiplications long, not 120 FMAs)
                double l[B];
#pragma unroll
                for (int j = 0; j < B; ++j) l[j] = G[r * LD + j0 + j];
#pragma unroll
                for (int j = 0; j < B; ++j) {
                    l[j] *= dinv[j0 + j];
#pragma unroll
                    for (int k = j + 1; k < B; ++k) l[k] = fma(-l[j], G[(j0 + k) * LD + j0 + j], l[k]);
                }
#pragma unroll
                for (int j = 0; j < B; ++j) G[r * LD + j0 + j] = l[j];
            }
        }
        __syncthreads();
        {
            // Trailing lower triangle.  Wave 0 updates the next diagonal tile (tile 0) and factors it straight away,
            // while the other three waves share the remaining tiles: the one-wave factorisation, the longest step of
            // a block, runs beside the update instead of after it.
            const int m = NB - 1 - p;
            const int n_tiles = m * (m + 1) / 2;
            if (wv == 0) {
                if (n_tiles > 0) {
                    update_tile(p, 0);
                    factor_diagonal(p + 1);
                }
            } else {
                for (int t = wv; t < n_tiles; t += 3) update_tile(p, t);
            }
        }
        __syncthreads();
    }
    // X = L^-1.  X[k][c] (k > c) is kept at G[c][k], in the unused upper triangle; X[c][c] = dinv[c].
    // First the eight diagonal tiles T_I = L_II^-1, all at once: thread c solves column c of its tile (the chain
    // through the 16 rows is paid once, not once per block row).
    if (tid < kP) {
        const int c = tid, i0 = c & ~(B - 1);
        double x[B];
#pragma unroll
        for (int ii = 0; ii < B; ++ii) x[ii] = i0 + ii == c ? 1.0 : 0.0;
#pragma unroll
        for (int ii = 0; ii < B; ++ii) {
            x[ii] = i0 + ii < c ? 0.0 : x[ii] * dinv[i0 + ii];
#pragma unroll
            for (int jj = ii + 1; jj < B; ++jj) x[jj] = fma(-G[(i0 + jj) * LD + i0 + ii], x[ii], x[jj]);
        }
#pragma unroll
        for (int ii = 0; ii < B; ++ii)
            if (i0 + ii > c) G[c * LD + i0 + ii] = x[ii];
    }
    __syncthreads();
    // Then block row I by tiles on the fp64 matrix cores:
    //   S(I, C) = -sum_{K=C}^{I-1} L(I, K) X(K, C)   (X(K, C) sits transposed in the upper triangle, so both operands
    //                                                 are read along rows of G; X(C, C) = T_C is lower triangular)
    //   X(I, C) = T_I S(I, C)                         (register v of the result S is row 4 v + kk: exactly the lane's
    //                                                 operand of contraction step v, so S never leaves the registers)
    for (int I = 1; I < NB; ++I) {
        const int i0 = B * I;
        const int c = lane & 15, kk = lane >> 4;
        for (int C = wv; C < I; C += 4) {                            // wave w takes the column tiles w and w + 4
            f64x4_t acc = {0.0, 0.0, 0.0, 0.0};
            for (int K = C; K < I; ++K) {
#pragma unroll
                for (int sx = 0; sx < 4; ++sx) {
                    const int k = 4 * sx + kk;                       // row of X / column of L inside tile K
                    const double av = -G[(i0 + c) * LD + B * K + k];
                    double bv = G[(B * C + c) * LD + B * K + k];
                    if (K == C) bv = k > c ? bv : (k == c ? dinv[B * C + c] : 0.0);
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
                }
            }
            f64x4_t xt = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int sx = 0; sx < 4; ++sx) {
                const int k = 4 * sx + kk;                           // T_I[c][k], kept at G[i0 + k][i0 + c] for k < c
                const double tv = k < c ? G[(i0 + k) * LD + i0 + c] : (k == c ? dinv[i0 + c] : 0.0);
                xt = __builtin_amdgcn_mfma_f64_16x16x4f64(tv, acc[sx], xt, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) G[(B * C + c) * LD + i0 + 4 * v + kk] = xt[v];
        }
        __syncthreads();
    }
    // Rinv = (L^-1)^T: Rinv[c][i] = X[i][c], zero for i < c.  Written once, in rows, after the loop: a store to
    // global memory inside it would be waited for at every workgroup barrier.
    for (int e = tid; e < kP * kP; e += 256) {
        const int c = e >> 7, i = e & (kP - 1);
        Rinv[e] = i > c ? (float)G[c * LD + i] : (i == c ? (float)dinv[c] : 0.f);
    }
}

MatrixPlan plan_matrix(int N, int D) {
    MatrixPlan p;
    p.stat_chunks = N < 128 * 64 ? (N + 63) / 64 : 128;
    p.stat_chunk = (N + p.stat_chunks - 1) / p.stat_chunks;
    p.stat_chunks = (N + p.stat_chunk - 1) / p.stat_chunk;
    // split of the token sum in W = X^T Z: enough workgroups for the chip, partials kept modest
    const int row_blocks = (D + 63) / 64;
    int kc = (1024 + row_blocks - 1) / row_blocks;
    if (kc > 16) kc = 16;
    const int max_kc = (N + 255) / 256;
    if (kc > max_kc) kc = max_kc;
    if (kc < 1) kc = 1;
    p.w_chunk = ((N + kc - 1) / kc + 15) / 16 * 16;
    p.w_chunks = (N + p.w_chunk - 1) / p.w_chunk;
    // Gram of W: 64-row slices (one staged tile per workgroup: 14 + 7 us against 20 + 5 with 128 rows at D = 4096); Gram of the projected tokens: one workgroup per CU at most, whole 64-row tiles each
    p.gram_rows = kGramRows;
    p.gram_slices = (D + p.gram_rows - 1) / p.gram_rows;
    p.zgram_rows = ((N + 255) / 256 + kGramRows - 1) / kGramRows * kGramRows;
    p.zgram_slices = (N + p.zgram_rows - 1) / p.zgram_rows;
    // the eigenvalue kernel reads one already summed chunk
    p.ep.n_chunks = 1;
    p.ep.chunk = N;
    p.ep.gram_off = 0;
    p.ep.sum_off = (size_t)kP * kP * sizeof(float);
    p.ep.bytes = p.ep.sum_off + (size_t)kP * sizeof(float);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    p.ep_off = take(p.ep.bytes);
    p.statpart_off = take((size_t)p.stat_chunks * 2 * D * sizeof(double));
    p.s_off = take((size_t)D * sizeof(double));
    p.trace_off = take((size_t)(2 + 2 * ((D + 255) / 256)) * sizeof(double));     // the traces, then per-workgroup shares
    p.zsum_off = take((size_t)(1 + D / kQRows) * kP * sizeof(double));     // the sums, then the row blocks' shares
    p.q_off = take((size_t)D * kP * sizeof(float));
    p.w_off = take((size_t)D * kP * sizeof(float));
    // token chunks of the MFMA version of W = X^T Z (whole rounds of 128 tokens)
    int tn = (512 + D / 128 - 1) / (D / 128);
    if (tn > 16) tn = 16;
    if (tn < 1) tn = 1;
    p.t_chunk = ((N + tn - 1) / tn + 127) / 128 * 128;
    p.t_chunks = (N + p.t_chunk - 1) / p.t_chunk;
    p.wpart_off = take((size_t)(p.w_chunks > p.t_chunks ? p.w_chunks : p.t_chunks) * D * kP * sizeof(float));
    p.z_off = take((size_t)N * kP * sizeof(float));
    const int max_slices = p.gram_slices > p.zgram_slices ? p.gram_slices : p.zgram_slices;
    p.gpart_off = take((size_t)(max_slices + 1) * kP * kP * sizeof(double));     // slices, then their sum
    p.spart_off = take((size_t)p.zgram_slices * kP * sizeof(double));
    p.rinv_off = take((size_t)kP * kP * sizeof(float));
    // bf16 MFMA products: Q^T as two bf16 halves, partial Z of the split over d
    const int row_wgs = (N + 255) / 256;
    int zs = (512 + row_wgs - 1) / row_wgs;
    if (zs > 8) zs = 8;
    if (zs > D / 256) zs = D / 256;
    if (zs < 1) zs = 1;
    p.z_splits = zs;
    p.qt_off = take((size_t)2 * kP * D * sizeof(bf16_bits));
    p.zpart_off = take(zs > 1 ? (size_t)zs * N * kP * sizeof(float) : 0);
    p.zsplit_off = take((((size_t)N + 127) / 128 * 128) * kP * sizeof(bf16_bits));      // Z^T rounded to bf16
    p.bytes = off;
    return p;
}

template <typename T>
static hipError_t run_matrix_entropy(const T* X, int n_mat, int N, int D, int64_t mat_stride, int64_t ldx,
                                     int k_trunc, unsigned flags, int n_iter, const MatrixPlan& p, char* ws,
                                     float* entropy_out, float* eig_out, const Env& env) {
    hipStream_t s = env.s;
    const bool center = (flags & UNCOMP_CENTER) != 0;
    double* statpart = reinterpret_cast<double*>(ws + p.statpart_off);
    double* sv = reinterpret_cast<double*>(ws + p.s_off);
    double* trace = reinterpret_cast<double*>(ws + p.trace_off);
    double* zsum = reinterpret_cast<double*>(ws + p.zsum_off);
    float* Q = reinterpret_cast<float*>(ws + p.q_off);
    float* W = reinterpret_cast<float*>(ws + p.w_off);
    float* Wpart = reinterpret_cast<float*>(ws + p.wpart_off);
    float* Z = reinterpret_cast<float*>(ws + p.z_off);
    double* gpart = reinterpret_cast<double*>(ws + p.gpart_off);
    double* gsum = gpart + (size_t)(p.gram_slices > p.zgram_slices ? p.gram_slices : p.zgram_slices) * kP * kP;
    double* spart = reinterpret_cast<double*>(ws + p.spart_off);
    float* Rinv = reinterpret_cast<float*>(ws + p.rinv_off);
    const size_t chol_lds = (size_t)kP * (kP + 1) * sizeof(double);
    const unsigned dp_blocks = (unsigned)(((int64_t)D * kP + 255) / 256);
    // bf16 inputs with 16-byte aligned rows take the MFMA products, everything else the fp32 ALUs
    // (rows at most 2^22 elements apart: those kernels address 256 rows with 32-bit byte offsets)
    bool mfma = false;
    if constexpr (sizeof(T) == 2)
        mfma = !env.force_alu && (ldx % 8) == 0 && (mat_stride % 8) == 0 && (reinterpret_cast<uintptr_t>(X) & 15u) == 0 &&
               ldx <= ((int64_t)1 << 22);
    bf16_bits* Qt_hi = reinterpret_cast<bf16_bits*>(ws + p.qt_off);
    bf16_bits* Qt_lo = Qt_hi + (size_t)kP * D;
    // Q = orth(W): Cholesky QR with the Gram in fp64; the last kernel also leaves the bf16 halves of Q^T and the
    // shares of s^T Q for the round that follows
    auto orth = [&]() {
        sub_gram64_kernel<0><<<dim3((unsigned)p.gram_slices), dim3(256), 0, s>>>(W, 0, kP, D, p.gram_rows, gpart, nullptr, nullptr, nullptr);
        sub_gram64_sum_kernel<<<dim3(kP * kP / 256), dim3(256), 0, s>>>(gpart, p.gram_slices, gsum);
        sub_chol_kernel<<<dim3(1), dim3(256), chol_lds, s>>>(gsum, Rinv);
        sub_q_kernel<<<dim3((unsigned)(D / kQRows)), dim3(256), 0, s>>>(W, Rinv, D, center ? sv : nullptr, Q,
                                                                       mfma ? Qt_hi : nullptr, Qt_lo, zsum + kP);
    };
    float* Zpart = reinterpret_cast<float*>(ws + p.zpart_off);
    bf16_bits* Zt = reinterpret_cast<bf16_bits*>(ws + p.zsplit_off);
    hipError_t perr = hipSuccess;
    // Z is always rounded to bf16 on its way into W = X^T Z (2^-9 relative error per element, averaged over the
    // tokens of the sum); Q enters Z = X Q as its high bf16 half in all rounds but the last, and as both halves in
    // the last round and in the final projection.  What a round with rounded factors gets wrong is a small tilt of
    // the iterated subspace, which the next round removes like any other component outside the dominant subspace,
    // and the eigenvalues of the projection move only with the square of the tilt that is left (measured against
    // the fp64 reference: entropy off by 1.6e-6 relative at most; 5e-5 if the last round rounds Q as well; keeping
    // both halves of Z in the last round too changes nothing).
    const int first_precise = n_iter - 1;
    bool zt_ready = false;                                // the last projection left the transposed halves of Z, not Z
    auto project = [&](const T* Xm, bool precise, bool for_round) {       // Z = X Q
        zt_ready = false;
        if constexpr (sizeof(T) == 2) {
            if (mfma) {
                hipError_t e = launch_xq_mfma(Xm, ldx, N, D, Qt_hi, Qt_lo, p.z_splits, Zpart, Z, s, precise, for_round, Zt,
                                              &zt_ready);
                if (e != hipSuccess) perr = e;
                return;
            }
        }
        sub_gemm_kernel<T, false><<<dim3((unsigned)((N + 63) / 64), 1), dim3(256), 0, s>>>(Xm, ldx, Q, N, D, D, Z);
    };
    for (int m = 0; m < n_mat; ++m) {
        const T* Xm = X + (int64_t)m * mat_stride;
        env.begin("matrix_colstats");
        sub_colstats_kernel<T><<<dim3((unsigned)((D / 8 + 63) / 64), (unsigned)p.stat_chunks), dim3(256), 0, s>>>(
            Xm, N, D, ldx, p.stat_chunk, statpart);
        sub_colstats_finish_kernel<<<dim3((unsigned)((D + 255) / 256)), dim3(256), 0, s>>>(statpart, p.stat_chunks, D, N, sv,
                                                                                          trace + 2);
        sub_trace_kernel<<<dim3(1), dim3(64), 0, s>>>(trace + 2, (D + 255) / 256, trace);
        env.end();
        env.begin("matrix_subspace");
        sub_start_kernel<<<dim3(dp_blocks), dim3(256), 0, s>>>(W, D);
        orth();
        for (int it = 0; it < n_iter; ++it) {
            const bool precise = it >= first_precise;
            project(Xm, precise, true);
            if (center) {
                sub_zsum_kernel<<<dim3(1), dim3(1024), 0, s>>>(zsum + kP, D / kQRows, zsum);
            }
            int w_parts = p.w_chunks;
            bool done = false;
            if constexpr (sizeof(T) == 2) {
                if (mfma) {
                    hipError_t e = launch_xtz_mfma(Xm, ldx, Z, N, D, Zt, p.t_chunk, p.t_chunks, Wpart, s, zt_ready);
                    if (e != hipSuccess) return e;
                    w_parts = p.t_chunks;
                    done = true;
                }
            }
            if (!done)
                sub_gemm_kernel<T, true><<<dim3((unsigned)((D + 63) / 64), (unsigned)p.w_chunks), dim3(256), 0, s>>>(
                    Xm, ldx, Z, D, N, p.w_chunk, Wpart);
            sub_reduce_kernel<<<dim3(dp_blocks), dim3(256), 0, s>>>(Wpart, w_parts, D, center ? sv : nullptr, zsum,
                                                                    1.0 / (double)N, W);
            orth();
            if (it == n_iter - 1) {          // once more: the last Q is orthonormal to fp32 rounding
                hipError_t e = hipMemcpyAsync(W, Q, (size_t)D * kP * sizeof(float), hipMemcpyDeviceToDevice, s);
                if (e != hipSuccess) return e;
                orth();
            }
        }
        project(Xm, true, false);
        env.end();
        if (perr != hipSuccess) return perr;
        // the projected tokens go through the 128-wide entropy path; trace(C) replaces its own trace
        env.begin("matrix_gram");
        float* fpart = reinterpret_cast<float*>(gpart);          // the region of the fp64 slices, free by now
        sub_gram64_kernel<1><<<dim3((unsigned)p.zgram_slices), dim3(256), 0, s>>>(Z, 0, kP, N, p.zgram_rows, nullptr, fpart, spart, nullptr);
        sub_zgram_finish_kernel<<<dim3(kP * kP / 64 + 1), dim3(256), 0, s>>>(
            fpart, spart, p.zgram_slices, reinterpret_cast<float*>(ws + p.ep_off + p.ep.gram_off),
            reinterpret_cast<float*>(ws + p.ep_off + p.ep.sum_off));
        env.end();
        hipError_t e = launch_tridiag_entropy(1, N, k_trunc, flags, p.ep, ws + p.ep_off, entropy_out + m,
                                   eig_out != nullptr ? eig_out + (int64_t)m * kP : nullptr, env,
                                   trace);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

hipError_t launch_matrix_entropy(const void* X, uncomp_dtype dt, int n_mat, int N, int D, int64_t mat_stride,
                                 int64_t ldx, int k_trunc, unsigned flags, int n_iter, const MatrixPlan& p, char* ws,
                                 float* entropy_out, float* eig_out, const Env& env) {
    if (dt == UNCOMP_BF16)
        return run_matrix_entropy(static_cast<const bf16_bits*>(X), n_mat, N, D, mat_stride, ldx, k_trunc, flags, n_iter,
                                  p, ws, entropy_out, eig_out, env);
    return run_matrix_entropy(static_cast<const float*>(X), n_mat, N, D, mat_stride, ldx, k_trunc, flags, n_iter, p, ws,
                              entropy_out, eig_out, env);
}

hipError_t init_subspace_mfma_kernels();

hipError_t init_subspace_kernels() {
    hipError_t e = init_subspace_mfma_kernels();
    if (e != hipSuccess) return e;
    return allow_dynamic_lds(reinterpret_cast<const void*>(sub_chol_kernel), (size_t)kP * (kP + 1) * sizeof(double));
}

}  // namespace uncomp
