// Eigen stage of the truncated matrix entropy (Lemma 2: entropy from the eigenvalues of
// the covariance; Sec. 3.2 Eq. 5: only the k largest enter; proof of Lemma 4: unit trace).
//
// One workgroup per matrix:
//   1. add the Gram partials of the matrix in fp64, subtract the mean term s s^T / N
//      (Eq. 1; the common factor 1/(N-1) drops out under the unit-trace scaling), divide
//      by the trace and keep the 128x128 result as fp32 columns in LDS;
//   2. one-sided (Hestenes) Jacobi: plane rotations make the columns mutually orthogonal;
//      for a symmetric positive semi-definite matrix the column norms then equal the
//      eigenvalues.  Round-robin ordering gives 64 independent column pairs per round,
//      each handled by four adjacent lanes (32 rows each) that combine their partial dot
//      products by lane shuffles;
//   3. column norms -> descending order by rank counting -> truncated entropy in fp64.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kThreads = 256;
constexpr int kLd = kJacobiLd;
// A sweep whose largest |cos| between paired columns stayed below this leaves, after its
// own rotations, angles of the order of the square of it: eigenvalue errors at fp32 rounding.
constexpr float kStopCos2 = 5e-3f * 5e-3f;

struct Smem {
    float A[kD * kLd];       // column j at A + j*kLd
    double s[kD];            // column sums of X (for the mean correction)
    double red[8];
    float lam[kD];
    float sorted[kD];
    float flag[4];
};

__device__ __forceinline__ double block_sum(double v, double* red, int tid) {
    v = wave_sum(v);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

__device__ __forceinline__ float quad_sum(float v) {
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    return v;
}

}  // namespace

__global__ __launch_bounds__(kThreads) void jacobi_entropy_kernel(
    const float* __restrict__ gram_part, const float* __restrict__ sum_part, int n_chunks, int N,
    int k_trunc, unsigned flags, float* __restrict__ entropy_out, float* __restrict__ eig_out) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const float* Gm = gram_part + (int64_t)m * n_chunks * (kD * kD);
    const float* Sm = sum_part + (int64_t)m * n_chunks * kD;

    // ---- 1. reduce partials, centre, unit trace ------------------------------------------
    if (tid < kD) {
        double acc = 0.0;
        for (int c = 0; c < n_chunks; ++c) acc += (double)Sm[c * kD + tid];
        sm.s[tid] = acc;
    }
    __syncthreads();
    const bool center = (flags & UNCOMP_CENTER) != 0;
    const double inv_n = 1.0 / (double)N;
    // trace first (diagonal only), so the scaled matrix can be written in one go
    double tr_c = 0.0, tr_u = 0.0;
    if (tid < kD) {
        double acc = 0.0;
        for (int c = 0; c < n_chunks; ++c) acc += (double)Gm[(int64_t)c * (kD * kD) + tid * (kD + 1)];
        tr_u = acc;
        tr_c = center ? acc - sm.s[tid] * sm.s[tid] * inv_n : acc;
    }
    const double trace = block_sum(tr_c, sm.red, tid);
    const double trace_u = block_sum(tr_u, sm.red, tid);
    // Zero spread: a single token, or a centred trace so far below the second moment that
    // the fp32 partial sums cannot tell it from zero.
    const bool degenerate = !(trace > 0.0) || (center && (N < 2 || trace < trace_u * 0x1p-20));
    if (degenerate) {
        if (tid == 0) entropy_out[m] = 0.f;
        if (eig_out != nullptr && tid < kD) eig_out[(int64_t)m * kD + tid] = 0.f;
        return;
    }
    const double inv_tr = 1.0 / trace;
    for (int k = 0; k < 64; ++k) {
        int e = tid + k * kThreads;          // element e = i*128 + j
        int i = e >> 7, j = e & 127;
        double acc = 0.0;
        for (int c = 0; c < n_chunks; ++c) acc += (double)Gm[(int64_t)c * (kD * kD) + e];
        if (center) acc -= sm.s[i] * sm.s[j] * inv_n;
        sm.A[j * kLd + i] = (float)(acc * inv_tr);
    }
    __syncthreads();

    // ---- 2. one-sided Jacobi ---------------------------------------------------------------
    const int slot = tid >> 2;     // which of the 64 pairs of a round
    const int sub = tid & 3;       // which quarter of the rows (interleaved float4 groups)
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        float max_cos2 = 0.f;
        for (int r = 0; r < kD - 1; ++r) {
            int p, q;
            if (slot == 0) {
                p = kD - 1;
                q = r;
            } else {
                p = r + slot;
                if (p >= kD - 1) p -= kD - 1;
                q = r - slot;
                if (q < 0) q += kD - 1;
            }
            float4* cp = reinterpret_cast<float4*>(sm.A + p * kLd);
            float4* cq = reinterpret_cast<float4*>(sm.A + q * kLd);
            float4 ap[8], aq[8];
            float alpha = 0.f, beta = 0.f, gamma = 0.f;
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                ap[v] = cp[4 * v + sub];
                aq[v] = cq[4 * v + sub];
                alpha += ap[v].x * ap[v].x + ap[v].y * ap[v].y + ap[v].z * ap[v].z + ap[v].w * ap[v].w;
                beta += aq[v].x * aq[v].x + aq[v].y * aq[v].y + aq[v].z * aq[v].z + aq[v].w * aq[v].w;
                gamma += ap[v].x * aq[v].x + ap[v].y * aq[v].y + ap[v].z * aq[v].z + ap[v].w * aq[v].w;
            }
            alpha = quad_sum(alpha);
            beta = quad_sum(beta);
            gamma = quad_sum(gamma);
            const float ab = alpha * beta;
            const float g2 = gamma * gamma;
            if (ab > 0.f && g2 > 1e-14f * ab) {        // same decision in all four lanes
                max_cos2 = fmaxf(max_cos2, g2 / ab);
                float zeta = (beta - alpha) / (2.f * gamma);
                float t = copysignf(1.f, zeta) / (fabsf(zeta) + sqrtf(1.f + zeta * zeta));
                float c = rsqrtf(1.f + t * t);
                float s = c * t;
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    float4 np, nq;
                    np.x = c * ap[v].x - s * aq[v].x;  nq.x = s * ap[v].x + c * aq[v].x;
                    np.y = c * ap[v].y - s * aq[v].y;  nq.y = s * ap[v].y + c * aq[v].y;
                    np.z = c * ap[v].z - s * aq[v].z;  nq.z = s * ap[v].z + c * aq[v].z;
                    np.w = c * ap[v].w - s * aq[v].w;  nq.w = s * ap[v].w + c * aq[v].w;
                    cp[4 * v + sub] = np;
                    cq[4 * v + sub] = nq;
                }
            }
            __syncthreads();
        }
        // every thread learns the sweep's largest cos^2
        max_cos2 = wave_max(max_cos2);
        if ((tid & 63) == 0) sm.flag[tid >> 6] = max_cos2;
        __syncthreads();
        float mc = fmaxf(fmaxf(sm.flag[0], sm.flag[1]), fmaxf(sm.flag[2], sm.flag[3]));
        __syncthreads();
        if (mc < kStopCos2) break;
    }

    // ---- 3. eigenvalues, ordering, entropy -----------------------------------------------
    if (tid < kD) {
        const float* col = sm.A + tid * kLd;
        double n2 = 0.0;
        for (int i = 0; i < kD; ++i) n2 += (double)col[i] * (double)col[i];
        sm.lam[tid] = (float)sqrt(n2);
    }
    __syncthreads();
    if (tid < kD) {
        float mine = sm.lam[tid];
        int rank = 0;
        for (int i = 0; i < kD; ++i) {
            float o = sm.lam[i];
            rank += (o > mine || (o == mine && i < tid)) ? 1 : 0;
        }
        sm.sorted[rank] = mine;
    }
    __syncthreads();
    const int k = k_trunc < kD ? k_trunc : kD;
    double mine = tid < kD ? (double)sm.sorted[tid] : 0.0;
    const double total = block_sum(mine, sm.red, tid);
    const double topk = block_sum(tid < k ? mine : 0.0, sm.red, tid);
    const double denom = (flags & UNCOMP_TRUNC_RENORM) ? topk : total;
    double term = 0.0;
    if (tid < k && mine > 0.0 && denom > 0.0) {
        double sgm = mine / denom;
        term = -sgm * log(sgm);
    }
    const double H = block_sum(term, sm.red, tid);
    if (tid == 0) entropy_out[m] = (float)H;
    if (eig_out != nullptr && tid < kD)
        eig_out[(int64_t)m * kD + tid] = total > 0.0 ? (float)(mine / total) : 0.f;
}

hipError_t launch_jacobi_entropy(int n_mat, int N, int k_trunc, unsigned flags,
                                 const EntropyPlan& p, char* ws, float* entropy_out,
                                 float* eig_out, const Env& env) {
    hipStream_t s = env.s;
    static_assert(sizeof(Smem) <= 160 * 1024, "LDS budget");
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(jacobi_entropy_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Smem));
    if (e != hipSuccess) return e;
    const float* gram = reinterpret_cast<const float*>(ws + p.gram_off);
    const float* sums = reinterpret_cast<const float*>(ws + p.sum_off);
    env.begin("jacobi_entropy");
    jacobi_entropy_kernel<<<dim3(n_mat), dim3(kThreads), sizeof(Smem), s>>>(
        gram, sums, p.n_chunks, N, k_trunc, flags, entropy_out, eig_out);
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
