// Eigen stage of the truncated matrix entropy (Lemma 2: entropy from the eigenvalues of
// the covariance; Sec. 3.2 Eq. 5: only the k largest enter; proof of Lemma 4: unit trace).
//
// One workgroup per matrix:
//   1. add the Gram partials of the matrix in fp64, subtract the mean term s s^T / N
//      (Eq. 1; the common factor 1/(N-1) drops out under the unit-trace scaling), divide
//      by the trace and keep the 128x128 result as fp32 columns in LDS;
//   2. one-sided (Hestenes) Jacobi: plane rotations make the columns mutually orthogonal;
//      for a symmetric positive semi-definite matrix the column norms then equal the
//      eigenvalues.  Each pair of columns is handled by four adjacent lanes (32 rows each)
//      that combine their partial dot products with DPP quad permutes, 16 pairs per wave
//      per round.  The sweep is ordered in two levels so that waves rarely have to meet:
//      the 128 columns form 8 half-blocks of 16; a sweep is 7 block rounds (round-robin
//      over the half-blocks, each wave owning one pair of half-blocks and running its 16
//      cross rounds on its own) plus one phase of pairs inside the half-blocks.  That is
//      8 workgroup barriers per sweep for the same 127 rounds / 8128 rotations;
//   3. column norms -> descending order by rank counting -> truncated entropy in fp64.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

constexpr int kThreads = 256;
constexpr int kLd = kJacobiLd;
// A sweep whose largest |cos| between paired columns stayed below this leaves, after its
// own rotations, angles of the order of the square of it: eigenvalue errors at fp32 rounding.
constexpr float kStopCos2 = 1e-2f * 1e-2f;

struct Smem {
    float A[kD * kLd];       // column j at A + j*kLd
    double s[kD];            // column sums of X (for the mean correction)
    double red[8];
    float lam[kD];
    float sorted[kD];
    float dsc[kD];           // column j of the matrix is dsc[j] * A[j]
    float n2[kD];            // running squared norms of the columns
    float flag[4];
};

__device__ __forceinline__ double block_sum(double v, double* red, int tid) {
    v = wave_sum(v);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// Sum over the four lanes of a quad (all four get the same bits): DPP quad_perm [1,0,3,2]
// then [2,3,0,1].
__device__ __forceinline__ float quad_sum(float v) {
    v += __uint_as_float(__builtin_amdgcn_mov_dpp(__float_as_uint(v), 0xB1, 0xF, 0xF, true));
    v += __uint_as_float(__builtin_amdgcn_mov_dpp(__float_as_uint(v), 0x4E, 0xF, 0xF, true));
    return v;
}

// Sum of v over the four lanes {k, k+16, k+32, k+48}, delivered to all four with identical bits.
// v_permlane32_swap(a,b) -> ([a.lo32, b.lo32], [a.hi32, b.hi32]);
// v_permlane16_swap(a,b) -> ([a.r0, b.r0, a.r2, b.r2], [a.r1, b.r1, a.r3, b.r3])  (r = row of 16 lanes).
__device__ __forceinline__ float rows_allreduce(float v) {
    auto s1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    const float h = __uint_as_float(s1[0]) + __uint_as_float(s1[1]);      // rows 0,2: v0+v2; rows 1,3: v1+v3
    auto s2 = __builtin_amdgcn_permlane16_swap(__float_as_uint(h), __float_as_uint(h), false, false);
    return __uint_as_float(s2[0]) + __uint_as_float(s2[1]);
}

// Rotates a register by one lane inside each row of 16 lanes (DPP row_ror:1).
__device__ __forceinline__ float row_rotate(float v) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x121, 0xF, 0xF, false));
}

}  // namespace

__global__ __launch_bounds__(kThreads) void jacobi_entropy_kernel(
    const float* __restrict__ gram_part, const float* __restrict__ sum_part, int n_chunks, int N,
    int k_trunc, unsigned flags, float* __restrict__ entropy_out, float* __restrict__ eig_out, int eig_ld) {
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
        if (eig_out != nullptr && tid < eig_ld) eig_out[(int64_t)m * eig_ld + tid] = 0.f;
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
    // Rotations are applied in scaled form: column j is kept as dsc[j] * A[j], so that
    //   a_p' = c (a_p - t a_q),  a_q' = c (a_q + t a_p)
    // costs one multiply-add per element (A_p -= (t dsc_q/dsc_p) A_q, A_q += (t dsc_p/dsc_q) A_p)
    // and the common factor c goes into dsc.  Squared column norms are carried along
    // (|a_p'|^2 = |a_p|^2 - t gamma, |a_q'|^2 = |a_q|^2 + t gamma), leaving one dot product per
    // pair.  Scales are folded back into the columns at every workgroup barrier and the norms
    // are recomputed from the columns at the start of every sweep.
    const int wv = tid >> 6;
    const int slot = (tid >> 2) & 15;   // which of the wave's 16 pairs
    const int sub = tid & 3;            // which quarter of the rows (interleaved float4 groups)
    float max_cos2 = 0.f;
    if (tid < kD) sm.dsc[tid] = 1.f;
    auto fold_scales = [&](bool with_norms) {       // between two barriers
        if (tid < kD) {
            float4* col = reinterpret_cast<float4*>(sm.A + tid * kLd);
            const float d = sm.dsc[tid];
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll 8
            for (int i = 0; i < kD / 4; ++i) {
                float4 v = col[i];
                v.x *= d; v.y *= d; v.z *= d; v.w *= d;
                col[i] = v;
                acc0 += v.x * v.x + v.y * v.y;
                acc1 += v.z * v.z + v.w * v.w;
            }
            sm.dsc[tid] = 1.f;
            if (with_norms) sm.n2[tid] = acc0 + acc1;
        }
    };
    auto rotate_pair = [&](int p, int q) {
        float4* cp = reinterpret_cast<float4*>(sm.A + p * kLd);
        float4* cq = reinterpret_cast<float4*>(sm.A + q * kLd);
        float4 ap[8], aq[8];
        float ga[2] = {0.f, 0.f};
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            ap[v] = cp[4 * v + sub];
            aq[v] = cq[4 * v + sub];
        }
        const float dp = sm.dsc[p], dq = sm.dsc[q];
        const float alpha = sm.n2[p], beta = sm.n2[q];
#pragma unroll
        for (int v = 0; v < 8; ++v)
            ga[v & 1] += ap[v].x * aq[v].x + ap[v].y * aq[v].y + ap[v].z * aq[v].z + ap[v].w * aq[v].w;
        const float gamma = quad_sum(ga[0] + ga[1]) * (dp * dq);
        const float ab = alpha * beta;
        const float g2 = gamma * gamma;
        if (ab > 0.f && g2 > 1e-14f * ab) {            // same decision in all four lanes
            max_cos2 = fmaxf(max_cos2, g2 * __builtin_amdgcn_rcpf(ab));
            // tan of the rotation angle: smaller root of t^2 + 2 zeta t - 1 = 0
            const float zeta = (beta - alpha) * __builtin_amdgcn_rcpf(2.f * gamma);
            const float t = copysignf(1.f, zeta) *
                            __builtin_amdgcn_rcpf(fabsf(zeta) + __builtin_amdgcn_sqrtf(fmaf(zeta, zeta, 1.f)));
            const float c = __builtin_amdgcn_rsqf(fmaf(t, t, 1.f));
            const float ratio = dq * __builtin_amdgcn_rcpf(dp);
            const float tp = -t * ratio, tq = t * __builtin_amdgcn_rcpf(ratio);
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                float4 np, nq;
                np.x = fmaf(tp, aq[v].x, ap[v].x);  nq.x = fmaf(tq, ap[v].x, aq[v].x);
                np.y = fmaf(tp, aq[v].y, ap[v].y);  nq.y = fmaf(tq, ap[v].y, aq[v].y);
                np.z = fmaf(tp, aq[v].z, ap[v].z);  nq.z = fmaf(tq, ap[v].z, aq[v].z);
                np.w = fmaf(tp, aq[v].w, ap[v].w);  nq.w = fmaf(tq, ap[v].w, aq[v].w);
                cp[4 * v + sub] = np;
                cq[4 * v + sub] = nq;
            }
            if (sub == 0) {
                const float tg = t * gamma;
                sm.dsc[p] = dp * c;
                sm.dsc[q] = dq * c;
                sm.n2[p] = fmaxf(alpha - tg, 0.f);
                sm.n2[q] = beta + tg;
            }
        }
        // the wave's own LDS traffic is ordered; keep the compiler from moving it
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        max_cos2 = 0.f;
        __syncthreads();
        fold_scales(true);
        __syncthreads();
        // pairs inside half-blocks 2wv and 2wv+1: round-robin over 16 columns, 8 pairs each
        {
            const int hb = 2 * wv + (slot >> 3), k = slot & 7;
            for (int t = 0; t < 15; ++t) {
                int i, j;
                if (k == 0) {
                    i = 15;
                    j = t;
                } else {
                    i = t + k;
                    if (i >= 15) i -= 15;
                    j = t - k;
                    if (j < 0) j += 15;
                }
                rotate_pair(16 * hb + i, 16 * hb + j);
            }
        }
        // cross pairs: round-robin over the 8 half-blocks, one pair of half-blocks (X, Y) per
        // wave.  The 32 columns stay in registers for the 16 rounds of the block: lane
        // (k = lane%16, s = lane/16) holds quarter s of column X[k] and of one Y column; after
        // every round the Y slices (with their scale and norm) move one lane along their row of
        // 16, so lane k meets every Y column once and after 16 moves each is back where it
        // started.  No LDS traffic or barrier inside a block.
        __syncthreads();
        fold_scales(false);
        for (int br = 0; br < 7; ++br) {
            __syncthreads();
            int X, Y;
            if (wv == 0) {
                X = 7;
                Y = br;
            } else {
                X = br + wv;
                if (X >= 7) X -= 7;
                Y = br - wv;
                if (Y < 0) Y += 7;
            }
            const int k = tid & 15, s4 = (tid >> 4) & 3;
            const int px = 16 * X + k, py = 16 * Y + k;
            float4* cx = reinterpret_cast<float4*>(sm.A + px * kLd);
            float4* cy = reinterpret_cast<float4*>(sm.A + py * kLd);
            float4 xa[8], ya[8];
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                xa[v] = cx[4 * v + s4];
                ya[v] = cy[4 * v + s4];
            }
            float nx = sm.n2[px], ny = sm.n2[py], dx = 1.f, dy = 1.f;
            for (int t = 0; t < 16; ++t) {
                float ga[2] = {0.f, 0.f};
#pragma unroll
                for (int v = 0; v < 8; ++v)
                    ga[v & 1] += xa[v].x * ya[v].x + xa[v].y * ya[v].y + xa[v].z * ya[v].z + xa[v].w * ya[v].w;
                const float gamma = rows_allreduce(ga[0] + ga[1]) * (dx * dy);
                const float ab = nx * ny;
                const float g2 = gamma * gamma;
                if (ab > 0.f && g2 > 1e-14f * ab) {        // same decision in the four lanes of a pair
                    max_cos2 = fmaxf(max_cos2, g2 * __builtin_amdgcn_rcpf(ab));
                    const float zeta = (ny - nx) * __builtin_amdgcn_rcpf(2.f * gamma);
                    const float tn = copysignf(1.f, zeta) *
                                     __builtin_amdgcn_rcpf(fabsf(zeta) + __builtin_amdgcn_sqrtf(fmaf(zeta, zeta, 1.f)));
                    const float c = __builtin_amdgcn_rsqf(fmaf(tn, tn, 1.f));
                    const float ratio = dy * __builtin_amdgcn_rcpf(dx);
                    const float tp = -tn * ratio, tq = tn * __builtin_amdgcn_rcpf(ratio);
#pragma unroll
                    for (int v = 0; v < 8; ++v) {
                        const float4 ox = xa[v], oy = ya[v];
                        xa[v].x = fmaf(tp, oy.x, ox.x);  ya[v].x = fmaf(tq, ox.x, oy.x);
                        xa[v].y = fmaf(tp, oy.y, ox.y);  ya[v].y = fmaf(tq, ox.y, oy.y);
                        xa[v].z = fmaf(tp, oy.z, ox.z);  ya[v].z = fmaf(tq, ox.z, oy.z);
                        xa[v].w = fmaf(tp, oy.w, ox.w);  ya[v].w = fmaf(tq, ox.w, oy.w);
                    }
                    const float tg = tn * gamma;
                    dx *= c;
                    dy *= c;
                    nx = fmaxf(nx - tg, 0.f);
                    ny += tg;
                }
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    ya[v].x = row_rotate(ya[v].x);
                    ya[v].y = row_rotate(ya[v].y);
                    ya[v].z = row_rotate(ya[v].z);
                    ya[v].w = row_rotate(ya[v].w);
                }
                dy = row_rotate(dy);
                ny = row_rotate(ny);
            }
            // scales folded in on the way back; every Y slice is home again after 16 moves
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                cx[4 * v + s4] = make_float4(xa[v].x * dx, xa[v].y * dx, xa[v].z * dx, xa[v].w * dx);
                cy[4 * v + s4] = make_float4(ya[v].x * dy, ya[v].y * dy, ya[v].z * dy, ya[v].w * dy);
            }
            if (s4 == 0) {
                sm.n2[px] = nx;
                sm.n2[py] = ny;
            }
        }
        // every thread learns the sweep's largest cos^2
        max_cos2 = wave_max(max_cos2);
        if ((tid & 63) == 0) sm.flag[tid >> 6] = max_cos2;
        __syncthreads();
        const float mc = fmaxf(fmaxf(sm.flag[0], sm.flag[1]), fmaxf(sm.flag[2], sm.flag[3]));
        __syncthreads();
        if (mc < kStopCos2) break;
    }
    fold_scales(false);
    __syncthreads();

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
    if (eig_out != nullptr && tid < eig_ld)        // eig_ld values per matrix: all 128, or the leading 64 of a 64-wide input
        eig_out[(int64_t)m * eig_ld + tid] = total > 0.0 ? (float)(mine / total) : 0.f;
}

hipError_t launch_jacobi_entropy(int n_mat, int N, int k_trunc, unsigned flags,
                                 const EntropyPlan& p, char* ws, float* entropy_out,
                                 float* eig_out, const Env& env, int eig_ld) {
    hipStream_t s = env.s;
    static_assert(sizeof(Smem) <= 160 * 1024, "LDS budget");
    const float* gram = reinterpret_cast<const float*>(ws + p.gram_off);
    const float* sums = reinterpret_cast<const float*>(ws + p.sum_off);
    env.begin("jacobi_entropy");
    jacobi_entropy_kernel<<<dim3(n_mat), dim3(kThreads), sizeof(Smem), s>>>(
        gram, sums, p.n_chunks, N, k_trunc, flags, entropy_out, eig_out, eig_ld);
    env.end();
    return hipGetLastError();
}

hipError_t init_jacobi_kernels() {
    return allow_dynamic_lds(reinterpret_cast<const void*>(jacobi_entropy_kernel), sizeof(Smem));
}

}  // namespace uncomp
