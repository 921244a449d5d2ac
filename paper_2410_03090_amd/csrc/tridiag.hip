// Eigen stage of the truncated matrix entropy (Lemma 2: entropy from the eigenvalues of
// the covariance; Sec. 3.2 Eq. 5: only the k largest enter; proof of Lemma 4: unit trace),
// by Householder tridiagonalisation and Sturm-sequence multisection, all in fp64.
//
// One workgroup of 256 threads per matrix:
//   1. add the Gram partials of the matrix in fp64, subtract the mean term s s^T / N
//      (Eq. 1; the common factor 1/(N-1) drops out under the unit-trace scaling) and divide
//      by the trace.  The matrix lives in registers: thread (c, hf) holds rows 64*hf .. +64
//      of column c as 64 doubles.
//   2. 126 Householder reflections H = I - beta v v^T bring it to tridiagonal form
//      (A <- A - v w^T - w v^T with p = beta A v, w = p - (beta/2)(v^T p) v).  Per reflection:
//      the pivot row was left in LDS by the previous update, every wave forms the norm of its
//      tail on its own (identical bits in all waves, so the whole workgroup takes the same
//      branch), a matrix-vector product with v read from LDS at wave-uniform addresses, one
//      exchange of the two row halves, every wave forms v^T A v on its own, and the rank-2
//      update; three workgroup barriers.  Rows that are already done are skipped by uniform
//      branches; no register is ever indexed dynamically.
//   3. The eigenvalues of the tridiagonal matrix (d, e) are found by counting sign changes of
//      the characteristic-polynomial recurrence p_i = (d_i - x) p_{i-1} - e_{i-1}^2 p_{i-2}
//      (= number of eigenvalues below x; no division, rescaled against underflow): every
//      wanted eigenvalue owns a group of L lanes that cut its bracket into L+1 pieces per
//      round (ballot + count-trailing-zeros picks the piece).  Brackets start at
//      [0, 1 + 2^-10]: the matrix has unit trace and is positive semi-definite up to rounding,
//      and an eigenvalue that rounding pushed below zero is reported as zero, which is what
//      the definition asks for.  Only the k largest are computed unless the caller wants the
//      whole spectrum.
//   4. truncated entropy in fp64.
#include "common.h"
#include "device_utils.h"

namespace uncomp {

namespace {

// The kernel comes in two shapes.  kParts = 4: 512 threads per matrix, 32 rows of a column per
// thread, two waves per SIMD from the one matrix a CU works on (a launch with fewer matrices
// than the chip can hold two per CU).  kParts = 2: 256 threads, 64 rows per thread, registers
// capped so that two matrices share a CU and fill each other's waits (large launches).

template <int kParts>
struct TriSmem {
    double s[kD];            // column sums of X (for the mean correction)
    double red[8];
    double xbuf[kD];         // pivot row i, entries at columns <= i zeroed
    double ybuf[kD];         // row i + 1
    double pbuf[kParts][kD]; // the row slices of A x
    double2 vw[kD];          // (v_r, w_r)
    double2 de[kD];          // (d_i, e_{i-1}^2), e_{-1} = 0
    double lam[kD];          // eigenvalues, descending
};

template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes, delivered to every lane with identical bits: rotations inside the
// rows of 16 lanes (DPP row_ror 8, 4, 2, 1), then the four rows with
// v_permlane32_swap(a,b) -> ([a.lo32, b.lo32], [a.hi32, b.hi32]) and
// v_permlane16_swap(a,b) -> ([a.r0, b.r0, a.r2, b.r2], [a.r1, b.r1, a.r3, b.r3]).
__device__ __forceinline__ double wave_allsum(double v) {
    v += dpp_move<0x128>(v);
    v += dpp_move<0x124>(v);
    v += dpp_move<0x122>(v);
    v += dpp_move<0x121>(v);
    {
        const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
        auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        v = __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
    }
    {
        const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
        auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        v = __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
    }
    return v;
}

template <int kWaves>
__device__ __forceinline__ double block_sum(double v, double* red, int tid) {
    v = wave_allsum(v);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    double t = red[0];
#pragma unroll
    for (int x = 1; x < kWaves; ++x) t += red[x];
    return t;
}

// Number of eigenvalues of the tridiagonal matrix below x: sign changes along
// 1, p_0, p_1, ..., p_{n-1} (a zero takes the sign '+', which gives the same total as the
// textbook rule because the next term then has the opposite sign of the previous one).
// The (d_i, e_{i-1}^2) pairs come from LDS eight at a time, the next eight requested before
// the current eight are used.
__device__ __forceinline__ int sturm_count(const double2* de, double x) {
    double pp = 0.0, p = 1.0;                      // p_{-2}, p_{-1}
    int cnt = 0;
    double2 cur[8], nxt[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) cur[u] = de[u];
#pragma clang loop unroll(disable)
    for (int base = 0; base < kD; base += 8) {
        const int nb = base + 8 < kD ? base + 8 : base;          // the last prefetch re-reads its own chunk
#pragma unroll
        for (int u = 0; u < 8; ++u) nxt[u] = de[nb + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const double pn = fma(cur[u].x - x, p, -(cur[u].y * pp));
            cnt += (int)((unsigned)(__double2hiint(pn) ^ __double2hiint(p)) >> 31);
            pp = p;
            p = pn;
        }
        // |p| shrinks by at most ~2^-35 per step and grows by at most 1.25: keep it normal
        const double sc = fabs(p) < 0x1p-300 ? 0x1p300 : 1.0;
        p *= sc;
        pp *= sc;
#pragma unroll
        for (int u = 0; u < 8; ++u) cur[u] = nxt[u];
    }
    return cnt;
}

}  // namespace

template <int kParts>
__global__ __launch_bounds__(kD * kParts, kParts == 2 ? 2 : 1) void tridiag_entropy_kernel(
    const float* __restrict__ gram_part, const float* __restrict__ sum_part, int n_chunks, int N,
    int k_trunc, unsigned flags, float* __restrict__ entropy_out, float* __restrict__ eig_out, int eig_ld,
    const double* __restrict__ trace_total) {
    constexpr int kThreads = kD * kParts, kWaves = kThreads / 64;
    constexpr int kHalf = kD / kParts;                           // rows of a column per thread
    __shared__ TriSmem<kParts> sm;
    const int m = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int c = tid & (kD - 1);
    const int hf = __builtin_amdgcn_readfirstlane(tid >> 7);     // wave-uniform: which slice of rows
    const int col_hi = __builtin_amdgcn_readfirstlane(c | 63);   // last column of this wave
    const float* Gm = gram_part + (int64_t)m * n_chunks * (kD * kD);
    const float* Sm = sum_part + (int64_t)m * n_chunks * kD;

    // ---- 1. reduce partials, centre, unit trace ------------------------------------------
    if (tid < kD) {
        double acc = 0.0;
        for (int ch = 0; ch < n_chunks; ++ch) acc += (double)Sm[ch * kD + tid];
        sm.s[tid] = acc;
    }
    __syncthreads();
    const bool center = (flags & UNCOMP_CENTER) != 0;
    const double inv_n = 1.0 / (double)N;
    double tr_c = 0.0, tr_u = 0.0;
    if (tid < kD) {
        double acc = 0.0;
        for (int ch = 0; ch < n_chunks; ++ch) acc += (double)Gm[(int64_t)ch * (kD * kD) + tid * (kD + 1)];
        tr_u = acc;
        tr_c = center ? acc - sm.s[tid] * sm.s[tid] * inv_n : acc;
    }
    const double trace = block_sum<kWaves>(tr_c, sm.red, tid);
    const double trace_u = block_sum<kWaves>(tr_u, sm.red, tid);
    // Zero spread: a single token, or a centred trace so far below the second moment that
    // the fp32 partial sums cannot tell it from zero.
    bool degenerate = !(trace > 0.0) || (center && (N < 2 || trace < trace_u * 0x1p-20));
    // A projection of a larger matrix: the verdict comes from the larger matrix' own traces
    // (centred, uncentred; accumulated in fp64), the projection of a constant matrix being noise.
    double whole_raw = 0.0;
    if (trace_total != nullptr) {
        whole_raw = center ? trace_total[0] : trace_total[1];
        degenerate = degenerate || !(whole_raw > 0.0) || (center && whole_raw < trace_total[1] * 0x1p-30);
    }
    if (degenerate) {
        if (tid == 0) entropy_out[m] = 0.f;
        if (eig_out != nullptr && tid < eig_ld) eig_out[(int64_t)m * eig_ld + tid] = 0.f;
        return;
    }
    double a[kHalf];                                             // a[k] = A[64 hf + k][c]
#pragma unroll
    for (int k = 0; k < kHalf; ++k) a[k] = 0.0;
    for (int ch = 0; ch < n_chunks; ++ch) {
        const float* g = Gm + (int64_t)ch * (kD * kD) + (hf * kHalf) * kD + c;
#pragma unroll
        for (int kb = 0; kb < kHalf; kb += 16) {                 // 16 independent loads in flight
            float t[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) t[u] = g[(kb + u) * kD];
#pragma unroll
            for (int u = 0; u < 16; ++u) a[kb + u] += (double)t[u];
        }
    }
    {
        const double inv_tr = 1.0 / trace;
        const double sc = center ? sm.s[c] * inv_n : 0.0;
#pragma unroll
        for (int k = 0; k < kHalf; ++k) a[k] = (a[k] - sm.s[hf * kHalf + k] * sc) * inv_tr;
    }

    // ---- 2. Householder tridiagonalisation ---------------------------------------------------
    // Leaves rows `row` and `row + 1` of the matrix in LDS for the next reflection: row `row` in
    // xbuf with the entries at columns <= row zeroed (its diagonal entry goes to de[row].x), row
    // `row + 1` in ybuf.  A row is held by the 128 threads of one half in a register whose number
    // depends on the row; a switch on that (wave-uniform) number reaches it without indexing.
#define UNCOMP_TRI_CASE(K)                                                      \
    case K:                                                                     \
        if constexpr (K < kHalf) {                                              \
            sm.xbuf[c] = c > row ? a[K] : 0.0;                                  \
            if (c == row) sm.de[row].x = a[K];                                  \
            if (K + 1 < kHalf) sm.ybuf[c] = a[K + 1 < kHalf ? K + 1 : K];       \
        }                                                                       \
        break;
#define UNCOMP_TRI_CASE8(K)                                                                          \
    UNCOMP_TRI_CASE(K) UNCOMP_TRI_CASE(K + 1) UNCOMP_TRI_CASE(K + 2) UNCOMP_TRI_CASE(K + 3)          \
    UNCOMP_TRI_CASE(K + 4) UNCOMP_TRI_CASE(K + 5) UNCOMP_TRI_CASE(K + 6) UNCOMP_TRI_CASE(K + 7)
    auto publish2 = [&](int row) {
        switch (row - hf * kHalf) {
            case -1:                                             // row + 1 is the first row of this half
                sm.ybuf[c] = a[0];
                break;
            UNCOMP_TRI_CASE8(0) UNCOMP_TRI_CASE8(8) UNCOMP_TRI_CASE8(16) UNCOMP_TRI_CASE8(24)
            UNCOMP_TRI_CASE8(32) UNCOMP_TRI_CASE8(40) UNCOMP_TRI_CASE8(48) UNCOMP_TRI_CASE8(56)
            default:
                break;
        }
    };
#undef UNCOMP_TRI_CASE8
#undef UNCOMP_TRI_CASE
    publish2(0);
    for (int i = 0; i < kD - 2; ++i) {
        __syncthreads();                                         // xbuf = row i (masked), ybuf = row i + 1
        const double x1 = sm.xbuf[i + 1];
        const double xa = lane > i + 1 ? sm.xbuf[lane] : 0.0;
        const double xb = lane + 64 > i + 1 ? sm.xbuf[lane + 64] : 0.0;
        // This thread's part of (A x)_c over the rows of its half (x is zero on the rows that are
        // done).  It does not depend on the reflection's scalars, so it runs beside their reduction.
        double p0 = 0.0, p1 = 0.0, p2 = 0.0, p3 = 0.0;
        // rows of this slice still in play, and columns of this wave still in play (both wave-uniform)
        const bool half_live = hf * kHalf + kHalf - 1 > i && col_hi > i;
        if (half_live) {
#pragma unroll
            for (int k = 0; k < kHalf; k += 4) {
                const double2 xv0 = *reinterpret_cast<const double2*>(&sm.xbuf[hf * kHalf + k]);
                const double2 xv1 = *reinterpret_cast<const double2*>(&sm.xbuf[hf * kHalf + k + 2]);
                p0 = fma(a[k], xv0.x, p0);
                p1 = fma(a[k + 1], xv0.y, p1);
                p2 = fma(a[k + 2], xv1.x, p2);
                p3 = fma(a[k + 3], xv1.y, p3);
            }
        }
        const double tail = wave_allsum(xa * xa + xb * xb);      // sum_{r > i+1} x_r^2, same bits in every wave
        if (tail == 0.0) {
            // the column is already in tridiagonal form: nothing to reflect
            if (tid == 0) sm.de[i + 1].y = x1 * x1;
            __syncthreads();                                     // both rows read by all before they are replaced
        } else {
            // v = x - alpha e_{i+1};  A v = A x - alpha (row i + 1)
            const double sigma = tail + x1 * x1;
            const double nrm = sqrt(sigma);
            const double alpha = x1 >= 0.0 ? -nrm : nrm;
            const double den = sigma - alpha * x1;               // = sigma + |x1| sqrt(sigma) > 0
            double beta = __builtin_amdgcn_rcp(den);
            beta = fma(fma(-den, beta, 1.0), beta, beta);        // two Newton steps on the hardware estimate
            beta = fma(fma(-den, beta, 1.0), beta, beta);
            if (tid == 0) sm.de[i + 1].y = sigma;                // e_i^2 = alpha^2
            sm.pbuf[hf][c] = (p0 + p1) + (p2 + p3);
            __syncthreads();
            auto v_of = [&](int r) { return sm.xbuf[r] - (r == i + 1 ? alpha : 0.0); };
            auto Av_of = [&](int r) {
                double t = sm.pbuf[0][r];
#pragma unroll
                for (int x = 1; x < kParts; ++x) t += sm.pbuf[x][r];
                return t - alpha * sm.ybuf[r];
            };
            const double vAv = wave_allsum(v_of(lane) * Av_of(lane) + v_of(lane + 64) * Av_of(lane + 64));
            const double K = 0.5 * beta * beta * vAv;
            const double vc = v_of(c);
            const double wc = c > i ? beta * Av_of(c) - K * vc : 0.0;
            if (hf == 0) sm.vw[c] = make_double2(vc, wc);
            __syncthreads();
            if (half_live) {
#pragma unroll
                for (int k = 0; k < kHalf; ++k) {
                    const double2 t = sm.vw[hf * kHalf + k];
                    a[k] = fma(-t.x, wc, fma(-t.y, vc, a[k]));
                }
            }
        }
        publish2(i + 1);
    }
    __syncthreads();                                             // xbuf = row 126 (masked)
    if (tid == 0) {
        sm.de[kD - 1].y = sm.xbuf[kD - 1] * sm.xbuf[kD - 1];
        sm.de[0].y = 0.0;
    }
    if (tid == kThreads - 1) sm.de[kD - 1].x = a[kHalf - 1];
    if (tid < kD) sm.lam[tid] = 0.0;
    __syncthreads();

    // ---- 3. eigenvalues by multisection on the Sturm count ------------------------------------
    const int k = k_trunc < kD ? k_trunc : kD;
    const int n_need = eig_out != nullptr ? kD : k;
    // lanes per eigenvalue: as many as the workgroup can give every wanted eigenvalue
    const int L = kThreads / 16 >= n_need ? 16 : (kThreads / 8 >= n_need ? 8 : (kThreads / 4 >= n_need ? 4 : 2));
    const int rounds = L == 16 ? 8 : (L == 8 ? 10 : (L == 4 ? 14 : 20));           // (L+1)^rounds >= 2^31
    {
        const int q = tid / L, s = tid % L;                      // eigenvalue q (0 = largest), piece s
        const int j = kD - 1 - q;                                // its index in ascending order
        const double inv = 1.0 / (double)(L + 1);
        double lo = 0.0, hi = 1.0 + 0x1p-10;
        for (int it = 0; it < rounds; ++it) {
            const double step = (hi - lo) * inv;
            const int cnt = sturm_count(sm.de, lo + step * (double)(s + 1));
            const unsigned long long mask = __ballot(cnt > j);
            const unsigned bits = (unsigned)(mask >> (lane - s)) & ((1u << L) - 1u);
            const int piece = bits ? __builtin_ctz(bits) : L;    // first cut with more than j eigenvalues below it
            const double nlo = lo + step * (double)piece;
            hi = piece == L ? hi : lo + step * (double)(piece + 1);
            lo = nlo;
        }
        if (s == 0 && q < n_need) {
            const double v = 0.5 * (lo + hi);
            sm.lam[q] = v > 0.0 ? v : 0.0;
        }
    }
    __syncthreads();

    // ---- 4. entropy --------------------------------------------------------------------------
    const double mine = tid < kD ? sm.lam[tid] : 0.0;
    const double total = block_sum<kWaves>(tid < kD ? sm.de[tid].x : 0.0, sm.red, tid);   // the trace: sum of all eigenvalues
    const double topk = block_sum<kWaves>(tid < k ? mine : 0.0, sm.red, tid);
    // total = 1 up to rounding (the matrix was scaled to unit trace).  When the matrix is a projection
    // of a larger one, the eigenvalues' share of the larger trace is what Eq. 5 and eig_out mean.
    const double whole = trace_total != nullptr ? total * (whole_raw / trace) : total;
    const double denom = (flags & UNCOMP_TRUNC_RENORM) ? topk : whole;
    double term = 0.0;
    if (tid < k && mine > 0.0 && denom > 0.0) {
        const double sgm = mine / denom;
        term = -sgm * log(sgm);
    }
    const double H = block_sum<kWaves>(term, sm.red, tid);
    if (tid == 0) entropy_out[m] = (float)H;
    if (eig_out != nullptr && tid < eig_ld)        // eig_ld values per matrix: all 128, or the leading 64 of a 64-wide input
        eig_out[(int64_t)m * eig_ld + tid] = whole > 0.0 ? (float)(mine / whole) : 0.f;
}

hipError_t launch_tridiag_entropy(int n_mat, int N, int k_trunc, unsigned flags, const EntropyPlan& p,
                                  char* ws, float* entropy_out, float* eig_out, const Env& env,
                                  const double* trace_total, int eig_ld) {
    const float* gram = reinterpret_cast<const float*>(ws + p.gram_off);
    const float* sums = reinterpret_cast<const float*>(ws + p.sum_off);
    env.begin("tridiag_entropy");
    if (n_mat < 512)
        tridiag_entropy_kernel<4><<<dim3(n_mat), dim3(4 * kD), 0, env.s>>>(gram, sums, p.n_chunks, N, k_trunc, flags,
                                                                         entropy_out, eig_out, eig_ld, trace_total);
    else
        tridiag_entropy_kernel<2><<<dim3(n_mat), dim3(2 * kD), 0, env.s>>>(gram, sums, p.n_chunks, N, k_trunc, flags,
                                                                         entropy_out, eig_out, eig_ld, trace_total);
    env.end();
    return hipGetLastError();
}

}  // namespace uncomp
