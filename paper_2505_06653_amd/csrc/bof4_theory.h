// bof4_theory.h - theoretical (data-free) MSE centroids for a tabulated symmetric weight distribution.
//
// Section 3.2 eq. 5 (the boxed general centroid of appendix B.2) with the conditional expectation of the appendix's
// "Expectation of Normalized Weights" and p_M, F_X of appendix B.1 substituted; the factors common to numerator and
// denominator cancelled:
//     level(l) = INT m [Phi1(m x)]_a^b A(m)^(I-2) p_W(m) dm  /  INT m^2 [F_W(m x)]_a^b A(m)^(I-2) p_W(m) dm,
// a, b the region's thresholds, A = 2 F_W - 1, Phi1(t) = INT_-inf^t u p_W(u) du = -Psi(|t|), Psi(t) = INT_t^inf u p_W.
// p_W and F_W come as tables on a uniform grid over [0, u_max]; Psi is made from p_W by the trapezoid rule, values
// between grid points by linear interpolation, the integrals over m by the composite Simpson rule on the same grid.
// This is a small quadrature (16 x n evaluations), not a streaming pass: one workgroup per level.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace bof4 {

// Psi[k] = sum over the segments from k on of h/2 (u_i p_i + u_{i+1} p_{i+1}); one workgroup, any n.
__global__ __launch_bounds__(1024) void theory_psi_kernel(const double* __restrict__ pdf, uint32_t n, double h,
                                                          double* __restrict__ psi) {
    __shared__ double chunk_sum[1024];
    const uint32_t tid = threadIdx.x, n_seg = n - 1;
    const uint32_t per = (n_seg + 1023) / 1024;
    const uint32_t s0 = tid * per, s1 = (s0 + per < n_seg) ? s0 + per : n_seg;
    double sum = 0.0;
    for (uint32_t i = s0; i < s1; ++i)
        sum += 0.5 * h * ((double)i * h * pdf[i] + (double)(i + 1) * h * pdf[i + 1]);
    chunk_sum[tid] = s0 < n_seg ? sum : 0.0;
    __syncthreads();
    double behind = 0.0;  // the chunks after this one
    for (uint32_t c = 1023; c > tid; --c) behind += chunk_sum[c];
    // suffix sums inside the chunk, from its end
    double run = behind;
    for (uint32_t i = s1; i > s0; --i) {
        run += 0.5 * h * ((double)(i - 1) * h * pdf[i - 1] + (double)i * h * pdf[i]);
        psi[i - 1] = run;
    }
    if (tid == 0) psi[n - 1] = 0.0;
}

__device__ __forceinline__ double table_at(const double* __restrict__ t, uint32_t n, double pos) {
    uint32_t k = (uint32_t)pos;
    if (k > n - 2) k = n - 2;
    const double fr = pos - (double)k;
    return t[k] + fr * (t[k + 1] - t[k]);
}

struct TheoryRegions {
    double a[16], b[16];  // thresholds of every level's region
    uint32_t skip_mask;   // pinned levels
};

// One workgroup per level: Simpson sums of the two integrands, reduced in a fixed order.
__global__ __launch_bounds__(256) void theory_centroid_kernel(const double* __restrict__ pdf,
                                                              const double* __restrict__ cdf,
                                                              const double* __restrict__ psi, uint32_t n, double h,
                                                              uint32_t block, TheoryRegions rg,
                                                              double* __restrict__ out /* [16][2]: num, den */) {
    __shared__ double red[2][256];
    const uint32_t l = blockIdx.x, tid = threadIdx.x;
    double num = 0.0, den = 0.0;
    if (!((rg.skip_mask >> l) & 1u)) {
        const double a = rg.a[l], b = rg.b[l];
        const double inv_h = 1.0 / h;
        for (uint32_t j = 1 + tid; j < n; j += 256) {  // the term at m = 0 vanishes
            const double m = (double)j * h;
            const double wS = (j == n - 1 ? 1.0 : (j & 1u) ? 4.0 : 2.0) * (h / 3.0);
            const double core = pow(2.0 * cdf[j] - 1.0, (double)(block - 2)) * pdf[j];
            const double pa = fabs(a) * m * inv_h, pb = fabs(b) * m * inv_h;  // positions of |m a|, |m b| in the tables
            const double Fa = a < 0.0 ? 1.0 - table_at(cdf, n, pa) : table_at(cdf, n, pa);
            const double Fb = b < 0.0 ? 1.0 - table_at(cdf, n, pb) : table_at(cdf, n, pb);
            const double dPhi = table_at(psi, n, pa) - table_at(psi, n, pb);  // Phi1(m b) - Phi1(m a), Phi1 = -Psi
            num += wS * m * dPhi * core;
            den += wS * m * m * (Fb - Fa) * core;
        }
    }
    red[0][tid] = num;
    red[1][tid] = den;
    __syncthreads();
    for (uint32_t s = 128; s >= 1; s >>= 1) {
        if (tid < s) {
            red[0][tid] += red[0][tid + s];
            red[1][tid] += red[1][tid + s];
        }
        __syncthreads();
    }
    if (tid == 0) {
        out[2 * l] = red[0][0];
        out[2 * l + 1] = red[1][0];
    }
}

}  // namespace bof4
