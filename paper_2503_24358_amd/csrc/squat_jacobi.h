// One-sided (Hestenes) Jacobi on the ROWS of a symmetric positive semi-definite
// n x n matrix held in LDS in fp64, used for the eigen-decomposition behind
// Qhat (Section 3.2 of the paper: top singular vectors of the prompt queries)
// and for the small r x r systems of the update matrix.
//
// Rotating rows p, q of A = G until all rows are mutually orthogonal leaves
// row i = lambda_i * v_i^T with (lambda_i, v_i) an eigenpair of G: the row
// norms are the eigenvalues and the normalised rows the eigenvectors, so no
// separate eigenvector matrix is kept.  Pairs follow a round-robin tournament
// (n - 1 rounds of n / 2 disjoint pairs), one team of lanes per pair.
#pragma once

#include <hip/hip_runtime.h>

namespace squat {

// Team-wide sum over TS consecutive lanes (TS a power of two <= 64).
template <int TS>
__device__ __forceinline__ double team_sum(double v) {
#pragma unroll
    for (int off = TS >> 1; off > 0; off >>= 1) v += __shfl_xor(v, off, TS);
    return v;
}

// A: n x n row-major with leading dimension ld (doubles) in LDS; n even, n/2 * TS <= THREADS.
// `flag` is one int in LDS.  Returns the number of sweeps done.  All threads of the block
// must call it.
template <int THREADS, int TS>
__device__ int jacobi_rows(double* A, int n, int ld, int* flag, int max_sweeps, double tol) {
    const int tid = threadIdx.x;
    const int team = tid / TS;
    const int tl = tid % TS;
    const int pairs = n >> 1;
    const int m = n - 1;
    int sweep = 0;
    for (; sweep < max_sweeps; ++sweep) {
        if (tid == 0) *flag = 0;
        __syncthreads();
        for (int round = 0; round < m; ++round) {
            if (team < pairs) {
                int p, q;
                if (team == 0) {
                    p = m;
                    q = round;
                } else {
                    p = (round + team) % m;
                    q = (round - team + m) % m;
                }
                double* x = A + p * ld;
                double* y = A + q * ld;
                double al = 0.0, be = 0.0, ga = 0.0;
                for (int c = tl; c < n; c += TS) {
                    const double xv = x[c], yv = y[c];
                    al += xv * xv;
                    be += yv * yv;
                    ga += xv * yv;
                }
                al = team_sum<TS>(al);
                be = team_sum<TS>(be);
                ga = team_sum<TS>(ga);
                if (fabs(ga) > tol * sqrt(al * be) && ga != 0.0) {
                    const double zeta = (be - al) / (2.0 * ga);
                    const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    const double cs = 1.0 / sqrt(1.0 + t * t);
                    const double sn = cs * t;
                    for (int c = tl; c < n; c += TS) {
                        const double xv = x[c], yv = y[c];
                        x[c] = cs * xv - sn * yv;
                        y[c] = sn * xv + cs * yv;
                    }
                    if (tl == 0) *flag = 1;
                }
            }
            __syncthreads();
        }
        const int any = *flag;
        __syncthreads();
        if (!any) {
            ++sweep;
            break;
        }
    }
    return sweep;
}

}  // namespace squat
