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
//
// Cost per round is kept low in three ways: squared row norms are cached and
// updated algebraically (one dot product per pair instead of three, refreshed
// from scratch every sweep); the rotation angle is computed in fp32 (any angle
// gives an exactly orthogonal rotation; its accuracy only sets how completely
// one rotation annihilates the pair, and later sweeps finish the job), while
// cos/sin are normalised in fp64 by Newton steps; team reductions use DPP
// moves instead of LDS permutes.
#pragma once

#include <hip/hip_runtime.h>

namespace squat {

__device__ __forceinline__ double dpp_move(double v, int ctrl_sel) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    switch (ctrl_sel) {
        case 0:  // quad_perm [1,0,3,2]
            lo = __builtin_amdgcn_mov_dpp(lo, 0xB1, 0xF, 0xF, true);
            hi = __builtin_amdgcn_mov_dpp(hi, 0xB1, 0xF, 0xF, true);
            break;
        case 1:  // quad_perm [2,3,0,1]
            lo = __builtin_amdgcn_mov_dpp(lo, 0x4E, 0xF, 0xF, true);
            hi = __builtin_amdgcn_mov_dpp(hi, 0x4E, 0xF, 0xF, true);
            break;
        case 2:  // row_half_mirror
            lo = __builtin_amdgcn_mov_dpp(lo, 0x141, 0xF, 0xF, true);
            hi = __builtin_amdgcn_mov_dpp(hi, 0x141, 0xF, 0xF, true);
            break;
        default:  // row_mirror
            lo = __builtin_amdgcn_mov_dpp(lo, 0x140, 0xF, 0xF, true);
            hi = __builtin_amdgcn_mov_dpp(hi, 0x140, 0xF, 0xF, true);
            break;
    }
    return __hiloint2double(hi, lo);
}

// Sum over TS consecutive lanes (TS a power of two <= 64, teams aligned); every lane gets the total.
template <int TS>
__device__ __forceinline__ double team_sum(double v) {
    if constexpr (TS >= 2) v += dpp_move(v, 0);
    if constexpr (TS >= 4) v += dpp_move(v, 1);
    if constexpr (TS >= 8) v += dpp_move(v, 2);     // partner quad of the same half-row holds the other sum
    if constexpr (TS >= 16) v += dpp_move(v, 3);    // partner half-row
    if constexpr (TS >= 32) v += __shfl_xor(v, 16, 64);
    if constexpr (TS >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

// A: n x n row-major with leading dimension ld (doubles) in LDS; n even, n/2 * TS <= THREADS.
// nrm2: n doubles in LDS (scratch for the squared row norms).  `flag` is one int in LDS.
// Returns the number of sweeps done.  All threads of the block must call it.
template <int THREADS, int TS>
__device__ int jacobi_rows(double* A, int n, int ld, double* nrm2, int* flag, int max_sweeps, double tol) {
    const int tid = threadIdx.x;
    const int team = tid / TS;
    const int tl = tid % TS;
    const int pairs = n >> 1;
    const int m = n - 1;
    const double tol2 = tol * tol;
    int sweep = 0;
    for (; sweep < max_sweeps; ++sweep) {
        // refresh the cached squared norms (one team per row, several passes if needed)
        for (int row = team; row < n; row += THREADS / TS) {
            double s = 0.0;
            for (int c = tl; c < n; c += TS) {
                const double v = A[row * ld + c];
                s += v * v;
            }
            s = team_sum<TS>(s);
            if (tl == 0) nrm2[row] = s;
        }
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
                double ga = 0.0;
                for (int c = tl; c < n; c += TS) ga += x[c] * y[c];
                ga = team_sum<TS>(ga);
                const double al = nrm2[p], be = nrm2[q];
                if (ga * ga > tol2 * al * be && ga != 0.0) {
                    // tan of the rotation angle in fp32, cos/sin normalised in fp64
                    const float gf = static_cast<float>(ga), df = static_cast<float>(be - al);
                    float zf;
                    if (fabsf(gf) > 1e-30f && fabsf(df) < 1e30f)
                        zf = df / (2.0f * gf);
                    else   // outside fp32's comfortable range: take the ratio in fp64 (rare)
                        zf = static_cast<float>((be - al) / (2.0 * ga));
                    float tf;
                    if (fabsf(zf) < 1e15f)
                        tf = copysignf(1.0f, zf) / (fabsf(zf) + sqrtf(1.0f + zf * zf));
                    else
                        tf = 0.5f / zf;
                    const double t = static_cast<double>(tf);
                    const double a = 1.0 + t * t;
                    double cs = static_cast<double>(rsqrtf(static_cast<float>(a)));
                    cs = cs * (1.5 - 0.5 * a * cs * cs);
                    cs = cs * (1.5 - 0.5 * a * cs * cs);
                    const double sn = cs * t;
                    for (int c = tl; c < n; c += TS) {
                        const double xv = x[c], yv = y[c];
                        x[c] = cs * xv - sn * yv;
                        y[c] = sn * xv + cs * yv;
                    }
                    if (tl == 0) {
                        // exact for the exact angle; the fp32 angle leaves an O(1e-7) relative drift that
                        // the per-sweep refresh removes
                        nrm2[p] = cs * cs * al - 2.0 * cs * sn * ga + sn * sn * be;
                        nrm2[q] = sn * sn * al + 2.0 * cs * sn * ga + cs * cs * be;
                        *flag = 1;
                    }
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
