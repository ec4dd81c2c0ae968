// Block power (subspace) iteration on the 128 x 128 Gram matrix of a KV head, followed by a Rayleigh-Ritz
// step: the cheaper route to Qhat that Algorithm 1 of the paper points to in its remark on the SVD line
// ("can be accelerated using block power method"), and the one that can start from a previous Qhat when
// the Gram matrix has only grown by a few queries.
//
// One 512-thread workgroup per head, everything in fp64:
//   - the Gram matrix lives in REGISTERS for the whole kernel (thread (row pair, l) holds columns
//     l, l + 8, ..., l + 120 of two rows), the block X (128 x 32) and Y = G X in LDS;
//   - Y = G X: every thread forms its 2 x 32 partial products over its 16 columns (16-byte LDS reads of X,
//     conflict-free with a row stride of 34 doubles) and the 8 lanes of a row pair add up through DPP moves;
//   - X <- orth(Y) by Cholesky-QR: S = Y^T Y (thread per two entries), S = C C^T by one wavefront with a row
//     per lane in registers, X = Y C^-T by one thread per row of Y (the factor is read as LDS broadcasts);
//   - Rayleigh-Ritz: T = X^T (G X) diagonalised by the one-sided Jacobi routine inside one wavefront, Ritz
//     vectors x_i = X w_i, residuals ||G x_i - theta_i x_i||, ranking, sign convention, output rows
//     sqrt(theta_i) x_i.
// The block is always 32 wide: for r < 32 the extra columns are free oversampling (the iteration then converges
// like (lambda_33 / lambda_r)^k).  A block that turns out rank-deficient (a Cholesky pivot below 1e-13 of the
// largest) flags the head; the caller redoes flagged heads with the exact solver.
#pragma once

#include <hip/hip_runtime.h>

#include "squat_internal.h"
#include "squat_jacobi.h"

namespace squat {

constexpr int kItP = 32;                 // block width
constexpr int kItLd = 34;                // doubles per row of X, Y, S in LDS
constexpr int kItThreads = 512;
constexpr int kItX = 0;                  // [128][34]
constexpr int kItY = kItX + kD * kItLd;  // [128][34]
constexpr int kItS = kItY + kD * kItLd;  // [32][34]
constexpr int kItMisc = kItS + kItP * kItLd;   // theta [32], resid [32], nrm2 [32], then ints
constexpr int kItLdsDoubles = kItMisc + 160;
constexpr size_t kItLdsBytes = static_cast<size_t>(kItLdsDoubles) * sizeof(double);

__device__ __forceinline__ double it_readlane(double v, int src) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
    return __hiloint2double(hi, lo);
}

// dst = G src (both [128][kItLd] in LDS).  g[a][c] = G[2 rp + a][8 c + l].
__device__ __forceinline__ void it_mul(const double (&g)[2][16], const double* src, double* dst, int tid) {
    const int rp = tid >> 3, l = tid & 7;
#pragma unroll 2
    for (int jb = 0; jb < kItP / 2; ++jb) {
        double a00 = 0.0, a01 = 0.0, a10 = 0.0, a11 = 0.0;
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const double2 x = *reinterpret_cast<const double2*>(src + (8 * c + l) * kItLd + 2 * jb);
            a00 = fma(g[0][c], x.x, a00);
            a01 = fma(g[0][c], x.y, a01);
            a10 = fma(g[1][c], x.x, a10);
            a11 = fma(g[1][c], x.y, a11);
        }
        a00 = team_sum<8>(a00);
        a01 = team_sum<8>(a01);
        a10 = team_sum<8>(a10);
        a11 = team_sum<8>(a11);
        if ((jb & 7) == l) {
            *reinterpret_cast<double2*>(dst + (2 * rp) * kItLd + 2 * jb) = double2{a00, a01};
            *reinterpret_cast<double2*>(dst + (2 * rp + 1) * kItLd + 2 * jb) = double2{a10, a11};
        }
    }
}

// S[i][k] = 1/2 sum_c (A[c][i] B[c][k] + A[c][k] B[c][i])  (A = B gives A^T A; A = X, B = G X the symmetrised X^T G X)
__device__ __forceinline__ void it_cross(const double* A, const double* B, double* S, int tid, bool same) {
    const int i = tid >> 4, k = 2 * (tid & 15);
    double s0 = 0.0, s1 = 0.0;
    if (same) {
#pragma unroll 8
        for (int c = 0; c < kD; ++c) {
            const double ai = A[c * kItLd + i];
            const double2 ak = *reinterpret_cast<const double2*>(A + c * kItLd + k);
            s0 = fma(ai, ak.x, s0);
            s1 = fma(ai, ak.y, s1);
        }
    } else {
#pragma unroll 4
        for (int c = 0; c < kD; ++c) {
            const double ai = A[c * kItLd + i], bi = B[c * kItLd + i];
            const double2 ak = *reinterpret_cast<const double2*>(A + c * kItLd + k);
            const double2 bk = *reinterpret_cast<const double2*>(B + c * kItLd + k);
            s0 = fma(ai, bk.x, fma(bi, ak.x, s0));
            s1 = fma(ai, bk.y, fma(bi, ak.y, s1));
        }
        s0 *= 0.5;
        s1 *= 0.5;
    }
    *reinterpret_cast<double2*>(S + i * kItLd + k) = double2{s0, s1};
}

// In-place Cholesky S = C C^T of the 32 x 32 matrix in LDS by ONE wavefront (lane = row, the row in registers,
// right-looking); C is stored with 1 / C_jj on the diagonal and zeros above it.  Returns false (to every lane) if
// the pivots span more than 1e13 or one is not positive.
__device__ __forceinline__ bool it_chol(double* S, int lane) {
    const int row = lane & 31;
    double a[kItP];
#pragma unroll
    for (int c = 0; c < kItP; ++c) a[c] = S[row * kItLd + c];
    double pmin = 1e300, pmax = 0.0;
#pragma unroll
    for (int j = 0; j < kItP; ++j) {
        const double piv = it_readlane(a[j], j);
        pmin = fmin(pmin, piv);
        pmax = fmax(pmax, piv);
        const double rs = piv > 0.0 ? 1.0 / sqrt(piv) : 0.0;
        const double lj = a[j] * rs;
        a[j] = row == j ? rs : lj;
#pragma unroll
        for (int k2 = j + 1; k2 < kItP; ++k2) a[k2] = fma(-lj, it_readlane(lj, k2), a[k2]);
    }
    if (lane < 32) {
#pragma unroll
        for (int c = 0; c < kItP; ++c) S[row * kItLd + c] = c > row ? 0.0 : a[c];
    }
    return pmin > 1e-13 * pmax;       // false for NaN as well
}

// dst[row][:] = src[row][:] C^-T, i.e. the solution x of x C^T = y for every row y of src (threads 0..127, one
// row each; the entries of C are wave-uniform LDS reads).
__device__ __forceinline__ void it_apply(const double* src, const double* C, double* dst, int tid) {
    if (tid < kD) {
        double y[kItP];
#pragma unroll
        for (int k = 0; k < kItP; k += 2) {
            const double2 v = *reinterpret_cast<const double2*>(src + tid * kItLd + k);
            y[k] = v.x;
            y[k + 1] = v.y;
        }
#pragma unroll
        for (int k = 0; k < kItP; ++k) {
            double s = y[k];
#pragma unroll
            for (int j = 0; j < k; ++j) s = fma(-y[j], C[k * kItLd + j], s);
            y[k] = s * C[k * kItLd + k];                        // diagonal holds the reciprocal
        }
#pragma unroll
        for (int k = 0; k < kItP; k += 2)
            *reinterpret_cast<double2*>(dst + tid * kItLd + k) = double2{y[k], y[k + 1]};
    }
}

// X <- orth(src) by Cholesky-QR; returns false if the block is numerically rank-deficient.  All threads call it.
__device__ __forceinline__ bool it_orth(const double* src, double* X, double* S, int* flag, int tid) {
    it_cross(src, src, S, tid, true);
    __syncthreads();
    if (tid < 64) {
        const bool ok = it_chol(S, tid);
        if (tid == 0) *flag = ok ? 0 : 1;
    }
    __syncthreads();
    const bool ok = *flag == 0;
    if (ok) it_apply(src, S, X, tid);
    __syncthreads();
    return ok;
}

// g64: this head's Gram matrix [128][128]; prev: previous Qhat of this head [r_prev][128] or NULL; qhat [r][128],
// eig [r] or NULL, resid: one float or NULL.  L: kItLdsBytes of LDS.  Returns false if the head must be redone
// by the exact solver (nothing is written then).
__device__ __forceinline__ bool subspace_iterate(const double* g64, const float* prev, int r_prev, int r, int iterations,
                                                 float* qhat, float* eig, float* resid_out, double* L) {
    const int tid = threadIdx.x;
    double* X = L + kItX;
    double* Y = L + kItY;
    double* S = L + kItS;
    double* theta = L + kItMisc;
    double* resid = theta + 32;
    double* nrm2 = resid + 32;
    int* ibuf = reinterpret_cast<int*>(nrm2 + 32);      // [0..1] Jacobi flags, [2] breakdown flag, [3] columns taken
    int* rank = ibuf + 8;                               // [32]
    int* slot = rank + 32;                              // [32] column of the start block a previous row goes to

    // ---- the Gram matrix into registers
    double g[2][16];
    {
        const int rp = tid >> 3, l = tid & 7;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 16; ++c) g[a][c] = g64[(2 * rp + a) * kD + 8 * c + l];
    }
    // ---- start block: the previous directions (non-zero rows, normalised), completed with coordinate vectors
    for (int idx = tid; idx < kD * kItLd; idx += kItThreads) X[idx] = 0.0;
    if (prev && r_prev > 0) {
        const int i = tid >> 4, part = tid & 15;
        double s = 0.0;
        if (i < r_prev)
            for (int c = part; c < kD; c += 16) {
                const double v = static_cast<double>(prev[i * kD + c]);
                s = fma(v, v, s);
            }
        s = team_sum<16>(s);
        if (part == 0) nrm2[i] = i < r_prev ? s : 0.0;
    }
    __syncthreads();
    if (tid == 0) {
        int k = 0;
        for (int i = 0; i < kItP; ++i) {
            const bool take = prev && i < r_prev && nrm2[i] > 0.0;
            slot[i] = take ? k : -1;
            k += take ? 1 : 0;
        }
        ibuf[3] = k;
    }
    __syncthreads();
    {
        const int k = ibuf[3];
        if (k > 0) {
            for (int idx = tid; idx < r_prev * kD; idx += kItThreads) {
                const int i = idx >> 7, c = idx & (kD - 1);
                if (slot[i] >= 0) X[c * kItLd + slot[i]] = static_cast<double>(prev[idx]) / sqrt(nrm2[i]);
            }
        }
        if (k < kItP && tid < kItP - k) X[(tid * (kD / (kItP - k))) * kItLd + k + tid] = 1.0;
    }
    __syncthreads();
    // previous directions next to coordinate vectors can be nearly dependent: orthonormalise twice
    if (!it_orth(X, Y, S, ibuf + 2, tid)) return false;
    if (!it_orth(Y, X, S, ibuf + 2, tid)) return false;

    // ---- power iterations
    for (int it = 0; it < iterations; ++it) {
        it_mul(g, X, Y, tid);
        __syncthreads();
        if (!it_orth(Y, X, S, ibuf + 2, tid)) return false;
    }

    // ---- Rayleigh-Ritz
    it_mul(g, X, Y, tid);
    __syncthreads();
    it_cross(X, Y, S, tid, false);
    __syncthreads();
    if (tid < 64) jacobi_rows<64, 4, 8, false>(S, kItP, kItLd, nrm2, ibuf, 60, 1e-14);
    __syncthreads();
    {
        // row i of S is now theta_i w_i^T
        const int i = tid >> 4, part = tid & 15;
        double s = 0.0;
        for (int c = part; c < kItP; c += 16) s = fma(S[i * kItLd + c], S[i * kItLd + c], s);
        s = team_sum<16>(s);
        if (part == 0) theta[i] = sqrt(s);
    }
    __syncthreads();
    if (tid < kItP) {
        const double mine = theta[tid];
        int rk = 0;
        for (int j = 0; j < kItP; ++j) {
            const double o = theta[j];
            rk += (o > mine || (o == mine && j < tid)) ? 1 : 0;
        }
        rank[tid] = rk;
    }
    double top = 0.0;
    for (int j = 0; j < kItP; ++j) top = fmax(top, theta[j]);
    // Ritz vectors x_i = X w_i and the residual vectors G x_i - theta_i x_i = (G X) w_i - theta_i x_i: thread
    // (c, block of 8 i) keeps its results in registers until every thread has read its row of X and Y
    {
        const int c = tid >> 2, i0 = 8 * (tid & 3);
        double xr[8], dr[8];
        double xrow[kItP], yrow[kItP];
#pragma unroll
        for (int k = 0; k < kItP; k += 2) {
            const double2 xv = *reinterpret_cast<const double2*>(X + c * kItLd + k);
            const double2 yv = *reinterpret_cast<const double2*>(Y + c * kItLd + k);
            xrow[k] = xv.x; xrow[k + 1] = xv.y;
            yrow[k] = yv.x; yrow[k + 1] = yv.y;
        }
#pragma unroll
        for (int ii = 0; ii < 8; ++ii) {
            const int i = i0 + ii;
            const double th = theta[i];
            const double inv = th > 1e-300 ? 1.0 / th : 0.0;
            double sx = 0.0, sy = 0.0;
#pragma unroll
            for (int k = 0; k < kItP; ++k) {
                const double w = S[i * kItLd + k];
                sx = fma(xrow[k], w, sx);
                sy = fma(yrow[k], w, sy);
            }
            xr[ii] = sx * inv;
            dr[ii] = sy * inv - th * xr[ii];
        }
        __syncthreads();
#pragma unroll
        for (int ii = 0; ii < 8; ++ii) {
            X[c * kItLd + i0 + ii] = xr[ii];
            Y[c * kItLd + i0 + ii] = dr[ii];
        }
    }
    __syncthreads();
    // residual norms, and per Ritz vector the component of largest magnitude (sign convention)
    {
        const int i = tid >> 4, part = tid & 15;
        double s = 0.0, best = -1.0, bestv = 0.0;
        int besti = kD;
        for (int c = part; c < kD; c += 16) {
            const double dv = Y[c * kItLd + i];
            s = fma(dv, dv, s);
            const double v = X[c * kItLd + i];
            if (fabs(v) > best) { best = fabs(v); bestv = v; besti = c; }
        }
        s = team_sum<16>(s);
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) {
            const double ob = __shfl_xor(best, off, 16);
            const double ov = __shfl_xor(bestv, off, 16);
            const int oi = __shfl_xor(besti, off, 16);
            if (ob > best || (ob == best && oi < besti)) { best = ob; bestv = ov; besti = oi; }
        }
        if (part == 0) {
            resid[i] = top > 0.0 ? sqrt(s) / top : 0.0;
            nrm2[i] = bestv < 0.0 ? -1.0 : 1.0;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < kItP * kD; idx += kItThreads) {
        const int i = idx >> 7, c = idx & (kD - 1);
        const int rk = rank[i];
        if (rk < r) qhat[rk * kD + c] = static_cast<float>(nrm2[i] * sqrt(theta[i]) * X[c * kItLd + i]);
    }
    if (tid < kItP && rank[tid] < r && eig) eig[rank[tid]] = static_cast<float>(theta[tid]);
    if (tid == 0 && resid_out) {
        double worst = 0.0;
        for (int i = 0; i < kItP; ++i)
            if (rank[i] < r) worst = fmax(worst, resid[i]);
        *resid_out = static_cast<float>(worst);
    }
    return true;
}

}  // namespace squat
