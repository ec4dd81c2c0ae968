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
// The per-round instruction count is what bounds this routine, so: squared row
// norms are cached and updated algebraically (one dot product per pair instead
// of three, refreshed from scratch every sweep); each lane keeps its slice of
// both rows in registers between the dot product and the update (16-byte LDS
// accesses); the rotation angle is computed in fp32 with hardware reciprocal /
// square-root approximations (ANY angle gives an exactly orthogonal rotation;
// its accuracy only sets how completely one rotation annihilates the pair, and
// later sweeps finish the job) while cos/sin are normalised in fp64 by Newton
// steps; team reductions use DPP moves instead of LDS permutes; the sweep that
// would only confirm convergence is skipped when the largest relative
// off-diagonal seen in a sweep is already below sqrt(tol) (Jacobi converges
// quadratically).
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

// A: n x n row-major with leading dimension ld (doubles, even; A 16-byte aligned) in LDS; n even,
// n/2 * TS <= THREADS, n <= MAXE * TS.  FULL promises n == MAXE * TS (no column predicates).
// nrm2: n doubles in LDS (scratch for the squared row norms).  `flag`: two ints in LDS.
// Returns the number of sweeps done.  All threads of the block must call it.
// THREADS == 64 runs the whole problem inside one wavefront (tid = lane): the synchronisation points
// are then wave-level fences instead of workgroup barriers, so several problems can share a workgroup.
template <int THREADS>
__device__ __forceinline__ void team_sync() {
    if constexpr (THREADS == 64) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        __syncthreads();
    }
}

template <int THREADS, int TS, int MAXE, bool FULL>
__device__ int jacobi_rows(double* A, int n, int ld, double* nrm2, int* flag, int max_sweeps, double tol) {
    constexpr int MAXP = (MAXE + 1) / 2;     // column pairs per lane
    const int tid = THREADS == 64 ? (threadIdx.x & 63) : threadIdx.x;
    const int team = tid / TS;
    const int tl = tid % TS;
    const int pairs = n >> 1;
    const int m = n - 1;
    const float tol2 = static_cast<float>(tol * tol);
    const float early2 = static_cast<float>(tol);           // (sqrt(tol))^2
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
        if (tid == 0) {
            flag[0] = 0;      // any rotation in this sweep
            flag[1] = 0;      // any pair whose relative off-diagonal exceeded sqrt(tol)
        }
        team_sync<THREADS>();
        for (int round = 0; round < m; ++round) {
            if (team < pairs) {
                int p, q;
                if (team == 0) {
                    p = m;
                    q = round;
                } else {
                    p = round + team;
                    p = p >= m ? p - m : p;
                    q = round - team;
                    q = q < 0 ? q + m : q;
                }
                double* x = A + p * ld;
                double* y = A + q * ld;
                double2 xv[MAXP], yv[MAXP];
                double g0 = 0.0, g1 = 0.0;
#pragma unroll
                for (int e = 0; e < MAXP; ++e) {
                    const int c = 2 * (tl + e * TS);
                    if (FULL || c < n) {
                        xv[e] = *reinterpret_cast<const double2*>(x + c);
                        yv[e] = *reinterpret_cast<const double2*>(y + c);
                    } else {
                        xv[e] = double2{0.0, 0.0};
                        yv[e] = double2{0.0, 0.0};
                    }
                    g0 = fma(xv[e].x, yv[e].x, g0);
                    g1 = fma(xv[e].y, yv[e].y, g1);
                }
                const double ga = team_sum<TS>(g0 + g1);
                const double al = nrm2[p], be = nrm2[q];
                // the decision and the angle only need fp32 (the range guard sends the rare pair whose
                // magnitudes leave fp32's range through fp64)
                float gf = static_cast<float>(ga), af = static_cast<float>(al), bf = static_cast<float>(be);
                float df = static_cast<float>(be - al);
                const float big = fmaxf(af, bf);
                if (!(big < 1e18f && big > 1e-18f)) {
                    // rescale by a power of two: the ratios below are scale-free
                    int ex;
                    (void)frexp(fmax(al, be), &ex);
                    gf = static_cast<float>(ldexp(ga, -ex));
                    af = static_cast<float>(ldexp(al, -ex));
                    bf = static_cast<float>(ldexp(be, -ex));
                    df = static_cast<float>(ldexp(be - al, -ex));
                }
                const float g2 = gf * gf, ab = af * bf;
                if (g2 > tol2 * ab && gf != 0.0f) {
                    const float zf = df * __builtin_amdgcn_rcpf(2.0f * gf);
                    const float az = fabsf(zf);
                    // tan = sign(z) / (|z| + sqrt(1 + z^2));   |z| huge: 1 / (2 z)
                    const float den = az < 1e18f ? az + __builtin_amdgcn_sqrtf(fmaf(zf, zf, 1.0f)) : 2.0f * az;
                    const float tf = copysignf(__builtin_amdgcn_rcpf(den), zf);
                    const double t = static_cast<double>(tf);
                    const double a = fma(t, t, 1.0);
                    double cs = static_cast<double>(__builtin_amdgcn_rsqf(static_cast<float>(a)));
                    cs = cs * fma(-0.5 * a, cs * cs, 1.5);
                    cs = cs * fma(-0.5 * a, cs * cs, 1.5);
                    const double sn = cs * t;
#pragma unroll
                    for (int e = 0; e < MAXP; ++e) {
                        const int c = 2 * (tl + e * TS);
                        if (FULL || c < n) {
                            *reinterpret_cast<double2*>(x + c) =
                                double2{fma(cs, xv[e].x, -sn * yv[e].x), fma(cs, xv[e].y, -sn * yv[e].y)};
                            *reinterpret_cast<double2*>(y + c) =
                                double2{fma(sn, xv[e].x, cs * yv[e].x), fma(sn, xv[e].y, cs * yv[e].y)};
                        }
                    }
                    if (tl == 0) {
                        // exact for ANY rotation angle; rounding drift is removed by the per-sweep refresh
                        const double cc = cs * cs, ss = sn * sn, x2 = 2.0 * cs * sn * ga;
                        nrm2[p] = cc * al - x2 + ss * be;
                        nrm2[q] = ss * al + x2 + cc * be;
                        flag[0] = 1;
                        if (g2 > early2 * ab) flag[1] = 1;
                    }
                }
            }
            team_sync<THREADS>();
        }
        const int any = flag[0], coarse = flag[1];
        team_sync<THREADS>();
        if (!any || !coarse) {
            // no rotation at all, or every off-diagonal of this sweep was already below sqrt(tol)
            // before its rotation: quadratic convergence puts the next sweep below tol
            ++sweep;
            break;
        }
    }
    return sweep;
}


// The same sweep for the full-size problem (n = MAXE * TS rows, n / 2 teams of TS lanes, all threads
// busy), re-ordered so that half of the row traffic stays in registers.  LDS bandwidth, not
// arithmetic, bounds the routine above at this size: every round each team reads two rows and writes
// two rows.  Here the pairs of one sweep are visited level by level: at the level with span S the teams
// form blocks of S teams over 2 S consecutive rows; team j of a block keeps row (base + j) in REGISTERS
// for the S rounds of the level and meets rows base + S + ((j + round) mod S), which alone travel
// through LDS.  Spans n/2, n/4, ..., 1 give n - 1 rounds in which every pair of rows meets exactly
// once (pairs across the two halves of a block at this level, pairs inside a half at the deeper
// levels), i.e. a cyclic ordering like the tournament above, with half its LDS traffic.
template <int THREADS, int TS, int MAXE>
__device__ int jacobi_rows_resident(double* A, int ld, double* nrm2, int* flag, int max_sweeps, double tol) {
    constexpr int N = MAXE * TS;
    constexpr int MAXP = MAXE / 2;           // column pairs per lane
    static_assert(THREADS == (N / 2) * TS && MAXE % 2 == 0, "one team of TS lanes per row pair");
    const int tid = threadIdx.x;
    const int team = tid / TS;
    const int tl = tid % TS;
    const float tol2 = static_cast<float>(tol * tol);
    const float early2 = static_cast<float>(tol);           // (sqrt(tol))^2
    int sweep = 0;
    for (; sweep < max_sweeps; ++sweep) {
        // refresh the cached squared norms (one team per row, two passes)
        for (int row = team; row < N; row += THREADS / TS) {
            double s = 0.0;
            for (int c = tl; c < N; c += TS) {
                const double v = A[row * ld + c];
                s += v * v;
            }
            s = team_sum<TS>(s);
            if (tl == 0) nrm2[row] = s;
        }
        if (tid == 0) {
            flag[0] = 0;      // any rotation in this sweep
            flag[1] = 0;      // any pair whose relative off-diagonal exceeded sqrt(tol)
        }
        __syncthreads();
        for (int span = N / 2; span >= 1; span >>= 1) {
            const int base = (team / span) * (2 * span);
            const int j = team % span;
            const int p = base + j;
            double* x = A + p * ld;
            double2 xv[MAXP];
#pragma unroll
            for (int e = 0; e < MAXP; ++e) xv[e] = *reinterpret_cast<const double2*>(x + 2 * (tl + e * TS));
            double al = nrm2[p];
            for (int round = 0; round < span; ++round) {
                int jq = j + round;
                jq = jq >= span ? jq - span : jq;
                const int q = base + span + jq;
                double* y = A + q * ld;
                double2 yv[MAXP];
                double g0 = 0.0, g1 = 0.0;
#pragma unroll
                for (int e = 0; e < MAXP; ++e) {
                    yv[e] = *reinterpret_cast<const double2*>(y + 2 * (tl + e * TS));
                    g0 = fma(xv[e].x, yv[e].x, g0);
                    g1 = fma(xv[e].y, yv[e].y, g1);
                }
                const double ga = team_sum<TS>(g0 + g1);
                const double be = nrm2[q];
                // the decision and the angle only need fp32 (the range guard sends the rare pair whose
                // magnitudes leave fp32's range through fp64)
                float gf = static_cast<float>(ga), af = static_cast<float>(al), bf = static_cast<float>(be);
                float df = static_cast<float>(be - al);
                const float big = fmaxf(af, bf);
                if (!(big < 1e18f && big > 1e-18f)) {
                    int ex;
                    (void)frexp(fmax(al, be), &ex);
                    gf = static_cast<float>(ldexp(ga, -ex));
                    af = static_cast<float>(ldexp(al, -ex));
                    bf = static_cast<float>(ldexp(be, -ex));
                    df = static_cast<float>(ldexp(be - al, -ex));
                }
                const float g2 = gf * gf, ab = af * bf;
                if (g2 > tol2 * ab && gf != 0.0f) {
                    const float zf = df * __builtin_amdgcn_rcpf(2.0f * gf);
                    const float az = fabsf(zf);
                    // tan = sign(z) / (|z| + sqrt(1 + z^2));   |z| huge: 1 / (2 z)
                    const float den = az < 1e18f ? az + __builtin_amdgcn_sqrtf(fmaf(zf, zf, 1.0f)) : 2.0f * az;
                    const float tf = copysignf(__builtin_amdgcn_rcpf(den), zf);
                    const double t = static_cast<double>(tf);
                    const double a = fma(t, t, 1.0);
                    double cs = static_cast<double>(__builtin_amdgcn_rsqf(static_cast<float>(a)));
                    cs = cs * fma(-0.5 * a, cs * cs, 1.5);
                    cs = cs * fma(-0.5 * a, cs * cs, 1.5);
                    const double sn = cs * t;
#pragma unroll
                    for (int e = 0; e < MAXP; ++e) {
                        const double2 xo = xv[e];
                        xv[e] = double2{fma(cs, xo.x, -sn * yv[e].x), fma(cs, xo.y, -sn * yv[e].y)};
                        *reinterpret_cast<double2*>(y + 2 * (tl + e * TS)) =
                            double2{fma(sn, xo.x, cs * yv[e].x), fma(sn, xo.y, cs * yv[e].y)};
                    }
                    // exact for ANY rotation angle; rounding drift is removed by the per-sweep refresh
                    const double cc = cs * cs, ss = sn * sn, x2 = 2.0 * cs * sn * ga;
                    if (tl == 0) {
                        nrm2[q] = ss * al + x2 + cc * be;
                        flag[0] = 1;
                        if (g2 > early2 * ab) flag[1] = 1;
                    }
                    al = cc * al - x2 + ss * be;
                }
                __syncthreads();
            }
            // the level is over: the resident row goes back for the next level's pairing
#pragma unroll
            for (int e = 0; e < MAXP; ++e) *reinterpret_cast<double2*>(x + 2 * (tl + e * TS)) = xv[e];
            if (tl == 0) nrm2[p] = al;
            __syncthreads();
        }
        const int any = flag[0], coarse = flag[1];
        __syncthreads();
        if (!any || !coarse) {
            ++sweep;
            break;
        }
    }
    return sweep;
}

}  // namespace squat
