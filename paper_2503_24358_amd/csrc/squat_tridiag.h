// Top-r eigenpairs (r <= 64) of a symmetric positive semi-definite 128 x 128 matrix by the
// classical dense route, one 512-thread workgroup per matrix (Section 3.2: the
// right singular vectors and singular values of the query matrix are the
// eigenpairs of its Gram matrix):
//
//   1. Householder reduction to tridiagonal form T.  The matrix lives in the
//      REGISTERS of the first four wavefronts, dealt out cyclically: thread
//      (team, lane l of the team of 8) holds rows team, 32 + team, 64 + team,
//      96 + team at columns l, 8 + l, .., 120 + l, so the trailing block
//      shrinks in every thread at once; per step only the column being
//      eliminated, the product A v and two scalars travel through LDS (two
//      barriers per step).
//   2. The r largest eigenvalues of T by 17-section on Sturm counts (16 trial
//      shifts per eigenvalue and round, 14 rounds from [-3, 3] ||T||): the count
//      is the number of sign changes of the three-term recurrence of the leading
//      principal minors, division-free, rescaled by a power of two every 8 terms.
//   3. Eigenvectors of T by inverse iteration with those shifts (made distinct by
//      a few ulps where eigenvalues coincide): two solves per vector by Gaussian
//      elimination with partial pivoting, one lane per vector; then the Gram
//      matrix of the vectors decides whether they are orthonormal to 1e-10
//      already (separated eigenvalues), need one symmetric correction step (close
//      eigenvalues) or go through Cholesky-QR (coincident ones).
//   4. Rayleigh quotients = eigenvalues; residuals ||T x - lambda x|| checked.
//   5. Back-transformation by the stored reflectors (kept in LDS during step 1,
//      parked in global memory while steps 2-4 use that LDS block).
//
// A matrix whose result fails the checks of step 4 (never seen with fp64, kept as
// a safety net) is flagged and handed to the Jacobi kernel.  About 40 times fewer
// floating-point operations than cyclic Jacobi on the full matrix.
#pragma once

#include "squat_internal.h"
#include "squat_jacobi.h"

namespace squat {

constexpr int kTriN = 128;
constexpr int kTriRows = 4;              // matrix rows per thread in the reduction (one wavefront per SIMD holds the matrix:
                                         // the step's scalar chain and its two wavefront sums are then done once per
                                         // SIMD, not twice; 6 us of 325 against two rows per thread on all eight)
constexpr int kTriRedThreads = kTriN / kTriRows * 8;   // threads that hold the matrix: a row's 128 columns are spread over 8 lanes
constexpr int kTriThreads = 512;
static_assert(kTriRedThreads <= kTriThreads && (kTriN / kTriRows) % 8 == 0, "whole wavefronts of 8 teams hold the matrix");
constexpr int kTriMaxR = 32;            // vectors the LDS plan holds
constexpr int kTriPts = 16;             // trial shifts per eigenvalue and round (32 eigenvalues x 16 = every thread of the block)
constexpr int kTriRounds = 14;          // 17^14 > 6 * 2^53
constexpr double kTriAccept = 1e-9;     // ||T x - lambda x|| / ||T|| and |x_i . x_j| allowed before the fallback

// LDS plan, in doubles
constexpr int kTriXs = 0;               // [2][128] column being eliminated (double-buffered)
constexpr int kTriPs = 256;             // [2][128] beta * A v
constexpr int kTriDd = 512;             // [128] diagonal of T (then normalised)
constexpr int kTriEe = 640;             // [128] sub-diagonal (then normalised)
constexpr int kTriBet = 768;            // [128] beta of every reflector
constexpr int kTriDe = 896;             // [128][2] (d_i, e_{i-1}^2) normalised, for the Sturm recurrence
constexpr int kTriLam = 1152;           // [32] eigenvalues, [32] shifts, [32] Rayleigh quotients, [32] scratch
constexpr int kTriMisc = 1280;          // [64] reductions and flags
constexpr int kTriX = 1344;             // [128][32] vectors, element-major
constexpr int kTriU0 = kTriX + 4096;    // [128][32] reciprocal pivots
constexpr int kTriU1 = kTriU0 + 4096;
constexpr int kTriU2 = kTriU1 + 4096;
constexpr int kTriS = kTriU2 + 4096;    // [32][33] Gram matrix / Cholesky factor
constexpr int kTriLdsDoubles = kTriS + 32 * 33;
constexpr size_t kTriLdsBytes = static_cast<size_t>(kTriLdsDoubles) * sizeof(double);
static_assert(kTriLdsBytes <= 160 * 1024, "LDS plan exceeds a compute unit");
static_assert(kTriPts * kTriMaxR <= kTriThreads && (kTriPts & (kTriPts - 1)) == 0 && kTriPts <= 32, "one thread per (eigenvalue, trial shift); a team's points are one aligned run of lanes");
static_assert(kTriX + 16384 == kTriS, "vectors and factors form one 128 KB block (reused for the reflectors)");

__device__ __forceinline__ double tri_block_max(double v, double* scratch, int tid) {
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) v = fmax(v, __shfl_xor(v, s, 64));
    __syncthreads();                                      // scratch may still be read from an earlier use
    if ((tid & 63) == 0) scratch[tid >> 6] = v;
    __syncthreads();
    double m = scratch[0];
#pragma unroll
    for (int w = 1; w < kTriThreads / 64; ++w) m = fmax(m, scratch[w]);
    return m;
}

__device__ __forceinline__ double tri_pow2(int e) {       // 2^e, -1022 <= e <= 1023
    return __hiloint2double((e + 1023) << 20, 0);
}

// Workgroup barrier that orders LDS traffic only (the Householder loop touches nothing else; the full
// barrier would also wait for the vector-memory counter).
__device__ __forceinline__ void tri_lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ double tri_readlane(double v, int src) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
    return __hiloint2double(hi, lo);
}

// Sum over an aligned team of 32 lanes (two rows of 16): row sums by lane permutes, then the two rows
// trade their sums with the row-swap instruction (no trip through the LDS crossbar).
__device__ __forceinline__ double tri_sum32(double v) {
    v = team_sum<16>(v);
    const uint32_t lo = static_cast<uint32_t>(__double2loint(v)), hi = static_cast<uint32_t>(__double2hiint(v));
    const auto sl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto sh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __hiloint2double(static_cast<int>(sh[0]), static_cast<int>(sl[0])) +
           __hiloint2double(static_cast<int>(sh[1]), static_cast<int>(sl[1]));
}

// Sum over the wavefront, the same value (bit for bit) in every lane and in every wavefront that sums the same
// numbers: row sums, rows 0 + 1 and 2 + 3, then the two halves (all by lane permutes and swaps: the route through
// scalar registers, four v_readlane pairs and scalar-operand adds, cost about 100 cycles more per sum).
__device__ __forceinline__ double tri_wave_sum(double v) {
    v = tri_sum32(v);
    const uint32_t lo = static_cast<uint32_t>(__double2loint(v)), hi = static_cast<uint32_t>(__double2hiint(v));
    const auto sl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto sh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __hiloint2double(static_cast<int>(sh[0]), static_cast<int>(sl[0])) +
           __hiloint2double(static_cast<int>(sh[1]), static_cast<int>(sl[1]));
}

// 1 / sqrt(x) and 1 / x from the hardware approximations and Newton steps (short dependent chains: the
// library routines would sit on the critical path of every Householder step).  The approximations are good
// to 5e-8 relative (measured over 2^22 arguments across 120 binades), so two steps reach the last bit: the
// largest relative error after one step is 4e-15, after two 2.6e-16 (reciprocal: 0 against the library's
// division), and a third changes nothing.
__device__ __forceinline__ double tri_rsqrt(double x) {
    double y = __builtin_amdgcn_rsq(x);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const double e = fma(-x * y, y, 1.0);
        y = fma(0.5 * y, e, y);
    }
    return y;
}
__device__ __forceinline__ double tri_rcp(double x) {
    double y = __builtin_amdgcn_rcp(x);
#pragma unroll
    for (int it = 0; it < 2; ++it) y = fma(y, fma(-x, y, 1.0), y);
    return y;
}

// Eight Householder steps, columns k = 8 CC .. 8 CC + 7 (CC is a compile-time register index).  Rows and columns
// are dealt out cyclically: thread (team, l) holds rows team, RG + team, ... (RG = 128 / kTriRows rows per group) at
// columns 8 c + l, c = 0 .. 15.  The trailing block of step k then shrinks in every thread at once: registers c < CC
// hold finished columns for every lane (skipped at compile time), a group of rows is finished once k passes its
// last row, and the wavefronts stay equally loaded until the last group thins out.  Per step every wavefront
// recomputes sigma, alpha, beta and K and re-reads its part of v and p from LDS.  The eliminated column goes to LDS
// with zeros down to the diagonal (no masks afterwards: finished rows and columns meet zeros of v and p), and the
// rank-two update v w' + w v' is applied as two multiply-adds per element.  Threads beyond kTriRedThreads hold no
// part of the matrix and only keep the barriers.
template <int CC>
__device__ __forceinline__ void tri_steps(double (&a)[kTriRows][16], int team, int l, int tid, double* L) {
    constexpr int RG = kTriN / kTriRows;                  // rows per group = teams
    constexpr int R0 = 8 * CC / RG;                       // first row register that can be live
    const int lane = tid & 63, wave = tid >> 6;
    const bool active = tid < kTriRedThreads;
#pragma nounroll
    for (int ll = 0; ll < 8; ++ll) {
        const int k = 8 * CC + ll;
        if (k > kTriN - 3) return;                        // uniform
        double* xs = L + kTriXs + (k & 1) * kTriN;
        double* ps = L + kTriPs + (k & 1) * kTriN;
        if (active && l == ll) {
#pragma unroll
            for (int r = 0; r < kTriRows; ++r) {
                const int row = RG * r + team;
                xs[row] = row > k ? a[r][CC] : 0.0;
                if (row == k) L[kTriDd + k] = a[r][CC];
            }
        }
        tri_lds_barrier();
        // this wavefront still owns rows of the trailing block (its last group's last row is beyond k)
        const bool rows_live = active && RG * (kTriRows - 1) + 8 * wave + 7 > k;
        double alpha = 0.0, beta = 0.0;
        double p_i[kTriRows], v_i[kTriRows];
#pragma unroll
        for (int r = 0; r < kTriRows; ++r) p_i[r] = v_i[r] = 0.0;
        double vj[16];
        bool live = false;
        double xa = 0.0, xb = 0.0;                        // column entries lane and lane + 64 (used again for K)
        if (rows_live || wave == 0) {
            xa = xs[lane];
            xb = xs[lane + 64];
            const double x0 = xs[k + 1];
            // sigma = |x|^2 without its first element
            double r2 = fma(xb, xb, xa * xa);
            r2 = tri_wave_sum(r2) - x0 * x0;
            // (cancellation in the line above only matters when the rest is ~1e-16 |x0|^2: then the reflector is
            // the identity to working precision either way; a tiny negative result takes the identity branch)
            live = r2 > 0.0;
            alpha = x0;
            if (live) {
                const double sigma = fma(x0, x0, r2);
                const double sq = sigma * tri_rsqrt(sigma);
                alpha = x0 >= 0.0 ? -sq : sq;
                beta = tri_rcp(fma(fabs(x0), sq, sigma)); // 2 / v'v with v = x - alpha e_1
                if (rows_live) {
#pragma unroll
                    for (int c = CC; c < 16; ++c) vj[c] = xs[8 * c + l];
                    // column k + 1 sits in lane (ll + 1) mod 8, one register further when the lane wraps
                    if (l == ((ll + 1) & 7)) {
                        if (ll < 7) vj[CC] -= alpha;
                        if constexpr (CC < 15) {
                            if (ll == 7) vj[CC + 1] -= alpha;
                        }
                    }
#pragma unroll
                    for (int r = R0; r < kTriRows; ++r) {
                        if (!(RG * r + 8 * wave + 7 > k)) continue;   // uniform: this group's rows are done here
                        const int row = RG * r + team;
                        double q4[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                        for (int c = CC; c < 16; ++c) q4[c & 3] = fma(a[r][c], vj[c], q4[c & 3]);
                        const double q = team_sum<8>((q4[0] + q4[1]) + (q4[2] + q4[3]));
                        v_i[r] = xs[row];
                        if (row == k + 1) v_i[r] -= alpha;
                        p_i[r] = row > k ? beta * q : 0.0;
                    }
                }
            }
        }
        // rows that are done contribute zeros; every row writes so that nothing stale is read
        if (active && l == 0) {
#pragma unroll
            for (int r = 0; r < kTriRows; ++r) {
                const int row = RG * r + team;
                ps[row] = p_i[r];
                L[kTriX + k * kTriN + row] = v_i[r];      // reflector k (the block of the later phases is free now)
            }
        }
        if (tid == 0) {
            L[kTriEe + k] = alpha;
            L[kTriBet + k] = beta;
        }
        tri_lds_barrier();
        if (live && rows_live) {
            // K = beta/2 p'v ; w = p - K v ; A -= v w' + w v'
            double s;
            {
                double va = xa, vb = xb;
                if (lane == k + 1) va -= alpha;
                if (lane + 64 == k + 1) vb -= alpha;
                s = fma(ps[lane], va, ps[lane + 64] * vb);
            }
            const double K = 0.5 * beta * tri_wave_sum(s);
            double w[16];
#pragma unroll
            for (int c = CC; c < 16; ++c) w[c] = fma(-K, vj[c], ps[8 * c + l]);
#pragma unroll
            for (int r = R0; r < kTriRows; ++r) {
                if (!(RG * r + 8 * wave + 7 > k)) continue;           // uniform
                const double nw = fma(K, v_i[r], -p_i[r]), nv = -v_i[r];
#pragma unroll
                for (int c = CC; c < 16; ++c) a[r][c] = fma(nv, w[c], fma(nw, vj[c], a[r][c]));
            }
        }
    }
}

// g: the matrix (row-major doubles, symmetric positive semi-definite); vws: 128 x 128 doubles of
// scratch in global memory; qhat: r rows of 128 floats = sqrt(lambda_j) v_j, eigenvalues descending;
// eig: r floats or NULL; r <= 2 kTriMaxR.  Returns (to every thread) whether the result was accepted; if not, the
// outputs are to be redone as a whole (a first batch of rows may have been written).  All kTriThreads threads of
// the block must call it; L: kTriLdsBytes of LDS, 16-byte aligned.
__device__ __forceinline__ bool tridiag_top_eigs(const double* g, double* vws, int r, float* qhat, float* eig,
                                                 double* L) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int team = tid >> 3, l = tid & 7;               // this thread's rows team, 32 + team, ... and columns 8 c + l
    double* misc = L + kTriMisc;

    // ---- load, scale by a power of two so that the largest entry is in [1, 2)
    double a[kTriRows][16];
#pragma unroll
    for (int r = 0; r < kTriRows; ++r) {
        const double* src = g + (kTriN / kTriRows * r + team) * kTriN + l;
#pragma unroll
        for (int c = 0; c < 16; ++c) a[r][c] = tid < kTriRedThreads ? src[8 * c] : 0.0;
    }
    double amax = 0.0;
#pragma unroll
    for (int r = 0; r < kTriRows; ++r)
#pragma unroll
        for (int c = 0; c < 16; ++c) amax = fmax(amax, fabs(a[r][c]));
    amax = tri_block_max(amax, misc, tid);
    if (!(amax > 0.0) || !(amax < 1e300)) {
        // zero matrix: zero eigenvalues, zero rows (also taken for NaN / Inf input: nothing sensible exists)
        for (int e = tid; e < r * kTriN; e += kTriThreads) qhat[e] = 0.0f;
        if (eig)
            for (int e = tid; e < r; e += kTriThreads) eig[e] = 0.0f;
        return true;
    }
    const int aexp = ((__double2hiint(amax) >> 20) & 0x7FF) - 1023;
    const int sexp = aexp < -1000 ? -1000 : (aexp > 1000 ? 1000 : aexp);
    const double down = tri_pow2(-sexp), up = tri_pow2(sexp);
#pragma unroll
    for (int r = 0; r < kTriRows; ++r)
#pragma unroll
        for (int c = 0; c < 16; ++c) a[r][c] *= down;

    // ---- 1. Householder reduction
    for (int e = tid; e < 4 * kTriN; e += kTriThreads) L[e] = 0.0;      // column and product buffers: never read uninitialised
    __syncthreads();
    tri_steps<0>(a, team, l, tid, L);
    tri_steps<1>(a, team, l, tid, L);
    tri_steps<2>(a, team, l, tid, L);
    tri_steps<3>(a, team, l, tid, L);
    tri_steps<4>(a, team, l, tid, L);
    tri_steps<5>(a, team, l, tid, L);
    tri_steps<6>(a, team, l, tid, L);
    tri_steps<7>(a, team, l, tid, L);
    tri_steps<8>(a, team, l, tid, L);
    tri_steps<9>(a, team, l, tid, L);
    tri_steps<10>(a, team, l, tid, L);
    tri_steps<11>(a, team, l, tid, L);
    tri_steps<12>(a, team, l, tid, L);
    tri_steps<13>(a, team, l, tid, L);
    tri_steps<14>(a, team, l, tid, L);
    tri_steps<15>(a, team, l, tid, L);
    // the last 2 x 2 block: rows 126 and 127 are the last two teams' last rows, columns 126 and 127 lanes 6 and 7
    // at register 15
    constexpr int kLastTeam = kTriN / kTriRows - 1;
    if (team == kLastTeam - 1 && l == 6) L[kTriDd + kTriN - 2] = a[kTriRows - 1][15];
    if (team == kLastTeam && l == 7) {
        L[kTriDd + kTriN - 1] = a[kTriRows - 1][15];
        L[kTriEe + kTriN - 1] = 0.0;
        L[kTriBet + kTriN - 2] = 0.0;
        L[kTriBet + kTriN - 1] = 0.0;
    }
    if (team == kLastTeam && l == 6) L[kTriEe + kTriN - 2] = a[kTriRows - 1][15];
    __syncthreads();
    // the reflectors leave LDS (their block is needed for the vectors and factors) and come back for step 5
    for (int e = tid * 2; e < (kTriN - 2) * kTriN; e += 2 * kTriThreads)
        *reinterpret_cast<double2*>(vws + e) = *reinterpret_cast<const double2*>(L + kTriX + e);

    // ---- normalise T to max |entry| = 1
    double tmax = 0.0;
    if (tid < kTriN) tmax = fmax(fabs(L[kTriDd + tid]), fabs(L[kTriEe + tid]));
    tmax = tri_block_max(tmax, misc, tid);                // > 0: the trace is preserved
    const double tinv = 1.0 / tmax;
    __syncthreads();
    if (tid < kTriN) {
        const double dn = L[kTriDd + tid] * tinv, en = L[kTriEe + tid] * tinv;
        L[kTriDd + tid] = dn;
        L[kTriEe + tid] = en;
        L[kTriDe + 2 * tid] = dn;
        if (tid + 1 < kTriN) L[kTriDe + 2 * (tid + 1) + 1] = en * en;
        if (tid == 0) L[kTriDe + 1] = 0.0;
    }
    __syncthreads();

    // Steps 2-5 take the eigenpairs in batches of kTriMaxR, largest first (the LDS plan holds that many vectors): r <= 32
    // is one batch; for more, T and the reflectors serve every batch.  (Two inlined copies of the batch rather than
    // a loop around one: inside a loop the compiler spills a hundred registers.)
    double lam_edge = 0.0;                                // smallest eigenvalue of the batch before
    auto batch = [&](const int joff, const int rb) -> bool {
        // ---- 2. the rb largest eigenvalues by 17-section on Sturm counts
        if (tid < kTriPts * rb) {
            const int j = tid / kTriPts, pt = tid % kTriPts;
            const int below_target = kTriN - 1 - (joff + j);  // eigenvalue joff + j (descending) has this many below it
            double lo = -3.0001, hi = 3.0001;
            const double* de = L + kTriDe;
            for (int round = 0; round < kTriRounds; ++round) {
                asm volatile("" ::: "memory");                // keep the 128 LDS reads inside the round (not hoisted into registers)
                const double step = (hi - lo) * (1.0 / (kTriPts + 1));
                const double x = fma(step, static_cast<double>(pt + 1), lo);
                double p0 = 1.0, p1 = de[0] - x;
                // The signs of the minors are shifted into a register, newest at bit 0 (one instruction per term);
                // a block's sign changes are then the ones of (signs ^ signs >> 1) over its terms.  The sign of
                // p_0 = 1 is 0, so the first minor's own sign is a change.
                uint32_t signs = static_cast<uint32_t>(__double2hiint(p1)) >> 31;
                int cnt = static_cast<int>(signs);
                auto block = [&](int b, auto nt_tag) {
                    constexpr int NTERMS = decltype(nt_tag)::value;
#pragma unroll
                    for (int u = 0; u < NTERMS; ++u) {
                        const double2 t = *reinterpret_cast<const double2*>(de + 2 * (b + u));
                        const double p2 = fma(t.x - x, p1, -(t.y * p0));
                        signs = __builtin_amdgcn_alignbit(signs, static_cast<uint32_t>(__double2hiint(p2)), 31);
                        p0 = p1;
                        p1 = p2;
                    }
                    cnt += __popc((signs ^ (signs >> 1)) & ((1u << NTERMS) - 1u));
                    // rescale the pair by a power of two (the larger one to [1, 2))
                    const double m = fmax(fabs(p0), fabs(p1));
                    const int ex = ((__double2hiint(m) >> 20) & 0x7FF) - 1023;
                    if (ex > -1000 && ex < 1000) {
                        const double f = tri_pow2(-ex);
                        p0 *= f;
                        p1 *= f;
                    }
                };
                static_assert((kTriN - 1) % 8 == 7, "15 blocks of 8 terms and one of 7");
                for (int b = 1; b + 8 <= kTriN; b += 8) block(b, std::integral_constant<int, 8>{});
                block(kTriN - 7, std::integral_constant<int, 7>{});
                // the team's points are ascending: those with count <= target are a prefix
                const unsigned long long mask = __ballot(cnt <= below_target);
                const int nb = __popc(static_cast<unsigned>((mask >> (lane & ~(kTriPts - 1))) & ((1u << kTriPts) - 1u)));
                const double nlo = nb == 0 ? lo : fma(step, static_cast<double>(nb), lo);
                const double nhi = nb == kTriPts ? hi : fma(step, static_cast<double>(nb + 1), lo);
                lo = nlo;
                hi = nhi;
            }
            if (pt == 0) L[kTriLam + j] = 0.5 * (lo + hi);
        }
        __syncthreads();
        // A later batch stands on its own only if its eigenvalues are clear of the batch before (vectors of eigenvalues
        // closer than this could share a subspace, which only a joint orthonormalisation would see)
        if (joff > 0 && !(lam_edge - L[kTriLam] >= 1e-7)) return false;      // uniform
        lam_edge = L[kTriLam + rb - 1];

        // ---- 3. inverse iteration, one lane per vector
        if (tid == 0) {
            const double sep = 10.0 * 2.220446049250313e-16;  // coincident eigenvalues get shifts a few ulps apart
            double prev = L[kTriLam];
            L[kTriLam + 32] = prev;
            for (int j = 1; j < rb; ++j) {
                double s = L[kTriLam + j];
                s = s > prev - sep ? prev - sep : s;
                L[kTriLam + 32 + j] = s;
                prev = s;
            }
        }
        // columns rb .. 31 are padding (unit vectors, never used)
        for (int e = tid; e < kTriN * 32; e += kTriThreads) {
            const int row = e >> 5, colj = e & 31;
            // start vectors: a fixed pseudo-random pattern in (-1, 1)
            uint32_t h = static_cast<uint32_t>(row) * 2654435761u + static_cast<uint32_t>(colj) * 40503u + 12345u;
            h ^= h >> 15;
            h *= 2246822519u;
            h ^= h >> 13;
            const double rnd = (static_cast<double>(h >> 8) + 0.5) * (2.0 / 16777216.0) - 1.0;
            L[kTriX + e] = colj < rb ? rnd : (row == colj ? 1.0 : 0.0);
        }
        __syncthreads();
        if (tid < rb) {
            const int j = tid;
            const double shift = L[kTriLam + 32 + j];
            const double pivmin = 2.0e-19;
            const double* dn = L + kTriDd;
            const double* en = L + kTriEe;
            double* X = L + kTriX + j;
            double* U0 = L + kTriU0 + j;
            double* U1 = L + kTriU1 + j;
            double* U2 = L + kTriU2 + j;
            double scale = 1.0;
            for (int it = 0; it < 2; ++it) {
                // forward elimination with row interchanges, applied to the right-hand side on the fly
                double ca = dn[0] - shift, cc = en[0], cf = 0.0, cb = X[0] * scale;
                for (int row = 0; row < kTriN - 1; ++row) {
                    const double na = en[row], nc = dn[row + 1] - shift, nf = row + 1 < kTriN - 1 ? en[row + 1] : 0.0;
                    const double nb = X[32 * (row + 1)] * scale;
                    const bool keep = fabs(ca) >= fabs(na);
                    double pa = keep ? ca : na, pc = keep ? cc : nc, pf = keep ? cf : nf, pb = keep ? cb : nb;
                    const double oa = keep ? na : ca, oc = keep ? nc : cc, of = keep ? nf : cf, ob = keep ? nb : cb;
                    if (fabs(pa) < pivmin) pa = pa < 0.0 ? -pivmin : pivmin;
                    const double inv = tri_rcp(pa);
                    const double mlt = oa * inv;
                    U0[32 * row] = inv;
                    U1[32 * row] = pc;
                    U2[32 * row] = pf;
                    X[32 * row] = pb;
                    ca = fma(-mlt, pc, oc);
                    cc = fma(-mlt, pf, of);
                    cf = 0.0;
                    cb = fma(-mlt, pb, ob);
                }
                if (fabs(ca) < pivmin) ca = ca < 0.0 ? -pivmin : pivmin;
                // back substitution
                double x2 = 0.0, x1 = cb * tri_rcp(ca), big = fabs(x1);
                X[32 * (kTriN - 1)] = x1;
                for (int row = kTriN - 2; row >= 0; --row) {
                    const double x = (X[32 * row] - U1[32 * row] * x1 - U2[32 * row] * x2) * U0[32 * row];
                    X[32 * row] = x;
                    big = fmax(big, fabs(x));
                    x2 = x1;
                    x1 = x;
                }
                scale = big > 0.0 && big < 1e300 ? 1.0 / big : 1.0;
            }
            // unit 2-norm
            double s2 = 0.0;
            for (int row = 0; row < kTriN; ++row) {
                const double x = X[32 * row] * scale;
                s2 = fma(x, x, s2);
            }
            const double nrm = scale * (s2 > 0.0 ? 1.0 / sqrt(s2) : 0.0);
            for (int row = 0; row < kTriN; ++row) X[32 * row] *= nrm;
        }
        __syncthreads();

        // ---- orthonormality: Gram matrix of the 32 columns; Cholesky-QR (twice) only if it is not the identity
        double* S = L + kTriS;
        bool ok = true;
        for (int pass = 0; pass < 3; ++pass) {
            double dev = 0.0;
            if (tid < 256) {
                const int a2 = tid >> 4, b2 = tid & 15;
                double s00 = 0.0, s01 = 0.0, s10 = 0.0, s11 = 0.0;
                for (int row = 0; row < kTriN; ++row) {
                    const double2 xa = *reinterpret_cast<const double2*>(L + kTriX + 32 * row + 2 * a2);
                    const double2 xb = *reinterpret_cast<const double2*>(L + kTriX + 32 * row + 2 * b2);
                    s00 = fma(xa.x, xb.x, s00);
                    s01 = fma(xa.x, xb.y, s01);
                    s10 = fma(xa.y, xb.x, s10);
                    s11 = fma(xa.y, xb.y, s11);
                }
                S[(2 * a2) * 33 + 2 * b2] = s00;
                S[(2 * a2) * 33 + 2 * b2 + 1] = s01;
                S[(2 * a2 + 1) * 33 + 2 * b2] = s10;
                S[(2 * a2 + 1) * 33 + 2 * b2 + 1] = s11;
                // only the rb real columns count (the padding columns are never used)
                const double i00 = a2 == b2 ? 1.0 : 0.0;
                const bool ra0 = 2 * a2 < rb, ra1 = 2 * a2 + 1 < rb, rb0 = 2 * b2 < rb, rb1 = 2 * b2 + 1 < rb;
                dev = fmax(fmax(ra0 && rb0 ? fabs(s00 - i00) : 0.0, ra1 && rb1 ? fabs(s11 - i00) : 0.0),
                           fmax(ra0 && rb1 ? fabs(s01) : 0.0, ra1 && rb0 ? fabs(s10) : 0.0));
            }
            dev = tri_block_max(dev, misc, tid);
            if (!(dev == dev)) ok = false;
            if (dev <= 1e-10 || !ok) break;
            if (pass == 2) {
                ok = dev <= kTriAccept;
                break;
            }
            if (dev <= 1e-5) {
                // nearly orthonormal (close eigenvalues, not coincident ones): one symmetric step
                // X <- X (3/2 I - 1/2 S) squares the deviation
                constexpr int NP = kTriN * 8 / kTriThreads;    // row passes per thread
                const int j0 = 4 * (tid & 7);
                double out[NP][4];
#pragma unroll
                for (int ps2 = 0; ps2 < NP; ++ps2) {
                    const double* xr = L + kTriX + 32 * ((tid >> 3) + ps2 * (kTriThreads / 8));
#pragma unroll
                    for (int c = 0; c < 4; ++c) out[ps2][c] = 0.0;
                    for (int k2 = 0; k2 < rb; ++k2) {
                        const double xk = xr[k2];
#pragma unroll
                        for (int c = 0; c < 4; ++c) out[ps2][c] = fma(xk, S[k2 * 33 + j0 + c], out[ps2][c]);
                    }
#pragma unroll
                    for (int c = 0; c < 4; ++c) out[ps2][c] = fma(-0.5, out[ps2][c], 1.5 * xr[j0 + c]);
                }
                __syncthreads();
#pragma unroll
                for (int ps2 = 0; ps2 < NP; ++ps2)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (j0 + c < rb) L[kTriX + 32 * ((tid >> 3) + ps2 * (kTriThreads / 8)) + j0 + c] = out[ps2][c];
                __syncthreads();
                continue;
            }
            // Cholesky S = C C' in place (lower triangle), one wavefront, lane = row
            if (wave == 0) {
                int bad = 0;
                for (int j = 0; j < rb; ++j) {
                    double acc = 0.0;
                    if (lane < rb && lane >= j) {
                        acc = S[lane * 33 + j];
                        for (int k2 = 0; k2 < j; ++k2) acc = fma(-S[lane * 33 + k2], S[j * 33 + k2], acc);
                    }
                    const double piv = __shfl(acc, j, 64);
                    if (!(piv > 1e-280)) bad = 1;
                    const double rs = bad ? 0.0 : 1.0 / sqrt(piv);
                    if (lane < rb && lane >= j) S[lane * 33 + j] = lane == j ? rs : acc * rs;      // diagonal: 1 / C_jj
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
                if (lane == 0) misc[32] = bad ? 1.0 : 0.0;
            }
            __syncthreads();
            if (misc[32] != 0.0) {
                ok = false;
                break;
            }
            // X <- X C^-T : row by row, y_j = (x_j - sum_{k<j} C_jk y_k) / C_jj
            if (tid < kTriN) {
                double* xr = L + kTriX + 32 * tid;
                double y[32];
#pragma unroll
                for (int j = 0; j < 32; ++j) {
                    if (j < rb) {                              // uniform
                        double acc = xr[j];
#pragma unroll
                        for (int k2 = 0; k2 < j; ++k2) acc = fma(-S[j * 33 + k2], y[k2], acc);
                        y[j] = acc * S[j * 33 + j];
                    }
                }
#pragma unroll
                for (int j = 0; j < 32; ++j)
                    if (j < rb) xr[j] = y[j];
            }
            __syncthreads();
        }

        // ---- 4. Rayleigh quotients and residuals: team of 32 lanes per vector, 4 elements per lane, NV
        // vectors per thread
        constexpr int NV = 32 * 32 / kTriThreads;
        const int sub = tid & 31;
        double xv[NV][4];
        {
            double worst = 0.0;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const int vj = (tid >> 5) + q * (kTriThreads / 32);
                double num = 0.0, den = 0.0;
                double yv[4];
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const int row = sub + 32 * m;
                    const double x = L[kTriX + 32 * row + vj];
                    const double xm = row > 0 ? L[kTriX + 32 * (row - 1) + vj] : 0.0;
                    const double xp = row < kTriN - 1 ? L[kTriX + 32 * (row + 1) + vj] : 0.0;
                    const double em = row > 0 ? L[kTriEe + row - 1] : 0.0;
                    const double y = fma(L[kTriDd + row], x, fma(em, xm, L[kTriEe + row] * xp));
                    xv[q][m] = x;
                    yv[m] = y;
                    num = fma(x, y, num);
                    den = fma(x, x, den);
                }
                num = tri_sum32(num);
                den = tri_sum32(den);
                const double rq = den > 0.0 ? num / den : 0.0;
                double res = 0.0;
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const double t = yv[m] - rq * xv[q][m];
                    res = fma(t, t, res);
                }
                res = tri_sum32(res);
                if (sub == 0) L[kTriLam + 64 + vj] = rq;
                double w = vj < rb ? sqrt(res) : 0.0;
                if (!(w == w)) w = 1e300;
                worst = fmax(worst, w);
            }
            worst = tri_block_max(worst, misc, tid);
            if (!(worst <= kTriAccept)) ok = false;
        }
        if (!ok) return false;                                // uniform: every thread saw the same flags

        // ---- 5. back-transformation: team of 16 lanes per vector (every thread of the block: 32 vectors), lane s holds
        // elements s, s + 16, ..., s + 112.  Per reflector and lane: one dot product over 8 elements, a sum over the 16
        // lanes (four lane-permute stages; with 32 lanes and two vectors per thread the sums were most of the
        // instructions), 8 multiply-adds; the next reflector's entries are fetched meanwhile.  The vectors are read
        // from LDS in this layout before the reflectors come back from global memory into their block.
        static_assert(kTriThreads == 16 * kTriMaxR, "one team of 16 lanes per vector");
        const int bvj = tid >> 4, bs = tid & 15;
        double xb[8];
#pragma unroll
        for (int m = 0; m < 8; ++m) xb[m] = L[kTriX + 32 * (bs + 16 * m) + bvj];
        __syncthreads();
        __threadfence_block();
        {
            double* V = L + kTriX;
            // (unrolled, so that the loads of several trips are in flight together: one trip at a time, each of the 16
            // trips waits out a whole global-memory round trip)
#pragma unroll 8
            for (int e = tid * 2; e < (kTriN - 2) * kTriN; e += 2 * kTriThreads)
                *reinterpret_cast<double2*>(V + e) = *reinterpret_cast<const double2*>(vws + e);
            __syncthreads();
            double vn[8];
#pragma unroll
            for (int m = 0; m < 8; ++m) vn[m] = V[(kTriN - 3) * kTriN + bs + 16 * m];
            // (a wavefront holds four vectors: one whose vectors are all padding skips the loop)
            for (int k = 4 * wave < rb ? kTriN - 3 : -1; k >= 0; --k) {
                const double beta = L[kTriBet + k];
                double v[8];
#pragma unroll
                for (int m = 0; m < 8; ++m) v[m] = vn[m];
                if (k > 0) {
#pragma unroll
                    for (int m = 0; m < 8; ++m) vn[m] = V[(k - 1) * kTriN + bs + 16 * m];
                }
                if (beta == 0.0) continue;                    // uniform
                double s0 = 0.0, s1 = 0.0;
#pragma unroll
                for (int m = 0; m < 8; m += 2) {
                    s0 = fma(v[m], xb[m], s0);
                    s1 = fma(v[m + 1], xb[m + 1], s1);
                }
                const double sc = team_sum<16>(s0 + s1) * beta;
#pragma unroll
                for (int m = 0; m < 8; ++m) xb[m] = fma(-sc, v[m], xb[m]);
            }
        }

        // ---- output: rank by eigenvalue, sign so that the largest component is positive, rows sqrt(lambda) v
        if (bvj < rb) {                                        // uniform per team of 16 lanes
            const double lam = L[kTriLam + 64 + bvj];
            int rank = 0;
            for (int o = 0; o < rb; ++o) {
                const double lo = L[kTriLam + 64 + o];
                rank += (lo > lam) || (lo == lam && o < bvj);
            }
            double best = -1.0, bestv = 0.0;
            int besti = kTriN;
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const double av = fabs(xb[m]);
                if (av > best) { best = av; bestv = xb[m]; besti = bs + 16 * m; }
            }
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) {
                const double ob = __shfl_xor(best, off, 64);
                const double ov = __shfl_xor(bestv, off, 64);
                const int oi = __shfl_xor(besti, off, 64);
                if (ob > best || (ob == best && oi < besti)) { best = ob; bestv = ov; besti = oi; }
            }
            const double lam_true = fmax(lam, 0.0) * tmax * up;
            const double sc = (bestv < 0.0 ? -1.0 : 1.0) * sqrt(lam_true);
            float* dst = qhat + (joff + rank) * kTriN;
#pragma unroll
            for (int m = 0; m < 8; ++m) dst[bs + 16 * m] = static_cast<float>(xb[m] * sc);
            if (eig && bs == 0) eig[joff + rank] = static_cast<float>(lam_true);
        }
        __syncthreads();                                  // the next batch reuses every LDS block
        return true;
    };
    if (!batch(0, r < kTriMaxR ? r : kTriMaxR)) return false;
    if (r > kTriMaxR) {
        if (!batch(kTriMaxR, r - kTriMaxR)) return false;
    }
    return true;
}

}  // namespace squat
