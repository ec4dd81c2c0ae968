// squat_prepare: the per-head update matrix U of Lemma 2 / Lemma 3 of the paper,
//     U[t g :, (t-1) g : t g] = B_t H_t,    t = 1 .. d/g - 1.
// Eliminating the free tail of Lemma 2's problem gives B_t H_t = -P[tg:,tg:]^{-1} P[tg:,blk]
// with P = I + lambda Qhat^T Qhat, and the Woodbury identity (the paper's O(r d^2) footnote)
// reduces this to an r x r problem:
//     W_t = -Qr^T (I/lambda + Qr Qr^T)^{-1} Qb,     Qb = Qhat[:, blk], Qr = Qhat[:, tg:].
// One workgroup per (head, t) works in fp64: it forms S = I/lambda + Qr Qr^T in LDS,
// diagonalises it with the one-sided Jacobi routine (rows a_i = mu_i v_i), and applies
// S^+ = sum_i a_i a_i^T / mu_i^3.  lambda = +inf drops the I/lambda term and discards the
// (numerically) zero mu_i, which yields -pinv(Qr) Qb.  By default the result is stored as fp32 numbers that
// are exactly representable in fp16; squat_prepare_ex can store the plain fp32 rounding instead.
#include <math.h>

#include "squat_internal.h"
#include "squat_jacobi.h"

using namespace squat;

// Scratch of squat_prepare_noalloc: lives in the code object, one copy per device that loads the library,
// for the life of the process.  In host code this name only stands for the symbol; the device address is
// looked up once per device (scratch_address below) and the kernels get that pointer.
constexpr size_t kStaticScratchBytes = size_t(4) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kPrepThreads = 1024;

struct PrepParams {
    const float* qhat;    // [heads][r][d]
    float* update;        // [heads][d][d]
    double* ws;           // per workgroup: y [rp][g] then z [rp][d]
    int r, rp, g, nsteps; // rp = r rounded up to even
    int nprob;            // heads * nsteps
    double inv_lambda;    // 0 for lambda = +inf
    int hard;
    int full;             // 1: store the fp32 rounding of the fp64 result; 0: round it to the fp16 grid first
};

// The stored form of an entry of U.  On the fp16 grid (relative 2^-12) the quantize kernels contract with two
// fp16 matrix passes instead of three.
__device__ __forceinline__ float stored_entry(double v, int full) {
    const float f = static_cast<float>(v);
    return full ? f : static_cast<float>(static_cast<_Float16>(f));
}

__global__ void __launch_bounds__(256) zero_fill(float* p, int64_t n4) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n4) reinterpret_cast<f32x4*>(p)[i] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// Large r (> 32; up to 64 with a finite lambda only for the heads the Cholesky kernel flags): one 1024-thread
// workgroup per (head, t) panel; intermediate products go through the global workspace.
template <int TS>
__global__ void __launch_bounds__(kPrepThreads) prepare_kernel(const PrepParams p, const int* need) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (need && need[blockIdx.x / p.nsteps] == 0) return;  // done by the Cholesky kernel
    constexpr int THREADS = kPrepThreads;
    const int r = p.r, rp = p.rp, g = p.g;
    double* S = reinterpret_cast<double*>(smem);     // rp x rp
    double* mu = S + rp * rp;                         // rp
    int* flag = reinterpret_cast<int*>(mu + rp);
    const int head = blockIdx.x / p.nsteps;
    const int t = blockIdx.x % p.nsteps + 1;          // 1 .. d/g - 1
    const int c0 = t * g;                             // first remaining channel
    const int nrest = kD - c0;
    const float* Q = p.qhat + static_cast<int64_t>(head) * r * kD;
    double* y = p.ws + static_cast<int64_t>(blockIdx.x) * rp * (g + kD);
    double* z = y + rp * g;
    const int tid = threadIdx.x;

    // S = I/lambda + Qr Qr^T  (padded row/column rp-1 is zero when r is odd)
    for (int idx = tid; idx < rp * rp; idx += THREADS) {
        const int i = idx / rp, k = idx % rp;
        double s = 0.0;
        if (i < r && k < r) {
            for (int c = c0; c < kD; ++c) s += static_cast<double>(Q[i * kD + c]) * static_cast<double>(Q[k * kD + c]);
            if (i == k) s += p.inv_lambda;
        }
        S[idx] = s;
    }
    __syncthreads();
    jacobi_rows<THREADS, TS, (kD + TS - 1) / TS, false>(S, rp, rp, mu, flag, 60, 1e-13);
    __syncthreads();

    if (tid < rp) {
        double s = 0.0;
        for (int c = 0; c < rp; ++c) s += S[tid * rp + c] * S[tid * rp + c];
        mu[tid] = sqrt(s);
    }
    __syncthreads();
    double mumax = 0.0;
    for (int i = 0; i < rp; ++i) mumax = fmax(mumax, mu[i]);
    // pseudo-inverse cut: with a finite lambda every true mu_i >= 1/lambda, so only the
    // padding row falls below it
    const double cut = p.hard ? mumax * 1e-12 : 0.5 * p.inv_lambda;

    // y_i[j] = a_i . Qb[:, j] / mu_i^3 ;  z_i[c] = sum_k Qr[k, c] a_i[k]
    for (int idx = tid; idx < rp * g; idx += THREADS) {
        const int i = idx / g, j = idx % g;
        double s = 0.0;
        const double m = mu[i];
        if (m > cut && m > 0.0) {
            for (int k = 0; k < r; ++k) s += S[i * rp + k] * static_cast<double>(Q[k * kD + (c0 - g) + j]);
            s /= (m * m * m);
        }
        y[idx] = s;
    }
    for (int idx = tid; idx < rp * nrest; idx += THREADS) {
        const int i = idx / nrest, c = idx % nrest;
        double s = 0.0;
        for (int k = 0; k < r; ++k) s += S[i * rp + k] * static_cast<double>(Q[k * kD + c0 + c]);
        z[i * kD + c] = s;
    }
    __threadfence_block();
    __syncthreads();
    // W[c][j] = - sum_i z_i[c] y_i[j]
    float* U = p.update + static_cast<int64_t>(head) * kD * kD;
    for (int idx = tid; idx < nrest * g; idx += THREADS) {
        const int c = idx / g, j = idx % g;
        double s = 0.0;
        for (int i = 0; i < rp; ++i) s += z[i * kD + c] * y[i * g + j];
        U[(c0 + c) * kD + (c0 - g) + j] = stored_entry(-s, p.full);
    }
}

// r <= 32 (the paper's usual range): one workgroup per head, one WAVEFRONT per panel t.  The r x r
// Jacobi then needs no workgroup barrier (it is bound by synchronisation latency, not arithmetic), the
// head's Qhat is staged once in LDS as fp32, and all intermediates stay in LDS:
//   X = S^+ Qb = sum_i a_i (a_i . Qb) / mu_i^3   (rp x g),      W = -Qr^T X.
__global__ void __launch_bounds__(192) prepare_wave_kernel(const PrepParams p, const int* need) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (need && need[blockIdx.x] == 0) return;             // done by the Cholesky kernel
    const int r = p.r, rp = p.rp, g = p.g;
    constexpr int QLD = kD + 1;       // odd row stride: column reads across rows hit distinct LDS banks
    const int ld = rp + 2;            // padded row: teams of 4 lanes read different rows at the same column
    const int head = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float* Qf = reinterpret_cast<float*>(smem);                          // [rp][128]
    const size_t per = (static_cast<size_t>(rp) * ld + rp + 2 + 2 * static_cast<size_t>(rp) * g) * sizeof(double);
    double* S = reinterpret_cast<double*>(smem + ((static_cast<size_t>(rp) * QLD * sizeof(float) + 15) & ~size_t(15)) + wave * per);
    double* mu = S + rp * ld;
    int* flag = reinterpret_cast<int*>(mu + rp);
    double* y = mu + rp + 2;                                             // [rp][g]
    double* X = y + rp * g;                                              // [rp][g]
    const float* Q = p.qhat + static_cast<int64_t>(head) * r * kD;
    for (int idx = threadIdx.x; idx < rp * kD; idx += blockDim.x)
        Qf[(idx >> 7) * QLD + (idx & 127)] = idx < r * kD ? Q[idx] : 0.0f;
    __syncthreads();

    const int t = wave + 1;
    const int c0 = t * g, nrest = kD - c0;
    for (int idx = lane; idx < rp * rp; idx += 64) {
        const int i = idx / rp, k = idx % rp;
        double s = (i == k && i < r) ? p.inv_lambda : 0.0;
        for (int c = c0; c < kD; ++c) s = fma(static_cast<double>(Qf[i * QLD + c]), static_cast<double>(Qf[k * QLD + c]), s);
        S[i * ld + k] = s;
    }
    team_sync<64>();
    jacobi_rows<64, 4, 8, false>(S, rp, ld, mu, flag, 60, 1e-13);
    team_sync<64>();
    for (int i = lane; i < rp; i += 64) {
        double s = 0.0;
        for (int c = 0; c < rp; ++c) s = fma(S[i * ld + c], S[i * ld + c], s);
        mu[i] = sqrt(s);
    }
    team_sync<64>();
    double mumax = 0.0;
    for (int i = 0; i < rp; ++i) mumax = fmax(mumax, mu[i]);
    const double cut = p.hard ? mumax * 1e-12 : 0.5 * p.inv_lambda;
    for (int idx = lane; idx < rp * g; idx += 64) {
        const int i = idx / g, j = idx % g;
        double s = 0.0;
        const double m = mu[i];
        if (m > cut && m > 0.0) {
            for (int k = 0; k < rp; ++k) s = fma(S[i * ld + k], static_cast<double>(Qf[k * QLD + (c0 - g) + j]), s);
            s /= (m * m * m);
        }
        y[idx] = s;
    }
    team_sync<64>();
    for (int idx = lane; idx < rp * g; idx += 64) {
        const int k = idx / g, j = idx % g;
        double s = 0.0;
        for (int i = 0; i < rp; ++i) s = fma(S[i * ld + k], y[i * g + j], s);
        X[idx] = s;
    }
    team_sync<64>();
    float* U = p.update + static_cast<int64_t>(head) * kD * kD;
    for (int idx = lane; idx < nrest * g; idx += 64) {
        const int c = idx / g, j = idx % g;
        double s = 0.0;
        for (int k = 0; k < rp; ++k) s = fma(static_cast<double>(Qf[k * QLD + c0 + c]), X[k * g + j], s);
        U[(c0 + c) * kD + (c0 - g) + j] = stored_entry(-s, p.full);
    }
}

// r <= 64 and finite lambda: S = I/lambda + Qr Qr^T is positive definite with smallest eigenvalue
// >= 1/lambda, so X = S^-1 Qb comes from a Cholesky factorisation instead of an eigen-decomposition.
// One 512-thread workgroup per head does all panels, arranged so that no thread runs a long chain of
// dependent LDS reads (RP = 32 or 64 rows: r rounded up; rows and columns >= r are the identity and cost nothing):
//   - S: RP = 32: thread (i, k) accumulates the three 32-channel pieces of Q_i . Q_k side by side and sums them
//     from the back (S_t needs the channels from t g on); RP = 64: a thread per 2 x 2 block of the upper triangle,
//     mirrored;
//   - Cholesky: one wavefront per panel, lane = row, the row in REGISTERS, right-looking (the column
//     being eliminated goes through an LDS buffer of the wavefront, which every lane reads back at
//     uniform addresses; 1 / sqrt(pivot) from the hardware approximation and two Newton steps, branch-free);
//   - triangular solves: one wavefront per panel, lane = COLUMN of Qb with its RP unknowns in registers, so a
//     step needs no exchange between lanes: the factor's entries are read at uniform LDS addresses, fetched ahead
//     of their use, and the whole substitution is straight-line code;
//   - W = -Qr^T X with a thread per 2 x 2 block of outputs and four accumulators per entry.
// A panel whose pivots span more than 1e9 (lambda times the largest eigenvalue of Qr Qr^T that large)
// sets the head's flag: the eigen-route kernel, launched afterwards, redoes exactly the flagged heads.
constexpr int kCholThreads = 512;           // 256 registers per thread: the Cholesky keeps a row of RP doubles in them

constexpr size_t chol_lds_bytes(int rp, int nsteps, int g) {
    // Qhat as fp32, the panels' matrices / factors, (RP = 32: the solutions,) the columns in flight, one flag;
    // RP = 64 writes a panel's solutions over its factor, which is not needed any more by then
    return ((static_cast<size_t>(rp) * (kD + 1) * sizeof(float) + 15) & ~size_t(15)) +
           static_cast<size_t>(nsteps) * rp * ((rp + 1) + (rp == 32 ? g : 0) + 1) * sizeof(double) + 16;
}

template <int RP>
__global__ void __launch_bounds__(kCholThreads) prepare_chol_kernel(const PrepParams p, int* need) {
    static_assert(RP == 32 || RP == 64, "rows of a panel's matrix: one or two per lane pair of a wavefront");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int r = p.r, g = p.g, nsteps = p.nsteps;
    constexpr int QLD = kD + 1;
    constexpr int LD = RP + 1;
    constexpr bool kAlias = RP == 64;                     // the solutions X_t overwrite the factor of panel t
    const int head = blockIdx.x, tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    float* Qf = reinterpret_cast<float*>(smem);                                   // [RP][129]
    double* Sall = reinterpret_cast<double*>(smem + ((RP * QLD * sizeof(float) + 15) & ~size_t(15)));   // [nsteps][RP][LD]
    double* Xall = kAlias ? Sall : Sall + nsteps * RP * LD;                       // [nsteps][RP][g] (aliased: at the panel's factor)
    const int xstride = kAlias ? RP * LD : RP * g;                                // doubles between the panels' solutions
    double* colbuf = Sall + nsteps * RP * LD + (kAlias ? 0 : nsteps * RP * g);    // [nsteps][RP] column in flight
    int* bad = reinterpret_cast<int*>(colbuf + nsteps * RP);
    const float* Q = p.qhat + static_cast<int64_t>(head) * r * kD;
    for (int idx = tid; idx < RP * kD; idx += kCholThreads)
        Qf[(idx >> 7) * QLD + (idx & 127)] = idx < r * kD ? Q[idx] : 0.0f;
    if (tid == 0) bad[0] = 0;
    // Everything of this head's matrix outside the panels is zero: row i from the start of its own block of g
    // columns on (the panels, written at the end or by the eigen route, are the columns before it).
    {
        float* Uz = p.update + static_cast<int64_t>(head) * kD * kD;
        for (int idx = tid; idx < kD * (kD / 4); idx += kCholThreads) {
            const int row = idx / (kD / 4), col = 4 * (idx % (kD / 4));
            if (col >= row / g * g) *reinterpret_cast<f32x4*>(Uz + row * kD + col) = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    __syncthreads();

    // S_t[i][k] = [i == k] / lambda + sum_{c >= (t+1) g} Q[i][c] Q[k][c]   (rows / columns >= r: identity)
    if constexpr (RP == 32) {
        for (int e = tid; e < 1024; e += kCholThreads) {
            const int i = e >> 5, k = e & 31;
            const float* qi = Qf + i * QLD;
            const float* qk = Qf + k * QLD;
            double piece[3] = {0.0, 0.0, 0.0};                // channels 32..63, 64..95, 96..127
#pragma unroll 8
            for (int c = 0; c < 32; ++c) {
#pragma unroll
                for (int b = 0; b < 3; ++b)
                    piece[b] = fma(static_cast<double>(qi[32 * (b + 1) + c]), static_cast<double>(qk[32 * (b + 1) + c]), piece[b]);
            }
            const double diag = i == k ? (i < r ? p.inv_lambda : 1.0) : 0.0;
            for (int t = 0; t < nsteps; ++t) {
                double s = diag;
                for (int b = (t + 1) * (g / 32) - 1; b < 3; ++b) s += piece[b];
                Sall[(t * RP + i) * LD + k] = s;
            }
        }
    } else {
        // 2 x 2 blocks (rows 2 ti.., columns 2 tk.., ti <= tk) of the upper triangle: 528 of them, folded into a
        // 16 x 33 rectangle of indices
        for (int e = tid; e < 528; e += kCholThreads) {
            const int fa = e / 33, fb = e % 33;
            const int ti = fb > fa ? fa : 31 - fa;
            const int tk = fb > fa ? fb - 1 : 31 - fa + fb;
            const int i0 = 2 * ti, k0 = 2 * tk;
            double piece[2][2][3];
#pragma unroll
            for (int q = 0; q < 12; ++q) (&piece[0][0][0])[q] = 0.0;
            if (k0 < r) {                                 // (i0 <= k0; beyond r the rows of Qhat are zero)
                const float* qi = Qf + i0 * QLD;
                const float* qk = Qf + k0 * QLD;
#pragma unroll 4
                for (int c = 0; c < 32; ++c) {
#pragma unroll
                    for (int b = 0; b < 3; ++b) {
                        const double i_0 = static_cast<double>(qi[32 * (b + 1) + c]), i_1 = static_cast<double>(qi[QLD + 32 * (b + 1) + c]);
                        const double k_0 = static_cast<double>(qk[32 * (b + 1) + c]), k_1 = static_cast<double>(qk[QLD + 32 * (b + 1) + c]);
                        piece[0][0][b] = fma(i_0, k_0, piece[0][0][b]);
                        piece[0][1][b] = fma(i_0, k_1, piece[0][1][b]);
                        piece[1][0][b] = fma(i_1, k_0, piece[1][0][b]);
                        piece[1][1][b] = fma(i_1, k_1, piece[1][1][b]);
                    }
                }
            }
#pragma unroll
            for (int ia = 0; ia < 2; ++ia)
#pragma unroll
                for (int ka = 0; ka < 2; ++ka) {
                    const int i = i0 + ia, k = k0 + ka;
                    const double diag = i == k ? (i < r ? p.inv_lambda : 1.0) : 0.0;
                    for (int t = 0; t < nsteps; ++t) {
                        double s = diag;
                        for (int b = (t + 1) * (g / 32) - 1; b < 3; ++b) s += piece[ia][ka][b];
                        Sall[(t * RP + i) * LD + k] = s;
                        Sall[(t * RP + k) * LD + i] = s;
                    }
                }
        }
    }
    __syncthreads();

    // Cholesky S = C C^T, one wavefront per panel; C goes back to LDS with 1 / C_jj on the diagonal
    if (wave < nsteps) {
        double* S = Sall + wave * RP * LD;
        double* col = colbuf + wave * RP;
        const int row = lane & (RP - 1);                  // RP = 32: lanes 32..63 mirror lanes 0..31 (same values, same addresses)
        double a[RP];
#pragma unroll
        for (int c = 0; c < RP; ++c) a[c] = S[row * LD + c];
        double pmin = 1e300, pmax = 0.0;
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            if (j < r) {                                  // uniform; the rows and columns from r on are the identity already
                // column j of the trailing matrix: through the wavefront's own buffer (a wavefront's LDS accesses
                // complete in order, so the reads see this write), read back at addresses that are the same in every lane
                col[row] = a[j];
                const double piv = col[j];
                pmin = fmin(pmin, piv);
                pmax = fmax(pmax, piv);
                // 1 / sqrt(pivot) without the library routines' branches (with them the compiler keeps the column's
                // loads live across the branch and spills); two Newton steps reach the last bit
                double y = __builtin_amdgcn_rsq(piv);
#pragma unroll
                for (int it = 0; it < 2; ++it) {
                    const double e = fma(-piv * y, y, 1.0);
                    y = fma(0.5 * y, e, y);
                }
                const double rs = piv > 0.0 ? y : 0.0;
                const double lj = a[j] * rs;              // column j of C (rows > j), garbage above the diagonal
                a[j] = row == j ? rs : lj;
#pragma unroll
                for (int k2 = j + 1; k2 < RP; ++k2) {
                    a[k2] = fma(-lj, col[k2] * rs, a[k2]);
                    // (half a long column at a time, so that its loads and the row fit the registers)
                    if (RP == 64 && k2 == j + 32) asm volatile("" ::: "memory");
                }
                asm volatile("" ::: "memory");            // the next step's write stays behind these reads
            }
        }
        if (lane < RP) {
#pragma unroll
            for (int c = 0; c < RP; ++c) S[row * LD + c] = c > row ? 0.0 : a[c];
        }
        if (lane == 0 && !(pmin > 1e-9 * pmax)) atomicOr(bad, 1);       // also catches NaN
    }
    __syncthreads();
    if (bad[0]) {                                          // uniform: leave this head to the eigen route
        if (tid == 0) need[head] = 1;
        return;
    }
    if (tid == 0) need[head] = 0;

    // X = S^-1 Qb, one wavefront per panel, lane j = column j of Qb (g = 32: half a wavefront): the column's
    // entries live in registers and both substitutions are straight-line code whose only memory traffic is the
    // factor, read at addresses that are the same in every lane.  (With a lane per ROW and the unknown of every
    // step broadcast between the lanes, the LDS crossbar bounded this phase: 26 of the kernel's 50 us.)
    if (wave < nsteps && lane < g) {
        const double* C = Sall + wave * RP * LD;
        double b[RP];
#pragma unroll
        for (int k = 0; k < RP; ++k) b[k] = static_cast<double>(Qf[k * QLD + wave * g + lane]);
        if constexpr (RP == 32) {
            // The factor's column (row) of step k + 1 is fetched while step k computes; the fences keep the compiler
            // from hoisting every load of the block to its top (which spills the registers).
            double cur[32], nxt[32];
            // forward: y_k = b_k / C_kk, then b_i -= C_ik y_k for i > k
#pragma unroll
            for (int i = 0; i < 32; ++i) cur[i] = C[i * LD];
#pragma unroll
            for (int k = 0; k < 32; ++k) {
                if (k + 1 < 32) {
#pragma unroll
                    for (int i = k + 1; i < 32; ++i) nxt[i] = C[i * LD + k + 1];
                }
                b[k] *= cur[k];                           // the diagonal holds 1 / C_kk
#pragma unroll
                for (int i = k + 1; i < 32; ++i) b[i] = fma(-cur[i], b[k], b[i]);
                asm volatile("" ::: "memory");
#pragma unroll
                for (int i = k + 1; i < 32; ++i) cur[i] = nxt[i];
            }
            // backward: x_k = y_k / C_kk, then y_i -= C_ki x_k for i < k
#pragma unroll
            for (int i = 0; i < 32; ++i) cur[i] = C[31 * LD + i];
#pragma unroll
            for (int k = 31; k >= 0; --k) {
                if (k > 0) {
#pragma unroll
                    for (int i = 0; i < k; ++i) nxt[i] = C[(k - 1) * LD + i];
                }
                b[k] *= cur[k];
#pragma unroll
                for (int i = 0; i < k; ++i) b[i] = fma(-cur[i], b[k], b[i]);
                asm volatile("" ::: "memory");
#pragma unroll
                for (int i = 0; i < k; ++i) cur[i] = nxt[i];
            }
        } else {
            // 64 unknowns leave room for 16 entries of the factor at a time and 16 more on their way: a step's column
            // (row) is taken in pieces of 16, the next piece (of this step or the next) fetched while one is used.
            // Steps from r on meet zeros and the identity and are skipped (uniform).
            constexpr int PC = 16;
            double cur[PC], nxt[PC], dcur, dnxt = 0.0;
            // forward: y_k = b_k / C_kk, then b_i -= C_ik y_k for i > k
            dcur = C[0];
#pragma unroll
            for (int e = 0; e < PC; ++e) cur[e] = C[(1 + e) * LD];
#pragma unroll
            for (int k = 0; k < RP; ++k) {
                if (k >= r) continue;                     // uniform: the unknowns from r on are zero
                b[k] *= dcur;                             // the diagonal holds 1 / C_kk
                if (k + 1 < RP) dnxt = C[(k + 1) * LD + k + 1];
#pragma unroll
                for (int pc = 0; pc < RP / PC; ++pc) {    // (a constant number of trips, so that the loop unrolls)
                    const int i0 = k + 1 + pc * PC;
                    if (i0 >= RP) continue;
                    // the piece after this one: further down this column, or the head of the next
                    if (i0 + PC < RP) {
#pragma unroll
                        for (int e = 0; e < PC; ++e)
                            if (i0 + PC + e < RP) nxt[e] = C[(i0 + PC + e) * LD + k];
                    } else if (k + 2 < RP) {
#pragma unroll
                        for (int e = 0; e < PC; ++e)
                            if (k + 2 + e < RP) nxt[e] = C[(k + 2 + e) * LD + k + 1];
                    }
#pragma unroll
                    for (int e = 0; e < PC; ++e)
                        if (i0 + e < RP) b[i0 + e] = fma(-cur[e], b[k], b[i0 + e]);
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int e = 0; e < PC; ++e) cur[e] = nxt[e];
                }
                dcur = dnxt;
            }
            // backward: x_k = y_k / C_kk, then y_i -= C_ki x_k for i < k (row k of the factor, from its start); the
            // first step that counts is r - 1, so every step fetches its own first piece and the later ones ahead
#pragma unroll
            for (int k = RP - 1; k >= 0; --k) {
                if (k >= r) continue;                     // uniform
                dcur = C[k * LD + k];
#pragma unroll
                for (int e = 0; e < PC; ++e)
                    if (e < k) cur[e] = C[k * LD + e];
                b[k] *= dcur;
#pragma unroll
                for (int pc = 0; pc < RP / PC; ++pc) {
                    const int i0 = pc * PC;
                    if (i0 >= k) continue;
                    if (i0 + PC < k) {
#pragma unroll
                        for (int e = 0; e < PC; ++e)
                            if (i0 + PC + e < k) nxt[e] = C[k * LD + i0 + PC + e];
                    }
#pragma unroll
                    for (int e = 0; e < PC; ++e)
                        if (i0 + e < k) b[i0 + e] = fma(-cur[e], b[k], b[i0 + e]);
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int e = 0; e < PC; ++e) cur[e] = nxt[e];
                }
            }
        }
        // (aliased: every lane of the wavefront is past its last read of the factor here)
#pragma unroll
        for (int k = 0; k < RP; ++k) Xall[wave * xstride + k * g + lane] = b[k];
    }
    __syncthreads();

    // W_t[c][j] = -sum_k Q[k][(t+1) g + c] X_t[k][j], a thread per 2 x 2 block of outputs (two LDS reads feed
    // four multiply-adds), the blocks of all panels dealt out in one run (1536 at g = 32: three per thread)
    float* U = p.update + static_cast<int64_t>(head) * kD * kD;
    const int hg = g / 2;
    int total = 0;
    for (int t = 0; t < nsteps; ++t) total += (kD - (t + 1) * g) * g / 4;
    for (int q0 = tid; q0 < total; q0 += kCholThreads) {
        int t = 0, q = q0;
        while (q >= (kD - (t + 1) * g) * g / 4) {
            q -= (kD - (t + 1) * g) * g / 4;
            ++t;
        }
        const int c0 = (t + 1) * g;
        const int c = 2 * (q / hg), j = 2 * (q % hg);
        const double* X = Xall + t * xstride + j;
        const float* Qc = Qf + c0 + c;
        double s4[2][2][4];
#pragma unroll
        for (int e = 0; e < 16; ++e) (&s4[0][0][0])[e] = 0.0;
        auto term = [&](int k, int slot) {
            const double qa = static_cast<double>(Qc[k * QLD]), qb = static_cast<double>(Qc[k * QLD + 1]);
            const double2 x = *reinterpret_cast<const double2*>(X + k * g);
            s4[0][0][slot] = fma(qa, x.x, s4[0][0][slot]);
            s4[0][1][slot] = fma(qa, x.y, s4[0][1][slot]);
            s4[1][0][slot] = fma(qb, x.x, s4[1][0][slot]);
            s4[1][1][slot] = fma(qb, x.y, s4[1][1][slot]);
        };
        if constexpr (RP == 32) {
#pragma unroll
            for (int k = 0; k < 32; ++k) term(k, k & 3);
        } else {
            const int kmax = (r + 3) & ~3;                // rows from r on are zero on both sides
#pragma unroll 2
            for (int k4 = 0; k4 < kmax; k4 += 4) {
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) term(k4 + kk, kk);
            }
        }
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            float2 o;
            o.x = stored_entry(-((s4[a][0][0] + s4[a][0][1]) + (s4[a][0][2] + s4[a][0][3])), p.full);
            o.y = stored_entry(-((s4[a][1][0] + s4[a][1][1]) + (s4[a][1][2] + s4[a][1][3])), p.full);
            *reinterpret_cast<float2*>(U + (c0 + c + a) * kD + (c0 - g) + j) = o;
        }
    }
}

int team_size(int rp) {
    int ts = 64;
    while (ts > 1 && (rp / 2) * ts > kPrepThreads) ts >>= 1;
    return ts;
}

}  // namespace

extern "C" size_t squat_prepare_workspace(int n_heads, int d, int r, int g) {
    if (d != kD || n_heads < 1 || r < 0 || r > d || (g != 32 && g != 64 && g != 128)) return 0;
    const int nsteps = d / g - 1;
    const int rp = (r + 1) & ~1;
    const size_t per = static_cast<size_t>(rp) * (g + kD) * sizeof(double);
    const size_t total = ((static_cast<size_t>(n_heads) * nsteps * per + 255) & ~size_t(255)) +
                         ((static_cast<size_t>(n_heads) * sizeof(int) + 255) & ~size_t(255));   // + one flag per head
    return total < 256 ? 256 : total;
}

namespace {

// Bytes of the two scratch pieces a call uses: `yz` (intermediate products of the r > 32 kernel) and
// `flags` (one int per head, written by the Cholesky kernel and read by the eigen-route kernel that follows
// it).  Both are fully written before they are read, so neither needs clearing.
struct PrepScratch {
    size_t yz_bytes, flag_bytes;
};
PrepScratch prep_scratch(int n_heads, int r, int g, bool hard) {
    const int nsteps = kD / g - 1;
    const int rp = (r + 1) & ~1;
    PrepScratch out{0, 0};
    if (rp > 32)
        out.yz_bytes = (static_cast<size_t>(n_heads) * nsteps * rp * (g + kD) * sizeof(double) + 255) & ~size_t(255);
    if (!hard && rp <= 64)
        out.flag_bytes = (static_cast<size_t>(n_heads) * sizeof(int) + 255) & ~size_t(255);
    return out;
}

int prepare_impl(const float* qhat, int n_heads, int r, float lambda, int g, unsigned flags_arg, float* update,
                 double* yz, int* flags, hipStream_t s) {
    const int nsteps = kD / g - 1;
    const bool trivial = (r == 0 || lambda == 0.0f || nsteps == 0);
    // The Cholesky route's kernel clears its heads' matrices itself; every other route starts from a cleared tensor.
    const bool chol_route = !trivial && r <= 64 && !isinf(lambda);
    int rc = SQUAT_OK;
    if (!chol_route) {
        const int64_t n4 = static_cast<int64_t>(n_heads) * kD * kD / 4;
        hipLaunchKernelGGL(zero_fill, dim3(static_cast<unsigned>((n4 + 255) / 256)), dim3(256), 0, s, update, n4);
        rc = check_launch();
    }
    if (rc || trivial) return rc;

    PrepParams p;
    p.qhat = qhat;
    p.update = update;
    p.ws = yz;
    p.r = r;
    p.rp = (r + 1) & ~1;
    p.g = g;
    p.nsteps = nsteps;
    p.hard = isinf(lambda) ? 1 : 0;
    p.full = (flags_arg & SQUAT_PREPARE_FULL_PRECISION) ? 1 : 0;
    p.inv_lambda = p.hard ? 0.0 : 1.0 / static_cast<double>(lambda);
    p.nprob = n_heads * nsteps;
    const int* need = nullptr;
    if (chol_route) {
        static std::atomic<uint64_t> chol32_done{0}, chol64_done{0};
        if (p.rp <= 32) {
            if ((rc = set_max_lds_once(chol32_done, reinterpret_cast<const void*>(prepare_chol_kernel<32>), 140 * 1024))) return rc;
            hipLaunchKernelGGL(prepare_chol_kernel<32>, dim3(n_heads), dim3(kCholThreads), chol_lds_bytes(32, nsteps, g), s, p, flags);
        } else {
            if ((rc = set_max_lds_once(chol64_done, reinterpret_cast<const void*>(prepare_chol_kernel<64>), 140 * 1024))) return rc;
            hipLaunchKernelGGL(prepare_chol_kernel<64>, dim3(n_heads), dim3(kCholThreads), chol_lds_bytes(64, nsteps, g), s, p, flags);
        }
        rc = check_launch();
        if (rc) return rc;
        need = flags;                                     // the eigen route below redoes the flagged heads only
    }
    if (p.rp <= 32) {
        // one workgroup per head, one wavefront per panel
        const size_t lds = ((static_cast<size_t>(p.rp) * (kD + 1) * sizeof(float) + 15) & ~size_t(15)) +
                           nsteps * (static_cast<size_t>(p.rp) * (p.rp + 2) + p.rp + 2 + 2 * static_cast<size_t>(p.rp) * g) * sizeof(double);
        static std::atomic<uint64_t> wave_done{0};
        if ((rc = set_max_lds_once(wave_done, reinterpret_cast<const void*>(prepare_wave_kernel), 140 * 1024))) return rc;
        hipLaunchKernelGGL(prepare_wave_kernel, dim3(n_heads), dim3(64 * nsteps), lds, s, p, need);
        return check_launch();
    }
    const size_t lds = (static_cast<size_t>(p.rp) * p.rp + p.rp) * sizeof(double) + 16;
    const dim3 grid(static_cast<unsigned>(p.nprob));
    const int ts = team_size(p.rp);
#define SQUAT_PREP_LAUNCH(TS)                                                                              \
    do {                                                                                                   \
        static std::atomic<uint64_t> done{0};                                                              \
        if ((rc = set_max_lds_once(done, reinterpret_cast<const void*>(prepare_kernel<TS>), 140 * 1024)))  \
            return rc;                                                                                     \
        hipLaunchKernelGGL(prepare_kernel<TS>, grid, dim3(kPrepThreads), lds, s, p, need);                 \
    } while (0)
    if (ts == 64) SQUAT_PREP_LAUNCH(64);
    else if (ts == 32) SQUAT_PREP_LAUNCH(32);
    else SQUAT_PREP_LAUNCH(16);
#undef SQUAT_PREP_LAUNCH
    return check_launch();
}

int prepare_check(const float* qhat, int n_heads, int d, int r, float lambda, int g, const float* update) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (n_heads < 0 || r < 0 || r > d) return SQUAT_E_BADSHAPE;
    if (g != 32 && g != 64 && g != 128) return SQUAT_E_BADSHAPE;
    if (!(lambda >= 0.0f)) return SQUAT_E_BADVALUE;       // also rejects NaN
    if (n_heads == 0) return SQUAT_OK;
    if (!update || (r > 0 && !qhat)) return SQUAT_E_NULLPTR;
    if (!aligned(update, 16)) return SQUAT_E_ALIGN;
    return SQUAT_OK;
}

}  // namespace

extern "C" int squat_prepare(const float* qhat, int n_heads, int d, int r, float lambda, int g, float* update,
                             void* ws, size_t ws_bytes, squat_stream stream) {
    return squat_prepare_ex(qhat, n_heads, d, r, lambda, g, 0u, update, ws, ws_bytes, stream);
}

extern "C" int squat_prepare_ex(const float* qhat, int n_heads, int d, int r, float lambda, int g, unsigned flags_arg,
                                float* update, void* ws, size_t ws_bytes, squat_stream stream) {
    if (flags_arg & ~unsigned(SQUAT_PREPARE_FULL_PRECISION)) return SQUAT_E_BADVALUE;
    if (int rc = prepare_check(qhat, n_heads, d, r, lambda, g, update)) return rc;
    if (n_heads == 0) return SQUAT_OK;
    const int nsteps = d / g - 1;
    const bool trivial = (r == 0 || lambda == 0.0f || nsteps == 0);
    int* flags = nullptr;
    if (!trivial) {
        if (!ws || ws_bytes < squat_prepare_workspace(n_heads, d, r, g)) return SQUAT_E_WORKSPACE;
        if (!aligned(ws, 256)) return SQUAT_E_ALIGN;
        // the flags follow the (r-independent) room for the intermediate products
        const int rp = (r + 1) & ~1;
        flags = reinterpret_cast<int*>(static_cast<unsigned char*>(ws) +
                                       ((static_cast<size_t>(n_heads) * nsteps * rp * (g + kD) * sizeof(double) + 255) & ~size_t(255)));
    }
    return prepare_impl(qhat, n_heads, r, lambda, g, flags_arg, update, static_cast<double*>(ws), flags,
                        static_cast<hipStream_t>(stream));
}

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (each device holds its own copy at its own address).
int scratch_address(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SQUAT_E_HIP;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return SQUAT_E_HIP;
        }
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // threads that race store the same address
    }
    *out = ptr;
    return SQUAT_OK;
}

}  // namespace

extern "C" int squat_prepare_noalloc(const float* qhat, int n_heads, int d, int r, float lambda, int g,
                                     float* update, squat_stream stream) {
    if (int rc = prepare_check(qhat, n_heads, d, r, lambda, g, update)) return rc;
    if (n_heads == 0) return SQUAT_OK;
    const bool trivial = (r == 0 || lambda == 0.0f || d / g - 1 == 0);
    double* yz = nullptr;
    int* flags = nullptr;
    if (!trivial) {
        const PrepScratch need = prep_scratch(n_heads, r, g, isinf(lambda));
        if (need.yz_bytes + need.flag_bytes > kStaticScratchBytes) return SQUAT_E_WORKSPACE;
        void* base = nullptr;
        if (int rc = scratch_address(&base)) return rc;
        // the intermediate products first (if any), the flags behind them
        yz = static_cast<double*>(base);
        flags = reinterpret_cast<int*>(static_cast<unsigned char*>(base) + need.yz_bytes);
    }
    return prepare_impl(qhat, n_heads, r, lambda, g, 0u, update, yz, flags, static_cast<hipStream_t>(stream));
}
