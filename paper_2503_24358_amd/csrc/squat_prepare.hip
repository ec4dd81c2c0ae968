// squat_prepare: the per-head update matrix U of Lemma 2 / Lemma 3 of the paper,
//     U[t g :, (t-1) g : t g] = B_t H_t,    t = 1 .. d/g - 1.
// Eliminating the free tail of Lemma 2's problem gives B_t H_t = -P[tg:,tg:]^{-1} P[tg:,blk]
// with P = I + lambda Qhat^T Qhat, and the Woodbury identity (the paper's O(r d^2) footnote)
// reduces this to an r x r problem:
//     W_t = -Qr^T (I/lambda + Qr Qr^T)^{-1} Qb,     Qb = Qhat[:, blk], Qr = Qhat[:, tg:].
// One workgroup per (head, t) works in fp64: it forms S = I/lambda + Qr Qr^T in LDS,
// diagonalises it with the one-sided Jacobi routine (rows a_i = mu_i v_i), and applies
// S^+ = sum_i a_i a_i^T / mu_i^3.  lambda = +inf drops the I/lambda term and discards the
// (numerically) zero mu_i, which yields -pinv(Qr) Qb.  The result is stored as fp32 numbers that are
// exactly representable in fp16.
#include <math.h>

#include "squat_internal.h"
#include "squat_jacobi.h"

using namespace squat;

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
};

__global__ void __launch_bounds__(256) zero_fill(float* p, int64_t n4) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n4) reinterpret_cast<f32x4*>(p)[i] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// Large r (> 32): one 1024-thread workgroup per (head, t) panel; intermediate products go through the
// global workspace.
template <int TS>
__global__ void __launch_bounds__(kPrepThreads) prepare_kernel(const PrepParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
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
        // Entries are rounded to the fp16 grid (relative 2^-12): the quantize kernel then needs two
        // matrix passes instead of three, and both sides of any comparison use this same matrix.
        U[(c0 + c) * kD + (c0 - g) + j] = static_cast<float>(static_cast<_Float16>(static_cast<float>(-s)));
    }
}

// r <= 32 (the paper's usual range): one workgroup per head, one WAVEFRONT per panel t.  The r x r
// Jacobi then needs no workgroup barrier (it is bound by synchronisation latency, not arithmetic), the
// head's Qhat is staged once in LDS as fp32, and all intermediates stay in LDS:
//   X = S^+ Qb = sum_i a_i (a_i . Qb) / mu_i^3   (rp x g),      W = -Qr^T X.
__global__ void __launch_bounds__(192) prepare_wave_kernel(const PrepParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
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
        // rounded to the fp16 grid, as in the large-r kernel
        U[(c0 + c) * kD + (c0 - g) + j] = static_cast<float>(static_cast<_Float16>(static_cast<float>(-s)));
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
    const size_t total = static_cast<size_t>(n_heads) * nsteps * per;
    return total < 256 ? 256 : total;
}

extern "C" int squat_prepare(const float* qhat, int n_heads, int d, int r, float lambda, int g, float* update,
                             void* ws, size_t ws_bytes, squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (n_heads < 0 || r < 0 || r > d) return SQUAT_E_BADSHAPE;
    if (g != 32 && g != 64 && g != 128) return SQUAT_E_BADSHAPE;
    if (!(lambda >= 0.0f)) return SQUAT_E_BADVALUE;       // also rejects NaN
    if (n_heads == 0) return SQUAT_OK;
    if (!update || (r > 0 && !qhat)) return SQUAT_E_NULLPTR;
    if (!aligned(update, 16)) return SQUAT_E_ALIGN;
    const int nsteps = d / g - 1;
    const bool trivial = (r == 0 || lambda == 0.0f || nsteps == 0);
    if (!trivial) {
        if (!ws || ws_bytes < squat_prepare_workspace(n_heads, d, r, g)) return SQUAT_E_WORKSPACE;
        if (!aligned(ws, 256)) return SQUAT_E_ALIGN;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t n4 = static_cast<int64_t>(n_heads) * kD * kD / 4;
    hipLaunchKernelGGL(zero_fill, dim3(static_cast<unsigned>((n4 + 255) / 256)), dim3(256), 0, s, update, n4);
    int rc = check_launch();
    if (rc || trivial) return rc;

    PrepParams p;
    p.qhat = qhat;
    p.update = update;
    p.ws = static_cast<double*>(ws);
    p.r = r;
    p.rp = (r + 1) & ~1;
    p.g = g;
    p.nsteps = nsteps;
    p.hard = isinf(lambda) ? 1 : 0;
    p.inv_lambda = p.hard ? 0.0 : 1.0 / static_cast<double>(lambda);
    p.nprob = n_heads * nsteps;
    if (p.rp <= 32) {
        // one workgroup per head, one wavefront per panel
        const size_t lds = ((static_cast<size_t>(p.rp) * (kD + 1) * sizeof(float) + 15) & ~size_t(15)) +
                           nsteps * (static_cast<size_t>(p.rp) * (p.rp + 2) + p.rp + 2 + 2 * static_cast<size_t>(p.rp) * g) * sizeof(double);
        static bool done = false;
        if (!done) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(prepare_wave_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 140 * 1024) != hipSuccess)
                return SQUAT_E_HIP;
            done = true;
        }
        hipLaunchKernelGGL(prepare_wave_kernel, dim3(n_heads), dim3(64 * nsteps), lds, s, p);
        return check_launch();
    }
    const size_t lds = (static_cast<size_t>(p.rp) * p.rp + p.rp) * sizeof(double) + 16;
    const dim3 grid(static_cast<unsigned>(p.nprob));
    const int ts = team_size(p.rp);
#define SQUAT_PREP_LAUNCH(TS)                                                                              \
    do {                                                                                                   \
        static bool done = false;                                                                          \
        if (!done) {                                                                                       \
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(prepare_kernel<TS>),                     \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 140 * 1024) != hipSuccess) \
                return SQUAT_E_HIP;                                                                        \
            done = true;                                                                                   \
        }                                                                                                  \
        hipLaunchKernelGGL(prepare_kernel<TS>, grid, dim3(kPrepThreads), lds, s, p);                       \
    } while (0)
    if (ts == 64) SQUAT_PREP_LAUNCH(64);
    else if (ts == 32) SQUAT_PREP_LAUNCH(32);
    else SQUAT_PREP_LAUNCH(16);
#undef SQUAT_PREP_LAUNCH
    return check_launch();
}
