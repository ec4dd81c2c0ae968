// squat_build_subspace: Qhat = diag(Sigma[:r]) V[:r] of the pooled prompt queries
// (Section 3.2 and Algorithm 1 of the paper; GQA pooling as in its appendix),
// computed as the top-r eigenpairs of the Gram matrix Q^T Q.
//
//   gram_partial  MFMA kernel.  A wavefront streams 16-token chunks of one query
//                 head; lane (hh, m) loads tokens 8*hh + 0..7, channels 4m..4m+3,
//                 and regroups them in registers (v_perm) into four MFMA
//                 operands X_a, a = 0..3, whose row m is channel 4m + a.  The
//                 same registers serve as A and B operand of X_a^T X_b, so no
//                 LDS transpose is needed; only the 10 tile products with
//                 a <= b are formed (symmetry).  fp32 accumulation per
//                 workgroup, partial tiles go to the workspace.
//   gram_reduce   sums the workgroups' partials in fp64 in a fixed order
//                 (deterministic), un-permutes channels and mirrors;
//   gram_reduce_tiles  the same with a workgroup per (tile, head), for
//                 heads with many partials.
//   eig_tridiag_kernel  r <= 64: Householder tridiagonalisation, Sturm-count search
//                 for the r largest eigenvalues, inverse iteration, back-transformation
//                 (squat_tridiag.h), one workgroup per KV head; flags a head whose result
//                 fails its own residual checks.
//   eig_kernel    cyclic one-sided Jacobi in fp64 on the 128 x 128 Gram matrix in
//                 LDS, one workgroup per KV head, then picks the r largest: r > 64, and
//                 the heads the kernel above flagged.
#include "squat_internal.h"
#include "squat_jacobi.h"
#include "squat_tridiag.h"
#include "squat_subiter.h"

using namespace squat;

namespace {

constexpr int kGramWaves = 4;
constexpr int kTiles = 10;                     // (a, b) with a <= b, a, b in 0..3
constexpr int kPartialFloats = kTiles * 1024;  // one workgroup's partial Gram

struct GramParams {
    const unsigned char* q;
    int64_t sh, st;              // strides in BYTES
    int64_t n_tokens;
    int q_per_kv;
    int wgs_per_head;
    int64_t chunks_per_qhead;    // ceil(n_tokens / 16)
    int64_t units_per_head;      // q_per_kv * chunks_per_qhead
    float* partial;              // [n_kv_heads][wgs_per_head][10][1024]
};

__host__ __device__ constexpr int tile_index(int a, int b) {   // a <= b
    int c = 0;
    for (int i = 0; i < 4; ++i)
        for (int j = i; j < 4; ++j) {
            if (i == a && j == b) return c;
            ++c;
        }
    return -1;
}

template <int DT>
struct GramOps;

// 16-bit inputs: operand of one MFMA = 8 tokens per lane, packed pairs.
template <>
struct GramOps<SQUAT_BF16> {
    typedef bf16x8 op_t;
    static __device__ __forceinline__ f32x16 mfma(op_t a, op_t b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <>
struct GramOps<SQUAT_F16> {
    typedef half8 op_t;
    static __device__ __forceinline__ f32x16 mfma(op_t a, op_t b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};

// Accumulate one workgroup's share of Q^T Q.  16-bit element types.
template <int DT>
__global__ void __launch_bounds__(kGramWaves * kWave, 1) gram_partial_16(const GramParams p) {
    typedef typename GramOps<DT>::op_t op_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5, m = lane & 31;
    const int kvh = blockIdx.x / p.wgs_per_head;
    const int wg = blockIdx.x % p.wgs_per_head;

    f32x16 acc[kTiles];
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;

    const int64_t ustride = static_cast<int64_t>(p.wgs_per_head) * kGramWaves;
    const int64_t cpq = p.chunks_per_qhead;
    const int64_t last_unit = p.units_per_head - 1;

    // Position of a unit (chunk of 16 tokens of one query head), kept in scalar registers and advanced
    // without a division: units of a wavefront are `ustride` apart.
    struct Cursor {
        int64_t u, qh, c;        // unit, its query head, its chunk inside the query head
    };
    auto advance = [&](Cursor& k) {
        k.u += ustride;
        k.c += ustride;
        while (k.c >= cpq) {     // wave-uniform
            k.c -= cpq;
            ++k.qh;
        }
    };
    Cursor ci;                   // next unit to load
    ci.u = static_cast<int64_t>(wg) * kGramWaves + wave;
    ci.qh = ci.u / cpq;
    ci.c = ci.u - ci.qh * cpq;
    Cursor cc = ci;              // next unit to multiply

    // Lane (hh, m) loads bytes 8 m .. 8 m + 7 of rows 8 hh + j, j = 0..7, of a chunk: one 32-bit offset per
    // row from the chunk's (scalar) base address.
    const uint32_t st32 = static_cast<uint32_t>(p.st);
    uint32_t voff[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) voff[j] = static_cast<uint32_t>(8 * hh + j) * st32 + static_cast<uint32_t>(m) * 8u;

    // kDepth chunks of 16 tokens are in flight per wavefront (4 KB each).  Loads are unconditional:
    // units past the end re-read the last unit, rows past the end of a query head re-read its last
    // row; both are discarded below by wave-uniform tests, so the load stream stays straight-line.
    constexpr int kDepth = 4;
    u32x2 raw[kDepth][8];
    auto issue = [&](const Cursor& k, u32x2* dst) {
        const bool past = k.u > last_unit;
        const int64_t qh = past ? p.q_per_kv - 1 : k.qh;
        const int64_t tokc = (past ? cpq - 1 : k.c) * 16;
        const unsigned char* head = p.q + (static_cast<int64_t>(kvh) * p.q_per_kv + qh) * p.sh;
        if (tokc + 16 <= p.n_tokens) {                   // whole chunk (wave-uniform)
            const unsigned char* base = head + tokc * p.st;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                dst[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(base + voff[j]));
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                int64_t tok = tokc + 8 * hh + j;
                tok = tok < p.n_tokens ? tok : p.n_tokens - 1;
                dst[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(head + tok * p.st + m * 8));
            }
        }
    };
    auto consume = [&](const Cursor& k, u32x2* src) {
        if (k.u > last_unit) return;                     // wave-uniform
        const int64_t tokc = k.c * 16;
        if (tokc + 16 > p.n_tokens) {                    // ragged last chunk of a query head (wave-uniform)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (tokc + 8 * hh + j >= p.n_tokens) src[j] = u32x2{0u, 0u};
        }
        // regroup: operand X_a holds, for channel 4m + a, the 8 tokens of this lane
        uint32_t x[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[0][i] = __builtin_amdgcn_perm(src[2 * i + 1][0], src[2 * i][0], 0x05040100u);
            x[1][i] = __builtin_amdgcn_perm(src[2 * i + 1][0], src[2 * i][0], 0x07060302u);
            x[2][i] = __builtin_amdgcn_perm(src[2 * i + 1][1], src[2 * i][1], 0x05040100u);
            x[3][i] = __builtin_amdgcn_perm(src[2 * i + 1][1], src[2 * i][1], 0x07060302u);
        }
        op_t ops[4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
            ops[a] = __builtin_bit_cast(op_t, u32x4{x[a][0], x[a][1], x[a][2], x[a][3]});
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = a; b < 4; ++b)
                acc[tile_index(a, b)] = GramOps<DT>::mfma(ops[a], ops[b], acc[tile_index(a, b)]);
    };

    if (cc.u <= last_unit) {
#pragma unroll
        for (int i = 0; i < kDepth; ++i) {
            issue(ci, raw[i]);
            advance(ci);
        }
        while (cc.u <= last_unit) {
#pragma unroll
            for (int i = 0; i < kDepth; ++i) {
                consume(cc, raw[i]);
                advance(cc);
                issue(ci, raw[i]);
                advance(ci);
            }
        }
    }

    // reduce the four wavefronts through LDS (two rounds), wave 0 writes the partial
    float* red = reinterpret_cast<float*>(smem);        // [2][10][16][64]
    auto put = [&](int slot) {
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[((slot * kTiles + t) * 16 + e) * 64 + lane] = acc[t][e];
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][e] += red[((slot * kTiles + t) * 16 + e) * 64 + lane];
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        add(0);
        float* dst = p.partial + (static_cast<int64_t>(kvh) * p.wgs_per_head + wg) * kPartialFloats;
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) dst[(t * 16 + e) * 64 + lane] = acc[t][e];
    }
}

// fp32 inputs: products on the fp32 matrix cores (32x32x2), two tokens per step.
__global__ void __launch_bounds__(kGramWaves * kWave, 1) gram_partial_f32(const GramParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hh = lane >> 5, m = lane & 31;
    const int kvh = blockIdx.x / p.wgs_per_head;
    const int wg = blockIdx.x % p.wgs_per_head;

    f32x16 acc[kTiles];
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;

    const int64_t ustride = static_cast<int64_t>(p.wgs_per_head) * kGramWaves;
    for (int64_t unit = static_cast<int64_t>(wg) * kGramWaves + wave; unit < p.units_per_head; unit += ustride) {
        const int64_t qh = unit / p.chunks_per_qhead;
        const int64_t tok0 = (unit - qh * p.chunks_per_qhead) * 16;
        const unsigned char* base = p.q + (static_cast<int64_t>(kvh) * p.q_per_kv + qh) * p.sh + m * 16;
        f32x4 raw[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t tok = tok0 + 2 * j + hh;
            if (tok < p.n_tokens)
                raw[j] = *reinterpret_cast<const f32x4*>(base + tok * p.st);
            else
                raw[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = a; b < 4; ++b)
                    acc[tile_index(a, b)] =
                        __builtin_amdgcn_mfma_f32_32x32x2f32(raw[j][a], raw[j][b], acc[tile_index(a, b)], 0, 0, 0);
    }

    float* red = reinterpret_cast<float*>(smem);
    auto put = [&](int slot) {
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[((slot * kTiles + t) * 16 + e) * 64 + lane] = acc[t][e];
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][e] += red[((slot * kTiles + t) * 16 + e) * 64 + lane];
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        add(0);
        float* dst = p.partial + (static_cast<int64_t>(kvh) * p.wgs_per_head + wg) * kPartialFloats;
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) dst[(t * 16 + e) * 64 + lane] = acc[t][e];
    }
}

// partial[(t*16 + e)*64 + lane] is element (row mm, col nn) of tile t = (a, b) with
// nn = lane & 31, mm = 8*(e>>2) + 4*(lane>>5) + (e&3), i.e. G[4*mm + a][4*nn + b].
constexpr int kRedLd = kD + 1;          // padded row of the LDS copy: the mirrored writes spread over the banks
constexpr int kRedThreads = 512;
static_assert(kPartialFloats % kRedThreads == 0, "whole entries per thread");
constexpr size_t kRedLdsBytes = static_cast<size_t>(kD) * kRedLd * sizeof(double);

// The tile layout is scattered over the matrix, so the sums are placed (both triangles) in an LDS copy of the
// matrix first and written out row by row.
// accumulate != 0: the sums are added to what g64 holds (more queries of the same heads have arrived).
__global__ void __launch_bounds__(kRedThreads) gram_reduce(const float* partial, int wgs_per_head,
                                                           double* g64, float* gram_out, int accumulate) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    double* L = reinterpret_cast<double*>(smem);
    const int kvh = blockIdx.x;
    const float* src = partial + static_cast<int64_t>(kvh) * wgs_per_head * kPartialFloats;
    double* g = g64 + static_cast<int64_t>(kvh) * kD * kD;
    float* go = gram_out ? gram_out + static_cast<int64_t>(kvh) * kD * kD : nullptr;
    // Partials outermost, the thread's kRedPer entries inside: the loads of one partial (and, unrolled, of the next)
    // are all in flight together, while every entry is still summed in the order of the partials.  (With the
    // partials innermost a thread's loads followed one another: 165 us for 32 partials per head.)
    constexpr int kRedPer = kPartialFloats / kRedThreads;
    double sums[kRedPer];
#pragma unroll
    for (int k = 0; k < kRedPer; ++k) sums[k] = 0.0;
#pragma unroll 2
    for (int w = 0; w < wgs_per_head; ++w) {
        const float* pw = src + static_cast<int64_t>(w) * kPartialFloats + threadIdx.x;
        float v[kRedPer];
#pragma unroll
        for (int k = 0; k < kRedPer; ++k) v[k] = __builtin_nontemporal_load(pw + k * kRedThreads);
#pragma unroll
        for (int k = 0; k < kRedPer; ++k) sums[k] += static_cast<double>(v[k]);
    }
#pragma unroll
    for (int k = 0; k < kRedPer; ++k) {
        const int idx = threadIdx.x + k * kRedThreads;
        const double s = sums[k];
        const int t = idx >> 10, e = (idx >> 6) & 15, lane = idx & 63;
        int a = 0, b = 0;
        {
            int c = 0;
            for (int i = 0; i < 4; ++i)
                for (int j = i; j < 4; ++j) {
                    if (c == t) { a = i; b = j; }
                    ++c;
                }
        }
        const int nn = lane & 31;
        const int mm = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        const int row = 4 * mm + a, col = 4 * nn + b;
        // diagonal tiles hold both (row, col) and (col, row); keep the upper one for an exactly symmetric result
        if (a != b || row <= col) {
            L[row * kRedLd + col] = s;
            L[col * kRedLd + row] = s;
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kD * kD; idx += kRedThreads) {
        double v = L[(idx >> 7) * kRedLd + (idx & (kD - 1))];
        if (accumulate) v += g[idx];
        g[idx] = v;
        if (go) go[idx] = static_cast<float>(v);
    }
}

// The same sums when a head has several partials (a launch with few heads: every head's Gram kernel workgroups
// left one each): one workgroup per (tile, head) instead of one per head, which then is bound by what one compute
// unit can read (1.3 MB for the 32 partials of a head of a single layer: 28 us); the sums go straight to their two
// places in the matrix (the scattered 8-byte writes are 128 KB per head).  Same order of additions, same bits.
__global__ void __launch_bounds__(kRedThreads) gram_reduce_tiles(const float* partial, int wgs_per_head,
                                                                 double* g64, float* gram_out, int accumulate) {
    const int kvh = blockIdx.y, t = blockIdx.x;
    const float* src = partial + static_cast<int64_t>(kvh) * wgs_per_head * kPartialFloats + t * 1024 + threadIdx.x;
    double* g = g64 + static_cast<int64_t>(kvh) * kD * kD;
    float* go = gram_out ? gram_out + static_cast<int64_t>(kvh) * kD * kD : nullptr;
    constexpr int kPer = 1024 / kRedThreads;
    double sums[kPer];
#pragma unroll
    for (int k = 0; k < kPer; ++k) sums[k] = 0.0;
#pragma unroll 8
    for (int w = 0; w < wgs_per_head; ++w) {
        float v[kPer];
#pragma unroll
        for (int k = 0; k < kPer; ++k)
            v[k] = __builtin_nontemporal_load(src + static_cast<int64_t>(w) * kPartialFloats + k * kRedThreads);
#pragma unroll
        for (int k = 0; k < kPer; ++k) sums[k] += static_cast<double>(v[k]);
    }
    int a = 0, b = 0;
    {
        int c = 0;
        for (int i = 0; i < 4; ++i)
            for (int j = i; j < 4; ++j) {
                if (c == t) { a = i; b = j; }
                ++c;
            }
    }
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
        const int idx = threadIdx.x + k * kRedThreads;
        const int e = (idx >> 6) & 15, lane = idx & 63;
        const int nn = lane & 31;
        const int mm = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        const int row = 4 * mm + a, col = 4 * nn + b;
        if (a != b || row <= col) {
            double v = sums[k];
            if (accumulate) v += g[row * kD + col];
            g[row * kD + col] = v;
            g[col * kD + row] = v;
            if (go) {
                go[row * kD + col] = static_cast<float>(v);
                go[col * kD + row] = static_cast<float>(v);
            }
        }
    }
}

constexpr int kEigTeam = 16;                    // lanes per row pair
constexpr int kEigThreads = 64 * kEigTeam;
constexpr int kEigLd = kD;       // rows are read with unit stride by consecutive lanes

__global__ void __launch_bounds__(kTriThreads) eig_tridiag_kernel(const double* g64, double* vws, int r, float* qhat,
                                                                  float* eig, int* need) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int64_t kvh = blockIdx.x;
    const bool ok = tridiag_top_eigs(g64 + kvh * kD * kD, vws + kvh * kD * kD, r, qhat + kvh * r * kD,
                                     eig ? eig + kvh * r : nullptr, reinterpret_cast<double*>(smem));
    if (threadIdx.x == 0) need[kvh] = ok ? 0 : 1;
}

// Block power iteration + Rayleigh-Ritz (squat_subiter.h), one workgroup per KV head; need[head] = 1 asks the
// exact solver to redo a head whose block broke down.
__global__ void __launch_bounds__(kItThreads) subspace_iter_kernel(const double* g64, const float* prev, int r_prev,
                                                                   int r, int iterations, float* qhat, float* eig,
                                                                   float* resid, int* need) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int64_t kvh = blockIdx.x;
    const bool ok = subspace_iterate(g64 + kvh * kD * kD, prev ? prev + kvh * r_prev * kD : nullptr, r_prev, r,
                                     iterations, qhat + kvh * r * kD, eig ? eig + kvh * r : nullptr,
                                     resid ? resid + kvh : nullptr, reinterpret_cast<double*>(smem));
    if (threadIdx.x == 0) {
        need[kvh] = ok ? 0 : 1;
        if (!ok && resid) resid[kvh] = 0.0f;        // the exact solver takes this head
    }
}

__global__ void __launch_bounds__(256) fill_float(float* p, int n, float v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// need: NULL = every head; else only the heads with need[head] != 0
__global__ void __launch_bounds__(kEigThreads) eig_kernel(const double* g64, int r, float* qhat, float* eig,
                                                          int* sweeps_out, const int* need) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (need && need[blockIdx.x] == 0) return;
    double* A = reinterpret_cast<double*>(smem);                 // 128 x 128
    double* nrm = A + kD * kEigLd;                               // 128
    int* rank = reinterpret_cast<int*>(nrm + kD);                // 128
    int* flag = rank + kD;
    const int kvh = blockIdx.x;
    const double* g = g64 + static_cast<int64_t>(kvh) * kD * kD;
    for (int i = threadIdx.x; i < kD * kD; i += kEigThreads) A[i] = g[i];
    __syncthreads();
    const int sweeps = jacobi_rows_resident<kEigThreads, kEigTeam, kD / kEigTeam>(A, kEigLd, nrm, flag, 60, 1e-13);
    __syncthreads();
    if (sweeps_out && threadIdx.x == 0) sweeps_out[kvh] = sweeps;

    // eigenvalue of row i = its norm
    for (int row = threadIdx.x >> 3; row < kD; row += kEigThreads / 8) {     // 8 lanes per row
        const int tl = threadIdx.x & 7;
        double s = 0.0;
        for (int c = tl; c < kD; c += 8) s += A[row * kEigLd + c] * A[row * kEigLd + c];
        s = team_sum<8>(s);
        if (tl == 0) nrm[row] = sqrt(s);
    }
    __syncthreads();
    if (threadIdx.x < kD) {
        const int i = threadIdx.x;
        const double ni = nrm[i];
        int rk = 0;
        for (int j = 0; j < kD; ++j) {
            const double nj = nrm[j];
            rk += (nj > ni) || (nj == ni && j < i);
        }
        rank[i] = rk;
    }
    __syncthreads();
    // row i with rank < r  ->  qhat[rank] = row / sqrt(norm), sign: largest |component| positive
    for (int row = threadIdx.x >> 3; row < kD; row += kEigThreads / 8) {
        const int tl = threadIdx.x & 7;
        const int rk = rank[row];
        if (rk < r) {
            double best = -1.0, bestv = 0.0;
            int besti = kD;
            for (int c = tl; c < kD; c += 8) {
                const double v = A[row * kEigLd + c];
                if (fabs(v) > best) { best = fabs(v); bestv = v; besti = c; }
            }
#pragma unroll
            for (int off = 4; off > 0; off >>= 1) {
                const double ob = __shfl_xor(best, off, 8);
                const double ov = __shfl_xor(bestv, off, 8);
                const int oi = __shfl_xor(besti, off, 8);
                if (ob > best || (ob == best && oi < besti)) { best = ob; bestv = ov; besti = oi; }
            }
            const double lam = nrm[row];
            const double sc = lam > 0.0 ? (bestv < 0.0 ? -1.0 : 1.0) / sqrt(lam) : 0.0;
            float* dst = qhat + (static_cast<int64_t>(kvh) * r + rk) * kD;
            for (int c = tl; c < kD; c += 8) dst[c] = static_cast<float>(A[row * kEigLd + c] * sc);
            if (eig && tl == 0) eig[static_cast<int64_t>(kvh) * r + rk] = static_cast<float>(lam);
        }
    }
}

struct SubspacePlan {
    int wgs_per_head;
    size_t off_partial, off_g64, off_v, off_need, total;
};

SubspacePlan plan(int64_t n_tokens, int n_kv_heads, int q_per_kv, int cus) {
    SubspacePlan pl;
    const int64_t units = q_per_kv * ((n_tokens + 15) / 16);
    int64_t per = (cus + n_kv_heads - 1) / n_kv_heads;          // one workgroup per CU in total
    const int64_t need = (units + kGramWaves * 8 - 1) / (kGramWaves * 8);   // at least 8 chunks per wavefront
    if (per > need) per = need;
    if (per < 1) per = 1;
    pl.wgs_per_head = static_cast<int>(per);
    pl.off_partial = 0;
    size_t partial = static_cast<size_t>(n_kv_heads) * per * kPartialFloats * sizeof(float);
    pl.off_g64 = (partial + 255) & ~size_t(255);
    const size_t mat = static_cast<size_t>(n_kv_heads) * kD * kD * sizeof(double);
    pl.off_v = pl.off_g64 + mat;                               // Householder reflectors of every head
    pl.off_need = pl.off_v + mat;                              // per head: 1 = the Jacobi kernel must redo it
    pl.total = pl.off_need + ((static_cast<size_t>(n_kv_heads) * sizeof(int) + 255) & ~size_t(255));
    return pl;
}

constexpr int kPlanCUs = 256;   // workspace size must not depend on the device: plan for MI355X's 256 CUs

}  // namespace

extern "C" size_t squat_build_subspace_workspace(int64_t n_tokens, int n_kv_heads, int q_per_kv, int d, int r) {
    (void)r;
    if (d != kD || n_tokens < 1 || n_kv_heads < 1 || q_per_kv < 1) return 0;
    return plan(n_tokens, n_kv_heads, q_per_kv, kPlanCUs).total;
}

namespace {

constexpr size_t kEigLdsBytes = kD * kEigLd * sizeof(double) + kD * sizeof(double) + kD * sizeof(int) + 16;
constexpr size_t kGramLdsBytes = 2 * kPartialFloats * sizeof(float);      // 80 KB

int raise_lds_limits() {
    // one flag per kernel: a failed call is retried by the next launch, a raced one only repeated
    static std::atomic<uint64_t> done[7];
    const struct { const void* kernel; size_t bytes; } limits[7] = {
        {reinterpret_cast<const void*>(gram_partial_16<SQUAT_BF16>), kGramLdsBytes},
        {reinterpret_cast<const void*>(gram_partial_16<SQUAT_F16>), kGramLdsBytes},
        {reinterpret_cast<const void*>(gram_partial_f32), kGramLdsBytes},
        {reinterpret_cast<const void*>(eig_kernel), kEigLdsBytes},
        {reinterpret_cast<const void*>(eig_tridiag_kernel), static_cast<size_t>(kTriLdsBytes)},
        {reinterpret_cast<const void*>(gram_reduce), static_cast<size_t>(kRedLdsBytes)},
        {reinterpret_cast<const void*>(subspace_iter_kernel), static_cast<size_t>(kItLdsBytes)}};
    for (int i = 0; i < 7; ++i)
        if (int rc = set_max_lds_once(done[i], limits[i].kernel, static_cast<int>(limits[i].bytes))) return rc;
    return SQUAT_OK;
}

int check_queries(const void* q, squat_dtype q_dt, int n_kv_heads, int q_per_kv, int d, int64_t q_stride_head,
                  int64_t q_stride_token) {
    if (q_dt != SQUAT_F32 && q_dt != SQUAT_F16 && q_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (!q) return SQUAT_E_NULLPTR;
    if (q_stride_token < d || q_stride_head < 0) return SQUAT_E_BADSHAPE;
    if ((q_stride_token % 8) || (q_stride_head % 8) || !aligned(q, 16)) return SQUAT_E_ALIGN;
    if (static_cast<int64_t>(n_kv_heads) * q_per_kv > (int64_t(1) << 24)) return SQUAT_E_BADSHAPE;
    // a chunk's 16 rows are addressed by 32-bit byte offsets from its first row
    if (q_stride_token * elem_size(q_dt) >= (int64_t(1) << 27)) return SQUAT_E_BADSHAPE;
    return SQUAT_OK;
}

// Pooled Gram matrices of the queries into g64 (fp64 [n_kv_heads, d, d]; added to it if accumulate), optionally
// also as fp32 into gram_out.
int run_gram(const void* q, squat_dtype q_dt, int64_t n_tokens, int n_kv_heads, int q_per_kv, int64_t q_stride_head,
             int64_t q_stride_token, const SubspacePlan& pl, void* ws, double* g64, float* gram_out, int accumulate,
             hipStream_t s) {
    const int es = elem_size(q_dt);
    GramParams p;
    p.q = static_cast<const unsigned char*>(q);
    p.sh = q_stride_head * es;
    p.st = q_stride_token * es;
    p.n_tokens = n_tokens;
    p.q_per_kv = q_per_kv;
    p.wgs_per_head = pl.wgs_per_head;
    p.chunks_per_qhead = (n_tokens + 15) / 16;
    p.units_per_head = p.chunks_per_qhead * q_per_kv;
    p.partial = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + pl.off_partial);
    const dim3 grid(static_cast<unsigned>(n_kv_heads) * pl.wgs_per_head);
    switch (q_dt) {
        case SQUAT_BF16: hipLaunchKernelGGL(gram_partial_16<SQUAT_BF16>, grid, dim3(kGramWaves * kWave), kGramLdsBytes, s, p); break;
        case SQUAT_F16: hipLaunchKernelGGL(gram_partial_16<SQUAT_F16>, grid, dim3(kGramWaves * kWave), kGramLdsBytes, s, p); break;
        default: hipLaunchKernelGGL(gram_partial_f32, grid, dim3(kGramWaves * kWave), kGramLdsBytes, s, p); break;
    }
    int rc = check_launch();
    if (rc) return rc;
    if (pl.wgs_per_head >= 4 && n_kv_heads <= 65535)
        hipLaunchKernelGGL(gram_reduce_tiles, dim3(kTiles, static_cast<unsigned>(n_kv_heads)), dim3(kRedThreads), 0, s, p.partial,
                           pl.wgs_per_head, g64, gram_out, accumulate);
    else
        hipLaunchKernelGGL(gram_reduce, dim3(n_kv_heads), dim3(kRedThreads), kRedLdsBytes, s, p.partial, pl.wgs_per_head,
                           g64, gram_out, accumulate);
    return check_launch();
}

// Exact top-r eigenpairs of the Gram matrices in g64: tridiagonal route (r <= 64, in batches of 32 vectors), Jacobi
// for larger r and for the heads that route flags.
int run_exact_solver(const double* g64, int n_kv_heads, int r, float* qhat, float* eig, const SubspacePlan& pl, void* ws,
                     hipStream_t s) {
    int rc = SQUAT_OK;
    int* need = nullptr;
    if (r <= 2 * kTriMaxR) {
        need = reinterpret_cast<int*>(static_cast<unsigned char*>(ws) + pl.off_need);
        double* vws = reinterpret_cast<double*>(static_cast<unsigned char*>(ws) + pl.off_v);
        hipLaunchKernelGGL(eig_tridiag_kernel, dim3(n_kv_heads), dim3(kTriThreads), kTriLdsBytes, s, g64, vws, r, qhat,
                           eig, need);
        rc = check_launch();
        if (rc) return rc;
    }
    hipLaunchKernelGGL(eig_kernel, dim3(n_kv_heads), dim3(kEigThreads), kEigLdsBytes, s, g64, r, qhat, eig,
                       static_cast<int*>(nullptr), static_cast<const int*>(need));
    return check_launch();
}

}  // namespace

extern "C" int squat_build_subspace(const void* q, squat_dtype q_dt, int64_t n_tokens, int n_kv_heads,
                                    int q_per_kv, int d, int64_t q_stride_head, int64_t q_stride_token,
                                    int r, float* qhat, float* eig, float* gram, void* ws, size_t ws_bytes,
                                    squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (n_tokens < 1 || n_kv_heads < 0 || q_per_kv < 1 || r < 0 || r > d) return SQUAT_E_BADSHAPE;
    if (q_dt != SQUAT_F32 && q_dt != SQUAT_F16 && q_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (n_kv_heads == 0) return SQUAT_OK;
    if (!q || (r > 0 && !qhat)) return SQUAT_E_NULLPTR;
    if (int rc = check_queries(q, q_dt, n_kv_heads, q_per_kv, d, q_stride_head, q_stride_token)) return rc;
    const SubspacePlan pl = plan(n_tokens, n_kv_heads, q_per_kv, kPlanCUs);
    if (!ws || ws_bytes < pl.total) return SQUAT_E_WORKSPACE;
    if (!aligned(ws, 256)) return SQUAT_E_ALIGN;
    if (int rc = raise_lds_limits()) return rc;

    hipStream_t s = static_cast<hipStream_t>(stream);
    double* g64 = reinterpret_cast<double*>(static_cast<unsigned char*>(ws) + pl.off_g64);
    int rc = run_gram(q, q_dt, n_tokens, n_kv_heads, q_per_kv, q_stride_head, q_stride_token, pl, ws, g64, gram, 0, s);
    if (rc || r == 0) return rc;
    return run_exact_solver(g64, n_kv_heads, r, qhat, eig, pl, ws, s);
}

extern "C" size_t squat_refresh_subspace_workspace(int64_t n_new, int n_kv_heads, int q_per_kv, int d, int r) {
    (void)r;
    if (d != kD || n_new < 0 || n_kv_heads < 1 || q_per_kv < 1) return 0;
    // as squat_build_subspace (the slot of its own fp64 Gram matrix stays unused: the state is the caller's)
    return plan(n_new < 1 ? 1 : n_new, n_kv_heads, q_per_kv, kPlanCUs).total;
}

extern "C" int squat_refresh_subspace(const void* q_new, squat_dtype q_dt, int64_t n_new, int n_kv_heads, int q_per_kv,
                                      int d, int64_t q_stride_head, int64_t q_stride_token, int accumulate,
                                      double* gram_state, int r, int iterations, const float* qhat_prev, int r_prev,
                                      float* qhat, float* eig, float* residual, void* ws, size_t ws_bytes,
                                      squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (n_new < 0 || n_kv_heads < 0 || q_per_kv < 1 || r < 0 || r > d || r_prev < 0 || r_prev > kItP)
        return SQUAT_E_BADSHAPE;
    if (iterations >= 0 && r > kItP) return SQUAT_E_BADSHAPE;         // the iteration's block is 32 wide
    if (iterations > 1000) return SQUAT_E_BADSHAPE;
    if (n_new == 0 && !accumulate) return SQUAT_E_BADSHAPE;            // nothing to build the state from
    if (n_kv_heads == 0) return SQUAT_OK;
    if (!gram_state || (r > 0 && !qhat)) return SQUAT_E_NULLPTR;
    if (!aligned(gram_state, 16)) return SQUAT_E_ALIGN;
    if (n_new > 0)
        if (int rc = check_queries(q_new, q_dt, n_kv_heads, q_per_kv, d, q_stride_head, q_stride_token)) return rc;
    const SubspacePlan pl = plan(n_new < 1 ? 1 : n_new, n_kv_heads, q_per_kv, kPlanCUs);
    if (!ws || ws_bytes < pl.total) return SQUAT_E_WORKSPACE;
    if (!aligned(ws, 256)) return SQUAT_E_ALIGN;
    if (int rc = raise_lds_limits()) return rc;

    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = SQUAT_OK;
    if (n_new > 0) {
        rc = run_gram(q_new, q_dt, n_new, n_kv_heads, q_per_kv, q_stride_head, q_stride_token, pl, ws, gram_state,
                      nullptr, accumulate ? 1 : 0, s);
        if (rc) return rc;
    }
    if (r == 0) return rc;
    if (iterations < 0) {
        if (residual) {
            hipLaunchKernelGGL(fill_float, dim3((n_kv_heads + 255) / 256), dim3(256), 0, s, residual, n_kv_heads, 0.0f);
            rc = check_launch();
            if (rc) return rc;
        }
        return run_exact_solver(gram_state, n_kv_heads, r, qhat, eig, pl, ws, s);
    }
    int* need = reinterpret_cast<int*>(static_cast<unsigned char*>(ws) + pl.off_need);
    hipLaunchKernelGGL(subspace_iter_kernel, dim3(n_kv_heads), dim3(kItThreads), kItLdsBytes, s, gram_state,
                       (qhat_prev && r_prev > 0) ? qhat_prev : static_cast<const float*>(nullptr), r_prev, r, iterations,
                       qhat, eig, residual, need);
    rc = check_launch();
    if (rc) return rc;
    // heads whose block broke down (rank-deficient Gram matrix or start block): exact solver, exits at once otherwise
    hipLaunchKernelGGL(eig_kernel, dim3(n_kv_heads), dim3(kEigThreads), kEigLdsBytes, s, gram_state, r, qhat, eig,
                       static_cast<int*>(nullptr), static_cast<const int*>(need));
    return check_launch();
}
