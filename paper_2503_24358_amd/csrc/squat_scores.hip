// squat_key_scores: attention logits of decode-time queries against the packed
// key store, out_scale * q . deq(code)^T, without materialising the keys
// (Section 2: deq(c) = c * Delta + m; decoding phase of Algorithm 1: the tokens
// that have left the residual buffer are only available quantized).
//
// Per token and group of channels,  q . deq = Delta * sum_c q_c code_c + m * sum_c q_c.
// The first sum is a small dense contraction and runs on the matrix cores
// (v_mfma_f32_16x16x32_f16: 16 query rows x 16 tokens x 32 channels = one
// quantization group of 32 channels per instruction):
//   - A operand (constant per wavefront): the queries of the KV head's query
//     heads, each split into an fp16 high and low row, so rows = (query head,
//     part); products with the integer codes are then exact.
//   - B operand: the codes themselves.  A packed word is rotated and masked in
//     place: a code at bit position s of a 16-bit half IS the fp16 subnormal
//     number code * 2^(s-24), so two codes become one operand register with a
//     rotate and an and; the power of two is undone in the A operand.  Codes are
//     only taken from bits 6..9 of a half: the matrix cores align products by
//     their exponent FIELDS, and a subnormal with many leading zeros would push
//     its product's low bits out of the adder (measured: 2^-14 relative with
//     codes at bits 0..1, fp32-exact with codes at bits 6..9).
//   - the second sum is one more matrix product per 16 tokens: zero-points (fp16
//     as stored) times the per-group sums of the queries.
// The accumulator puts a token in a lane (column) and the (query head, part)
// rows in its registers, so Delta of the lane's own token scales the four group
// results, high and low rows add inside the lane, and consecutive lanes store
// consecutive tokens of one query head.
#include "squat_internal.h"

using namespace squat;

namespace {

constexpr int kDepth = 4;              // units whose loads are in flight per wavefront (software pipeline)
#define SC_LOAD(p) __builtin_nontemporal_load(p)       // the store is streamed once

typedef float f32x4v __attribute__((ext_vector_type(4)));

constexpr int kUnitTokens = 16;        // tokens per matrix product (MFMA N)
constexpr int kMaxUnitsPerWave = 32;   // 16-token units a wavefront aims at (amortises its operand set-up; up to 1.5x) ...
constexpr int kMinUnitsPerWave = 4;    // ... unless the sequence is short: then all four wavefronts share it
constexpr int kScoreWaves = 4;

struct ScoreParams {
    const uint32_t* codes;
    const uint16_t* scale;
    const uint16_t* zero;
    const unsigned char* q;
    int q_dt;
    int64_t qsb, qsh;                // query strides in ELEMENTS
    float* scores;
    int64_t ssb, ssh;                // score strides in elements
    int64_t n_tokens;
    int64_t store_stride;            // tokens per (batch, KV head) in the store (>= n_tokens)
    int n_kv_heads;
    int qpk;
    float out_scale;
    int units_per_wave;
    int wide_loads;                  // rows of the store are 16-byte aligned: whole units are fetched with 16-byte loads
};

__device__ __forceinline__ uint32_t pack_halves(_Float16 lo, _Float16 hi) {
    return static_cast<uint32_t>(__builtin_bit_cast(uint16_t, lo)) |
           (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, hi)) << 16);
}

// grid: x over slabs of kScoreWaves * units_per_wave units, y / z over (batch, KV head)
template <int BITS, int NG, int QDT>
__global__ void __launch_bounds__(kScoreWaves* kWave) key_scores_kernel(const ScoreParams p) {
    constexpr int WPK = kD * BITS / 32;                   // packed words per key
    constexpr int CPG = 4 / NG;                           // 32-channel chunks per group
    // A code at bit s of a half-word is the fp16 number code * 2^(s - 24); the query side carries
    // 2^(TOP - s), so every product is code * q * 2^(TOP - 24).  2-bit codes are read at s = 6 and 8,
    // 4-bit codes at s = 6.
    constexpr int TOP = BITS == 2 ? 8 : 6;
    constexpr float DESCALE = static_cast<float>(1 << (24 - TOP));

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));   // uniform: scalar loop control
    const int kb = lane >> 4;                             // K block of an operand / row block of the result
    const int col = lane & 15;                            // operand row (A) or token (B, result)
    const int64_t bh = static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y;
    const int64_t b = bh / p.n_kv_heads;
    const int kvh = static_cast<int>(bh - b * p.n_kv_heads);

    // ---- this wavefront's 16-token units; the loads of its first units are issued before anything else, so
    // that their latency overlaps the set-up of the query-side operands
    // 32-bit token indices inside this (batch, KV head): the host rejects sequences of 2^25 tokens or more
    const int n_tok = static_cast<int>(p.n_tokens);
    const int n_units = (n_tok + kUnitTokens - 1) / kUnitTokens;
    const int u0 = (static_cast<int>(blockIdx.x) * kScoreWaves + wave) * p.units_per_wave;
    const int u1 = min(u0 + p.units_per_wave, n_units);
    const int64_t row0 = bh * p.store_stride;
    // A unit's packed words (16 tokens x WPK words, contiguous in memory) and its scales and zero-points (two
    // contiguous runs of 32 NG bytes) pass through a small per-wavefront LDS tile, from which every lane picks
    // the words of its K block and the metadata of its token.
    constexpr int PPT = WPK / 4;                          // 16-byte pieces of codes per token
    constexpr int CL = kUnitTokens * PPT;                 // lanes that load codes (32 or 64)
    constexpr int MP = 2 * NG;                            // 16-byte pieces of scales (and of zero-points) per unit
    constexpr int CS = WPK * 4 + 16;                      // LDS bytes per token of codes (padded)
    constexpr int META0 = kUnitTokens * CS;               // scales: 2 NG bytes per token from META0, zero-points from ZOFF
    constexpr int ZOFF = META0 + MP * 16;
    constexpr int SPARE = META0 + 256;                    // 16 bytes per lane for the lanes with nothing to deliver
    constexpr int TILE = SPARE + kWave * 16;
    // Whole units, in pairs: one 16-byte load per lane and unit (a second one for the metadata of 4-bit stores),
    // contiguous over the wavefront, kDepth units in flight.  Lanes left over after the codes and the metadata
    // repeat a neighbour's load and drop it into a spare LDS slot: no lane tests in the loop.
    const int n_full = n_tok / kUnitTokens;
    int nf = 0;
    if (p.wide_loads) nf = max(min(u1, n_full) - u0, 0) & ~1;
    const int uf = u0 + nf;
    const int ml = BITS == 2 ? (lane - 32) & 31 : lane;   // index among the lanes that may load metadata
    const int mm = ml & (2 * MP - 1);
    const int m_lds = ml < 2 * MP ? META0 + mm * 16 : SPARE + lane * 16;
    const int c_lds = (lane / PPT) * CS + (lane % PPT) * 16;
    // 2-bit: lanes 0..31 deliver codes, lanes 32.. metadata, with one instruction
    const bool code_lane = BITS == 4 || lane < CL;
    const int g_lds = code_lane ? c_lds : m_lds;
    const uint32_t gstep = code_lane ? kUnitTokens * WPK * 4 : kUnitTokens * 2 * NG;
    const unsigned char* mptr;
    const unsigned char* gp;
    {
        const int64_t trow = row0 + static_cast<int64_t>(u0) * kUnitTokens;
        mptr = reinterpret_cast<const unsigned char*>(mm >= MP ? p.zero : p.scale) + trow * (2 * NG) + (mm & (MP - 1)) * 16;
        const unsigned char* cptr = reinterpret_cast<const unsigned char*>(p.codes) + trow * (WPK * 4) + lane * 16;
        gp = code_lane ? cptr : mptr;
    }
    struct Raw {
        u32x4 c;
        u32x4 m;
    };
    Raw ring[kDepth];
    auto fetch = [&](Raw& r) {
        r.c = SC_LOAD(reinterpret_cast<const u32x4*>(gp));
        gp += gstep;
        if constexpr (BITS == 4) {
            r.m = SC_LOAD(reinterpret_cast<const u32x4*>(mptr));
            mptr += kUnitTokens * 2 * NG;
        }
    };
#pragma unroll
    for (int i = 0; i < kDepth; ++i) {
        ring[i].c = u32x4{0u, 0u, 0u, 0u};
        ring[i].m = u32x4{0u, 0u, 0u, 0u};
        if (i < nf) fetch(ring[i]);
    }

    // ---- the KV head's queries -> LDS as fp32 (one wide load per thread instead of 32 two-byte loads per
    // lane: vector-memory instructions are what this kernel runs out of first)
    constexpr int QLD = kD + 1;                           // row stride in floats (odd: spreads the banks)
    __shared__ float qlds[8 * QLD];
    {
        const int e0 = 4 * static_cast<int>(threadIdx.x);            // 4 consecutive channels of one query head
        const int qrow = e0 / kD, qch = e0 % kD;
        if (qrow < p.qpk) {
            const int64_t qoff = b * p.qsb + (static_cast<int64_t>(kvh) * p.qpk + qrow) * p.qsh + qch;
            float v[4];
            if constexpr (QDT == SQUAT_F32) {
                const f32x4 t = *reinterpret_cast<const f32x4*>(p.q + qoff * 4);
                v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
            } else {
                const u32x2 t = *reinterpret_cast<const u32x2*>(p.q + qoff * 2);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t raw = (i & 1) ? (t[i >> 1] >> 16) : (t[i >> 1] & 0xFFFFu);
                    v[i] = QDT == SQUAT_BF16 ? as_f32(raw << 16)
                                             : static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(raw)));
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) qlds[qrow * QLD + qch + i] = v[i];
        }
    }
    __syncthreads();

    // ---- A operands.  Result row 4 kb + i belongs to query head kb + 4 (i >> 1), part i & 1 (high or low
    // half of the fp16 split), so that with up to four query heads every lane of the result holds exactly
    // one of them; K = 8 kb + 2 j + pp.
    const int qh = (col >> 2) + 4 * ((col >> 1) & 1), part = col & 1;
    const bool row_live = qh < p.qpk;
    // Wavefront w builds the operand of chunk w (and that chunk's sum of q per row); the four share them
    // through LDS.
    __shared__ __attribute__((aligned(16))) u32x4 aop_lds[4 * kWave];
    __shared__ float csum_lds[4 * kWave];
    {
        const int g = wave;
        float cs = 0.0f;
        u32x4 a;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            _Float16 h[2];
#pragma unroll
            for (int pp = 0; pp < 2; ++pp) {
                int ch, sh;
                if constexpr (BITS == 2) {
                    ch = 32 * g + 16 * (kb >> 1) + 4 * (kb & 1) + j + 8 * pp;
                    sh = TOP - (6 + 2 * (j & 1));
                } else {
                    ch = 32 * g + 8 * kb + j + 4 * pp;
                    sh = 0;
                }
                const float v = row_live ? qlds[qh * QLD + ch] : 0.0f;
                cs += v;
                const float vs = v * static_cast<float>(1 << sh);
                const _Float16 hi = static_cast<_Float16>(vs);
                h[pp] = part == 0 ? hi : static_cast<_Float16>(vs - static_cast<float>(hi));
            }
            a[j] = pack_halves(h[0], h[1]);
        }
        // all K blocks of the row: lanes col, col + 16, col + 32, col + 48
        cs += __shfl_xor(cs, 16, 64);
        cs += __shfl_xor(cs, 32, 64);
        aop_lds[g * kWave + lane] = a;
        csum_lds[g * kWave + lane] = cs;
    }
    __syncthreads();
    u32x4 aop[4];
    float csum[4];                                        // sum of q over each chunk, for this lane's row
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        aop[g] = aop_lds[g * kWave + lane];
        csum[g] = csum_lds[g * kWave + lane];
    }
    // Zero-points: one more matrix product per unit, K = g.  The B operand is the token's stored zero-points
    // as they lie in memory (K = g in K block 0; the other K blocks hold the same numbers and meet zero rows
    // here); the A operand carries the group sums of q, their fp16 high part in the rows of part 0 and the
    // low part in the rows of part 1, which are added after the product anyway.
    u32x4 azp = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < (NG + 1) / 2; ++i) {
        _Float16 h[2] = {static_cast<_Float16>(0.0f), static_cast<_Float16>(0.0f)};
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int g = 2 * i + e;
            if (g < NG) {
                float s = 0.0f;
#pragma unroll
                for (int c = 0; c < CPG; ++c) s += csum[g * CPG + c];
                const _Float16 hi = static_cast<_Float16>(s);
                h[e] = part == 0 ? hi : static_cast<_Float16>(s - static_cast<float>(hi));
            }
        }
        azp[i] = kb == 0 ? pack_halves(h[0], h[1]) : 0u;
    }

    // ---- stream the units
    if (u0 >= u1) return;
    const int widx0 = BITS == 2 ? (kb >> 1) : kb;          // word of chunk 0 this lane unpacks
    // right-rotations that bring this lane's codes to bits 6..9 of both halves: 2-bit, codes c0, c0 + 1
    // (c0 = 4 (kb & 1), at bits 2 c0) then c0 + 2, c0 + 3; a rotation by 32 - k is a left shift by k
    const uint32_t rot_a = (kb & 1) ? 2u : 26u, rot_b = (kb & 1) ? 6u : 30u;
    const bool two = p.qpk > 4;                           // a lane holds a second query head (kb + 4)
    const bool st0 = kb < p.qpk, st1 = kb + 4 < p.qpk;
    float* const out0 = p.scores + b * p.ssb + (static_cast<int64_t>(kvh) * p.qpk + kb) * p.ssh;
    const int64_t out1 = 4 * p.ssh;
    const float fin = p.out_scale;

    __shared__ __attribute__((aligned(16))) unsigned char lds_all[kScoreWaves * TILE];
    unsigned char* lds = lds_all + wave * TILE;

    // tile -> logits of the lane's token for the lane's query head(s)
    auto unit_scores = [&](float& s0, float& s1) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint32_t w[4];
#pragma unroll
        for (int g = 0; g < 4; ++g)
            w[g] = *reinterpret_cast<const uint32_t*>(lds + col * CS + (g * (WPK / 4) + widx0) * 4);
        uint32_t sraw[2] = {0u, 0u}, zraw[2] = {0u, 0u};
        if constexpr (NG == 4) {
            const u32x2 sv = *reinterpret_cast<const u32x2*>(lds + META0 + col * 8);
            const u32x2 zv = *reinterpret_cast<const u32x2*>(lds + ZOFF + col * 8);
            sraw[0] = sv[0]; sraw[1] = sv[1];
            zraw[0] = zv[0]; zraw[1] = zv[1];
        } else if constexpr (NG == 2) {
            sraw[0] = *reinterpret_cast<const uint32_t*>(lds + META0 + col * 4);
            zraw[0] = *reinterpret_cast<const uint32_t*>(lds + ZOFF + col * 4);
        } else {
            sraw[0] = *reinterpret_cast<const uint16_t*>(lds + META0 + col * 2);
            zraw[0] = *reinterpret_cast<const uint16_t*>(lds + ZOFF + col * 2);
        }
        // the next unit's tile must not overtake these reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        f32x4v acc[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g] = f32x4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            u32x4 bop;
            if constexpr (BITS == 2) {
                const uint32_t wa = __builtin_amdgcn_alignbit(w[g], w[g], rot_a);
                const uint32_t wb = __builtin_amdgcn_alignbit(w[g], w[g], rot_b);
                bop = u32x4{wa & 0x00C000C0u, wa & 0x03000300u, wb & 0x00C000C0u, wb & 0x03000300u};
            } else {
                // code j (and j + 4 in the upper half) sits at bit 4 j: rotate it to bit 6
                bop = u32x4{__builtin_amdgcn_alignbit(w[g], w[g], 26u) & 0x03C003C0u,
                            __builtin_amdgcn_alignbit(w[g], w[g], 30u) & 0x03C003C0u,
                            __builtin_amdgcn_alignbit(w[g], w[g], 2u) & 0x03C003C0u,
                            __builtin_amdgcn_alignbit(w[g], w[g], 6u) & 0x03C003C0u};
            }
            acc[g / CPG] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop[g]),
                                                                  __builtin_bit_cast(half8, bop), acc[g / CPG], 0, 0, 0);
        }
        const u32x4 zop = {zraw[0], zraw[1], 0u, 0u};
        f32x4v zacc = {0.0f, 0.0f, 0.0f, 0.0f};
        zacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, azp), __builtin_bit_cast(half8, zop),
                                                      zacc, 0, 0, 0);
        // Delta of this lane's token scales each group's result.  The conversions are kept apart from the
        // multiply-adds on purpose: the mixed-precision multiply-add the compiler would fuse them into issues
        // at half the rate of a plain one.
        float sc[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const uint32_t word = sraw[g >> 1];
            sc[g] = static_cast<float>(
                __builtin_bit_cast(_Float16, static_cast<uint16_t>((g & 1) ? (word >> 16) : (word & 0xFFFFu))));
            asm volatile("" : "+v"(sc[g]));
        }
        // rows 4 kb + {0, 1}: high and low part of query head kb; rows + {2, 3}: query head kb + 4
        {
            float r0 = sc[0] * acc[0][0], r1 = sc[0] * acc[0][1];
#pragma unroll
            for (int g = 1; g < NG; ++g) {
                r0 = fmaf(sc[g], acc[g][0], r0);
                r1 = fmaf(sc[g], acc[g][1], r1);
            }
            s0 = fin * (fmaf(DESCALE, r0 + r1, zacc[0] + zacc[1]));
        }
        if (two) {
            float r2 = sc[0] * acc[0][2], r3 = sc[0] * acc[0][3];
#pragma unroll
            for (int g = 1; g < NG; ++g) {
                r2 = fmaf(sc[g], acc[g][2], r2);
                r3 = fmaf(sc[g], acc[g][3], r3);
            }
            s1 = fin * (fmaf(DESCALE, r2 + r3, zacc[2] + zacc[3]));
        }
    };

    // ---- whole units, in pairs
    if (nf > 0) {
        auto deliver = [&](const Raw& r) {
            *reinterpret_cast<u32x4*>(lds + g_lds) = r.c;
            if constexpr (BITS == 4) *reinterpret_cast<u32x4*>(lds + m_lds) = r.m;
        };
        float* optr = out0 + static_cast<int64_t>(u0) * kUnitTokens + col;
        float held0 = 0.0f, held1 = 0.0f;
        // Two consecutive units fill one 128-byte line of a score row: the first unit of a pair keeps its results
        // until the second one is done, and both halves are stored back to back (stored a unit apart, the halves
        // reach memory as two partial line writes).
        auto pair_step = [&](int i, bool more) {
            float s0 = 0.0f, s1 = 0.0f;
            deliver(ring[i]);
            if (more) fetch(ring[i]);
            unit_scores(s0, s1);
            if ((i & 1) == 0) {
                held0 = s0;
                held1 = s1;
            } else {
                if (st0) {
                    __builtin_nontemporal_store(held0, optr);
                    __builtin_nontemporal_store(s0, optr + kUnitTokens);
                }
                if (st1) {
                    __builtin_nontemporal_store(held1, optr + out1);
                    __builtin_nontemporal_store(s1, optr + out1 + kUnitTokens);
                }
                optr += 2 * kUnitTokens;
            }
        };
        static_assert(kDepth % 2 == 0, "pairs of units");
        int u = u0;
        for (; u + kDepth <= uf; u += kDepth) {
#pragma unroll
            for (int i = 0; i < kDepth; ++i) pair_step(i, u + i + kDepth < uf);
        }
        // nf is even: an even number of units below kDepth is left, all of them in flight
#pragma unroll
        for (int i = 0; i < kDepth - 2; i += 2) {
            if (u + i < uf) {
                pair_step(i, false);
                pair_step(i + 1, false);
            }
        }
    }

    // ---- what is left: a single unit after the pairs, the ragged end of the sequence, or everything when the
    // store's rows are not aligned for the wide loads.  Every lane fetches for itself; rows past the end of the
    // keys re-read the last key and are not stored.
    {
        const int sl = BITS == 2 ? lane - 32 : lane;          // index among the lanes that load metadata
        const bool is_c = lane < CL, is_m = sl >= 0 && sl < 32;
        const int c_tok = lane / PPT, c_piece = lane % PPT;
        const int m_tok = sl & 15;
        const uint32_t* c_base = p.codes + row0 * WPK + c_piece * 4;
        const uint16_t* m_base = ((sl & 16) ? p.zero : p.scale) + row0 * NG;
        unsigned char* m_dst = lds + ((sl & 16) ? ZOFF : META0) + m_tok * (2 * NG);
#pragma nounroll
        for (int u = uf; u < u1; ++u) {
            if (is_c) {
                const int t = min(u * kUnitTokens + c_tok, n_tok - 1);
                *reinterpret_cast<u32x4*>(lds + c_tok * CS + c_piece * 16) =
                    SC_LOAD(reinterpret_cast<const u32x4*>(c_base + static_cast<uint32_t>(t) * WPK));
            }
            if (is_m) {
                const int t = min(u * kUnitTokens + m_tok, n_tok - 1);
                if constexpr (NG == 4) {
                    *reinterpret_cast<u32x2*>(m_dst) =
                        SC_LOAD(reinterpret_cast<const u32x2*>(m_base + static_cast<uint32_t>(t) * 4));
                } else if constexpr (NG == 2) {
                    *reinterpret_cast<uint32_t*>(m_dst) =
                        SC_LOAD(reinterpret_cast<const uint32_t*>(m_base + static_cast<uint32_t>(t) * 2));
                } else {
                    *reinterpret_cast<uint16_t*>(m_dst) = SC_LOAD(m_base + static_cast<uint32_t>(t));
                }
            }
            float s0 = 0.0f, s1 = 0.0f;
            unit_scores(s0, s1);
            const int tok = u * kUnitTokens + col;
            if (tok < n_tok) {
                if (st0) __builtin_nontemporal_store(s0, out0 + tok);
                if (st1) __builtin_nontemporal_store(s1, out0 + out1 + tok);
            }
        }
    }
}

template <int BITS, int NG>
int launch_dt(const ScoreParams& p, dim3 grid, hipStream_t s) {
    const dim3 block(kScoreWaves * kWave);
    switch (p.q_dt) {
        case SQUAT_F32: hipLaunchKernelGGL((key_scores_kernel<BITS, NG, SQUAT_F32>), grid, block, 0, s, p); break;
        case SQUAT_F16: hipLaunchKernelGGL((key_scores_kernel<BITS, NG, SQUAT_F16>), grid, block, 0, s, p); break;
        case SQUAT_BF16: hipLaunchKernelGGL((key_scores_kernel<BITS, NG, SQUAT_BF16>), grid, block, 0, s, p); break;
        default: return SQUAT_E_BADDTYPE;
    }
    return check_launch();
}

template <int BITS>
int launch_ng(int ng, const ScoreParams& p, dim3 grid, hipStream_t s) {
    switch (ng) {
        case 4: return launch_dt<BITS, 4>(p, grid, s);
        case 2: return launch_dt<BITS, 2>(p, grid, s);
        case 1: return launch_dt<BITS, 1>(p, grid, s);
    }
    return SQUAT_E_BADSHAPE;
}

}  // namespace

// squat_key_scores over the first n_tokens tokens of a store that holds store_stride tokens per
// (batch, KV head).
int squat::key_scores_from(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t n_batch,
                           int n_kv_heads, int64_t n_tokens, int64_t store_stride, int d, int bits, int group,
                           const void* q, squat_dtype q_dt, int q_per_kv, int64_t q_stride_batch,
                           int64_t q_stride_head, float out_scale, float* scores, int64_t s_stride_batch,
                           int64_t s_stride_head, squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    if (group != 32 && group != 64 && group != 128) return SQUAT_E_BADSHAPE;
    if (q_per_kv < 1 || q_per_kv > 8) return SQUAT_E_BADSHAPE;
    if (n_batch < 0 || n_kv_heads < 0 || n_tokens < 0 || n_tokens >= (int64_t(1) << 25)) return SQUAT_E_BADSHAPE;
    if (store_stride < n_tokens) return SQUAT_E_BADSHAPE;
    if (q_dt != SQUAT_F32 && q_dt != SQUAT_F16 && q_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (!(out_scale == out_scale)) return SQUAT_E_BADVALUE;
    if (n_batch == 0 || n_kv_heads == 0 || n_tokens == 0) return SQUAT_OK;
    if (!codes || !scale || !zero || !q || !scores) return SQUAT_E_NULLPTR;
    if (q_stride_head < d || q_stride_batch < 0 || s_stride_head < n_tokens || s_stride_batch < 0) return SQUAT_E_BADSHAPE;
    if ((q_stride_head % 8) || (q_stride_batch % 8)) return SQUAT_E_ALIGN;
    if (!aligned(codes, 16) || !aligned(scale, 8) || !aligned(zero, 8) || !aligned(scores, 4) || !aligned(q, 16))
        return SQUAT_E_ALIGN;

    ScoreParams p;
    p.codes = codes;
    p.scale = scale;
    p.zero = zero;
    p.q = static_cast<const unsigned char*>(q);
    p.q_dt = static_cast<int>(q_dt);
    p.qsb = q_stride_batch;
    p.qsh = q_stride_head;
    p.scores = scores;
    p.ssb = s_stride_batch;
    p.ssh = s_stride_head;
    p.n_tokens = n_tokens;
    p.store_stride = store_stride;
    p.n_kv_heads = n_kv_heads;
    p.qpk = q_per_kv;
    p.out_scale = out_scale;
    {
        const int64_t meta_row = 2 * (128 / group);       // bytes of scales (or zero-points) per key
        p.wide_loads = (store_stride * meta_row) % 16 == 0 && aligned(scale, 16) && aligned(zero, 16);
    }

    const int64_t n_units = (n_tokens + kUnitTokens - 1) / kUnitTokens;
    // Workgroups along the sequence: about kScoreWaves * kMaxUnitsPerWave units each, the count rounded to
    // nearest and the units then spread evenly, so that no workgroup pays the operand set-up for a sliver
    // (2080 tokens = 130 units used to run as 128 + 2 and took 60 % longer than 2048 tokens).
    const int64_t slab = static_cast<int64_t>(kScoreWaves) * kMaxUnitsPerWave;
    int64_t gx = (n_units + slab / 2) / slab;
    if (gx < 1) gx = 1;
    int64_t upw = (n_units + kScoreWaves * gx - 1) / (kScoreWaves * gx);
    if (upw < kMinUnitsPerWave) upw = kMinUnitsPerWave;
    upw += upw & 1;                                       // even: every wavefront's range starts on a 32-token line
    p.units_per_wave = static_cast<int>(upw);
    gx = (n_units + kScoreWaves * upw - 1) / (kScoreWaves * upw);
    const int64_t bh = n_batch * n_kv_heads;
    int64_t gy = bh, gz = 1;
    if (gy > 65535) {
        gy = 0;
        for (int64_t cand = 65535; cand >= 1; --cand)
            if (bh % cand == 0) { gy = cand; break; }
        gz = bh / gy;
    }
    if (gx > 0x7FFFFFFF || gz > 65535) return SQUAT_E_BADSHAPE;
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy), static_cast<unsigned>(gz));
    hipStream_t s = static_cast<hipStream_t>(stream);
    return bits == 2 ? launch_ng<2>(128 / group, p, grid, s) : launch_ng<4>(128 / group, p, grid, s);
}

extern "C" int squat_key_scores(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                                int64_t n_batch, int n_kv_heads, int64_t n_tokens, int d, int bits, int group,
                                const void* q, squat_dtype q_dt, int q_per_kv, int64_t q_stride_batch,
                                int64_t q_stride_head, float out_scale, float* scores,
                                int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream) {
    return squat::key_scores_from(codes, scale, zero, n_batch, n_kv_heads, n_tokens, n_tokens, d, bits, group, q,
                                  q_dt, q_per_kv, q_stride_batch, q_stride_head, out_scale, scores,
                                  s_stride_batch, s_stride_head, stream);
}
