// squat_key_scores_rope: attention logits against keys that were quantized BEFORE
// the rotary position embedding (the pre-RoPE variant of Section 4: the cache
// stores pre-RoPE keys and applies positions on the fly after dequantization),
//     scores[b, hq, t] = out_scale * q . RoPE_{pos0 + t}(deq(code_t)),
// channel pairs (c, c + 64) rotated by (pos0 + t) * inv_freq[c]; per-token store.
//
// The rotation sits between the codes and the contraction, so the codes cannot
// go to the matrix cores raw as in squat_key_scores: every key is dequantized in
// registers (code * Delta + m, fp32), rotated, rounded to fp16 and only then
// multiplied with the fp16 high/low rows of the queries
// (v_mfma_f32_16x16x32_f16, token = column, (query head, part) = row).  This
// kernel is bound by vector arithmetic (270 instructions per 16 tokens against
// about 60 in the unrotated kernel), which is the price of that variant; it
// still never writes a key to memory.
//
// A lane owns, for its token, channels 32 g + 8 kb + i (g < 4, i < 8): both
// members of every rotary pair (chunks g and g + 2), so the rotation needs no
// lane exchange.  cos / sin of the lane's 16 angles are carried in registers
// and advanced by 16 positions per unit with the addition theorems; they are
// seeded per wavefront from fp64 range reduction (position * inv_freq reduced to
// a fraction of a turn before the fp32 sincospi), so the recurrence runs for at
// most ~48 steps (error ~ 1e-5 of a radian, far below the fp16 rounding of the
// rotated key, 2^-11 relative, which sets the accuracy of this call).
//
// squat_key_scores_rope_per_channel is the same computation over the per-channel
// store (statistics per channel over 32 tokens, the grouping Algorithm 1 prints):
// a wavefront takes whole token groups, the lane roles and the arithmetic after
// the dequantize step are unchanged.
//
// Score stores: a 128-byte line of a score row is written by two 16-lane stores;
// they are issued in consecutive instructions (the per-token kernel keeps the
// even unit of a pair in registers until the odd one is done), because halves
// stored a unit of work apart reach memory as two partial line writes.
#include "squat_internal.h"

using namespace squat;

namespace {

constexpr int kRopeDepth = 3;          // units whose loads are in flight per wavefront
#define RP_LOAD(p) __builtin_nontemporal_load(p)

typedef float f32x4v __attribute__((ext_vector_type(4)));

constexpr int kRopeUnit = 16;          // tokens per matrix product (MFMA N)
constexpr int kRopeMaxUnitsPerWave = 32;
constexpr int kRopeMinUnitsPerWave = 4;
constexpr int kRopeWaves = 4;

struct RopeParams {
    const uint32_t* codes;
    const uint16_t* scale;
    const uint16_t* zero;
    const unsigned char* q;
    const float* inv_freq;           // [64]
    int64_t pos0;
    int q_dt;
    int64_t qsb, qsh;                // query strides in ELEMENTS
    float* scores;
    int64_t ssb, ssh;
    int64_t n_tokens;
    int64_t store_stride;            // tokens per (batch, KV head) in the store (>= n_tokens)
    int n_kv_heads;
    int qpk;
    float out_scale;
    int units_per_wave;
};

__device__ __forceinline__ uint32_t pack_h2(_Float16 lo, _Float16 hi) {
    return static_cast<uint32_t>(__builtin_bit_cast(uint16_t, lo)) |
           (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, hi)) << 16);
}

template <int BITS, int NG, int QDT>
__global__ void __launch_bounds__(kRopeWaves* kWave) key_scores_rope_kernel(const RopeParams p) {
    constexpr int WPK = kD * BITS / 32;                   // packed words per key
    constexpr int CPG = 4 / NG;                           // 32-channel chunks per group

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));   // uniform: scalar loop control
    const int kb = lane >> 4;                             // K block of an operand / row block of the result
    const int col = lane & 15;                            // operand row (A) or token (B, result)
    const int64_t bh = static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y;
    const int64_t b = bh / p.n_kv_heads;
    const int kvh = static_cast<int>(bh - b * p.n_kv_heads);

    // ---- the KV head's queries -> LDS as fp32 (rows past q_per_kv zero); rotation of 16 positions per
    // frequency -> LDS
    constexpr int QLD = kD + 1;
    __shared__ float qlds[8 * QLD];
    __shared__ float step_cs[2 * 64];
    {
        const int e0 = 4 * static_cast<int>(threadIdx.x);
        const int qrow = e0 / kD, qch = e0 % kD;
        float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (qrow < p.qpk) {
            const int64_t qoff = b * p.qsb + (static_cast<int64_t>(kvh) * p.qpk + qrow) * p.qsh + qch;
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
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) qlds[qrow * QLD + qch + i] = v[i];
        if (threadIdx.x < 64) {
            float c, s;
            turn_sincos(static_cast<double>(kRopeUnit), p.inv_freq[threadIdx.x], c, s);
            step_cs[2 * threadIdx.x] = c;
            step_cs[2 * threadIdx.x + 1] = s;
        }
    }
    __syncthreads();

    // ---- A operands: row `col` = (query head col / 2, fp16 high / low part col % 2);
    // register r of chunk g holds K = 8 kb + 2 r + {0, 1}  <->  channels 32 g + 8 kb + 2 r + {0, 1}
    const int qh = col >> 1, part = col & 1;
    u32x4 aop[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            _Float16 h[2];
#pragma unroll
            for (int pp = 0; pp < 2; ++pp) {
                const float v = qlds[qh * QLD + 32 * g + 8 * kb + 2 * r + pp];
                const _Float16 hi = static_cast<_Float16>(v);
                h[pp] = part == 0 ? hi : static_cast<_Float16>(v - static_cast<float>(hi));
            }
            aop[g][r] = pack_h2(h[0], h[1]);
        }

    // ---- this wavefront's 16-token units
    const int n_units = static_cast<int>((p.n_tokens + kRopeUnit - 1) / kRopeUnit);
    const int u0 = (static_cast<int>(blockIdx.x) * kRopeWaves + wave) * p.units_per_wave;
    const int u1 = min(u0 + p.units_per_wave, n_units);
    if (u0 >= u1) return;                                 // after the last workgroup barrier

    // rotary state of this lane: frequency index 8 g' + i  <->  channel pair (32 g' + 8 kb + i, + 64)
    float cs[16], sn[16], dc[16], ds[16];
    {
        const double position = static_cast<double>(p.pos0 + static_cast<int64_t>(u0) * kRopeUnit + col);
#pragma unroll
        for (int f = 0; f < 16; ++f) {
            const int ch = 32 * (f >> 3) + 8 * kb + (f & 7);
            turn_sincos(position, p.inv_freq[ch], cs[f], sn[f]);
            dc[f] = step_cs[2 * ch];
            ds[f] = step_cs[2 * ch + 1];
        }
    }

    const int64_t row0 = bh * p.store_stride;
    const int widx0 = BITS == 2 ? (kb >> 1) : kb;         // word of chunk 0 this lane unpacks
    const uint32_t wshift = BITS == 2 ? 16u * (kb & 1) : 0u;
    float* out0 = p.scores + b * p.ssb + (static_cast<int64_t>(kvh) * p.qpk + 2 * kb) * p.ssh;
    const bool st0 = 2 * kb < p.qpk, st1 = 2 * kb + 1 < p.qpk;
    const float fin = p.out_scale;

    // loads: per unit ONE 16-byte load by the lanes that cover the unit's codes and ONE load of the
    // scales and zero-points, through a small per-wavefront LDS tile (as in the unrotated kernel)
    constexpr int PPT = WPK / 4;
    constexpr int CL = kRopeUnit * PPT;
    constexpr int CS = WPK * 4 + 16;
    constexpr int META0 = kRopeUnit * CS;
    constexpr int TILE = META0 + 256;
    __shared__ __attribute__((aligned(16))) unsigned char lds_all[kRopeWaves * TILE];
    unsigned char* lds = lds_all + wave * TILE;
    struct Raw {
        u32x4 c;
        u32x2 m;
    };
    const int n_tok = static_cast<int>(p.n_tokens);
    const int ml = BITS == 2 ? lane - 32 : lane;
    const bool is_c = lane < CL, is_m = ml >= 0 && ml < 32;
    const int c_tok = lane / PPT, c_piece = lane % PPT;
    const int m_tok = ml & 15;
    const uint32_t* c_base = p.codes + row0 * WPK + c_piece * 4;
    const uint16_t* m_base = ((ml & 16) ? p.zero : p.scale) + row0 * NG;
    auto fetch = [&](int u, Raw& r) {
        r.c = u32x4{0u, 0u, 0u, 0u};
        r.m = u32x2{0u, 0u};
        if (is_c) {
            const int t = min(u * kRopeUnit + c_tok, n_tok - 1);
            r.c = RP_LOAD(reinterpret_cast<const u32x4*>(c_base + static_cast<uint32_t>(t) * WPK));
        }
        if (is_m) {
            const int t = min(u * kRopeUnit + m_tok, n_tok - 1);
            if constexpr (NG == 4) {
                r.m = RP_LOAD(reinterpret_cast<const u32x2*>(m_base + static_cast<uint32_t>(t) * 4));
            } else if constexpr (NG == 2) {
                r.m[0] = RP_LOAD(reinterpret_cast<const uint32_t*>(m_base + static_cast<uint32_t>(t) * 2));
            } else {
                r.m[0] = RP_LOAD(m_base + static_cast<uint32_t>(t));
            }
        }
    };

    float held0 = 0.0f, held1 = 0.0f;
    auto compute = [&](int u, const Raw& raw) {
        // registers -> LDS tile -> the words of this lane's K block, the metadata of its token
        if (is_c) *reinterpret_cast<u32x4*>(lds + c_tok * CS + c_piece * 16) = raw.c;
        if (is_m) *reinterpret_cast<u32x2*>(lds + META0 + (ml & 16) * 8 + m_tok * 8) = raw.m;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint32_t w[4];
#pragma unroll
        for (int g = 0; g < 4; ++g)
            w[g] = *reinterpret_cast<const uint32_t*>(lds + col * CS + (g * (WPK / 4) + widx0) * 4) >> wshift;
        const u32x2 sv = *reinterpret_cast<const u32x2*>(lds + META0 + col * 8);
        const u32x2 zv = *reinterpret_cast<const u32x2*>(lds + META0 + 128 + col * 8);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        float sc[NG], zp[NG];
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
            const uint32_t sw = gi < 2 ? sv[0] : sv[1], zw = gi < 2 ? zv[0] : zv[1];
            sc[gi] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>((gi & 1) ? (sw >> 16) : (sw & 0xFFFFu))));
            zp[gi] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>((gi & 1) ? (zw >> 16) : (zw & 0xFFFFu))));
        }
        // dequantize this lane's 32 channels (Section 2: code * Delta + m)
        float k[4][8];
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t code = (w[g] >> (BITS * i)) & ((1u << BITS) - 1u);
                k[g][i] = fmaf(static_cast<float>(code), sc[g / CPG], zp[g / CPG]);
            }
        // rotate the pairs (chunk g', chunk g' + 2), then move the angles on by 16 positions
#pragma unroll
        for (int f = 0; f < 16; ++f) {
            const int g = f >> 3, i = f & 7;
            const float a = k[g][i], bb = k[g + 2][i];
            k[g][i] = fmaf(a, cs[f], -(bb * sn[f]));
            k[g + 2][i] = fmaf(bb, cs[f], a * sn[f]);
            const float c2 = fmaf(cs[f], dc[f], -(sn[f] * ds[f]));
            sn[f] = fmaf(sn[f], dc[f], cs[f] * ds[f]);
            cs[f] = c2;
        }
        f32x4v acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            u32x4 bop;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                bop[r] = pack_h2(static_cast<_Float16>(k[g][2 * r]), static_cast<_Float16>(k[g][2 * r + 1]));
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop[g]), __builtin_bit_cast(half8, bop),
                                                         acc, 0, 0, 0);
        }
        // rows 4 kb + {0, 1}: high and low part of query head 2 kb; rows + {2, 3}: query head 2 kb + 1
        // two consecutive units fill one 128-byte line of a score row: the first of an (even, odd) pair is
        // kept and stored together with the second (a unit apart they reach memory as partial line writes)
        const int tok = u * kRopeUnit + col;
        const float s0 = fin * (acc[0] + acc[1]), s1 = fin * (acc[2] + acc[3]);
        if ((u & 1) == 0 && u + 1 < u1) {
            held0 = s0;
            held1 = s1;
        } else {
            const bool pair = (u & 1) && u > u0;          // the held unit is complete: u exists
            float* const d0 = out0 + tok;
            float* const d1 = d0 + p.ssh;
            if (pair && (u + 1) * kRopeUnit <= n_tok) {
                // the usual case, all tests wave-uniform but the lane's rows: four stores, the two halves
                // of a line in consecutive instructions
                if (st0) {
                    __builtin_nontemporal_store(held0, d0 - kRopeUnit);
                    __builtin_nontemporal_store(s0, d0);
                }
                if (st1) {
                    __builtin_nontemporal_store(held1, d1 - kRopeUnit);
                    __builtin_nontemporal_store(s1, d1);
                }
            } else {
                const bool mine = tok < n_tok;
                if (st0) {
                    if (pair) __builtin_nontemporal_store(held0, d0 - kRopeUnit);
                    if (mine) __builtin_nontemporal_store(s0, d0);
                }
                if (st1) {
                    if (pair) __builtin_nontemporal_store(held1, d1 - kRopeUnit);
                    if (mine) __builtin_nontemporal_store(s1, d1);
                }
            }
        }
    };

    // software pipeline; every unit of the range is computed in order (the angles advance with it)
    Raw ring[kRopeDepth];
#pragma unroll
    for (int i = 0; i < kRopeDepth; ++i) fetch(min(u0 + i, u1 - 1), ring[i]);
    // whole groups of kRopeDepth units run without a test (a skipped unit inside the loop costs a register
    // copy per value the loop carries: the 32 angles); the last, shorter group is handled after it
    int u = u0;
    for (; u + kRopeDepth <= u1; u += kRopeDepth) {
#pragma unroll
        for (int i = 0; i < kRopeDepth; ++i) {
            const Raw cur = ring[i];
            fetch(min(u + i + kRopeDepth, u1 - 1), ring[i]);
            compute(u + i, cur);
        }
    }
    static_assert(kRopeDepth <= 3, "the tail picks its unit from ring[0] / ring[1]");
#pragma nounroll
    for (int i = 0; u + i < u1; ++i) {                    // at most kRopeDepth - 1 units; one copy of the code
        Raw cur = ring[0];
        if (i == 1) cur = ring[1];
        compute(u + i, cur);
    }
}

// The same against the PER-CHANNEL store (statistics per channel over 32 tokens: codes
// [tile][channel][BITS words], token j of the tile at bit BITS * (j mod 32 / BITS) of word j / (32 / BITS);
// scale / zero [tile][channel]).  A wavefront goes over tiles of 32 tokens: the tile's words and metadata come
// in with contiguous 16-byte loads, pass through a wavefront-private LDS tile, and are consumed as two units of
// 16 tokens (lane = token of the unit x K block, as above; the lane's 32 channels each give one word per unit).
// p.n_tokens and p.store_stride are multiples of 32; p.units_per_wave counts TILES here.
template <int BITS, int QDT>
__global__ void __launch_bounds__(kRopeWaves* kWave) key_scores_pc_rope_kernel(const RopeParams p) {
    constexpr int TW = kD * BITS;                         // packed words per tile
    constexpr int NCL = TW / 256;                         // 16-byte code loads per lane and tile
    constexpr int DEPTH = BITS == 4 ? 2 : kRopeDepth;     // tiles in flight (4-bit tiles take twice the registers)

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));   // uniform: scalar loop control
    const int kb = lane >> 4;
    const int col = lane & 15;
    const int64_t bh = static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y;
    const int64_t b = bh / p.n_kv_heads;
    const int kvh = static_cast<int>(bh - b * p.n_kv_heads);

    constexpr int QLD = kD + 1;
    __shared__ float qlds[8 * QLD];
    __shared__ float step_cs[2 * 64];
    {
        const int e0 = 4 * static_cast<int>(threadIdx.x);
        const int qrow = e0 / kD, qch = e0 % kD;
        float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (qrow < p.qpk) {
            const int64_t qoff = b * p.qsb + (static_cast<int64_t>(kvh) * p.qpk + qrow) * p.qsh + qch;
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
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) qlds[qrow * QLD + qch + i] = v[i];
        if (threadIdx.x < 64) {
            float c, s;
            turn_sincos(static_cast<double>(kRopeUnit), p.inv_freq[threadIdx.x], c, s);
            step_cs[2 * threadIdx.x] = c;
            step_cs[2 * threadIdx.x + 1] = s;
        }
    }
    __syncthreads();

    const int qh = col >> 1, part = col & 1;
    u32x4 aop[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            _Float16 h[2];
#pragma unroll
            for (int pp = 0; pp < 2; ++pp) {
                const float v = qlds[qh * QLD + 32 * g + 8 * kb + 2 * r + pp];
                const _Float16 hi = static_cast<_Float16>(v);
                h[pp] = part == 0 ? hi : static_cast<_Float16>(v - static_cast<float>(hi));
            }
            aop[g][r] = pack_h2(h[0], h[1]);
        }

    // ---- this wavefront's tiles
    const int n_tiles = static_cast<int>(p.n_tokens / 32);
    const int t0 = (static_cast<int>(blockIdx.x) * kRopeWaves + wave) * p.units_per_wave;
    const int t1 = min(t0 + p.units_per_wave, n_tiles);
    if (t0 >= t1) return;                                 // after the last workgroup barrier

    float cs[16], sn[16], dc[16], ds[16];
    {
        const double position = static_cast<double>(p.pos0 + static_cast<int64_t>(t0) * 32 + col);
#pragma unroll
        for (int f = 0; f < 16; ++f) {
            const int ch = 32 * (f >> 3) + 8 * kb + (f & 7);
            turn_sincos(position, p.inv_freq[ch], cs[f], sn[f]);
            dc[f] = step_cs[2 * ch];
            ds[f] = step_cs[2 * ch + 1];
        }
    }

    const int64_t tile0 = bh * (p.store_stride / 32);
    float* out0 = p.scores + b * p.ssb + (static_cast<int64_t>(kvh) * p.qpk + 2 * kb) * p.ssh;
    const bool st0 = 2 * kb < p.qpk, st1 = 2 * kb + 1 < p.qpk;
    const float fin = p.out_scale;

    constexpr int TILE_BYTES = TW * 4 + 512;              // words, then 128 scales and 128 zero-points (fp16)
    __shared__ __attribute__((aligned(16))) unsigned char lds_all[kRopeWaves * TILE_BYTES];
    unsigned char* lds = lds_all + wave * TILE_BYTES;
    const uint32_t* ldsw = reinterpret_cast<const uint32_t*>(lds);
    struct Raw {
        u32x4 c[NCL];
        u32x4 m;
    };
    const bool is_m = lane < 32;                          // lanes 0..15: scales, 16..31: zero-points (8 channels each)
    auto fetch = [&](int t, Raw& r) {
        const int64_t tile = tile0 + t;
        const uint32_t* cw = p.codes + tile * TW;
#pragma unroll
        for (int i = 0; i < NCL; ++i) r.c[i] = RP_LOAD(reinterpret_cast<const u32x4*>(cw + (i * 64 + lane) * 4));
        r.m = u32x4{0u, 0u, 0u, 0u};
        if (is_m) {
            const uint16_t* mb = ((lane & 16) ? p.zero : p.scale) + tile * kD + 8 * (lane & 15);
            r.m = RP_LOAD(reinterpret_cast<const u32x4*>(mb));
        }
    };

    auto compute = [&](int t, const Raw& raw) {
#pragma unroll
        for (int i = 0; i < NCL; ++i) *reinterpret_cast<u32x4*>(lds + (i * 64 + lane) * 16) = raw.c[i];
        if (is_m) *reinterpret_cast<u32x4*>(lds + TW * 4 + lane * 16) = raw.m;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // scales and zero-points of this lane's channels 32 g + 8 kb .. + 7 (fp16 pairs)
        u32x4 sraw[4], zraw[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            sraw[g] = *reinterpret_cast<const u32x4*>(lds + TW * 4 + (32 * g + 8 * kb) * 2);
            zraw[g] = *reinterpret_cast<const u32x4*>(lds + TW * 4 + 256 + (32 * g + 8 * kb) * 2);
        }
        float res[2][2];
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            // token 16 hf + col of the tile: word and bit of its code inside a channel's words
            const int widx = BITS == 2 ? hf : 2 * hf + (col >> 3);
            const uint32_t bit = BITS == 2 ? 2u * col : 4u * (col & 7);
            uint32_t w[4][8];
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int i = 0; i < 8; ++i) w[g][i] = ldsw[(32 * g + 8 * kb + i) * BITS + widx];
            float k[4][8];
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t sw = sraw[g][i >> 1], zw = zraw[g][i >> 1];
                    const float sc = static_cast<float>(
                        __builtin_bit_cast(_Float16, static_cast<uint16_t>((i & 1) ? (sw >> 16) : (sw & 0xFFFFu))));
                    const float zp = static_cast<float>(
                        __builtin_bit_cast(_Float16, static_cast<uint16_t>((i & 1) ? (zw >> 16) : (zw & 0xFFFFu))));
                    const uint32_t code = (w[g][i] >> bit) & ((1u << BITS) - 1u);
                    k[g][i] = fmaf(static_cast<float>(code), sc, zp);
                }
#pragma unroll
            for (int f = 0; f < 16; ++f) {
                const int g = f >> 3, i = f & 7;
                const float a = k[g][i], bb = k[g + 2][i];
                k[g][i] = fmaf(a, cs[f], -(bb * sn[f]));
                k[g + 2][i] = fmaf(bb, cs[f], a * sn[f]);
                const float c2 = fmaf(cs[f], dc[f], -(sn[f] * ds[f]));
                sn[f] = fmaf(sn[f], dc[f], cs[f] * ds[f]);
                cs[f] = c2;
            }
            f32x4v acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x4 bop;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    bop[r] = pack_h2(static_cast<_Float16>(k[g][2 * r]), static_cast<_Float16>(k[g][2 * r + 1]));
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop[g]),
                                                             __builtin_bit_cast(half8, bop), acc, 0, 0, 0);
            }
            res[hf][0] = fin * (acc[0] + acc[1]);
            res[hf][1] = fin * (acc[2] + acc[3]);
            __builtin_amdgcn_sched_barrier(0);            // keep the halves apart: interleaved they need > 256 registers
        }
        // both halves of the group's 128-byte line of a score row, back to back
        const int64_t tok = static_cast<int64_t>(t) * 32 + col;
        if (st0) {
            __builtin_nontemporal_store(res[0][0], out0 + tok);
            __builtin_nontemporal_store(res[1][0], out0 + tok + 16);
        }
        if (st1) {
            __builtin_nontemporal_store(res[0][1], out0 + p.ssh + tok);
            __builtin_nontemporal_store(res[1][1], out0 + p.ssh + tok + 16);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    Raw ring[DEPTH];
#pragma unroll
    for (int i = 0; i < DEPTH; ++i) fetch(min(t0 + i, t1 - 1), ring[i]);
    int t = t0;                                           // whole groups of DEPTH tiles, then the shorter last one
    for (; t + DEPTH <= t1; t += DEPTH) {
#pragma unroll
        for (int i = 0; i < DEPTH; ++i) {
            const Raw cur = ring[i];
            fetch(min(t + i + DEPTH, t1 - 1), ring[i]);
            compute(t + i, cur);
        }
    }
    static_assert(DEPTH <= 3, "the tail picks its tile from ring[0] / ring[1]");
#pragma nounroll
    for (int i = 0; t + i < t1; ++i) {                    // at most DEPTH - 1 tiles; one copy of the code
        Raw cur = ring[0];
        if (i == 1) cur = ring[1];
        compute(t + i, cur);
    }
}

template <int BITS>
int launch_pc_dt(const RopeParams& p, dim3 grid, hipStream_t s) {
    const dim3 block(kRopeWaves * kWave);
    switch (p.q_dt) {
        case SQUAT_F32: hipLaunchKernelGGL((key_scores_pc_rope_kernel<BITS, SQUAT_F32>), grid, block, 0, s, p); break;
        case SQUAT_F16: hipLaunchKernelGGL((key_scores_pc_rope_kernel<BITS, SQUAT_F16>), grid, block, 0, s, p); break;
        case SQUAT_BF16: hipLaunchKernelGGL((key_scores_pc_rope_kernel<BITS, SQUAT_BF16>), grid, block, 0, s, p); break;
        default: return SQUAT_E_BADDTYPE;
    }
    return check_launch();
}

template <int BITS, int NG>
int launch_dt(const RopeParams& p, dim3 grid, hipStream_t s) {
    const dim3 block(kRopeWaves * kWave);
    switch (p.q_dt) {
        case SQUAT_F32: hipLaunchKernelGGL((key_scores_rope_kernel<BITS, NG, SQUAT_F32>), grid, block, 0, s, p); break;
        case SQUAT_F16: hipLaunchKernelGGL((key_scores_rope_kernel<BITS, NG, SQUAT_F16>), grid, block, 0, s, p); break;
        case SQUAT_BF16: hipLaunchKernelGGL((key_scores_rope_kernel<BITS, NG, SQUAT_BF16>), grid, block, 0, s, p); break;
        default: return SQUAT_E_BADDTYPE;
    }
    return check_launch();
}

template <int BITS>
int launch_ng(int ng, const RopeParams& p, dim3 grid, hipStream_t s) {
    switch (ng) {
        case 4: return launch_dt<BITS, 4>(p, grid, s);
        case 2: return launch_dt<BITS, 2>(p, grid, s);
        case 1: return launch_dt<BITS, 1>(p, grid, s);
    }
    return SQUAT_E_BADSHAPE;
}

}  // namespace

// squat_key_scores_rope over the first n_tokens tokens of a store that holds store_stride tokens per (batch, KV
// head): what a cache reads with.
int squat::key_scores_rope_from(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t n_batch,
                                int n_kv_heads, int64_t n_tokens, int64_t store_stride, int d, int bits, int group,
                                const float* inv_freq, int64_t pos0, const void* q, squat_dtype q_dt, int q_per_kv,
                                int64_t q_stride_batch, int64_t q_stride_head, float out_scale, float* scores,
                                int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (store_stride < n_tokens) return SQUAT_E_BADSHAPE;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    if (group != 32 && group != 64 && group != 128) return SQUAT_E_BADSHAPE;
    if (q_per_kv < 1 || q_per_kv > 8) return SQUAT_E_BADSHAPE;
    if (n_batch < 0 || n_kv_heads < 0 || n_tokens < 0 || n_tokens >= (int64_t(1) << 25)) return SQUAT_E_BADSHAPE;
    if (pos0 < 0 || pos0 >= (int64_t(1) << 40)) return SQUAT_E_BADSHAPE;
    if (q_dt != SQUAT_F32 && q_dt != SQUAT_F16 && q_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (!(out_scale == out_scale)) return SQUAT_E_BADVALUE;
    if (n_batch == 0 || n_kv_heads == 0 || n_tokens == 0) return SQUAT_OK;
    if (!codes || !scale || !zero || !q || !scores || !inv_freq) return SQUAT_E_NULLPTR;
    if (q_stride_head < d || q_stride_batch < 0 || s_stride_head < n_tokens || s_stride_batch < 0) return SQUAT_E_BADSHAPE;
    if ((q_stride_head % 8) || (q_stride_batch % 8)) return SQUAT_E_ALIGN;
    if (!aligned(codes, 16) || !aligned(scale, 8) || !aligned(zero, 8) || !aligned(scores, 4) || !aligned(q, 16) ||
        !aligned(inv_freq, 4))
        return SQUAT_E_ALIGN;

    RopeParams p;
    p.codes = codes;
    p.scale = scale;
    p.zero = zero;
    p.q = static_cast<const unsigned char*>(q);
    p.inv_freq = inv_freq;
    p.pos0 = pos0;
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

    // workgroups along the sequence: about kRopeWaves * kRopeMaxUnitsPerWave units each, spread evenly
    const int64_t n_units = (n_tokens + kRopeUnit - 1) / kRopeUnit;
    const int64_t slab = static_cast<int64_t>(kRopeWaves) * kRopeMaxUnitsPerWave;
    int64_t gx = (n_units + slab / 2) / slab;
    if (gx < 1) gx = 1;
    int64_t upw = (n_units + kRopeWaves * gx - 1) / (kRopeWaves * gx);
    if (upw < kRopeMinUnitsPerWave) upw = kRopeMinUnitsPerWave;
    upw += upw & 1;                                       // even: every wavefront's range starts on a 32-token line
    p.units_per_wave = static_cast<int>(upw);
    gx = (n_units + kRopeWaves * upw - 1) / (kRopeWaves * upw);
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

extern "C" int squat_key_scores_rope(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                                     int64_t n_batch, int n_kv_heads, int64_t n_tokens, int d, int bits, int group,
                                     const float* inv_freq, int64_t pos0, const void* q, squat_dtype q_dt,
                                     int q_per_kv, int64_t q_stride_batch, int64_t q_stride_head, float out_scale,
                                     float* scores, int64_t s_stride_batch, int64_t s_stride_head,
                                     squat_stream stream) {
    return squat::key_scores_rope_from(codes, scale, zero, n_batch, n_kv_heads, n_tokens, n_tokens, d, bits, group,
                                       inv_freq, pos0, q, q_dt, q_per_kv, q_stride_batch, q_stride_head, out_scale,
                                       scores, s_stride_batch, s_stride_head, stream);
}

// Per-channel store: the first n_tokens tokens (a multiple of 32) of a store that holds store_tokens per (batch, KV head).
int squat::key_scores_pc_rope_from(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t n_batch,
                                   int n_kv_heads, int64_t n_tokens, int64_t store_tokens, int d, int bits, int group,
                                   const float* inv_freq, int64_t pos0, const void* q, squat_dtype q_dt, int q_per_kv,
                                   int64_t q_stride_batch, int64_t q_stride_head, float out_scale, float* scores,
                                   int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    if (group != kTileTokens) return SQUAT_E_BADSHAPE;
    if (q_per_kv < 1 || q_per_kv > 8) return SQUAT_E_BADSHAPE;
    if (n_batch < 0 || n_kv_heads < 0 || n_tokens < 0 || n_tokens >= (int64_t(1) << 25) || n_tokens % group)
        return SQUAT_E_BADSHAPE;
    if (store_tokens < n_tokens || store_tokens % group) return SQUAT_E_BADSHAPE;
    if (pos0 < 0 || pos0 >= (int64_t(1) << 40)) return SQUAT_E_BADSHAPE;
    if (q_dt != SQUAT_F32 && q_dt != SQUAT_F16 && q_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (!(out_scale == out_scale)) return SQUAT_E_BADVALUE;
    if (n_batch == 0 || n_kv_heads == 0 || n_tokens == 0) return SQUAT_OK;
    if (!codes || !scale || !zero || !q || !scores || !inv_freq) return SQUAT_E_NULLPTR;
    if (q_stride_head < d || q_stride_batch < 0 || s_stride_head < n_tokens || s_stride_batch < 0) return SQUAT_E_BADSHAPE;
    if ((q_stride_head % 8) || (q_stride_batch % 8)) return SQUAT_E_ALIGN;
    if (!aligned(codes, 16) || !aligned(scale, 16) || !aligned(zero, 16) || !aligned(scores, 4) || !aligned(q, 16) ||
        !aligned(inv_freq, 4))
        return SQUAT_E_ALIGN;

    RopeParams p;
    p.codes = codes;
    p.scale = scale;
    p.zero = zero;
    p.q = static_cast<const unsigned char*>(q);
    p.inv_freq = inv_freq;
    p.pos0 = pos0;
    p.q_dt = static_cast<int>(q_dt);
    p.qsb = q_stride_batch;
    p.qsh = q_stride_head;
    p.scores = scores;
    p.ssb = s_stride_batch;
    p.ssh = s_stride_head;
    p.n_tokens = n_tokens;
    p.store_stride = store_tokens;
    p.n_kv_heads = n_kv_heads;
    p.qpk = q_per_kv;
    p.out_scale = out_scale;

    // workgroups along the sequence: about kRopeWaves * kRopeMaxUnitsPerWave / 2 tiles each, spread evenly
    const int64_t n_tiles = n_tokens / group;
    const int64_t slab = static_cast<int64_t>(kRopeWaves) * (kRopeMaxUnitsPerWave / 2);
    int64_t gx = (n_tiles + slab / 2) / slab;
    if (gx < 1) gx = 1;
    int64_t tpw = (n_tiles + kRopeWaves * gx - 1) / (kRopeWaves * gx);
    if (tpw < kRopeMinUnitsPerWave / 2) tpw = kRopeMinUnitsPerWave / 2;
    p.units_per_wave = static_cast<int>(tpw);
    gx = (n_tiles + kRopeWaves * tpw - 1) / (kRopeWaves * tpw);
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
    return bits == 2 ? launch_pc_dt<2>(p, grid, s) : launch_pc_dt<4>(p, grid, s);
}

extern "C" int squat_key_scores_rope_per_channel(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                                                 int64_t n_batch, int n_kv_heads, int64_t n_tokens, int d, int bits,
                                                 int group, const float* inv_freq, int64_t pos0, const void* q,
                                                 squat_dtype q_dt, int q_per_kv, int64_t q_stride_batch,
                                                 int64_t q_stride_head, float out_scale, float* scores,
                                                 int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream) {
    return squat::key_scores_pc_rope_from(codes, scale, zero, n_batch, n_kv_heads, n_tokens, n_tokens, d, bits, group,
                                          inv_freq, pos0, q, q_dt, q_per_kv, q_stride_batch, q_stride_head, out_scale,
                                          scores, s_stride_batch, s_stride_head, stream);
}
