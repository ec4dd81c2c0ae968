// squat_key_scores_rope: attention logits against keys that were quantized BEFORE
// the rotary position embedding (the pre-RoPE variant of Section 4: the cache
// stores pre-RoPE keys and applies positions on the fly after dequantization),
//     scores[b, hq, t] = out_scale * q . RoPE_{pos0 + t}(deq(code_t)),
// channel pairs (c, c + 64) rotated by (pos0 + t) * inv_freq[c]; per-token store.
//
// The rotation sits between the codes and the contraction, so the codes cannot
// go to the matrix cores raw as in squat_key_scores: every key is dequantized
// and rotated in registers and only then multiplied with the fp16 high/low rows
// of the queries (v_mfma_f32_16x16x32_f16, token = column, (query head, part) =
// row).  The kernels are bound by vector arithmetic (about 160 instructions per 16
// tokens against about 90 in the unrotated kernel), which is the price of that
// variant; they still never write a key to memory.  How the arithmetic is kept
// that small (angle split into a per-epoch and a per-token part, packed fp16 on
// rotary pairs) is described at the shared pieces below.
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
#include <type_traits>

#include "squat_internal.h"

using namespace squat;

namespace {

constexpr int kRopeDepth = 3;          // units whose loads are in flight per wavefront
#define RP_LOAD(p) __builtin_nontemporal_load(p)

typedef float f32x4v __attribute__((ext_vector_type(4)));

constexpr int kRopeUnit = 16;          // tokens per matrix product (MFMA N)
constexpr int kRopeMaxUnitsPerWave = 64;
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
    int wide_loads;                  // per-token store: rows 16-byte aligned, whole units fetched with 16-byte loads
};

__device__ __forceinline__ uint32_t pack_h2(_Float16 lo, _Float16 hi) {
    return static_cast<uint32_t>(__builtin_bit_cast(uint16_t, lo)) |
           (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, hi)) << 16);
}

// ---- shared pieces of the two kernels -----------------------------------------------------------------------
//
// Angle of token t and frequency f:  (pos0 + t) f = theta_E + theta_l  with E the first token of t's EPOCH of 64
// tokens and l = t - E.  R(theta) = R(theta_E) R(theta_l), and  q . R(theta) k = (R(-theta_E) q) . (R(theta_l) k):
//   - key side: theta_l runs over 64 x 64 fixed values, the same for every epoch, wavefront and position offset:
//     their (cos, sin) sit in an LDS table as packed fp16 pairs, filled once per workgroup;
//   - query side: R(-theta_E) q is rebuilt once per epoch and wavefront in fp32 (cos / sin of theta_E advance by the
//     addition theorems, seeded from an fp64 range reduction), split into exact fp16 high / low parts, and becomes
//     the A operand of the epoch's matrix products.
// The key itself is dequantized and rotated in PACKED fp16: a register holds a rotary pair (k_c, k_{c+64}) of the
// lane's token, so x' = (a cos - b sin, b cos + a sin) is one packed multiply and one packed multiply-add on the
// pair and its swapped copy, and the result is the B operand as it stands (the contraction index is ordered
// pair by pair on both sides).  Rounding: the dequantized value, the table entries, the product and the result are
// each rounded to fp16: |error of x'| <= 4 * 2^-11 * sqrt(a^2 + b^2) in the worst case (typically a quarter of it).
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

constexpr int kEpochUnits = 4;                 // units of 16 tokens that share one query-side operand
constexpr int kEpochTokens = kEpochUnits * kRopeUnit;
constexpr int kTrigLd = 68;                    // words per table row (64 + 4: 16-byte lane reads fall on distinct banks)
constexpr int kATileLd = 68;                   // words per row of the A-operand exchange tile
constexpr float kCodeScale = 512.0f;           // codes enter the multiply-add as code * 2^-9, the scales times 2^9

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t h2_bits(h2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ uint32_t pack_rne(float lo, float hi) {
    return pack_h2(static_cast<_Float16>(lo), static_cast<_Float16>(hi));
}

// (a cos - b sin, b cos + a sin) for the pair x = (a, b) and cs = (cos, sin)
__device__ __forceinline__ h2 rotate_pair(h2 x, h2 cs) {
    const h2 cc = __builtin_shufflevector(cs, cs, 0, 0);
    const h2 sw = __builtin_shufflevector(x, x, 1, 0);
    const h2 ss = {-cs[1], cs[1]};
    return __builtin_elementwise_fma(sw, ss, x * cc);
}

// Word index of frequency f inside a row of the LDS tables: lane K-block kb = (f >> 3) & 3 first, then the
// 32-channel chunk g = f >> 5, then i = f & 7, so that the 16 entries of one lane are 64 contiguous bytes.
__device__ __forceinline__ int freq_slot(int f) { return ((f >> 3) & 3) * 16 + (f >> 5) * 8 + (f & 7); }

// Fills the key-side table trig[l][slot(f)] = (cos, sin)(l * inv_freq[f]) and step64[f] = (cos, sin)(64 inv_freq[f]).
// 256 threads; thread (f, quarter) covers l = 16 quarter .. + 15 by the addition theorems from an fp64-reduced start.
__device__ __forceinline__ void fill_trig_tables(const float* inv_freq, uint32_t* trig, float* step64) {
    const int f = threadIdx.x & 63, quarter = threadIdx.x >> 6;
    const float fr = inv_freq[f];
    float c, s, c1, s1;
    turn_sincos(static_cast<double>(16 * quarter), fr, c, s);
    turn_sincos(1.0, fr, c1, s1);
    const int slot = freq_slot(f);
#pragma unroll 4
    for (int l = 0; l < 16; ++l) {
        trig[(16 * quarter + l) * kTrigLd + slot] = pack_rne(c, s);
        const float c2 = fmaf(c, c1, -(s * s1));
        s = fmaf(s, c1, c * s1);
        c = c2;
    }
    if (quarter == 0) {
        float ce, se;
        turn_sincos(static_cast<double>(kEpochTokens), fr, ce, se);
        step64[2 * f] = ce;
        step64[2 * f + 1] = se;
    }
}

// Query side of one wavefront.  With more than four query heads per KV head lane (h = lane >> 3, fb = lane & 7)
// owns the NF = 8 pairs (q_h[f], q_h[f + 64]), f = 8 fb + i; with at most four (the usual grouped-query case) lane
// (h = lane >> 4, fb = lane & 15) owns NF = 4 pairs, f = 4 fb + i, and the rows of query heads 4 .. 7 stay zero (WIDE,
// a template parameter: the narrow form keeps half the state in registers).  `build`
// writes R(-theta_E) q as fp16 high (row 4 (h & 3) + 2 (h >> 2)) and low (the row after it) parts into the
// wavefront's exchange tile (so that result lane block kb holds query heads kb and kb + 4), from
// which every lane reads the 16 registers of its A operands.
template <bool WIDE>
struct QuerySide {
    static constexpr int NF = WIDE ? 8 : 4;
    float ce[NF], se[NF];        // cos / sin of theta_E (the only state that lives across epochs)
    const float* qrow;           // this lane's query head in LDS (fp32)
    const float* step;           // (cos, sin) of one epoch's rotation (64 positions) per frequency, LDS
    int f0;                      // first frequency of this lane

    __device__ __forceinline__ void init(const float* qlds, int qld, const float* step64, const float* inv_freq,
                                         double position, int lane, int qpk, uint32_t* atile) {
        (void)qpk;
        const int h = WIDE ? lane >> 3 : lane >> 4;
        f0 = WIDE ? 8 * (lane & 7) : 4 * (lane & 15);
        qrow = qlds + h * qld;
        step = step64;
#pragma unroll
        for (int i = 0; i < NF; ++i) turn_sincos(position, inv_freq[f0 + i], ce[i], se[i]);
        // rows that `build` never writes (query heads past 4 in the narrow form) must read as zero
        for (int idx = lane; idx < 16 * kATileLd; idx += kWave) atile[idx] = 0u;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    __device__ __forceinline__ void rotate_and_store(uint32_t* dst) {
        uint32_t hi[NF], lo[NF];
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            const float qa = qrow[f0 + i], qb = qrow[64 + f0 + i];
            const float dc = step[2 * (f0 + i)], ds = step[2 * (f0 + i) + 1];
            // R(-theta): (a cos + b sin, b cos - a sin)
            const float ra = fmaf(qa, ce[i], qb * se[i]);
            const float rb = fmaf(qb, ce[i], -(qa * se[i]));
            const auto hv = __builtin_amdgcn_cvt_pkrtz(ra, rb);
            hi[i] = __builtin_bit_cast(uint32_t, hv);
            lo[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(ra - static_cast<float>(hv[0]),
                                                                            rb - static_cast<float>(hv[1])));
            const float c2 = fmaf(ce[i], dc, -(se[i] * ds));
            se[i] = fmaf(se[i], dc, ce[i] * ds);
            ce[i] = c2;
        }
#pragma unroll
        for (int i = 0; i < NF; i += 4) {
            *reinterpret_cast<u32x4*>(dst + i) = u32x4{hi[i], hi[i + 1], hi[i + 2], hi[i + 3]};
            *reinterpret_cast<u32x4*>(dst + kATileLd + i) = u32x4{lo[i], lo[i + 1], lo[i + 2], lo[i + 3]};
        }
    }
    // A operands of the epoch whose angles are current, then the angles move on by one epoch
    __device__ __forceinline__ void build(uint32_t* atile, int lane, u32x4 (&aop)[4]) {
        if constexpr (WIDE) {
            // frequencies 8 fb .. 8 fb + 7 are K-block fb & 3, chunk fb >> 2: 8 consecutive words of a row
            const int h = lane >> 3, fb = lane & 7;
            rotate_and_store(atile + (4 * (h & 3) + 2 * (h >> 2)) * kATileLd + (fb & 3) * 16 + (fb >> 2) * 8);
        } else {
            // frequencies 4 fb .. 4 fb + 3: K-block (fb >> 1) & 3, chunk fb >> 3, pairs 4 (fb & 1) .. + 3
            const int h = lane >> 4, fb = lane & 15;
            rotate_and_store(atile + (4 * h) * kATileLd + ((fb >> 1) & 3) * 16 + (fb >> 3) * 8 + (fb & 1) * 4);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint32_t* src = atile + (lane & 15) * kATileLd + (lane >> 4) * 16;
#pragma unroll
        for (int m = 0; m < 4; ++m) aop[m] = *reinterpret_cast<const u32x4*>(src + 4 * m);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
};

// Loads the KV head's queries into LDS as fp32 (rows past q_per_kv zero).  256 threads, 8 x 128 values.
template <int QDT>
__device__ __forceinline__ void stage_queries(const RopeParams& p, int64_t b, int kvh, float* qlds, int qld) {
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
    for (int i = 0; i < 4; ++i) qlds[qrow * qld + qch + i] = v[i];
}

// Per-token store.  Lane (kb = lane >> 4, col = lane & 15): token col of the unit, rotary pairs
// (32 g + 8 kb + i, + 64), g < 2, i < 8.  Matrix product m = 2 g + (i >> 2) takes the pairs i & 3 = 0..3 of chunk g
// as its K slots 8 kb .. 8 kb + 7 (both operands), rows = (query head, fp16 high / low part).
// (Registers are capped at three wavefronts per SIMD: the 4-bit forms for more than four query heads per KV head
// would otherwise take a few more and run two, 6 % slower.)
template <int BITS, int NG, int QDT, bool WIDE>
__global__ void __launch_bounds__(kRopeWaves* kWave) __attribute__((amdgpu_waves_per_eu(3)))
key_scores_rope_kernel(const RopeParams p) {
    constexpr int WPK = kD * BITS / 32;                   // packed words per key
    constexpr int CPR = 8 / BITS;                         // codes of a pair register whose bits stay below bit 8 of a half
    constexpr int NSRC = 8 / CPR;                         // such source registers per chunk pair: 2 (2-bit), 4 (4-bit)

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));   // uniform: scalar loop control
    const int kb = lane >> 4;
    const int col = lane & 15;
    const int64_t bh = static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y;
    const int64_t b = bh / p.n_kv_heads;
    const int kvh = static_cast<int>(bh - b * p.n_kv_heads);

    // ---- this wavefront's 16-token units (whole epochs; the range starts on an epoch boundary).  The loads of its
    // first units are issued before anything else: their latency overlaps the set-up of queries and tables.
    const int n_tok = static_cast<int>(p.n_tokens);
    const int n_units = (n_tok + kRopeUnit - 1) / kRopeUnit;
    const int u0 = (static_cast<int>(blockIdx.x) * kRopeWaves + wave) * p.units_per_wave;
    const int u1 = min(u0 + p.units_per_wave, n_units);
    const int64_t row0 = bh * p.store_stride;
    // A unit's packed words (contiguous in memory) and its scales and zero-points (two contiguous runs of 32 NG
    // bytes) pass through a small per-wavefront LDS tile, as in the unrotated kernel: whole units with one 16-byte
    // load per lane (a second one for the metadata of 4-bit stores) and no lane tests; lanes left over repeat a
    // neighbour's load and drop it into a spare LDS slot.
    constexpr int PPT = WPK / 4;                          // 16-byte pieces of codes per token
    constexpr int CL = kRopeUnit * PPT;                   // lanes that load codes (32 or 64)
    constexpr int MP = 2 * NG;                            // 16-byte pieces of scales (and of zero-points) per unit
    constexpr int CS = WPK * 4 + 16;                      // LDS bytes per token of codes (padded)
    constexpr int META0 = kRopeUnit * CS;                 // scales: 2 NG bytes per token from META0, zero-points from ZOFF
    constexpr int ZOFF = META0 + MP * 16;
    constexpr int SPARE = META0 + 256;
    constexpr int TILE = SPARE + kWave * 16;
    const int n_full = n_tok / kRopeUnit;
    int nf = 0;
    if (p.wide_loads) nf = max(min(u1, n_full) - u0, 0) & ~1;
    const int uf = u0 + nf;
    const int ml = BITS == 2 ? (lane - 32) & 31 : lane;   // index among the lanes that may load metadata
    const int mm = ml & (2 * MP - 1);
    const int m_lds = ml < 2 * MP ? META0 + mm * 16 : SPARE + lane * 16;
    const int c_lds = (lane / PPT) * CS + (lane % PPT) * 16;
    const bool code_lane = BITS == 4 || lane < CL;        // 2-bit: lanes 0..31 deliver codes, lanes 32.. metadata
    const int g_lds = code_lane ? c_lds : m_lds;
    const uint32_t gstep = code_lane ? kRopeUnit * WPK * 4 : kRopeUnit * 2 * NG;
    const unsigned char* mptr;
    const unsigned char* gp;
    {
        const int64_t trow = row0 + static_cast<int64_t>(u0) * kRopeUnit;
        mptr = reinterpret_cast<const unsigned char*>(mm >= MP ? p.zero : p.scale) + trow * (2 * NG) + (mm & (MP - 1)) * 16;
        const unsigned char* cptr = reinterpret_cast<const unsigned char*>(p.codes) + trow * (WPK * 4) + lane * 16;
        gp = code_lane ? cptr : mptr;
    }
    struct Raw {
        u32x4 c;
        u32x4 m;
    };
    Raw ring[kEpochUnits];
    auto fetch = [&](Raw& r) {
        r.c = RP_LOAD(reinterpret_cast<const u32x4*>(gp));
        gp += gstep;
        if constexpr (BITS == 4) {
            r.m = RP_LOAD(reinterpret_cast<const u32x4*>(mptr));
            mptr += kRopeUnit * 2 * NG;
        }
    };
#pragma unroll
    for (int i = 0; i < kEpochUnits; ++i) {
        ring[i].c = u32x4{0u, 0u, 0u, 0u};
        ring[i].m = u32x4{0u, 0u, 0u, 0u};
        if (i < nf) fetch(ring[i]);
    }

    constexpr int QLD = kD + 1;
    __shared__ float qlds[8 * QLD];
    __shared__ float step64[2 * 64];
    __shared__ __attribute__((aligned(16))) uint32_t trig[kEpochTokens * kTrigLd];
    __shared__ __attribute__((aligned(16))) uint32_t atiles[kRopeWaves * 16 * kATileLd];
    stage_queries<QDT>(p, b, kvh, qlds, QLD);
    fill_trig_tables(p.inv_freq, trig, step64);
    __syncthreads();
    if (u0 >= u1) return;                                 // after the last workgroup barrier

    uint32_t* atile = atiles + wave * 16 * kATileLd;
    QuerySide<WIDE> qs;
    qs.init(qlds, QLD, step64, p.inv_freq, static_cast<double>(p.pos0 + static_cast<int64_t>(u0) * kRopeUnit), lane,
            p.qpk, atile);

    // result rows 4 kb + {0, 1}: high and low part of query head kb; rows + {2, 3}: query head kb + 4
    constexpr bool two = WIDE;
    const bool st0 = kb < p.qpk, st1 = kb + 4 < p.qpk;
    float* const out0 = p.scores + b * p.ssb + (static_cast<int64_t>(kvh) * p.qpk + kb) * p.ssh;
    const int64_t out1 = 4 * p.ssh;
    const float fin = p.out_scale;

    __shared__ __attribute__((aligned(16))) unsigned char lds_all[kRopeWaves * TILE];
    unsigned char* lds = lds_all + wave * TILE;

    // where this lane's codes sit: 2-bit: 16 bits (one half of a word) per chunk; 4-bit: one word per chunk
    const int widx0 = BITS == 2 ? (kb >> 1) : kb;
    const uint32_t half_sel = (kb & 1) ? 0x07060302u : 0x05040100u;       // v_perm: (hi : lo) <- the same half of both words

    u32x4 aop[4];
    // LDS tile -> logits of the lane's token (unit v of the epoch) for the lane's query head(s)
    auto unit_scores = [&](int v, float& s0, float& s1) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint32_t w[4];
#pragma unroll
        for (int g = 0; g < 4; ++g)
            w[g] = *reinterpret_cast<const uint32_t*>(lds + col * CS + (g * (WPK / 4) + widx0) * 4);
        // scales and zero-points of the token: NG fp16 numbers each
        uint32_t sv[2] = {0u, 0u}, zv[2] = {0u, 0u};
        if constexpr (NG == 4) {
            const u32x2 s2 = *reinterpret_cast<const u32x2*>(lds + META0 + col * 8);
            const u32x2 z2 = *reinterpret_cast<const u32x2*>(lds + ZOFF + col * 8);
            sv[0] = s2[0]; sv[1] = s2[1];
            zv[0] = z2[0]; zv[1] = z2[1];
        } else if constexpr (NG == 2) {
            sv[0] = *reinterpret_cast<const uint32_t*>(lds + META0 + col * 4);
            zv[0] = *reinterpret_cast<const uint32_t*>(lds + ZOFF + col * 4);
        } else {
            sv[0] = *reinterpret_cast<const uint16_t*>(lds + META0 + col * 2);
            zv[0] = *reinterpret_cast<const uint16_t*>(lds + ZOFF + col * 2);
        }
        // key-side angles of token 16 v + col of the epoch, this lane's 16 frequencies
        u32x4 tr[4];
        {
            const uint32_t* trow = trig + (kRopeUnit * v + col) * kTrigLd + kb * 16;
#pragma unroll
            for (int m = 0; m < 4; ++m) tr[m] = *reinterpret_cast<const u32x4*>(trow + 4 * m);
        }
        // the next unit's tile must not overtake these reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // scale and zero-point of the two members of a pair of chunk g: groups (g, g + 2) * NG / 4, as one packed
        // pair per chunk (one byte permute each at most)
        uint32_t sw[2], zw[2];
        if constexpr (NG == 4) {
            sw[0] = __builtin_amdgcn_perm(sv[1], sv[0], 0x05040100u);        // (s0, s2)
            sw[1] = __builtin_amdgcn_perm(sv[1], sv[0], 0x07060302u);        // (s1, s3)
            zw[0] = __builtin_amdgcn_perm(zv[1], zv[0], 0x05040100u);
            zw[1] = __builtin_amdgcn_perm(zv[1], zv[0], 0x07060302u);
        } else if constexpr (NG == 2) {
            sw[0] = sw[1] = sv[0];                                           // (s0, s1) for both chunks
            zw[0] = zw[1] = zv[0];
        } else {
            sw[0] = sw[1] = __builtin_amdgcn_perm(sv[0], sv[0], 0x01000100u);   // (s0, s0)
            zw[0] = zw[1] = __builtin_amdgcn_perm(zv[0], zv[0], 0x01000100u);
        }
        // scales are non-negative fp16 numbers: their bit patterns order like their values (127.0 = 0x57F0; Inf
        // and NaN land on the careful side as well): the largest of the four, compared as packed 16-bit integers
        typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
        const u16x2 smax = __builtin_elementwise_max(__builtin_bit_cast(u16x2, sw[0]), __builtin_bit_cast(u16x2, sw[1]));
        const u16x2 scap = __builtin_elementwise_min(smax, u16x2{0x57F0, 0x57F0});
        const bool big = __builtin_bit_cast(uint32_t, smax) != __builtin_bit_cast(uint32_t, scap);
        const h2 dsc[2] = {as_h2(sw[0]), as_h2(sw[1])};
        const h2 dzp[2] = {as_h2(zw[0]), as_h2(zw[1])};
        // dequantize into rotary pairs (Section 2: code * Delta + m), rotate, and contract
        f32x4v acc = {0.0f, 0.0f, 0.0f, 0.0f};
        auto body = [&](auto fast_tag) {
            constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                // source registers: (codes of chunk g + 2 : codes of chunk g), each code below bit 8 of its half
                uint32_t src[NSRC];
                if constexpr (BITS == 2) {
                    src[0] = __builtin_amdgcn_perm(w[g + 2], w[g], half_sel);
                    src[1] = src[0] >> 8;
                } else {
                    src[0] = __builtin_amdgcn_perm(w[g + 2], w[g], 0x05040100u);
                    src[1] = src[0] >> 8;
                    src[2] = __builtin_amdgcn_perm(w[g + 2], w[g], 0x07060302u);
                    src[3] = src[2] >> 8;
                }
                const h2 sc9 = FAST ? dsc[g] * h2{static_cast<_Float16>(kCodeScale), static_cast<_Float16>(kCodeScale)} : dsc[g];
                u32x4 bop[2];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int sr = i / CPR, pos = i % CPR;
                    constexpr uint32_t CM = (1u << BITS) - 1u;
                    const uint32_t bitsv = src[sr] & ((CM | (CM << 16)) << (BITS * pos));
                    h2 kv;
                    if constexpr (FAST) {
                        // the masked bits ARE the fp16 subnormals code * 2^(BITS pos - 24): times 2^(15 - BITS pos)
                        // gives code * 2^-9 exactly
                        const _Float16 kf = static_cast<_Float16>(static_cast<float>(1u << (15 - BITS * pos)));
                        const h2 t = as_h2(bitsv) * h2{kf, kf};
                        kv = __builtin_elementwise_fma(t, sc9, dzp[g]);
                    } else {
                        const float ca = static_cast<float>((bitsv & 0xFFFFu) >> (BITS * pos));
                        const float cb = static_cast<float>(bitsv >> (16 + BITS * pos));
                        kv = h2{static_cast<_Float16>(fmaf(ca, static_cast<float>(sc9[0]), static_cast<float>(dzp[g][0]))),
                                static_cast<_Float16>(fmaf(cb, static_cast<float>(sc9[1]), static_cast<float>(dzp[g][1])))};
                    }
                    const h2 xr = rotate_pair(kv, as_h2(tr[2 * g + (i >> 2)][i & 3]));
                    bop[i >> 2][i & 3] = h2_bits(xr);
                }
#pragma unroll
                for (int mm2 = 0; mm2 < 2; ++mm2)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop[2 * g + mm2]),
                                                                 __builtin_bit_cast(half8, bop[mm2]), acc, 0, 0, 0);
            }
        };
        if (__builtin_amdgcn_ballot_w64(big) == 0ull)
            body(std::true_type{});
        else
            body(std::false_type{});
        s0 = fin * (acc[0] + acc[1]);
        if (two) s1 = fin * (acc[2] + acc[3]);
    };

    // ---- whole units, in pairs, an epoch at a time; the loads of the next epoch's units are in flight while this
    // epoch is computed.  Two consecutive units fill one 128-byte line of a score row: the first of a pair is kept
    // and stored together with the second (a unit apart they reach memory as partial line writes).
    if (nf > 0) {
        auto deliver = [&](const Raw& r) {
            *reinterpret_cast<u32x4*>(lds + g_lds) = r.c;
            if constexpr (BITS == 4) *reinterpret_cast<u32x4*>(lds + m_lds) = r.m;
        };
        float* optr = out0 + static_cast<int64_t>(u0) * kRopeUnit + col;
        float held0 = 0.0f, held1 = 0.0f;
        auto pair_step = [&](int v, bool more) {
            float s0 = 0.0f, s1 = 0.0f;
            deliver(ring[v]);
            if (more) fetch(ring[v]);
            unit_scores(v, s0, s1);
            if ((v & 1) == 0) {
                held0 = s0;
                held1 = s1;
            } else {
                if (st0) {
                    __builtin_nontemporal_store(held0, optr);
                    __builtin_nontemporal_store(s0, optr + kRopeUnit);
                }
                if (st1) {
                    __builtin_nontemporal_store(held1, optr + out1);
                    __builtin_nontemporal_store(s1, optr + out1 + kRopeUnit);
                }
                optr += 2 * kRopeUnit;
            }
        };
        static_assert(kEpochUnits == 4, "an epoch is two pairs of units");
        for (int e = u0; e < uf; e += kEpochUnits) {
            qs.build(atile, lane, aop);
            pair_step(0, e + kEpochUnits < uf);
            pair_step(1, e + 1 + kEpochUnits < uf);
            if (e + 2 < uf) {                             // wave-uniform; nf is even
                pair_step(2, e + 2 + kEpochUnits < uf);
                pair_step(3, e + 3 + kEpochUnits < uf);
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
            const int v = (u - u0) & (kEpochUnits - 1);
            if (v == 0) qs.build(atile, lane, aop);           // a new epoch starts here
            if (is_c) {
                const int t = min(u * kRopeUnit + c_tok, n_tok - 1);
                *reinterpret_cast<u32x4*>(lds + c_tok * CS + c_piece * 16) =
                    RP_LOAD(reinterpret_cast<const u32x4*>(c_base + static_cast<uint32_t>(t) * WPK));
            }
            if (is_m) {
                const int t = min(u * kRopeUnit + m_tok, n_tok - 1);
                if constexpr (NG == 4) {
                    *reinterpret_cast<u32x2*>(m_dst) =
                        RP_LOAD(reinterpret_cast<const u32x2*>(m_base + static_cast<uint32_t>(t) * 4));
                } else if constexpr (NG == 2) {
                    *reinterpret_cast<uint32_t*>(m_dst) =
                        RP_LOAD(reinterpret_cast<const uint32_t*>(m_base + static_cast<uint32_t>(t) * 2));
                } else {
                    *reinterpret_cast<uint16_t*>(m_dst) = RP_LOAD(m_base + static_cast<uint32_t>(t));
                }
            }
            float s0 = 0.0f, s1 = 0.0f;
            unit_scores(v, s0, s1);
            const int tok = u * kRopeUnit + col;
            if (tok < n_tok) {
                if (st0) __builtin_nontemporal_store(s0, out0 + tok);
                if (st1) __builtin_nontemporal_store(s1, out0 + out1 + tok);
            }
        }
    }
}

// The same against the PER-CHANNEL store (statistics per channel over 32 tokens: codes
// [tile][channel][BITS words], token j of the tile at bit BITS * (j mod 32 / BITS) of word j / (32 / BITS);
// scale / zero [tile][channel]).  A wavefront goes over tiles of 32 tokens, two per epoch: the tile's words and
// metadata come in with contiguous 16-byte loads, pass through a wavefront-private LDS tile, and are consumed as two
// units of 16 tokens (lane = token of the unit x K block, as above).  A rotary pair's two codes come from two
// channels' words: one v_perm picks the byte that holds the lane's token from both, one v_and leaves the two codes
// as fp16 subnormals at a lane-constant bit, one packed multiply by a lane-constant power of two normalises them.
// p.n_tokens and p.store_stride are multiples of 32; p.units_per_wave counts TILES here (a multiple of 2).
template <int BITS, int QDT, bool WIDE>
__global__ void __launch_bounds__(kRopeWaves* kWave) key_scores_pc_rope_kernel(const RopeParams p) {
    constexpr int TW = kD * BITS;                         // packed words per tile
    constexpr int NCL = TW / 256;                         // 16-byte code loads per lane and tile
    constexpr int DEPTH = 2;                              // tiles in flight = one epoch
    constexpr uint32_t CM = (1u << BITS) - 1u;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));   // uniform: scalar loop control
    const int kb = lane >> 4;
    const int col = lane & 15;
    const int64_t bh = static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y;
    const int64_t b = bh / p.n_kv_heads;
    const int kvh = static_cast<int>(bh - b * p.n_kv_heads);

    // ---- this wavefront's tiles (whole epochs of two)
    const int n_tiles = static_cast<int>(p.n_tokens / 32);
    const int t0 = (static_cast<int>(blockIdx.x) * kRopeWaves + wave) * p.units_per_wave;
    const int t1 = min(t0 + p.units_per_wave, n_tiles);
    const int64_t tile0 = bh * (p.store_stride / 32);
    struct Raw {
        u32x4 c[NCL];
        u32x4 m;
    };
    // metadata: lanes 0..15 scales, 16..31 zero-points (8 channels each); lanes 32..63 repeat those loads and
    // drop them into a spare LDS slot (no lane tests)
    auto fetch = [&](int t, Raw& r) {
        const int64_t tile = tile0 + t;
        const uint32_t* cw = p.codes + tile * TW;
#pragma unroll
        for (int i = 0; i < NCL; ++i) r.c[i] = RP_LOAD(reinterpret_cast<const u32x4*>(cw + (i * 64 + lane) * 4));
        r.m = RP_LOAD(reinterpret_cast<const u32x4*>(((lane & 16) ? p.zero : p.scale) + tile * kD + 8 * (lane & 15)));
    };

    constexpr int QLD = kD + 1;
    __shared__ float qlds[8 * QLD];
    __shared__ float step64[2 * 64];
    __shared__ __attribute__((aligned(16))) uint32_t trig[kEpochTokens * kTrigLd];
    __shared__ __attribute__((aligned(16))) uint32_t atiles[kRopeWaves * 16 * kATileLd];
    stage_queries<QDT>(p, b, kvh, qlds, QLD);
    fill_trig_tables(p.inv_freq, trig, step64);
    __syncthreads();
    if (t0 >= t1) return;                                 // after the last workgroup barrier

    uint32_t* atile = atiles + wave * 16 * kATileLd;
    QuerySide<WIDE> qs;
    qs.init(qlds, QLD, step64, p.inv_freq, static_cast<double>(p.pos0 + static_cast<int64_t>(t0) * 32), lane, p.qpk, atile);

    // result rows 4 kb + {0, 1}: high and low part of query head kb; rows + {2, 3}: query head kb + 4
    constexpr bool two = WIDE;
    float* const out0 = p.scores + b * p.ssb + (static_cast<int64_t>(kvh) * p.qpk + kb) * p.ssh;
    const bool st0 = kb < p.qpk, st1 = kb + 4 < p.qpk;
    const float fin = p.out_scale;

    constexpr int TILE_BYTES = TW * 4 + 512 + 512;        // words, 128 scales and 128 zero-points (fp16), spare slots
    __shared__ __attribute__((aligned(16))) unsigned char lds_all[kRopeWaves * TILE_BYTES];
    unsigned char* lds = lds_all + wave * TILE_BYTES;
    const uint32_t* ldsw = reinterpret_cast<const uint32_t*>(lds);

    // where the code of this lane's token (16 hf + col of the tile) sits inside a channel's words
    //   2-bit: word hf, bit 2 col;  4-bit: word 2 hf + (col >> 3), bit 4 (col & 7)
    const int tbit = BITS == 2 ? 2 * col : 4 * (col & 7);
    const int wsub = BITS == 2 ? 0 : (col >> 3);
    const uint32_t bsel = 0x0C000C00u | (static_cast<uint32_t>(4 + (tbit >> 3)) << 16) | static_cast<uint32_t>(tbit >> 3);
    const int sh = tbit & 7;
    const uint32_t cmask = (CM | (CM << 16)) << sh;
    const _Float16 kf = static_cast<_Float16>(static_cast<float>(1u << (15 - sh)));      // code * 2^(sh - 24) -> code * 2^-9
    const h2 knorm = {kf, kf};
    const h2 k512 = {static_cast<_Float16>(kCodeScale), static_cast<_Float16>(kCodeScale)};

    u32x4 aop[4];
    // registers -> LDS tile (the registers are free afterwards); returns whether this lane saw a scale beyond the
    // packed range
    auto deliver = [&](const Raw& raw) -> bool {
#pragma unroll
        for (int i = 0; i < NCL; ++i) *reinterpret_cast<u32x4*>(lds + (i * 64 + lane) * 16) = raw.c[i];
        *reinterpret_cast<u32x4*>(lds + TW * 4 + lane * 16) = raw.m;      // lanes 32..63: the spare slots
        // the lanes that loaded the scales look for one beyond the packed range (scales are non-negative fp16
        // numbers: bit patterns order like values, 127.0 = 0x57F0)
        bool big = false;
        if (lane < 16) {
#pragma unroll
            for (int w = 0; w < 4; ++w) big = big || (raw.m[w] & 0xFFFFu) > 0x57F0u || (raw.m[w] >> 16) > 0x57F0u;
        }
        return big;
    };
    auto compute = [&](int t, int v, bool big) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const bool fast = __builtin_amdgcn_ballot_w64(big) == 0ull;

        f32x4v acc[2] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
        auto body = [&](auto fast_tag) {
            constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                // (scale, zero-point) of the two members of pair i: channels 32 g + 8 kb + i and + 64
                h2 dsc[8], dzp[8];
                {
                    const u32x4 sa = *reinterpret_cast<const u32x4*>(lds + TW * 4 + (32 * g + 8 * kb) * 2);
                    const u32x4 sb = *reinterpret_cast<const u32x4*>(lds + TW * 4 + (32 * g + 64 + 8 * kb) * 2);
                    const u32x4 za = *reinterpret_cast<const u32x4*>(lds + TW * 4 + 256 + (32 * g + 8 * kb) * 2);
                    const u32x4 zb = *reinterpret_cast<const u32x4*>(lds + TW * 4 + 256 + (32 * g + 64 + 8 * kb) * 2);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
                        const h2 sc = as_h2(__builtin_amdgcn_perm(sb[i >> 1], sa[i >> 1], sel));
                        dsc[i] = FAST ? sc * k512 : sc;
                        dzp[i] = as_h2(__builtin_amdgcn_perm(zb[i >> 1], za[i >> 1], sel));
                    }
                }
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const uint32_t* trow = trig + (2 * kRopeUnit * v + kRopeUnit * hf + col) * kTrigLd + kb * 16 + 8 * g;
                    const u32x4 tr0 = *reinterpret_cast<const u32x4*>(trow);
                    const u32x4 tr1 = *reinterpret_cast<const u32x4*>(trow + 4);
                    u32x4 bop[2];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int ca = 32 * g + 8 * kb + i;
                        const uint32_t wa = ldsw[ca * BITS + (BITS / 2) * hf + wsub];
                        const uint32_t wb = ldsw[(ca + 64) * BITS + (BITS / 2) * hf + wsub];
                        const uint32_t pr = __builtin_amdgcn_perm(wb, wa, bsel) & cmask;
                        h2 kv;
                        if constexpr (FAST) {
                            kv = __builtin_elementwise_fma(as_h2(pr) * knorm, dsc[i], dzp[i]);
                        } else {
                            const float fa = static_cast<float>((pr & 0xFFFFu) >> sh);
                            const float fb = static_cast<float>(pr >> (16 + sh));
                            kv = h2{static_cast<_Float16>(fmaf(fa, static_cast<float>(dsc[i][0]), static_cast<float>(dzp[i][0]))),
                                    static_cast<_Float16>(fmaf(fb, static_cast<float>(dsc[i][1]), static_cast<float>(dzp[i][1])))};
                        }
                        const uint32_t cs = i < 4 ? tr0[i & 3] : tr1[i & 3];
                        bop[i >> 2][i & 3] = h2_bits(rotate_pair(kv, as_h2(cs)));
                    }
#pragma unroll
                    for (int mm = 0; mm < 2; ++mm)
                        acc[hf] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop[2 * g + mm]),
                                                                         __builtin_bit_cast(half8, bop[mm]), acc[hf], 0, 0, 0);
                }
            }
        };
        if (fast)
            body(std::true_type{});
        else
            body(std::false_type{});
        // both halves of the group's 128-byte line of a score row, back to back
        const int64_t tok = static_cast<int64_t>(t) * 32 + col;
        if (st0) {
            __builtin_nontemporal_store(fin * (acc[0][0] + acc[0][1]), out0 + tok);
            __builtin_nontemporal_store(fin * (acc[1][0] + acc[1][1]), out0 + tok + 16);
        }
        if (two) {
            if (st1) {
                __builtin_nontemporal_store(fin * (acc[0][2] + acc[0][3]), out0 + 4 * p.ssh + tok);
                __builtin_nontemporal_store(fin * (acc[1][2] + acc[1][3]), out0 + 4 * p.ssh + tok + 16);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    Raw ring[DEPTH];
#pragma unroll
    for (int i = 0; i < DEPTH; ++i) fetch(min(t0 + i, t1 - 1), ring[i]);
    for (int e = t0; e < t1; e += DEPTH) {
        qs.build(atile, lane, aop);
#pragma unroll
        for (int v = 0; v < DEPTH; ++v) {
            if (e + v < t1) {                             // wave-uniform
                const bool big = deliver(ring[v]);
                fetch(min(e + v + DEPTH, t1 - 1), ring[v]);
                compute(e + v, v, big);
            }
        }
    }
}

// (WIDE: more than four query heads per KV head)
template <int BITS, int QDT>
void launch_pc_wide(const RopeParams& p, dim3 grid, dim3 block, hipStream_t s) {
    if (p.qpk > 4)
        hipLaunchKernelGGL((key_scores_pc_rope_kernel<BITS, QDT, true>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((key_scores_pc_rope_kernel<BITS, QDT, false>), grid, block, 0, s, p);
}

template <int BITS>
int launch_pc_dt(const RopeParams& p, dim3 grid, hipStream_t s) {
    const dim3 block(kRopeWaves * kWave);
    switch (p.q_dt) {
        case SQUAT_F32: launch_pc_wide<BITS, SQUAT_F32>(p, grid, block, s); break;
        case SQUAT_F16: launch_pc_wide<BITS, SQUAT_F16>(p, grid, block, s); break;
        case SQUAT_BF16: launch_pc_wide<BITS, SQUAT_BF16>(p, grid, block, s); break;
        default: return SQUAT_E_BADDTYPE;
    }
    return check_launch();
}

template <int BITS, int NG, int QDT>
void launch_wide(const RopeParams& p, dim3 grid, dim3 block, hipStream_t s) {
    if (p.qpk > 4)
        hipLaunchKernelGGL((key_scores_rope_kernel<BITS, NG, QDT, true>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((key_scores_rope_kernel<BITS, NG, QDT, false>), grid, block, 0, s, p);
}

template <int BITS, int NG>
int launch_dt(const RopeParams& p, dim3 grid, hipStream_t s) {
    const dim3 block(kRopeWaves * kWave);
    switch (p.q_dt) {
        case SQUAT_F32: launch_wide<BITS, NG, SQUAT_F32>(p, grid, block, s); break;
        case SQUAT_F16: launch_wide<BITS, NG, SQUAT_F16>(p, grid, block, s); break;
        case SQUAT_BF16: launch_wide<BITS, NG, SQUAT_BF16>(p, grid, block, s); break;
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
    {
        const int64_t meta_row = 2 * (128 / group);       // bytes of scales (or zero-points) per key
        p.wide_loads = (store_stride * meta_row) % 16 == 0 && aligned(scale, 16) && aligned(zero, 16);
    }

    // workgroups along the sequence: about kRopeWaves * kRopeMaxUnitsPerWave units each, spread evenly
    const int64_t n_units = (n_tokens + kRopeUnit - 1) / kRopeUnit;
    const int64_t slab = static_cast<int64_t>(kRopeWaves) * kRopeMaxUnitsPerWave;
    int64_t gx = (n_units + slab / 2) / slab;
    if (gx < 1) gx = 1;
    int64_t upw = (n_units + kRopeWaves * gx - 1) / (kRopeWaves * gx);
    if (upw < kRopeMinUnitsPerWave) upw = kRopeMinUnitsPerWave;
    upw = (upw + kEpochUnits - 1) / kEpochUnits * kEpochUnits;       // whole epochs: a range starts where the query-side operand changes
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
    tpw += tpw & 1;                                       // whole epochs of two tiles
    p.wide_loads = 0;
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
