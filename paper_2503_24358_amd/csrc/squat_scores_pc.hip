// squat_key_scores_per_channel: attention logits of decode-time queries against
// the PER-CHANNEL packed key store (the grouping Algorithm 1's Quant prints:
// one scale / zero-point per channel and group of 32 tokens), out_scale * q .
// deq(code)^T without materialising the keys (Section 2: deq(c) = c * Delta + m).
//
// For token t of token group T,
//     q . deq = sum_c (q_c Delta_{T,c}) code_{c,t}  +  sum_c q_c m_{T,c}.
// The scales sit INSIDE the contraction here, so the query-side operand is
// rebuilt for every token group: a_c = q_c Delta_c as an fp16 high / low pair
// (rows = (query head, part), as in the per-token kernel), formed with packed
// fp16 arithmetic from the fp16 parts of q and the fp16 Delta as stored:
//     hi = rn(q_hi Delta),  lo = fma(q_hi, Delta, -hi) [exact] (+ q_lo Delta).
// Two wave-uniform powers of two keep that inside fp16's range whatever the data:
// q is normalised by the exponent of max |q| of the KV head, Delta by the
// exponent of the largest Delta of the token group (both undone in fp32 at the
// end).  The codes are the other operand, as raw bits: a code at bit s of a
// 16-bit half IS the fp16 subnormal code * 2^(s-24), and codes are only read at
// bits 6..9 (the matrix cores align products by exponent fields; lower positions
// lose bits).  A packed word holds 16 (2-bit) or 8 (4-bit) TOKENS of one channel
// while a matrix operand wants consecutive CHANNELS of one token in a lane, so
// the group's words go through a small per-wavefront LDS tile, regrouped on the
// way in as (low halves, high halves) of the words of two neighbouring channels
// (one v_perm each); a lane then reads such a pair and one rotate + mask puts
// its token's two codes into an operand register: one instruction per code.  The zero-point term is one more matrix product per
// chunk with the zero-points as stored as the other operand (every column gets
// the same sum, so each lane finds it next to its own token's result).
#include "squat_internal.h"

using namespace squat;

namespace {

constexpr int kPcDepth = 2;            // token groups whose loads are in flight per wavefront
constexpr int kPcWaves = 4;
constexpr int kPcTilesPerWave = 16;    // token groups a wavefront aims at (amortises its set-up) ...
constexpr int kPcMinTilesPerWave = 2;  // ... unless the sequence is short
#define PC_LOAD(p) __builtin_nontemporal_load(p)

typedef float f32x4v __attribute__((ext_vector_type(4)));

struct ScorePcParams {
    const uint32_t* codes;
    const uint16_t* scale;
    const uint16_t* zero;
    const unsigned char* q;
    int q_dt;
    int64_t qsb, qsh;                // query strides in ELEMENTS
    float* scores;
    int64_t ssb, ssh;                // score strides in elements
    int n_tiles;                     // token groups per (batch, KV head) to read
    int64_t store_tiles;             // token groups per (batch, KV head) in the store (>= n_tiles)
    int n_kv_heads;
    int qpk;
    float out_scale;
    int tiles_per_wave;
};

__device__ __forceinline__ uint32_t pack2(_Float16 lo, _Float16 hi) {
    return static_cast<uint32_t>(__builtin_bit_cast(uint16_t, lo)) |
           (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, hi)) << 16);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max(uint32_t v) {
    const uint32_t o = static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, false));
    return v > o ? v : o;
}

// grid: x over slabs of kPcWaves * tiles_per_wave token groups, y / z over (batch, KV head).
// NT = token groups per step.  With at most four query heads per KV head only 8 of the 16 operand rows
// are in use, so NT = 2 gives rows 0..7 to one token group and rows 8..15 to the next one (same queries,
// the other group's scales): the instructions that build the query-side operand then serve two groups,
// and lanes of K blocks 0, 1 find the first group's results in their registers, K blocks 2, 3 the second's.
template <int BITS, int QDT, int NT>
__global__ void __launch_bounds__(kPcWaves* kWave) key_scores_pc_kernel(const ScorePcParams p) {
    constexpr int W = BITS;                               // packed words per channel and token group
    constexpr int TH = 16 / BITS;                         // tokens per 16-bit half of a word: 8 or 4
    constexpr uint32_t MASK = BITS == 2 ? 0x00C000C0u : 0x03C003C0u;   // a code at bits 6.. of both halves
    // LDS tile of one wavefront: region (i, k) = word k of every channel of group i, per pair of channels the
    // low halves of both words, then the high halves (128 words; 32 spare bytes shift the banks of consecutive
    // regions), then scales of group 0 (, 1), zero-points of group 0 (, 1)
    constexpr int RSTRIDE = 512 + 32;
    constexpr int META = NT * W * RSTRIDE, ZOFF = NT * 256, TILE = META + 2 * NT * 256;
    constexpr int ML = 2 * NT;                            // metadata dwords a lane loads

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));   // uniform: scalar loop control
    const int kb = lane >> 4;                             // K block of an operand / row block of the result
    const int col = lane & 15;                            // operand row (A) or column (B, result)
    const int64_t bh = static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y;
    const int64_t b = bh / p.n_kv_heads;
    const int kvh = static_cast<int>(bh - b * p.n_kv_heads);

    // ---- this wavefront's token groups (tiles_per_wave is a multiple of NT); the loads of its first steps are
    // issued before anything else, so that their latency overlaps the set-up of the query-side registers
    const int t0 = (static_cast<int>(blockIdx.x) * kPcWaves + wave) * p.tiles_per_wave;
    const int t1 = min(t0 + p.tiles_per_wave, p.n_tiles);
    const int64_t tile0 = bh * p.store_tiles;
    // loads per token group: lane L fetches the words of channels 2 L and 2 L + 1 (16 or 32 contiguous
    // bytes); metadata per step: 2 NT arrays of 128 halves (scales of group 0 (, 1), zero-points of group
    // 0 (, 1)), 4 NT halves per lane
    const uint32_t* c_base = p.codes + tile0 * (kD * W) + lane * (2 * W);
    constexpr int LPA = 32 / NT;                          // lanes per metadata array
    const int m_arr = lane / LPA;                         // which array this lane loads from
    const int m_tile = m_arr % NT;
    const uint16_t* m_base = (m_arr < NT ? p.scale : p.zero) + tile0 * kD + (lane % LPA) * (4 * NT);
    typedef uint32_t mvec __attribute__((ext_vector_type(ML)));
    struct Raw {
        u32x4 c[NT][BITS / 2];
        mvec m;
    };
    // a group past the end of this wavefront's range re-reads its last group (never used)
    auto fetch = [&](int t, Raw& r) {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const uint32_t tt = static_cast<uint32_t>(min(t + i, t1 - 1));
#pragma unroll
            for (int k = 0; k < BITS / 2; ++k)
                r.c[i][k] = PC_LOAD(reinterpret_cast<const u32x4*>(c_base + tt * (kD * W) + 4 * k));
        }
        const uint32_t tm = static_cast<uint32_t>(min(t + m_tile, t1 - 1));
        r.m = PC_LOAD(reinterpret_cast<const mvec*>(m_base + tm * kD));
    };

    Raw ring[kPcDepth];
    if (t0 < t1) {
#pragma unroll
        for (int i = 0; i < kPcDepth; ++i) fetch(t0 + NT * i, ring[i]);
    }

    // ---- the KV head's queries -> LDS as fp32, rows past q_per_kv zero
    constexpr int QLD = kD + 1;
    __shared__ float qlds[8 * QLD];
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
    }
    __syncthreads();

    // ---- power of two that brings max |q| of this KV head into [1, 2)
    float qmax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int e = lane + 64 * i;
        qmax = fmaxf(qmax, fabsf(qlds[(e / kD) * QLD + (e % kD)]));
    }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) qmax = fmaxf(qmax, __shfl_xor(qmax, s, 64));
    uint32_t eb = as_u32(qmax) >> 23;
    eb = eb < 1u ? 1u : (eb > 253u ? 253u : eb);
    const float inv_q = as_f32((254u - eb) << 23);        // 2^-(eb - 127)
    const float fin = p.out_scale * as_f32(eb << 23);     // out_scale * 2^(eb - 127)

    // ---- constant query-side operands: row `col` = (token group col / 8 if NT = 2, query head, part);
    // register r of chunk g holds K = 8 kb + 2 r + {0, 1}  <->  channels 32 g + 8 kb + 2 r + {0, 1}.
    // The operand register of a row is  fma(q_hi, Delta, -sub)  with sub = rn(q_sub Delta): high rows keep
    // q_sub = 0 (the result is rn(q_hi Delta)), low rows q_sub = q_hi (the result is the exact remainder),
    // so both kinds of row run the same two instructions.
    const int arow = NT == 2 ? (col & 7) : col;
    const int ahalf = NT == 2 ? (col >> 3) : 0;           // token group whose scales this lane's row uses
    const int qh = arow >> 1, part = arow & 1;
    // They live in LDS, not in registers (32 to 48 of them would cost a wavefront per SIMD): wavefront g builds
    // chunk g for every lane position, and a step reads a chunk back with one 16-byte read per kind.
    __shared__ __attribute__((aligned(16))) u32x4 qhi_lds[4 * kWave];
    __shared__ __attribute__((aligned(16))) u32x4 qsub_lds[4 * kWave];
    __shared__ __attribute__((aligned(16))) u32x4 qlo_lds[QDT == SQUAT_F32 ? 4 * kWave : 1];   // fp32 queries only: low part (low rows), else 0
    {
        const int g = wave;
        u32x4 vh, vs, vl;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int c = 32 * g + 8 * kb + 2 * r;
            const float v0 = qlds[qh * QLD + c] * inv_q, v1 = qlds[qh * QLD + c + 1] * inv_q;
            const _Float16 h0 = static_cast<_Float16>(v0), h1 = static_cast<_Float16>(v1);
            const _Float16 l0 = static_cast<_Float16>(v0 - static_cast<float>(h0));
            const _Float16 l1 = static_cast<_Float16>(v1 - static_cast<float>(h1));
            vh[r] = pack2(h0, h1);
            vs[r] = part == 0 ? 0u : pack2(h0, h1);
            vl[r] = part == 0 ? 0u : pack2(l0, l1);
        }
        qhi_lds[g * kWave + lane] = vh;
        qsub_lds[g * kWave + lane] = vs;
        if constexpr (QDT == SQUAT_F32) qlo_lds[g * kWave + lane] = vl;
    }
    __syncthreads();

    if (t0 >= t1) return;                                 // after the last workgroup barrier

    __shared__ __attribute__((aligned(16))) unsigned char lds_all[kPcWaves * TILE];
    unsigned char* lds = lds_all + wave * TILE;
    // This lane's tokens.  4-bit: word wsel of a channel, position j in both of its 16-bit halves, i.e. tokens
    // tokA and tokA + 4.  2-bit: a half holds 8 tokens, and two NEIGHBOURING tokens can be taken from one rotated
    // register (bits 6..7 and 8..9; the second comes out times 4, undone in the final scale): word wsel, half
    // hsel, tokens tokA = 2 jp and tokA + 1.
    constexpr int TOKB = BITS == 2 ? 1 : TH;              // distance of the second product's token
    const int wsel = BITS == 2 ? col >> 3 : col / TH;
    const int hsel = BITS == 2 ? (col >> 2) & 1 : 0;
    const int j = BITS == 2 ? 2 * (col & 3) : col % TH;
    const uint32_t rot = static_cast<uint32_t>(BITS * j - 6) & 31u;      // right-rotation: code -> bits 6..
    const int tokA = (32 / W) * wsel + 8 * hsel + j;
    const int kbh = NT == 2 ? (kb & 1) : kb;              // pair of query heads in this lane's result rows
    const int rhalf = NT == 2 ? (kb >> 1) : 0;            // token group of this lane's result rows
    float* out0 = p.scores + b * p.ssb + (static_cast<int64_t>(kvh) * p.qpk + 2 * kbh) * p.ssh;
    const bool st0 = 2 * kbh < p.qpk, st1 = 2 * kbh + 1 < p.qpk;
    const unsigned char* rd_codes = lds + wsel * RSTRIDE + 32 * kb + 16 * hsel;
    const unsigned char* rd_scale = lds + META + ahalf * 256 + 16 * kb;
    // zero-points: the group of the COLUMN (every K block of a column must see the same group)
    const unsigned char* rd_zero = lds + META + ZOFF + (NT == 2 ? (col >> 3) * 256 : 0) + 16 * kb;
    const bool z_mine = NT == 1 || (col >> 3) == rhalf;

    // registers -> LDS tile; returns the lane's largest scale pattern (the registers are free afterwards)
    auto deliver = [&](const Raw& raw) -> uint32_t {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            // word k of the lane's two channels, regrouped as (low halves, high halves): a half-word pair is
            // what an operand register of the reader holds, so the regrouping is done once here, not per reader
            // (4-bit: the two kinds alternate, a reader takes both; 2-bit: per block of 8 channels the four low
            // pairs, then the four high pairs, a reader takes one kind with one 16-byte read)
            unsigned char* reg = lds + i * W * RSTRIDE + (BITS == 2 ? (lane >> 2) * 32 + (lane & 3) * 4 : 8 * lane);
#pragma unroll
            for (int k = 0; k < W; ++k) {
                const uint32_t we = raw.c[i][0][k];
                const uint32_t wo = BITS == 2 ? raw.c[i][0][2 + k] : raw.c[i][BITS / 2 - 1][k];
                const uint32_t pl = __builtin_amdgcn_perm(wo, we, 0x05040100u);
                const uint32_t ph = __builtin_amdgcn_perm(wo, we, 0x07060302u);
                if constexpr (BITS == 2) {
                    *reinterpret_cast<uint32_t*>(reg + k * RSTRIDE) = pl;
                    *reinterpret_cast<uint32_t*>(reg + k * RSTRIDE + 16) = ph;
                } else {
                    *reinterpret_cast<u32x2*>(reg + k * RSTRIDE) = u32x2{pl, ph};
                }
            }
        }
        *reinterpret_cast<mvec*>(lds + META + 4 * ML * lane) = raw.m;
        // largest Delta of each token group: fp16 patterns of non-negative numbers order like integers;
        // lanes 0..15 (row 0) hold scales of group 0, lanes 16..31 (row 1) of group NT - 1; the rows of
        // the zero-points are reduced too and never read
        uint32_t mx = 0u;
#pragma unroll
        for (int i = 0; i < ML; ++i) {
            const uint32_t v = raw.m[i];
            mx = max(mx, max(v & 0xFFFFu, v >> 16));
        }
        return mx;
    };
    auto compute = [&](int t, uint32_t mx) {
        mx = dpp_max<0xB1>(mx);                           // quad_perm [1,0,3,2]
        mx = dpp_max<0x4E>(mx);                           // quad_perm [2,3,0,1]
        mx = dpp_max<0x141>(mx);                          // row_half_mirror
        mx = dpp_max<0x140>(mx);                          // row_mirror
        const uint32_t m0 = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(mx), 0));
        const uint32_t m1 = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(mx), 16));
        // Delta * 2^(field - 15) < 2 (< 4 at the top of fp16's range); a negative or NaN "scale" only
        // ends up at the clamp
        int field[2];
        field[0] = 30 - static_cast<int>((NT == 2 ? m0 : max(m0, m1)) >> 10);
        field[1] = 30 - static_cast<int>(m1 >> 10);
#pragma unroll
        for (int i = 0; i < 2; ++i) field[i] = field[i] < 1 ? 1 : field[i];
        const int fa = NT == 2 && ahalf ? field[1] : field[0];
        const int fr = NT == 2 && rhalf ? field[1] : field[0];
        const uint32_t sp = static_cast<uint32_t>(fa) << 10;
        const half2v spack = __builtin_bit_cast(half2v, sp | (sp << 16));
        const float descale = as_f32(static_cast<uint32_t>(127 + 33 - fr) << 23);     // 2^18 * 2^(15 - field)

        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        f32x4v acc[NT][2];
#pragma unroll
        for (int i = 0; i < NT; ++i) acc[i][0] = acc[i][1] = f32x4v{0.0f, 0.0f, 0.0f, 0.0f};
        f32x4v zacc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const u32x4 sc = *reinterpret_cast<const u32x4*>(rd_scale + 64 * g);
            const u32x4 zm = *reinterpret_cast<const u32x4*>(rd_zero + 64 * g);
            const u32x4 qh4 = qhi_lds[g * kWave + lane];
            const u32x4 qs4 = qsub_lds[g * kWave + lane];
            u32x4 ql4 = {0u, 0u, 0u, 0u};
            if constexpr (QDT == SQUAT_F32) ql4 = qlo_lds[g * kWave + lane];
            u32x4 aop;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // (bit-casting the vector ELEMENT expression directly makes this compiler read element 0)
                const uint32_t sraw = sc[r], qhr = qh4[r], qsr = qs4[r], qlr = ql4[r];
                const half2v dl = __builtin_bit_cast(half2v, sraw) * spack;
                const half2v sub = __builtin_bit_cast(half2v, qsr) * dl;
                half2v a = __builtin_elementwise_fma(__builtin_bit_cast(half2v, qhr), dl, -sub);
                if constexpr (QDT == SQUAT_F32) a = __builtin_elementwise_fma(__builtin_bit_cast(half2v, qlr), dl, a);
                aop[r] = __builtin_bit_cast(uint32_t, a);
            }
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const unsigned char* src = rd_codes + i * W * RSTRIDE + 128 * g;
                u32x4 bopA, bopB;
                if constexpr (BITS == 2) {
                    const u32x4 wq = *reinterpret_cast<const u32x4*>(src);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const uint32_t wr = wq[r];
                        const uint32_t x = __builtin_amdgcn_alignbit(wr, wr, rot);
                        bopA[r] = x & MASK;                   // token tokA of channels 2 r, 2 r + 1
                        bopB[r] = x & (MASK << 2);            // token tokA + 1, times 4
                    }
                } else {
                    const u32x4 wlo = *reinterpret_cast<const u32x4*>(src);
                    const u32x4 whi = *reinterpret_cast<const u32x4*>(src + 16);
                    const uint32_t w[8] = {wlo[0], wlo[1], wlo[2], wlo[3], whi[0], whi[1], whi[2], whi[3]};
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // low / high halves of the words of channels 2 r, 2 r + 1: tokens j / TH + j of the word
                        bopA[r] = __builtin_amdgcn_alignbit(w[2 * r], w[2 * r], rot) & MASK;
                        bopB[r] = __builtin_amdgcn_alignbit(w[2 * r + 1], w[2 * r + 1], rot) & MASK;
                    }
                }
                acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop),
                                                                   __builtin_bit_cast(half8, bopA), acc[i][0], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop),
                                                                   __builtin_bit_cast(half8, bopB), acc[i][1], 0, 0, 0);
            }
            u32x4 az;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // high rows: q_hi (q_sub = 0), low rows: q_lo (q_sub = q_hi)
                az[r] = qh4[r] ^ qs4[r];
                if constexpr (QDT == SQUAT_F32) az[r] |= ql4[r];
            }
            zacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, az), __builtin_bit_cast(half8, zm),
                                                          zacc, 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // rows 4 kb + {0, 1}: high and low part of the first query head of the lane, rows + {2, 3}: the second
        float z0 = zacc[0] + zacc[1], z1 = zacc[2] + zacc[3];
        if constexpr (NT == 2) {
            // the zero-point sums of this lane's group sit 8 columns away when the column is the other group's
            const float y0 = as_f32(static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(as_u32(z0)), 0x128, 0xF, 0xF, false)));
            const float y1 = as_f32(static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(as_u32(z1)), 0x128, 0xF, 0xF, false)));
            z0 = z_mine ? z0 : y0;
            z1 = z_mine ? z1 : y1;
        }
        float r0[2], r1[2];
#pragma unroll
        for (int sgn = 0; sgn < 2; ++sgn) {
            f32x4v v = acc[0][sgn];
            if constexpr (NT == 2) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = rhalf ? acc[NT - 1][sgn][e] : v[e];
            }
            const float ds = (BITS == 2 && sgn == 1) ? 0.25f * descale : descale;
            r0[sgn] = fin * fmaf(ds, v[0] + v[1], z0);
            r1[sgn] = fin * fmaf(ds, v[2] + v[3], z1);
        }
        const int tr = t + rhalf;
        if (tr < t1) {
            const int64_t tok = static_cast<int64_t>(tr) * 32 + tokA;
            if (st0) {
                __builtin_nontemporal_store(r0[0], out0 + tok);
                __builtin_nontemporal_store(r0[1], out0 + tok + TOKB);
            }
            if (st1) {
                __builtin_nontemporal_store(r1[0], out0 + p.ssh + tok);
                __builtin_nontemporal_store(r1[1], out0 + p.ssh + tok + TOKB);
            }
        }
    };

    // whole groups of kPcDepth steps run without a test (a skipped step inside the loop costs a register copy
    // per value the loop carries); the last, shorter group is handled after it
    int t = t0;
    for (; t + NT * (kPcDepth - 1) < t1; t += NT * kPcDepth) {
#pragma unroll
        for (int i = 0; i < kPcDepth; ++i) {
            const uint32_t mx = deliver(ring[i]);
            fetch(t + NT * (i + kPcDepth), ring[i]);
            compute(t + NT * i, mx);
        }
    }
    static_assert(kPcDepth <= 3, "the tail picks its step from ring[0] / ring[1]");
#pragma nounroll
    for (int i = 0; t + NT * i < t1; ++i) {               // at most kPcDepth - 1 steps; one copy of the code
        Raw cur = ring[0];
        if (i == 1) cur = ring[1];
        const uint32_t mx = deliver(cur);
        compute(t + NT * i, mx);
    }
}

template <int BITS, int NT>
int launch_dt(const ScorePcParams& p, dim3 grid, hipStream_t s) {
    const dim3 block(kPcWaves * kWave);
    switch (p.q_dt) {
        case SQUAT_F32: hipLaunchKernelGGL((key_scores_pc_kernel<BITS, SQUAT_F32, NT>), grid, block, 0, s, p); break;
        case SQUAT_F16: hipLaunchKernelGGL((key_scores_pc_kernel<BITS, SQUAT_F16, NT>), grid, block, 0, s, p); break;
        case SQUAT_BF16: hipLaunchKernelGGL((key_scores_pc_kernel<BITS, SQUAT_BF16, NT>), grid, block, 0, s, p); break;
        default: return SQUAT_E_BADDTYPE;
    }
    return check_launch();
}

}  // namespace

// squat_key_scores_per_channel over the first n_tokens tokens of a store that holds store_tokens tokens
// (a multiple of 32) per (batch, KV head).
int squat::key_scores_pc_from(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t n_batch,
                              int n_kv_heads, int64_t n_tokens, int64_t store_tokens, int d, int bits, int group,
                              const void* q, squat_dtype q_dt, int q_per_kv, int64_t q_stride_batch,
                              int64_t q_stride_head, float out_scale, float* scores, int64_t s_stride_batch,
                              int64_t s_stride_head, squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    if (group != 32) return SQUAT_E_BADSHAPE;
    if (q_per_kv < 1 || q_per_kv > 8) return SQUAT_E_BADSHAPE;
    if (n_batch < 0 || n_kv_heads < 0 || n_tokens < 0 || n_tokens >= (int64_t(1) << 25)) return SQUAT_E_BADSHAPE;
    if ((n_tokens % 32) || (store_tokens % 32) || store_tokens < n_tokens) return SQUAT_E_BADSHAPE;
    if (q_dt != SQUAT_F32 && q_dt != SQUAT_F16 && q_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (!(out_scale == out_scale)) return SQUAT_E_BADVALUE;
    if (n_batch == 0 || n_kv_heads == 0 || n_tokens == 0) return SQUAT_OK;
    if (!codes || !scale || !zero || !q || !scores) return SQUAT_E_NULLPTR;
    if (q_stride_head < d || q_stride_batch < 0 || s_stride_head < n_tokens || s_stride_batch < 0) return SQUAT_E_BADSHAPE;
    if ((q_stride_head % 8) || (q_stride_batch % 8)) return SQUAT_E_ALIGN;
    if (!aligned(codes, 16) || !aligned(scale, 16) || !aligned(zero, 16) || !aligned(scores, 4) || !aligned(q, 16))
        return SQUAT_E_ALIGN;

    ScorePcParams p;
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
    p.n_tiles = static_cast<int>(n_tokens / 32);
    p.store_tiles = store_tokens / 32;
    p.n_kv_heads = n_kv_heads;
    p.qpk = q_per_kv;
    p.out_scale = out_scale;

    // workgroups along the sequence: about kPcWaves * kPcTilesPerWave token groups each, spread evenly
    const int64_t n_tiles = p.n_tiles;
    const int64_t slab = static_cast<int64_t>(kPcWaves) * kPcTilesPerWave;
    int64_t gx = (n_tiles + slab / 2) / slab;
    if (gx < 1) gx = 1;
    int64_t tpw = (n_tiles + kPcWaves * gx - 1) / (kPcWaves * gx);
    if (tpw < kPcMinTilesPerWave) tpw = kPcMinTilesPerWave;
    const bool two = q_per_kv <= 4;                       // two token groups per step (see the kernel)
    if (two) tpw += tpw & 1;
    p.tiles_per_wave = static_cast<int>(tpw);
    gx = (n_tiles + kPcWaves * tpw - 1) / (kPcWaves * tpw);
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
    if (two) return bits == 2 ? launch_dt<2, 2>(p, grid, s) : launch_dt<4, 2>(p, grid, s);
    return bits == 2 ? launch_dt<2, 1>(p, grid, s) : launch_dt<4, 1>(p, grid, s);
}

extern "C" int squat_key_scores_per_channel(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                                            int64_t n_batch, int n_kv_heads, int64_t n_tokens, int d, int bits,
                                            int group, const void* q, squat_dtype q_dt, int q_per_kv,
                                            int64_t q_stride_batch, int64_t q_stride_head, float out_scale,
                                            float* scores, int64_t s_stride_batch, int64_t s_stride_head,
                                            squat_stream stream) {
    return squat::key_scores_pc_from(codes, scale, zero, n_batch, n_kv_heads, n_tokens, n_tokens, d, bits, group, q,
                                     q_dt, q_per_kv, q_stride_batch, q_stride_head, out_scale, scores,
                                     s_stride_batch, s_stride_head, stream);
}
