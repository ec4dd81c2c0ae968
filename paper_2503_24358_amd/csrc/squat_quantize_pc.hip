// squat_quantize_keys_per_channel: the iteration of Algorithm 1's `Quant` with
// the block update of Lemma 2 in the paper's own grouping: every channel of a
// key block is quantized over a group of 32 consecutive TOKENS (KIVI's layout
// for keys, Section 2 / Algorithm 1), on gfx950.
//
// One wavefront owns a tile of 32 tokens x 128 channels = one quantization
// group of every channel.  The working copy lives in registers in the MFMA
// 32x32 accumulator layout with a CHANNEL as a column: lane (hh, n) holds, for
// channel n of each 32-channel tile, tokens 16*hh .. 16*hh+15.  In that layout
//   - a channel's min/max over the group is an in-register reduction plus one
//     exchange with lane ^ 32,
//   - 16 two-bit codes of a lane are one 32-bit word of the token-major packed
//     output.
// The update of Lemma 2 is  X[:, rest] += E (tokens x g) * W^T (g x rest):  the
// error tile is the A operand, which wants a token per lane, so it takes one
// trip through LDS (4-byte writes, 16-byte reads), and the working copy itself
// is the accumulator of the matrix product.  Each error (in the keys' own
// units) is split into an fp16 high part and a low part scaled by 2^11, which
// sit side by side along the MFMA K dimension (K = channel x {high, low}); the
// matching B operand holds every update-matrix entry twice, the second copy
// scaled by 2^-11.  The scaling keeps the low part a normal fp16 number
// whenever the high part is one, so the pair carries the error to 2^-21
// relative (or 2^-35 absolute) for every step size fp16 can hold.
// 16-bit keys reach the accumulator layout through the matrix cores as well:
// the raw key rows (16-byte pieces, the A operand as it lies in memory) times a
// 0/1 selection matrix is an exact conversion to fp32 and a transposition in
// one step.
#include <type_traits>

#include "squat_internal.h"

using namespace squat;

namespace {

constexpr int NT = kD / 32;          // 32-channel tiles per key

constexpr float kLoGain = 2048.0f;   // the low part of an error enters the matrix product times 2^11
constexpr float kFastOffset = 32.0f; // largest |zero| / scale for which the one-multiply-add path is used
constexpr float kFastStep = 0.015625f;  // smallest step size for which the cheap error split is used (see below)

// Wavefronts per workgroup (one workgroup per CU): bounded by LDS (update panels + one staging tile
// per wavefront) and by registers (168 per lane at 12 wavefronts).
__host__ __device__ constexpr int pc_waves_for(int dt, int bt) {
    (void)bt;
    return dt == SQUAT_F32 ? 6 : 12;
}

struct PcParams {
    const unsigned char* k;
    int64_t sb, sh, st;              // key strides in BYTES
    const float* update;
    int64_t usb;                     // update stride per outer-batch entry, elements
    uint32_t* codes;
    uint16_t* scale;
    uint16_t* zero;
    int64_t n_inner;                 // batch entries that share one update matrix
    int n_heads;
    int64_t tiles_per_seq;
    int64_t out_tiles, out_tile0;    // token groups per (batch, head) in the output store, first one written
    int64_t units_per_prob;          // n_inner * tiles_per_seq, < 2^31
    int wgs_per_prob;
    uint32_t div_mul;                // unit / tiles_per_seq == (unit * div_mul) >> div_shift for unit < 2^31
    uint32_t div_shift;
};

template <int DT>
__device__ __forceinline__ float load_elem(const unsigned char* src) {
    if constexpr (DT == SQUAT_F32) {
        return *reinterpret_cast<const float*>(src);
    } else if constexpr (DT == SQUAT_BF16) {
        return as_f32(static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(src)) << 16);
    } else {
        return static_cast<float>(__builtin_bit_cast(_Float16, *reinterpret_cast<const uint16_t*>(src)));
    }
}

template <int BITS, int BT, int DT>
__global__ void __launch_bounds__(pc_waves_for(DT, BT) * kWave, 1) quantize_pc_kernel(const PcParams p) {
    constexpr int kWaves = pc_waves_for(DT, BT);
    constexpr int ES = (DT == SQUAT_F32) ? 4 : 2;
    constexpr int ROWB = kD * ES;                 // bytes of one key
    constexpr int LROW = ROWB + 16;               // padded LDS row of the staging tile
    constexpr int CPR = ROWB / 16;                // 16-byte chunks per key
    constexpr int NLOAD = 32 * CPR / kWave;       // 16-byte loads per lane per tile
    constexpr int NPAIRS = n_pairs(BT);
    constexpr int NB = NT / BT;                   // blocks (iterations) per key
    constexpr int WPT = BITS / 2;                 // packed words per lane per tile
    constexpr int CPH = 16 / BITS;                // codes per 16-bit half-word
    constexpr int EROW = 32 * BT + 4;             // dwords per row of the error tile in LDS (padded)
    constexpr int NCH = 4 * BT;                   // MFMA K-chunks per block: 8 channels x {high, low} each
    constexpr float LV = static_cast<float>((1 << BITS) - 1);
    constexpr bool XL = DT != SQUAT_F32;          // load through the matrix cores (16-bit keys)
    static_assert(NPAIRS == 0 || 32 * EROW * 4 <= 32 * LROW, "the error tile reuses the staging tile's LDS");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    half8* wlds = reinterpret_cast<half8*>(smem);           // [NPAIRS][4 chunks][hi, lo][64 lanes]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5;
    const int n = lane & 31;
    unsigned char* stage = smem + NPAIRS * 8192 + wave * (32 * LROW);
    uint32_t* ebuf = reinterpret_cast<uint32_t*>(stage);

    const int64_t prob = blockIdx.x / p.wgs_per_prob;
    const int wg = blockIdx.x % p.wgs_per_prob;
    const int head = static_cast<int>(prob % p.n_heads);
    const int64_t bo = prob / p.n_heads;

    // The first tile's loads are issued before the panels are converted: their latency overlaps that work.
    const uint32_t st32 = static_cast<uint32_t>(p.st);
    u32x4 pre[NLOAD];
    // unit -> (batch entry, tile): exact multiply-shift division by tiles_per_seq (units < 2^31)
    auto locate = [&](uint32_t u, uint32_t& bi, uint32_t& tile) {
        bi = static_cast<uint32_t>((static_cast<uint64_t>(u) * p.div_mul) >> p.div_shift);
        tile = u - bi * static_cast<uint32_t>(p.tiles_per_seq);
    };
    // lane part of a load address: 16-byte chunk (lane % CPR) of row (lane / CPR); load i adds 64 / CPR rows
    const uint32_t lane_off = static_cast<uint32_t>(lane / CPR) * st32 + static_cast<uint32_t>(lane % CPR) * 16;
    auto issue_loads = [&](uint32_t u) {
        uint32_t bi, tile;
        locate(u, bi, tile);
        // wave-uniform by construction; say so, so that the loads take a scalar base and one lane offset
        // (the builtin returns a signed int: widen both halves as unsigned)
        const uint64_t voff = static_cast<uint64_t>((bo + bi) * p.sb + head * p.sh +
                                                    static_cast<int64_t>(tile) * kTileTokens * p.st);
        const uint32_t off_hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(voff >> 32)));
        const uint32_t off_lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(voff & 0xFFFFFFFFull)));
        const unsigned char* base = p.k + ((static_cast<uint64_t>(off_hi) << 32) | static_cast<uint64_t>(off_lo));
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            // streamed once: non-temporal, so the tile does not displace the update panels in L2
            pre[i] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4*>(base + static_cast<int64_t>(i * (kWave / CPR)) * p.st + lane_off));
        }
    };

    const uint32_t nunits = static_cast<uint32_t>(p.units_per_prob);
    const uint32_t ustride = static_cast<uint32_t>(p.wgs_per_prob) * kWaves;
    // Wavefront v of workgroup w starts at tile v * workgroups + w: a problem with few tiles (a decode-time flush)
    // is spread over the workgroups first, so its wavefronts do not share a SIMD.
    uint32_t unit = static_cast<uint32_t>(wave) * static_cast<uint32_t>(p.wgs_per_prob) + wg;
    if (unit < nunits) issue_loads(unit);


    // Panels whose entries are all fp16 numbers (as squat_prepare writes them) have a zero low part:
    // the product with it is skipped for the whole head.
    bool need_lo = false;
    int* lo_flag = reinterpret_cast<int*>(smem + NPAIRS * 8192 + kWaves * (32 * LROW));
    // Selection matrices for the load: B operand of chunk c (16 channels of a 32-channel tile): lane (hb, m)
    // holds B[k = 8 hb + i][m] = 1 if m == 16 c + 8 hb + i, in the keys' own 16-bit format.
    u32x4* sel_lds = reinterpret_cast<u32x4*>(smem + NPAIRS * 8192 + kWaves * (32 * LROW) + 16);
    if constexpr (XL) {
        constexpr uint32_t ONE = DT == SQUAT_BF16 ? 0x3F80u : 0x3C00u;
        for (int idx = tid; idx < 2 * 64; idx += kWaves * kWave) {
            const int c = idx >> 6, l = idx & 63;
            const int i1 = (l & 31) - 16 * c - 8 * (l >> 5);        // the i with a one, if in 0..7
            u32x4 v;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                v[w] = (i1 == 2 * w ? ONE : 0u) | (i1 == 2 * w + 1 ? ONE << 16 : 0u);
            sel_lds[idx] = v;
        }
        if constexpr (NPAIRS == 0) __syncthreads();
    }
    if constexpr (NPAIRS > 0) {
        if (tid == 0) *lo_flag = 0;
        __syncthreads();
        // B operand of pair (jt, s), chunk c: lane (hb, m) holds, for output channel 32 jt + m, the
        // entries U[32 jt + m][32 s + 8 c + 4 hb + i], i = 0..3, each one twice: K = 2 i meets the high
        // part of the error, K = 2 i + 1 its low part times 2^11, so that copy is scaled by 2^-11.
        const float* U = p.update + bo * p.usb + static_cast<int64_t>(head) * kD * kD;
        for (int idx = tid; idx < NPAIRS * 4 * 64; idx += kWaves * kWave) {
            const int pr = idx >> 8;
            const int c = (idx >> 6) & 3;
            const int l = idx & 63;
            int jt = 0, s = 0;
            {
                int cnt = 0;
                for (int ss = 0; ss < NT; ++ss)
                    for (int j = (ss / BT + 1) * BT; j < NT; ++j) {
                        if (cnt == pr) { jt = j; s = ss; }
                        ++cnt;
                    }
            }
            const int hb = l >> 5, m = l & 31;
            const f32x4 v = *reinterpret_cast<const f32x4*>(U + (32 * jt + m) * kD + 32 * s + 8 * c + 4 * hb);
            half8 hi, lo;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const _Float16 h = static_cast<_Float16>(v[i]);
                const _Float16 r = static_cast<_Float16>(v[i] - static_cast<float>(h));
                hi[2 * i] = h; hi[2 * i + 1] = static_cast<_Float16>(static_cast<float>(h) * (1.0f / kLoGain));
                lo[2 * i] = r; lo[2 * i + 1] = static_cast<_Float16>(static_cast<float>(r) * (1.0f / kLoGain));
            }
            wlds[((pr * 4 + c) * 2 + 0) * 64 + l] = hi;
            wlds[((pr * 4 + c) * 2 + 1) * 64 + l] = lo;
            const u32x4 lb = __builtin_bit_cast(u32x4, lo);
            if (((lb[0] | lb[1] | lb[2] | lb[3]) & 0x7FFF7FFFu) != 0u) *lo_flag = 1;
        }
        __syncthreads();
        need_lo = *lo_flag != 0;
    }

    while (unit < nunits) {
        // ---- registers -> LDS (token-major rows), then read back one channel per lane
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const int flat = i * kWave + lane;
            const int tok = flat / CPR, ch = flat % CPR;
            // token 16 a + 4 b + c goes to row 8 b + 4 a + c: the row of the MFMA accumulator whose
            // register 4 b + c in lane half a stands for it
            const int row = 8 * ((tok >> 2) & 3) + 4 * (tok >> 4) + (tok & 3);
            *reinterpret_cast<u32x4*>(stage + row * LROW + ch * 16) = pre[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        const uint32_t cur = unit;
        unit += ustride;

        // x[j][e]: token 16 hh + e of the tile, channel 32 j + n
        f32x16 x[NT];
        if constexpr (XL) {
            const u32x4 sel0 = sel_lds[lane], sel1 = sel_lds[64 + lane];
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                // A operand: lane (hh, n) holds row n, K = 8 hh .. 8 hh + 7 of each 16-channel chunk
                const u32x4 a0 = *reinterpret_cast<const u32x4*>(stage + n * LROW + (32 * j + 8 * hh) * ES);
                const u32x4 a1 = *reinterpret_cast<const u32x4*>(stage + n * LROW + (32 * j + 16 + 8 * hh) * ES);
                f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                if constexpr (DT == SQUAT_BF16) {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a0),
                                                                  __builtin_bit_cast(bf16x8, sel0), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a1),
                                                                  __builtin_bit_cast(bf16x8, sel1), acc, 0, 0, 0);
                } else {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a0),
                                                                 __builtin_bit_cast(half8, sel0), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a1),
                                                                 __builtin_bit_cast(half8, sel1), acc, 0, 0, 0);
                }
                x[j] = acc;
            }
        } else {
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    x[j][e] = load_elem<DT>(stage + (8 * (e >> 2) + 4 * hh + (e & 3)) * LROW + (32 * j + n) * ES);
        }

        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // The next tile is prefetched into registers; with several blocks the loads are issued only once
        // the first half of the blocks is frozen, so that they reuse the registers of those tiles.
        constexpr int PF_BLK = NB >= 2 ? NB / 2 - 1 : -1;
        if constexpr (PF_BLK < 0)
            if (unit < nunits) issue_loads(unit);

        uint32_t words[NT][WPT];
        uint16_t sbits[NT], zbits[NT];

#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            // ---- statistics of this block's channels over the 32 tokens (current values)
            float b_zero[BT], b_inv[BT], b_top[BT], b_step[BT];
            bool risky = false;
#pragma unroll
            for (int jj = 0; jj < BT; ++jj) {
                const int j = blk * BT + jj;
                float mn = x[j][0], mx = x[j][0];
#pragma unroll
                for (int e = 1; e < 16; ++e) {
                    mn = fminf(mn, x[j][e]);
                    mx = fmaxf(mx, x[j][e]);
                }
                mn = pair_min(mn);
                mx = pair_max(mx);
                // Correctly rounded (max - min) / (2^b - 1) by one Newton step on the rounded reciprocal
                // of the constant divisor: an exact quotient stays exact, so a tie of the fp16 rounding
                // below breaks to even, as the definition does.
                const float rng = mx - mn;
                constexpr float RL = 1.0f / LV;
                const float q0 = rng * RL;
                const float dl = fmaf(fmaf(-q0, LV, rng), RL, q0);
                const float sh = round_f16(dl, sbits[j]);
                const float zh = round_f16(mn, zbits[j]);
                const bool live = sh > 0.0f;
                const float sp = live ? sh : 1.0f;
                float inv = __builtin_amdgcn_rcpf(sp);
                inv = fmaf(fmaf(-sp, inv, 1.0f), inv, inv);
                b_zero[jj] = zh;
                b_inv[jj] = inv;
                b_top[jj] = live ? LV : 0.0f;
                b_step[jj] = sp;
                risky = risky || !(sh >= kFastStep) || fabsf(zh) * inv > kFastOffset;
            }
            // Two versions of the block.  The careful one clamps to [0, 2^b - 1] (which can only bite when
            // the fp16 rounding of zero/scale moved the group's ends by more than half a step: scale not a
            // normal fp16 number, incl. 0, or |zero| / scale > 256), computes (x - m) / Delta as written
            // and takes the high part of the error from a real conversion to fp16, exact for any size.
            // The cheap one folds the zero-point into one multiply-add, x * (1/Delta) - m/Delta, whose
            // rounding error grows with |m| / Delta, and masks the high part in fp32, which loses up to
            // 2^-24 (absolute) when the error is below fp16's normal range.  The whole wavefront takes it
            // only while |m| / Delta <= 32 and Delta >= 2^-6 in every channel of the block (both errors
            // then stay below 5e-6 steps).
            const bool clamp = __builtin_amdgcn_ballot_w64(risky) != 0ull;
            auto quant_block = [&](auto clamp_tag) {
                constexpr bool CLAMP = decltype(clamp_tag)::value;
#pragma unroll
                for (int jj = 0; jj < BT; ++jj) {
                    const int j = blk * BT + jj;
                    const float mh = b_zero[jj], inv = b_inv[jj], top = b_top[jj];
                    const float sp = b_step[jj];       // step size (1 for a constant channel: the error is m - x)
                    const float nmi = -mh * inv;
                    // codes are collected per half-word as exact small floats (Horner), then converted once
                    uint32_t hw[16 / CPH];
#pragma unroll
                    for (int q = 16 / CPH - 1; q >= 0; --q) {
                        float accf = 0.0f;
#pragma unroll
                        for (int e = CPH - 1; e >= 0; --e) {
                            const int c = q * CPH + e;
                            float u, code, et = 0.0f;
                            if constexpr (CLAMP) {
                                const float dd = x[j][c] - mh;
                                u = __builtin_amdgcn_fmed3f(dd * inv, 0.0f, top);
                                code = __builtin_rintf(u);
                                if (blk < NB - 1)
                                    et = __builtin_amdgcn_fmed3f(fmaf(-inv, dd, code) * sp, -60000.0f, 60000.0f);
                            } else {
                                u = fmaf(x[j][c], inv, nmi);
                                code = __builtin_rintf(u);
                                if (blk < NB - 1) et = (code - u) * sp;
                            }
                            accf = fmaf(accf, static_cast<float>(1 << BITS), code);
                            if (blk < NB - 1) {
                                // error  deq - x  split into a part with 11 significant bits (exact in
                                // fp16) and the remainder times 2^11
                                float eh;
                                if constexpr (CLAMP)
                                    eh = static_cast<float>(static_cast<_Float16>(et));
                                else
                                    eh = as_f32(as_u32(et) & 0xFFFFE000u);
                                const float el = (et - eh) * kLoGain;
                                // row of the MFMA A operand that stands for token 16 hh + c
                                const int mrow = 8 * (c >> 2) + 4 * hh + (c & 3);
                                if constexpr (NPAIRS > 0)
                                    ebuf[mrow * EROW + 32 * jj + n] =
                                        __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(eh, el));
                            }
                        }
                        hw[q] = static_cast<uint32_t>(accf);
                    }
#pragma unroll
                    for (int w = 0; w < WPT; ++w) words[j][w] = hw[2 * w] | (hw[2 * w + 1] << 16);
                }
            };
            if (clamp)
                quant_block(std::true_type{});
            else
                quant_block(std::false_type{});
            // ---- Lemma 2: remaining channels += error * U[rest, block]^T
            if constexpr (NPAIRS > 0) {
                if (blk < NB - 1) {
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    // A operand, chunk c: lane (ha, m) holds row m, K = 8 ha .. 8 ha + 7, i.e. channels
                    // 8 c + 4 ha .. + 3 of the block, each as (high, low)
                    half8 aop[NCH];
#pragma unroll
                    for (int c = 0; c < NCH; ++c)
                        aop[c] = __builtin_bit_cast(
                            half8, *reinterpret_cast<const u32x4*>(ebuf + n * EROW + 8 * c + 4 * hh));
                    // The working copy is the accumulator.  The chains of the remaining tiles are
                    // interleaved (K-chunk outermost), so that no matrix product waits for the one
                    // issued just before it.  Accumulator register e is row 8 (e >> 2) + 4 hh + (e & 3),
                    // i.e. token 16 hh + e.  The products with the low parts of the panels follow as a
                    // second, conditional pass over the same accumulators (straight-line code in both
                    // passes, operand reads issued ahead; one pass with the choice inside would make the
                    // two versions hand the working copy over in different registers).
                    auto pass = [&](auto part_tag) {
                        constexpr int PART = decltype(part_tag)::value;
#pragma unroll
                        for (int jj = 0; jj < BT; ++jj)
#pragma unroll
                            for (int c = 0; c < 4; ++c)
#pragma unroll
                                for (int jt = (blk + 1) * BT; jt < NT; ++jt) {
                                    const int pr = pair_index(BT, jt, blk * BT + jj);
                                    const half8 w = wlds[((pr * 4 + c) * 2 + PART) * 64 + lane];
                                    x[jt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop[4 * jj + c], w, x[jt], 0, 0, 0);
                                }
                    };
                    pass(std::integral_constant<int, 0>{});
                    if (need_lo) pass(std::integral_constant<int, 1>{});
                    // the next block's error tile must not overtake this block's operand reads
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
            }
            if (blk == PF_BLK) {
                if (unit < nunits) {
                    issue_loads(unit);
                } else {
                    // the loop ends after this tile: say that the old contents are dead, or they would be
                    // kept in registers up to this point
                    // (an empty statement that "writes" them: no instruction, unlike a frozen undefined value,
                    // which is materialised as zeros)
#pragma unroll
                    for (int i = 0; i < NLOAD; ++i)
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            uint32_t dead;
                            asm volatile("" : "=v"(dead));
                            pre[i][w] = dead;
                        }
                }
            }
        }

        // ---- outputs
        uint32_t bi, tile;
        locate(cur, bi, tile);
        const int64_t gt = ((bo + bi) * p.n_heads + head) * p.out_tiles + p.out_tile0 + tile;     // wave-uniform
        // codes[tile][channel][BITS words]: this lane's 16 tokens are words hh * WPT .. of its channel
        uint32_t* cdst = p.codes + gt * (kD * BITS) + n * BITS + hh * WPT;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            if constexpr (WPT == 1)
                __builtin_nontemporal_store(words[j][0], cdst + 32 * j * BITS);
            else
                __builtin_nontemporal_store(u32x2{words[j][0], words[j][1]},
                                            reinterpret_cast<u32x2*>(cdst + 32 * j * BITS));
        }
        // lanes 0..31 write the scales, lanes 32..63 the zero-points; even lanes store their
        // neighbour's value with their own (two channels per 32-bit word)
        uint16_t* mbase = (hh ? p.zero : p.scale) + gt * kD + n;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const uint32_t mine = hh ? zbits[j] : sbits[j];
            const uint32_t other = static_cast<uint32_t>(
                __builtin_amdgcn_mov_dpp(static_cast<int>(mine), 0xB1, 0xF, 0xF, true));
            if ((n & 1) == 0)
                __builtin_nontemporal_store(mine | (other << 16), reinterpret_cast<uint32_t*>(mbase + 32 * j));
        }
    }
}

template <int BITS, int BT, int DT>
int launch(const PcParams& p, int64_t n_prob, hipStream_t stream) {
    constexpr int ES = (DT == SQUAT_F32) ? 4 : 2;
    constexpr int kWaves = pc_waves_for(DT, BT);
    constexpr size_t lds = n_pairs(BT) * 8192 + kWaves * 32 * (kD * ES + 16) + 16 + 2 * 64 * 16;
    auto kern = quantize_pc_kernel<BITS, BT, DT>;
    static std::atomic<uint64_t> attr_done{0};
    if (int rc = set_max_lds_once(attr_done, reinterpret_cast<const void*>(kern), static_cast<int>(lds))) return rc;
    const dim3 grid(static_cast<unsigned>(n_prob * p.wgs_per_prob));
    hipLaunchKernelGGL(kern, grid, dim3(kWaves * kWave), lds, stream, p);
    return check_launch();
}

template <int BITS, int BT>
int dispatch_dt(squat_dtype dt, const PcParams& p, int64_t n_prob, hipStream_t s) {
    switch (dt) {
        case SQUAT_F32: return launch<BITS, BT, SQUAT_F32>(p, n_prob, s);
        case SQUAT_F16: return launch<BITS, BT, SQUAT_F16>(p, n_prob, s);
        case SQUAT_BF16: return launch<BITS, BT, SQUAT_BF16>(p, n_prob, s);
    }
    return SQUAT_E_BADDTYPE;
}
template <int BITS>
int dispatch_bt(int bt, squat_dtype dt, const PcParams& p, int64_t n_prob, hipStream_t s) {
    switch (bt) {
        case 1: return dispatch_dt<BITS, 1>(dt, p, n_prob, s);
        case 2: return dispatch_dt<BITS, 2>(dt, p, n_prob, s);
        case 4: return dispatch_dt<BITS, 4>(dt, p, n_prob, s);
    }
    return SQUAT_E_BADSHAPE;
}

}  // namespace

// The launch shape of squat_quantize_keys_per_channel for a problem size (shared with squat_quantize_keys_plan).
int squat::plan_quantize_pc(squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens, bool has_update,
                            int64_t update_stride_batch, int g, QuantPlan& out) {
    if (g != 32 && g != 64 && g != 128) return SQUAT_E_BADSHAPE;
    if (k_dt != SQUAT_F32 && k_dt != SQUAT_F16 && k_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (n_batch < 1 || n_heads < 1 || n_tokens < 1 || n_tokens % kTileTokens || update_stride_batch < 0)
        return SQUAT_E_BADSHAPE;
    if (n_batch * n_heads > (int64_t(1) << 30)) return SQUAT_E_BADSHAPE;
    out.tiles_per_seq = n_tokens / kTileTokens;
    // Workgroups are bound to one update matrix: per head when it is shared across the
    // batch, per (batch, head) otherwise.
    if (has_update && update_stride_batch != 0) {
        out.n_prob = n_batch * n_heads;
        out.n_inner = 1;
    } else {
        out.n_prob = n_heads;
        out.n_inner = n_batch;
    }
    out.units_per_prob = out.n_inner * out.tiles_per_seq;
    if (out.units_per_prob >= (int64_t(1) << 31) || out.tiles_per_seq >= (int64_t(1) << 31)) return SQUAT_E_BADSHAPE;
    const int bt = has_update ? g / 32 : 4;      // no update matrix: one block, plain round-to-nearest
    out.waves = pc_waves_for(k_dt, bt);
    int64_t per = (static_cast<int64_t>(device_cu_count()) + out.n_prob - 1) / out.n_prob;     // fill every CU once
    const int64_t need = out.units_per_prob;     // at least one tile per workgroup
    if (per > need) per = need;
    if (per < 1) per = 1;
    if (out.n_prob * per > 0x7FFFFFFF) return SQUAT_E_BADSHAPE;
    out.wgs_per_prob = static_cast<int>(per);
    return SQUAT_OK;
}

// squat_quantize_keys_per_channel into a store that holds out_stride tokens per (batch, head), starting at
// token out_offset (both multiples of 32).
int squat::quantize_keys_pc_into(const void* k, squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens,
                                 int d, int64_t k_stride_batch, int64_t k_stride_head, int64_t k_stride_token,
                                 const float* update, int64_t update_stride_batch, int bits, int group, int g,
                                 uint32_t* codes, uint16_t* scale, uint16_t* zero, int64_t out_stride,
                                 int64_t out_offset, squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (out_stride % kTileTokens || out_offset % kTileTokens || out_offset < 0 || out_offset + n_tokens > out_stride)
        return SQUAT_E_BADSHAPE;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    if (group != kTileTokens) return SQUAT_E_BADSHAPE;
    if (g != 32 && g != 64 && g != 128) return SQUAT_E_BADSHAPE;
    if (n_batch < 0 || n_heads < 0 || n_tokens < 0) return SQUAT_E_BADSHAPE;
    if (n_tokens % group) return SQUAT_E_BADSHAPE;
    if (k_dt != SQUAT_F32 && k_dt != SQUAT_F16 && k_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (n_batch == 0 || n_heads == 0 || n_tokens == 0) return SQUAT_OK;
    if (!k || !codes || !scale || !zero) return SQUAT_E_NULLPTR;
    if (k_stride_token < d || k_stride_batch < 0 || k_stride_head < 0 || update_stride_batch < 0)
        return SQUAT_E_BADSHAPE;
    if ((k_stride_token % 8) || (k_stride_head % 8) || (k_stride_batch % 8)) return SQUAT_E_ALIGN;
    if (!aligned(k, 16) || !aligned(codes, 16) || !aligned(scale, 4) || !aligned(zero, 4)) return SQUAT_E_ALIGN;
    if (update && (!aligned(update, 16) || (update_stride_batch % 4))) return SQUAT_E_ALIGN;
    if (n_batch * n_heads > (int64_t(1) << 30)) return SQUAT_E_BADSHAPE;

    const int es = elem_size(k_dt);
    PcParams p;
    p.k = static_cast<const unsigned char*>(k);
    p.sb = k_stride_batch * es;
    p.sh = k_stride_head * es;
    p.st = k_stride_token * es;
    p.update = update;
    p.usb = update_stride_batch;
    p.codes = codes;
    p.scale = scale;
    p.zero = zero;
    p.n_heads = n_heads;
    p.tiles_per_seq = n_tokens / kTileTokens;
    p.out_tiles = out_stride / kTileTokens;
    p.out_tile0 = out_offset / kTileTokens;

    QuantPlan plan;
    if (int rc = plan_quantize_pc(k_dt, n_batch, n_heads, n_tokens, update != nullptr, update_stride_batch, g, plan))
        return rc;
    if (k_stride_token * es >= (int64_t(1) << 26)) return SQUAT_E_BADSHAPE;
    const int64_t n_prob = plan.n_prob;
    p.n_inner = plan.n_inner;
    p.units_per_prob = plan.units_per_prob;
    p.wgs_per_prob = plan.wgs_per_prob;
    {
        // floor(u / dv) for u < 2^31: shift = 31 + ceil(log2 dv), mul = floor(2^shift / dv) + 1
        const uint64_t dv = static_cast<uint64_t>(p.tiles_per_seq);
        uint32_t l = 0;
        while ((uint64_t(1) << l) < dv) ++l;
        p.div_shift = 31 + l;
        p.div_mul = static_cast<uint32_t>(((uint64_t(1) << p.div_shift) / dv) + 1);
    }
    const int bt = update ? g / 32 : 4;      // no update matrix: one block, plain round-to-nearest

    hipStream_t s = static_cast<hipStream_t>(stream);
    return bits == 2 ? dispatch_bt<2>(bt, k_dt, p, n_prob, s) : dispatch_bt<4>(bt, k_dt, p, n_prob, s);
}

extern "C" int squat_quantize_keys_per_channel(const void* k, squat_dtype k_dt, int64_t n_batch, int n_heads,
                                               int64_t n_tokens, int d, int64_t k_stride_batch,
                                               int64_t k_stride_head, int64_t k_stride_token,
                                               const float* update, int64_t update_stride_batch, int bits,
                                               int group, int g, uint32_t* codes, uint16_t* scale,
                                               uint16_t* zero, squat_stream stream) {
    return squat::quantize_keys_pc_into(k, k_dt, n_batch, n_heads, n_tokens, d, k_stride_batch, k_stride_head,
                                        k_stride_token, update, update_stride_batch, bits, group, g, codes, scale,
                                        zero, n_tokens < 0 ? 0 : n_tokens, 0, stream);
}
