// squat_quantize_keys: the iteration of Algorithm 1's `Quant` with the block
// update of Lemma 2, for per-token groups of channels, on gfx950.
//
// One wavefront owns a tile of 32 tokens x 128 channels.  The working copy of
// the keys lives in registers in the MFMA 32x32 accumulator layout with a token
// as a COLUMN: lane (hh, n) holds, for token n, channels 16*hh .. 16*hh+15 of
// each 32-channel tile.  In that layout
//   - a group's min/max is an in-register reduction plus one exchange with
//     lane ^ 32,
//   - the normalised rounding error of a frozen tile is already the B operand
//     of  W (channels x g) * E (g x tokens), so the update of Lemma 2 needs no
//     data movement between lanes,
//   - 16 two-bit codes of a lane are exactly one 32-bit word of the packed
//     output.
// The contraction runs on the fp16 matrix cores with both operands split into
// a high and a low fp16 part (three products per tile), accumulating in fp32;
// the error is kept in units of the group's scale so that its fp16 split has a
// fixed range.  Workgroups are persistent and bound to one head: the head's
// update panels are converted once into LDS, in MFMA A-operand order.
#include <type_traits>

#include "squat_internal.h"

using namespace squat;

namespace {

constexpr int NT = kD / 32;          // 32-channel tiles per key
// Wavefronts per workgroup: one workgroup per CU, sized by LDS (update panels + one staging tile per
// wavefront) and registers: 12 waves (3 per SIMD) for 16-bit keys, 6 for fp32 keys.
// Variants that keep more live state (two tiles per block, or statistics over four tiles) get 8 waves so
// that each may use 256 registers instead of spilling at 168.
__host__ __device__ constexpr int waves_for(int dt, int gt, int bt) {
    return dt == SQUAT_F32 ? 6 : ((bt == 2 || (gt == 4 && bt == 1)) ? 8 : 12);
}
constexpr int kWgsPerCU = 1;
constexpr float kFastOffset = 32.0f;   // largest |zero| / scale for which the one-multiply-add path is used

struct QuantParams {
    const unsigned char* k;
    int64_t sb, sh, st;              // key strides in BYTES
    const float* update;
    int64_t usb;                     // update stride per outer-batch entry, elements
    uint32_t* codes;
    uint16_t* scale;
    uint16_t* zero;
    int64_t n_tokens;
    int64_t out_stride;              // tokens per (batch, head) in the output store (>= n_tokens)
    int64_t out_offset;              // first output token
    int64_t n_inner;                 // batch entries that share one update matrix
    int n_heads;
    int64_t tiles_per_seq;
    int64_t units_per_prob;          // n_inner * tiles_per_seq, < 2^31
    int wgs_per_prob;
    uint32_t div_mul;                // unit / tiles_per_seq == (unit * div_mul) >> div_shift for unit < 2^31
    uint32_t div_shift;
};

template <int DT>
struct Elem {
    static constexpr int size = (DT == SQUAT_F32) ? 4 : 2;
};

// 16 consecutive channels (raw bytes in LDS) -> 16 floats.
template <int DT>
__device__ __forceinline__ void load16(const unsigned char* src, float* out) {
    if constexpr (DT == SQUAT_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f32x4 v = *reinterpret_cast<const f32x4*>(src + 16 * i);
            out[4 * i + 0] = v[0]; out[4 * i + 1] = v[1]; out[4 * i + 2] = v[2]; out[4 * i + 3] = v[3];
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            u32x4 v = *reinterpret_cast<const u32x4*>(src + 16 * i);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                if constexpr (DT == SQUAT_BF16) {
                    out[8 * i + 2 * w + 0] = as_f32(v[w] << 16);
                    out[8 * i + 2 * w + 1] = as_f32(v[w] & 0xFFFF0000u);
                } else {
                    const uint32_t word = v[w];
                    out[8 * i + 2 * w + 0] =
                        static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(word & 0xFFFFu)));
                    out[8 * i + 2 * w + 1] =
                        static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(word >> 16)));
                }
            }
        }
    }
}

// After the call lanes 32..63 of `a` hold what lanes 0..31 of `b` held and vice versa.
__device__ __forceinline__ void swap_halves(uint32_t& a, uint32_t& b) {
    auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    a = r[0];
    b = r[1];
}

// Split 8 floats into packed fp16 high and low parts (hi + lo ~ value to 2^-22).
__device__ __forceinline__ void split8(const float* v, half8& hi, half8& lo) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        _Float16 h = static_cast<_Float16>(v[i]);
        hi[i] = h;
        lo[i] = static_cast<_Float16>(v[i] - static_cast<float>(h));
    }
}

template <int BITS, int GT, int BT, int DT>
__global__ void __launch_bounds__(waves_for(DT, GT, BT) * kWave, kWgsPerCU) quantize_kernel(const QuantParams p) {
    constexpr int kWaves = waves_for(DT, GT, BT);
    constexpr int ES = Elem<DT>::size;
    constexpr int ROWB = kD * ES;                 // bytes of one key
    constexpr int LROW = ROWB + 16;               // padded LDS row: conflict-free b128 column reads
    constexpr int CPR = ROWB / 16;                // 16-byte chunks per key
    constexpr int NLOAD = 32 * CPR / kWave;       // 16-byte loads per lane per tile
    constexpr int NPAIRS = n_pairs(BT);
    constexpr int NB = NT / BT;                   // blocks (iterations) per key
    constexpr int NG = NT / GT;                   // groups per key
    constexpr int WPT = BITS / 2;                 // packed words per lane per tile
    constexpr int CPH = 16 / BITS;                // codes per 16-bit half-word
    constexpr float LV = static_cast<float>((1 << BITS) - 1);

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    half8* wlds = reinterpret_cast<half8*>(smem);           // [NPAIRS][2 kk][hi, lo][64 lanes]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5;
    const int n = lane & 31;
    unsigned char* stage = smem + NPAIRS * 4096 + wave * (32 * LROW);

    const int64_t prob = blockIdx.x / p.wgs_per_prob;
    const int wg = blockIdx.x % p.wgs_per_prob;
    const int head = static_cast<int>(prob % p.n_heads);
    const int64_t bo = prob / p.n_heads;

    // The first tile's loads are issued before the panels are converted: their latency overlaps that work.
    const uint32_t st32 = static_cast<uint32_t>(p.st);
    u32x4 pre[NLOAD];
    // unit -> (batch entry, first token): exact multiply-shift division by tiles_per_seq (units < 2^31)
    auto locate = [&](uint32_t u, uint32_t& bi, int64_t& tok0) {
        bi = static_cast<uint32_t>((static_cast<uint64_t>(u) * p.div_mul) >> p.div_shift);
        tok0 = static_cast<int64_t>(u - bi * static_cast<uint32_t>(p.tiles_per_seq)) * kTileTokens;
    };
    auto issue_loads = [&](uint32_t u) {
        uint32_t bi;
        int64_t tok0;
        locate(u, bi, tok0);
        const unsigned char* base = p.k + (bo + bi) * p.sb + head * p.sh + tok0 * p.st;
        const int64_t left = p.n_tokens - tok0;                 // >= 1 valid rows in this tile
        const int last = left >= kTileTokens ? kTileTokens - 1 : static_cast<int>(left) - 1;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const int flat = i * kWave + lane;
            int row = flat / CPR;
            const int ch = flat % CPR;
            row = row < last ? row : last;      // rows past the end re-read the last valid key; their outputs are not stored
            // streamed once: non-temporal, so the tile does not displace the update panels in L2
            pre[i] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4*>(base + (static_cast<uint32_t>(row) * st32 + ch * 16)));
        }
    };

    const uint32_t nunits = static_cast<uint32_t>(p.units_per_prob);
    const uint32_t ustride = static_cast<uint32_t>(p.wgs_per_prob) * kWaves;
    // Wavefront v of workgroup w starts at tile v * workgroups + w: a problem with few tiles (a decode-time flush)
    // is spread over the workgroups first, so its wavefronts do not share a SIMD.
    uint32_t unit = static_cast<uint32_t>(wave) * static_cast<uint32_t>(p.wgs_per_prob) + wg;
    if (unit < nunits) issue_loads(unit);


    // Panels whose entries are all fp16 numbers (as squat_prepare writes them) have a zero low part:
    // the third matrix product is skipped for the whole head.
    bool need_lo = false;
    int* lo_flag = reinterpret_cast<int*>(smem + NPAIRS * 4096 + kWaves * (32 * LROW));
    if constexpr (NPAIRS > 0) {
        if (tid == 0) *lo_flag = 0;
        __syncthreads();
        // Convert this head's panels once: A operand of pair (jt, s), MFMA kk: lane (ha, m)
        // holds U[32 jt + channel(m)][32 s + 16 ha + 8 kk + 0..7].
        const float* U = p.update + bo * p.usb + static_cast<int64_t>(head) * kD * kD;
        for (int idx = tid; idx < NPAIRS * 2 * 64; idx += kWaves * kWave) {
            const int pr = idx >> 7;
            const int kk = (idx >> 6) & 1;
            const int l = idx & 63;
            int jt = 0, s = 0;
            {
                int c = 0;
                for (int ss = 0; ss < NT; ++ss)
                    for (int j = (ss / BT + 1) * BT; j < NT; ++j) {
                        if (c == pr) { jt = j; s = ss; }
                        ++c;
                    }
            }
            const int ha = l >> 5, m = l & 31;
            const int row = 32 * jt + row_to_channel(m);
            const int col = 32 * s + 16 * ha + 8 * kk;
            const f32x4* src = reinterpret_cast<const f32x4*>(U + row * kD + col);
            const f32x4 a = src[0], b = src[1];
            const float v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
            half8 hi, lo;
            split8(v, hi, lo);
            wlds[((pr * 2 + kk) * 2 + 0) * 64 + l] = hi;
            wlds[((pr * 2 + kk) * 2 + 1) * 64 + l] = lo;
            const u32x4 lb = __builtin_bit_cast(u32x4, lo);
            if (((lb[0] | lb[1] | lb[2] | lb[3]) & 0x7FFF7FFFu) != 0u) *lo_flag = 1;
        }
        __syncthreads();
        need_lo = *lo_flag != 0;
    }

    while (unit < nunits) {
        // ---- registers -> LDS (token-major rows), then read back channel-major per lane
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const int flat = i * kWave + lane;
            const int row = flat / CPR, ch = flat % CPR;
            *reinterpret_cast<u32x4*>(stage + row * LROW + ch * 16) = pre[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        const uint32_t cur = unit;
        unit += ustride;

        float x[NT][16];
#pragma unroll
        for (int j = 0; j < NT; ++j)
            load16<DT>(stage + n * LROW + (32 * j + 16 * hh) * ES, x[j]);

        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        if (unit < nunits) issue_loads(unit);   // prefetch the next tile

        uint32_t words[NT][WPT];
        uint16_t sbits[NG], zbits[NG];
        float g_scale[NG], g_inv[NG], g_zero[NG], g_top[NG];
        bool g_risky[NG];

#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            // ---- statistics of the groups that start in this block (current values)
#pragma unroll
            for (int j = blk * BT; j < (blk + 1) * BT; ++j) {
                if (j % GT == 0) {
                    const int gi = j / GT;
                    float mn = x[j][0], mx = x[j][0];
#pragma unroll
                    for (int jj = j; jj < j + GT; ++jj)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            mn = fminf(mn, x[jj][e]);
                            mx = fmaxf(mx, x[jj][e]);
                        }
                    mn = pair_min(mn);
                    mx = pair_max(mx);
                    // Correctly rounded (max - min) / (2^b - 1) by one Newton step on the rounded
                    // reciprocal of the constant divisor: an exact quotient (frequent with 16-bit
                    // inputs) stays exact, so a tie of the fp16 rounding below breaks to even, as the
                    // definition does.
                    const float rng = mx - mn;
                    constexpr float RL = 1.0f / LV;
                    const float q0 = rng * RL;
                    const float dl = fmaf(fmaf(-q0, LV, rng), RL, q0);
                    const float sh = round_f16(dl, sbits[gi]);
                    g_zero[gi] = round_f16(mn, zbits[gi]);
                    const bool live = sh > 0.0f;
                    const float sp = live ? sh : 1.0f;
                    float inv = __builtin_amdgcn_rcpf(sp);
                    inv = fmaf(fmaf(-sp, inv, 1.0f), inv, inv);
                    g_scale[gi] = sp;
                    g_inv[gi] = inv;
                    g_top[gi] = live ? LV : 0.0f;
                    g_risky[gi] = !(sh >= 6.2e-5f) || fabsf(g_zero[gi]) * inv > kFastOffset;
                }
            }
            // ---- quantize and freeze the block; keep its normalised error as MFMA B operands
            // Two versions of the block.  The careful one clamps to [0, 2^b - 1] (which can only bite when
            // the fp16 rounding of zero/scale moved the group's ends by more than half a step: scale not a
            // normal fp16 number, incl. 0, or |zero| / scale > 256) and computes (x - m) / Delta as
            // written.  The cheap one folds the zero-point into one multiply-add, x * (1/Delta) - m/Delta,
            // whose rounding error grows with |m| / Delta: the whole wavefront takes it only while that
            // ratio stays below 32 in every group of the block (error < 5e-6 steps).
            bool risky = false;
#pragma unroll
            for (int jj = 0; jj < BT; ++jj) {
                const int gi = (blk * BT + jj) / GT;
                risky = risky || g_risky[gi];
            }
            // A group that spans several blocks (G > g) has its later blocks updated after its statistics
            // were taken: those can leave the range, so there the clamp is part of the definition.
            const bool clamp = (GT > BT && (blk * BT) % GT != 0) || __builtin_amdgcn_ballot_w64(risky) != 0ull;
            u32x4 bhi[BT][2], blo[BT][2];
            auto quant_block = [&](auto clamp_tag) {
                constexpr bool CLAMP = decltype(clamp_tag)::value;
#pragma unroll
                for (int jj = 0; jj < BT; ++jj) {
                    const int j = blk * BT + jj;
                    const int gi = j / GT;
                    const float mh = g_zero[gi], inv = g_inv[gi], top = g_top[gi];
                    const float nmi = -mh * inv;
                    // codes are collected per half-word as exact small floats (Horner), then converted once
                    uint32_t hw[16 / CPH];
                    float eh[16], el[16];
#pragma unroll
                    for (int q = 16 / CPH - 1; q >= 0; --q) {
                        float accf = 0.0f;
#pragma unroll
                        for (int e = CPH - 1; e >= 0; --e) {
                            const int c = q * CPH + e;
                            float code, et;
                            if constexpr (CLAMP) {
                                const float dd = x[j][c] - mh;
                                const float u = __builtin_amdgcn_fmed3f(dd * inv, 0.0f, top);
                                code = __builtin_rintf(u);
                                et = fmaf(-inv, dd, code);
                            } else {
                                const float u = fmaf(x[j][c], inv, nmi);
                                code = __builtin_rintf(u);
                                et = code - u;
                            }
                            accf = fmaf(accf, static_cast<float>(1 << BITS), code);
                            if (blk < NB - 1) {
                                // normalised error  code - (x - m)/Delta  split into a part with 11
                                // significant bits (exact in fp16) and the exact remainder
                                eh[c] = as_f32(as_u32(et) & 0xFFFFE000u);
                                el[c] = et - eh[c];
                            }
                        }
                        hw[q] = static_cast<uint32_t>(accf);
                    }
#pragma unroll
                    for (int w = 0; w < WPT; ++w) words[j][w] = hw[2 * w] | (hw[2 * w + 1] << 16);
                    if (blk < NB - 1) {
#pragma unroll
                        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                bhi[jj][kk][i] = __builtin_bit_cast(
                                    uint32_t, __builtin_amdgcn_cvt_pkrtz(eh[8 * kk + 2 * i], eh[8 * kk + 2 * i + 1]));
                                blo[jj][kk][i] = __builtin_bit_cast(
                                    uint32_t, __builtin_amdgcn_cvt_pkrtz(el[8 * kk + 2 * i], el[8 * kk + 2 * i + 1]));
                            }
                    }
                }
            };
            if (clamp)
                quant_block(std::true_type{});
            else
                quant_block(std::false_type{});
            // ---- Lemma 2: remaining channels += U[rest, block] * error
            if constexpr (NPAIRS > 0) {
                if (blk < NB - 1) {
                    // Straight-line code, so that the operand reads of a chain can be issued ahead of its
                    // matrix products.  The products with the low parts of the panels, needed only when some
                    // panel entry is not an fp16 number, are a second, conditional pass (one pass with the
                    // choice inside makes its two versions hand the working copy over in different registers:
                    // a register move per value where they join).
                    auto pass = [&](auto lo_tag) {
                        constexpr bool LO = decltype(lo_tag)::value;
#pragma unroll
                        for (int jt = (blk + 1) * BT; jt < NT; ++jt) {
#pragma unroll
                            for (int jj = 0; jj < BT; ++jj) {
                                const int s = blk * BT + jj;
                                const int pr = pair_index(BT, jt, s);
                                f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                                for (int kk = 0; kk < 2; ++kk) {
                                    const half8 w = wlds[((pr * 2 + kk) * 2 + (LO ? 1 : 0)) * 64 + lane];
                                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(w, __builtin_bit_cast(half8, bhi[jj][kk]), acc, 0, 0, 0);
                                    if constexpr (!LO)
                                        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(w, __builtin_bit_cast(half8, blo[jj][kk]), acc, 0, 0, 0);
                                }
                                const float sc = g_scale[s / GT];
#pragma unroll
                                for (int e = 0; e < 16; ++e) x[jt][e] = fmaf(sc, acc[e], x[jt][e]);
                            }
                        }
                    };
                    pass(std::false_type{});
                    if (need_lo) pass(std::true_type{});
                }
            }
        }

        // ---- outputs
        uint32_t bi;
        int64_t tok0;
        locate(cur, bi, tok0);
        const bool valid = tok0 + n < p.n_tokens;
        const int64_t row0 = ((bo + bi) * p.n_heads + head) * p.out_stride + p.out_offset + tok0;     // wave-uniform

        // lower half-wave collects the first half of a key's words, upper the second
#pragma unroll
        for (int w = 0; w < WPT; ++w) {
            swap_halves(words[0][w], words[2][w]);
            swap_halves(words[1][w], words[3][w]);
        }
        if (valid) {
            uint32_t* dst = p.codes + row0 * (NT * 2 * WPT) + (n * (NT * 2 * WPT) + hh * (NT * WPT));
            if constexpr (WPT == 1) {
                __builtin_nontemporal_store(u32x4{words[0][0], words[2][0], words[1][0], words[3][0]},
                                            reinterpret_cast<u32x4*>(dst));
            } else {
                __builtin_nontemporal_store(u32x4{words[0][0], words[0][1], words[2][0], words[2][1]},
                                            reinterpret_cast<u32x4*>(dst));
                __builtin_nontemporal_store(u32x4{words[1][0], words[1][1], words[3][0], words[3][1]},
                                            reinterpret_cast<u32x4*>(dst + 4));
            }
            // lanes 0..31 write the scales, lanes 32..63 the zero-points
            uint16_t* mdst = (hh ? p.zero : p.scale) + row0 * NG + n * NG;
            if constexpr (NG == 4) {
                const uint32_t lo = hh ? (zbits[0] | (uint32_t(zbits[1]) << 16)) : (sbits[0] | (uint32_t(sbits[1]) << 16));
                const uint32_t hi = hh ? (zbits[2] | (uint32_t(zbits[3]) << 16)) : (sbits[2] | (uint32_t(sbits[3]) << 16));
                __builtin_nontemporal_store(u32x2{lo, hi}, reinterpret_cast<u32x2*>(mdst));
            } else if constexpr (NG == 2) {
                __builtin_nontemporal_store(
                    hh ? (zbits[0] | (uint32_t(zbits[1]) << 16)) : (sbits[0] | (uint32_t(sbits[1]) << 16)),
                    reinterpret_cast<uint32_t*>(mdst));
            } else {
                *mdst = hh ? zbits[0] : sbits[0];
            }
        }
    }
}

template <int BITS, int GT, int BT, int DT>
int launch(const QuantParams& p, int64_t n_prob, hipStream_t stream) {
    constexpr int ES = Elem<DT>::size;
    constexpr int kWaves = waves_for(DT, GT, BT);
    constexpr size_t lds = n_pairs(BT) * 4096 + kWaves * 32 * (kD * ES + 16) + 16;
    auto kern = quantize_kernel<BITS, GT, BT, DT>;
    static std::atomic<uint64_t> attr_done{0};
    if (int rc = set_max_lds_once(attr_done, reinterpret_cast<const void*>(kern), static_cast<int>(lds))) return rc;
    const dim3 grid(static_cast<unsigned>(n_prob * p.wgs_per_prob));
    hipLaunchKernelGGL(kern, grid, dim3(kWaves * kWave), lds, stream, p);
    return check_launch();
}

template <int BITS, int GT, int BT>
int dispatch_dt(squat_dtype dt, const QuantParams& p, int64_t n_prob, hipStream_t s) {
    switch (dt) {
        case SQUAT_F32: return launch<BITS, GT, BT, SQUAT_F32>(p, n_prob, s);
        case SQUAT_F16: return launch<BITS, GT, BT, SQUAT_F16>(p, n_prob, s);
        case SQUAT_BF16: return launch<BITS, GT, BT, SQUAT_BF16>(p, n_prob, s);
    }
    return SQUAT_E_BADDTYPE;
}
template <int BITS, int GT>
int dispatch_bt(int bt, squat_dtype dt, const QuantParams& p, int64_t n_prob, hipStream_t s) {
    switch (bt) {
        case 1: return dispatch_dt<BITS, GT, 1>(dt, p, n_prob, s);
        case 2: return dispatch_dt<BITS, GT, 2>(dt, p, n_prob, s);
        case 4: return dispatch_dt<BITS, GT, 4>(dt, p, n_prob, s);
    }
    return SQUAT_E_BADSHAPE;
}
template <int BITS>
int dispatch_gt(int gt, int bt, squat_dtype dt, const QuantParams& p, int64_t n_prob, hipStream_t s) {
    switch (gt) {
        case 1: return dispatch_bt<BITS, 1>(bt, dt, p, n_prob, s);
        case 2: return dispatch_bt<BITS, 2>(bt, dt, p, n_prob, s);
        case 4: return dispatch_bt<BITS, 4>(bt, dt, p, n_prob, s);
    }
    return SQUAT_E_BADSHAPE;
}

}  // namespace

// The launch shape of squat_quantize_keys for a problem size: shared by the launcher and by
// squat_quantize_keys_plan, so that what a caller is told is what runs.
int squat::plan_quantize(squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens, bool has_update,
                         int64_t update_stride_batch, int group, int g, QuantPlan& out) {
    if (group != 32 && group != 64 && group != 128) return SQUAT_E_BADSHAPE;
    if (g != 32 && g != 64 && g != 128) return SQUAT_E_BADSHAPE;
    if (k_dt != SQUAT_F32 && k_dt != SQUAT_F16 && k_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (n_batch < 1 || n_heads < 1 || n_tokens < 1 || update_stride_batch < 0) return SQUAT_E_BADSHAPE;
    if (n_batch * n_heads > (int64_t(1) << 30)) return SQUAT_E_BADSHAPE;
    out.tiles_per_seq = (n_tokens + kTileTokens - 1) / kTileTokens;
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
    const int gt = group / 32;
    const int bt = has_update ? g / 32 : 4;      // no update matrix: one block, plain round-to-nearest
    if (!(gt % bt == 0 || bt % gt == 0)) return SQUAT_E_BADSHAPE;
    out.waves = waves_for(k_dt, gt, bt);
    const int64_t target = kWgsPerCU * static_cast<int64_t>(device_cu_count());   // fill every CU once
    int64_t per = (target + out.n_prob - 1) / out.n_prob;
    const int64_t need = out.units_per_prob;     // at least one tile per workgroup
    if (per > need) per = need;
    if (per < 1) per = 1;
    if (out.n_prob * per > 0x7FFFFFFF) return SQUAT_E_BADSHAPE;
    out.wgs_per_prob = static_cast<int>(per);
    return SQUAT_OK;
}

// squat_quantize_keys with the outputs placed at tokens out_offset .. of a store that holds out_stride
// tokens per (batch, head): what a cache appends with.
int squat::quantize_keys_into(const void* k, squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens,
                              int d, int64_t k_stride_batch, int64_t k_stride_head, int64_t k_stride_token,
                              const float* update, int64_t update_stride_batch, int bits, int group, int g,
                              uint32_t* codes, uint16_t* scale, uint16_t* zero, int64_t out_stride,
                              int64_t out_offset, squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    if (group != 32 && group != 64 && group != 128) return SQUAT_E_BADSHAPE;
    if (g != 32 && g != 64 && g != 128) return SQUAT_E_BADSHAPE;
    if (n_batch < 0 || n_heads < 0 || n_tokens < 0) return SQUAT_E_BADSHAPE;
    if (out_offset < 0 || out_stride < out_offset + n_tokens) return SQUAT_E_BADSHAPE;
    if (k_dt != SQUAT_F32 && k_dt != SQUAT_F16 && k_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (n_batch == 0 || n_heads == 0 || n_tokens == 0) return SQUAT_OK;
    if (!k || !codes || !scale || !zero) return SQUAT_E_NULLPTR;
    if (k_stride_token < d || k_stride_batch < 0 || k_stride_head < 0 || update_stride_batch < 0)
        return SQUAT_E_BADSHAPE;
    if ((k_stride_token % 8) || (k_stride_head % 8) || (k_stride_batch % 8)) return SQUAT_E_ALIGN;
    if (!aligned(k, 16) || !aligned(codes, 16) || !aligned(scale, 8) || !aligned(zero, 8)) return SQUAT_E_ALIGN;
    // the kernel stores 16-byte pieces of codes and 8-byte pieces of metadata per key
    if ((out_stride * (d * bits / 8)) % 16 || (out_offset * (d * bits / 8)) % 16) return SQUAT_E_ALIGN;
    if (update && (!aligned(update, 16) || (update_stride_batch % 4))) return SQUAT_E_ALIGN;
    if (n_batch * n_heads > (int64_t(1) << 30)) return SQUAT_E_BADSHAPE;

    const int es = elem_size(k_dt);
    QuantParams p;
    p.k = static_cast<const unsigned char*>(k);
    p.sb = k_stride_batch * es;
    p.sh = k_stride_head * es;
    p.st = k_stride_token * es;
    p.update = update;
    p.usb = update_stride_batch;
    p.codes = codes;
    p.scale = scale;
    p.zero = zero;
    p.n_tokens = n_tokens;
    p.out_stride = out_stride;
    p.out_offset = out_offset;
    p.n_heads = n_heads;
    p.tiles_per_seq = (n_tokens + kTileTokens - 1) / kTileTokens;

    QuantPlan plan;
    if (int rc = plan_quantize(k_dt, n_batch, n_heads, n_tokens, update != nullptr, update_stride_batch, group, g, plan))
        return rc;
    if (k_stride_token * es >= (int64_t(1) << 26)) return SQUAT_E_BADSHAPE;
    const int64_t n_prob = plan.n_prob;
    p.n_inner = plan.n_inner;
    p.units_per_prob = plan.units_per_prob;
    p.wgs_per_prob = plan.wgs_per_prob;
    {
        // floor(u / d) for u < 2^31: shift = 31 + ceil(log2 d), mul = floor(2^shift / d) + 1
        const uint64_t dv = static_cast<uint64_t>(p.tiles_per_seq);
        uint32_t l = 0;
        while ((uint64_t(1) << l) < dv) ++l;
        p.div_shift = 31 + l;
        p.div_mul = static_cast<uint32_t>(((uint64_t(1) << p.div_shift) / dv) + 1);
    }
    const int gt = group / 32;
    const int bt = update ? g / 32 : 4;      // no update matrix: one block, plain round-to-nearest

    if (!(gt % bt == 0 || bt % gt == 0)) return SQUAT_E_BADSHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return bits == 2 ? dispatch_gt<2>(gt, bt, k_dt, p, n_prob, s)
                     : dispatch_gt<4>(gt, bt, k_dt, p, n_prob, s);
}

extern "C" int squat_quantize_keys(const void* k, squat_dtype k_dt, int64_t n_batch, int n_heads,
                                   int64_t n_tokens, int d, int64_t k_stride_batch,
                                   int64_t k_stride_head, int64_t k_stride_token,
                                   const float* update, int64_t update_stride_batch, int bits,
                                   int group, int g, uint32_t* codes, uint16_t* scale,
                                   uint16_t* zero, squat_stream stream) {
    return squat::quantize_keys_into(k, k_dt, n_batch, n_heads, n_tokens, d, k_stride_batch, k_stride_head,
                                     k_stride_token, update, update_stride_batch, bits, group, g, codes, scale,
                                     zero, n_tokens, 0, stream);
}
