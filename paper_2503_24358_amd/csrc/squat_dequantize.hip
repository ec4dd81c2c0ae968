// squat_dequantize_keys: deq(c) = c * Delta + m (Section 2 of the paper) over the
// packed store written by squat_quantize_keys.  Pure streaming: one thread turns
// 16 channels of one key (one or two packed words, one scale, one zero) into 16
// output elements; a wavefront covers 8 consecutive keys, so code reads are one
// contiguous 256/512-byte run and output writes one contiguous 2/4-KB run.
//
// squat_dequantize_keys_per_channel reads the token-major store of the
// per-channel mode: one wavefront rebuilds one tile of 32 tokens; a lane owns 8
// consecutive channels (one 16-byte piece of an output row) of 8 tokens, so it
// needs 8 packed words, 8 scales and 8 zero-points, and writes whole rows.
#include "squat_internal.h"

using namespace squat;

namespace {

struct DeqParams {
    const uint32_t* codes;
    const uint16_t* scale;
    const uint16_t* zero;
    unsigned char* out;
    int64_t ob, oh, ot;      // output strides in BYTES
    int64_t n_tokens;
    int n_heads;
    uint32_t div_mul, div_shift;    // bh / n_heads == (bh * div_mul) >> div_shift for bh < 2^31
};

// Two floats -> two bf16 (round to nearest even, NaN stays NaN) in one word: the hardware conversion.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

template <int DT>
__device__ __forceinline__ void store16(unsigned char* dst, const float* v) {
    if constexpr (DT == SQUAT_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<f32x4*>(dst + 16 * i) = f32x4{v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]};
    } else {
        uint32_t w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (DT == SQUAT_F16) {
                half2v h;
                h[0] = static_cast<_Float16>(v[2 * i]);
                h[1] = static_cast<_Float16>(v[2 * i + 1]);
                w[i] = __builtin_bit_cast(uint32_t, h);
            } else {
                w[i] = pack_bf16(v[2 * i], v[2 * i + 1]);
            }
        }
        *reinterpret_cast<u32x4*>(dst) = u32x4{w[0], w[1], w[2], w[3]};
        *reinterpret_cast<u32x4*>(dst + 16) = u32x4{w[4], w[5], w[6], w[7]};
    }
}

// grid: x over (token, 16-channel chunk), y/z over (batch, head)
template <int BITS, int GROUP, int DT>
__global__ void __launch_bounds__(256) dequantize_kernel(const DeqParams p) {
    constexpr int ES = (DT == SQUAT_F32) ? 4 : 2;
    constexpr int WPK = kD * BITS / 32;       // words per key
    constexpr int NG = kD / GROUP;            // groups per key
    constexpr int WPC = BITS / 2;             // words per 16-channel chunk
    const int64_t bh = static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y;
    const int64_t flat = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t tok = flat >> 3;
    const int chunk = static_cast<int>(flat & 7);
    if (tok >= p.n_tokens) return;
    // exact multiply-shift division (a 64-bit division is ~60 scalar instructions in front of every
    // wavefront's first load, and the wavefronts of this kernel are short)
    const int64_t b = static_cast<int64_t>((static_cast<uint64_t>(bh) * p.div_mul) >> p.div_shift);
    const int64_t h = bh - b * p.n_heads;
    const int64_t row = bh * p.n_tokens + tok;

    uint32_t w[WPC];
    if constexpr (WPC == 1) {
        w[0] = p.codes[row * WPK + chunk];
    } else {
        const u32x2 v = *reinterpret_cast<const u32x2*>(p.codes + row * WPK + 2 * chunk);
        w[0] = v[0];
        w[1] = v[1];
    }
    const int gi = chunk * 16 / GROUP;
    float sc = static_cast<float>(__builtin_bit_cast(_Float16, p.scale[row * NG + gi]));
    float zp = static_cast<float>(__builtin_bit_cast(_Float16, p.zero[row * NG + gi]));
    // converted once: folded into the 16 multiply-adds as mixed-precision operands they would issue at half rate
    asm volatile("" : "+v"(sc), "+v"(zp));

    float v[16];
    constexpr int IPW = 32 / BITS;
    constexpr uint32_t MASK = (1u << BITS) - 1u;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t c = (w[i / IPW] >> (BITS * (i % IPW))) & MASK;
        v[i] = fmaf(static_cast<float>(c), sc, zp);
    }
    unsigned char* dst = p.out + b * p.ob + h * p.oh + tok * p.ot + chunk * 16 * ES;
    store16<DT>(dst, v);
}

// One wavefront per tile of 32 tokens.  Lane (s = lane >> 4, pc = lane & 15): channels 8 pc .. 8 pc + 7,
// tokens 8 s .. 8 s + 7 of the tile.  Token j of the tile sits in word j / (32 / BITS) of its channel
// at bit BITS * (j mod 32 / BITS), so the lane's 8 tokens are BITS consecutive bytes of one word.
template <int BITS, int DT>
__global__ void __launch_bounds__(256) dequantize_pc_kernel(const DeqParams p, const int64_t tiles_per_seq) {
    constexpr int ES = (DT == SQUAT_F32) ? 4 : 2;
    const int lane = threadIdx.x & 63;
    const int64_t bh = static_cast<int64_t>(blockIdx.z) * gridDim.y + blockIdx.y;
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (tile >= tiles_per_seq) return;
    // exact multiply-shift division (a 64-bit division is ~60 scalar instructions in front of every
    // wavefront's first load, and the wavefronts of this kernel are short)
    const int64_t b = static_cast<int64_t>((static_cast<uint64_t>(bh) * p.div_mul) >> p.div_shift);
    const int64_t h = bh - b * p.n_heads;
    const int64_t gt = bh * tiles_per_seq + tile;
    const int s = lane >> 4, pc = lane & 15;

    const int widx = 8 * s * BITS / 32;               // word of the channel that holds tokens 8 s .. 8 s + 7
    const int shift0 = (8 * s * BITS) % 32;
    // The tile's packed words come in with one (two for 4 bits) 16-byte load per lane, contiguous over the
    // wavefront, and go through a wavefront-private LDS tile to the lanes that unpack them (a lane's own 8
    // words are 4 BITS bytes apart in memory: fetched directly, every load instruction touched 16 to 32
    // sectors for 256 bytes).  Every 16 words of the tile are followed by 4 words of padding, which spreads
    // the 16 lanes of a token group over the banks.
    constexpr int TW = kD * BITS;                     // words per tile
    __shared__ __attribute__((aligned(16))) uint32_t tile_lds[4][TW + TW / 4];
    uint32_t* tl = tile_lds[threadIdx.x >> 6];
    const uint32_t* ct = p.codes + gt * TW;
#pragma unroll
    for (int i = 0; i < TW / 256; ++i) {
        const int idx = (i * 64 + lane) * 4;
        *reinterpret_cast<u32x4*>(tl + idx + (idx >> 4) * 4) =
            __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ct + idx));
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint32_t w[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int idx = (8 * pc + c) * BITS + widx;
        w[c] = tl[idx + (idx >> 4) * 4] >> shift0;
    }
    const u32x4 sraw = *reinterpret_cast<const u32x4*>(p.scale + gt * kD + 8 * pc);
    const u32x4 zraw = *reinterpret_cast<const u32x4*>(p.zero + gt * kD + 8 * pc);
    float sc[8], zp[8];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        sc[2 * c] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(sraw[c] & 0xFFFFu)));
        sc[2 * c + 1] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(sraw[c] >> 16)));
        zp[2 * c] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(zraw[c] & 0xFFFFu)));
        zp[2 * c + 1] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(zraw[c] >> 16)));
    }
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    unsigned char* dst = p.out + b * p.ob + h * p.oh + (tile * kTileTokens + 8 * s) * p.ot + pc * 8 * ES;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float v[8];
#pragma unroll
        for (int c = 0; c < 8; ++c)
            v[c] = fmaf(static_cast<float>((w[c] >> (BITS * i)) & MASK), sc[c], zp[c]);
        unsigned char* o = dst + i * p.ot;
        if constexpr (DT == SQUAT_F32) {
            *reinterpret_cast<f32x4*>(o) = f32x4{v[0], v[1], v[2], v[3]};
            *reinterpret_cast<f32x4*>(o + 16) = f32x4{v[4], v[5], v[6], v[7]};
        } else {
            uint32_t pk[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if constexpr (DT == SQUAT_F16) {
                    half2v hv;
                    hv[0] = static_cast<_Float16>(v[2 * c]);
                    hv[1] = static_cast<_Float16>(v[2 * c + 1]);
                    pk[c] = __builtin_bit_cast(uint32_t, hv);
                } else {
                    pk[c] = pack_bf16(v[2 * c], v[2 * c + 1]);
                }
            }
            *reinterpret_cast<u32x4*>(o) = u32x4{pk[0], pk[1], pk[2], pk[3]};
        }
    }
}

template <int BITS>
int launch_pc(squat_dtype dt, const DeqParams& p, int64_t tiles, dim3 grid, hipStream_t s) {
    switch (dt) {
        case SQUAT_F32: hipLaunchKernelGGL((dequantize_pc_kernel<BITS, SQUAT_F32>), grid, dim3(256), 0, s, p, tiles); break;
        case SQUAT_F16: hipLaunchKernelGGL((dequantize_pc_kernel<BITS, SQUAT_F16>), grid, dim3(256), 0, s, p, tiles); break;
        case SQUAT_BF16: hipLaunchKernelGGL((dequantize_pc_kernel<BITS, SQUAT_BF16>), grid, dim3(256), 0, s, p, tiles); break;
        default: return SQUAT_E_BADDTYPE;
    }
    return check_launch();
}

// (batch, head) pairs over grid y / z: an exact factorisation so that every (y, z) is a real pair.
bool split_bh(int64_t bh, int64_t& gy, int64_t& gz) {
    gy = bh;
    gz = 1;
    if (gy > 65535) {
        gy = 0;
        for (int64_t cand = 65535; cand >= 1; --cand)
            if (bh % cand == 0) { gy = cand; break; }
        gz = bh / gy;
    }
    return gz <= 65535;
}

template <int BITS, int GROUP>
int launch_dt(squat_dtype dt, const DeqParams& p, dim3 grid, hipStream_t s) {
    switch (dt) {
        case SQUAT_F32: hipLaunchKernelGGL((dequantize_kernel<BITS, GROUP, SQUAT_F32>), grid, dim3(256), 0, s, p); break;
        case SQUAT_F16: hipLaunchKernelGGL((dequantize_kernel<BITS, GROUP, SQUAT_F16>), grid, dim3(256), 0, s, p); break;
        case SQUAT_BF16: hipLaunchKernelGGL((dequantize_kernel<BITS, GROUP, SQUAT_BF16>), grid, dim3(256), 0, s, p); break;
        default: return SQUAT_E_BADDTYPE;
    }
    return check_launch();
}

template <int BITS>
int launch_group(int group, squat_dtype dt, const DeqParams& p, dim3 grid, hipStream_t s) {
    switch (group) {
        case 32: return launch_dt<BITS, 32>(dt, p, grid, s);
        case 64: return launch_dt<BITS, 64>(dt, p, grid, s);
        case 128: return launch_dt<BITS, 128>(dt, p, grid, s);
    }
    return SQUAT_E_BADSHAPE;
}

}  // namespace

extern "C" int squat_dequantize_keys(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                                     int64_t n_batch, int n_heads, int64_t n_tokens, int d, int bits,
                                     int group, void* k_out, squat_dtype out_dt, int64_t o_stride_batch,
                                     int64_t o_stride_head, int64_t o_stride_token, squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    if (group != 32 && group != 64 && group != 128) return SQUAT_E_BADSHAPE;
    if (n_batch < 0 || n_heads < 0 || n_tokens < 0) return SQUAT_E_BADSHAPE;
    if (out_dt != SQUAT_F32 && out_dt != SQUAT_F16 && out_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (n_batch == 0 || n_heads == 0 || n_tokens == 0) return SQUAT_OK;
    if (!codes || !scale || !zero || !k_out) return SQUAT_E_NULLPTR;
    if (o_stride_token < d || o_stride_batch < 0 || o_stride_head < 0) return SQUAT_E_BADSHAPE;
    if ((o_stride_token % 8) || (o_stride_head % 8) || (o_stride_batch % 8)) return SQUAT_E_ALIGN;
    if (!aligned(k_out, 16) || !aligned(codes, 16) || !aligned(scale, 2) || !aligned(zero, 2)) return SQUAT_E_ALIGN;

    const int es = elem_size(out_dt);
    DeqParams p;
    p.codes = codes;
    p.scale = scale;
    p.zero = zero;
    p.out = static_cast<unsigned char*>(k_out);
    p.ob = o_stride_batch * es;
    p.oh = o_stride_head * es;
    p.ot = o_stride_token * es;
    p.n_tokens = n_tokens;
    p.n_heads = n_heads;
    if (n_batch * n_heads >= (int64_t(1) << 31)) return SQUAT_E_BADSHAPE;
    {
        // floor(u / d) for u < 2^31: shift = 31 + ceil(log2 d), mul = floor(2^shift / d) + 1
        const uint64_t dv = static_cast<uint64_t>(n_heads);
        uint32_t l = 0;
        while ((uint64_t(1) << l) < dv) ++l;
        p.div_shift = 31 + l;
        p.div_mul = static_cast<uint32_t>(((uint64_t(1) << p.div_shift) / dv) + 1);
    }

    const int64_t gx = (n_tokens * 8 + 255) / 256;
    int64_t gy, gz;
    if (!split_bh(n_batch * n_heads, gy, gz) || gx > 0x7FFFFFFF) return SQUAT_E_BADSHAPE;
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy), static_cast<unsigned>(gz));
    hipStream_t s = static_cast<hipStream_t>(stream);
    return bits == 2 ? launch_group<2>(group, out_dt, p, grid, s)
                     : launch_group<4>(group, out_dt, p, grid, s);
}

extern "C" int squat_dequantize_keys_per_channel(const uint32_t* codes, const uint16_t* scale,
                                                 const uint16_t* zero, int64_t n_batch, int n_heads,
                                                 int64_t n_tokens, int d, int bits, int group, void* k_out,
                                                 squat_dtype out_dt, int64_t o_stride_batch,
                                                 int64_t o_stride_head, int64_t o_stride_token,
                                                 squat_stream stream) {
    if (d != kD) return SQUAT_E_BADSHAPE;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    if (group != kTileTokens) return SQUAT_E_BADSHAPE;
    if (n_batch < 0 || n_heads < 0 || n_tokens < 0 || n_tokens % group) return SQUAT_E_BADSHAPE;
    if (out_dt != SQUAT_F32 && out_dt != SQUAT_F16 && out_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (n_batch == 0 || n_heads == 0 || n_tokens == 0) return SQUAT_OK;
    if (!codes || !scale || !zero || !k_out) return SQUAT_E_NULLPTR;
    if (o_stride_token < d || o_stride_batch < 0 || o_stride_head < 0) return SQUAT_E_BADSHAPE;
    if ((o_stride_token % 8) || (o_stride_head % 8) || (o_stride_batch % 8)) return SQUAT_E_ALIGN;
    if (!aligned(k_out, 16) || !aligned(codes, 16) || !aligned(scale, 16) || !aligned(zero, 16)) return SQUAT_E_ALIGN;

    const int es = elem_size(out_dt);
    DeqParams p;
    p.codes = codes;
    p.scale = scale;
    p.zero = zero;
    p.out = static_cast<unsigned char*>(k_out);
    p.ob = o_stride_batch * es;
    p.oh = o_stride_head * es;
    p.ot = o_stride_token * es;
    p.n_tokens = n_tokens;
    p.n_heads = n_heads;
    if (n_batch * n_heads >= (int64_t(1) << 31)) return SQUAT_E_BADSHAPE;
    {
        // floor(u / d) for u < 2^31: shift = 31 + ceil(log2 d), mul = floor(2^shift / d) + 1
        const uint64_t dv = static_cast<uint64_t>(n_heads);
        uint32_t l = 0;
        while ((uint64_t(1) << l) < dv) ++l;
        p.div_shift = 31 + l;
        p.div_mul = static_cast<uint32_t>(((uint64_t(1) << p.div_shift) / dv) + 1);
    }

    const int64_t tiles = n_tokens / kTileTokens;
    const int64_t gx = (tiles + 3) / 4;
    int64_t gy, gz;
    if (!split_bh(n_batch * n_heads, gy, gz) || gx > 0x7FFFFFFF) return SQUAT_E_BADSHAPE;
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy), static_cast<unsigned>(gz));
    hipStream_t s = static_cast<hipStream_t>(stream);
    return bits == 2 ? launch_pc<2>(out_dt, p, tiles, grid, s) : launch_pc<4>(out_dt, p, tiles, grid, s);
}
