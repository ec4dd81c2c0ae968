// Internal helpers shared by the HIP sources of libsquat (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "squat.h"

namespace squat {

constexpr int kD = 128;            // head size supported by this version
constexpr int kWave = 64;          // CDNA wavefront
constexpr int kTileTokens = 32;    // tokens per wavefront tile (MFMA N dimension)

inline int elem_size(squat_dtype dt) {
    switch (dt) {
        case SQUAT_F32: return 4;
        case SQUAT_F16: return 2;
        case SQUAT_BF16: return 2;
    }
    return 0;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? SQUAT_OK : SQUAT_E_HIP;
}

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// Round an fp32 value to fp16 (nearest even) and return it widened again.
__device__ __forceinline__ float round_f16(float v, uint16_t& bits) {
    _Float16 h = static_cast<_Float16>(v);
    bits = __builtin_bit_cast(uint16_t, h);
    return static_cast<float>(h);
}

// MFMA 32x32 accumulator layout on a 64-lane wavefront: lane (hh = lane >> 5,
// n = lane & 31) owns column n and rows 8*q + 4*hh + i for q, i in 0..3, in
// accumulator register 4*q + i.  The kernels that keep a 32-channel tile of a
// key in such an accumulator name the rows so that each lane owns 16
// CONSECUTIVE channels: row m  <->  channel 16*((m>>2)&1) + 4*(m>>3) + (m&3),
// i.e. lane half hh, register e  <->  channel 16*hh + e of the tile.
__host__ __device__ __forceinline__ int row_to_channel(int m) {
    return 16 * ((m >> 2) & 1) + 4 * (m >> 3) + (m & 3);
}

// Tile pairs (jt, s) of 32-channel tiles with a non-zero update panel: block(jt) > block(s), BT tiles
// per block, kD / 32 tiles per key.  Enumerated in the order the panels are laid out in LDS.
__host__ __device__ constexpr int n_pairs(int BT) {
    int c = 0;
    for (int s = 0; s < kD / 32; ++s)
        for (int jt = (s / BT + 1) * BT; jt < kD / 32; ++jt) ++c;
    return c;
}
__host__ __device__ constexpr int pair_index(int BT, int jt, int s) {
    int c = 0;
    for (int ss = 0; ss < kD / 32; ++ss)
        for (int j = (ss / BT + 1) * BT; j < kD / 32; ++j) {
            if (ss == s && j == jt) return c;
            ++c;
        }
    return -1;
}

// min / max as the single machine instruction (the C library functions add one instruction per
// operand that only matters for signalling NaNs when the operands come out of a lane exchange).
__device__ __forceinline__ float raw_min(float a, float b) {
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float raw_max(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// min (or max) of a value with the same value in lane ^ 32.
__device__ __forceinline__ float pair_min(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(as_u32(v), as_u32(v), false, false);
    return raw_min(as_f32(r[0]), as_f32(r[1]));
}
__device__ __forceinline__ float pair_max(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(as_u32(v), as_u32(v), false, false);
    return raw_max(as_f32(r[0]), as_f32(r[1]));
}

// Entry points with an explicit output / input placement inside a larger store (used by the cache).
int quantize_keys_into(const void* k, squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens, int d,
                       int64_t k_stride_batch, int64_t k_stride_head, int64_t k_stride_token, const float* update,
                       int64_t update_stride_batch, int bits, int group, int g, uint32_t* codes, uint16_t* scale,
                       uint16_t* zero, int64_t out_stride, int64_t out_offset, squat_stream stream);
int quantize_keys_pc_into(const void* k, squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens, int d,
                          int64_t k_stride_batch, int64_t k_stride_head, int64_t k_stride_token, const float* update,
                          int64_t update_stride_batch, int bits, int group, int g, uint32_t* codes, uint16_t* scale,
                          uint16_t* zero, int64_t out_stride, int64_t out_offset, squat_stream stream);
int key_scores_from(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t n_batch,
                    int n_kv_heads, int64_t n_tokens, int64_t store_stride, int d, int bits, int group,
                    const void* q, squat_dtype q_dt, int q_per_kv, int64_t q_stride_batch, int64_t q_stride_head,
                    float out_scale, float* scores, int64_t s_stride_batch, int64_t s_stride_head,
                    squat_stream stream);
int key_scores_pc_from(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t n_batch,
                       int n_kv_heads, int64_t n_tokens, int64_t store_tokens, int d, int bits, int group,
                       const void* q, squat_dtype q_dt, int q_per_kv, int64_t q_stride_batch, int64_t q_stride_head,
                       float out_scale, float* scores, int64_t s_stride_batch, int64_t s_stride_head,
                       squat_stream stream);

int key_scores_rope_from(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t n_batch,
                         int n_kv_heads, int64_t n_tokens, int64_t store_stride, int d, int bits, int group,
                         const float* inv_freq, int64_t pos0, const void* q, squat_dtype q_dt, int q_per_kv,
                         int64_t q_stride_batch, int64_t q_stride_head, float out_scale, float* scores,
                         int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream);

int key_scores_pc_rope_from(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t n_batch,
                            int n_kv_heads, int64_t n_tokens, int64_t store_tokens, int d, int bits, int group,
                            const float* inv_freq, int64_t pos0, const void* q, squat_dtype q_dt, int q_per_kv,
                            int64_t q_stride_batch, int64_t q_stride_head, float out_scale, float* scores,
                            int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream);

#if defined(__HIPCC__)
// cos and sin of position * freq: the product is reduced to a fraction of a turn in fp64 first
__device__ __forceinline__ void turn_sincos(double position, float freq, float& c, float& s) {
    const double turns = position * static_cast<double>(freq) * 0.15915494309189535;   // / (2 pi)
    const double frac = turns - rint(turns);                                           // [-0.5, 0.5]
    sincospif(static_cast<float>(2.0 * frac), &s, &c);
}
#endif

// Raises a kernel's dynamic-LDS limit once per device and process.  `done` holds one bit per device
// ordinal; threads that race only repeat the (idempotent) runtime call.
inline int set_max_lds_once(std::atomic<uint64_t>& done, const void* kernel, int bytes) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SQUAT_E_HIP;
    const uint64_t bit = uint64_t(1) << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return SQUAT_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return SQUAT_E_HIP;
    }
    done.fetch_or(bit, std::memory_order_release);
    return SQUAT_OK;
}

// How a quantize launch spreads its 32-token tiles: `problems` update matrices, each served by
// `wgs_per_prob` persistent workgroups of `waves` wavefronts that stride over `units_per_prob` tiles.
struct QuantPlan {
    int64_t n_prob;
    int64_t n_inner;         // batch entries that share one update matrix
    int64_t tiles_per_seq;
    int64_t units_per_prob;
    int wgs_per_prob;
    int waves;
};
int plan_quantize(squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens, bool has_update,
                  int64_t update_stride_batch, int group, int g, QuantPlan& out);
int plan_quantize_pc(squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens, bool has_update,
                     int64_t update_stride_batch, int g, QuantPlan& out);

// Number of compute units of the current device (256 if the query fails).
inline int device_cu_count() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return 256;
    return cus;
}

}  // namespace squat
