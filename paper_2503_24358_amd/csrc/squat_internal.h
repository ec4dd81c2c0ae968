// Internal helpers shared by the HIP sources of libsquat (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

}  // namespace squat
