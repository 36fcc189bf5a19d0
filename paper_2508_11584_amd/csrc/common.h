// Shared device-side vocabulary for the gfx950 kernels: element types, vector types,
// the LDS chunk swizzle, and small conversion helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vpe {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;

// Source position of one output row (or column) of an aligned-corner bilinear resize, sy = y (in - 1) / (out - 1):
// lower tap and the weight of the upper one (i0 + 1, clamped to the last sample).
struct AcTap { int i0; float w1; };

// One 16-byte chunk holds CE elements of T.
template <typename T> struct Elem;
template <> struct Elem<bf16>  { static constexpr int CE = 8; };
template <> struct Elem<float> { static constexpr int CE = 4; };

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

// LDS tiles are stored as rows of 16-byte chunks; chunk c of row r lives at physical chunk
// c ^ ((r >> 1) & 7).  The gfx950 LDS has 64 banks of 4 bytes (256 bytes per cycle): a 128-byte row
// covers half of them, rows r and r + 1 the two halves, so 16 consecutive rows reading the same
// logical chunk land on 16 different 16-byte bank groups (measured: ds_read_b128 at 5.25 cycles per
// wave-instruction, the same as a linear pattern; XOR with r & 7 costs 8.0, no swizzle 32).
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ u32x4 ld_global_16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }

// Sum over the 64 lanes of a wave (butterfly), result in every lane.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__host__ __device__ constexpr int cdiv(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ constexpr int64_t rup(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

}  // namespace vpe
