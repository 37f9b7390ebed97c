// Device-side helpers shared by the libitq3s kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace itq3s {

constexpr int kBlock = 256;        // elements per quantization block (the transform length)
constexpr int kTileRows = 16;      // rows per storage tile
constexpr int kTileWords = 384;    // uint32 per tile: 256 low-plane + 128 high-plane
constexpr int kTileLoWords = 256;
constexpr int kWave = 64;

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }

__device__ __forceinline__ float f16_bits_to_f32(uint32_t bits16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}

// Cross-lane exchange with lane (l ^ mask), 32-bit payload.
__device__ __forceinline__ int xor_lane_i32(int v, int mask) { return __shfl_xor(v, mask, 64); }
__device__ __forceinline__ float xor_lane_f32(float v, int mask) { return __shfl_xor(v, mask, 64); }
__device__ __forceinline__ double xor_lane_f64(double v, int mask) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_xor(lo, mask, 64);
    hi = __shfl_xor(hi, mask, 64);
    return __hiloint2double(hi, lo);
}

// value of lane (l ^ MASK), MASK < 32, through the LDS crossbar (ds_swizzle in bit-mask mode: no
// memory access).  One instruction per 32 bits for any distance, and it runs beside the vector ALU
// rather than on it -- data-parallel-primitive moves need two per distance 4 or 8 and measured 12 %
// slower in the fp64 butterfly kernels, which are bound by vector-ALU issue.
template <int MASK>
__device__ __forceinline__ int row_xor_i32(int x) {
    return __builtin_amdgcn_ds_swizzle(x, (MASK << 10) | 0x1F);
}
template <int MASK>
__device__ __forceinline__ double row_xor_f64(double v) {
    const int lo = row_xor_i32<MASK>(__double2loint(v)), hi = row_xor_i32<MASK>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

}  // namespace itq3s
