// Device-side types and small helpers shared by the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace fdc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef uint16_t bf16_t;   // storage type in global memory

// float -> bf16 bits, round to nearest even (the hardware conversion)
__device__ __forceinline__ uint16_t f2bf(float f) {
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}
__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// float -> fp16 bits, round to nearest even, saturating at the largest finite value
__device__ __forceinline__ uint16_t f2h(float f) {
    const float c = fminf(fmaxf(f, -65504.0f), 65504.0f);   // NaN stays NaN
    return __builtin_bit_cast(uint16_t, (_Float16)(f != f ? f : c));
}

// split a float into a bf16 head and a bf16 tail with head + tail ~ f to 2^-17
__device__ __forceinline__ void split_bf16(float f, uint16_t& hi, uint16_t& lo) {
    hi = f2bf(f);
    lo = f2bf(f - bf2f(hi));
}

// Operand order of the activation side of v_mfma_f32_16x16x32_bf16 for a
// [16 rows][K] matrix: element (m, k) of row tile mt lives at this offset
// (in bf16 elements) of a [mt][K/32][64 lanes][8] array.
__device__ __forceinline__ size_t act_frag_index(int m, int k, int KT) {
    const int mt = m >> 4, kt = k >> 5, kg = (k & 31) >> 3, e = k & 7;
    return ((((size_t)mt * KT + kt) * 64) + (m & 15) + 16 * kg) * 8 + e;
}

// K cache: 32-key tiles; inside a tile the operand order of the key side of
// v_mfma_f32_32x32x16_bf16: [D/16 steps][64 lanes][8], lane = key%32 + 32*((d%16)/8).
template <int D>
__device__ __forceinline__ size_t k_tile_index(int key_in_tile, int d) {
    const int j = d >> 4, h = (d & 15) >> 3, e = d & 7;
    return ((size_t)(j * 64 + key_in_tile + 32 * h)) * 8 + e;
}

// V cache: 32-key tiles holding V^T in the operand order of the value side of
// the P*V product: [D/32][2 halves of 16 keys][64 lanes][8], lane = d%32 + 32*hh,
// where inside a 16-key half key = 8*(e/4) + 4*hh + e%4 - the order in which the
// score tile of the 32x32 instruction leaves the accumulator registers.
template <int D>
__device__ __forceinline__ size_t v_tile_index(int key_in_tile, int d) {
    const int s = key_in_tile >> 4, k16 = key_in_tile & 15;
    const int e = 4 * (k16 >> 3) + (k16 & 3), hh = (k16 & 7) >> 2;
    const int dt = d >> 5;
    return ((size_t)((dt * 2 + s) * 64 + (d & 31) + 32 * hh)) * 8 + e;
}

}  // namespace fdc
