// Device-side helpers shared by the gfx950 kernels.
//
// Matrix-core tiles use v_mfma_f32_32x32x16_bf16 (wave64): operand A is 32 rows x 16 k, operand B
// is 16 k x 32 columns, each lane l = 32*g + i carries 8 bf16 of row/column i, k-group g; the
// accumulator lane l holds column l%32 and rows 8*(v/4) + 4*(l/32) + v%4 for v = 0..15.
// An operand fragment is therefore 64 lanes x 16 bytes = one contiguous 1 KiB read when the data
// is stored in fragment order (expert weights, packed tokens, activations).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ef {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ floatx16 mfma32(uint4 a, uint4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ floatx16 mfma32v(u32x4_t a, u32x4_t b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// The second FFN half runs the matrix cores in fp16 (fp32 accumulation): the intermediate activation
// silu(g) * u is stored with 11 significant bits instead of bf16's 8, and the W2 section of an expert blob
// holds the fp16 numbers equal to the bf16 weights (a bf16 value of magnitude in [2^-24, 65504] is an fp16
// number; the packing call checks the upper end, values below the lower end round to the nearest
// multiple of 2^-24).  Same operand fragment layout as the bf16 instruction.
__device__ __forceinline__ floatx16 mfma32h(u32x4_t a, u32x4_t b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b),
                                                  c, 0, 0, 0);
}

// two activations -> one dword of two fp16 (round to nearest even; magnitudes beyond the largest
// finite fp16 saturate to it instead of becoming infinite)
__device__ __forceinline__ uint32_t pack_act2(float v0, float v1) {
    const float lim = 65504.f;
    v0 = fminf(fmaxf(v0, -lim), lim);
    v1 = fminf(fmaxf(v1, -lim), lim);
    return __builtin_bit_cast(uint32_t, half2_t{(_Float16)v0, (_Float16)v1});
}

// streaming (read-once) 16-byte load: keeps expert weights from displacing reused data in L2
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ void zero16(floatx16 &a) {
#pragma unroll
    for (int v = 0; v < 16; ++v) a[v] = 0.f;
}

}  // namespace ef
