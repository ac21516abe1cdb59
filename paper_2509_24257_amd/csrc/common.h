// Shared device helpers for the gfx950 kernels: bf16 storage, 64-lane wave reductions, vector types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vl {

typedef __bf16 bf16;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte register quad for staged copies
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int WAVE = 64;

// Tiled image of a K-contiguous bf16 matrix [rows][K] (K a multiple of 32; rows padded to a multiple of 256): blocks of
// 256 rows, and inside a block one contiguous 16 KB piece per k-tile of 32 (256 rows x 64 bytes).  This is exactly
// what one k-step of a 256-row GEMM tile loads, so every such load covers whole 128-byte lines.  The operands of the
// bf16 GEMMs (weights, normalised rows, attention output, SwiGLU output) live in this layout.
constexpr int TL_ROWS = 256, TL_K = 32, TL_PIECE = TL_ROWS * TL_K;
__host__ __device__ __forceinline__ int64_t tiled_off(int64_t row, int64_t k, int64_t K) {
    return ((row >> 8) * (K >> 5) + (k >> 5)) * TL_PIECE + (row & 255) * TL_K + (k & 31);
}

// Storage-type conversions.  float -> bf16 is the hardware convert (round to nearest, ties to even).
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// silu(g) * u of the bf16 GEMM epilogues.  The result is rounded to bf16 (8 bits), so the hardware reciprocal (1 ulp of
// fp32) replaces the division sequence, which was a third of the SwiGLU epilogue's instructions.  Both bf16 GEMM kernels
// use this one expression, so the prefill and the token-by-token path round alike.
__device__ __forceinline__ float silu_mul(float g, float u) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u; }

// Butterfly reductions over the 64 lanes of a wave; every lane ends with the result.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}

}  // namespace vl
