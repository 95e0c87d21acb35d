// Device-side helpers: bf16 <-> float/double conversion, MFMA operand types, slot addressing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "ltri_internal.h"

namespace ltri {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}

// fp32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// fp64 -> bf16 in ONE rounding (nearest even); avoids the double rounding of going
// through fp32. Finite inputs in the normal bf16 range; tiny values flush to +-0.
__device__ __forceinline__ uint16_t f64_to_bf16(double x) {
  uint64_t u = (uint64_t)__double_as_longlong(x);
  uint32_t sign = (uint32_t)(u >> 63) << 15;
  int64_t e = (int64_t)((u >> 52) & 0x7FF) - 1023 + 127;   // rebias
  if (e <= 0) return (uint16_t)sign;
  uint64_t mant = u & 0x000FFFFFFFFFFFFFull;               // 52 bits; keep the top 7
  uint64_t keep = mant >> 45;
  uint64_t rest = mant & ((1ull << 45) - 1);
  uint64_t half = 1ull << 44;
  uint32_t r = ((uint32_t)e << 7) | (uint32_t)keep;
  if (rest > half || (rest == half && (keep & 1ull))) r += 1;   // carries into the exponent correctly
  if (r >= 0x7F80u) r = 0x7F7Fu;                            // clamp instead of inf
  return (uint16_t)(sign | r);
}

template <int DT> struct Elt;
template <> struct Elt<LTRI_F32> {
  typedef float type;
  __device__ static __forceinline__ double to_f64(float v) { return (double)v; }
  __device__ static __forceinline__ float to_f32(float v) { return v; }
  __device__ static __forceinline__ float from_f64(double v) { return (float)v; }
  __device__ static __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Elt<LTRI_BF16> {
  typedef uint16_t type;
  __device__ static __forceinline__ double to_f64(uint16_t v) { return (double)bf16_to_f32(v); }
  __device__ static __forceinline__ float to_f32(uint16_t v) { return bf16_to_f32(v); }
  __device__ static __forceinline__ uint16_t from_f64(double v) { return f64_to_bf16(v); }
  __device__ static __forceinline__ uint16_t from_f32(float v) { return f32_to_bf16(v); }
};

__device__ __forceinline__ int slot_of(const Dims& D, int layer, int seq, int h) {
  return (layer * D.n_seqs + seq) * D.Hkv + h;
}
// Element offset of token 0 of a slot inside a KV arena.
__device__ __forceinline__ size_t arena_off(const Dims& D, int slot) {
  return (size_t)slot * (size_t)D.arena_rows * (size_t)D.d;
}
// Row, inside its slot, of token `tok` of the chunk that starts at token c0 (the chunk's rows are consecutive).
__device__ __forceinline__ int chunk_tok_row(const Dims& D, int c0, int tok) {
  return D.ring0 + (c0 & D.ring_mask) + (tok - c0);
}
// Row of a token of the local window (any token among the latest ring_mask + 1 ones).
__device__ __forceinline__ int window_tok_row(const Dims& D, int tok) {
  return D.ring0 + (tok & D.ring_mask);
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Value of lane (lane ^ M) for M = 1 .. 32, on the vector ALU (DPP / lane-swap instructions)
// instead of the LDS crossbar that __shfl_xor goes through.
template <int M>
__device__ __forceinline__ uint32_t lane_xor_c(uint32_t v) {
  if constexpr (M == 1) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);          // quad_perm [1,0,3,2]
  } else if constexpr (M == 2) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);          // quad_perm [2,3,0,1]
  } else if constexpr (M == 4) {
    int r = __builtin_amdgcn_update_dpp(0, (int)v, 0x104, 0xF, 0x5, false);           // banks 0, 2 <- lane + 4
    r = __builtin_amdgcn_update_dpp(r, (int)v, 0x114, 0xF, 0xA, false);               // banks 1, 3 <- lane - 4
    return (uint32_t)r;
  } else if constexpr (M == 8) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xF, 0xF, true);         // row_ror:8
  } else if constexpr (M == 16) {
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return (threadIdx.x & 16) ? r[0] : r[1];
  } else {
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (threadIdx.x & 32) ? r[0] : r[1];
  }
}
__device__ __forceinline__ bool key_less(uint64_t a1, uint32_t a2, uint64_t b1, uint32_t b2) {
  return (a1 < b1) || (a1 == b1 && a2 < b2);
}

}  // namespace ltri
