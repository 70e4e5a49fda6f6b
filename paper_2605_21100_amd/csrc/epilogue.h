// Output epilogue shared by every kernel that writes rows in their final form (the Phase 4 merge, the tile
// reduction, and the tile kernels' direct path): float32, bfloat16 or OCP FP8 E4M3FN with a caller-supplied scale.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "nanocp.h"

namespace nanocp {

// float -> bfloat16 bits, round to nearest even
__device__ inline uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// float -> OCP FP8 E4M3FN code (bias 7, max 448, no infinity): round to nearest even, saturating; NaN -> 0x7f.
// Written with integer arithmetic from the format's definition, so the result does not depend on a conversion
// instruction's saturation mode.
__device__ inline uint32_t f32_to_e4m3(float f) {
  const uint32_t u = __float_as_uint(f);
  const uint32_t sign = (u >> 24) & 0x80u;
  uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return sign | 0x7fu;
  if (a >= 0x43e00000u) return sign | 0x7eu;  // |f| >= 448 (infinity included): the largest finite code
  if (a < 0x3c800000u) {                      // below 2^-6: multiples of 2^-9; 8 * 2^-9 is the smallest normal, code 8
    return sign | (uint32_t)__float2int_rn(__uint_as_float(a) * 512.f);
  }
  a += 0x7ffffu + ((a >> 20) & 1u);           // keep 3 fraction bits, ties to even (a carry moves to the exponent)
  return sign | ((a >> 20) - (120u << 3));    // rebias 127 -> 7; at most 0x7e because a < 448 rounds to <= 448
}

// Store N consecutive elements (N = 1, 4 or 8; idx a multiple of N) of a final row.
// kind: NANOCP_F32, NANOCP_BF16, or NANOCP_FP8_E4M3 (code of value / scale).
template <int N>
__device__ inline void store_final(void* out, size_t idx, int kind, float scale, const float (&v)[N]) {
  static_assert(N == 1 || N == 4 || N == 8, "vector width");
  if (kind == NANOCP_F32) {
    float* o = (float*)out + idx;
    if (N == 1) {
      o[0] = v[0];
    } else {
#pragma unroll
      for (int i = 0; i < N; i += 4) *(float4*)(o + i) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
    }
  } else if (kind == NANOCP_BF16) {
    uint16_t* o = (uint16_t*)out + idx;
    if (N == 1) {
      o[0] = (uint16_t)f32_to_bf16_rne(v[0]);
    } else {
      uint32_t w[N >= 2 ? N / 2 : 1];
#pragma unroll
      for (int i = 0; i < N / 2; ++i) w[i] = f32_to_bf16_rne(v[2 * i]) | (f32_to_bf16_rne(v[2 * i + 1]) << 16);
      if (N == 4) *(uint2*)o = make_uint2(w[0], w[1]);
      if (N == 8) *(uint4*)o = make_uint4(w[0], w[1], w[N == 8 ? 2 : 0], w[N == 8 ? 3 : 0]);
    }
  } else {
    uint8_t* o = (uint8_t*)out + idx;
    if (N == 1) {
      o[0] = (uint8_t)f32_to_e4m3(v[0] / scale);
    } else {
      uint32_t w[N >= 4 ? N / 4 : 1];
#pragma unroll
      for (int i = 0; i < N / 4; ++i)
        w[i] = f32_to_e4m3(v[4 * i] / scale) | (f32_to_e4m3(v[4 * i + 1] / scale) << 8) |
               (f32_to_e4m3(v[4 * i + 2] / scale) << 16) | (f32_to_e4m3(v[4 * i + 3] / scale) << 24);
      if (N == 4) *(uint32_t*)o = w[0];
      if (N == 8) *(uint2*)o = make_uint2(w[0], w[N == 8 ? 1 : 0]);
    }
  }
}

// a row of zeros in the given format (+0 in all three)
template <int N>
__device__ inline void store_final_zero(void* out, size_t idx, int kind) {
  const float z[N] = {};
  store_final<N>(out, idx, kind == NANOCP_FP8_E4M3 ? NANOCP_FP8_E4M3 : kind, 1.f, z);
}

inline bool final_dtype_ok(int dt) { return dt == NANOCP_F32 || dt == NANOCP_BF16 || dt == NANOCP_FP8_E4M3; }
inline float out_scale_of(const nanocp_attn_desc& d) { return d.out_scale > 0.f ? d.out_scale : 1.f; }

}  // namespace nanocp
