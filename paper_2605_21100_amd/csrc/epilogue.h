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

// Two floats -> two OCP FP8 E4M3FN codes in the low 16 bits (first value in the low byte): round to nearest even,
// saturating at +-448 (the format has no infinity; the conversion instruction alone would produce NaN beyond the
// range), NaN -> a NaN code.  gfx950's packed conversion produces the OCP format; the saturation is done here.
__device__ inline uint32_t f32x2_to_e4m3(float a, float b) {
  a = a != a ? a : __builtin_amdgcn_fmed3f(a, -448.f, 448.f);  // the clamp must not turn a NaN into a number
  b = b != b ? b : __builtin_amdgcn_fmed3f(b, -448.f, 448.f);
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false) & 0xffffu;
}

// Store N consecutive elements (N = 1, 4 or 8; idx a multiple of N) of a final row.
// kind: NANOCP_F32, NANOCP_BF16, or NANOCP_FP8_E4M3 (code of value * inv_scale, inv_scale = 1 / out_scale in fp32).
template <int N>
__device__ inline void store_final(void* out, size_t idx, int kind, float inv_scale, const float (&v)[N]) {
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
      o[0] = (uint8_t)f32x2_to_e4m3(v[0] * inv_scale, 0.f);
    } else {
      uint32_t w[N >= 4 ? N / 4 : 1];
#pragma unroll
      for (int i = 0; i < N / 4; ++i)
        w[i] = f32x2_to_e4m3(v[4 * i] * inv_scale, v[4 * i + 1] * inv_scale) |
               (f32x2_to_e4m3(v[4 * i + 2] * inv_scale, v[4 * i + 3] * inv_scale) << 16);
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
// multiplier of the fp8 epilogue: 1 / out_scale rounded to fp32 (out_scale <= 0 means 1)
inline float out_inv_scale_of(const nanocp_attn_desc& d) { return d.out_scale > 0.f ? 1.f / d.out_scale : 1.f; }

}  // namespace nanocp
