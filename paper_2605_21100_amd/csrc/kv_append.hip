// Writer for the paged KV layouts the attention kernels read (include/nanocp.h, "Memory layouts"): scatters the
// K / V rows of n tokens into their pages.  A decode step appends one token per request to the instance's own KV
// partition before Phase 2 (paper: Data Plane, per-instance KV partition); a bulk call converts a plain cache.
// Pure data movement: one thread per 16-byte vector of the source rows.
#include <hip/hip_runtime.h>

#include "plan.h"

namespace nanocp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// kEl = bytes per kv element, x = 16 / kEl elements per 16-byte vector
template <int kEl>
__global__ __launch_bounds__(kThreads) void kv_append_kernel(const char* __restrict__ k_new, const char* __restrict__ v_new,
                                                             const int32_t* __restrict__ bt_row,
                                                             const int32_t* __restrict__ position, int n,
                                                             char* __restrict__ k_pool, char* __restrict__ v_pool,
                                                             const int32_t* __restrict__ block_table, int max_blocks,
                                                             int Hkv, int Dk, int Dv, int ps, int mla) {
  constexpr int x = 16 / kEl;
  const int kvec = Dk / x, vvec = mla ? 0 : Dv / x;  // 16-byte vectors per (token, head) of K and of V
  const int64_t per_tok = (int64_t)Hkv * (kvec + vvec);
  const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (id >= (int64_t)n * per_tok) return;
  const int t = (int)(id / per_tok);
  int rest = (int)(id % per_tok);
  const int h = rest / (kvec + vvec);
  rest %= kvec + vvec;
  const int pos = position[t];
  const size_t page = (size_t)block_table[(size_t)bt_row[t] * max_blocks + pos / ps];
  const int slot = pos % ps;
  if (mla) {
    // k_pool [pages, ps, Dk]: plain rows
    const u32x4 v = *(const u32x4*)(k_new + ((size_t)t * Dk + (size_t)rest * x) * kEl);
    *(u32x4*)(k_pool + ((page * ps + slot) * Dk + (size_t)rest * x) * kEl) = v;
    return;
  }
  const int grp = slot / (4 * x), w = slot % (4 * x);  // token group of 4x slots, slot inside it
  if (rest < kvec) {
    // k_pool [pages, Hkv, ps/4x, Dk/x, 4x, x]: vector (c, w) = dims [cx, cx + x) of slot w
    const int c = rest;
    const u32x4 v = *(const u32x4*)(k_new + (((size_t)t * Hkv + h) * Dk + (size_t)c * x) * kEl);
    const size_t vec = (((page * Hkv + h) * (ps / (4 * x)) + grp) * kvec + c) * (4 * x) + w;
    *(u32x4*)(k_pool + vec * 16) = v;
  } else {
    // v_pool [pages, Hkv, ps/x, Dv, x]: slot w = 16b + 4g + i of group grp is element 4b + i of vector u = 4 grp + g
    const int c0 = (rest - kvec) * x;  // first of the x dims this thread moves
    const int b = w / 16, g = (w % 16) / 4, i = w % 4;
    const int u = 4 * grp + g, e = 4 * b + i;
    const char* src = v_new + (((size_t)t * Hkv + h) * Dv + c0) * kEl;
    char* dst = v_pool + ((((page * Hkv + h) * (ps / x) + u) * Dv + c0) * x + e) * kEl;
#pragma unroll
    for (int j = 0; j < x; ++j) {
      if (kEl == 4) *(uint32_t*)(dst + (size_t)j * 16) = *(const uint32_t*)(src + j * 4);
      if (kEl == 2) *(uint16_t*)(dst + (size_t)j * 16) = *(const uint16_t*)(src + j * 2);
      if (kEl == 1) *(uint8_t*)(dst + (size_t)j * 16) = *(const uint8_t*)(src + j);
    }
  }
}

}  // namespace
}  // namespace nanocp

extern "C" nanocp_status nanocp_kv_append(const nanocp_attn_desc* desc, const void* k_new, const void* v_new,
                                          const int32_t* bt_row, const int32_t* position, int32_t n, void* k_pool,
                                          void* v_pool, const int32_t* block_table, int32_t max_blocks_per_row,
                                          void* stream) {
  using namespace nanocp;
  if (!desc || n < 0 || max_blocks_per_row <= 0) return NANOCP_EINVAL;
  const nanocp_status st = check_desc(*desc);
  if (st != NANOCP_OK) return st;
  if (n == 0) return NANOCP_OK;
  const bool mla = desc->kind == NANOCP_MLA;
  if (!k_new || !bt_row || !position || !k_pool || !block_table || (!mla && (!v_new || !v_pool))) return NANOCP_EINVAL;
  if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_pool | (uintptr_t)v_pool) & 15) return NANOCP_EINVAL;
  const int el = desc->kv_dtype == NANOCP_F32 ? 4 : desc->kv_dtype == NANOCP_BF16 ? 2 : 1;
  const int x = 16 / el;
  if (!mla && desc->head_dim_v % x) return NANOCP_ESHAPE;
  const int64_t vecs =
      (int64_t)n * desc->num_kv_heads * (desc->head_dim_qk / x + (mla ? 0 : desc->head_dim_v / x));
  const int64_t blocks = (vecs + kThreads - 1) / kThreads;
  if (blocks > 0x7fffffff) return NANOCP_EBOUNDS;
  auto launch = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, (const char*)k_new,
                       (const char*)v_new, bt_row, position, (int)n, (char*)k_pool, (char*)v_pool, block_table,
                       (int)max_blocks_per_row, (int)desc->num_kv_heads, (int)desc->head_dim_qk, (int)desc->head_dim_v,
                       (int)desc->page_size, (int)mla);
  };
  if (el == 4)
    launch(kv_append_kernel<4>);
  else if (el == 2)
    launch(kv_append_kernel<2>);
  else
    launch(kv_append_kernel<1>);
  return hipGetLastError() == hipSuccess ? NANOCP_OK : NANOCP_EHIP;
}
