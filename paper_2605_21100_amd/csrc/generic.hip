// Shape-generic tile kernel (any head counts, dims <= 576/512, page sizes, f32 / bf16 / fp8 KV, GQA or MLA).
// Plain fp32 FMA arithmetic; it is the path for fp32 inputs (where 1e-5 parity needs fp32 products)
// and for shapes the MFMA kernels do not cover.  One workgroup runs the tiles of one chunk; for each
// tile it walks the tokens 64 at a time:  scores -> online softmax (wavefront reductions) -> P*V.
// Paper: Data Plane, Phase 2 (partial attention output and its LSE over the local KV partition).
#include <hip/hip_runtime.h>

#include "epilogue.h"
#include "plan.h"

namespace nanocp {

namespace {

constexpr int kTok = 64;     // tokens per step
constexpr int kHeads = 16;   // query heads processed together
constexpr int kMaxDk = 576;
constexpr int kAccPerThread = (kHeads * 512) / kThreads;  // 32

__device__ inline float ld_elem(const float* p, size_t i) { return p[i]; }
__device__ inline float ld_elem(const uint16_t* p, size_t i) { return __uint_as_float((uint32_t)p[i] << 16); }
__device__ inline float ld_elem(const uint8_t* p, size_t i) {
  // OCP E4M3FN -> float (hardware conversion of byte 0 of the source dword)
  return __builtin_amdgcn_cvt_f32_fp8((int)p[i], 0);
}

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <typename QT, typename KT>
__global__ __launch_bounds__(kThreads) void generic_partial_kernel(KParams p) {
  __shared__ float qs[kHeads * kMaxDk];
  __shared__ float sc[kHeads][kTok];
  __shared__ float m_s[kHeads], l_s[kHeads], alpha_s[kHeads];
  __shared__ int page_s[kTok], slot_s[kTok];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const QT* q = (const QT*)p.q;
  const KT* kp = (const KT*)p.k_pool;
  const KT* vp = (const KT*)p.v_pool;
  constexpr int x = 16 / (int)sizeof(KT);
  const bool mla = p.kind == NANOCP_MLA;
  const bool fp8 = sizeof(KT) == 1;
  const int Dk = p.Dk, Dv = p.Dv, ps = p.ps, Hkv = p.Hkv, G = p.G;

  // plan image: launched for the bucket's capacity; an image of another kernel variant, or one with grouped final
  // rows but no final output, is not run
  if (p.header && ((int)blockIdx.x >= p.header[0] || p.header[4] != p.variant || (p.header[5] != 0 && !p.final_out)))
    return;
  const int t0 = p.chunk_offsets[blockIdx.x], t1 = p.chunk_offsets[blockIdx.x + 1];
  for (int ti = t0; ti < t1; ++ti) {
    const DevTile tile = p.tiles[ti];
    uint64_t clk0 = 0;
    if (p.tile_clock && tid == 0) clk0 = wall_clock64();
    const int h = tile.kv_head;
    const int32_t* bt = p.block_table + (size_t)tile.bt_row * p.max_blocks;

    for (int g0 = 0; g0 < G; g0 += kHeads) {
      const int GH = min(kHeads, G - g0);
      const int a0 = h * G + g0;  // first query head of the group
      __syncthreads();
      for (int i = tid; i < GH * Dk; i += kThreads) {
        const int g = i / Dk, d = i - g * Dk;
        qs[g * Dk + d] = ld_elem(q, ((size_t)tile.q_row * p.Hq + a0 + g) * Dk + d);
      }
      if (tid < kHeads) {
        m_s[tid] = -INFINITY;
        l_s[tid] = 0.f;
      }
      float acc[kAccPerThread];
#pragma unroll
      for (int i = 0; i < kAccPerThread; ++i) acc[i] = 0.f;
      __syncthreads();

      for (int tb = tile.tok_begin; tb < tile.tok_end; tb += kTok) {
        const int n = min(kTok, tile.tok_end - tb);
        if (tid < n) {
          const int t = tb + tid;
          page_s[tid] = bt[t / ps];
          slot_s[tid] = t % ps;
        }
        __syncthreads();
        // scores
        for (int i = tid; i < GH * kTok; i += kThreads) {
          const int g = i / kTok, j = i - g * kTok;
          float s = -INFINITY;
          if (j < n) {
            const int page = page_s[j], slot = slot_s[j];
            const float* qg = qs + g * Dk;
            float dot = 0.f;
            if (mla) {
              const size_t base = ((size_t)page * ps + slot) * Dk;
              for (int d = 0; d < Dk; ++d) dot = fmaf(qg[d], ld_elem(kp, base + d), dot);
            } else {
              // K: token groups of 4x slots, [group][Dk/x][4x][x]
              const size_t base = (((size_t)page * Hkv + h) * (ps / (4 * x)) + slot / (4 * x)) * (size_t)(Dk / x) * 4 * x * x;
              for (int c = 0; c < Dk / x; ++c) {
                const size_t vb = base + ((size_t)c * 4 * x + slot % (4 * x)) * x;
#pragma unroll
                for (int e = 0; e < x; ++e) dot = fmaf(qg[c * x + e], ld_elem(kp, vb + e), dot);
              }
            }
            if (fp8) dot *= p.k_scale[(size_t)page * Hkv + h];
            s = dot * p.scale;
          }
          sc[g][j] = s;
        }
        __syncthreads();
        // online softmax, one wavefront per head
        for (int g = wave; g < GH; g += kThreads / 64) {
          const float s = sc[g][lane];
          const float m_old = m_s[g];
          const float m_new = fmaxf(m_old, wave_max(s));  // finite: the step holds at least one token
          float pj = lane < n ? expf(s - m_new) : 0.f;
          const float sum = wave_sum(pj);
          const float alpha = expf(m_old - m_new);  // exp(-inf) = 0 on the first step
          if (fp8 && lane < n) pj *= p.v_scale[(size_t)page_s[lane] * Hkv + h];
          sc[g][lane] = pj;
          if (lane == 0) {
            m_s[g] = m_new;
            l_s[g] = l_s[g] * alpha + sum;
            alpha_s[g] = alpha;
          }
        }
        __syncthreads();
        // acc = acc * alpha + P V
#pragma unroll
        for (int i = 0; i < kAccPerThread; ++i) {
          const int o = tid + i * kThreads;
          if (o < GH * Dv) {
            const int g = o / Dv, dv = o - g * Dv;
            float a = acc[i] * alpha_s[g];
            for (int j = 0; j < n; ++j) {
              const int page = page_s[j], slot = slot_s[j];
              size_t idx;
              if (mla)
                idx = ((size_t)page * ps + slot) * Dk + dv;
              else {
                // V vector/element of a slot: groups of 4x slots, slot 16b+4g+i -> vector g, element 4b+i
                const int w = slot % (4 * x);
                const int u = 4 * (slot / (4 * x)) + (w % 16) / 4, e = 4 * (w / 16) + (w % 4);
                idx = ((((size_t)page * Hkv + h) * (ps / x) + u) * Dv + dv) * x + e;
              }
              a = fmaf(sc[g][j], ld_elem(mla ? kp : vp, idx), a);
            }
            acc[i] = a;
          }
        }
        __syncthreads();
      }
      // write the tile's partial: normalised output and natural-log LSE
      float* dst_o;
      float* dst_l;
      if (tile.dst >= 0) {
        dst_o = p.ws_o + ((size_t)tile.dst * G + g0) * Dv;
        dst_l = p.ws_lse + (size_t)tile.dst * G + g0;
      } else {
        dst_o = p.out_o + ((size_t)tile.shard * p.Hq + a0) * Dv;
        dst_l = p.out_lse + (size_t)tile.lse_shard * p.Hq + a0;
      }
      const bool fin = tile.dst < 0 && p.final_out && tile.final_row >= 0;  // the shard alone is an output row
      if (fin) {
        const size_t fo = ((size_t)tile.final_row * p.Hq + a0) * Dv;
#pragma unroll
        for (int i = 0; i < kAccPerThread; ++i) {
          const int o = tid + i * kThreads;
          if (o < GH * Dv) {
            const float v = acc[i] / l_s[o / Dv];
            const float v1[1] = {v};
            store_final<1>(p.final_out, fo + o, p.final_kind, p.out_inv_scale, v1);
          }
        }
        if (tid < GH) {
          const float lse = m_s[tid] + logf(l_s[tid]);
          dst_l[tid] = lse;
          if (p.final_lse) p.final_lse[(size_t)tile.final_row * p.Hq + a0 + tid] = lse;
        }
      } else {
#pragma unroll
        for (int i = 0; i < kAccPerThread; ++i) {
          const int o = tid + i * kThreads;
          if (o < GH * Dv) dst_o[o] = acc[i] / l_s[o / Dv];
        }
        if (tid < GH) dst_l[tid] = m_s[tid] + logf(l_s[tid]);
      }
    }
    if (p.tile_clock && tid == 0) {
      p.tile_clock[3 * (size_t)ti] = clk0;
      p.tile_clock[3 * (size_t)ti + 1] = wall_clock64();
      p.tile_clock[3 * (size_t)ti + 2] = blockIdx.x;
    }
  }
}

}  // namespace

hipError_t launch_generic(const nanocp_attn_desc& d, const KParams& p, int num_blocks, hipStream_t st) {
  dim3 grid(num_blocks), block(kThreads);
  if (d.kv_dtype == NANOCP_F32)
    hipLaunchKernelGGL((generic_partial_kernel<float, float>), grid, block, 0, st, p);
  else if (d.kv_dtype == NANOCP_BF16)
    hipLaunchKernelGGL((generic_partial_kernel<uint16_t, uint16_t>), grid, block, 0, st, p);
  else
    hipLaunchKernelGGL((generic_partial_kernel<uint16_t, uint8_t>), grid, block, 0, st, p);
  return hipGetLastError();
}

}  // namespace nanocp
