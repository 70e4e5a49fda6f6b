// MFMA tile kernel for MLA-absorbed decode (DeepSeek-V3-like shapes): 128 query heads (or 64, with 4 wavefronts)
// share one latent row of 576 dims per token (512 latent + 64 rope); V is the first 512 dims of the same row, so a
// page is read from HBM once and used for both products.  bf16, page size 64.
// Paper: Data Plane, Phase 2 (partial attention + LSE over the local KV partition); the MoE-bound
// instance's Q row has hidden size 512 (+64) and 128 heads.
//
// One workgroup = 8 wavefronts (two per SIMD) = one chunk of the work queue at a time, one workgroup per CU.
// A page (72 KB) is copied HBM -> LDS by direct-to-LDS 16-byte loads (no registers in between) into one of
// two buffers while the previous page is being computed.  Wavefront w owns query heads 16w..16w+15; its Q
// fragments (72 registers) and its 16 x 512 accumulator (128 registers) stay resident for the whole tile:
//   scores:  S^T[token, head] = K[token, :] . Q[head, :]     A = K rows from LDS (ds_read_b128), B = Q (registers)
//   output:  O^T[dim, head]  += V^T[dim, token] P^T[token, head]   A = V^T via the LDS transpose read
//            (ds_read_b64_tr_b16: 16 lanes fetch a 4-token x 16-dim block, each lane gets 4 tokens of one dim)
// so no wavefront needs another's probabilities or accumulators; the only barriers are the two per page
// that guard the LDS buffers.  P is split into two bf16 terms as in the GQA kernels.
// LDS rows are XOR-swizzled in units of 16 bytes so that both read patterns are bank-conflict free.
#include <hip/hip_runtime.h>

#include <mutex>

#include "epilogue.h"
#include "plan.h"

namespace nanocp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kDk = 576, kDv = 512, kPS = 64;
constexpr int kHB = 1;  // 16-head blocks per wavefront (2 was measured: half the LDS reads, but Q and O no longer fit 256 registers)
// kKD, kVD below: how far the LDS reads run ahead of the matrix instructions that use them (K: units of two
// fragments, V: fragments); bounded by the registers left beside Q and the accumulators: (1, 2) with 256 registers
// per wavefront.  Measured with 512 registers (64-head variant): going deeper than this does not help -- the
// transpose read itself is the limit (about 100 B/clk per CU against 210 for 16-byte reads, measured with a
// stand-alone probe), and it carries 64 KB per wavefront and page.
constexpr int kMla64KD = 2, kMla64VD = 4;
constexpr int kRowBytes = kDk * 2;        // 1152: one token's latent row in HBM
constexpr int kRowA = kDv * 2;            // 1024: dims 0..511 (the V part), LDS region A row
constexpr int kRowB = (kDk - kDv) * 2;    // 128:  dims 512..575 (rope part), LDS region B row
constexpr int kRegionA = kPS * kRowA;     // 65536
constexpr int kBufBytes = kRegionA + kPS * kRowB;  // 73728 per page buffer
constexpr int kSteps = kDk / 32;          // 18 k-steps of 32 dims
constexpr int kStepsA = kDv / 32;         // 16 of them in region A

template <typename T>
using cptr = const __attribute__((address_space(4))) T*;
template <typename T>
__device__ inline cptr<T> as_const(const T* ptr) {
  return (cptr<T>)(uintptr_t)ptr;
}
typedef __attribute__((address_space(3))) char* lds_ptr;

// 64 lanes x 16 bytes from global (scalar base + per-lane offset) straight into LDS at lds_addr + 16*lane
__device__ inline void dma16(uint64_t base, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_addr)
               : "memory");
}
// workgroup barrier without the memory fences of __syncthreads(): copies in flight stay in flight
__device__ inline void wg_barrier() { __builtin_amdgcn_s_barrier(); }

__device__ inline f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ inline uint32_t pack_bf16(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ inline void split8(const float* p, bf16x8& hi, bf16x8& lo) {
  u32x4 h, l;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t hp = pack_bf16(p[2 * i], p[2 * i + 1]);
    const float h0 = __uint_as_float(hp << 16), h1 = __uint_as_float(hp & 0xffff0000u);
    h[i] = hp;
    l[i] = pack_bf16(p[2 * i] - h0, p[2 * i + 1] - h1);
  }
  hi = __builtin_bit_cast(bf16x8, h);
  lo = __builtin_bit_cast(bf16x8, l);
}
// Butterfly over the four 16-lane rows of a wavefront (lanes l, l^16, l^32, l^48 hold the same head) with the
// row-swap instructions of the vector ALU (v_permlane16_swap / v_permlane32_swap) -- no trip through LDS.
// swap16(x, x) = {rows x0 x0 x2 x2, rows x1 x1 x3 x3};  swap32(x, x) = {x0 x1 x0 x1, x2 x3 x2 x3}.
__device__ inline float xor_max(float v) {
  typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
  const uint32_t u = __float_as_uint(v);
  const u32x2_t a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float w = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const uint32_t uw = __float_as_uint(w);
  const u32x2_t b = __builtin_amdgcn_permlane32_swap(uw, uw, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ inline float xor_sum(float v) {
  typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
  const uint32_t u = __float_as_uint(v);
  const u32x2_t a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float w = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const uint32_t uw = __float_as_uint(w);
  const u32x2_t b = __builtin_amdgcn_permlane32_swap(uw, uw, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// kMlaWaves wavefronts of 16 heads each: 8 for 128 query heads (DeepSeek-V3-like), 4 for 64 (Kimi-K2-like)
template <int kMlaWaves, int kKD, int kVD>
__device__ __forceinline__ void mla_mfma_body(const KParams& p) {
  constexpr int kHq = 16 * kHB * kMlaWaves;
  constexpr int kSlabs = 8 / kMlaWaves;  // rope slabs (8 rows each) one wavefront copies
  extern __shared__ __attribute__((aligned(16))) char smem[];  // 2 page buffers
  __shared__ int next_s;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, g = lane >> 4;
  const float c_log2 = p.scale * 1.4426950408889634f;
  const lds_ptr lds = (lds_ptr)smem;

  const cptr<int32_t> chunk_offsets = as_const(p.chunk_offsets);
  const cptr<int32_t> tile_words = as_const((const int32_t*)p.tiles);

  // ---- per-lane constants of the LDS read patterns.  A row's 16-byte chunk c is stored at position
  // c ^ (row & 15) (region A) or c ^ ((row >> 1) & 7) (region B).  For the rows a lane reads, the XOR mask is a
  // per-lane constant, and the compile-time part of c only touches other bits, so a handful of precomputed
  // offsets plus immediates address everything.
  // K fragment (token block tb, k-step s): lane (r, g) reads token 16tb + r, chunk 4s+g:
  //   region A: r*1024 + (((s & 3) << 2) ^ g ^ r) * 16 + [16tb*1024 + (s >> 2)*256]
  //   region B: r*128  + ((((s - 16) << 2) | g) ^ (r >> 1)) * 16 + [16tb*128]
  // V fragment (dim block dvb, tokens 32j + 16hf + 4g + 0..3): lane r supplies token row 4g + (r >> 2) (+32j+16hf),
  //   8 bytes at chunk 2dvb + ((r & 3) >> 1), half (r & 1):
  //   (4g + (r >> 2))*1024 + ((((dvb & 7) << 1) ^ x) * 16) + (r & 1)*8 + [(32j+16hf)*1024 + (dvb >> 3)*256],
  //   x = ((r & 3) >> 1) ^ (4g + (r >> 2))
  // Because a 16-byte shift distributes over XOR, each family of offsets is one per-lane base XOR a small
  // compile-time constant: k = K0 ^ ((s & 3) << 6), kb = KB0 ^ ((s - 16) << 6), v = V0 ^ ((dvb & 7) << 5).
  const uint32_t K0 = (uint32_t)(r * kRowA + ((g ^ r) << 4));
  const uint32_t KB0 = (uint32_t)(kRegionA + r * kRowB + ((g ^ (r >> 1)) << 4));
  uint32_t V0;
  {
    const int vrow = 4 * g + (r >> 2);
    const int x = ((r & 3) >> 1) ^ vrow;
    V0 = (uint32_t)(vrow * kRowA + (x << 4) + (r & 1) * 8);
  }

  // global-side lane offsets of the page copy: token row tok = w + 4j is stored with chunk l ^ (tok & 15) at
  // position l (four masks per wavefront); the rope slabs of rows 8i..8i+7, i = 2w, 2w+1, with chunk
  // (l & 7) ^ ((row >> 1) & 7)
  // (the masks of rows w, w + kMlaWaves, ... differ only in the bits above log2(kMlaWaves): base XOR constant)
  const uint32_t D0 = (uint32_t)((lane ^ wave) << 4);
  uint32_t dma_slab[kSlabs];
#pragma unroll
  for (int a = 0; a < kSlabs; ++a) {
    const int row = 8 * (kSlabs * wave + a) + (lane >> 3);
    dma_slab[a] = (uint32_t)((lane >> 3) * kRowBytes + kRowA + (((lane & 7) ^ ((row >> 1) & 7)) * 16));
  }
  const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

  // plan image: the counts live on the device; an image of another kernel variant, or one with grouped final rows
  // but no final output, is not run
  if (p.header && (as_const(p.header)[4] != p.variant || (as_const(p.header)[5] != 0 && !p.final_out))) return;
  const int num_chunks = p.header ? as_const(p.header)[0] : p.num_chunks;
  for (int chunk = blockIdx.x; chunk < num_chunks;) {
    const int t0 = chunk_offsets[chunk], t1 = chunk_offsets[chunk + 1];
    for (int ti = t0; ti < t1; ++ti) {
      DevTile tile;
      {
        const cptr<int32_t> w = tile_words + (size_t)ti * (sizeof(DevTile) / 4);
        tile.q_row = w[0], tile.bt_row = w[1], tile.kv_head = w[2], tile.shard = w[3];
        tile.tok_begin = w[4], tile.tok_end = w[5], tile.dst = w[6], tile.seg = w[7];
        tile.n_parts = w[8], tile.slot_begin = w[9], tile.final_row = w[10], tile.lse_shard = w[11];
      }
      uint64_t clk0 = 0;
      if (p.tile_clock && tid == 0) clk0 = wall_clock64();
      const cptr<int32_t> bt = as_const(p.block_table + (size_t)tile.bt_row * p.max_blocks);
      const int tb = tile.tok_begin, te = tile.tok_end;
      const int pg0 = tb / kPS, pg1 = (te - 1) / kPS + 1;  // pages [pg0, pg1) of the row

      // direct-to-LDS copy of one page; wavefront w brings token rows w, w+8, ... and one slab of the rope part.
      // Written as inline assembly so that the compiler does not serialise these copies against the LDS reads
      // of the page being computed (it cannot tell the two buffers apart); completion is awaited explicitly.
      auto issue_page = [&](int pg, int buf) {
        const int page = bt[pg];
        const uint64_t src = (uint64_t)(uintptr_t)p.k_pool + (uint64_t)page * (kPS * kRowBytes);
        const uint32_t dst = lds_base + (uint32_t)(buf * kBufBytes);
#pragma unroll
        for (int j = 0; j < kPS / kMlaWaves; ++j) {
          const int tok = wave + kMlaWaves * j;
          dma16(src + (uint64_t)(tok * kRowBytes), D0 ^ (uint32_t)(((kMlaWaves * j) & 15) << 4), dst + (uint32_t)(tok * kRowA));
        }
#pragma unroll
        for (int a = 0; a < kSlabs; ++a)
          dma16(src + (uint64_t)(8 * (kSlabs * wave + a) * kRowBytes), dma_slab[a],
                dst + (uint32_t)(kRegionA + (kSlabs * wave + a) * 1024));
      };

      // Q fragments of this wavefront's heads (B operand): lane (g, n = r) holds Q[16hb + n][dims 8(4s+g) .. +8]
      bf16x8 qf[kHB][kSteps];
#pragma unroll
      for (int hb = 0; hb < kHB; ++hb) {
        const char* qrow = (const char*)p.q + ((size_t)tile.q_row * kHq + 16 * (kHB * wave + hb) + r) * (kDk * 2);
#pragma unroll
        for (int s = 0; s < kSteps; ++s) qf[hb][s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + (4 * s + g) * 16));
      }

      f32x4 acc[kHB][kDv / 16];
#pragma unroll
      for (int hb = 0; hb < kHB; ++hb)
#pragma unroll
        for (int j = 0; j < kDv / 16; ++j) acc[hb][j] = f32x4{0.f, 0.f, 0.f, 0.f};
      float m_run[kHB], l_run[kHB];
#pragma unroll
      for (int hb = 0; hb < kHB; ++hb) m_run[hb] = -INFINITY, l_run[hb] = 0.f;

      issue_page(pg0, 0);
      for (int pg = pg0; pg < pg1; ++pg) {
        const int buf = (pg - pg0) & 1;
        // this page's copy (issued one iteration ago, or before the loop) and, on the first page, Q have landed ...
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        wg_barrier();  // ... in every wavefront
        // start the next page's copy; it overlaps this page's compute (its buffer was released by the barrier
        // that ended the previous iteration)
        if (pg + 1 < pg1) issue_page(pg + 1, buf ^ 1);
        const lds_ptr A = lds + buf * kBufBytes;
        const uint32_t boff = (uint32_t)(buf * kBufBytes);
        const uint32_t KA = K0 + boff, KBA = KB0 + boff, VA = V0 + boff;  // this buffer's lane bases
        const int tok0 = pg * kPS;
        const bool ragged = tok0 < tb || tok0 + kPS > te;  // uniform
        if (ragged) {
          // token slots outside [tb, te) may hold NaN patterns: clear their V part so that 0 * V stays 0
#pragma unroll
          for (int pass = 0; pass < kPS / kMlaWaves; ++pass) {
            const int row = pass * kMlaWaves + wave;
            const int tok = tok0 + row;
            if (tok < tb || tok >= te) *(__attribute__((address_space(3))) u32x4*)(A + row * kRowA + lane * 16) = u32x4{0, 0, 0, 0};
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          wg_barrier();
        }

        // ---- scores S^T[16 tokens x 16 heads] for the 4 token blocks of the page (x kHB head blocks): independent
        // accumulators, so consecutive matrix instructions do not wait for each other
        f32x4 S[4][kHB];
#pragma unroll
        for (int tbk = 0; tbk < 4; ++tbk)
#pragma unroll
          for (int hb = 0; hb < kHB; ++hb) S[tbk][hb] = f32x4{0.f, 0.f, 0.f, 0.f};
        // software pipeline over units u = (k-step s, token-block pair) of 2 fragments and 2*kHB MFMAs: the
        // fragments of unit u+kKD are read while the MFMAs of unit u run; scheduling barriers keep the compiler
        // from hoisting all LDS reads to the top (register blow-up)
        auto load_k = [&](bf16x8* kf, int u) {
          const int s = u >> 1;
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2) {
            const int tbk = 2 * (u & 1) + t2;
            const lds_ptr kp = s < kStepsA ? lds + (KA ^ (uint32_t)((s & 3) << 6)) + (16 * tbk * kRowA + (s >> 2) * 256)
                                           : lds + (KBA ^ (uint32_t)((s - kStepsA) << 6)) + 16 * tbk * kRowB;
            kf[t2] = __builtin_bit_cast(bf16x8, *(__attribute__((address_space(3))) const u32x4*)kp);
          }
        };
        {
          bf16x8 kf[kKD + 1][2];
#pragma unroll
          for (int u = 0; u < kKD; ++u) load_k(kf[u], u);
#pragma unroll
          for (int u = 0; u < 2 * kSteps; ++u) {
            if (u + kKD < 2 * kSteps) load_k(kf[(u + kKD) % (kKD + 1)], u + kKD);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
              for (int hb = 0; hb < kHB; ++hb)
                S[2 * (u & 1) + t2][hb] = mfma16(kf[u % (kKD + 1)][t2], qf[hb][u >> 1], S[2 * (u & 1) + t2][hb]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // ---- online softmax (log2 domain); S[tbk][hb][i] is token tok0 + 16tbk + 4g + i, head 16hb + r
        bf16x8 hi[kHB][2], lo[kHB][2];  // k-blocks j = 0, 1: tokens 32j + 16hf + 4g + i  <->  element 4hf + i
#pragma unroll
        for (int hb = 0; hb < kHB; ++hb) {
          float y[16];
          float mloc = -INFINITY;
#pragma unroll
          for (int tbk = 0; tbk < 4; ++tbk)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              float v = S[tbk][hb][i] * c_log2;
              if (ragged) {
                const int tok = tok0 + 16 * tbk + 4 * g + i;
                v = (tok >= tb && tok < te) ? v : -INFINITY;
              }
              y[tbk * 4 + i] = v;
              mloc = fmaxf(mloc, v);
            }
          mloc = xor_max(mloc);
          const float m_new = fmaxf(m_run[hb], mloc);  // finite: every page of the tile holds a token of its range
          if (__any(m_new > m_run[hb])) {
            const float alpha = __builtin_amdgcn_exp2f(m_run[hb] - m_new);
            l_run[hb] *= alpha;
            // the accumulators live in accumulation registers the vector ALU cannot address: rescale them a few
            // at a time so that the round trip needs only a few temporaries
#pragma unroll
            for (int j = 0; j < kDv / 16; ++j) {
              acc[hb][j] *= alpha;
              if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);
            }
            m_run[hb] = m_new;
          }
          float psum = 0.f;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            y[e] = __builtin_amdgcn_exp2f(y[e] - m_run[hb]);
            psum += y[e];
          }
          l_run[hb] += psum;
          split8(y, hi[hb][0], lo[hb][0]);
          split8(y + 8, hi[hb][1], lo[hb][1]);
        }

        // ---- O^T += V^T P^T over units u = (dim block dvb, token half j): one fragment (two transpose reads) feeds
        // 2*kHB MFMAs (hi and lo term of P); kVD fragments are kept in flight
        auto load_v = [&](int u) {
          const int dvb = u >> 1, j = u & 1;
          u32x4 vf;
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            const lds_ptr ap = lds + (VA ^ (uint32_t)((dvb & 7) << 5)) + ((32 * j + 16 * hf) * kRowA + (dvb >> 3) * 256);
            const s16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)ap);
            const u32x2 t2 = __builtin_bit_cast(u32x2, t);
            vf[2 * hf] = t2[0];
            vf[2 * hf + 1] = t2[1];
          }
          return __builtin_bit_cast(bf16x8, vf);
        };
        {
          constexpr int kUnits = 2 * (kDv / 16);
          bf16x8 vfr[kVD + 1];
#pragma unroll
          for (int u = 0; u < kVD; ++u) vfr[u] = load_v(u);
#pragma unroll
          for (int u = 0; u < kUnits; ++u) {
            if (u + kVD < kUnits) vfr[(u + kVD) % (kVD + 1)] = load_v(u + kVD);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int hb = 0; hb < kHB; ++hb) acc[hb][u >> 1] = mfma16(vfr[u % (kVD + 1)], hi[hb][u & 1], acc[hb][u >> 1]);
#pragma unroll
            for (int hb = 0; hb < kHB; ++hb) acc[hb][u >> 1] = mfma16(vfr[u % (kVD + 1)], lo[hb][u & 1], acc[hb][u >> 1]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wg_barrier();  // the buffer may be overwritten by the copy issued at the top of the next iteration
      }

      // ---- write this wavefront's heads: normalised output rows and natural-log LSE
      float* dst_o;
      float* dst_l;
      if (tile.dst >= 0) {
        dst_o = p.ws_o + (size_t)tile.dst * kHq * kDv;
        dst_l = p.ws_lse + (size_t)tile.dst * kHq;
      } else {
        dst_o = p.out_o + (size_t)tile.shard * kHq * kDv;
        dst_l = p.out_lse + (size_t)tile.lse_shard * kHq;
      }
      const bool fin = tile.dst < 0 && p.final_out && tile.final_row >= 0;  // the shard alone is an output row
#pragma unroll
      for (int hb = 0; hb < kHB; ++hb) {
        const float l = xor_sum(l_run[hb]);
        const float inv = 1.f / l;
        const int head = 16 * (kHB * wave + hb) + r;
        const float lse = (m_run[hb] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
        if (g == 0) dst_l[head] = lse;
        if (fin) {
          // acc[hb][dvb][i] = dim 16dvb + 4g + i of that head
          const size_t fo = ((size_t)tile.final_row * kHq + head) * kDv + 4 * g;
#pragma unroll
          for (int dvb = 0; dvb < kDv / 16; ++dvb) {
            const f32x4 v = acc[hb][dvb] * inv;
            const float v4[4] = {v[0], v[1], v[2], v[3]};
            store_final<4>(p.final_out, fo + 16 * dvb, p.final_kind, p.out_inv_scale, v4);
            if ((dvb & 3) == 3) __builtin_amdgcn_sched_barrier(0);
          }
          if (g == 0 && p.final_lse) p.final_lse[(size_t)tile.final_row * kHq + head] = lse;
        } else {
          float* orow = dst_o + (size_t)head * kDv + 4 * g;  // acc[hb][dvb][i] = dim 16dvb + 4g + i of that head
#pragma unroll
          for (int dvb = 0; dvb < kDv / 16; ++dvb) {
            *(f32x4*)(orow + 16 * dvb) = acc[hb][dvb] * inv;
            if ((dvb & 3) == 3) __builtin_amdgcn_sched_barrier(0);
          }
        }
      }

      if (p.tile_clock && tid == 0) {
        p.tile_clock[3 * (size_t)ti] = clk0;
        p.tile_clock[3 * (size_t)ti + 1] = wall_clock64();
        p.tile_clock[3 * (size_t)ti + 2] = blockIdx.x;
      }
    }
    if (tid == 0) next_s = (int)gridDim.x + atomicAdd(&p.sync[0], 1);
    __syncthreads();
    chunk = __builtin_amdgcn_readfirstlane(next_s);
    __syncthreads();
  }
  if (tid == 0) {
    const int done = atomicAdd(&p.sync[1], 1);
    if (done == (int)gridDim.x - 1) {
      p.sync[0] = 0;
      p.sync[1] = 0;
    }
  }
}

// 128 heads: two wavefronts per SIMD, 256 registers each
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void mla_mfma_kernel(KParams p) {
  mla_mfma_body<8, 1, 2>(p);
}
// 64 heads: one wavefront per SIMD, 512 registers: the LDS reads run far ahead
__global__ __launch_bounds__(256, 1) void mla64_mfma_kernel(KParams p) {
  mla_mfma_body<4, kMla64KD, kMla64VD>(p);
}

// The dynamic-LDS limit is an attribute of the kernel on ONE device: it is raised once per device and kernel, with
// that device current, the first time the kernel is launched there.
template <typename K>
hipError_t allow_big_lds(K kernel, int bytes, int slot) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static bool done[2][kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!done[slot][dev]) {
    e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    done[slot][dev] = true;
  }
  return hipSuccess;
}

}  // namespace

hipError_t launch_mla_mfma(const KParams& p, int num_blocks, hipStream_t st) {
  if (p.Hq == 128) {
    const hipError_t attr = allow_big_lds(mla_mfma_kernel, 2 * kBufBytes, 0);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(mla_mfma_kernel, dim3(num_blocks), dim3(512), 2 * kBufBytes, st, p);
  } else if (p.Hq == 64) {
    const hipError_t attr = allow_big_lds(mla64_mfma_kernel, 2 * kBufBytes, 1);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(mla64_mfma_kernel, dim3(num_blocks), dim3(256), 2 * kBufBytes, st, p);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace nanocp
