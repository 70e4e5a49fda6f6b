// MFMA tile kernels for MLA-absorbed decode (DeepSeek-V3-like shapes): 128 query heads (or 64) share one latent
// row of 576 dims per token (512 latent + 64 rope); V is the first 512 dims of the same row, so a page is read from
// HBM once and used for both products.  bf16, page size 64.
// Paper: Data Plane, Phase 2 (partial attention + LSE over the local KV partition); the MoE-bound
// instance's Q row has hidden size 512 (+64) and 128 heads.
//
// One workgroup = 8 wavefronts (two per SIMD) = one chunk of the work queue at a time, one workgroup per CU.  A page
// (72 KB) sits in LDS while it is computed on, the next one arrives meanwhile (who copies it: see mla_mfma_body).  The
// two products are split over the computing wavefronts (all 8 with 128 heads, 4 with 64) in different ways:
//   scores (split by heads):  wavefront w owns query heads 16w..16w+15, its Q fragments stay in registers
//       S^T[token, head] = K[token, :] . Q[head, :]          A = K rows from LDS (ds_read_b128), B = Q
//     one 16-token block at a time, each followed at once by the softmax of its scores; the page's probabilities go
//     to LDS as fp16 B-operand fragments.
//   output (split by V dims): wavefront w owns a slice of the 512 dims of ALL heads (accumulator 128 registers)
//       O^T[dim, head] += V^T[dim, token] P^T[token, head]   A = V^T via the LDS transpose read
//       (ds_read_b64_tr_b16: 16 lanes fetch a 4-token x 16-dim block, each lane gets 4 tokens of one dim), B = P
//     so every V^T fragment is fetched from LDS once per page (not once per wavefront) and feeds one matrix
//     instruction per head block; the only data all wavefronts read are the probabilities (16 KB per page).
// Precision of P.  One fp16 term (11 significant bits) instead of the two bf16 terms of the GQA kernels: the P.V
// product is then half the matrix instructions.  Two things make that sufficient:
//   * the softmax reference is an INTEGER exponent m (a ceiling of log2-domain scores that may lag the running
//     maximum, see kHeadroom), and p = 2^frac(y) * 2^(floor(y) - m): the significand of p does not depend on m,
//     every rescale is an exact power of two, so a token's rounded probability is the same number (up to that power
//     of two) whatever tile or shard it is processed in -- a request's merged partials and its unsharded result
//     differ only by fp32 summation order;
//   * V (bf16, 8 significant bits) is widened to fp16 exactly (in registers, by the wavefront that owns the dims).
//     fp16's range applies: |V| above 65504 saturates, |V| below 6e-8 flushes to zero.  P is scaled by a power of
//     two so that probabilities down to 2^-20 of the reference stay normal fp16 numbers.
// LDS rows are XOR-swizzled in units of 16 bytes so that both read patterns are bank-conflict free.
// The tiles of one (shard, head-set) that was cut are combined by mla_reduce_kernel below, launched right after the
// tile kernel (it also writes the rows of shards without tokens).
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

#include "epilogue.h"
#include "plan.h"

namespace nanocp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kDk = 576, kDv = 512, kPS = 64;
constexpr int kRowBytes = kDk * 2;        // 1152: one token's latent row in HBM
constexpr int kRowA = kDv * 2;            // 1024: dims 0..511 (the V part), LDS region A row
constexpr int kRowB = (kDk - kDv) * 2;    // 128:  dims 512..575 (rope part), LDS region B row
constexpr int kRegionA = kPS * kRowA;     // 65536 per page buffer
constexpr int kSteps = kDk / 32;          // 18 k-steps of 32 dims
constexpr int kStepsA = kDv / 32;         // 16 of them in region A
// Probabilities are handed to the matrix cores as 2^(y - m_ref) * 2^kPShift, where m_ref is a per-head integer
// REFERENCE exponent that is allowed to lag the running maximum by up to kHeadroom: it moves (and the accumulators
// are rescaled, by an exact power of two) only when a score exceeds it by more than that -- after a tile's first page
// almost never, whereas the running maximum of 128 heads moves on nearly every page.  Largest value fed to the
// matrix cores: 2^(kHeadroom + kPShift) = 2^14 (fp16 holds up to 2^16); values stay normal fp16 numbers down to
// 2^-20 of the reference (2^-28 of the largest possible maximum).
constexpr int kHeadroom = 8;
constexpr int kPShift = 6;
constexpr float kMaskedScore = -1073741824.f;  // -2^30: score of a token slot outside the tile's range

// LDS map: two buffers for the V part of a page (double-buffered: the copy of page n+1 runs under the compute of
// page n), ONE for the rope part (only the score product reads it; it is refilled as soon as that product is done),
// the probabilities of one page, and the small per-head exchange arrays.
constexpr int kOffRope = 2 * kRegionA;                  // 131072, 8 KB
constexpr int kOffP = kOffRope + kPS * kRowB;           // 139264, up to 16 KB: [head block][token half][lane] x 16 B
constexpr int kOffAlpha = kOffP + 8 * 2 * 1024;         // [16 r][8 hb] floats: this page's accumulator rescale factors
constexpr int kOffM = kOffAlpha + 512;                  // [128] per-head running maximum (tile end)
constexpr int kOffL = kOffM + 512;                      // [128] per-head sum of probabilities (tile end)
constexpr int kOffMoved = kOffL + 512;                  // [2] per page parity: some head's reference moved on that page
constexpr int kOffNext = kOffMoved + 8;                 // next work-queue entry, broadcast to the workgroup
constexpr int kLdsBytes = kOffMoved + 16;               // 157200

template <typename T>
using cptr = const __attribute__((address_space(4))) T*;
template <typename T>
__device__ inline cptr<T> as_const(const T* ptr) {
  return (cptr<T>)(uintptr_t)ptr;
}
typedef __attribute__((address_space(3))) char* lds_ptr;
#define LDS_AS(T, ptr) ((__attribute__((address_space(3))) T*)(ptr))

// 64 lanes x 16 bytes from global (scalar base + per-lane offset) straight into LDS at lds_addr + 16*lane
__device__ inline void dma16(uint64_t base, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_addr)
               : "memory");
}
// workgroup barrier without the memory fences of __syncthreads(): copies in flight stay in flight
__device__ inline void wg_barrier() { __builtin_amdgcn_s_barrier(); }

__device__ inline f32x4 mfma_bf16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ inline f32x4 mfma_f16(f16x8 a, f16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
// two bf16 (one dword) -> two fp16 (one dword), exact inside fp16's range (the conversion rounds toward zero, which
// only matters outside it: too large saturates to 65504, too small flushes toward zero)
__device__ inline uint32_t bf16x2_to_f16x2(uint32_t w) {
  const float lo = __uint_as_float(w << 16), hi = __uint_as_float(w & 0xffff0000u);
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
__device__ inline uint32_t pack_f16(float a, float b) {
  f16x2 v = {(_Float16)a, (_Float16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}
// Butterfly over the four 16-lane rows of a wavefront (lanes l, l^16, l^32, l^48 hold the same head) with the
// row-swap instructions of the vector ALU (v_permlane16_swap / v_permlane32_swap) -- no trip through LDS.
// (the maxima are written as instructions: fmaxf() on values that come out of a bit cast first spends an
// instruction per operand on quieting NaNs)
__device__ inline float max_raw(uint32_t a, uint32_t b) {
  float o;
  asm("v_max_f32 %0, %1, %2" : "=v"(o) : "v"(a), "v"(b));
  return o;
}
__device__ inline float xor_max(float v) {
  const uint32_t u = __float_as_uint(v);
  const u32x2 a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const uint32_t uw = __float_as_uint(max_raw(a[0], a[1]));
  const u32x2 b = __builtin_amdgcn_permlane32_swap(uw, uw, false, false);
  return max_raw(b[0], b[1]);
}
__device__ inline float xor_sum(float v) {
  const uint32_t u = __float_as_uint(v);
  const u32x2 a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float w = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const uint32_t uw = __float_as_uint(w);
  const u32x2 b = __builtin_amdgcn_permlane32_swap(uw, uw, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
// W computing wavefronts: 8 for 128 query heads (DeepSeek-V3-like), 4 for 64 (Kimi-K2-like); the workgroup always has
// 8 wavefronts.  Who issues the page copies matters: the memory pipeline takes a one-kilobyte direct-to-LDS copy only
// every hundred-odd cycles, a wavefront that issues the next one earlier sits blocked at the issue, and everything
// behind it in program order -- its matrix instructions -- waits too (measured: 16 copies in front of a 72-instruction
// score product tripled its duration).  So the copies belong to wavefronts that can afford to block:
//   64 heads:  wavefronts 4..7 do nothing else (they need no registers to speak of and spend their time blocked or
//              at the barriers); the four computing wavefronts never touch global memory inside the page loop;
//   128 heads: all 8 wavefronts compute, two per SIMD, and the hardware favours the older one of a pair, which then
//              waits at each barrier for the younger one.  Wavefronts 0..3 (the older ones) issue all copies, one
//              between every two units of their score product: their blocked time comes out of that slack and leaves
//              the SIMD to the younger wavefront.
// kRing: K fragments in registers; the LDS reads run kRing - 1 matrix instructions ahead.
template <int W, int kRing, int kOut>
__device__ __forceinline__ void mla_mfma_body(const KParams& p) {
  constexpr int kHq = 16 * W;        // query heads = head blocks of 16 x W
  constexpr int kDW = 32 / W;        // 16-dim blocks of V one wavefront owns (4 or 8)
  constexpr int kND = 4;             // copying wavefronts; each brings kPS / kND token rows and 8 / kND rope slabs
  extern __shared__ __attribute__((aligned(16))) char smem[];  // the only LDS object: its offset is 0, so LDS
                                                               // addresses are plain lane offsets plus immediates

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 15, g = lane >> 4;
  const float c_log2 = p.scale * 1.4426950408889634f;
  const lds_ptr lds = (lds_ptr)smem;
  const bool computes = W == 8 || wave < W;          // wavefront-uniform
  const bool copies = W == 8 ? wave < kND : wave >= W;
  const int cw = W == 8 ? wave : wave - W;           // index among the copying wavefronts (if `copies`)

  const cptr<int32_t> chunk_offsets = as_const(p.chunk_offsets);
  const cptr<int32_t> tile_words = as_const((const int32_t*)p.tiles);

  // ---- per-lane constants of the LDS read patterns.  A row's 16-byte chunk c is stored at position
  // c ^ (row & 15) (region A) or c ^ ((row >> 1) & 7) (rope region).  For the rows a lane reads, the XOR mask is a
  // per-lane constant, and the compile-time part of c only touches other bits, so a handful of precomputed
  // offsets plus immediates address everything.
  // K fragment (token block tb, k-step s): lane (r, g) reads token 16tb + r, chunk 4s+g:
  //   region A: r*1024 + (((s & 3) << 2) ^ g ^ r) * 16 + [16tb*1024 + (s >> 2)*256]
  //   rope:     r*128  + ((((s - 16) << 2) | g) ^ (r >> 1)) * 16 + [16tb*128]
  // V fragment (dim block dvb, tokens 32j + 16hf + 4g + 0..3): lane r supplies token row 4g + (r >> 2) (+32j+16hf),
  //   8 bytes at chunk 2dvb + ((r & 3) >> 1), half (r & 1):
  //   (4g + (r >> 2))*1024 + ((((dvb & 7) << 1) ^ x) * 16) + (r & 1)*8 + [(32j+16hf)*1024 + (dvb >> 3)*256],
  //   x = ((r & 3) >> 1) ^ (4g + (r >> 2))
  // Because a 16-byte shift distributes over XOR, each family of offsets is one per-lane base XOR a small
  // compile-time constant: k = K0 ^ ((s & 3) << 6), kb = KB0 ^ ((s - 16) << 6), v = V0 ^ ((dvb & 7) << 5).
  // The lane-dependent offsets below are recomputed from the lane id once per page (a dozen integer instructions
  // against thousands of cycles of page time) instead of being kept in registers across the whole tile loop: with
  // Q (72) and the accumulators (128) resident, the registers they would occupy are the ones that decide
  // between no spills and spills in the page loop.  fresh() hands the lane id through an empty asm statement so
  // that the compiler does not hoist the computations back out of the loop.
  auto fresh = [&]() {
    int l = lane;
    asm volatile("" : "+v"(l));
    return l;
  };
  const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
  // a zero the compiler cannot trace back to a constant it already holds somewhere (which here would be a register
  // that lives, spilled, across the whole tile loop)
  auto fresh_zero = [] {
    uint32_t z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
  };

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
      const uint64_t clk0 = wall_clock64();  // (unconditional: a scalar read; the condition would cost a register)
      const cptr<int32_t> bt = as_const(p.block_table + (size_t)tile.bt_row * p.max_blocks);
      const int tb = tile.tok_begin, te = tile.tok_end;
      const int pg0 = tb / kPS, pg1 = (te - 1) / kPS + 1;  // pages [pg0, pg1) of the row

      // direct-to-LDS copies of one page; copying wavefront c brings token rows c, c + kND, ... of the V part and
      // 8 / kND slabs (8 rows each) of the rope part.  Written as inline assembly so that the compiler does not
      // serialise these copies against the LDS reads of the page being computed; completion is awaited explicitly.
      // Global-side lane offsets: token row tok is stored with chunk l ^ (tok & 15) at position l; the rope slab of
      // rows 8i..8i+7 with chunk (l & 7) ^ ((row >> 1) & 7).  The lane offset is recomputed per copy (two
      // instructions) rather than held in a register.
      auto page_src = [&](int pg) { return (uint64_t)(uintptr_t)p.k_pool + (uint64_t)bt[pg] * (kPS * kRowBytes); };
      auto issue_a_row = [&](uint64_t src, int buf, int j) {
        const int tok = cw + kND * j;
        dma16(src + (uint64_t)(tok * kRowBytes), (uint32_t)((fresh() ^ (tok & 15)) << 4),
              lds_base + (uint32_t)(buf * kRegionA) + (uint32_t)(tok * kRowA));
      };
      auto issue_page_a = [&](int pg, int buf) {  // all rows of this wavefront in one burst
        const uint64_t src = page_src(pg);
#pragma unroll
        for (int j = 0; j < kPS / kND; ++j) issue_a_row(src, buf, j);
      };
      auto issue_page_rope = [&](int pg) {
        const uint64_t src = page_src(pg);
        const int l = fresh();
#pragma unroll
        for (int a = 0; a < 8 / kND; ++a) {
          const int slab = (8 / kND) * cw + a;
          const int row = 8 * slab + (l >> 3);
          const uint32_t off = (uint32_t)((l >> 3) * kRowBytes + kRowA + (((l & 7) ^ ((row >> 1) & 7)) * 16));
          dma16(src + (uint64_t)(8 * slab * kRowBytes), off, lds_base + (uint32_t)(kOffRope + slab * 1024));
        }
      };

      if (!computes) {
        // A copying-only wavefront (64-head kernel): the same barriers as the computing ones.  It has registers to
        // spare, so its share of a page (16 rows of the V part, 2 rope slabs: 18 KB) travels through registers --
        // ordinary 16-byte global loads, then ds_write_b128 -- instead of direct-to-LDS copies: that path tops out
        // near 6 TB/s over the whole chip (measured with nothing else running), below what this kernel can consume,
        // and a page staged in registers can be requested a whole page earlier than its LDS buffer becomes free.
        const int l = fresh();
        u32x4 va[kPS / kND], vr[8 / kND];
        // (global address space stated explicitly: through a generic pointer these would be FLAT loads, which count on
        // the LDS counter as well)  Same placement as the direct copies: position l of row tok holds chunk l ^ (tok & 15).
        typedef const __attribute__((address_space(1))) char* gchar;
        typedef const __attribute__((address_space(1))) u32x4* gvec;
        auto fetch_rows = [&](int pg) {
          const gchar src = (gchar)(uintptr_t)page_src(pg);
#pragma unroll
          for (int j = 0; j < kPS / kND; ++j) {
            const int tok = cw + kND * j;
            va[j] = __builtin_nontemporal_load((gvec)(src + (uint32_t)(tok * kRowBytes + ((l ^ (tok & 15)) << 4))));
          }
        };
        auto fetch_rope = [&](int pg) {
          const gchar src = (gchar)(uintptr_t)page_src(pg);
#pragma unroll
          for (int a = 0; a < 8 / kND; ++a) {
            const int slab = (8 / kND) * cw + a;
            const int row = 8 * slab + (l >> 3);
            vr[a] = __builtin_nontemporal_load(
                (gvec)(src + (uint32_t)(row * kRowBytes + kRowA + (((l & 7) ^ ((row >> 1) & 7)) << 4))));
          }
        };
        auto store_a = [&](int buf) {
#pragma unroll
          for (int j = 0; j < kPS / kND; ++j)
            *LDS_AS(u32x4, lds + buf * kRegionA + (cw + kND * j) * kRowA + l * 16) = va[j];
        };
        auto store_rope = [&]() {
#pragma unroll
          for (int a = 0; a < 8 / kND; ++a) *LDS_AS(u32x4, lds + kOffRope + ((8 / kND) * cw + a) * 1024 + l * 16) = vr[a];
        };
        fetch_rows(pg0);
        fetch_rope(pg0);
        store_a(0);
        store_rope();
        if (pg0 + 1 < pg1) {  // in flight while the computing wavefronts work on the first page
          fetch_rows(pg0 + 1);
          fetch_rope(pg0 + 1);
        }
        for (int pg = pg0; pg < pg1; ++pg) {
          const int tok0 = pg * kPS;
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wavefront's share of page pg is in LDS
          wg_barrier();                                        // top of the page
          if (tok0 < tb || tok0 + kPS > te) wg_barrier();      // ragged page: after the clearing of unused rows
          // The rows of page pg + 1 go to LDS (that buffer was last read by the P.V of page pg - 1) and the rows of
          // page pg + 2 are requested at once: they have a whole page time to arrive.
          if (pg + 1 < pg1) store_a(((pg - pg0) & 1) ^ 1);
          if (pg + 2 < pg1) fetch_rows(pg + 2);
          asm volatile("" ::: "memory");  // (keeps the loads here: the compiler otherwise sinks them towards their use)
          wg_barrier();                                        // probabilities written; the rope buffer is free
          if (pg + 1 < pg1) store_rope();
          if (pg + 2 < pg1) fetch_rope(pg + 2);
          asm volatile("" ::: "memory");
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wg_barrier();  // the two barriers of the tile epilogue
        wg_barrier();
        continue;
      }

      // Q fragments of this wavefront's heads (B operand): lane (g, n = r) holds Q[16w + n][dims 8(4s+g) .. +8]
      bf16x8 qf[kSteps];
      {
        // uniform base + 32-bit lane offset from a re-read lane id (see the note on output addresses below)
        const char* qrows = (const char*)p.q + ((size_t)tile.q_row * kHq + 16 * wave) * (kDk * 2);
        const int lq0 = fresh();
        const uint32_t qoff = (uint32_t)((lq0 & 15) * (kDk * 2) + (lq0 >> 4) * 16);
#pragma unroll
        for (int s = 0; s < kSteps; ++s) qf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrows + (qoff + (uint32_t)(64 * s))));
      }

      // accumulator of this wavefront's dims (16-dim blocks kDW*w .. kDW*w + kDW - 1) for all head blocks:
      // acc[dl][hb][i] = O^T[dim 16(kDW*w + dl) + 4g + i][head 16hb + r], scaled by 2^kPShift and not yet normalised
      f32x4 acc[kDW][W];
#pragma unroll
      for (int dl = 0; dl < kDW; ++dl)
#pragma unroll
        for (int hb = 0; hb < W; ++hb) acc[dl][hb] = f32x4{0.f, 0.f, 0.f, 0.f};
      float m_run = -INFINITY;  // integer-valued reference exponent (log2 domain) of head 16w + r, see kHeadroom
      float l_run = 0.f;        // this lane's share of the running sum of probabilities (times 2^kPShift)
      // derived from m_run whenever it moves: which form of the exponential applies (wavefront-uniform), the integer
      // kPShift - m_run and the factor 2^(kPShift - m_run)
      bool p_plain = true;
      int p_off = 0;
      float p_unit = 0.f;

      // Q must count as arrived BEFORE the page loop: the compiler tracks its own global loads with the same counter
      // the page copies use, and would otherwise wait inside the loop -- at each Q fragment's first use -- for "all
      // but n outstanding loads", which there means: for the next page's copy.  Naming every fragment as an asm
      // operand makes it place those waits here.
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        u32x4 t = __builtin_bit_cast(u32x4, qf[s]);
        asm volatile("" : "+v"(t));
        qf[s] = __builtin_bit_cast(bf16x8, t);
      }
      if (copies) {  // 128 heads: wavefronts 0..3
        issue_page_a(pg0, 0);
        issue_page_rope(pg0);
      }
      for (int pg = pg0; pg < pg1; ++pg) {
        const int buf = (pg - pg0) & 1;
        // this page's copies (V part issued one iteration ago, rope part half an iteration ago, or both before the
        // loop) and, on the first page, Q have landed ...
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        wg_barrier();  // ... in every wavefront; and every wavefront is done with the previous page
        const bool more = pg + 1 < pg1;  // the next page is copied under this page's compute
        const uint32_t boff = (uint32_t)(buf * kRegionA);
        const int tok0 = pg * kPS;
        const bool ragged = tok0 < tb || tok0 + kPS > te;  // uniform over the workgroup
        // re-arm the other parity's "a reference moved" flag (last read during the previous page's P.V).  The flag is
        // a shortcut only: set means "read the rescale factors", and they are written on every page.
        if (wave == 0 && fresh() == 0) *LDS_AS(uint32_t, lds + kOffMoved + (buf ^ 1) * 4) = fresh_zero();
        // this page's lane bases (see the comment on the read patterns above)
        const int lq = fresh();
        const int rq = lq & 15, gq = lq >> 4;
        const uint32_t KA = (uint32_t)(rq * kRowA + ((gq ^ rq) << 4)) + boff;
        const uint32_t KBA = (uint32_t)(kOffRope + rq * kRowB + ((gq ^ (rq >> 1)) << 4));
        const uint32_t PA = (uint32_t)(kOffP + lq * 16);  // probabilities: fragment (hb, j) of lane l at +((hb*2+j)*64)*16
        if (ragged) {
          // token slots outside [tb, te) may hold NaN patterns: clear their V part so that 0 * V stays 0
          const uint32_t z = fresh_zero();  // materialised here, not kept (and spilled) across the tile loop
          const u32x4 zero = {z, z, z, z};
#pragma unroll
          for (int pass = 0; pass < kPS / W; ++pass) {
            const int row = pass * W + wave;
            const int tok = tok0 + row;
            if (tok < tb || tok >= te) *LDS_AS(u32x4, lds + boff + row * kRowA + lane * 16) = zero;
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          wg_barrier();
        }

        // ---- scores and probabilities, one 16-token block at a time: S^T[16 tokens x 16 heads] = K . Q (18 matrix
        // instructions on one accumulator), then at once the softmax of those 4 scores per lane, while the LDS reads of
        // the next block are in flight.  The wavefront's instruction stream alternates between bursts of matrix and of
        // vector instructions; the two wavefronts of a SIMD fall into opposite phases by themselves (whoever loses
        // the matrix pipe is the one with vector work to do), and bursts from different wavefronts DO run
        // concurrently (measured: 2 x {18 matrix, 30 vector} per SIMD take the time of the 36 matrix instructions
        // alone), whereas a separate softmax phase for the whole page leaves the matrix pipes idle for its duration.
        // This order is possible because the reference m_ref of a head is allowed to lag its running maximum (see
        // kHeadroom): the scores of a block are turned into probabilities against the CURRENT reference, and only
        // when one of them exceeds it by more than the headroom does the slow path below run, which also rescales
        // what this page has produced so far.
        uint32_t kb[6];  // the six XOR-ed lane bases of the page (the rest of a fragment's address is an immediate)
#pragma unroll
        for (int x = 0; x < 4; ++x) kb[x] = KA ^ (uint32_t)(x << 6);
        kb[4] = KBA;
        kb[5] = KBA ^ 64u;
        auto load_kf = [&](int i) {  // fragment i = 18 * token block + k-step
          const int tbk = i / kSteps, ks = i % kSteps;
          const lds_ptr kp = ks < kStepsA ? lds + kb[ks & 3] + (16 * tbk * kRowA + (ks >> 2) * 256)
                                          : lds + kb[4 + (ks - kStepsA)] + 16 * tbk * kRowB;
          return __builtin_bit_cast(bf16x8, *LDS_AS(const u32x4, kp));
        };
        u32x4 frag[2] = {u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}};  // the page's probabilities as fp16 B-operand fragments:
                                                                // token half j holds tokens 32j + 16hf + 4g + i as element 4hf + i
        float alpha_page = 1.f;  // rescale factor of everything accumulated before this page (a power of two)

        auto softmax_block = [&](int tbk, f32x4 Sb) {
          if (ragged) {
            // Masked token slots score -2^30 (not -inf: the general form below converts the integer part of a score
            // to an int): exp2 of it is exactly 0.  (Scores are assumed to lie within +-2^30 in the log2 domain.)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int tok = tok0 + 16 * tbk + 4 * g + i;
              Sb[i] = (tok >= tb && tok < te) ? Sb[i] : kMaskedScore;
            }
            asm volatile("" ::: "memory");  // keeps this a branch taken on ragged pages only, not selects on every page
          }
          const float mx = fmaxf(fmaxf(Sb[0], Sb[1]), fmaxf(Sb[2], Sb[3]));  // raw scores: the softmax scale is positive
          if (__any(mx * c_log2 > m_run + (float)kHeadroom)) {
            // Slow path (a tile's first block; afterwards only when a score beats everything seen so far by a factor
            // of 2^8): the reference of such a head moves to the ceiling of the block's maximum.
            const float mb = xor_max(mx);            // over the 4 lane groups: all 16 tokens of the block, head r
            const bool real = mb > -5.0e8f;           // the block holds a token of this tile's range
            const float m_blk = __builtin_ceilf(mb * c_log2);
            const float m_new = (real && m_blk > m_run + (float)kHeadroom) ? m_blk : m_run;
            // 2^(m_run - m_new), exact; 0 while nothing has been accumulated (m_run = -inf)
            const int down = (int)fmaxf(m_run - m_new, -200.f);  // <= 0
            const float alpha = __builtin_amdgcn_ldexpf(1.f, down);
            m_run = m_new;
            l_run *= alpha;
            alpha_page *= alpha;
            // What this page has produced so far was scaled by the old reference: multiply the fp16 pairs by 2^down,
            // as up to three packed fp16 factors of at least 2^-14 each (a single fp16 factor would underflow
            // where the product does not; beyond 2^-42 every product is 0 anyway).
            if (__any(down != 0)) {
              int e = down;
#pragma unroll
              for (int round = 0; round < 3; ++round) {
                const int step = e > -14 ? e : -14;
                e -= step;
                const uint32_t bits = (uint32_t)(step + 15) << 10;  // fp16 2^step
                const f16x2 f = __builtin_bit_cast(f16x2, bits | (bits << 16));
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                  for (int q = 0; q < 4; ++q) {
                    const uint32_t w = frag[j][q];  // (a bit cast applied to the vector element itself reads element 0)
                    frag[j][q] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, w) * f);
                  }
              }
            }
            // p * 2^kPShift = 2^frac(y) * 2^(floor(y) - m + kPShift): the significand depends on the score alone.
            // While every reference of this wavefront lies in [-100, 118] (any sane input) that is exp2(y) * 2^(kPShift
            // - m) with the hardware's exp2 over its normal range: three instructions per score instead of six;
            // scores below -126 then give 0 instead of at most 2^-20 of the reference.  A head that has seen no token
            // yet (m = -inf) takes that form with factor 0.
            const bool none = !(m_run > -INFINITY);
            p_plain = __all(none || (m_run >= -100.f && m_run <= 118.f));
            p_off = none ? 0 : kPShift - (int)m_run;
            p_unit = none ? 0.f : __builtin_amdgcn_ldexpf(1.f, p_off);
          }
          float pw[4];
          if (p_plain) {
#pragma unroll
            for (int i = 0; i < 4; ++i) pw[i] = __builtin_amdgcn_exp2f(Sb[i] * c_log2) * p_unit;
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float yv = Sb[i] * c_log2;
              const float ex = __builtin_amdgcn_exp2f(__builtin_amdgcn_fractf(yv));
              int fl;
              asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(fl) : "v"(yv));  // floor(y) as an integer, one instruction
              pw[i] = (m_run > -INFINITY) ? __builtin_amdgcn_ldexpf(ex, fl + p_off) : 0.f;
            }
          }
          frag[tbk >> 1][2 * (tbk & 1)] = pack_f16(pw[0], pw[1]);
          frag[tbk >> 1][2 * (tbk & 1) + 1] = pack_f16(pw[2], pw[3]);
          l_run += (pw[0] + pw[1]) + (pw[2] + pw[3]);  // sum of p * 2^kPShift before the fp16 rounding
        };

        auto score_product = [&](auto with_copies) {
          [[maybe_unused]] uint64_t next_src = 0;
          if constexpr (with_copies.value) next_src = page_src(pg + 1);
          constexpr int kFrags = 4 * kSteps;  // 72 K fragments per wavefront and page
          bf16x8 ring[kRing];
#pragma unroll
          for (int i = 0; i < kRing - 1; ++i) ring[i] = load_kf(i);
#pragma unroll
          for (int tbk = 0; tbk < 4; ++tbk) {
            f32x4 Sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < kSteps; ++ks) {
              const int i = tbk * kSteps + ks;
              if (i + kRing - 1 < kFrags) ring[(i + kRing - 1) % kRing] = load_kf(i + kRing - 1);
              if constexpr (with_copies.value) {  // one row of the next page every fourth matrix instruction
                if (i % 4 == 0 && i / 4 < kPS / kND) issue_a_row(next_src, buf ^ 1, i / 4);
              }
              __builtin_amdgcn_sched_barrier(0);
              Sb = mfma_bf16(ring[i % kRing], qf[ks], Sb);
              __builtin_amdgcn_sched_barrier(0);
            }
            softmax_block(tbk, Sb);
            __builtin_amdgcn_sched_barrier(0);
          }
        };
        if (W == 8 && copies && more) score_product(std::true_type{});
        else score_product(std::false_type{});

        // the page's probabilities and rescale factors go to LDS
        {
#pragma unroll
          for (int j = 0; j < 2; ++j) *LDS_AS(u32x4, lds + PA + (wave * 2 + j) * 1024) = frag[j];
          const int la = fresh();  // (an address built from the kernel's lane constants would be kept across the tile loop)
          if (la < 16) *LDS_AS(float, lds + kOffAlpha + (la * 8 + wave) * 4) = alpha_page;
          if (__any(alpha_page != 1.f) && la == 0) *LDS_AS(int, lds + kOffMoved + buf * 4) = 1;
        }
        uint32_t VA;
        {
          const int lv = fresh();
          const int vrow = 4 * (lv >> 4) + ((lv & 15) >> 2);
          const int x = ((lv & 3) >> 1) ^ vrow;
          VA = (uint32_t)(vrow * kRowA + (x << 4) + (lv & 1) * 8) + boff;
        }
        // raw V^T fragment (bf16 bits): two transpose reads; widened to fp16 later, in place, so that all reads of a
        // token half are in flight together (one LDS latency per half, not one per read)
        // XOR-ed lane base of each of this wavefront's dim blocks: held in registers (128 heads, 4 blocks), or
        // rebuilt at each use (64 heads, 8 blocks: two instructions, and the registers are needed elsewhere)
        constexpr bool kHoldBases = kDW <= 4;
        auto v_base = [&](int dl) {
          return (VA ^ (uint32_t)(((kDW * wave + dl) & 7) << 5)) + (uint32_t)(((kDW * wave + dl) >> 3) * 256);
        };
        uint32_t vb[kHoldBases ? kDW : 1];
        if constexpr (kHoldBases) {
#pragma unroll
          for (int dl = 0; dl < kDW; ++dl) {
            vb[dl] = v_base(dl);
            asm volatile("" : "+v"(vb[dl]));  // a finished base: the token offsets below stay instruction immediates
          }
        }
        auto load_v_raw = [&](int dl, int j) {
          u32x4 vf;
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            const lds_ptr ap = lds + (kHoldBases ? vb[kHoldBases ? dl : 0] : v_base(dl)) + (32 * j + 16 * hf) * kRowA;
            const s16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_AS(s16x4, ap));
            const u32x2 t2 = __builtin_bit_cast(u32x2, t);
            vf[2 * hf] = t2[0];
            vf[2 * hf + 1] = t2[1];
          }
          return vf;
        };
        // The first token half's V^T reads are requested BEFORE the barrier (V has been in LDS since the top of the
        // iteration): their latency passes while this wavefront waits for the others.  LDS operations complete in
        // order, so waiting until only those reads are outstanding means the probabilities have been written.
        // dim blocks in flight: the wavefront's kDW blocks are taken kDB at a time (two with 64 heads: the
        // registers four would take are not there)
        constexpr int kDB = W == 8 ? 4 : 2;
        u32x4 raw[kDB];
#pragma unroll
        for (int dl = 0; dl < kDB; ++dl) raw[dl] = load_v_raw(dl, 0);
        asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(2 * kDB) : "memory");
        wg_barrier();  // all probabilities and rescale factors of this page are in LDS; the rope part is free
        if (W == 8 && copies && more) issue_page_rope(pg + 1);

        // ---- rescale the accumulators if some head's reference moved (rare after the first pages of a tile)
        if (__builtin_amdgcn_readfirstlane(*LDS_AS(const int, lds + kOffMoved + buf * 4))) {
          float al[W];
#pragma unroll
          for (int q4 = 0; q4 < W / 4; ++q4) {
            const f32x4 a4 = *LDS_AS(const f32x4, lds + kOffAlpha + r * 32 + q4 * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i) al[4 * q4 + i] = a4[i];
          }
#pragma unroll
          for (int hb = 0; hb < W; ++hb) {
#pragma unroll
            for (int dl = 0; dl < kDW; ++dl) acc[dl][hb] *= al[hb];
            __builtin_amdgcn_sched_barrier(0);
          }
        }

        // ---- O^T += V^T P^T for this wavefront's dims and all heads.  Per token half j: kDW V^T fragments (two
        // transpose reads each, widened to fp16 in registers), then one probability fragment per head block
        // feeds kDW matrix instructions.
        auto widen_v = [&](u32x4 raw) {
          u32x4 o;
#pragma unroll
          for (int i = 0; i < 4; ++i) o[i] = bf16x2_to_f16x2(raw[i]);
          return __builtin_bit_cast(f16x8, o);
        };
        auto load_p = [&](int hb, int j) {
          return __builtin_bit_cast(f16x8, *LDS_AS(const u32x4, lds + PA + (hb * 2 + j) * 1024));
        };
#pragma unroll
        for (int dh = 0; dh < kDW / kDB; ++dh) {  // one pass (128 heads) or four (64 heads)
          // probability fragments are requested kPF - 1 units ahead (64 heads: two, one wavefront per SIMD has
          // nobody to hide an LDS latency behind; 128 heads: one, there is no register for a third fragment)
          constexpr int kPF = W == 8 ? 2 : 3;
          f16x8 pf[kPF];
#pragma unroll
          for (int a = 0; a < kPF - 1; ++a) pf[a] = load_p(a % W, a / W);
          __builtin_amdgcn_sched_barrier(0);
          f16x8 vf[kDB];
#pragma unroll
          for (int dl = 0; dl < kDB; ++dl) vf[dl] = widen_v(raw[dl]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int u = 0; u < 2 * W; ++u) {  // units (j, hb): one probability fragment feeds kDB matrix instructions
            const int j = u / W, hb = u % W;
            if (u + kPF - 1 < 2 * W) pf[(u + kPF - 1) % kPF] = load_p((u + kPF - 1) % W, (u + kPF - 1) / W);
            // the raw V^T fragments needed next (this pass's second token half, then the next pass's first) are
            // requested during the current half's units, one per unit over its last kDB units
            constexpr int kFirst = W - kDB;
            const bool next_pass = j == 1 && dh + 1 < kDW / kDB;
            if (hb >= kFirst && (j == 0 || next_pass)) raw[hb - kFirst] = load_v_raw(kDB * (dh + (j == 1 ? 1 : 0)) + hb - kFirst, j ^ 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int dl = 0; dl < kDB; ++dl) acc[kDB * dh + dl][hb] = mfma_f16(vf[dl], pf[u % kPF], acc[kDB * dh + dl][hb]);
            __builtin_amdgcn_sched_barrier(0);
            if (u == W - 1 || (u == 2 * W - 1 && dh + 1 < kDW / kDB)) {
#pragma unroll
              for (int dl = 0; dl < kDB; ++dl) vf[dl] = widen_v(raw[dl]);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        // the barrier at the top of the next iteration (or the one below) releases this page's buffers
      }

      // ---- tile epilogue: per-head maximum and sum go through LDS (every wavefront needs them for all heads)
      wg_barrier();  // every wavefront is done with the last page: LDS may be reused, copies may start
      {
        const float l = xor_sum(l_run);
        const int lw = fresh();
        if (lw < 16) {
          *LDS_AS(float, lds + kOffM + (16 * wave + lw) * 4) = m_run;
          *LDS_AS(float, lds + kOffL + (16 * wave + lw) * 4) = l;
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      wg_barrier();
      // Addresses from here on are built from a lane id that is re-read here: a wavefront-uniform base pointer plus
      // a 32-bit offset.  (Built from the kernel's lane constants, the addresses of all reads and stores below are
      // hoisted out of the tile loop and kept -- spilled -- across it; a kernel with spills needs scratch memory,
      // and a launch that needs scratch memory costs tens of microseconds more.)
      const int le = fresh();
      const int re = le & 15, ge = le >> 4;
      float inv[W], lse[W];  // of head 16hb + r
      {
        const uint32_t ml = (uint32_t)(kOffM + re * 4);
#pragma unroll
        for (int hb = 0; hb < W; ++hb) {
          const float m = *LDS_AS(const float, lds + ml + 64 * hb);
          const float l = *LDS_AS(const float, lds + ml + (kOffL - kOffM) + 64 * hb);
          inv[hb] = 1.f / l;  // the accumulators and l carry the same factor 2^kPShift
          lse[hb] = (m - (float)kPShift + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
        }
      }
      const uint32_t lane_col = (uint32_t)(re * kDv + 16 * kDW * wave + 4 * ge);  // head r, first dim of acc[0][.][0]

      // writes a finished row set (this wavefront's dims of all heads) in its final form or as fp32 partial rows
      auto write_rows = [&](const f32x4 (&o)[kDW][W], const float (&sc)[W], const float (&ls)[W]) {
        const bool fin = p.final_out && tile.final_row >= 0;
        if (wave == 0 && ge == 0) {
          float* lse_row = p.out_lse + (size_t)tile.lse_shard * kHq;
          float* fin_lse_row = (fin && p.final_lse) ? p.final_lse + (size_t)tile.final_row * kHq : nullptr;
#pragma unroll
          for (int hb = 0; hb < W; ++hb) {
            lse_row[(uint32_t)(16 * hb + re)] = ls[hb];
            if (fin_lse_row) fin_lse_row[(uint32_t)(16 * hb + re)] = ls[hb];
          }
        }
        constexpr int kElem = kOut == NANOCP_F32 ? 4 : kOut == NANOCP_BF16 ? 2 : 1;
        char* fin_row = fin ? (char*)p.final_out + (size_t)tile.final_row * kHq * kDv * kElem : nullptr;
        float* part_row = p.out_o + (size_t)tile.shard * kHq * kDv;
#pragma unroll
        for (int hb = 0; hb < W; ++hb) {
#pragma unroll
          for (int dl = 0; dl < kDW; ++dl) {
            const f32x4 v = o[dl][hb] * sc[hb];
            const uint32_t col = lane_col + (uint32_t)(16 * hb * kDv + 16 * dl);
            if (fin) {
              const float v4[4] = {v[0], v[1], v[2], v[3]};
              store_final<4>(fin_row, col, kOut, p.out_inv_scale, v4);
            } else {
              *(f32x4*)(part_row + col) = v;
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      };

      if (tile.dst < 0) {
        write_rows(acc, inv, lse);
      } else {
        // one of several tiles: store the normalised partial in register order ([wave][dl][hb][lane] x 16 bytes, so
        // every store covers 1 KB of contiguous memory) and its LSEs; mla_reduce_kernel combines them after this
        // kernel (a partial is 256 KB: reduced by the workgroup that delivers the last tile, as the GQA kernels do
        // with their 8 KB partials, every long request ended with one compute unit reading 1-3 MB alone)
        float* dst = p.ws_o + (size_t)tile.dst * ((size_t)kHq * kDv) + (size_t)wave * (kDW * W * 256);
        const uint32_t lane4 = (uint32_t)le * 4;
#pragma unroll
        for (int dl = 0; dl < kDW; ++dl)
#pragma unroll
          for (int hb = 0; hb < W; ++hb) *(f32x4*)(dst + (lane4 + (uint32_t)((dl * W + hb) * 256))) = acc[dl][hb] * inv[hb];
        if (wave == 0 && ge == 0) {
          float* lse_row = p.ws_lse + (size_t)tile.dst * kHq;
#pragma unroll
          for (int hb = 0; hb < W; ++hb) lse_row[(uint32_t)(16 * hb + re)] = lse[hb];
        }
      }

      if (p.tile_clock && wave == 0 && fresh() == 0) {
        p.tile_clock[3 * (size_t)ti] = clk0;
        p.tile_clock[3 * (size_t)ti + 1] = wall_clock64();
        p.tile_clock[3 * (size_t)ti + 2] = blockIdx.x;
      }
    }
    if (wave == 0 && fresh() == 0) *LDS_AS(int, lds + kOffNext) = (int)gridDim.x + atomicAdd(&p.sync[0], 1);
    __syncthreads();
    chunk = __builtin_amdgcn_readfirstlane(*LDS_AS(const int, lds + kOffNext));
    __syncthreads();
  }
  // the last workgroup to leave re-arms the queue for the next launch
  if (wave == 0 && fresh() == 0) {
    const int done = atomicAdd(&p.sync[1], 1);
    if (done == (int)gridDim.x - 1) {
      p.sync[0] = 0;
      p.sync[1] = 0;
    }
  }
}

// LSE-combine of the tile partials of one segment (same operator as the Phase 4 merge), reading the partials in
// the register order the tile kernel stored them in.  One thread per 16-byte unit; parts are taken 8 at a time with a
// running maximum.  Segments without parts are shards without tokens: O = 0, LSE = -inf.
template <int W, int kOut>
__global__ __launch_bounds__(256) void mla_reduce_kernel(KParams p, const Seg* __restrict__ segs) {
  constexpr int kHq = 16 * W, kDW = 32 / W;
  if (p.header && (int)blockIdx.x >= p.header[1]) return;  // plan image: launched for the bucket's capacity
  const Seg sg = segs[blockIdx.x];
  const int u = blockIdx.y * 256 + threadIdx.x;  // unit ((wave * kDW + dl) * W + hb) * 64 + lane
  const int lane = u & 63, hb = (u >> 6) % W, dl = ((u >> 6) / W) % kDW, wave = (u >> 6) / (W * kDW);
  const int head = 16 * hb + (lane & 15), dim0 = 16 * (kDW * wave + dl) + 4 * (lane >> 4);
  const size_t per_tile = (size_t)kHq * kDv;
  float top = -INFINITY, tot = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < sg.n_parts; k0 += 8) {
    float li[8];
    f32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {  // (the part count is the same for the whole workgroup: no load is issued twice)
      li[j] = -INFINITY;
      v[j] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (k0 + j < sg.n_parts) {
        const size_t slot = (size_t)(sg.slot_begin + k0 + j);
        li[j] = p.ws_lse[slot * kHq + head];
        v[j] = *(const f32x4*)(p.ws_o + slot * per_tile + (size_t)u * 4);
      }
    }
    float bm = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) bm = fmaxf(bm, li[j]);
    const float nt = fmaxf(top, bm);  // finite: tile partials are never empty
    const float sc = expf(top - nt);
    tot *= sc;
    acc *= sc;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool live = li[j] != -INFINITY;
      const float w = live ? expf(li[j] - nt) : 0.f;
      tot += w;
      if (live) acc += v[j] * w;
    }
    top = nt;
  }
  const bool empty = sg.n_parts == 0;
  const float inv = empty ? 0.f : 1.f / tot;
  const float lse = empty ? -INFINITY : top + logf(tot);
  const bool fin = p.final_out && sg.final_row >= 0;
  if (dim0 == 0) {
    p.out_lse[(size_t)sg.shard * kHq + head] = lse;
    if (fin && p.final_lse) p.final_lse[(size_t)sg.final_row * kHq + head] = lse;
  }
  const f32x4 o = acc * inv;
  const size_t col = (size_t)head * kDv + dim0;
  if (fin) {
    const float o4[4] = {o[0], o[1], o[2], o[3]};
    store_final<4>(p.final_out, (size_t)sg.final_row * kHq * kDv + col, kOut, p.out_inv_scale, o4);
  } else {
    *(f32x4*)(p.out_o + (size_t)sg.shard * kHq * kDv + col) = o;
  }
}

// Both kernels: 8 wavefronts, two per SIMD, 256 registers each.  128 heads: all of them compute.
template <int kOut>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void mla_mfma_kernel(KParams p) {
  mla_mfma_body<8, 4, kOut>(p);
}
// 64 heads: four compute, four copy
template <int kOut>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void mla64_mfma_kernel(KParams p) {
  mla_mfma_body<4, 4, kOut>(p);
}

// The dynamic-LDS limit is an attribute of the kernel on ONE device: it is raised once per device and kernel, with
// that device current, the first time the kernel is launched there.
template <typename K>
hipError_t allow_big_lds(K kernel, int bytes, int slot) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static bool done[6][kMaxDevices] = {};
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

template <int kOut>
hipError_t launch_out(const KParams& p, int num_blocks, hipStream_t st, int slot) {
  if (p.Hq == 128) {
    const hipError_t attr = allow_big_lds(mla_mfma_kernel<kOut>, kLdsBytes, slot);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(mla_mfma_kernel<kOut>, dim3(num_blocks), dim3(512), kLdsBytes, st, p);
  } else if (p.Hq == 64) {
    const hipError_t attr = allow_big_lds(mla64_mfma_kernel<kOut>, kLdsBytes, slot + 3);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(mla64_mfma_kernel<kOut>, dim3(num_blocks), dim3(512), kLdsBytes, st, p);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int kOut>
hipError_t launch_reduce_out(const KParams& p, const Seg* segs, int num_segs, hipStream_t st) {
  if (p.Hq == 128)
    hipLaunchKernelGGL((mla_reduce_kernel<8, kOut>), dim3(num_segs, 128 * kDv / 4 / 256), dim3(256), 0, st, p, segs);
  else if (p.Hq == 64)
    hipLaunchKernelGGL((mla_reduce_kernel<4, kOut>), dim3(num_segs, 64 * kDv / 4 / 256), dim3(256), 0, st, p, segs);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace

// the reduction that goes with the tile kernel's partial layout: `num_segs` segments (cut (shard, head-set)s and
// shards without tokens)
hipError_t launch_mla_reduce(const KParams& p, const Seg* segs, int num_segs, hipStream_t st) {
  if (num_segs <= 0) return hipSuccess;
  if (p.final_kind == NANOCP_BF16) return launch_reduce_out<NANOCP_BF16>(p, segs, num_segs, st);
  if (p.final_kind == NANOCP_FP8_E4M3) return launch_reduce_out<NANOCP_FP8_E4M3>(p, segs, num_segs, st);
  return launch_reduce_out<NANOCP_F32>(p, segs, num_segs, st);
}

hipError_t launch_mla_mfma(const KParams& p, int num_blocks, hipStream_t st) {
  if (p.final_kind == NANOCP_BF16) return launch_out<NANOCP_BF16>(p, num_blocks, st, 0);
  if (p.final_kind == NANOCP_FP8_E4M3) return launch_out<NANOCP_FP8_E4M3>(p, num_blocks, st, 1);
  return launch_out<NANOCP_F32>(p, num_blocks, st, 2);
}

}  // namespace nanocp
