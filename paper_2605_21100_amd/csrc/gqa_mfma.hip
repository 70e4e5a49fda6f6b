// MFMA tile kernels for GQA decode with 16 query heads per kv head, head dim 128, page size 64:
// bf16 KV and fp8 (OCP E4M3FN) KV.  Paper: Data Plane, Phase 2 (partial attention + LSE over the
// local KV partition).
//
// Work split.  One workgroup (4 wavefronts) runs the tiles of one chunk of the work-list.  Inside
// a tile the wavefronts take alternate steps of kStep tokens (32 for bf16, 64 for fp8), each keeping
// its own running max / sum / accumulator; they are combined through LDS once per tile.
//
// Data path.  K and V go from HBM straight into MFMA operand registers: the page layouts
// (token groups of 4x slots; [Dk/x][4x][x] for K, [4][Dv][x] for V, x = elements per 16 bytes) make every 16-byte vector a
// ready operand fragment, and 16 consecutive lanes always read 256 contiguous bytes (whole cache
// lines, each touched by exactly one load instruction, which is what lets the streaming hint pay).
//   scores:  S^T[token, head] = K[token, :] . Q[head, :]        v_mfma_f32_16x16x32_bf16, A = K, B = Q^T
//   output:  O^T[dim,  head] += V^T[dim, token] P^T[token, head]                       A = V^T, B = P^T
// The C layout of the first product gives lane group g (lanes 16g..16g+15) the token rows 4g..4g+3 of
// every 16-token block b; the B operand of the second wants lane group g to hold 8 (or 16) values of
// consecutive k.  The V page layout stores exactly those tokens {16b + 4g + i} together in vector g
// (element 4b + i), so the probabilities are in operand order as they come out of the softmax and no
// cross-lane data movement is needed.
// P is split into two bf16 terms (hi + lo) so that the P*V product keeps ~16 bits of P.
// fp8 K/V are widened to bf16 in registers (exact); the per-(page, head) scales are applied to the
// scores (K) and to P (V) in fp32.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <type_traits>

#include "arrive.h"
#include "epilogue.h"
#include "plan.h"

namespace nanocp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kG = 16;    // query heads per kv head
constexpr int kD = 128;   // head dim (qk and v)
constexpr int kPS = 64;   // page size
constexpr int kWaves = kThreads / 64;
constexpr int kOPad = kD + 4;  // LDS row stride (floats) of the combine buffer

// Read-only metadata (work-list, block table, fp8 scales) is never written by this kernel; reading it
// through the constant address space lets wave-uniform reads use the scalar unit (SGPR results, own
// wait counter) instead of occupying vector-memory slots.
template <typename T>
using cptr = const __attribute__((address_space(4))) T*;
template <typename T>
__device__ inline cptr<T> as_const(const T* ptr) {
  return (cptr<T>)(uintptr_t)ptr;
}

__device__ inline f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// 16-byte load of K/V; kNT adds the non-temporal hint (K/V are read exactly once)
template <bool kNT>
__device__ inline u32x4 ldg16(const void* base, uint32_t byte_off) {
  const u32x4* ptr = (const u32x4*)((const char*)base + byte_off);
  return kNT ? __builtin_nontemporal_load(ptr) : *ptr;
}

__device__ inline uint32_t pack_bf16(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}

// two OCP E4M3 bytes (low or high half of w) -> two bf16, exact: v_cvt_scalef32_pk_bf16_fp8 with scale 1
template <bool kHi>
__device__ inline uint32_t fp8x2_to_bf16x2(uint32_t w) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, kHi));
}

// 8 fp8 bytes (two dwords) -> 8 bf16
__device__ inline bf16x8 widen8(uint32_t w0, uint32_t w1) {
  u32x4 r = {fp8x2_to_bf16x2<false>(w0), fp8x2_to_bf16x2<true>(w0), fp8x2_to_bf16x2<false>(w1),
             fp8x2_to_bf16x2<true>(w1)};
  return __builtin_bit_cast(bf16x8, r);
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

// hi/lo bf16 split of 8 probabilities -> two B operands
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

template <bool kFp8>
struct StepRegs {
  // bf16: 32 tokens -> K 2 blocks x 4 k-steps, V 8 dim blocks, 16 bytes each
  // fp8:  64 tokens -> K 4 blocks x 2 loads (16 dims each), V 8 dim blocks (16 tokens each)
  u32x4 k[8];
  u32x4 v[8];
  float ks, vs;  // fp8 scales of the step's page
};

// kOut: element type of the final rows (nanocp_dtype), a compile-time constant so that each instantiation carries
// one output epilogue only -- the kernel's run time is sensitive to its instruction footprint (every tile walks
// through prologue and epilogue code that is cold by then).
template <bool kFp8, bool kNT, int kOut>
__global__ __launch_bounds__(kThreads, 1) void gqa_mfma_kernel(KParams p) {
  constexpr int kStep = kFp8 ? 64 : 32;            // tokens per step
  constexpr int kEl = kFp8 ? 1 : 2;                // bytes per kv element
  constexpr int kBlocks = kStep / 16;              // score MFMA blocks per step
  constexpr uint32_t kPageHeadBytes = kPS * kD * kEl;  // one (page, kv head) of K or of V
  constexpr int kNS = kStep / 4;                   // scores per lane per step

  __shared__ float o_s[kWaves][kG][kOPad];
  __shared__ float m_s[kWaves][kG], l_s[kWaves][kG];
  __shared__ int next_s, arrive_s;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: step indices, pages and branches stay uniform
  const int r = lane & 15, g = lane >> 4;
  const int Hkv = p.Hkv;
  const float c_log2 = p.scale * 1.4426950408889634f;

  // per-lane byte offsets inside a (page, head) block; the step's slot offset is added per step
  // K of a step's token group: vector (c, t) at (c*kStep + t)*16, t = slot inside the group.  Score block b,
  // row r  <->  slot 16b + r, so 16 lanes read 256 contiguous bytes and a step reads one contiguous 8 KB run
  const uint32_t k_lane = (uint32_t)((g * kStep + r) * 16);
  // V vector (u, c) at (u*Dv + c)*16.   lane (r, g): vector slot0/x + g of the step's token group, dim 16j + r
  const uint32_t v_lane = (uint32_t)((g * kD + r) * 16);

  // Work queue: workgroup b starts with chunk b, then pulls the next unclaimed chunk.  The queue is
  // ordered from large to small chunks, so differences in speed between workgroups even out at the end.
  const cptr<int32_t> chunk_offsets = as_const(p.chunk_offsets);
  const cptr<int32_t> tile_words = as_const((const int32_t*)p.tiles);
  auto load_tile = [&](int ti) {
    DevTile t;
    const cptr<int32_t> w = tile_words + (size_t)ti * (sizeof(DevTile) / 4);
    t.q_row = w[0], t.bt_row = w[1], t.kv_head = w[2], t.shard = w[3];
    t.tok_begin = w[4], t.tok_end = w[5], t.dst = w[6], t.seg = w[7];
    t.n_parts = w[8], t.slot_begin = w[9], t.final_row = w[10], t.lse_shard = w[11];
    return t;
  };
  // plan image: the counts live on the device.  An image packed for another kernel variant, or one whose shards
  // are grouped into final rows while no final rows were given, is not run at all (outputs stay untouched).
  if (p.header && (as_const(p.header)[4] != p.variant || (as_const(p.header)[5] != 0 && !p.final_out))) return;
  const int num_chunks = p.header ? as_const(p.header)[0] : p.num_chunks;
  for (int chunk = blockIdx.x; chunk < num_chunks;) {
  const int t0 = chunk_offsets[chunk], t1 = chunk_offsets[chunk + 1];
  DevTile tile_next = load_tile(t0);
  for (int ti = t0; ti < t1; ++ti) {
    const DevTile tile = tile_next;
    // the next tile's record is fetched now (scalar loads), so that its latency is not on the next tile's critical
    // path in front of the block-table and K/V loads; reading one record past the chunk is harmless only inside
    // the list, hence the clamp
    tile_next = load_tile(ti + 1 < t1 ? ti + 1 : ti);
    uint64_t clk0 = 0;
    if (p.tile_clock && tid == 0) clk0 = wall_clock64();
    const int h = tile.kv_head;
    const cptr<int32_t> bt = as_const(p.block_table + (size_t)tile.bt_row * p.max_blocks);
    const int tb = tile.tok_begin, te = tile.tok_end;

    // Q fragments (B operand): lane (g, n = r) holds Q[n][dims of k-step s]
    bf16x8 qf[4];
    {
      const char* qrow = (const char*)p.q + ((size_t)tile.q_row * p.Hq + (size_t)h * kG + r) * kD * 2;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        // bf16 KV: k-step s, group g <-> dim chunk 4s+g (8 dims).
        // fp8 KV:  load u = s/2 brings dims 16(g+4u)..+16; k-step s takes its half s%2.
        const int dim0 = kFp8 ? (16 * (g + 4 * (s >> 1)) + 8 * (s & 1)) : (8 * (4 * s + g));
        qf[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + dim0 * 2));
      }
    }

    f32x4 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;  // running max of scaled (log2-domain) scores of head r
    float l_run = 0.f;        // this lane's share of the running sum

    // Steps are kStep-aligned in the row's token coordinates.  Steps that lie entirely inside [tb, te)
    // ("full") run in the pipelined loop; the at most two ragged ones (shard begins / ends inside a step)
    // are taken separately, with masking, by the wavefronts that get the fewest full steps.
    const int u_first = tb / kStep, u_last = (te - 1) / kStep;
    const bool head_ragged = (tb % kStep) != 0, tail_ragged = (te % kStep) != 0;
    int fb = u_first + (head_ragged ? 1 : 0);  // full steps [fb, fe)
    int fe = u_last + 1 - (tail_ragged ? 1 : 0);
    int rag0 = head_ragged ? u_first : -1;     // ragged steps (or -1)
    int rag1 = (tail_ragged && !(head_ragged && u_last == u_first)) ? u_last : -1;
    if (fe < fb) fe = fb;
    const int u_end = fe;
    int u = fb + wave;

    auto page_of = [&](int uu) { return uu <= u_last ? bt[(uu * kStep) / kPS] : 0; };
    auto load_step = [&](StepRegs<kFp8>& sr, int uu, int page) {
      const int tok0 = uu * kStep;
      const uint32_t slot0 = (uint32_t)(tok0 % kPS);
      const size_t ph = ((size_t)page * Hkv + h) * kPageHeadBytes;
      const char* kb = (const char*)p.k_pool + ph;
      const char* vb = (const char*)p.v_pool + ph;
      if (kFp8) {
        sr.ks = as_const(p.k_scale)[(size_t)page * Hkv + h];
        sr.vs = as_const(p.v_scale)[(size_t)page * Hkv + h];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
          for (int q2 = 0; q2 < 2; ++q2)
            sr.k[b * 2 + q2] = ldg16<kNT>(kb, k_lane + (uint32_t)((4 * q2 * kStep + 16 * b) * 16));
#pragma unroll
        for (int j = 0; j < 8; ++j) sr.v[j] = ldg16<kNT>(vb, v_lane + (uint32_t)(((slot0 / 16) * kD + 16 * j) * 16));
      } else {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int s = 0; s < 4; ++s)
            sr.k[b * 4 + s] = ldg16<kNT>(kb, k_lane + (uint32_t)((slot0 * kD / 8 + 4 * s * kStep + 16 * b) * 16));
#pragma unroll
        for (int j = 0; j < 8; ++j) sr.v[j] = ldg16<kNT>(vb, v_lane + (uint32_t)(((slot0 / 8) * kD + 16 * j) * 16));
      }
    };

    auto compute_step = [&](StepRegs<kFp8>& sr, int uu, auto ragged_tag) {
      constexpr bool ragged = decltype(ragged_tag)::value;
      const int tok0 = uu * kStep;
      // ---- scores
      f32x4 S[kBlocks];
#pragma unroll
      for (int b = 0; b < kBlocks; ++b) {
        S[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (kFp8) {
#pragma unroll
          for (int q2 = 0; q2 < 2; ++q2) {
            const u32x4 w = sr.k[b * 2 + q2];
            S[b] = mfma16(widen8(w[0], w[1]), qf[2 * q2], S[b]);
            S[b] = mfma16(widen8(w[2], w[3]), qf[2 * q2 + 1], S[b]);
          }
        } else {
#pragma unroll
          for (int s = 0; s < 4; ++s) S[b] = mfma16(__builtin_bit_cast(bf16x8, sr.k[b * 4 + s]), qf[s], S[b]);
        }
      }
      // ---- online softmax in the log2 domain.  S[b][i] is token tok0 + 16b + 4g + i, which the V layout
      // stores as element 4b + i of the step's vector g: the scores are already in P*V operand order
      const float cs = kFp8 ? c_log2 * sr.ks : c_log2;
      float y[kNS];
      float mloc = -INFINITY;
#pragma unroll
      for (int b = 0; b < kBlocks; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v = S[b][i] * cs;
          if (ragged) {
            const int tok = tok0 + 16 * b + 4 * g + i;
            v = (tok >= tb && tok < te) ? v : -INFINITY;
          }
          y[b * 4 + i] = v;
          mloc = fmaxf(mloc, v);
        }
      mloc = xor_max(mloc);
      const float m_new = fmaxf(m_run, mloc);  // finite: every step overlaps the tile's range
      if (__any(m_new > m_run)) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= alpha;
        m_run = m_new;
      }
      float pr[kNS];
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < kNS; ++e) {
        pr[e] = __builtin_amdgcn_exp2f(y[e] - m_run);
        psum += pr[e];
      }
      l_run += psum;
      if (kFp8) {
#pragma unroll
        for (int e = 0; e < kNS; ++e) pr[e] *= sr.vs;
      }
      // ---- mask unused token slots of V (they may hold NaN patterns)
      if (ragged) {
        if (kFp8) {
          // lane's V vector: byte 4w + e  <->  token tok0 + 16w + 4g + e
          u32x4 mk;
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            uint32_t mw = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int tok = tok0 + 16 * w + 4 * g + e;
              if (tok >= tb && tok < te) mw |= 0xffu << (8 * e);
            }
            mk[w] = mw;
          }
#pragma unroll
          for (int j = 0; j < 8; ++j) sr.v[j] &= mk;
        } else {
          u32x4 mk;
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            uint32_t mw = 0;
#pragma unroll
            for (int e = 0; e < 2; ++e) {  // element 2w + e = 4b + i  <->  token tok0 + 16b + 4g + i
              const int tok = tok0 + 16 * (w >> 1) + 4 * g + 2 * (w & 1) + e;
              if (tok >= tb && tok < te) mw |= 0xffffu << (16 * e);
            }
            mk[w] = mw;
          }
#pragma unroll
          for (int j = 0; j < 8; ++j) sr.v[j] &= mk;
        }
      }
      // ---- O^T += V^T P^T
      if (kFp8) {
        bf16x8 hi0, lo0, hi1, lo1;  // vector elements 0..7 (score blocks 0,1) and 8..15 (blocks 2,3)
        split8(pr, hi0, lo0);
        split8(pr + 8, hi1, lo1);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const u32x4 w = sr.v[j];
          const bf16x8 va = widen8(w[0], w[1]), vb2 = widen8(w[2], w[3]);
          acc[j] = mfma16(va, hi0, acc[j]);
          acc[j] = mfma16(va, lo0, acc[j]);
          acc[j] = mfma16(vb2, hi1, acc[j]);
          acc[j] = mfma16(vb2, lo1, acc[j]);
        }
      } else {
        bf16x8 hi, lo;
        split8(pr, hi, lo);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bf16x8 va = __builtin_bit_cast(bf16x8, sr.v[j]);
          acc[j] = mfma16(va, hi, acc[j]);
          acc[j] = mfma16(va, lo, acc[j]);
        }
      }
    };

    // software pipeline over the full steps: the loads of step n+1 are in flight while step n is
    // computed, and the block-table entry of step n+2 is fetched one step ahead.  The steady state has
    // no conditional loads, so the wait for the older buffer is a counted one, not a drain.
    StepRegs<kFp8> ra, rb, rc;
    // the ragged step of this wavefront (the head by the last wavefront, the tail by the one before it) is
    // requested first and computed last: its latency hides behind the full steps
    const int ru = wave == kWaves - 1 ? rag0 : (wave == kWaves - 2 ? rag1 : -1);
    if (ru >= 0) load_step(rc, ru, page_of(ru));
    if (u < u_end) {
      load_step(ra, u, page_of(u));
      int pg_next = page_of(u + kWaves);
      while (true) {
        if (u + kWaves >= u_end) {
          compute_step(ra, u, std::false_type{});
          break;
        }
        load_step(rb, u + kWaves, pg_next);
        pg_next = page_of(u + 2 * kWaves);
        compute_step(ra, u, std::false_type{});
        u += kWaves;
        if (u + kWaves >= u_end) {
          compute_step(rb, u, std::false_type{});
          break;
        }
        load_step(ra, u + kWaves, pg_next);
        pg_next = page_of(u + 2 * kWaves);
        compute_step(rb, u, std::false_type{});
        u += kWaves;
      }
    }
    if (ru >= 0) compute_step(rc, ru, std::true_type{});

    // ---- combine the 4 wavefronts' partials
    l_run = xor_sum(l_run);
    if (g == 0) {
      m_s[wave][r] = m_run;
      l_s[wave][r] = l_run;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) *(f32x4*)&o_s[wave][r][16 * j + 4 * g] = acc[j];  // rows 4g+i of block j = dims 16j+4g+i
    __syncthreads();
    {
      // thread <-> (head n, 8 dims)
      const int n = tid >> 4, c16 = tid & 15;
      float mw[kWaves], M = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        mw[w] = m_s[w][n];
        M = fmaxf(M, mw[w]);
      }
      float L = 0.f, f[kWaves];
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        f[w] = __builtin_amdgcn_exp2f(mw[w] - M);  // a wavefront without steps has m = -inf -> weight 0
        L += f[w] * l_s[w][n];
      }
      const float inv = 1.f / L;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) f[w] *= inv;
      const float lse_nat = (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f;
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = 0.f;
      if (tile.dst < 0) {
        // the only tile of its (shard, head): final rows; the thread owns 8 consecutive dims (two 16-byte stores)
        const int d0 = c16 * 8;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const f32x4 a = *(const f32x4*)&o_s[w][n][d0], b = *(const f32x4*)&o_s[w][n][d0 + 4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[e] = fmaf(f[w], a[e], o[e]);
            o[4 + e] = fmaf(f[w], b[e], o[4 + e]);
          }
        }
        if (c16 == 0) p.out_lse[(size_t)tile.lse_shard * p.Hq + (size_t)h * kG + n] = lse_nat;
        if (p.final_out && tile.final_row >= 0) {
          // the shard alone is an output row: written in its final form, no merge needed
          const size_t fo = ((size_t)tile.final_row * p.Hq + (size_t)h * kG + n) * kD + d0;
          store_final<8>(p.final_out, fo, kOut, p.out_inv_scale, o);
          if (c16 == 0 && p.final_lse) p.final_lse[(size_t)tile.final_row * p.Hq + (size_t)h * kG + n] = lse_nat;
        } else {
          float* dst_o = p.out_o + ((size_t)tile.shard * p.Hq + (size_t)h * kG + n) * kD + d0;
          *(f32x4*)dst_o = f32x4{o[0], o[1], o[2], o[3]};
          *(f32x4*)(dst_o + 4) = f32x4{o[4], o[5], o[6], o[7]};
        }
      } else {
        // one of several tiles: publish the partial, and let the workgroup that delivers the last one
        // LSE-combine them (same operator as the Phase 4 merge) into the shard's rows.  Here the thread owns
        // the dim pairs 2 c16 + 32 e, + 1, so that each of the 8-byte device-scope stores / loads of 16 neighbouring
        // lanes covers 128 contiguous bytes (a device-scope access costs per instruction: four instead of eight).
#pragma unroll
        for (int w = 0; w < kWaves; ++w)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[2 * e] = fmaf(f[w], o_s[w][n][2 * c16 + 32 * e], o[2 * e]);
            o[2 * e + 1] = fmaf(f[w], o_s[w][n][2 * c16 + 32 * e + 1], o[2 * e + 1]);
          }
        float* dst_o = p.ws_o + ((size_t)tile.dst * kG + n) * kD + 2 * c16;
#pragma unroll
        for (int e = 0; e < 4; ++e) st_dev2(dst_o + 32 * e, o[2 * e], o[2 * e + 1]);
        if (c16 == 0) st_dev(p.ws_lse + (size_t)tile.dst * kG + n, lse_nat);
        // publish, count the arrival, and reduce if this workgroup delivered the last partial (csrc/arrive.h)
        if (arrive_is_last(&p.sync[kSyncSegBase + tile.seg], tile.n_parts, &arrive_s)) {
          const float* wl = p.ws_lse + (size_t)tile.slot_begin * kG + n;
          const float* wo = p.ws_o + ((size_t)tile.slot_begin * kG + n) * kD + 2 * c16;
          // One pass with a running maximum, four partials at a time: their 36 loads are issued together, so a
          // segment of n partials costs ceil(n / 4) memory round trips on this workgroup (it is the last one of the
          // segment: nothing else hides them).  Tile partials are never empty: every LSE is finite.
          float top = -INFINITY, tot = 0.f, r8[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) r8[e] = 0.f;
          for (int k0 = 0; k0 < tile.n_parts; k0 += 4) {
            float lw[4], v[4][8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              lw[j] = -INFINITY;
#pragma unroll
              for (int e = 0; e < 8; ++e) v[j][e] = 0.f;
              if (k0 + j < tile.n_parts) {  // uniform over the workgroup
                lw[j] = ld_dev(wl + (size_t)(k0 + j) * kG);
#pragma unroll
                for (int e = 0; e < 4; ++e) ld_dev2(wo + (size_t)(k0 + j) * kG * kD + 32 * e, v[j][2 * e], v[j][2 * e + 1]);
              }
            }
            const float nt = fmaxf(fmaxf(top, fmaxf(lw[0], lw[1])), fmaxf(lw[2], lw[3]));
            const float sc = expf(top - nt);  // 0 on the first batch (top = -inf)
            tot *= sc;
#pragma unroll
            for (int e = 0; e < 8; ++e) r8[e] *= sc;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const float w = expf(lw[j] - nt);  // 0 for the padding of the last batch
              tot += w;
#pragma unroll
              for (int e = 0; e < 8; ++e) r8[e] = fmaf(w, v[j][e], r8[e]);
            }
            top = nt;
          }
          const float rinv = 1.f / tot;
          const float lse_f = top + logf(tot);
          // (shards reduced as one group deliver the row's LSE at the group's first shard, whoever arrives last)
          if (c16 == 0) p.out_lse[(size_t)tile.lse_shard * p.Hq + (size_t)h * kG + n] = lse_f;
          if (p.final_out && tile.final_row >= 0) {
            const size_t fi = ((size_t)tile.final_row * p.Hq + (size_t)h * kG + n) * kD + 2 * c16;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float v1[1] = {r8[e] * rinv};
              store_final<1>(p.final_out, fi + 32 * (e >> 1) + (e & 1), kOut, p.out_inv_scale, v1);
            }
            if (c16 == 0 && p.final_lse) p.final_lse[(size_t)tile.final_row * p.Hq + (size_t)h * kG + n] = lse_f;
          } else {
            float* fo = p.out_o + ((size_t)tile.shard * p.Hq + (size_t)h * kG + n) * kD + 2 * c16;
#pragma unroll
            for (int e = 0; e < 4; ++e) *(float2*)(fo + 32 * e) = make_float2(r8[2 * e] * rinv, r8[2 * e + 1] * rinv);
          }
          if (tid == 0) arrive_reset(&p.sync[kSyncSegBase + tile.seg]);  // ready for the next launch
        }
      }
    }
    __syncthreads();
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
  // (shard, head) pairs without tokens (the plan lists no others for this kernel): O = 0, LSE = -inf
  {
    const int num_segs = p.header ? as_const(p.header)[1] : p.num_segs;
    const int n = tid >> 4, d0 = (tid & 15) * 8;
    for (int si = blockIdx.x; si < num_segs; si += gridDim.x) {
      const Seg sg = p.segs[si];
      if (sg.n_parts != 0) continue;
      const size_t head = (size_t)sg.kv_head * kG + n;
      if ((tid & 15) == 0) p.out_lse[(size_t)sg.shard * p.Hq + head] = -INFINITY;
      if (p.final_out && sg.final_row >= 0) {
        const size_t fo = ((size_t)sg.final_row * p.Hq + head) * kD + d0;
        store_final_zero<8>(p.final_out, fo, kOut);
        if ((tid & 15) == 0 && p.final_lse) p.final_lse[(size_t)sg.final_row * p.Hq + head] = -INFINITY;
      } else {
        float* dst_o = p.out_o + ((size_t)sg.shard * p.Hq + head) * kD + d0;
        *(f32x4*)dst_o = f32x4{0.f, 0.f, 0.f, 0.f};
        *(f32x4*)(dst_o + 4) = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
  }
  // the last workgroup to leave re-arms the queue for the next launch
  if (tid == 0) {
    const int done = atomicAdd(&p.sync[1], 1);
    if (done == (int)gridDim.x - 1) {
      p.sync[0] = 0;
      p.sync[1] = 0;
    }
  }
}

}  // namespace

template <bool kFp8, bool kNT>
void launch_out(const KParams& p, dim3 grid, dim3 block, hipStream_t st) {
  if (p.final_kind == NANOCP_BF16)
    hipLaunchKernelGGL((gqa_mfma_kernel<kFp8, kNT, NANOCP_BF16>), grid, block, 0, st, p);
  else if (p.final_kind == NANOCP_FP8_E4M3)
    hipLaunchKernelGGL((gqa_mfma_kernel<kFp8, kNT, NANOCP_FP8_E4M3>), grid, block, 0, st, p);
  else
    hipLaunchKernelGGL((gqa_mfma_kernel<kFp8, kNT, NANOCP_F32>), grid, block, 0, st, p);
}

hipError_t launch_gqa_mfma(int variant, const KParams& p, int num_blocks, hipStream_t st) {
  dim3 grid(num_blocks), block(kThreads);
  // K/V are read exactly once: the streaming (non-temporal) loads are the product path.  A -DNANOCP_TUNING build can
  // switch them off from the environment to measure what they buy.
#ifdef NANOCP_TUNING
  static const bool nt = [] {
    const char* v = std::getenv("NANOCP_KV_NONTEMPORAL");
    return !(v && v[0] == '0');
  }();
  if (!nt) {
    if (variant == kGqaMfmaBf16) launch_out<false, false>(p, grid, block, st);
    else if (variant == kGqaMfmaFp8) launch_out<true, false>(p, grid, block, st);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
#endif
  if (variant == kGqaMfmaBf16)
    launch_out<false, true>(p, grid, block, st);
  else if (variant == kGqaMfmaFp8)
    launch_out<true, true>(p, grid, block, st);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace nanocp
