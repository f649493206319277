// Attention of a whole chunk of new tokens over the compressed cache
// (App. A.1 Eq. 18 with Q in R^{T x d_h}, on K~ = K_down P_K^T, V~ = V_down P_V^T
// of Sec. 3.2 Eq. 7; causal: token t of the chunk sits at position n_prev + t and
// sees cache rows 0 .. n_prev + t).
//
// Unlike the single-query decode step this is a dense contraction, so it runs on
// the matrix cores (v_mfma_f32_32x32x16_bf16, float32 accumulate), in the factored
// form: Q~ = Q P_K, S = Q~ K_down^T, online softmax, A = P V_down, O = A P_V^T.
//
// Every product is computed transposed (keys or channels along the 32 result
// rows, the 32 query rows of a wave along the result columns).  In the result
// layout of the 32x32 MFMA a lane then holds 16 entries of ONE query row, so the
// softmax statistics of a row live in one lane (plus its partner 32 lanes up),
// the accumulator rescale is a per-lane scalar, and the probabilities are
// already laid out as the next product's B operand.
//
//   operand layout (wave of 64, ln = lane % 32, lh = lane / 32):
//     A[m = ln][k = 8 lh .. 8 lh + 7]      B[k = 8 lh .. 8 lh + 7][n = ln]
//     C register 4 i + j  <->  C[m = 8 i + 4 lh + j][n = ln]
//
// The contraction index of a product may be enumerated in any order as long as
// both operands agree; the orders are chosen so that every operand fetch is one
// 16-byte piece:
//   * P_K^T is staged in LDS with bits 2 and 3 of the channel index swapped, so
//     registers 8u..8u+7 of a Q~^T result block are channels 16 kb + 8 lh + 0..7
//     -- the B operand of score step kb, matching a plain 16-byte read of a key row.
//   * V_down tiles are transposed on their way into LDS ([channel][key position]),
//     with bits 2 and 3 of the key index swapped, so registers 8 kb..8 kb+7 of a
//     score block (keys 16 kb + 8 (s/4) + 4 lh + s%4) meet 8 contiguous positions.
//
// Precision.  Q~ (a float32 sum over d_h), the probabilities and the normalised
// mix are float32 numbers that the bf16 matrix cores cannot take directly.
// Each is split into a bf16 head and a bf16 remainder (x ~ hi + lo, relative
// error 2^-17) and fed as two products.  None of the three can do without its
// remainder: fed as one bf16 term (relative error 2^-9) the probabilities alone
// put the output 4e-3 .. 2e-2 from the float64 definition (relative to the
// largest entry of an output vector), the projected queries alone up to 2.5e-3
// and the normalised mix alone up to 2.2e-3, against a bound of 2e-3.
#include <type_traits>

#include "skv_device_util.h"
#include "skv_internal.h"

#ifndef SKV_MINB3_SUM
#define SKV_MINB3_SUM 112         // up to this r_K + r_V the staged-together schedule is held to three waves per SIMD
#endif
#ifndef SKV_PAGED
#define SKV_PAGED 0                 // 1: the caches are page pools addressed through a block table
#endif
#ifndef SKV_RK
#error "compile with -DSKV_RK=<key rank>"
#endif

namespace skv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int D = SKV_HEAD_DIM;
constexpr int KT = kPrefillKeyTile;     // keys per LDS tile
constexpr int NT = kPrefillThreads;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// x minus one half of a bf16 pair, in one instruction: the two-element dot product of the pair with
// (-1, -0) or (-0, -1), accumulated onto x.  The difference of a float32 number and its own bf16 head is a
// float32 number, so whatever rounding the instruction applies the result is the float32 subtraction's
// (checked bit for bit on the GPU over 4 M values from 2^-100 to 2^11 and zeros).  The multipliers are spelt
// with -0 rather than +0 on purpose: (-1, +0) is the bit pattern of an inline constant, and in that form the
// instruction was seen to subtract BOTH halves.
__device__ __forceinline__ float minus_low_half(uint32_t pair, float x) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, 0x8000bf80u), x, false);
}
__device__ __forceinline__ float minus_high_half(uint32_t pair, float x) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, 0xbf808000u), x, false);
}

// Eight float32 -> bf16 heads and bf16 remainders.
__device__ __forceinline__ void split8(const float* x, bf16x8& hi, bf16x8& lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    h[e] = pack_bf16x2(x[2 * e], x[2 * e + 1]);
    l[e] = pack_bf16x2(minus_low_half(h[e], x[2 * e]), minus_high_half(h[e], x[2 * e + 1]));
  }
  hi = __builtin_bit_cast(bf16x8, uint4{h[0], h[1], h[2], h[3]});
  lo = __builtin_bit_cast(bf16x8, uint4{l[0], l[1], l[2], l[3]});
}

__device__ __forceinline__ bf16x8 lds_frag(const uint16_t* p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p));
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// The maximum of a value and its counterpart 32 lanes away, by a vector lane swap (no trip through LDS).
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float max_with_other_half(float x) {
  const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}

// Swap bits 2 and 3 of an index.
__device__ __forceinline__ int swap23(int c) { return (c & ~12) | ((c & 4) << 1) | ((c & 8) >> 1); }

// Workgroups per CU the register allocation aims for (waves per SIMD): a wave issues at most
// one instruction every 8-10 cycles, so both the vector and the matrix pipe stay busy only with
// several waves resident; 3 where the live state fits in 168 registers without spilling.
constexpr int prefill_min_blocks(int rk, int rv, bool pipe) {
  // (every other build is held to two waves per SIMD rather than left to drop to one: at the large ranks the
  // live state sits at the 256-register line, and a kernel allowed one wave takes a few accumulation
  // registers beyond it and halves its residency -- 128/128 took 49 ms that way against 31)
  return (!pipe && rk + rv <= SKV_MINB3_SUM) ? 3 : 2;
}

template <int RK, int RV, bool PIPE>
__global__ __launch_bounds__(NT, prefill_min_blocks(RK, RV, PIPE)) void prefill_kernel(const PrefillParams p) {
  constexpr int KSTEPS = RK / 16;            // contraction steps of the score product
  constexpr int RKB = (RK + 31) / 32;        // 32-channel result blocks of Q~^T
  constexpr int RVB = (RV + 31) / 32;        // 32-channel result blocks of the mix
  constexpr int VSTEPS = RV / 16;            // contraction steps of the lift
  constexpr int KP = RK + 8;                 // LDS pitch of a key row (bf16 elements)
  constexpr int VP = KT + 8;                 // LDS pitch of a value channel
  constexpr int STAGE = KT * KP + RVB * 32 * VP;
  constexpr int BP = D + 8;                  // LDS pitch of a transposed basis row
  constexpr int BASIS = RKB * 32 * BP;
  constexpr int SMEM = 2 * STAGE > BASIS ? 2 * STAGE : BASIS;
  __shared__ __attribute__((aligned(16))) uint16_t smem[SMEM];

  constexpr int KC8 = RK / 8;                // 16-byte pieces per key row
  constexpr int KPIECES = KT * KC8;
  constexpr int KPT = (KPIECES + NT - 1) / NT;
  constexpr int VCP = RV / 2;                // channel pairs per value row
  constexpr int VUNITS = (KT / 8) * VCP;     // (8-key group, channel pair) units per tile
  constexpr int VPT = (VUNITS + NT - 1) / NT;

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int ln = lane & 31;
  const int lh = lane >> 5;

  // Workgroups are dealt to the 8 XCDs round-robin by their linear index; remap it so that
  // the workgroups of one (sequence, KV head), which stream the same rows, share an L2.
  const int total = gridDim.x;
  const int full = total & ~7;
  const int lid = blockIdx.x;
  const int vid = lid < full ? (lid & 7) * (full >> 3) + (lid >> 3) : lid;
  const int by = vid / p.n_tiles;
  const int bx = vid % p.n_tiles;

  const int hp = p.group >= 4 ? 4 : p.group;           // heads of a group per workgroup
  const int passes = p.group / hp;
  const int tile_tokens = 32 * (4 / hp);
  const int pass = by % passes;
  const int bkv = by / passes;
  const int kv = bkv % p.n_kv_heads;
  const int b = bkv / p.n_kv_heads;
  const int head = kv * p.group + pass * hp + wave % hp;
  const int t0 = (p.n_tiles - 1 - bx) * tile_tokens;   // longest contexts first
  const int tw0 = t0 + 32 * (wave / hp);               // first token of this wave's rows
  const bool wave_active = tw0 < p.T;
  const int tok = tw0 + ln;
  const int tok_c = tok < p.T ? tok : p.T - 1;
  const int limit = p.n_prev + tok;                    // last cache row this lane's query sees
  const int wave_last = tw0 + 31 < p.T ? tw0 + 31 : p.T - 1;

  const int t_end = t0 + tile_tokens < p.T ? t0 + tile_tokens : p.T;
  const int n_keys = p.n_prev + t_end;                 // rows any query of this workgroup sees
  const int n_tiles_k = (n_keys + KT - 1) / KT;
  const int last_row = n_keys - 1;

  // The caches as one run of rows per (sequence, KV head).  With a paged cache that run exists only
  // tile by tile: a key tile is 64 rows from a multiple of 64 and a page holds a multiple of 64 rows, so
  // a tile never straddles a page, and row j of tile `tile` is found at base(tile) + j * r with the base
  // moved back by the tile's first row (one table entry per tile, uniform over the workgroup).
  const uint16_t* kc_flat = p.k_cache + ((int64_t)b * p.n_kv_heads + kv) * p.capacity * RK;
  const uint16_t* vc_flat = p.v_cache + ((int64_t)b * p.n_kv_heads + kv) * p.capacity * RV;
  constexpr bool paged = SKV_PAGED != 0;              // a build of its own: the kernel has no scalar registers to spare
#if SKV_PAGED
  // Where each key tile of this (sequence, KV head) starts in the pools, in blocks of 64 rows: looked up
  // once, kept in LDS (4 bytes per tile, sized by the launcher), so that the loop below carries no table
  // pointer, stride or bounds in scalar registers.
  static_assert(KT == 64, "a key tile is one 64-row block of a page");
  extern __shared__ int32_t tile_block_s[];
  for (int i = tid; i < n_tiles_k; i += NT)
    tile_block_s[i] = (int32_t)(cache_row(p.pages, 0, p.n_kv_heads, b, kv, (int64_t)i * KT) >> 6);
  __syncthreads();
  auto page_shift_rows = [&](int tile) -> int64_t {        // physical minus logical first row of the tile
    return ((int64_t)__builtin_amdgcn_readfirstlane(tile_block_s[tile]) - tile) * KT;
  };
#else
  auto page_shift_rows = [&](int) -> int64_t { return 0; };
#endif
  // ---- key/value tiles: global -> registers -> LDS --------------------------------------
  // Tiles that lie wholly inside every query's visible range are fetched with addresses that
  // are a per-thread constant plus a uniform tile base; the last few tiles (the causal
  // diagonal, the end of the cache) clamp their rows instead.
  // (named registers, not an array: as an array the key pieces were seen to stay in scratch memory in some
  // instantiations -- every tile then went global -> wait -> scratch -> LDS, and the prefetch was gone)
  static_assert(KPT <= 4, "a thread holds at most four key pieces");
  uint4 kreg0 = {}, kreg1 = {}, kreg2 = {}, kreg3 = {};
  auto each_key_piece = [&](auto&& f) {
    f(0, kreg0);
    if constexpr (KPT > 1) f(1, kreg1);
    if constexpr (KPT > 2) f(2, kreg2);
    if constexpr (KPT > 3) f(3, kreg3);
  };
  uint32_t vreg[VPT][8];
  int voff[VPT];
#pragma unroll
  for (int u = 0; u < VPT; ++u) {
    const int i = tid + u * NT;
    const int cp = i % VCP, kg = i / VCP;
    voff[u] = (16 * (kg >> 1) + 4 * (kg & 1)) * RV + 2 * cp;
  }
  // INNER: the tile needs no clamping
  auto load_k = [&](auto inner_tag, int tile) {
    const int j0 = tile * KT;
    const uint16_t* kc = paged ? p.k_cache + page_shift_rows(tile) * RK : kc_flat;
    const uint16_t* kt = kc + (int64_t)j0 * RK;
    each_key_piece([&](int u, uint4& piece) {
      const int i = tid + u * NT;
      if (KPIECES % NT == 0 || i < KPIECES) {
        if (decltype(inner_tag)::value) {
          piece = *reinterpret_cast<const uint4*>(kt + (i / KC8) * RK + (i % KC8) * 8);
        } else {
          int row = j0 + i / KC8;
          row = row < last_row ? row : last_row;       // rows past the end re-read the last row; masked later
          piece = *reinterpret_cast<const uint4*>(kc + (int64_t)row * RK + (i % KC8) * 8);
        }
      }
    });
  };
  auto load_v = [&](auto inner_tag, int tile) {
    const int j0 = tile * KT;
    const uint16_t* vc = paged ? p.v_cache + page_shift_rows(tile) * RV : vc_flat;
    const uint16_t* vt = vc + (int64_t)j0 * RV;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
      const int i = tid + u * NT;
      if (VUNITS % NT == 0 || i < VUNITS) {
        const int cp = i % VCP, kg = i / VCP;
        const int kbase = 16 * (kg >> 1) + 4 * (kg & 1);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int dk = 8 * (e >> 2) + (e & 3);
          if (decltype(inner_tag)::value) {
            vreg[u][e] = *reinterpret_cast<const uint32_t*>(vt + voff[u] + dk * RV);
          } else {
            int row = j0 + kbase + dk;
            row = row < last_row ? row : last_row;
            vreg[u][e] = *reinterpret_cast<const uint32_t*>(vc + (int64_t)row * RV + 2 * cp);
          }
        }
      }
    }
  };
  auto store_k = [&](uint16_t* ks) {
    each_key_piece([&](int u, uint4& piece) {
      const int i = tid + u * NT;
      if (KPIECES % NT == 0 || i < KPIECES) {
        const int key = i / KC8, c8 = i % KC8;
        *reinterpret_cast<uint4*>(ks + key * KP + c8 * 8) = piece;
      }
    });
  };
  auto store_v = [&](uint16_t* vt) {
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
      const int i = tid + u * NT;
      if (VUNITS % NT == 0 || i < VUNITS) {
        const int cp = i % VCP, kg = i / VCP;
        // keys 16x + 8y + 4z + w (x = kg/2, z = kg%2) go to positions 16x + 8z + 4y + w
        const int pos = 16 * (kg >> 1) + 8 * (kg & 1);
        uint4 even, odd;
        uint32_t* ev = reinterpret_cast<uint32_t*>(&even);
        uint32_t* od = reinterpret_cast<uint32_t*>(&odd);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t a = vreg[u][2 * e], c = vreg[u][2 * e + 1];
          ev[e] = (a & 0xffffu) | (c << 16);
          od[e] = (a >> 16) | (c & 0xffff0000u);
        }
        *reinterpret_cast<uint4*>(vt + (2 * cp) * VP + pos) = even;
        *reinterpret_cast<uint4*>(vt + (2 * cp + 1) * VP + pos) = odd;
      }
    }
  };
  using inner_t = std::true_type;
  using edge_t = std::false_type;

  // ---- projected queries: Q~^T = P_K^T Q^T, scaled, split ------------------------------
  bf16x8 qhi[KSTEPS], qlo[KSTEPS];
  if (!p.folded) {
    const uint16_t* basis = p.p_k + (int64_t)kv * p.p_k_head_stride;
    for (int i = tid; i < D * KC8; i += NT) {
      const int d = i / KC8, c8 = i % KC8;
      const uint4 v = *reinterpret_cast<const uint4*>(basis + d * RK + c8 * 8);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        smem[swap23(c8 * 8 + 2 * e) * BP + d] = (uint16_t)(w[e] & 0xffffu);
        smem[swap23(c8 * 8 + 2 * e + 1) * BP + d] = (uint16_t)(w[e] >> 16);
      }
    }
    if (RK % 32) {                                      // rows of the last block that hold no channel
      for (int i = tid; i < (RKB * 32 - RK) * D; i += NT) smem[(RK + i / D) * BP + i % D] = 0;
    }
    __syncthreads();
    const uint16_t* qrow = p.q + (int64_t)b * p.q_stride_b + (int64_t)tok_c * p.q_stride_t +
                           (int64_t)head * p.q_stride_h;
    f32x16 qa[RKB];
#pragma unroll
    for (int cb = 0; cb < RKB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) qa[cb][r] = 0.f;
#pragma unroll
    for (int kd = 0; kd < D / 16; ++kd) {
      const bf16x8 bq = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qrow + 16 * kd + 8 * lh));
#pragma unroll
      for (int cb = 0; cb < RKB; ++cb)
        qa[cb] = mfma32(lds_frag(&smem[(32 * cb + ln) * BP + 16 * kd + 8 * lh]), bq, qa[cb]);
    }
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = qa[ks >> 1][8 * (ks & 1) + e] * p.scale_log2e;
      split8(x, qhi[ks], qlo[ks]);
    }
  } else {
    const uint16_t* qrow = p.q + (((int64_t)b * p.T + tok_c) * p.n_q_heads + head) * RK;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const uint4 v = *reinterpret_cast<const uint4*>(qrow + 16 * ks + 8 * lh);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      float x[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        x[2 * e] = bf16_lo(w[e]) * p.scale_log2e;
        x[2 * e + 1] = bf16_hi(w[e]) * p.scale_log2e;
      }
      split8(x, qhi[ks], qlo[ks]);
    }
  }
  // Tiles [0, n_full) are visible to every query row of the workgroup and end before the
  // last cached row; the rest cross the diagonal or the end of the cache.
  int n_full = (p.n_prev + t0 + 1) / KT;
  n_full = n_full < n_tiles_k ? n_full : n_tiles_k;
  auto fetch_k = [&](int tile) {
    if (tile < n_full) load_k(inner_t{}, tile);
    else if (tile < n_tiles_k) load_k(edge_t{}, tile);
  };
  auto fetch_v = [&](int tile) {
    if (tile < n_full) load_v(inner_t{}, tile);
    else if (tile < n_tiles_k) load_v(edge_t{}, tile);
  };
  // LDS: two key stages and two value stages.  Keys run one tile ahead of values: while the
  // softmax and the mix of tile i run, the scores of tile i + 1 are already being computed.
  auto kst = [&](int tile) { return smem + (tile & 1) * STAGE; };
  auto vst = [&](int tile) { return smem + (tile & 1) * STAGE + KT * KP; };
  fetch_k(0);
  __syncthreads();                                      // the basis is no longer needed: stages may be written
  // Value channels that do not exist read as zero -- except the first of them, which reads as one at every
  // key position: its row of the mix is then sum_j p_j, the softmax normaliser, computed by the matrix
  // cores from the very weights the mix uses, and the vector pipe (the bound of this kernel) is spared a
  // row sum of 32 additions per tile.  (Ranks that fill their last 32-channel block keep the additions.)
  constexpr bool kRowSumInMix = RV % 32 != 0;
  if (RV % 32) {
    for (int i = tid; i < 2 * (RVB * 32 - RV) * VP; i += NT) {
      const int s = i / ((RVB * 32 - RV) * VP), o = i % ((RVB * 32 - RV) * VP);
      smem[s * STAGE + KT * KP + RV * VP + o] = (o < KT) ? (uint16_t)0x3F80u : (uint16_t)0u;
    }
  }
  if (PIPE) {
    store_k(kst(0));
    fetch_k(1);
    fetch_v(0);
    __syncthreads();
  } else {
    fetch_v(0);
  }

  // ---- stream the cache ----------------------------------------------------------------
  f32x16 oacc[RVB];
#pragma unroll
  for (int vb = 0; vb < RVB; ++vb)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[vb][r] = 0.f;
  // Scores are accumulated on top of -m (m = the softmax reference, log2 units), held in 16
  // registers that serve as the C operand of each score block's first product, so the
  // subtraction costs nothing.  The reference moves only when a score exceeds it by more
  // than 8: weights stay <= 2^8 and the accumulator rescale leaves the steady state.
  f32x16 negm;
#pragma unroll
  for (int r = 0; r < 16; ++r) negm[r] = 0.f;
  float l_run = 0.f;                                    // this lane's share of the normaliser
  float thr = -INFINITY;                                // first tile: adopt its maximum whatever it is
  f32x16 s_cur[2], s_nxt[2];                            // scores of the tile being mixed / of the next one

  // scores of one tile (two blocks of 32 keys) relative to the reference
  auto scores = [&](auto masked_tag, const uint16_t* ks_s, int j0, f32x16 (&s)[2]) {
    if (PIPE) {                                         // two independent accumulation chains side by side
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          const bf16x8 ka = lds_frag(&ks_s[(32 * a + ln) * KP + 16 * ks + 8 * lh]);
          s[a] = mfma32(ka, qhi[ks], ks == 0 ? negm : s[a]);
          s[a] = mfma32(ka, qlo[ks], s[a]);
        }
      }
    } else {
#pragma unroll
      for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
          const bf16x8 ka = lds_frag(&ks_s[(32 * a + ln) * KP + 16 * ks + 8 * lh]);
          s[a] = mfma32(ka, qhi[ks], ks == 0 ? negm : s[a]);
          s[a] = mfma32(ka, qlo[ks], s[a]);
        }
      }
    }
    if (decltype(masked_tag)::value) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + 32 * a + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (key > limit) s[a][r] = -INFINITY;
        }
    }
  };
  // moves the reference if this tile's scores call for it (rare after the first tile)
  auto adjust = [&](f32x16 (&s)[2]) {
    float mx = s[0][0];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[a][r]);
    mx = max_with_other_half(mx);
    if (__any(mx > thr)) {
      const float dlt = mx > thr ? mx : 0.f;
      const float alpha = thr < 0.f ? 1.f : __builtin_amdgcn_exp2f(-dlt);   // nothing accumulated before the first tile
      l_run *= alpha;
#pragma unroll
      for (int vb = 0; vb < RVB; ++vb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[vb][r] *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) negm[r] -= dlt;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[a][r] -= dlt;
    }
    thr = 8.f;
  };
  // softmax weights of one tile and their mix with its values
  auto mix = [&](const uint16_t* vt_s, const f32x16 (&s)[2]) {
    bf16x8 phi[4], plo[4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = __builtin_amdgcn_exp2f(s[a][8 * kb + e]);
        split8(x, phi[2 * a + kb], plo[2 * a + kb]);
        if (!kRowSumInMix) {
#pragma unroll
          for (int e = 0; e < 8; ++e) l_run += x[e];
        }
      }
    if (PIPE) {
#pragma unroll
      for (int st = 0; st < 4; ++st)
#pragma unroll
        for (int vb = 0; vb < RVB; ++vb) {
          const bf16x8 va = lds_frag(&vt_s[(32 * vb + ln) * VP + 16 * st + 8 * lh]);
          oacc[vb] = mfma32(va, phi[st], oacc[vb]);
          oacc[vb] = mfma32(va, plo[st], oacc[vb]);
        }
    } else {
#pragma unroll
      for (int vb = 0; vb < RVB; ++vb)
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          const bf16x8 va = lds_frag(&vt_s[(32 * vb + ln) * VP + 16 * st + 8 * lh]);
          oacc[vb] = mfma32(va, phi[st], oacc[vb]);
          oacc[vb] = mfma32(va, plo[st], oacc[vb]);
        }
    }
  };
  auto visible = [&](int tile) { return wave_active && tile < n_tiles_k && tile * KT <= p.n_prev + wave_last; };

  if (PIPE) {
    // Keys run one tile ahead of values: the score products of tile it + 1 share a scheduling
    // region with the softmax and the mix products of tile it.
    if (visible(0)) {
      if (n_full > 0) scores(std::false_type{}, kst(0), 0, s_cur); else scores(std::true_type{}, kst(0), 0, s_cur);
      adjust(s_cur);
    }
    int it = 0;
    // steady state: tiles it and it + 1 wholly visible; the scores of tile it are in `cur` on entry, those
    // of tile it + 1 in `nxt` on exit
    auto steady = [&](int it, f32x16 (&cur)[2], f32x16 (&nxt)[2]) {
      store_k(kst(it + 1));
      store_v(vst(it));
      __syncthreads();
      fetch_k(it + 2);
      load_v(inner_t{}, it + 1);
      if (wave_active) {
        scores(std::false_type{}, kst(it + 1), (it + 1) * KT, nxt);
        mix(vst(it), cur);
        adjust(nxt);
      }
    };
    // two tiles per turn with the two score sets changing roles: no copy of 32 registers per tile
    for (; it + 2 < n_full; it += 2) {
      steady(it, s_cur, s_nxt);
      steady(it + 1, s_nxt, s_cur);
    }
    for (; it + 1 < n_full; ++it) {
      steady(it, s_cur, s_nxt);
      if (wave_active) {
        s_cur[0] = s_nxt[0];
        s_cur[1] = s_nxt[1];
      }
    }
    for (; it < n_tiles_k; ++it) {                      // the diagonal and the end of the cache
      if (it + 1 < n_tiles_k) store_k(kst(it + 1));
      store_v(vst(it));
      __syncthreads();
      fetch_k(it + 2);
      fetch_v(it + 1);
      const bool vis_next = visible(it + 1);
      if (vis_next) {
        if (it + 1 < n_full) scores(std::false_type{}, kst(it + 1), (it + 1) * KT, s_nxt);
        else scores(std::true_type{}, kst(it + 1), (it + 1) * KT, s_nxt);
      }
      if (visible(it)) mix(vst(it), s_cur);
      if (vis_next) {
        adjust(s_nxt);
        s_cur[0] = s_nxt[0];
        s_cur[1] = s_nxt[1];
      }
    }
  } else {
    // Keys and values of a tile are staged together; fewer live registers, more waves per SIMD.
    int it = 0;
    for (; it < n_full; ++it) {
      store_k(kst(it));
      store_v(vst(it));
      __syncthreads();
      fetch_k(it + 1);
      fetch_v(it + 1);
      if (wave_active) {
        scores(std::false_type{}, kst(it), it * KT, s_cur);
        adjust(s_cur);
        mix(vst(it), s_cur);
      }
    }
    for (; it < n_tiles_k; ++it) {
      store_k(kst(it));
      store_v(vst(it));
      __syncthreads();
      fetch_k(it + 1);
      fetch_v(it + 1);
      if (visible(it)) {
        scores(std::true_type{}, kst(it), it * KT, s_cur);
        adjust(s_cur);
        mix(vst(it), s_cur);
      }
    }
  }

  if (!wave_active) return;
  // the normaliser of this lane's query row: the two lanes' shares, or (row sum in the mix) the accumulator of
  // channel RV, which is register 8 of the last block in the lane of the lower half
  static_assert(!kRowSumInMix || RV % 32 == 16, "channel RV is expected at row 16 of its block");
  const float l_all = kRowSumInMix ? __shfl(oacc[RVB - 1][8], ln) : l_run + __shfl_xor(l_run, 32);
  const float inv = 1.f / l_all;
  const bool row_ok = tok < p.T;

  if (p.folded) {
    // rank-r_V coordinates: lane holds channels 32 vb + 8 i + 4 lh + (0..3) of its row
    float* orow = p.out + (((int64_t)b * p.T + tok_c) * p.n_q_heads + head) * RV;
#pragma unroll
    for (int vb = 0; vb < RVB; ++vb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = 32 * vb + 8 * i + 4 * lh;
        if (row_ok && c < RV)
          *reinterpret_cast<float4*>(orow + c) = float4{oacc[vb][4 * i] * inv, oacc[vb][4 * i + 1] * inv,
                                                         oacc[vb][4 * i + 2] * inv, oacc[vb][4 * i + 3] * inv};
      }
    return;
  }

  // ---- lift: O^T = P_V A^T --------------------------------------------------------------
  // Contraction step st of the lift covers channels 16 st + 8 (s/4) + 4 lh + s%4 (the order
  // the mix accumulators have them): two 8-byte pieces of a basis row per lane.
  bf16x8 ahi[VSTEPS], alo[VSTEPS];
#pragma unroll
  for (int st = 0; st < VSTEPS; ++st) {
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = oacc[st >> 1][8 * (st & 1) + e] * inv;
    split8(x, ahi[st], alo[st]);
  }
  const uint16_t* pv = p.p_v + (int64_t)kv * p.p_v_head_stride;
  float* orow = p.out + (((int64_t)b * p.T + tok_c) * p.n_q_heads + head) * D;
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    f32x16 o;
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r] = 0.f;
    const uint16_t* prow = pv + (32 * db + ln) * RV;
#pragma unroll
    for (int st = 0; st < VSTEPS; ++st) {
      const uint2 w0 = *reinterpret_cast<const uint2*>(prow + 16 * st + 4 * lh);
      const uint2 w1 = *reinterpret_cast<const uint2*>(prow + 16 * st + 8 + 4 * lh);
      const bf16x8 pa = __builtin_bit_cast(bf16x8, uint4{w0.x, w0.y, w1.x, w1.y});
      o = mfma32(pa, ahi[st], o);
      o = mfma32(pa, alo[st], o);
    }
    if (row_ok) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<float4*>(orow + 32 * db + 8 * i + 4 * lh) =
            float4{o[4 * i], o[4 * i + 1], o[4 * i + 2], o[4 * i + 3]};
    }
  }
}

// Default schedule per shape: where keeping keys a tile ahead measured faster on MI355X
// (chunk of 4096 tokens over 28672 cached rows, ranks 32..128); elsewhere its extra live
// registers cost more than the overlap gains.
constexpr bool pipe_default(int rk, int rv) {
  if (rk <= 32) return true;
  if (rk <= 48) return rv >= 32 && rv <= 112;
  if (rk <= 64) return rv <= 112;
  if (rk <= 80) return rv >= 32 && rv <= 80;
  if (rk <= 96) return rv <= 48;
  if (rk <= 112) return rv == 16 || rv == 48;
  return false;
}

template <int RV, bool PIPE>
hipError_t launch_variant(const PrefillParams& p, hipStream_t stream) {
  const dim3 grid((unsigned)((int64_t)p.n_tiles * p.n_rows_y));
  auto* kernel = prefill_kernel<SKV_RK, RV, PIPE>;
  size_t dyn = 0;
#if SKV_PAGED
  // one table entry per key tile of the longest context of the launch
  dyn = (((size_t)p.n_prev + p.T + KT - 1) / KT * sizeof(int32_t) + 15) & ~(size_t)15;
  if (dyn > 8192) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
    if (e != hipSuccess) return e;
  }
#endif
  hipLaunchKernelGGL(kernel, grid, dim3(NT), dyn, stream, p);
  return hipGetLastError();
}

template <int RV>
hipError_t launch_rv(int sched, const PrefillParams& p, hipStream_t stream) {
  const bool pipe = sched == 1 ? false : sched == 2 ? true : pipe_default(SKV_RK, RV);
  return pipe ? launch_variant<RV, true>(p, stream) : launch_variant<RV, false>(p, stream);
}

}  // namespace

#define SKV_CAT2(a, b) a##b
#define SKV_CAT(a, b) SKV_CAT2(a, b)

#if SKV_PAGED
#define SKV_PREFILL_LAUNCHER SKV_CAT(launch_prefill_paged_rk, SKV_RK)
#else
#define SKV_PREFILL_LAUNCHER SKV_CAT(launch_prefill_rk, SKV_RK)
#endif
hipError_t SKV_PREFILL_LAUNCHER(int r_v, int sched, const PrefillParams& p, hipStream_t stream) {
  switch (r_v) {
    case 16: return launch_rv<16>(sched, p, stream);
    case 32: return launch_rv<32>(sched, p, stream);
    case 48: return launch_rv<48>(sched, p, stream);
    case 64: return launch_rv<64>(sched, p, stream);
    case 80: return launch_rv<80>(sched, p, stream);
    case 96: return launch_rv<96>(sched, p, stream);
    case 112: return launch_rv<112>(sched, p, stream);
    case 128: return launch_rv<128>(sched, p, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace skv
