// The range kernel on the matrix cores.  Included by skv_decode_partial.hip inside its namespaces; uses its
// constants and helpers (format description, fresh-rows workgroups, softmax constants).

// ---------------------------------------------------------------------------------------------------
// The same range on the matrix cores.
//
// With G query heads per KV head the scores and the mix are products of a [G x r] block with the streamed
// rows: 2 G (r_K + r_V) multiply-adds per cache row, which at G = 4 keeps the vector pipe almost as busy as
// the memory system (and, over a quantised cache, busier: there the vector kernel is bound by arithmetic).
// Here both products run as 16x16x16 bf16 matrix instructions with the query heads in 4 of the 16 columns
// (the matrix pipe has two orders of magnitude to spare at this arithmetic intensity), and the vector pipe
// is left with the softmax and the operand conversions.
//
//   S^T [keys x queries]   = K_down [keys x r_K] . Q~^T          A = cache rows as they are loaded
//   O^T [r_V x queries]   += V_down^T [r_V x keys] . P^T         B = 2^(S^T - m): the accumulator layout of the
//                                                                 first product is the B layout of the second
// A wave works on tiles of 32 consecutive rows by itself (wave w of the workgroup takes tiles w, w + 4, ...
// of the range): no workgroup barrier in the loop.  Lane (m = lane % 16, g = lane / 16) loads the g-th
// quarter of key row m of each 16-row block (contiguous), which is the A operand if the contraction index
// is enumerated as channel = g r_K / 4 + 4 step + i; Q~ is laid out to match.  Value rows go through a
// per-wave LDS region, transposed on the way ([channel][key], 8-key runs per 16-byte store), and come back
// as A operands of the second product.  float32 operands (Q~, the weights) are split into two bf16 terms
// (x ~ hi + lo, relative error 2^-17), two products each, so the 2e-3 bound of the vector kernel holds.
//
// Quantised caches (Sec. 4.3).  The integer codes enter the products as they are and the ranges stay
// outside: key scales are already folded into Q~ (the key zero point shifts every score of a query alike
// and drops out); a value row j contributes (p_j scale_j) code_j + p_j zero_j per 64-channel group, i.e.
// the weights of the second product are p_j scale_j (one B operand per group) and sum_j p_j zero_j is kept
// beside the normaliser.
//
// A code needs no conversion at all: the 16-bit pattern 0x00nn IS a bf16 number, n * 2^-133 (subnormal
// below 128, the first normal binade from there on), and the bf16 matrix instructions of this part take
// subnormal inputs at their value.  So one byte-permute per PAIR of codes builds the operand (zero-extend
// two bytes; 4-bit codes after the usual mask / shift-and-mask of a word), where a conversion through
// float32 costs three instructions per pair -- and the vector pipe is what bounds these kernels.  The factor
// 2^-133 is carried by the other operand as far as float32 allows, so that no product leaves the normal
// range: the folded queries are multiplied by 2^100 (scores come out times 2^-33, put right by the one
// multiply-add that also subtracts the softmax reference), and the softmax weights are kept 2^64 above
// their usual size (the reference sits 64 below the running maximum; normaliser, zero sums and partial
// results are all in that convention, which is as valid a partial result as any), the last 2^133 going
// onto the mix once, before it is written.  What this asks of the data: the products of the leading weights,
// 2^64 .. 2^72 times a row's value scale times a code times 2^-133, must be normal float32 numbers, i.e. value
// scales between about 2^-50 and 2^50 (ranges from 1e-13 to 1e17 at 8 bits) -- far outside what a projected
// activation spans, and tested over 2^-20 .. 2^20 times the usual ranges.
// ---------------------------------------------------------------------------------------------------
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x4 mfma16(uint2 a, uint2 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// x minus one half of a bf16 pair in one instruction: the two-element dot product of the pair with (-1, -0)
// or (-0, -1), accumulated onto x.  The difference of a float32 number and its own bf16 head is a float32
// number, so the result is the float32 subtraction's bit for bit (checked on the GPU).  The multipliers carry
// -0, not +0: (-1, +0) is the pattern of an inline constant, and in that form the instruction was seen to
// subtract both halves.
__device__ __forceinline__ float minus_low_half(uint32_t pair, float x) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair), __builtin_bit_cast(bf16x2_t, 0x8000bf80u), x, false);
}
__device__ __forceinline__ float minus_high_half(uint32_t pair, float x) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair), __builtin_bit_cast(bf16x2_t, 0xbf808000u), x, false);
}
// four float32 -> bf16 heads and bf16 remainders, packed as matrix operands
__device__ __forceinline__ void split4(const float (&x)[4], uint2& hi, uint2& lo) {
  hi.x = pack_bf16_pair(x[0], x[1]);
  hi.y = pack_bf16_pair(x[2], x[3]);
  lo.x = pack_bf16_pair(minus_low_half(hi.x, x[0]), minus_high_half(hi.x, x[1]));
  lo.y = pack_bf16_pair(minus_low_half(hi.y, x[2]), minus_high_half(hi.y, x[3]));
}
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
// the 32-deep form: lane (m, g) supplies A[m][8 g .. 8 g + 7] and B[8 g .. 8 g + 7][n]; per multiply-add it
// occupies the matrix pipe about a third as long as the 16-deep one (measured), which matters where the
// kernel is bound by instruction issue (the quantised caches)
__device__ __forceinline__ f32x4 mfma16w(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
__device__ __forceinline__ void split8w(const float (&x)[8], uint4& hi, uint4& lo) {
  uint2 h0, l0, h1, l1;
  const float a[4] = {x[0], x[1], x[2], x[3]}, b[4] = {x[4], x[5], x[6], x[7]};
  split4(a, h0, l0);
  split4(b, h1, l1);
  hi = uint4{h0.x, h0.y, h1.x, h1.y};
  lo = uint4{l0.x, l0.y, l1.x, l1.y};
}
// Integer codes as bf16 operands: the pattern 0x00nn is the bf16 number n * 2^-133.
// byte N of lo into byte 0 and byte N of hi into byte 2 of the result, zeros between: one byte-permute
// (selector bytes: 0..3 pick from lo, 4..7 from hi, 0x0c gives zero)
template <int N>
__device__ __forceinline__ uint32_t byte_pair(uint32_t lo, uint32_t hi) {
  return __builtin_amdgcn_perm(hi, lo, 0x0c000c00u | (uint32_t)N | ((uint32_t)(4 + N) << 16));
}
// bytes 2 H and 2 H + 1 of a word, each zero-extended to 16 bits
template <int H>
__device__ __forceinline__ uint32_t byte_pair_of_word(uint32_t w) {
  return __builtin_amdgcn_perm(0u, w, H == 0 ? 0x0c010c00u : 0x0c030c02u);
}
[[maybe_unused]] constexpr float kKeyUp = 0x1p100f;          // on the folded queries
[[maybe_unused]] constexpr float kScoreBack = 0x1p33f;       // 2^133 / kKeyUp, on the scores
[[maybe_unused]] constexpr float kWeightBias = 64.f;         // log2 of what the softmax weights carry
[[maybe_unused]] constexpr float kMixBackA = 0x1p66f, kMixBackB = 0x1p67f;   // 2^133 in two steps, on the mix

#ifndef SKV_MMA_DEPTH
#define SKV_MMA_DEPTH 1          // register sets per wave: tiles it has requested or is working on (1 or 2)
#endif
constexpr int kMmaTileRows = 32;                 // rows a wave takes at a time
constexpr int kMmaVPitch = kMmaTileRows + 8;     // LDS pitch of a value channel (bf16 elements; 80 bytes)

// An empty statement that the compiler keeps in its place among the memory requests, and through which a
// requested word passes: whatever needs the word is scheduled after the requests that precede the statement.
__device__ __forceinline__ void keep_after_requests(float& x) { asm volatile("" : "+v"(x) : : "memory"); }
__device__ __forceinline__ void keep_after_requests(uint32_t& x) { asm volatile("" : "+v"(x) : : "memory"); }

// Workgroups per CU the register allocation is held to.  Two at least: the allocator then works within 256
// registers per lane, all of them ordinary ones.  Four (128 registers) over a quantised cache with both ranks
// up to 64, where the kernel is bound by the latency of its chain of dependent steps and the fourth wave per
// SIMD is worth more than the two registers it costs to stay under the line (larger ranks would spill; with
// eight heads a pass the workgroup's LDS allows three per CU anyway).
constexpr int mma_min_workgroups(int rk, int rv, int gt) { return (SKV_Q8 && rk <= 64 && rv <= 64 && gt <= 4) ? 4 : 2; }

template <int RK, int RV, int GT, int FMT, bool NT>
__global__ __launch_bounds__(kDecodeThreads, mma_min_workgroups(RK, RV, GT)) void decode_partial_mma_kernel(const DecodeParams p) {
  static_assert(FMT == kFmt, "format tag must match the build");
  // Quantised builds (ranks are multiples of 32 there) use the 32-deep matrix instruction: the contraction index
  // of the first product is then enumerated as channel = g r_K / 4 + 8 step + i, and the 32 rows of a tile are
  // ONE contraction of the second product, position 8 g + 4 b + i standing for row 16 b + 4 g + i (the rows whose
  // scores lane (n, g) holds after the first product).
  constexpr bool WIDE = SKV_Q8 != 0;
  static_assert(!WIDE || RK % 32 == 0, "the 32-deep form needs ranks that are multiples of 32");
  constexpr int KSTEPS = WIDE ? RK / 32 : RK / 16;   // contraction steps of the score product
  constexpr int VBLOCKS = RV / 16;               // 16-channel blocks of the mix
  constexpr int NG = (RV + 63) / 64;             // 64-channel groups of a value row (quantisation groups)
  // raw words per lane: a quarter of a key row per 16-row block; value tiles as units of VROWS rows by one
  // word (8 rows; 4 with 4-bit codes, whose words hold 8 channels: every lane then has a unit at r_V = 64)
  constexpr int KRAW = RK / 4 / kElemsPerDword;  // bf16: RK / 8, 8-bit: RK / 16, 4-bit: RK / 32
  constexpr int VWORDS = RV / kElemsPerDword;    // words in a value row
  constexpr int VROWS = SKV_QBITS == 4 ? 4 : 8;
  constexpr int VUNITS = (kMmaTileRows / VROWS) * VWORDS;
  constexpr int VPL = (VUNITS + 63) / 64;        // units per lane
  constexpr int VP = kMmaVPitch;
  static_assert(KRAW >= 1 && (RK / 4) % kElemsPerDword == 0, "rank not supported by this format");

  // The projection scratch is needed before the first tile only, the value tiles after it: one region.
  constexpr int kProjBytes = kProjectThreads * (GT < 4 ? GT : 4) * 8 * (int)sizeof(float);
  constexpr int kTileBytes = 4 * RV * VP * (int)sizeof(uint16_t);           // per wave: value tile, [channel][row]
  __shared__ __attribute__((aligned(16))) unsigned char scratch_s[kProjBytes > kTileBytes ? kProjBytes : kTileBytes];
  constexpr int kWaveTileBytes = RV * VP * (int)sizeof(uint16_t);
  static_assert(GT * (RV + 2) * (int)sizeof(float) <= kWaveTileBytes, "a wave's merge slots must fit in its value tile");
  __shared__ float px_s[GT * SKV_HEAD_DIM];
  __shared__ float py_s[GT * SKV_HEAD_DIM];
  float* ppart_s = reinterpret_cast<float*>(scratch_s);

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int lm = lane & 15;                      // row of a 16-row block (first product), channel (second), query column
  const int g = lane >> 4;

  int split = blockIdx.x;
  const int passes = p.group / GT;
  int col = blockIdx.y;
  const int n_cols = p.batch * p.n_kv_heads * passes;
  const bool fresh = col >= n_cols;              // the fresh-rows workgroups of a fused decode step
  if (fresh) {
    col = (col - n_cols) * (int)gridDim.x + split;
    if (col >= n_cols) return;
    split = p.n_stream;
  }
  const int pass = col % passes;
  const int bkv = col / passes;
  const int kv = bkv % p.n_kv_heads;
  const int b = bkv / p.n_kv_heads;
  const int hq0 = kv * p.group + pass * GT;
  if (fresh) {
#if SKV_Q8
    fresh_rows_block_q<RK, RV, GT>(p, b, kv, pass, hq0, px_s, ppart_s, py_s);
#else
    fresh_rows_block<RK, RV, GT>(p, b, kv, pass, hq0, px_s, ppart_s, py_s);
#endif
    return;
  }
  int t0, t1;
  const int seq_rows = (int)clamped_len(p.seq_lens, b, p.n_ctx - p.len_add) + p.len_add;
  range_of_split(seq_rows, p.n_stream, split, &t0, &t1);
  // whole tiles front to back for an even number of rows in the sequence, back to front for an odd one: the
  // same rule, for the same reason, as in the vector kernel (consecutive decode steps sweep the cache in
  // opposite directions and meet first what a last-level cache still holds)
  const bool backwards = (seq_rows & 1) != 0;

  float* out_acc = p.part_acc + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + split) * RV;
  float* out_ml = p.part_ml + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + split) * 2;
  const int64_t head_step_acc = (int64_t)p.n_splits * RV;
  const int64_t head_step_ml = (int64_t)p.n_splits * 2;
  if (t0 >= t1) {
    for (int i = tid; i < GT * RV; i += kDecodeThreads) out_acc[(i / RV) * head_step_acc + (i % RV)] = 0.f;
    if (tid < GT) { out_ml[tid * head_step_ml] = kNegBig; out_ml[tid * head_step_ml + 1] = 0.f; }
    return;
  }

  // ---- where the rows of a tile are ---------------------------------------------------------------
  // rows [row, row + 32) lie in one page (ranges start at multiples of 64, pages hold multiples of 64)
#if SKV_PAGED
  const int page_rows_mask = (1 << p.pages.page_shift) - 1;
  auto tile_base = [&](int row) -> int64_t {                     // index of the tile's first row, in rows
    const int page = clamped_page(p.pages, b, row >> p.pages.page_shift);   // wave-uniform: a scalar load
    return ((((int64_t)page * p.n_kv_heads + kv)) << p.pages.page_shift) + (row & page_rows_mask);
  };
#else
  const int64_t flat0 = ((int64_t)b * p.n_kv_heads + kv) * p.capacity;
  auto tile_base = [&](int row) -> int64_t { return flat0 + row; };
#endif

  // ---- tile loads: key quarters as they lie in memory, values as (8 rows x one word) units ----------------
  // Whole tiles first, each wave its own (wave w: tiles w, w + 4, ...); rows left over at the end of the range
  // make one more, partial tile, taken by the wave whose turn it would be, after its whole ones.
  const int n_whole = (t1 - t0) / kMmaTileRows;
  const bool has_tail = (t1 - t0) % kMmaTileRows != 0;
  struct TileRegsM {
    uint32_t k[2][KRAW];
    uint32_t v[VPL][VROWS];
#if SKV_Q8
    uint32_t vm[NG][2][4];                       // (scale | zero << 16) of rows 16 kb + 4 g + i, per group
#endif
  };
  // A whole tile: one address per stream and lane, the rest are constant offsets; streaming or ordinary loads
  // as the launch asks (NT).  Nothing here depends on a condition: the loop below relies on every request of a
  // tile being the same run of instructions (see there).
  auto issue_whole = [&](int tile, TileRegsM& tr) {
    const int row0 = t0 + (backwards ? n_whole - 1 - tile : tile) * kMmaTileRows;
    const int64_t base = tile_base(row0);
    {
      {
        const uint32_t* ksrc = p.k_cache + (base + lm) * (RK / kElemsPerDword) + g * KRAW;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const uint32_t* src = ksrc + 16 * kb * (RK / kElemsPerDword);
          if constexpr (KRAW % 4 == 0) {
#pragma unroll
            for (int k4 = 0; k4 < KRAW / 4; ++k4) {
              const u32x4 w = load_cache<NT>(reinterpret_cast<const u32x4*>(src + 4 * k4));
              tr.k[kb][4 * k4] = w.x; tr.k[kb][4 * k4 + 1] = w.y; tr.k[kb][4 * k4 + 2] = w.z; tr.k[kb][4 * k4 + 3] = w.w;
            }
          } else if constexpr (KRAW % 2 == 0) {
#pragma unroll
            for (int k2 = 0; k2 < KRAW / 2; ++k2) {
              const u32x2 w = load_cache<NT>(reinterpret_cast<const u32x2*>(src + 2 * k2));
              tr.k[kb][2 * k2] = w.x; tr.k[kb][2 * k2 + 1] = w.y;
            }
          } else {
#pragma unroll
            for (int k1 = 0; k1 < KRAW; ++k1) tr.k[kb][k1] = load_cache<NT>(src + k1);
          }
        }
#pragma unroll
        for (int u = 0; u < VPL; ++u) {
          const int i = lane + 64 * u;
          if (VUNITS % 64 == 0 || i < VUNITS) {
            const int cw = i % VWORDS, kg = i / VWORDS;
            const uint32_t* vsrc = p.v_cache + (base + VROWS * kg) * VWORDS + cw;
#pragma unroll
            for (int e = 0; e < VROWS; ++e) tr.v[u][e] = load_cache<NT>(vsrc + e * VWORDS);
          }
        }
#if SKV_Q8
        const uint32_t* msrc = p.v_meta + (base + 4 * g) * NG;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int gq = 0; gq < NG; ++gq) tr.vm[gq][kb][i] = load_cache<NT>(msrc + (16 * kb + i) * NG + gq);
#endif
      }
    }
  };
  // The partial tile at the end of the range: rows past the last one re-read it; their weights are zero.
  auto issue_tail = [&](TileRegsM& tr) {
    const int row0 = t0 + n_whole * kMmaTileRows;
    const int64_t base = tile_base(row0);
    const int last = t1 - 1 - row0;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      int r = 16 * kb + lm;
      r = r < last ? r : last;
      const uint32_t* src = p.k_cache + (base + r) * (RK / kElemsPerDword) + g * KRAW;
      if constexpr (KRAW % 4 == 0) {
#pragma unroll
        for (int k4 = 0; k4 < KRAW / 4; ++k4) {
          const uint4 w = *reinterpret_cast<const uint4*>(src + 4 * k4);
          tr.k[kb][4 * k4] = w.x; tr.k[kb][4 * k4 + 1] = w.y; tr.k[kb][4 * k4 + 2] = w.z; tr.k[kb][4 * k4 + 3] = w.w;
        }
      } else if constexpr (KRAW % 2 == 0) {
#pragma unroll
        for (int k2 = 0; k2 < KRAW / 2; ++k2) {
          const uint2 w = *reinterpret_cast<const uint2*>(src + 2 * k2);
          tr.k[kb][2 * k2] = w.x; tr.k[kb][2 * k2 + 1] = w.y;
        }
      } else {
#pragma unroll
        for (int k1 = 0; k1 < KRAW; ++k1) tr.k[kb][k1] = src[k1];
      }
    }
#pragma unroll
    for (int u = 0; u < VPL; ++u) {
      const int i = lane + 64 * u;
      if (VUNITS % 64 == 0 || i < VUNITS) {
        const int cw = i % VWORDS, kg = i / VWORDS;
#pragma unroll
        for (int e = 0; e < VROWS; ++e) {
          int r = VROWS * kg + e;
          r = r < last ? r : last;
          tr.v[u][e] = p.v_cache[(base + r) * VWORDS + cw];
        }
      }
    }
#if SKV_Q8
#pragma unroll
    for (int gq = 0; gq < NG; ++gq)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          int r = 16 * kb + 4 * g + i;
          r = r < last ? r : last;
          tr.vm[gq][kb][i] = p.v_meta[(base + r) * NG + gq];
        }
#endif
  };
  // the A operand of contraction step ks of key block kb
#if SKV_QBITS == 8
  auto key_operand = [&](const TileRegsM& tr, int kb, int ks) -> uint4 {
    const uint32_t w0 = tr.k[kb][2 * ks], w1 = tr.k[kb][2 * ks + 1];   // 8 codes
    return uint4{byte_pair_of_word<0>(w0), byte_pair_of_word<1>(w0), byte_pair_of_word<0>(w1), byte_pair_of_word<1>(w1)};
  };
#elif SKV_QBITS == 4
  auto key_operand = [&](const TileRegsM& tr, int kb, int ks) -> uint4 {
    const uint32_t w = tr.k[kb][ks];                             // 8 codes: the even channel in the low half of a byte
    const uint32_t ev = w & 0x0f0f0f0fu, od = (w >> 4) & 0x0f0f0f0fu;
    return uint4{byte_pair<0>(ev, od), byte_pair<1>(ev, od), byte_pair<2>(ev, od), byte_pair<3>(ev, od)};
  };
#else
  auto key_operand = [&](const TileRegsM& tr, int kb, int ks) -> uint2 {
    return make_uint2(tr.k[kb][2 * ks], tr.k[kb][2 * ks + 1]);
  };
#endif
  // the value tile into this wave's LDS region as bf16, transposed: channel c, rows 8 kg .. 8 kg + 7 as one 16-byte run
  uint16_t* vt = reinterpret_cast<uint16_t*>(scratch_s) + wave * (RV * VP);
  auto store_values = [&](const TileRegsM& tr) {
#pragma unroll
    for (int u = 0; u < VPL; ++u) {
      const int i = lane + 64 * u;
      if (VUNITS % 64 == 0 || i < VUNITS) {
        const int cw = i % VWORDS, kg = i / VWORDS;
#if SKV_QBITS == 8
        // a word holds channels 4 cw .. 4 cw + 3 of one row
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint32_t o[4];
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            // channel c of rows 2 e2 and 2 e2 + 1: the same byte of two words
            const uint32_t w0 = tr.v[u][2 * e2], w1 = tr.v[u][2 * e2 + 1];
            o[e2] = c == 0 ? byte_pair<0>(w0, w1) : c == 1 ? byte_pair<1>(w0, w1) : c == 2 ? byte_pair<2>(w0, w1) : byte_pair<3>(w0, w1);
          }
          uint16_t* dst = vt + (4 * cw + c) * VP + 16 * (kg & 1) + 4 * (kg >> 1);   // rows 8 kg + e at 16 (kg % 2) + 8 (e / 4) + 4 (kg / 2) + e % 4
          *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1]);
          *reinterpret_cast<uint2*>(dst + 8) = make_uint2(o[2], o[3]);
        }
#elif SKV_QBITS == 4
        // a word holds channels 8 cw .. 8 cw + 7 of one row: even ones in the low halves of its bytes; the
        // unit is rows 4 kg .. 4 kg + 3
        uint32_t ev[4], od[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ev[e] = tr.v[u][e] & 0x0f0f0f0fu;
          od[e] = (tr.v[u][e] >> 4) & 0x0f0f0f0fu;
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          uint32_t o[2];
#pragma unroll
          for (int e2 = 0; e2 < 2; ++e2) {
            const uint32_t a = (c & 1) ? od[2 * e2] : ev[2 * e2], bb = (c & 1) ? od[2 * e2 + 1] : ev[2 * e2 + 1];
            // channel c of rows 2 e2 and 2 e2 + 1: the same byte of two words, picked by one byte-permute
            o[e2] = (c >> 1) == 0 ? byte_pair<0>(a, bb) : (c >> 1) == 1 ? byte_pair<1>(a, bb)
                  : (c >> 1) == 2 ? byte_pair<2>(a, bb) : byte_pair<3>(a, bb);
          }
          // rows 4 kg + e at 16 ((kg / 2) % 2) + 8 (kg % 2) + 4 (kg / 4) + e: the 8-bit layout, half a unit each
          uint16_t* dst = vt + (8 * cw + c) * VP + 16 * ((kg >> 1) & 1) + 8 * (kg & 1) + 4 * (kg >> 2);
          *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1]);
        }
#else
        // a word holds channels 2 cw, 2 cw + 1 of one row
        uint4 even, odd;
        even.x = __builtin_amdgcn_perm(tr.v[u][1], tr.v[u][0], 0x05040100u);
        even.y = __builtin_amdgcn_perm(tr.v[u][3], tr.v[u][2], 0x05040100u);
        even.z = __builtin_amdgcn_perm(tr.v[u][5], tr.v[u][4], 0x05040100u);
        even.w = __builtin_amdgcn_perm(tr.v[u][7], tr.v[u][6], 0x05040100u);
        odd.x = __builtin_amdgcn_perm(tr.v[u][1], tr.v[u][0], 0x07060302u);
        odd.y = __builtin_amdgcn_perm(tr.v[u][3], tr.v[u][2], 0x07060302u);
        odd.z = __builtin_amdgcn_perm(tr.v[u][5], tr.v[u][4], 0x07060302u);
        odd.w = __builtin_amdgcn_perm(tr.v[u][7], tr.v[u][6], 0x07060302u);
        *reinterpret_cast<uint4*>(vt + (2 * cw) * VP + 8 * kg) = even;
        *reinterpret_cast<uint4*>(vt + (2 * cw + 1) * VP + 8 * kg) = odd;
#endif
      }
    }
  };

  // ---- projected queries as B operands: column lm is query head lm of the pass (zero beyond GT) ---------
  // Requests return in order and are waited for by count.  The waits the compiler places are exact only if,
  // wherever paths join, every path has made the same requests in the same order; otherwise a wait for one
  // tile becomes a wait for everything.  So in the loop over whole tiles every request is the same straight
  // run of loads and is made every time: a wave that has run out of tiles requests the range's last whole one
  // again and never looks at it.  First come the few words the queries need (from the workspace, or the basis
  // pieces and raw queries of the in-kernel projection), then the wave's first SKV_MMA_DEPTH tiles.
  // One register set per wave is the default.  Two (SKV_MMA_DEPTH = 2; the waits then leave the other set's
  // 20 requests in flight, checked in the generated code) measured no faster anywhere: b4/32K 64/64 from HBM,
  // bf16 46.9 against 45.6 us; 8-bit codes 27.2 us (three waves per SIMD for the registers) against 25.0.
  // The kernels are not short of bytes in flight.
  TileRegsM ta;
  const bool from_workspace = p.q == nullptr;
  constexpr int QW = SKV_Q8 ? 8 : 4;                              // query channels per contraction step and lane
  const int lmq = lm < GT ? lm : 0;                               // a lane beyond the pass's heads reads head 0 and keeps zero
  float xq[KSTEPS][QW];
  ProjectPieces pp;
  constexpr int kQElems = GT * SKV_HEAD_DIM;
  constexpr int kQPerLane = (kQElems + kDecodeThreads - 1) / kDecodeThreads;
  uint32_t qraw[kQPerLane];                                      // one raw query element each, in a register of its own
  if (from_workspace) {
    // already scaled (and, quantised, times the key scales)
    const float* qt = p.qt + ((int64_t)b * p.n_q_heads + hq0) * RK + lmq * RK + g * (RK / 4);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
      for (int i = 0; i < QW; ++i) xq[ks][i] = qt[QW * ks + i];
  } else {
    project_rows_issue(p.p_k + (int64_t)kv * p.p_k_head_stride, RK, pp);
    const uint16_t* qptr = p.q + ((int64_t)b * p.n_q_heads + hq0) * SKV_HEAD_DIM;
#pragma unroll
    for (int k = 0; k < kQPerLane; ++k) qraw[k] = qptr[(tid + k * kDecodeThreads) % kQElems];
  }
  // Queries projected here: the projection's few words (basis pieces, raw queries) are waited for BEFORE the
  // tiles go out -- every workgroup of the launch starts at the same moment, and behind the whole chip's
  // first tiles those words took 3-5 us to arrive; the tiles then stream while the projection runs.
  // (SKV_MMA_WORDS_FIRST = 0 sends the tiles after the words without waiting: 47.1 against 45.9 us per call at
  // b4/32K 64/64, level over the quantised caches)
#ifndef SKV_MMA_WORDS_FIRST
#define SKV_MMA_WORDS_FIRST 1
#endif
  if (SKV_MMA_WORDS_FIRST && !from_workspace) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  auto clamped_tile = [&](int tile) { return tile < n_whole ? tile : n_whole - 1; };
#if SKV_MMA_DEPTH == 2
  TileRegsM tb;
#endif
  if (n_whole > 0) {                                             // (the same for all waves of the workgroup)
    issue_whole(clamped_tile(wave), ta);
#if SKV_MMA_DEPTH == 2
    issue_whole(clamped_tile(wave + 4), tb);
#endif
  }
  // Nothing that needs the words requested above may be scheduled ahead of the tile's requests (an empty
  // statement the compiler must keep in place, through which those words pass).
  if (from_workspace) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
      for (int i = 0; i < QW; ++i) keep_after_requests(xq[ks][i]);
  } else {
#pragma unroll
    for (int k = 0; k < kQPerLane; ++k) keep_after_requests(qraw[k]);
  }
  float qscale = 1.f;
  if (!from_workspace) {
#pragma unroll
    for (int k = 0; k < kQPerLane; ++k)
      if (tid + k * kDecodeThreads < kQElems) px_s[tid + k * kDecodeThreads] = bf16_to_f32((uint16_t)qraw[k]);
    __syncthreads();
    project_query_rows<GT>(pp, RK, px_s, ppart_s, py_s);
    const float* qh = py_s + lmq * RK + g * (RK / 4);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
      for (int i = 0; i < QW; ++i) xq[ks][i] = qh[QW * ks + i];
    qscale = p.scale_log2e;
  }
  // quantised keys: <q~, code * scale + zero> = <q~ * scale, code> + const; the constant drops out of the softmax
  // (queries taken from the workspace carry the key scales already)
#if SKV_Q8
  auto key_scale_of = [&](int channel) -> float {
    return from_workspace ? 1.f : p.k_scale[kv * ((RK + 63) / 64) + (channel >> 6)];
  };
  uint4 qhi[KSTEPS], qlo[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = lm < GT ? xq[ks][i] * qscale * key_scale_of(g * (RK / 4) + 8 * ks + i) * kKeyUp : 0.f;
    split8w(x, qhi[ks], qlo[ks]);
  }
#else
  uint2 qhi[KSTEPS], qlo[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    float x[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = lm < GT ? xq[ks][i] * qscale : 0.f;
    split4(x, qhi[ks], qlo[ks]);
  }
#endif

  // ---- stream this wave's tiles -------------------------------------------------------------------
  // Per lane: query column lm, rows 4 g + i of each 16-row block.  m_ref is the softmax reference of the
  // column (log2 units; the same in the four lanes of a column), l this lane's share of the normaliser,
  // zsum (quantised) its share of sum_j p_j zero_j per group.
  float m_ref = 0.f, l = 0.f;
  float zsum[NG];
#pragma unroll
  for (int gq = 0; gq < NG; ++gq) zsum[gq] = 0.f;
  bool first = true;
  f32x4 oacc[VBLOCKS];
#pragma unroll
  for (int cb = 0; cb < VBLOCKS; ++cb) oacc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // A tile in two parts, between which its register set is free for the next request.
  // Part one: scores minus the reference (the reference rides in as the initial accumulator), the values into
  // LDS, the rows' value ranges unpacked.
  f32x4 sc[2];
#if SKV_Q8
  float vscale[NG][2][4], vzero[NG][2][4];
#endif
  auto scores_and_values = [&](const TileRegsM& tr) {
    // (the two 16-row blocks take turns, so that a product never waits for the one just issued)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) sc[kb] = SKV_Q8 ? f32x4{0.f, 0.f, 0.f, 0.f} : f32x4{-m_ref, -m_ref, -m_ref, -m_ref};
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
#if SKV_Q8
      const uint4 a0 = key_operand(tr, 0, ks), a1 = key_operand(tr, 1, ks);
      sc[0] = mfma16w(a0, qhi[ks], sc[0]);
      sc[1] = mfma16w(a1, qhi[ks], sc[1]);
      sc[0] = mfma16w(a0, qlo[ks], sc[0]);
      sc[1] = mfma16w(a1, qlo[ks], sc[1]);
#else
      const uint2 a0 = key_operand(tr, 0, ks), a1 = key_operand(tr, 1, ks);
      sc[0] = mfma16(a0, qhi[ks], sc[0]);
      sc[1] = mfma16(a1, qhi[ks], sc[1]);
      sc[0] = mfma16(a0, qlo[ks], sc[0]);
      sc[1] = mfma16(a1, qlo[ks], sc[1]);
#endif
    }
#if SKV_Q8
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 4; ++i) sc[kb][i] = fmaf(sc[kb][i], kScoreBack, -m_ref);
#endif
    store_values(tr);
#if SKV_Q8
#pragma unroll
    for (int gq = 0; gq < NG; ++gq)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          vscale[gq][kb][i] = bf16_lo(tr.vm[gq][kb][i]);
          vzero[gq][kb][i] = bf16_hi(tr.vm[gq][kb][i]);
        }
#endif
    __builtin_amdgcn_wave_barrier();
  };
  // Part two: softmax weights of the tile's rows and their mix with its values.
  auto weights_and_mix = [&](int row0, bool partial) {
    // rows past the end of the range do not count
    if (partial) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (row0 + 16 * kb + 4 * g + i >= t1) sc[kb][i] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                     fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    // over the four lanes of a column (16 and 32 apart): two vector lane swaps, not two trips through the LDS
    // pipeline -- this maximum sits in the middle of the tile's chain of dependent steps
    mx = halves_pair(rows_pair(mx, true), true);
    // (over a quantised cache the reference is held kWeightBias below where it would be: the weights are
    // that much larger, up to 2^(slack + bias))
    constexpr float kBias = SKV_Q8 ? kWeightBias : 0.f;
    if (first || mx > kRescaleSlack + kBias) {                   // the reference moves (lanes of a column agree)
      const float d = mx - kBias;
      const float f = first ? 0.f : fast_exp2(-d);
      m_ref = first ? d : m_ref + d;
      l *= f;
#pragma unroll
      for (int gq = 0; gq < NG; ++gq) zsum[gq] *= f;
#pragma unroll
      for (int cb = 0; cb < VBLOCKS; ++cb) oacc[cb] *= f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) sc[kb] -= d;
    }
    first = false;
    // the weights as B operands: one pair per 64-channel group when rows carry their own value scales
#if SKV_Q8
    float x[2][4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[kb][i] = fast_exp2(sc[kb][i]);
        l += x[kb][i];
      }
    uint4 phi[NG], plo[NG];
#pragma unroll
    for (int gq = 0; gq < NG; ++gq) {
      float xs[8];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          xs[4 * kb + i] = x[kb][i] * vscale[gq][kb][i];
          zsum[gq] = fmaf(x[kb][i], vzero[gq][kb][i], zsum[gq]);
        }
      split8w(xs, phi[gq], plo[gq]);
    }
    uint4 va[VBLOCKS];
#pragma unroll
    for (int cb = 0; cb < VBLOCKS; ++cb) va[cb] = *reinterpret_cast<const uint4*>(vt + (16 * cb + lm) * VP + 8 * g);
#pragma unroll
    for (int cb = 0; cb < VBLOCKS; ++cb) oacc[cb] = mfma16w(va[cb], phi[(16 * cb) / 64], oacc[cb]);
#pragma unroll
    for (int cb = 0; cb < VBLOCKS; ++cb) oacc[cb] = mfma16w(va[cb], plo[(16 * cb) / 64], oacc[cb]);
#else
    uint2 phi[2], plo[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      float x[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[i] = fast_exp2(sc[kb][i]);
        l += x[i];
      }
      split4(x, phi[kb], plo[kb]);
    }
#pragma unroll
    for (int cb = 0; cb < VBLOCKS; ++cb)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const uint2 a = *reinterpret_cast<const uint2*>(vt + (16 * cb + lm) * VP + 16 * kb + 4 * g);
        oacc[cb] = mfma16(a, phi[kb], oacc[cb]);
        oacc[cb] = mfma16(a, plo[kb], oacc[cb]);
      }
#endif
    __builtin_amdgcn_wave_barrier();
  };
  // One whole tile from register set tr, if the wave still has one (wave-uniform); next_tile (or the last
  // whole tile again) is requested into the set as soon as it is free.
  auto step = [&](int tile, TileRegsM& tr, int next_tile) {
    const bool valid = tile < n_whole;
    if (valid) scores_and_values(tr);
    issue_whole(clamped_tile(next_tile), tr);
    if (valid) weights_and_mix(t0 + tile * kMmaTileRows, false);
  };
  if (n_whole > 0) {
#if SKV_MMA_DEPTH == 2
    for (int tile = wave; tile < n_whole; tile += 8) {
      step(tile, ta, tile + 8);
      step(tile + 4, tb, tile + 12);
    }
#else
    for (int tile = wave; tile < n_whole; tile += 4) step(tile, ta, tile + 4);
#endif
  }
  if (has_tail && wave == (n_whole & 3)) {
    issue_tail(ta);
    scores_and_values(ta);
    weights_and_mix(t0 + n_whole * kMmaTileRows, true);
  }

  // ---- the four lanes of a column hold shares of l (and of the zero sums); then merge the 4 waves through
  //      LDS, in wave order.  A wave's results go where its value tiles were: it has read the last of them
  //      (its own LDS operations complete in order), and no other wave touches that region before the barrier.
  auto wave_red = [&](int w) -> float* { return reinterpret_cast<float*>(scratch_s + w * kWaveTileBytes); };
  l = halves_pair(rows_pair(l, false), false);
#if SKV_Q8
#pragma unroll
  for (int gq = 0; gq < NG; ++gq) {
    zsum[gq] = halves_pair(rows_pair(zsum[gq], false), false);
  }
#endif
  if (lm < GT) {
    float* r = wave_red(wave) + lm * (RV + 2);
#pragma unroll
    for (int cb = 0; cb < VBLOCKS; ++cb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float a = oacc[cb][i];
        // codes were taken as n * 2^-133; every channel of a group receives the group's zero sum
        if (SKV_Q8) a = fmaf(a * kMixBackA, kMixBackB, zsum[(16 * cb) / 64]);
        r[16 * cb + 4 * g + i] = a;
      }
    if (g == 0) {
      r[RV] = first ? kNegBig : m_ref;                           // a wave without tiles: the neutral element
      r[RV + 1] = l;
    }
  }
  __syncthreads();
  for (int i = tid; i < GT * (RV + 2); i += kDecodeThreads) {
    const int hg = i / (RV + 2), c = i % (RV + 2);
    float mt = wave_red(0)[hg * (RV + 2) + RV];
#pragma unroll
    for (int w = 1; w < 4; ++w) mt = fmaxf(mt, wave_red(w)[hg * (RV + 2) + RV]);
    if (c == RV) {
      out_ml[hg * head_step_ml] = mt;
    } else {
      const int src = c == RV + 1 ? RV + 1 : c;
      float a = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float* r = wave_red(w) + hg * (RV + 2);
        a += r[src] * fast_exp2(r[RV] - mt);
      }
      if (c == RV + 1) out_ml[hg * head_step_ml + 1] = a;
      else out_acc[hg * head_step_acc + c] = a;
    }
  }
}
