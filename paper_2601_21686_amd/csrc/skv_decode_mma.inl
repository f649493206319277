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
// Quantised caches (Sec. 4.3).  Integer codes are exact in bf16, so they enter the products as they are
// and the ranges stay outside: key scales are already folded into Q~ (the key zero point shifts every
// score of a query alike and drops out); a value row j contributes (p_j scale_j) code_j + p_j zero_j per
// 64-channel group, i.e. the weights of the second product are p_j scale_j (one B operand per group) and
// sum_j p_j zero_j is kept beside the normaliser.  8-bit codes are converted byte by byte
// (v_cvt_f32_ubyteN, then the high halves of two results packed).  4-bit codes n become the bf16 number
// 16 + n, whose bit pattern is 0x4180 + 8 n (one shift-or per pair): for keys the extra 16 sum_c q~_c is
// one more constant per query; for values it is taken back through the zero term (zero_j - 16 scale_j).
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
// four float32 -> bf16 heads and bf16 remainders, packed as matrix operands
__device__ __forceinline__ void split4(const float (&x)[4], uint2& hi, uint2& lo) {
  hi.x = pack_bf16_pair(x[0], x[1]);
  hi.y = pack_bf16_pair(x[2], x[3]);
  lo.x = pack_bf16_pair(x[0] - bf16_lo(hi.x), x[1] - bf16_hi(hi.x));
  lo.y = pack_bf16_pair(x[2] - bf16_lo(hi.y), x[3] - bf16_hi(hi.y));
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
// the high halves of two float32 numbers as a bf16 pair (exact when both are bf16 numbers already)
__device__ __forceinline__ uint32_t high_halves(float lo, float hi) {
  return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}
template <int N>
__device__ __forceinline__ float byte_to_f32(uint32_t w) { return (float)((w >> (8 * N)) & 0xffu); }
// two 4-bit codes (bits 0..3 of bytes NL of lo and NH of hi ... see callers) as bf16 numbers 16 + n
[[maybe_unused]] constexpr float kNibbleOffset = 16.f;
__device__ __forceinline__ uint32_t nibbles_to_bf16_pair(uint32_t pair_in_bytes_0_and_2) {
  return (pair_in_bytes_0_and_2 << 3) | 0x41804180u;
}
// byte N of lo into byte 0 and byte N of hi into byte 2 of the result, zeros between: one byte-permute
// (selector bytes: 0..3 pick from lo, 4..7 from hi, 0x0c gives zero)
template <int N>
__device__ __forceinline__ uint32_t byte_pair(uint32_t lo, uint32_t hi) {
  return __builtin_amdgcn_perm(hi, lo, 0x0c000c00u | (uint32_t)N | ((uint32_t)(4 + N) << 16));
}

#ifndef SKV_MMA_DEPTH
#define SKV_MMA_DEPTH 1          // tiles a wave has requested ahead of the one it computes on (1 or 2)
#endif
constexpr int kMmaTileRows = 32;                 // rows a wave takes at a time
constexpr int kMmaVPitch = kMmaTileRows + 8;     // LDS pitch of a value channel (bf16 elements; 80 bytes)

// An empty statement that the compiler keeps in its place among the memory requests, and through which a
// requested word passes: whatever needs the word is scheduled after the requests that precede the statement.
__device__ __forceinline__ void keep_after_requests(float& x) { asm volatile("" : "+v"(x) : : "memory"); }
__device__ __forceinline__ void keep_after_requests(uint32_t& x) { asm volatile("" : "+v"(x) : : "memory"); }

template <int RK, int RV, int GT, int FMT, bool NT>
__global__ __launch_bounds__(kDecodeThreads) void decode_partial_mma_kernel(const DecodeParams p) {
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
  // raw words per lane: a quarter of a key row per 16-row block; value tiles as units of 8 rows by one word
  constexpr int KRAW = RK / 4 / kElemsPerDword;  // bf16: RK / 8, 8-bit: RK / 16, 4-bit: RK / 32
  constexpr int VWORDS = RV / kElemsPerDword;    // words in a value row
  constexpr int VUNITS = 4 * VWORDS;
  constexpr int VPL = (VUNITS + 63) / 64;        // units per lane
  constexpr int VP = kMmaVPitch;
  static_assert(KRAW >= 1 && (RK / 4) % kElemsPerDword == 0, "rank not supported by this format");

  // The projection scratch is needed before the first tile only, the value tiles after it: one region.
  constexpr int kProjBytes = kProjectThreads * (GT < 4 ? GT : 4) * 8 * (int)sizeof(float);
  constexpr int kTileBytes = 4 * RV * VP * (int)sizeof(uint16_t);           // per wave: value tile, [channel][row]
  __shared__ __attribute__((aligned(16))) unsigned char scratch_s[kProjBytes > kTileBytes ? kProjBytes : kTileBytes];
  __shared__ float red[4 * GT * (RV + 2)];
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
    fresh_rows_block_q<RK, RV, GT>(p, b, kv, pass, hq0, px_s, ppart_s, py_s, SKV_QBITS == 4 ? kNibbleOffset : 0.f);
#else
    fresh_rows_block<RK, RV, GT>(p, b, kv, pass, hq0, px_s, ppart_s, py_s);
#endif
    return;
  }
  int t0, t1;
  range_of_split((int)clamped_len(p.seq_lens, b, p.n_ctx - p.len_add) + p.len_add, p.n_stream, split, &t0, &t1);

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
  const int n_tiles = (t1 - t0 + kMmaTileRows - 1) / kMmaTileRows;
  struct TileRegsM {
    uint32_t k[2][KRAW];
    uint32_t v[VPL][8];
#if SKV_Q8
    uint32_t vm[NG][2][4];                       // (scale | zero << 16) of rows 16 kb + 4 g + i, per group
#endif
  };
  auto issue_tile = [&](int tile, TileRegsM& tr) {
    const int row0 = t0 + tile * kMmaTileRows;
    const int64_t base = tile_base(row0);
    if (row0 + kMmaTileRows <= t1) {
      // A whole tile (all but the last of a range): one address per stream and lane, the rest are constant
      // offsets; streaming or ordinary loads as the launch asks (NT).
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
            const uint32_t* vsrc = p.v_cache + (base + 8 * kg) * VWORDS + cw;
#pragma unroll
            for (int e = 0; e < 8; ++e) tr.v[u][e] = load_cache<NT>(vsrc + e * VWORDS);
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
      return;
    }
    const int last = t1 - 1 - row0;                              // rows past it re-read it; their weights are zero
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
        for (int e = 0; e < 8; ++e) {
          int r = 8 * kg + e;
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
    return uint4{high_halves(byte_to_f32<0>(w0), byte_to_f32<1>(w0)), high_halves(byte_to_f32<2>(w0), byte_to_f32<3>(w0)),
                 high_halves(byte_to_f32<0>(w1), byte_to_f32<1>(w1)), high_halves(byte_to_f32<2>(w1), byte_to_f32<3>(w1))};
  };
#elif SKV_QBITS == 4
  auto key_operand = [&](const TileRegsM& tr, int kb, int ks) -> uint4 {
    const uint32_t w = tr.k[kb][ks];                             // 8 codes: the even channel in the low half of a byte
    const uint32_t ev = w & 0x0f0f0f0fu, od = (w >> 4) & 0x0f0f0f0fu;
    return uint4{nibbles_to_bf16_pair(byte_pair<0>(ev, od)), nibbles_to_bf16_pair(byte_pair<1>(ev, od)),
                 nibbles_to_bf16_pair(byte_pair<2>(ev, od)), nibbles_to_bf16_pair(byte_pair<3>(ev, od))};
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
            const uint32_t w0 = tr.v[u][2 * e2], w1 = tr.v[u][2 * e2 + 1];
            const float f0 = c == 0 ? byte_to_f32<0>(w0) : c == 1 ? byte_to_f32<1>(w0) : c == 2 ? byte_to_f32<2>(w0) : byte_to_f32<3>(w0);
            const float f1 = c == 0 ? byte_to_f32<0>(w1) : c == 1 ? byte_to_f32<1>(w1) : c == 2 ? byte_to_f32<2>(w1) : byte_to_f32<3>(w1);
            o[e2] = high_halves(f0, f1);
          }
          uint16_t* dst = vt + (4 * cw + c) * VP + 16 * (kg & 1) + 4 * (kg >> 1);   // rows 8 kg + e at 16 (kg % 2) + 8 (e / 4) + 4 (kg / 2) + e % 4
          *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1]);
          *reinterpret_cast<uint2*>(dst + 8) = make_uint2(o[2], o[3]);
        }
#elif SKV_QBITS == 4
        // a word holds channels 8 cw .. 8 cw + 7 of one row: even ones in the low halves of its bytes
        uint32_t ev[8], od[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          ev[e] = tr.v[u][e] & 0x0f0f0f0fu;
          od[e] = (tr.v[u][e] >> 4) & 0x0f0f0f0fu;
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          uint32_t o[4];
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t a = (c & 1) ? od[2 * e2] : ev[2 * e2], bb = (c & 1) ? od[2 * e2 + 1] : ev[2 * e2 + 1];
            // channel c of rows 2 e2 and 2 e2 + 1: the same byte of two words, picked by one byte-permute
            const uint32_t pair = (c >> 1) == 0 ? byte_pair<0>(a, bb) : (c >> 1) == 1 ? byte_pair<1>(a, bb)
                                : (c >> 1) == 2 ? byte_pair<2>(a, bb) : byte_pair<3>(a, bb);
            o[e2] = nibbles_to_bf16_pair(pair);
          }
          uint16_t* dst = vt + (8 * cw + c) * VP + 16 * (kg & 1) + 4 * (kg >> 1);
          *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1]);
          *reinterpret_cast<uint2*>(dst + 8) = make_uint2(o[2], o[3]);
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
  // SKV_MMA_DEPTH tiles per wave on their way while the queries are prepared, and from then on (one register
  // set each).  Measured: a second set is slower at every shape tried (45.1 against 43.5 us at b4/32K, 64/64).
  // The requests go out in an order and a shape that keep the waits exact: first the few words the queries
  // need (from the workspace, or the basis pieces and raw queries of the in-kernel projection), then the
  // wave's first tile, without a condition (a wave with no tile of its own requests the range's last one and
  // never looks at it).  A request made under a condition is waited for where the paths join again, and
  // requests return in order, so the other way round the queries would wait for the whole tile.
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
  // bf16 rows, queries projected here: the projection's few words (basis pieces, raw queries) are waited for
  // BEFORE the tiles go out -- every workgroup of the launch starts at the same moment, and behind the whole
  // chip's first tiles those words took 3-5 us to arrive -- and TWO tiles per wave are requested, so that the
  // memory system has work for the 2-3 us the projection then takes (one tile per wave is 16 MB over the chip,
  // 2 us of streaming).  From the third tile on a wave is one tile ahead, as before: a second set in flight
  // throughout measured slower.  Measured b4/32K 64/64, rows from HBM: 46.6-47.1 against 48.2 us per launch.
  constexpr bool kTwoEarly = !SKV_Q8 && SKV_MMA_DEPTH == 1;
  const bool two_early = kTwoEarly && !from_workspace;
  if (two_early) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  issue_tile(wave < n_tiles ? wave : n_tiles - 1, ta);
#if SKV_MMA_DEPTH == 2
  TileRegsM tb;
  if (wave + 4 < n_tiles) issue_tile(wave + 4, tb);
#else
  [[maybe_unused]] TileRegsM tb;
  if constexpr (kTwoEarly) {
    if (two_early && wave + 4 < n_tiles) issue_tile(wave + 4, tb);
  }
#endif
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
    for (int i = 0; i < 8; ++i) x[i] = lm < GT ? xq[ks][i] * qscale * key_scale_of(g * (RK / 4) + 8 * ks + i) : 0.f;
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

  // one tile from register set tr; the tile after next is requested into the same set once it is free
  // next_tile: the tile to request into the set once it is free (none if out of range)
  auto process_next = [&](int tile, TileRegsM& tr, int next_tile) {
    const int row0 = t0 + tile * kMmaTileRows;
    // scores minus the reference: the reference rides in as the initial accumulator
    f32x4 sc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      sc[kb] = f32x4{-m_ref, -m_ref, -m_ref, -m_ref};
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
#if SKV_Q8
        const uint4 a = key_operand(tr, kb, ks);
        sc[kb] = mfma16w(a, qhi[ks], sc[kb]);
        sc[kb] = mfma16w(a, qlo[ks], sc[kb]);
#else
        const uint2 a = key_operand(tr, kb, ks);
        sc[kb] = mfma16(a, qhi[ks], sc[kb]);
        sc[kb] = mfma16(a, qlo[ks], sc[kb]);
#endif
      }
    }
    store_values(tr);
#if SKV_Q8
    float vscale[NG][2][4], vzero[NG][2][4];
#pragma unroll
    for (int gq = 0; gq < NG; ++gq)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          vscale[gq][kb][i] = bf16_lo(tr.vm[gq][kb][i]);
          vzero[gq][kb][i] = bf16_hi(tr.vm[gq][kb][i]);
          if (SKV_QBITS == 4) vzero[gq][kb][i] = fmaf(-kNibbleOffset, vscale[gq][kb][i], vzero[gq][kb][i]);
        }
#endif
    __builtin_amdgcn_wave_barrier();
    if (next_tile >= 0 && next_tile < n_tiles) issue_tile(next_tile, tr);
    // rows past the end of the range do not count
    if (row0 + kMmaTileRows > t1) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (row0 + 16 * kb + 4 * g + i >= t1) sc[kb][i] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                     fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (first || mx > kRescaleSlack) {                           // the reference moves (lanes of a column agree)
      const float f = first ? 0.f : fast_exp2(-mx);
      m_ref = first ? mx : m_ref + mx;
      l *= f;
#pragma unroll
      for (int gq = 0; gq < NG; ++gq) zsum[gq] *= f;
#pragma unroll
      for (int cb = 0; cb < VBLOCKS; ++cb) oacc[cb] *= f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) sc[kb] -= mx;
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
#pragma unroll
    for (int cb = 0; cb < VBLOCKS; ++cb) {
      const uint4 a = *reinterpret_cast<const uint4*>(vt + (16 * cb + lm) * VP + 8 * g);
      const int gq = (16 * cb) / 64;
      oacc[cb] = mfma16w(a, phi[gq], oacc[cb]);
      oacc[cb] = mfma16w(a, plo[gq], oacc[cb]);
    }
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
  auto process = [&](int tile, TileRegsM& tr) { process_next(tile, tr, tile + 4 * SKV_MMA_DEPTH); };
#if SKV_MMA_DEPTH == 2
  for (int tile = wave; tile < n_tiles; tile += 8) {
    process(tile, ta);
    if (tile + 4 < n_tiles) process(tile + 4, tb);
  }
#else
  int first_tile = wave;
  if constexpr (kTwoEarly) {
    if (two_early) {                               // the two tiles requested before the projection
      if (wave < n_tiles) process_next(wave, ta, wave + 8);
      if (wave + 4 < n_tiles) process_next(wave + 4, tb, -1);
      first_tile = wave + 8;
    }
  }
  for (int tile = first_tile; tile < n_tiles; tile += 4) process(tile, ta);
#endif

  // ---- the four lanes of a column hold shares of l (and of the zero sums); then merge the 4 waves through
  //      LDS, in wave order ------------------------------------------------------------------------
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
#if SKV_Q8
#pragma unroll
  for (int gq = 0; gq < NG; ++gq) {
    zsum[gq] += __shfl_xor(zsum[gq], 16);
    zsum[gq] += __shfl_xor(zsum[gq], 32);
  }
#endif
  if (lm < GT) {
    float* r = red + (wave * GT + lm) * (RV + 2);
#pragma unroll
    for (int cb = 0; cb < VBLOCKS; ++cb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float a = oacc[cb][i];
        if (SKV_Q8) a += zsum[(16 * cb) / 64];                   // every channel of a group receives the group's zero sum
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
    float mt = red[(0 * GT + hg) * (RV + 2) + RV];
#pragma unroll
    for (int w = 1; w < 4; ++w) mt = fmaxf(mt, red[(w * GT + hg) * (RV + 2) + RV]);
    if (c == RV) {
      out_ml[hg * head_step_ml] = mt;
    } else {
      const int src = c == RV + 1 ? RV + 1 : c;
      float a = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float* r = red + (w * GT + hg) * (RV + 2);
        a += r[src] * fast_exp2(r[RV] - mt);
      }
      if (c == RV + 1) out_ml[hg * head_step_ml + 1] = a;
      else out_acc[hg * head_step_acc + c] = a;
    }
  }
}
