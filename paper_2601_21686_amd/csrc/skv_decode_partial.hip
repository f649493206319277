// Split-context decode attention over the compressed cache: scores, online
// softmax and value mix for one context range of one KV head.
//
// This file is compiled once per key rank (-DSKV_RK=16,32,...,128); each
// object holds the kernels for that r_K and every r_V in {16,...,128} and
// 1, 2 or 4 query heads per workgroup.  With -DSKV_QBITS=8 (or 4) it is compiled
// for the quantised cache (Sec. 4.3; 8 bits: ranks 32, 64, 96, 128, one byte per
// channel; 4 bits: ranks 64, 128, two channels per byte): key scales are already folded into q~ (the key zero point
// adds the same constant to every score of a query and drops out of the
// softmax), and every value row carries a (scale, zero) pair per 64-channel
// group: a~ = sum_j (p_j scale_j) code_j + sum_j p_j zero_j.
//
// What is computed (App. A.1 Eq. 18 on the reconstructed cache of Sec. 3.2
// Eq. 7, in the factored form q K~^T = (q P_K) K_down^T,
// softmax(.) V~ = (softmax(.) V_down) P_V^T), given
//   q~[g]   = (q[g] . P_K) * scale * log2(e)               per query head g of the group:
//   s[g][j] = <q~[g], K_down[j]>                            j in this range
//   m, l, a = running max, normaliser and sum_j 2^(s_j - m) V_down[j]
// written per (sequence, query head, range) for the combine kernel.
//
// Mapping.  The (b, kv-head) stream K_down[0:n][r_K] is one contiguous span, so
// any run of rows is a coalesced segment whatever the rank.  Eight lanes (an
// "octet") share one cache row: lane j of the octet owns the j-th eighth of
// the first 128 bytes of the row and the j-th eighth of the rest, which keeps
// every load a 4..16-byte piece that is contiguous across the octet.  A
// 64-lane wave therefore covers 8 consecutive rows per load, U loads deep.
// Scores are reduced across the octet with DPP adds (no LDS); the two quads of
// an octet each finish half of the query heads; each octet runs its own
// online-softmax stream and streams are merged once at the end.
// The projected query q~ comes from the projection kernel (skv_project.hip) or is computed here.
// Both range kernels exist with ordinary and with streaming (non-temporal) loads of the cache rows
// (last template argument); the launcher picks per launch (DecodeParams::stream_loads).
//
// Parts: this file holds the cache-format description, the vector-arithmetic range kernel and the
// launchers; skv_decode_fresh.inl the extra workgroups of a fused decode step (the new rows);
// skv_decode_mma.inl the same range on the matrix cores.
#include "skv_device_util.h"
#include "skv_internal.h"

#ifndef SKV_RK
#error "compile with -DSKV_RK=<key rank>"
#endif
#ifndef SKV_QBITS
#define SKV_QBITS 0                 // 0: bf16 rows; 8 or 4: integer codes of that width (Sec. 4.3)
#endif
#define SKV_Q8 (SKV_QBITS != 0)     // any quantised build: codes plus per-row value ranges
#ifndef SKV_PAGED
#define SKV_PAGED 0                 // 1: the caches are page pools addressed through a block table (bf16 rows only)
#endif
// Quantised rows in pages are served by the matrix-core kernel only: such a build leaves the vector kernel out.
#define SKV_VECTOR_KERNEL (!(SKV_PAGED && SKV_QBITS != 0))
#if SKV_QBITS != 0 && SKV_QBITS != 8 && SKV_QBITS != 4
#error "SKV_QBITS must be 0, 8 or 4"
#endif

namespace skv {
namespace {

constexpr float kNegBig = -1.0e30f;   // "no score seen yet"; finite so that differences stay finite
constexpr float kRescaleSlack = 8.0f; // log2 units a score may exceed the softmax reference before it moves

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// How the r channels of a row are dealt to the 8 lanes of an octet: lane j owns the j-th eighth
// of the first 64 channels and the j-th eighth of the rest.
#if SKV_QBITS == 8
constexpr int kElemsPerDword = 4;                // one byte per channel
constexpr int kFmt = SKV_PAGED ? 4 : 1;
#elif SKV_QBITS == 4
constexpr int kElemsPerDword = 8;                // two channels per byte, the even one in the low half
constexpr int kFmt = SKV_PAGED ? 5 : 2;
#else
constexpr int kElemsPerDword = 2;                // bf16
constexpr int kFmt = SKV_PAGED ? 3 : 0;
#endif
template <int R>
struct RowMap {
  static constexpr int NA = R < 64 ? R : 64;   // channels in the first segment
  static constexpr int NB = R - NA;            // channels in the second segment
  static constexpr int CA = NA / 8;            // channels per lane, first segment
  static constexpr int CB = NB / 8;            // second segment
  static constexpr int DA = CA / kElemsPerDword;   // dwords per lane
  static constexpr int DB = CB / kElemsPerDword;
  static constexpr int CPL = CA + CB;          // channels per lane
  static constexpr int DPL = DA + DB;          // dwords per lane
  static constexpr int ROW_DW = R / kElemsPerDword;    // dwords per row
  static constexpr int SEG_B_DW = 64 / kElemsPerDword; // where the second segment starts
  static constexpr int NG = (R + 63) / 64;     // 64-channel groups (quantisation groups)
  static_assert(CA % kElemsPerDword == 0 && CB % kElemsPerDword == 0, "rank not supported by this format");
  // channel held in slot i of lane j
  __device__ static constexpr int chan(int j, int i) {
    return i < CA ? j * CA + i : NA + j * CB + (i - CA);
  }
  // 64-channel group of slot i
  __device__ static constexpr int group_of_slot(int i) { return i < CA ? 0 : 1; }
};

// Cache rows are loaded either with ordinary loads or, when the launch's rows cannot be found in a
// cache again anyway (see DecodeParams::stream_loads), with streaming (non-temporal) ones.  The kind is a
// template parameter of the range kernels: a run-time branch at the point of issue costs the steady-state
// loop its exact wait counts (measured: 10-25 % slower).
template <bool NT, typename T>
__device__ __forceinline__ T load_cache(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int N, bool NT>
__device__ __forceinline__ void load_dwords(const uint32_t* p, uint32_t* w) {
  if constexpr (N == 1) {
    w[0] = load_cache<NT>(p);
  } else if constexpr (N == 2) {
    const u32x2 v = load_cache<NT>(reinterpret_cast<const u32x2*>(p));
    w[0] = v.x; w[1] = v.y;
  } else if constexpr (N == 3) {
    w[0] = load_cache<NT>(p);
    w[1] = load_cache<NT>(p + 1);
    w[2] = load_cache<NT>(p + 2);
  } else if constexpr (N == 4) {
    const u32x4 v = load_cache<NT>(reinterpret_cast<const u32x4*>(p));
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  }
}

template <int R, bool NT = false>
__device__ __forceinline__ void load_row(const uint32_t* row, int j, uint32_t (&w)[RowMap<R>::DPL]) {
  using M = RowMap<R>;
  load_dwords<M::DA, NT>(row + j * M::DA, &w[0]);
  if constexpr (M::DB > 0) load_dwords<M::DB, NT>(row + M::SEG_B_DW + j * M::DB, &w[M::DA]);
}

template <int R>
__device__ __forceinline__ void unpack_row(const uint32_t (&w)[RowMap<R>::DPL], float (&f)[RowMap<R>::CPL]) {
#pragma unroll
  for (int i = 0; i < RowMap<R>::DPL; ++i) {
#if SKV_QBITS == 8
    f[4 * i] = (float)(w[i] & 0xffu);
    f[4 * i + 1] = (float)((w[i] >> 8) & 0xffu);
    f[4 * i + 2] = (float)((w[i] >> 16) & 0xffu);
    f[4 * i + 3] = (float)(w[i] >> 24);
#elif SKV_QBITS == 4
    // even channels sit in the low halves of the bytes, odd ones in the high halves: two masks,
    // then one byte-to-float conversion per channel
    const uint32_t ev = w[i] & 0x0f0f0f0fu, od = (w[i] >> 4) & 0x0f0f0f0fu;
    f[8 * i] = (float)(ev & 0xffu);
    f[8 * i + 1] = (float)(od & 0xffu);
    f[8 * i + 2] = (float)((ev >> 8) & 0xffu);
    f[8 * i + 3] = (float)((od >> 8) & 0xffu);
    f[8 * i + 4] = (float)((ev >> 16) & 0xffu);
    f[8 * i + 5] = (float)((od >> 16) & 0xffu);
    f[8 * i + 6] = (float)(ev >> 24);
    f[8 * i + 7] = (float)(od >> 24);
#else
    f[2 * i] = bf16_lo(w[i]);
    f[2 * i + 1] = bf16_hi(w[i]);
#endif
  }
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Sum over the 8 lanes of an octet; every lane receives the same bits.
__device__ __forceinline__ float octet_sum(float x) {
  x += dpp_f32<0x141>(x);   // row_half_mirror: lane i <-> 7-i
  x += dpp_f32<0xB1>(x);    // quad_perm [1,0,3,2]
  x += dpp_f32<0x4E>(x);    // quad_perm [2,3,0,1]
  return x;
}

// Sum / maximum over the 8 lanes that sit 8, 16 and 32 apart (the same slot of the wave's 8 octets); every
// lane receives the same bits.  The exchanges are vector instructions: a rotation by 8 inside a row of 16
// lanes, then the swaps of odd and even rows and of the two halves of the wave.  (The same tree as three
// shuffles, with the same bits, without the round trips through the LDS pipeline: the end-of-range merge
// of 40-odd values per lane took 2.4 us with shuffles.)
__device__ __forceinline__ float rows_pair(float x, bool take_max) {
  const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return take_max ? fmaxf(__uint_as_float(r.x), __uint_as_float(r.y)) : __uint_as_float(r.x) + __uint_as_float(r.y);
}
__device__ __forceinline__ float halves_pair(float x, bool take_max) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return take_max ? fmaxf(__uint_as_float(r.x), __uint_as_float(r.y)) : __uint_as_float(r.x) + __uint_as_float(r.y);
}
__device__ __forceinline__ float octets_sum(float x) {
  x += dpp_f32<0x128>(x);          // row_ror:8: lane i <-> i ^ 8
  return halves_pair(rows_pair(x, false), false);
}
__device__ __forceinline__ float octets_max(float x) {
  x = fmaxf(x, dpp_f32<0x128>(x));
  return halves_pair(rows_pair(x, true), true);
}

// Build-time tunables (defaults are the measured best on MI355X).
#ifndef SKV_DW_IN_FLIGHT
#define SKV_DW_IN_FLIGHT 8       // dwords of keys (and of values) one lane requests per tile
#endif
#ifndef SKV_EARLY_TILES
#define SKV_EARLY_TILES 6        // tiles a long range requests before the in-kernel query projection (>= 2)
#endif
#ifndef SKV_EARLY_FROM
#define SKV_EARLY_FROM 24        // a range is long from this many whole tiles; a shorter one requests two
#endif
#ifndef SKV_PIPELINE
#define SKV_PIPELINE 1           // tiles requested ahead of the one being computed on (>= 1)
#endif

// Rows per lane and tile: about SKV_DW_IN_FLIGHT dwords of keys and of values.
template <int RK, int RV>
struct Depth {
  static constexpr int kMaxDw = RowMap<RK>::DPL > RowMap<RV>::DPL ? RowMap<RK>::DPL : RowMap<RV>::DPL;
  static constexpr int kRaw = SKV_DW_IN_FLIGHT / kMaxDw;
  static constexpr int U = kRaw < 1 ? 1 : (kRaw > 8 ? 8 : kRaw);
};

// The raw cache words of one tile: U rows of keys and of values per lane.
template <int RK, int RV, int U>
struct TileRegs {
  uint32_t kw[U][RowMap<RK>::DPL];
  uint32_t vw[U][RowMap<RV>::DPL];
#if SKV_Q8
  uint32_t vm[U][RowMap<RV>::NG];              // per row and group: bf16 scale (low half), bf16 zero (high half)
#endif
};

// Requests 8*U rows of a wave.  row0 is this lane's first row; the lane's rows
// are row0 + 8u.  With MASKED, rows >= t_end are redirected to row t_end-1 so
// that nothing outside [0, n_ctx) is ever read.
template <int RK, int RV, int U, bool MASKED, bool NT = false>
__device__ __forceinline__ void issue_rows(const uint32_t* __restrict__ kbase,
                                           const uint32_t* __restrict__ vbase,
                                           const uint32_t* __restrict__ mbase, int row0, int t_end,
                                           int j, TileRegs<RK, RV, U>& t) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int row = row0 + 8 * u;
    if constexpr (MASKED) row = row < t_end ? row : t_end - 1;
    load_row<RK, NT>(kbase + (int64_t)row * RowMap<RK>::ROW_DW, j, t.kw[u]);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int row = row0 + 8 * u;
    if constexpr (MASKED) row = row < t_end ? row : t_end - 1;
    load_row<RV, NT>(vbase + (int64_t)row * RowMap<RV>::ROW_DW, j, t.vw[u]);
#if SKV_Q8
#pragma unroll
    for (int g = 0; g < RowMap<RV>::NG; ++g) t.vm[u][g] = load_cache<NT>(mbase + (int64_t)row * RowMap<RV>::NG + g);
#endif
  }
}

// How the query heads of a pass are shared inside an octet.  With two or more heads the two
// quads of the octet split them: after the per-lane partial dot products every lane keeps the
// partial sums of "its" half (HL heads) and hands the other half to its mirror lane (i <-> 7-i,
// which sits in the other quad), so the cross-lane reduction, the running maximum, the
// exponentials and the normaliser are computed for HL heads per lane instead of GT.  The mix
// needs the weights of all GT heads; the other half comes from the mirror lane (i <-> 7-i),
// which sits in the other quad.  Accumulator slot a < HL belongs to head qd*HL + a (this
// lane's quad qd), slot HL + a to head (1-qd)*HL + a.
template <int GT>
struct HeadSplit {
  static constexpr bool kSplit = GT >= 2;
  static constexpr int HL = kSplit ? GT / 2 : GT;     // heads whose softmax this lane runs
  __device__ static int head_of_slot(int slot, int qd) {
    if (!kSplit) return slot;
    return slot < HL ? qd * HL + slot : (1 - qd) * HL + (slot - HL);
  }
};

// Scores, online softmax and value mix for the rows of one tile.
//   qreg: projected queries in slot order (HeadSplit), this lane's channels
//   m, l: softmax reference (log2 units; within kRescaleSlack below the running maximum) and
//         normaliser of this lane's HL heads
//   acc:  un-normalised mixes, slot order
template <int RK, int RV, int GT, int U, bool MASKED>
__device__ __forceinline__ void consume_rows(const TileRegs<RK, RV, U>& t, int row0, int t_end, int qd,
                                             const float (&qreg)[GT][RowMap<RK>::CPL],
                                             float (&m)[HeadSplit<GT>::HL], float (&l)[HeadSplit<GT>::HL],
                                             float (&acc)[GT][RowMap<RV>::CPL],
                                             float (&zacc)[GT][RowMap<RV>::NG]) {
  using KM = RowMap<RK>;
  using VM = RowMap<RV>;
  using HS = HeadSplit<GT>;
  constexpr int HL = HS::HL;
  // per-lane partial dot products for all GT heads, then keep this quad's half and reduce
  float s[U][HL];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float kf[KM::CPL];
    unpack_row<RK>(t.kw[u], kf);
    float d[GT];                                 // slot order: see HeadSplit
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      d[g] = 0.f;
#pragma unroll
      for (int i = 0; i < KM::CPL; ++i) d[g] = fmaf(qreg[g][i], kf[i], d[g]);
    }
#pragma unroll
    for (int a = 0; a < HL; ++a) {
      float x;
      if constexpr (HS::kSplit) {
        // slot HL+a of the mirror lane is the same head as slot a here: one add pairs the
        // two quads, two more finish the sum inside the quad
        x = d[a] + dpp_f32<0x141>(d[HL + a]);
        x += dpp_f32<0xB1>(x);
        x += dpp_f32<0x4E>(x);
      } else {
        x = octet_sum(d[a]);
      }
      if constexpr (MASKED) x = (row0 + 8 * u < t_end) ? x : kNegBig;
      s[u][a] = x;
    }
  }

  // online softmax of this lane's heads.  The reference m only follows the running maximum when
  // a score exceeds it by more than kRescaleSlack (weights then stay below 2^kRescaleSlack, far
  // inside float32 range, and every sum is rescaled consistently, so the result is unchanged);
  // after the first tile of a stream this almost never happens, and the rescale of the
  // accumulators is skipped unless some octet of the wave needs it.
  float c[HL];
  bool moved = false;
#pragma unroll
  for (int a = 0; a < HL; ++a) {
    float mx = s[0][a];
#pragma unroll
    for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u][a]);
    const bool jump = mx > m[a] + kRescaleSlack;
    const float mn = jump ? mx : m[a];
    moved = moved || jump;
    c[a] = fast_exp2(m[a] - mn);             // exactly 1 when the reference stays
    m[a] = mn;
  }
  if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
    for (int a = 0; a < HL; ++a) {
      l[a] *= c[a];
#pragma unroll
      for (int i = 0; i < VM::CPL; ++i) acc[a][i] *= c[a];
      if constexpr (HS::kSplit) {
        const float cr = dpp_f32<0x141>(c[a]);   // the other quad's factor for its head
#pragma unroll
        for (int i = 0; i < VM::CPL; ++i) acc[HL + a][i] *= cr;
#if SKV_Q8
#pragma unroll
        for (int g = 0; g < VM::NG; ++g) zacc[HL + a][g] *= cr;
#endif
      }
#if SKV_Q8
#pragma unroll
      for (int g = 0; g < VM::NG; ++g) zacc[a][g] *= c[a];
#endif
    }
  }

  float pw[U][GT];
#pragma unroll
  for (int a = 0; a < HL; ++a) {
    float lsum = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float pv = fast_exp2(s[u][a] - m[a]);
      if constexpr (MASKED) pv = (row0 + 8 * u < t_end) ? pv : 0.f;
      pw[u][a] = pv;
      if constexpr (HS::kSplit) pw[u][HL + a] = dpp_f32<0x141>(pv);
      lsum += pv;
    }
    l[a] += lsum;
  }

#pragma unroll
  for (int u = 0; u < U; ++u) {
    float vf[VM::CPL];
    unpack_row<RV>(t.vw[u], vf);
#if SKV_Q8
    float sc[VM::NG], zr[VM::NG];
#pragma unroll
    for (int gq = 0; gq < VM::NG; ++gq) {
      sc[gq] = bf16_lo(t.vm[u][gq]);
      zr[gq] = bf16_hi(t.vm[u][gq]);
    }
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float ps[VM::NG];
#pragma unroll
      for (int gq = 0; gq < VM::NG; ++gq) {
        ps[gq] = pw[u][g] * sc[gq];
        zacc[g][gq] = fmaf(pw[u][g], zr[gq], zacc[g][gq]);
      }
#pragma unroll
      for (int i = 0; i < VM::CPL; ++i) acc[g][i] = fmaf(ps[VM::group_of_slot(i)], vf[i], acc[g][i]);
    }
#else
#pragma unroll
    for (int g = 0; g < GT; ++g) {
#pragma unroll
      for (int i = 0; i < VM::CPL; ++i) acc[g][i] = fmaf(pw[u][g], vf[i], acc[g][i]);
    }
#endif
  }
}

#include "skv_decode_fresh.inl"

#if SKV_VECTOR_KERNEL
// FMT only names the cache format in the kernel's symbol (0: bf16 rows, 1: 8-bit codes, 2: 4-bit codes,
// 3: bf16 rows in pages, 4 and 5: 8- and 4-bit codes in pages).
template <int RK, int RV, int GT, int FMT, bool NT>
__global__ __launch_bounds__(kDecodeThreads) void decode_partial_kernel(const DecodeParams p) {
  static_assert(FMT == kFmt, "format tag must match the build");
  using KM = RowMap<RK>;
  using VM = RowMap<RV>;
  constexpr int U = Depth<RK, RV>::U;
  constexpr int ROWS_PER_WAVE = 8 * U;
  constexpr int ROWS_PER_WG = 4 * ROWS_PER_WAVE;

  __shared__ float red[4 * GT * (RV + 2)];       // cross-wave merge at the end of the range
#if !SKV_Q8
  // scratch of the in-kernel projections (queries; new rows of a fused decode step)
  __shared__ float px_s[GT * SKV_HEAD_DIM];
  __shared__ float ppart_s[kProjectThreads * GT * 8];
  __shared__ float py_s[GT * SKV_HEAD_DIM];
#endif

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int oct = lane >> 3;
  const int j = lane & 7;

  int split = blockIdx.x;
  const int passes = p.group / GT;
  int col = blockIdx.y;                          // ((b * H_KV + kv) * passes + pass)
  const int n_cols = p.batch * p.n_kv_heads * passes;
  // Grid rows past the last column hold the fresh-rows workgroups of a fused decode step, one per
  // column: they are dispatched after every streaming workgroup, so the streaming ones spread over
  // the compute units exactly as in a launch without them.
  const bool fresh = col >= n_cols;
  if (fresh) {
    col = (col - n_cols) * (int)gridDim.x + split;
    if (col >= n_cols) return;
    split = p.n_stream;
  }
  const int pass = col % passes;
  const int bkv = col / passes;
  const int kv = bkv % p.n_kv_heads;
  const int b = bkv / p.n_kv_heads;
  const int hq0 = kv * p.group + pass * GT;      // first query head of this pass

#if !SKV_Q8
  if (fresh) {                                   // the extra workgroup of a fused decode step
    fresh_rows_block<RK, RV, GT>(p, b, kv, pass, hq0, px_s, ppart_s, py_s);
    return;
  }
#endif
  int t0, t1;
  const int seq_rows = (int)clamped_len(p.seq_lens, b, p.n_ctx - p.len_add) + p.len_add;
  range_of_split(seq_rows, p.n_stream, split, &t0, &t1);

  float* out_acc = p.part_acc + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + split) * RV;
  float* out_ml = p.part_ml + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + split) * 2;
  const int64_t head_step_acc = (int64_t)p.n_splits * RV;
  const int64_t head_step_ml = (int64_t)p.n_splits * 2;

  if (t0 >= t1) {
    // Empty range: the neutral element of the merge.
    for (int i = tid; i < GT * RV; i += kDecodeThreads) out_acc[(i / RV) * head_step_acc + (i % RV)] = 0.f;
    if (tid < GT) { out_ml[tid * head_step_ml] = kNegBig; out_ml[tid * head_step_ml + 1] = 0.f; }
    return;
  }

  const int lane_row = wave * ROWS_PER_WAVE + oct;     // this lane's first row inside a tile
  const int n_full = (t1 - t0) / ROWS_PER_WG;         // tiles with every row valid
  // The full tiles of a range are taken front to back when the sequence holds an even number of rows and back
  // to front when it holds an odd number.  A decode loop adds a row per step, so consecutive steps sweep the
  // cache in opposite directions and a step meets first the rows the step before read last -- the ones a
  // last-level cache of about the cache's size still holds (a plain read of 256 MiB in 512 slices: 39.6 us per
  // launch always front to back, 35.6 us in alternating directions).  The order only permutes the terms of
  // sums; the same call gives the same bits.
  const bool backwards = (seq_rows & 1) != 0;
  auto row_of_tile = [&](int idx) { return t0 + (backwards ? n_full - 1 - idx : idx) * ROWS_PER_WG; };
  using Tile = TileRegs<RK, RV, U>;
  Tile ta;
#if SKV_PAGED
  // Ranges start at multiples of 64 rows and a page holds a multiple of 64 rows, so the 8*U <= 64 rows a
  // wave requests in a full tile lie in ONE page: the page is looked up once per wave and tile.  Lane i
  // keeps the table entry of the range's page (first + i); a full tile takes its entry with a lane read,
  // so no load sits between a tile and the addresses of its rows.  Ranges longer than 64 pages refill.
  static_assert(ROWS_PER_WAVE <= kRangeQuantum && kRangeQuantum % ROWS_PER_WAVE == 0, "a wave's rows must share a page");
  const int page_rows_mask = (1 << p.pages.page_shift) - 1;
  const int page_first = t0 >> p.pages.page_shift;
  const int pages_in_range = ((t1 - 1) >> p.pages.page_shift) - page_first + 1;
  int held_first = 0;                            // which page of the range lane 0 holds
  int held = lane < pages_in_range ? clamped_page(p.pages, b, page_first + lane) : 0;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // requests the full tile whose first row is `tile_row` (a multiple of ROWS_PER_WG past t0)
  auto issue_full = [&](int tile_row, Tile& t) {
    const int r = tile_row + wave_u * ROWS_PER_WAVE;           // this wave's first row: wave-uniform
    const int rel = (r >> p.pages.page_shift) - page_first;
    if (rel < held_first || rel - held_first >= 64) {          // (ranges are swept in either direction)
      held_first = rel & ~63;
      held = held_first + lane < pages_in_range ? clamped_page(p.pages, b, page_first + held_first + lane) : 0;
    }
    const int page = __builtin_amdgcn_readlane(held, rel - held_first);
    const int64_t blk = ((int64_t)page * p.n_kv_heads + kv) << p.pages.page_shift;
    issue_rows<RK, RV, U, false, NT>(p.k_cache + blk * KM::ROW_DW, p.v_cache + blk * VM::ROW_DW, nullptr,
                                     (r & page_rows_mask) + oct, 0, j, t);
  };
  // the ragged tail: rows clamped to the last valid one, each looked up by itself
  auto issue_tail = [&](int row0, Tile& t) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int row = row0 + 8 * u;
      row = row < t1 ? row : t1 - 1;
      const int64_t at = cache_row(p.pages, 0, p.n_kv_heads, b, kv, row);
      load_row<RK>(p.k_cache + at * KM::ROW_DW, j, t.kw[u]);
      load_row<RV>(p.v_cache + at * VM::ROW_DW, j, t.vw[u]);
    }
  };
#else
  const uint32_t* kbase = p.k_cache + ((int64_t)b * p.n_kv_heads + kv) * p.capacity * KM::ROW_DW;
  const uint32_t* vbase = p.v_cache + ((int64_t)b * p.n_kv_heads + kv) * p.capacity * VM::ROW_DW;
#if SKV_Q8
  const uint32_t* mbase = p.v_meta + ((int64_t)b * p.n_kv_heads + kv) * p.capacity * VM::NG;
#else
  const uint32_t* mbase = nullptr;
#endif
  auto issue_full = [&](int tile_row, Tile& t) {
    issue_rows<RK, RV, U, false, NT>(kbase, vbase, mbase, tile_row + lane_row, t1, j, t);
  };
  auto issue_tail = [&](int row0, Tile& t) { issue_rows<RK, RV, U, true>(kbase, vbase, mbase, row0, t1, j, t); };
#endif

  // ---- this lane's slice of the projected queries, in slot order.  They come from the workspace
  //      (prepared by the projection kernel) or, when the raw queries are handed over, are projected
  //      here: q~ = (q P_K) * scale * log2(e), the same sums as the projection kernel.  Either way the
  //      first tile of the range is requested before the queries are waited for. -----------------
  float qreg[GT][KM::CPL];
  // Tiles 1 .. kEarlyTiles-1 of a long range, requested together with tile 0 ahead of the query projection:
  // the projection takes about as long as four tiles take to arrive at the steady rate.  A wave cannot go on
  // to the projection before its requests are accepted, which under load is not much sooner than they are
  // served, so a range of few tiles, where the projection is a visible share of the whole, requests only two.
  constexpr int kEarlyTiles = SKV_EARLY_TILES;
  constexpr int kEarlyFrom = SKV_EARLY_FROM;
  static_assert(kEarlyTiles >= 2 && kEarlyFrom > kEarlyTiles, "a long range holds more tiles than it requests early");
  Tile early[kEarlyTiles - 1];
  bool pre = false, pre2 = false;
#if !SKV_Q8
  if (p.q != nullptr) {
    ProjectPieces pp;
    project_rows_issue(p.p_k + (int64_t)kv * p.p_k_head_stride, RK, pp);
    // Every lane requests its share of the raw queries without a condition (a lane beyond the last element
    // repeats an earlier one and keeps nothing): a request under a condition is waited for where the
    // condition ends, ahead of the cache rows that should already be on their way by then.
    const uint16_t* qptr = p.q + ((int64_t)b * p.n_q_heads + hq0) * SKV_HEAD_DIM;
    constexpr int kQElems = GT * SKV_HEAD_DIM;
    constexpr int kQPerLane = (kQElems + kDecodeThreads - 1) / kDecodeThreads;
    uint16_t qraw[kQPerLane];
#pragma unroll
    for (int k = 0; k < kQPerLane; ++k) qraw[k] = qptr[(tid + k * kDecodeThreads) % kQElems];
    // The rest of the projection, once for each way the range starts: the waits for the basis and the queries
    // count the requests made after them, and a count is only exact where the path to it is a single one.
    auto finish = [&]() {
#pragma unroll
      for (int k = 0; k < kQPerLane; ++k)
        if (tid + k * kDecodeThreads < kQElems) px_s[tid + k * kDecodeThreads] = bf16_to_f32(qraw[k]);
      __syncthreads();
      project_rows_finish<GT>(pp, RK, px_s, ppart_s, py_s);
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        const float* qh = py_s + HeadSplit<GT>::head_of_slot(g, j >> 2) * RK;
#pragma unroll
        for (int i = 0; i < KM::CPL; ++i) qreg[g][i] = qh[KM::chan(j, i)] * p.scale_log2e;
      }
    };
    pre = SKV_PIPELINE == 1 && n_full >= kEarlyFrom;
    pre2 = SKV_PIPELINE == 1 && !pre && n_full >= 3;
    if (pre) {
      issue_full(row_of_tile(0), ta);
#pragma unroll
      for (int k = 1; k < kEarlyTiles; ++k) issue_full(row_of_tile(k), early[k - 1]);
      finish();
    } else if (pre2) {
      issue_full(row_of_tile(0), ta);
      issue_full(row_of_tile(1), early[0]);
      finish();
    } else if (n_full > 0) {
      issue_full(row_of_tile(0), ta);
      finish();
    } else {
      finish();
    }
  } else
#endif
  {
    const float* qt = p.qt + ((int64_t)b * p.n_q_heads + hq0) * RK;
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      const float* qh = qt + HeadSplit<GT>::head_of_slot(g, j >> 2) * RK;
#pragma unroll
      for (int i = 0; i < KM::CPL; i += 2) {
        const float2 v = *reinterpret_cast<const float2*>(qh + KM::chan(j, i));
        qreg[g][i] = v.x;
        qreg[g][i + 1] = v.y;
      }
    }
    if (n_full > 0) issue_full(row_of_tile(0), ta);
  }

  // ---- stream the range ---------------------------------------------------------------
  using HS = HeadSplit<GT>;
  constexpr int HL = HS::HL;
  const int qd = j >> 2;                         // which quad of the octet this lane is in
  float m[HL], l[HL], acc[GT][VM::CPL];
#pragma unroll
  for (int a = 0; a < HL; ++a) {
    m[a] = kNegBig;
    l[a] = 0.f;
  }
  float zacc[GT][VM::NG];                        // quantised cache: sum_j p_j zero_j per head and group
#pragma unroll
  for (int g = 0; g < GT; ++g) {
#pragma unroll
    for (int i = 0; i < VM::CPL; ++i) acc[g][i] = 0.f;
#pragma unroll
    for (int gq = 0; gq < VM::NG; ++gq) zacc[g][gq] = 0.f;
  }

  // A ring of NBUF register tiles: while one is being consumed the next NBUF-1 are already on
  // their way.  The steady-state loop issues unconditionally, so that the wait before each
  // consume is exactly "everything older than the tiles requested since".
  constexpr int NBUF = SKV_PIPELINE + 1;
  static_assert(NBUF >= 2, "at least one tile is requested ahead");
  if (n_full > 0) {
    Tile ring[NBUF];
    ring[0] = ta;                                   // tile 0 was requested before the projection
#pragma unroll
    for (int k = 1; k < NBUF - 1; ++k)
      if (k < n_full) issue_full(row_of_tile(k), ring[k]);
    int i = 0;
    if constexpr (NBUF == 2) {
      if (pre) {                                    // tiles 0 .. kEarlyTiles-1 are on their way (n_full >= kEarlyFrom)
        consume_rows<RK, RV, GT, U, false>(ring[0], 0, t1, qd, qreg, m, l, acc, zacc);
#pragma unroll
        for (int k = 1; k < kEarlyTiles; ++k) {
          if (k == kEarlyTiles - 1) issue_full(row_of_tile(kEarlyTiles), ring[0]);
          consume_rows<RK, RV, GT, U, false>(early[k - 1], 0, t1, qd, qreg, m, l, acc, zacc);
        }
        i = kEarlyTiles;                            // ring[0] holds that tile: the loop's invariant
      } else if (pre2) {                            // tiles 0 and 1 are on their way (n_full >= 3)
        consume_rows<RK, RV, GT, U, false>(ring[0], 0, t1, qd, qreg, m, l, acc, zacc);
        issue_full(row_of_tile(2), ring[0]);
        consume_rows<RK, RV, GT, U, false>(early[0], 0, t1, qd, qreg, m, l, acc, zacc);
        i = 2;
      }
    }
    if constexpr (NBUF > 1) {
      while (i + 2 * NBUF - 2 < n_full) {           // ring[k] holds tile i+k for k < NBUF-1
#pragma unroll
        for (int k = 0; k < NBUF; ++k) {
          issue_full(row_of_tile((i + k + NBUF - 1)), ring[(k + NBUF - 1) % NBUF]);
          consume_rows<RK, RV, GT, U, false>(ring[k], 0, t1, qd, qreg, m, l, acc, zacc);
        }
        i += NBUF;
      }
    }
    // drain: fewer than 2*NBUF-1 tiles left; ring[k] holds tile i+k for k < NBUF-1 (where it exists)
#pragma unroll
    for (int k = 0; k < 2 * NBUF - 2 || k < 1; ++k) {
      if (i + k < n_full) {
        if (NBUF > 1 && i + k + NBUF - 1 < n_full)
          issue_full(row_of_tile((i + k + NBUF - 1)), ring[(k + NBUF - 1) % NBUF]);
        consume_rows<RK, RV, GT, U, false>(ring[k % NBUF], 0, t1, qd, qreg, m, l, acc, zacc);
      }
    }
  }
  if (t0 + n_full * ROWS_PER_WG < t1) {               // ragged tail of the range
    const int row0 = t0 + n_full * ROWS_PER_WG + lane_row;
    issue_tail(row0, ta);
    consume_rows<RK, RV, GT, U, true>(ta, row0, t1, qd, qreg, m, l, acc, zacc);
  }

#if SKV_Q8
  // every channel of a group receives that group's sum of weighted zero points
#pragma unroll
  for (int g = 0; g < GT; ++g)
#pragma unroll
    for (int i = 0; i < VM::CPL; ++i) acc[g][i] += zacc[g][VM::group_of_slot(i)];
#endif

  // ---- merge the 8 octet streams of the wave (lanes 8, 16, 32 apart) ---------------------
#pragma unroll
  for (int a = 0; a < HL; ++a) {
    const float mw = octets_max(m[a]);
    const float f = fast_exp2(m[a] - mw);
    l[a] = octets_sum(l[a] * f);
    m[a] = mw;
#pragma unroll
    for (int half = 0; half < (HS::kSplit ? 2 : 1); ++half) {
      const float fh = half == 0 ? f : dpp_f32<0x141>(f);   // slot HL+a: the mirror lane's head
#pragma unroll
      for (int i = 0; i < VM::CPL; ++i) {
        acc[half * HL + a][i] = octets_sum(acc[half * HL + a][i] * fh);
      }
    }
  }

  // ---- merge the 4 waves through LDS, in wave order -----------------------------------
  if (oct == 0) {
#pragma unroll
    for (int slot = 0; slot < GT; ++slot) {
      float* r = red + (wave * GT + HS::head_of_slot(slot, qd)) * (RV + 2);
#pragma unroll
      for (int i = 0; i < VM::CPL; ++i) r[VM::chan(j, i)] = acc[slot][i];
      if ((j & 3) == 0 && slot < HL) { r[RV] = m[slot]; r[RV + 1] = l[slot]; }
    }
  }
  __syncthreads();
  for (int i = tid; i < GT * (RV + 2); i += kDecodeThreads) {
    const int g = i / (RV + 2), c = i % (RV + 2);
    float mt = red[(0 * GT + g) * (RV + 2) + RV];
#pragma unroll
    for (int w = 1; w < 4; ++w) mt = fmaxf(mt, red[(w * GT + g) * (RV + 2) + RV]);
    if (c == RV) {
      out_ml[g * head_step_ml] = mt;
    } else {
      const int src = c == RV + 1 ? RV + 1 : c;
      float a = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float* r = red + (w * GT + g) * (RV + 2);
        a += r[src] * fast_exp2(r[RV] - mt);
      }
      if (c == RV + 1) out_ml[g * head_step_ml + 1] = a;
      else out_acc[g * head_step_acc + c] = a;
    }
  }
}

#endif  // SKV_VECTOR_KERNEL


#include "skv_decode_mma.inl"

// launches KERNEL<RK, RV, HEADS, format, kind of cache load>
#define SKV_LAUNCH_BY_LOADS(KERNEL, HEADS)                                                           \
  do {                                                                                               \
    if (p.stream_loads) hipLaunchKernelGGL((KERNEL<RK, RV, HEADS, kFmt, true>), grid, block, 0, stream, p);  \
    else hipLaunchKernelGGL((KERNEL<RK, RV, HEADS, kFmt, false>), grid, block, 0, stream, p);       \
  } while (0)

template <int RK, int RV>
hipError_t launch_rv(int heads, const DecodeParams& p, hipStream_t stream) {
  const int passes = p.group / heads;
  const int cols = p.batch * p.n_kv_heads * passes;
  const int fresh_rows = p.T_new > 0 ? (cols + p.n_stream - 1) / p.n_stream : 0;
  const dim3 grid((unsigned)p.n_stream, (unsigned)(cols + fresh_rows));
  const dim3 block(kDecodeThreads);
  if (p.engine == 1) {
    switch (heads) {
      case 1: SKV_LAUNCH_BY_LOADS(decode_partial_mma_kernel, 1); break;
      case 2: SKV_LAUNCH_BY_LOADS(decode_partial_mma_kernel, 2); break;
      case 4: SKV_LAUNCH_BY_LOADS(decode_partial_mma_kernel, 4); break;
      case 8: SKV_LAUNCH_BY_LOADS(decode_partial_mma_kernel, 8); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
#if SKV_VECTOR_KERNEL
  switch (heads) {
    case 1: SKV_LAUNCH_BY_LOADS(decode_partial_kernel, 1); break;
    case 2: SKV_LAUNCH_BY_LOADS(decode_partial_kernel, 2); break;
    case 4: SKV_LAUNCH_BY_LOADS(decode_partial_kernel, 4); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
#else
  return hipErrorInvalidValue;                   // this build holds the matrix-core kernel only
#endif
}

template <int RK>
hipError_t launch_rk(int r_v, int heads, const DecodeParams& p, hipStream_t stream) {
  switch (r_v) {
#if SKV_QBITS == 0
    case 16: return launch_rv<RK, 16>(heads, p, stream);
    case 48: return launch_rv<RK, 48>(heads, p, stream);
    case 80: return launch_rv<RK, 80>(heads, p, stream);
    case 112: return launch_rv<RK, 112>(heads, p, stream);
#endif
#if SKV_QBITS != 4
    case 32: return launch_rv<RK, 32>(heads, p, stream);
    case 96: return launch_rv<RK, 96>(heads, p, stream);
#endif
    case 64: return launch_rv<RK, 64>(heads, p, stream);
    case 128: return launch_rv<RK, 128>(heads, p, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace

#define SKV_CAT2(a, b) a##b
#define SKV_CAT(a, b) SKV_CAT2(a, b)
#if SKV_QBITS == 8 && SKV_PAGED
#define SKV_LAUNCHER_NAME SKV_CAT(launch_decode_partial_paged_q8_rk, SKV_RK)
#elif SKV_QBITS == 4 && SKV_PAGED
#define SKV_LAUNCHER_NAME SKV_CAT(launch_decode_partial_paged_q4_rk, SKV_RK)
#elif SKV_QBITS == 8
#define SKV_LAUNCHER_NAME SKV_CAT(launch_decode_partial_q8_rk, SKV_RK)
#elif SKV_QBITS == 4
#define SKV_LAUNCHER_NAME SKV_CAT(launch_decode_partial_q4_rk, SKV_RK)
#elif SKV_PAGED
#define SKV_LAUNCHER_NAME SKV_CAT(launch_decode_partial_paged_rk, SKV_RK)
#else
#define SKV_LAUNCHER_NAME SKV_CAT(launch_decode_partial_rk, SKV_RK)
#endif
hipError_t SKV_LAUNCHER_NAME(int r_v, int heads, const DecodeParams& p, hipStream_t stream) {
  return launch_rk<SKV_RK>(r_v, heads, p, stream);
}

}  // namespace skv
