// Internal declarations shared by the host layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skv.h"

namespace skv {

// Where the rows of a sequence live.  table == null: one contiguous run of `capacity` rows per
// (sequence, KV head).  Otherwise the cache is a pool of pages [n_pages][n_kv_heads][page rows][r] and
// table[b * table_stride + i] names the page that holds rows [i << page_shift, (i + 1) << page_shift) of
// sequence b; entries are clamped into [0, n_pages) so that no access leaves the pool.
struct PageMap {
  const int32_t* table;
  int32_t table_stride;
  int32_t page_shift;
  int32_t n_pages;
};

__device__ __forceinline__ int clamped_page(const PageMap& pm, int b, int logical_page) {
  const int v = pm.table[(int64_t)b * pm.table_stride + logical_page];
  return v < 0 ? 0 : (v >= pm.n_pages ? pm.n_pages - 1 : v);
}

// Index, in rows, of row t of (sequence b, KV head kv); multiply by the row width.
__device__ __forceinline__ int64_t cache_row(const PageMap& pm, int64_t capacity, int n_kv_heads, int b, int kv,
                                             int64_t t) {
  if (pm.table == nullptr) return ((int64_t)b * n_kv_heads + kv) * capacity + t;
  const int page = clamped_page(pm, b, (int)(t >> pm.page_shift));
  return ((((int64_t)page * n_kv_heads + kv)) << pm.page_shift) + (t & ((1 << pm.page_shift) - 1));
}

// Arguments of the decode kernels (passed by value).
struct DecodeParams {
  const uint32_t* k_cache;   // bf16 pairs
  const uint32_t* v_cache;
  const uint16_t* p_k;
  const uint16_t* p_v;
  const uint16_t* q;
  float* part_acc;           // [batch][n_q_heads][n_splits][r_v]
  float* part_ml;            // [batch][n_q_heads][n_splits][2]  (max in log2 units, normaliser)
  float* qt;                 // [batch][n_q_heads][r_k]: projected query times scale*log2(e)
  // 8-bit quantised cache only (null otherwise)
  const float* k_scale;      // [n_kv_heads][groups of r_k]: static key scales, folded into qt
  const float* k_zero;       // the matching zero points: only a fused step over a quantised cache needs them (new rows)
  const uint32_t* v_meta;    // [batch][n_kv_heads][capacity][groups of r_v]: bf16 scale | bf16 zero << 16
  float* out;                // [batch][n_q_heads][128]
  int64_t capacity;
  int64_t p_k_head_stride;
  int64_t p_v_head_stride;
  int32_t batch, n_q_heads, n_kv_heads, group;
  int32_t r_k, r_v;
  int32_t n_ctx;             // cache rows the context ranges cover
  int32_t n_splits;          // partial results per (sequence, head): what the combine kernel merges
  int32_t n_stream;          // context ranges over [0, n_ctx); n_splits - 1 when a fresh-rows block is added
  // Fused decode step (bf16 cache): the range kernel projects the queries itself (q != null) and one extra
  // workgroup per (sequence, KV head, pass) projects, stores and attends the T_new new rows [cur_len, cur_len + T_new).
  const uint16_t* k_new;
  const uint16_t* v_new;
  uint16_t* k_cache_w;
  uint16_t* v_cache_w;
  int64_t stride_b, stride_t, stride_h;
  int64_t cur_len;
  int32_t T_new;
  // Per-sequence lengths (device int32 [batch]) or null: sequence b then attends rows [0, len_b) with
  // len_b = seq_lens[b] clamped into [0, n_ctx]; in a fused step len_b is also where its new rows go.
  const int32_t* seq_lens;
  int32_t len_add;           // rows added to every per-sequence length (an append that ran just before): len_b =
                             // clamp(seq_lens[b], 0, n_ctx - len_add) + len_add
  PageMap pages;             // paged cache: k_cache / v_cache are the pools
  int32_t engine;            // range kernel over bf16 rows: 0 = vector arithmetic, 1 = matrix cores
  int32_t stream_loads;      // 1: the full tiles of the range kernel are read with streaming (non-temporal) loads,
                             // for rows that will not be found in a cache again anyway; 0: ordinary loads
  float scale_log2e;         // softmax scale times log2(e)
  int32_t lift;              // combine: 1 = multiply by P_V^T into out [..][128]; 0 = leave rank-r_v coordinates in out [..][r_v]
};

// Arguments of the append kernels.
struct AppendParams {
  uint16_t* k_cache;
  uint16_t* v_cache;
  const uint16_t* p_k;
  const uint16_t* p_v;
  const uint16_t* k_new;
  const uint16_t* v_new;
  int64_t capacity;
  int64_t p_k_head_stride;
  int64_t p_v_head_stride;
  int64_t stride_b, stride_t, stride_h;
  int64_t cur_len;
  const int32_t* cur_lens;   // device int32 [batch] or null: per-sequence first row, clamped into [0, cur_len]
  int32_t batch, n_kv_heads;
  int32_t r_k, r_v;
  int32_t T;
  // quantised cache only (null otherwise): the caches then hold qbits-wide codes (8: one byte per channel;
  // 4: two channels per byte, the even one in the low half)
  const float* k_scale;      // [n_kv_heads][groups of r_k]
  const float* k_zero;
  uint32_t* v_meta;          // [batch][n_kv_heads][capacity][groups of r_v]
  int32_t qbits;
  PageMap pages;             // paged cache (bf16 only): k_cache / v_cache are the pools
};

// Length of sequence b: the uniform value, or the per-sequence one clamped into [0, uniform].
__host__ __device__ inline int64_t clamped_len(const int32_t* lens, int b, int64_t uniform) {
  if (!lens) return uniform;
  const int64_t v = lens[b];
  return v < 0 ? 0 : (v > uniform ? uniform : v);
}

// Heads of one KV group handled per workgroup pass (1, 2 or 4).
inline int heads_per_pass(int group) { return group >= 4 ? 4 : group; }

// Arguments of the chunk (prefill) attention kernel.
struct PrefillParams {
  const uint16_t* k_cache;
  const uint16_t* v_cache;
  const uint16_t* p_k;       // unused when folded
  const uint16_t* p_v;
  const uint16_t* q;         // bf16; element (b,t,h,i) at b*q_stride_b + t*q_stride_t + h*q_stride_h + i,
                             // or packed [batch][T][n_q_heads][r_k] when folded
  float* out;                // [batch][T][n_q_heads][128], or [..][r_v] when folded
  int64_t capacity;
  int64_t p_k_head_stride;
  int64_t p_v_head_stride;
  int64_t q_stride_b, q_stride_t, q_stride_h;
  int32_t batch, n_q_heads, n_kv_heads, group;
  int32_t T;                 // tokens of the chunk
  int32_t n_prev;            // cache rows before the chunk; the chunk's own rows are already cached
  int32_t n_tiles;           // token tiles per (sequence, KV head, pass)
  int32_t n_rows_y;          // batch * n_kv_heads * passes
  float scale_log2e;
  int32_t folded;
  PageMap pages;             // paged cache: k_cache / v_cache are the pools; a key tile never straddles a page
};

constexpr int kPrefillKeyTile = 64;     // cache rows staged in LDS per step
constexpr int kPrefillThreads = 256;
// Paged chunk attention keeps one table entry per key tile in LDS: contexts up to this many rows.
constexpr int64_t kPagedPrefillMaxRows = (int64_t)kPrefillKeyTile * 16384;
// Tokens of the chunk handled by one workgroup: 4 waves of 32 query rows, split over
// min(G, 4) heads of the group.
inline int prefill_tile_tokens(int group) { return 32 * (4 / heads_per_pass(group)); }

// The context is cut into quanta of this many rows; a range is a run of whole quanta (the last
// one may be ragged), and the ranges of a call differ by at most one quantum.
constexpr int kRangeQuantum = 64;
constexpr int kDecodeThreads = 256;

// Number of context ranges for n_ctx tokens of this layer (bits: 0 for bf16 rows, else the width of the
// quantised codes; paged_codes: quantised rows in pages).  want <= 0: heuristic.  Returns false if `want`
// is out of range.
bool plan_splits(const skv_layer* L, int64_t n_ctx, int32_t want, int32_t* n_splits, int bits = 0,
                 bool paged_codes = false);

// Bytes of workspace skv_decode_attention uses for n_ctx rows of this layer (its own range plan; at most
// skv_decode_workspace_bytes).  Validates the layer and n_ctx as that call does.
skv_status decode_attention_workspace_need(const skv_layer* L, int64_t n_ctx, size_t* bytes);

// Rows [t0, t1) of range `split` out of n_splits over n_ctx rows: whole quanta, dealt as evenly
// as possible (the first `rem` ranges get one more); empty when t0 >= t1.
__host__ __device__ inline void range_of_split(int n_ctx, int n_splits, int split, int* t0, int* t1) {
  const int quanta = (n_ctx + kRangeQuantum - 1) / kRangeQuantum;
  const int q = quanta / n_splits, rem = quanta % n_splits;
  const int first = split * q + (split < rem ? split : rem);
  const int count = q + (split < rem ? 1 : 0);
  *t0 = first * kRangeQuantum;
  const int end = (first + count) * kRangeQuantum;
  *t1 = end < n_ctx ? end : n_ctx;
}


// Launchers defined in the kernel translation units.  One per key rank.
typedef hipError_t (*decode_partial_launcher)(int r_v, int heads, const DecodeParams& p,
                                              hipStream_t stream);
hipError_t launch_decode_partial_rk16(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_rk32(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_rk48(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_rk64(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_rk80(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_rk96(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_rk112(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_rk128(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_rk16(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_rk32(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_rk48(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_rk64(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_rk80(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_rk96(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_rk112(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_rk128(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_q8_rk32(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_q8_rk64(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_q8_rk96(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_q8_rk128(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_q4_rk64(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_q4_rk128(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_q8_rk32(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_q8_rk64(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_q8_rk96(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_q8_rk128(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_q4_rk64(int, int, const DecodeParams&, hipStream_t);
hipError_t launch_decode_partial_paged_q4_rk128(int, int, const DecodeParams&, hipStream_t);

// sched: 0 = the default schedule for the shape, 1 = keys and values staged together, 2 = keys a tile ahead
typedef hipError_t (*prefill_launcher)(int r_v, int sched, const PrefillParams& p, hipStream_t stream);
hipError_t launch_prefill_rk16(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_rk32(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_rk48(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_rk64(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_rk80(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_rk96(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_rk112(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_rk128(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_paged_rk16(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_paged_rk32(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_paged_rk48(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_paged_rk64(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_paged_rk80(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_paged_rk96(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_paged_rk112(int, int, const PrefillParams&, hipStream_t);
hipError_t launch_prefill_paged_rk128(int, int, const PrefillParams&, hipStream_t);

hipError_t launch_decode_combine(const DecodeParams& p, hipStream_t stream);
// dst [rows][r_pad] = src [rows][r] followed by zero columns (bf16 bit patterns)
hipError_t launch_pad_basis(const void* src, void* dst, int r, int r_pad, int64_t rows, hipStream_t stream);
// out bf16 [n][128][r_out]: leading r columns of the orthonormal factor of a float32 [n][128][128], zero columns behind
hipError_t launch_orthonormalize(const void* a, void* out, int n, int r, int r_out, hipStream_t stream);
hipError_t launch_append(const AppendParams& p, hipStream_t stream);
// Folded-weights variant: rows that arrive already projected.
hipError_t launch_copy_projected(const AppendParams& p, hipStream_t stream);      // k_new / v_new are [b][t][h][r] packed
hipError_t launch_scale_query(const DecodeParams& p, hipStream_t stream);        // q is [b][h_q][r_k]
hipError_t launch_folded_prepare(const AppendParams& ap, const DecodeParams& dp, hipStream_t stream);  // both, one launch

// Few-token appends (ap) and query projections (dp) in one launch; either may be null.
hipError_t launch_project(const AppendParams* ap, const DecodeParams* dp, hipStream_t stream);

// New tokens per sequence up to which a decode step folds its append into the range kernel.
constexpr int kFusedStepMaxTokens = 4;

// Token rows (batch * T) up to which an append runs as vector projections.
constexpr int kVectorAppendMaxRows = 64;

}  // namespace skv
