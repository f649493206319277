// Internal declarations shared by the host layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skv.h"

namespace skv {

// Arguments of the decode kernels (passed by value).
struct DecodeParams {
  const uint32_t* k_cache;   // bf16 pairs
  const uint32_t* v_cache;
  const uint16_t* p_k;
  const uint16_t* p_v;
  const uint16_t* q;
  float* part_acc;           // [batch][n_q_heads][n_splits][r_v]
  float* part_ml;            // [batch][n_q_heads][n_splits][2]  (max in log2 units, normaliser)
  float* out;                // [batch][n_q_heads][128]
  int64_t capacity;
  int64_t p_k_head_stride;
  int64_t p_v_head_stride;
  int32_t batch, n_q_heads, n_kv_heads, group;
  int32_t r_k, r_v;
  int32_t n_ctx;
  int32_t n_splits;
  int32_t chunk;             // tokens per split (multiple of kChunkQuantum)
  float scale_log2e;         // softmax scale times log2(e)
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
  int32_t batch, n_kv_heads;
  int32_t r_k, r_v;
  int32_t T;
};

constexpr int kChunkQuantum = 256;   // every split but the last covers a multiple of this many tokens
constexpr int kDecodeThreads = 256;

// Chooses (n_splits, chunk) for a context of n_ctx tokens.  want <= 0: heuristic.
// Returns false if `want` cannot be honoured.
bool plan_splits(int32_t batch, int32_t n_kv_heads, int32_t group, int64_t n_ctx,
                 int32_t want, int32_t* n_splits, int32_t* chunk);

// Heads of one KV group handled per workgroup pass (1, 2 or 4).
inline int heads_per_pass(int group) { return group >= 4 ? 4 : group; }

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

hipError_t launch_decode_combine(const DecodeParams& p, hipStream_t stream);
hipError_t launch_append(const AppendParams& p, hipStream_t stream);

}  // namespace skv
