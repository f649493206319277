// Host layer of the C ABI: argument checks, launch planning, rank selection.
// No device code here.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>

#include "skv_internal.h"

namespace skv {

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Softmax scale times log2(e); scale <= 0 selects 1/sqrt(head_dim), the ORIGINAL head dimension.
float scale_log2e_of(float scale) {
  const double sc = scale > 0.f ? (double)scale : 1.0 / std::sqrt((double)SKV_HEAD_DIM);
  return (float)(sc * 1.4426950408889634);
}

bool rank_ok(int32_t r) { return r >= 16 && r <= SKV_HEAD_DIM && (r % 16) == 0; }

// Workgroups the streaming launch aims for: two per compute unit of the 256-CU part.  Each
// workgroup keeps enough loads in flight by itself (it requests a tile ahead), so more
// workgroups only add per-workgroup start-up and merge cost; measured at batch 4 / 32K context,
// 8 or 16 ranges per (sequence, KV head) are the fastest, 32 and 64 are slower.
constexpr int kTargetWorkgroups = 512;

// Which range kernel streams the cache of this layer: 0 = vector arithmetic, 1 = matrix cores.  The layer's
// SKV_ENGINE_* flag decides when set.  By shape, the matrix kernel where it saves a pass over the cache (eight
// query heads per KV head) and over the quantised formats (bits = width of the codes, 0 for bf16 rows: there it
// needs fewer vector instructions per row, which is what bounds both kernels: measured 31.4 against 35.2 us at
// 8 bits); for bf16 rows in groups of four with both ranks 32 or 64 as well: measured 2-5 % ahead of the vector
// kernel there with either kind of load (b4/32K 64/64: 40.3 against 41.3 us per launch on one machine) and level
// at short contexts; level or behind at ranks 48, 80, 96, 128 (128/128 with streaming loads: 107 against 93 us),
// behind without grouping, and behind by 5-9 % for groups of two below 8K rows.  Quantised rows in pages are
// served by the matrix kernel only.
int engine_for(const skv_layer* L, int bits = 0, bool paged_codes = false) {
  if (paged_codes) return 1;
  const uint32_t want = L->flags & SKV_ENGINE_MASK;
  const int group = L->n_q_heads / L->n_kv_heads;
  if (want == SKV_ENGINE_VECTOR) return 0;
  if (want == SKV_ENGINE_MATRIX) return 1;
  if (group == 8 || bits != 0) return 1;
  // Measured per rank pair with rows that come from HBM alone (layers flagged SKV_READS_STREAMING, rotated over
  // more caches than the last-level cache holds; b4/32K, us per launch, vector / matrix): 32/32 26.2 / 26.8,
  // 32/64 36.3 / 35.2, 32/128 55.6 / 54.4, 48/32 30.9 / 33.0, 48/48 34.9 / 41.5, 48/64 39.5 / 39.3, 64/32 34.9 /
  // 39.9, 64/64 44.6 / 44.7, 64/96 55.0 / 58.2, 64/128 65.2 / 63.4; 96/64 55.4 / 66.5, 128/96 74.0 / 108.
  // Such layers take the matrix kernel where it is ahead by more than the 1 us these figures move from machine
  // to machine; the matrix kernel also keeps the small ranks of layers whose rows are re-read from the
  // last-level cache (level or up to 1 us ahead there).
  if ((L->flags & SKV_READS_MASK) == SKV_READS_STREAMING) {
    const bool ahead = group == 4 && ((L->r_v == 128 && (L->r_k == 32 || L->r_k == 64)) || (L->r_k == 32 && L->r_v == 64));
    return ahead ? 1 : 0;
  }
  const bool small_pow2 = (L->r_k == 32 || L->r_k == 64) && (L->r_v == 32 || L->r_v == 64);
  return (group == 4 && small_pow2) ? 1 : 0;
}

// How the range kernels read cache rows: 1 = streaming loads, 0 = ordinary loads.  The layer's SKV_READS_* flag
// decides when set.  By size: a launch whose rows add up to clearly more than the 256 MiB last-level cache cannot
// find them there on the next step and reads them with streaming loads (measured 8-10 % faster from 0.4 to
// 10 GB per launch); one that fits, or nearly fits, keeps ordinary loads (rows re-read step after step are
// partly served from that cache: at 256 MiB ordinary loads are 2 % ahead, at 288 MiB streaming ones 1 %,
// at 384 MiB 10 %).  A caller whose layers together exceed that cache sets SKV_READS_STREAMING on each.
constexpr int64_t kStreamAboveBytes = 288ll << 20;
int32_t stream_loads_for(const skv_layer* L, int64_t n_ctx, int bits = 0) {
  const uint32_t want = L->flags & SKV_READS_MASK;
  if (want == SKV_READS_STREAMING) return 1;
  if (want == SKV_READS_CACHED) return 0;
  const int64_t row_bits = (int64_t)(L->r_k + L->r_v) * (bits ? bits : 16);
  return (int64_t)L->batch * L->n_kv_heads * n_ctx * row_bits / 8 > kStreamAboveBytes ? 1 : 0;
}

// Query heads of a KV group one workgroup of the range kernel serves.  The vector kernel takes up to four (a
// group of eight streams the cache twice); the matrix kernel has the columns for all eight in one pass.
int decode_heads_per_pass(const skv_layer* L, int bits = 0, bool paged_codes = false) {
  const int group = L->n_q_heads / L->n_kv_heads;
  return (group == 8 && engine_for(L, bits, paged_codes) == 1) ? 8 : heads_per_pass(group);
}

// need_bases = false: the folded-weights entry points, which never touch p_k / p_v.
skv_status check_layer(const skv_layer* L, bool need_bases = true) {
  if (!L) return SKV_ERR_NULL;
  if (!L->k_cache || !L->v_cache) return SKV_ERR_NULL;
  if (need_bases && (!L->p_k || !L->p_v)) return SKV_ERR_NULL;
  if (L->head_dim != SKV_HEAD_DIM) return SKV_ERR_SHAPE;
  if (L->batch < 1 || L->n_kv_heads < 1 || L->n_q_heads < 1) return SKV_ERR_SHAPE;
  if (L->n_q_heads % L->n_kv_heads) return SKV_ERR_SHAPE;
  const int g = L->n_q_heads / L->n_kv_heads;
  if (!(g == 1 || g == 2 || g == 4 || g == 8)) return SKV_ERR_SHAPE;
  // one grid row per (sequence, KV head, pass) in the streaming launch: the grid's y limit
  if ((int64_t)L->batch * L->n_kv_heads * (g / heads_per_pass(g)) > 65535) return SKV_ERR_SHAPE;
  if (!rank_ok(L->r_k) || !rank_ok(L->r_v)) return SKV_ERR_RANK;
  if ((L->flags & ~(SKV_READS_MASK | SKV_ENGINE_MASK)) || L->reserved != 0) return SKV_ERR_SHAPE;
  if ((L->flags & SKV_READS_MASK) == SKV_READS_MASK || (L->flags & SKV_ENGINE_MASK) == SKV_ENGINE_MASK) return SKV_ERR_SHAPE;
  if (L->capacity < 1 || L->capacity > std::numeric_limits<int32_t>::max()) return SKV_ERR_CAPACITY;
  const int64_t sk = L->p_k_head_stride, sv = L->p_v_head_stride;
  if (need_bases && sk != 0 && sk < (int64_t)SKV_HEAD_DIM * L->r_k) return SKV_ERR_SHAPE;
  if (need_bases && sv != 0 && sv < (int64_t)SKV_HEAD_DIM * L->r_v) return SKV_ERR_SHAPE;
  if (need_bases && ((sk % 8) || (sv % 8))) return SKV_ERR_ALIGN;
  if (!aligned16(L->k_cache) || !aligned16(L->v_cache)) return SKV_ERR_ALIGN;
  if (need_bases && (!aligned16(L->p_k) || !aligned16(L->p_v))) return SKV_ERR_ALIGN;
  return SKV_OK;
}

size_t align256(size_t x) { return (x + 255u) & ~(size_t)255u; }

// Workspace layout (bytes): [projected queries][partial mixes][partial max/normaliser].  The
// first block does not depend on the split count, so it can be filled before that is known.
size_t qt_bytes(const skv_layer* L) {
  return align256((size_t)L->batch * L->n_q_heads * (size_t)L->r_k * sizeof(float));
}
size_t workspace_need(const skv_layer* L, int32_t n_splits) {
  return qt_bytes(L) +
         (size_t)L->batch * L->n_q_heads * (size_t)n_splits * (size_t)(L->r_v + 2) * sizeof(float);
}

void fill_decode_params(const skv_layer* L, DecodeParams* p, int32_t n_splits, void* workspace) {
  p->k_cache = static_cast<const uint32_t*>(L->k_cache);
  p->v_cache = static_cast<const uint32_t*>(L->v_cache);
  p->p_k = static_cast<const uint16_t*>(L->p_k);
  p->p_v = static_cast<const uint16_t*>(L->p_v);
  p->q = nullptr;
  p->out = nullptr;
  p->capacity = L->capacity;
  p->p_k_head_stride = L->p_k_head_stride;
  p->p_v_head_stride = L->p_v_head_stride;
  p->batch = L->batch;
  p->n_q_heads = L->n_q_heads;
  p->n_kv_heads = L->n_kv_heads;
  p->group = L->n_q_heads / L->n_kv_heads;
  p->r_k = L->r_k;
  p->r_v = L->r_v;
  p->n_ctx = 0;
  p->n_splits = n_splits;
  p->n_stream = n_splits;
  p->k_new = nullptr;
  p->v_new = nullptr;
  p->k_cache_w = static_cast<uint16_t*>(L->k_cache);
  p->v_cache_w = static_cast<uint16_t*>(L->v_cache);
  p->stride_b = p->stride_t = p->stride_h = 0;
  p->cur_len = 0;
  p->T_new = 0;
  p->seq_lens = nullptr;
  p->len_add = 0;
  p->pages = PageMap{nullptr, 0, 0, 0};
  p->engine = engine_for(L);
  p->stream_loads = 0;
  p->scale_log2e = 0.f;
  p->lift = 1;
  p->k_scale = nullptr;
  p->k_zero = nullptr;
  p->v_meta = nullptr;
  char* ws = static_cast<char*>(workspace);
  p->qt = reinterpret_cast<float*>(ws);
  p->part_acc = reinterpret_cast<float*>(ws + qt_bytes(L));
  p->part_ml = p->part_acc + (size_t)L->batch * L->n_q_heads * (size_t)n_splits * (size_t)L->r_v;
}

decode_partial_launcher partial_launcher_for(int r_k) {
  switch (r_k) {
    case 16: return launch_decode_partial_rk16;
    case 32: return launch_decode_partial_rk32;
    case 48: return launch_decode_partial_rk48;
    case 64: return launch_decode_partial_rk64;
    case 80: return launch_decode_partial_rk80;
    case 96: return launch_decode_partial_rk96;
    case 112: return launch_decode_partial_rk112;
    case 128: return launch_decode_partial_rk128;
  }
  return nullptr;
}

decode_partial_launcher paged_partial_launcher_for(int r_k) {
  switch (r_k) {
    case 16: return launch_decode_partial_paged_rk16;
    case 32: return launch_decode_partial_paged_rk32;
    case 48: return launch_decode_partial_paged_rk48;
    case 64: return launch_decode_partial_paged_rk64;
    case 80: return launch_decode_partial_paged_rk80;
    case 96: return launch_decode_partial_paged_rk96;
    case 112: return launch_decode_partial_paged_rk112;
    case 128: return launch_decode_partial_paged_rk128;
  }
  return nullptr;
}

skv_status check_decode_common(const skv_layer* L, int32_t n_splits, const void* workspace,
                               size_t workspace_bytes) {
  if (!workspace) return SKV_ERR_NULL;
  if (!aligned16(workspace)) return SKV_ERR_ALIGN;
  if (n_splits < 1 || n_splits > SKV_MAX_SPLITS) return SKV_ERR_SHAPE;
  if (workspace_bytes < workspace_need(L, n_splits)) return SKV_ERR_WORKSPACE;
  return SKV_OK;
}

}  // namespace

// Workgroups a range launch aims for.  The matrix kernel over a quantised cache is bound by instruction issue
// and by the latency of its chain of dependent steps, which more resident waves help: as many workgroups as a
// CU holds at once (four with both ranks up to 64, where the kernel is built for 128 registers per lane, three
// beyond; measured for b4/32K, 64/64, 8-bit: 26.2 us in 32 ranges against 28.4 in 24, where the bf16 kernels
// want 8..16).
bool fills_every_slot(const skv_layer* L, int bits, bool paged_codes) {
  return bits != 0 && engine_for(L, bits, paged_codes) == 1;
}
int64_t workgroup_target(const skv_layer* L, int bits, bool paged_codes) {
  if (!fills_every_slot(L, bits, paged_codes)) return kTargetWorkgroups;
  return (L->r_k <= 64 && L->r_v <= 64) ? 2 * kTargetWorkgroups : 3 * kTargetWorkgroups / 2;
}

bool plan_splits(const skv_layer* L, int64_t n_ctx, int32_t want, int32_t* n_splits, int bits, bool paged_codes) {
  const int32_t batch = L->batch, n_kv_heads = L->n_kv_heads, group = L->n_q_heads / L->n_kv_heads;
  if (n_ctx < 1 || n_ctx > std::numeric_limits<int32_t>::max() - kRangeQuantum) return false;
  if (want > 0) {
    if (want > SKV_MAX_SPLITS) return false;
    *n_splits = want;
    return true;
  }
  const int64_t quanta = (n_ctx + kRangeQuantum - 1) / kRangeQuantum;
  const int64_t columns = (int64_t)batch * n_kv_heads * (group / decode_heads_per_pass(L, bits, paged_codes));
  const int64_t target = workgroup_target(L, bits, paged_codes);
  int64_t s = (target + columns - 1) / (columns > 0 ? columns : 1);
  if (s > SKV_MAX_SPLITS) s = SKV_MAX_SPLITS;
  if (s > quanta) s = quanta;                 // never a range without rows
  if (s < 1) s = 1;
  // Short ranges do not pay: a workgroup's start-up (query projection, first round trip) and its merge cost
  // about as much as streaming a thousand rows.  More than one workgroup per CU only while each still has
  // 1024 rows, and no range of a single 64-row tile while more than a quarter of the CUs stay busy (measured
  // for one sequence, 64/64: 32K rows 22.3 us in 32 ranges against 24.4 in 64; 4K rows 11.9 in 32 against 14.4
  // in 64; four sequences of 8K rows: 21.1 in 8 against 22.4 in 16; 8-bit codes, one sequence of 16K rows:
  // 18.0 in 32 against 21.8 in 96).
  const int64_t one_per_cu = std::max<int64_t>(1, (kTargetWorkgroups / 2) / (columns > 0 ? columns : 1));
  const int64_t by_rows = quanta / 16;
  if (s > by_rows) s = std::max(by_rows, std::min(s, one_per_cu));
  while (s > 1 && quanta / s < 2 && s * columns > kTargetWorkgroups / 8) s = (s + 1) / 2;
  if (s < 1) s = 1;
  *n_splits = (int32_t)s;
  return true;
}

// A fused step launches, beside its columns x ranges workgroups, the ones that take the step's new rows (in
// rows of `ranges` workgroups).  Where the plan already fills every slot the CUs have, those would wait for a
// slot and finish last (measured b4/32K 64/64 8-bit: 31.0 us against 27.0 for the same launch without them):
// fewer ranges, so that all are resident from the start.
void leave_room_for_new_rows(const skv_layer* L, int bits, bool paged_codes, int32_t* s) {
  if (!fills_every_slot(L, bits, paged_codes)) return;
  const int64_t columns = (int64_t)L->batch * L->n_kv_heads *
                          ((L->n_q_heads / L->n_kv_heads) / decode_heads_per_pass(L, bits, paged_codes));
  const int64_t target = workgroup_target(L, bits, paged_codes);
  while (*s > 1 && (columns + (columns + *s - 1) / *s) * *s > target) --*s;
}

skv_status decode_attention_workspace_need(const skv_layer* L, int64_t n_ctx, size_t* bytes) {
  const skv_status st = check_layer(L);
  if (st != SKV_OK) return st;
  if (n_ctx < 1 || n_ctx > L->capacity) return SKV_ERR_CAPACITY;
  int32_t s = 0;
  if (!plan_splits(L, n_ctx, 0, &s)) return SKV_ERR_SHAPE;
  *bytes = workspace_need(L, s);
  return SKV_OK;
}

}  // namespace skv

using namespace skv;

extern "C" {

const char* skv_status_string(skv_status s) {
  switch (s) {
    case SKV_OK: return "SKV_OK";
    case SKV_ERR_NULL: return "SKV_ERR_NULL";
    case SKV_ERR_SHAPE: return "SKV_ERR_SHAPE";
    case SKV_ERR_RANK: return "SKV_ERR_RANK";
    case SKV_ERR_CAPACITY: return "SKV_ERR_CAPACITY";
    case SKV_ERR_ALIGN: return "SKV_ERR_ALIGN";
    case SKV_ERR_WORKSPACE: return "SKV_ERR_WORKSPACE";
    case SKV_ERR_BUDGET: return "SKV_ERR_BUDGET";
    case SKV_ERR_HIP: return "SKV_ERR_HIP";
  }
  return "SKV_ERR_UNKNOWN";
}

int32_t skv_decode_engine_for(const skv_layer* L, int32_t code_bits) {
  if (check_layer(L, false) != SKV_OK) return -1;
  if (code_bits != 0 && code_bits != 8 && code_bits != 4) return -1;
  return engine_for(L, code_bits);
}

int32_t skv_decode_streams_rows(const skv_layer* L, int64_t n_ctx, int32_t code_bits) {
  if (check_layer(L, false) != SKV_OK) return -1;
  if (code_bits != 0 && code_bits != 8 && code_bits != 4) return -1;
  if (n_ctx < 1 || n_ctx > L->capacity) return -1;
  return stream_loads_for(L, n_ctx, code_bits);
}

size_t skv_cache_bytes(const skv_layer* L, int64_t n_tokens) {
  if (!L || n_tokens < 0) return 0;
  return (size_t)L->batch * L->n_kv_heads * (size_t)n_tokens * (size_t)(L->r_k + L->r_v) * 2u;
}

size_t skv_decode_workspace_bytes(const skv_layer* L) {
  if (check_layer(L) != SKV_OK) return 0;
  return workspace_need(L, SKV_MAX_SPLITS);
}

skv_status skv_decode_range(int64_t n_ctx, int32_t n_splits, int32_t range, int64_t* first_row,
                            int64_t* end_row) {
  if (!first_row || !end_row) return SKV_ERR_NULL;
  if (n_ctx < 1 || n_ctx > std::numeric_limits<int32_t>::max() - kRangeQuantum) return SKV_ERR_CAPACITY;
  if (n_splits < 1 || n_splits > SKV_MAX_SPLITS || range < 0 || range >= n_splits) return SKV_ERR_SHAPE;
  int t0 = 0, t1 = 0;
  range_of_split((int)n_ctx, n_splits, range, &t0, &t1);
  if (t0 > t1) t0 = t1;
  *first_row = t0;
  *end_row = t1;
  return SKV_OK;
}

int32_t skv_decode_default_splits(const skv_layer* L, int64_t n_ctx) {
  if (check_layer(L) != SKV_OK) return 0;
  if (n_ctx < 1 || n_ctx > L->capacity) return 0;
  int32_t s = 0;
  if (!plan_splits(L, n_ctx, 0, &s)) return 0;
  return s;
}

}  // extern "C"

namespace {

// ---- checks (no side effects) ---------------------------------------------------------------

skv_status check_query_stage(const skv_layer* L, const void* q, float scale, const void* workspace,
                             size_t workspace_bytes) {
  skv_status st = check_layer(L);
  if (st != SKV_OK) return st;
  if (!q || !workspace) return SKV_ERR_NULL;
  if (!aligned16(q) || !aligned16(workspace)) return SKV_ERR_ALIGN;
  if (!(scale == scale) || std::isinf(scale)) return SKV_ERR_SHAPE;
  if (workspace_bytes < workspace_need(L, 1)) return SKV_ERR_WORKSPACE;
  return SKV_OK;
}

skv_status check_partial_stage(const skv_layer* L, int64_t n_ctx, int32_t n_splits,
                               const void* workspace, size_t workspace_bytes, int32_t* s_out, int bits = 0,
                               bool paged_codes = false) {
  skv_status st = check_layer(L);
  if (st != SKV_OK) return st;
  if (n_ctx < 1 || n_ctx > L->capacity) return SKV_ERR_CAPACITY;
  if (n_splits > SKV_MAX_SPLITS) return SKV_ERR_SHAPE;
  if (!plan_splits(L, n_ctx, n_splits, s_out, bits, paged_codes))
    return SKV_ERR_SHAPE;
  return check_decode_common(L, *s_out, workspace, workspace_bytes);
}

skv_status check_combine_stage(const skv_layer* L, const void* out, int32_t n_splits,
                               const void* workspace, size_t workspace_bytes) {
  skv_status st = check_layer(L);
  if (st != SKV_OK) return st;
  if (!out) return SKV_ERR_NULL;
  if (!aligned16(out)) return SKV_ERR_ALIGN;
  return check_decode_common(L, n_splits, workspace, workspace_bytes);
}

skv_status check_append(const skv_layer* L, const void* k_new, const void* v_new, int64_t stride_b,
                        int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len) {
  skv_status st = check_layer(L);
  if (st != SKV_OK) return st;
  if (T < 0) return SKV_ERR_SHAPE;
  if (cur_len < 0 || cur_len + (int64_t)T > L->capacity) return SKV_ERR_CAPACITY;
  if (T == 0) return SKV_OK;
  if (!k_new || !v_new) return SKV_ERR_NULL;
  if (stride_b < 0 || stride_t < 0 || stride_h < 0) return SKV_ERR_SHAPE;
  if ((int64_t)L->batch * T > std::numeric_limits<int32_t>::max() / 64) return SKV_ERR_SHAPE;
  if ((stride_b % 8) || (stride_t % 8) || (stride_h % 8)) return SKV_ERR_ALIGN;
  if (!aligned16(k_new) || !aligned16(v_new)) return SKV_ERR_ALIGN;
  return SKV_OK;
}

// Everything skv_decode_attention needs checked before its first launch; *n_splits: the range plan.
skv_status check_decode_attention(const skv_layer* L, const void* q, const void* out, int64_t n_ctx, float scale,
                                  const void* workspace, size_t workspace_bytes, int32_t* n_splits) {
  skv_status st = check_query_stage(L, q, scale, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  st = check_partial_stage(L, n_ctx, 0, workspace, workspace_bytes, n_splits);
  if (st != SKV_OK) return st;
  return check_combine_stage(L, out, *n_splits, workspace, workspace_bytes);
}

// How a decode step runs: fused (the new rows are projected, stored and attended by workgroups of the range
// launch: two launches) or as append + attention; n_splits: partial results the merge reads.
struct StepPlan {
  bool fused = false;
  int32_t n_splits = 0;
};

skv_status check_decode_step(const skv_layer* L, const void* k_new, const void* v_new, int64_t stride_b,
                             int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len, const void* q,
                             const void* out, float scale, const void* workspace, size_t workspace_bytes,
                             StepPlan* plan) {
  skv_status st = check_append(L, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
  if (st != SKV_OK) return st;
  int32_t s = 0;
  st = check_decode_attention(L, q, out, cur_len + T, scale, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  plan->fused = false;
  plan->n_splits = s;
  const int gq = L->n_q_heads / L->n_kv_heads;
  // (the fused launch adds up to one grid row per column: stay inside the grid's y limit)
  const bool grid_ok = 2 * (int64_t)L->batch * L->n_kv_heads * (gq / decode_heads_per_pass(L)) <= 65535;
  if (T > 0 && T <= kFusedStepMaxTokens && cur_len > 0 && grid_ok) {
    int32_t s_old = 0;
    if (!plan_splits(L, cur_len, 0, &s_old)) return SKV_ERR_SHAPE;
    if (s_old + 1 > SKV_MAX_SPLITS) s_old = SKV_MAX_SPLITS - 1;
    if (workspace_bytes < workspace_need(L, s_old + 1)) return SKV_ERR_WORKSPACE;   // one more partial than ranges
    plan->fused = true;
    plan->n_splits = s_old + 1;
  }
  return SKV_OK;
}

// ---- parameter blocks ---------------------------------------------------------------------

void fill_query_params(const skv_layer* L, DecodeParams* p, const void* q, float scale, void* workspace) {
  fill_decode_params(L, p, 1, workspace);
  p->q = static_cast<const uint16_t*>(q);
  p->scale_log2e = scale_log2e_of(scale);
}

void fill_append_params(const skv_layer* L, AppendParams* p, const void* k_new, const void* v_new,
                        int64_t stride_b, int64_t stride_t, int64_t stride_h, int32_t T,
                        int64_t cur_len) {
  p->k_cache = static_cast<uint16_t*>(L->k_cache);
  p->v_cache = static_cast<uint16_t*>(L->v_cache);
  p->p_k = static_cast<const uint16_t*>(L->p_k);
  p->p_v = static_cast<const uint16_t*>(L->p_v);
  p->k_new = static_cast<const uint16_t*>(k_new);
  p->v_new = static_cast<const uint16_t*>(v_new);
  p->capacity = L->capacity;
  p->p_k_head_stride = L->p_k_head_stride;
  p->p_v_head_stride = L->p_v_head_stride;
  p->stride_b = stride_b;
  p->stride_t = stride_t;
  p->stride_h = stride_h;
  p->cur_len = cur_len;
  p->cur_lens = nullptr;
  p->batch = L->batch;
  p->n_kv_heads = L->n_kv_heads;
  p->r_k = L->r_k;
  p->r_v = L->r_v;
  p->T = T;
  p->k_scale = nullptr;
  p->k_zero = nullptr;
  p->v_meta = nullptr;
  p->qbits = 0;
  p->pages = PageMap{nullptr, 0, 0, 0};
}

// ---- launches -----------------------------------------------------------------------------

decode_partial_launcher partial_q_launcher_for(int bits, int r_k) {
  if (bits == 4) {
    switch (r_k) {
      case 64: return launch_decode_partial_q4_rk64;
      case 128: return launch_decode_partial_q4_rk128;
    }
    return nullptr;
  }
  switch (r_k) {
    case 32: return launch_decode_partial_q8_rk32;
    case 64: return launch_decode_partial_q8_rk64;
    case 96: return launch_decode_partial_q8_rk96;
    case 128: return launch_decode_partial_q8_rk128;
  }
  return nullptr;
}

decode_partial_launcher paged_partial_q_launcher_for(int bits, int r_k) {
  if (bits == 4) {
    switch (r_k) {
      case 64: return launch_decode_partial_paged_q4_rk64;
      case 128: return launch_decode_partial_paged_q4_rk128;
    }
    return nullptr;
  }
  switch (r_k) {
    case 32: return launch_decode_partial_paged_q8_rk32;
    case 64: return launch_decode_partial_paged_q8_rk64;
    case 96: return launch_decode_partial_paged_q8_rk96;
    case 128: return launch_decode_partial_paged_q8_rk128;
  }
  return nullptr;
}

// q8: the quantised layer the call is for, or null for the bf16 cache.
skv_status run_partial(const skv_layer* L, int64_t n_ctx, int32_t s, void* workspace, void* stream,
                       const skv_q8_layer* q8 = nullptr, int bits = 8, const int32_t* seq_lens = nullptr,
                       int32_t len_add = 0, const PageMap* pages = nullptr) {
  DecodeParams p;
  fill_decode_params(L, &p, s, workspace);
  p.n_ctx = (int32_t)n_ctx;
  p.seq_lens = seq_lens;
  p.len_add = len_add;
  const int cbits = q8 ? bits : 0;
  const bool paged_codes = q8 && pages;          // quantised rows in pages: the matrix-core kernel only
  p.stream_loads = stream_loads_for(L, n_ctx, cbits);
  p.engine = engine_for(L, cbits, paged_codes);
  if (q8) p.v_meta = static_cast<const uint32_t*>(q8->v_meta);
  if (pages) p.pages = *pages;
  decode_partial_launcher launch = !q8     ? (pages ? paged_partial_launcher_for(L->r_k) : partial_launcher_for(L->r_k))
                                   : pages ? paged_partial_q_launcher_for(bits, L->r_k)
                                           : partial_q_launcher_for(bits, L->r_k);
  if (!launch) return SKV_ERR_RANK;
  if (launch(L->r_v, decode_heads_per_pass(L, cbits, paged_codes), p, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SKV_ERR_HIP;
  return SKV_OK;
}

// The range kernel with the query projection folded in (bf16 cache): s_stream context ranges over
// rows [0, n_ctx) and, when T_new > 0, one more partial from the workgroups that project, store
// and attend the new rows [n_ctx, n_ctx + T_new).
skv_status run_partial_fused(const skv_layer* L, const void* q, float scale, int64_t n_ctx, int32_t s_stream,
                             const void* k_new, const void* v_new, int64_t stride_b, int64_t stride_t,
                             int64_t stride_h, int32_t T_new, void* workspace, void* stream,
                             const int32_t* seq_lens = nullptr, int32_t len_add = 0, const PageMap* pages = nullptr) {
  DecodeParams p;
  const int32_t total = s_stream + (T_new > 0 ? 1 : 0);
  fill_decode_params(L, &p, total, workspace);
  p.n_stream = s_stream;
  p.n_ctx = (int32_t)n_ctx;
  p.q = static_cast<const uint16_t*>(q);
  p.scale_log2e = scale_log2e_of(scale);
  p.k_new = static_cast<const uint16_t*>(k_new);
  p.v_new = static_cast<const uint16_t*>(v_new);
  p.stride_b = stride_b;
  p.stride_t = stride_t;
  p.stride_h = stride_h;
  p.cur_len = n_ctx;
  p.T_new = T_new;
  p.seq_lens = seq_lens;
  p.len_add = len_add;
  p.stream_loads = stream_loads_for(L, n_ctx);
  if (pages) p.pages = *pages;
  decode_partial_launcher launch = pages ? paged_partial_launcher_for(L->r_k) : partial_launcher_for(L->r_k);
  if (!launch) return SKV_ERR_RANK;
  if (launch(L->r_v, decode_heads_per_pass(L), p, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status run_combine(const skv_layer* L, void* out, int32_t s, void* workspace, void* stream) {
  DecodeParams p;
  fill_decode_params(L, &p, s, workspace);
  p.out = static_cast<float*>(out);
  if (launch_decode_combine(p, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return SKV_OK;
}

}  // namespace

extern "C" {

skv_status skv_decode_project_query(const skv_layer* L, const void* q, float scale, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  const skv_status st = check_query_stage(L, q, scale, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  DecodeParams p;
  fill_query_params(L, &p, q, scale, workspace);
  if (launch_project(nullptr, &p, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status skv_decode_partial(const skv_layer* L, int64_t n_ctx, int32_t n_splits, void* workspace,
                              size_t workspace_bytes, void* stream) {
  int32_t s = 0;
  const skv_status st = check_partial_stage(L, n_ctx, n_splits, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  return run_partial(L, n_ctx, s, workspace, stream);
}

skv_status skv_decode_partial_q(const skv_layer* L, const void* q, float scale, int64_t n_ctx, int32_t n_splits,
                                void* workspace, size_t workspace_bytes, void* stream) {
  skv_status st = check_query_stage(L, q, scale, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  int32_t s = 0;
  st = check_partial_stage(L, n_ctx, n_splits, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  return run_partial_fused(L, q, scale, n_ctx, s, nullptr, nullptr, 0, 0, 0, 0, workspace, stream);
}

skv_status skv_decode_combine(const skv_layer* L, void* out, int32_t n_splits, void* workspace,
                              size_t workspace_bytes, void* stream) {
  const skv_status st = check_combine_stage(L, out, n_splits, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  return run_combine(L, out, n_splits, workspace, stream);
}

skv_status skv_decode_attention(const skv_layer* L, const void* q, void* out, int64_t n_ctx,
                                float scale, void* workspace, size_t workspace_bytes,
                                void* stream) {
  // Check everything the stages need before the first launch, so that an error
  // never leaves part of the work enqueued.
  int32_t s = 0;
  skv_status st = check_decode_attention(L, q, out, n_ctx, scale, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  // two launches: the range kernel projects the queries itself
  st = run_partial_fused(L, q, scale, n_ctx, s, nullptr, nullptr, 0, 0, 0, 0, workspace, stream);
  if (st != SKV_OK) return st;
  return run_combine(L, out, s, workspace, stream);
}

skv_status skv_decode_attention_layers(const skv_layer* layers, int32_t n_layers, const void* const* q,
                                       void* const* out, int64_t n_ctx, float scale, void* workspace,
                                       size_t workspace_bytes, void* stream) {
  if (n_layers < 0) return SKV_ERR_SHAPE;
  if (n_layers == 0) return SKV_OK;
  if (!layers || !q || !out) return SKV_ERR_NULL;
  for (int32_t l = 0; l < n_layers; ++l) {              // every layer is checked before the first launch
    int32_t s = 0;
    const skv_status st = check_decode_attention(&layers[l], q[l], out[l], n_ctx, scale, workspace, workspace_bytes, &s);
    if (st != SKV_OK) return st;
  }
  for (int32_t l = 0; l < n_layers; ++l) {
    const skv_status st = skv_decode_attention(&layers[l], q[l], out[l], n_ctx, scale, workspace, workspace_bytes, stream);
    if (st != SKV_OK) return st;
  }
  return SKV_OK;
}

skv_status skv_project_append(const skv_layer* L, const void* k_new, const void* v_new,
                              int64_t stride_b, int64_t stride_t, int64_t stride_h, int32_t T,
                              int64_t cur_len, void* stream) {
  const skv_status st = check_append(L, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
  if (st != SKV_OK || T == 0) return st;
  AppendParams p;
  fill_append_params(L, &p, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
  if (launch_append(p, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status skv_decode_step(const skv_layer* L, const void* k_new, const void* v_new,
                           int64_t stride_b, int64_t stride_t, int64_t stride_h, int32_t T,
                           int64_t cur_len, const void* q, void* out, float scale, void* workspace,
                           size_t workspace_bytes, void* stream) {
  StepPlan plan;
  skv_status st = check_decode_step(L, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len, q, out, scale,
                                    workspace, workspace_bytes, &plan);
  if (st != SKV_OK) return st;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int64_t n_ctx = cur_len + T;
  const int32_t s = plan.n_splits;
  if (plan.fused) {
    // The usual decode step, two launches: context ranges over the rows already cached, plus one
    // workgroup per (sequence, KV head) that projects, stores and attends the new rows; then the merge.
    st = run_partial_fused(L, q, scale, cur_len, s - 1, k_new, v_new, stride_b, stride_t, stride_h, T, workspace,
                           stream);
    if (st != SKV_OK) return st;
    return run_combine(L, out, s, workspace, stream);
  }
  if (T > 0) {
    AppendParams ap;
    fill_append_params(L, &ap, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
    if (launch_append(ap, hs) != hipSuccess) return SKV_ERR_HIP;
  }
  st = run_partial_fused(L, q, scale, n_ctx, s, nullptr, nullptr, 0, 0, 0, 0, workspace, stream);
  if (st != SKV_OK) return st;
  return run_combine(L, out, s, workspace, stream);
}

skv_status skv_decode_step_layers(const skv_layer* layers, int32_t n_layers, const void* const* k_new,
                                  const void* const* v_new, int64_t stride_b, int64_t stride_t, int64_t stride_h,
                                  int32_t T, int64_t cur_len, const void* const* q, void* const* out, float scale,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (n_layers < 0) return SKV_ERR_SHAPE;
  if (n_layers == 0) return SKV_OK;
  if (!layers || !q || !out || (T > 0 && (!k_new || !v_new))) return SKV_ERR_NULL;
  for (int32_t l = 0; l < n_layers; ++l) {              // every layer is checked before the first launch
    StepPlan plan;
    const skv_status st = check_decode_step(&layers[l], T > 0 ? k_new[l] : nullptr, T > 0 ? v_new[l] : nullptr, stride_b,
                                            stride_t, stride_h, T, cur_len, q[l], out[l], scale, workspace,
                                            workspace_bytes, &plan);
    if (st != SKV_OK) return st;
  }
  for (int32_t l = 0; l < n_layers; ++l) {
    const skv_status st = skv_decode_step(&layers[l], T > 0 ? k_new[l] : nullptr, T > 0 ? v_new[l] : nullptr, stride_b,
                                          stride_t, stride_h, T, cur_len, q[l], out[l], scale, workspace,
                                          workspace_bytes, stream);
    if (st != SKV_OK) return st;
  }
  return SKV_OK;
}

}  // extern "C"

namespace {

prefill_launcher prefill_launcher_for(int r_k) {
  switch (r_k) {
    case 16: return launch_prefill_rk16;
    case 32: return launch_prefill_rk32;
    case 48: return launch_prefill_rk48;
    case 64: return launch_prefill_rk64;
    case 80: return launch_prefill_rk80;
    case 96: return launch_prefill_rk96;
    case 112: return launch_prefill_rk112;
    case 128: return launch_prefill_rk128;
  }
  return nullptr;
}

prefill_launcher paged_prefill_launcher_for(int r_k) {
  switch (r_k) {
    case 16: return launch_prefill_paged_rk16;
    case 32: return launch_prefill_paged_rk32;
    case 48: return launch_prefill_paged_rk48;
    case 64: return launch_prefill_paged_rk64;
    case 80: return launch_prefill_paged_rk80;
    case 96: return launch_prefill_paged_rk96;
    case 112: return launch_prefill_paged_rk112;
    case 128: return launch_prefill_paged_rk128;
  }
  return nullptr;
}

// Checks of the chunk attention that do not depend on where the queries come from.
skv_status check_prefill(const skv_layer* L, bool folded, const void* q, const void* out, int32_t T,
                         int64_t n_prev, float scale, int32_t mode) {
  const skv_status st = check_layer(L, !folded);
  if (st != SKV_OK) return st;
  if (T < 0) return SKV_ERR_SHAPE;
  if (mode & ~(SKV_PREFILL_SCHED_TOGETHER | SKV_PREFILL_SCHED_AHEAD)) return SKV_ERR_SHAPE;
  if ((mode & SKV_PREFILL_SCHED_TOGETHER) && (mode & SKV_PREFILL_SCHED_AHEAD)) return SKV_ERR_SHAPE;
  if (!(scale == scale) || std::isinf(scale)) return SKV_ERR_SHAPE;
  if (n_prev < 0 || n_prev + (int64_t)T > L->capacity) return SKV_ERR_CAPACITY;
  if (T == 0) return SKV_OK;
  if (!q || !out) return SKV_ERR_NULL;
  if (!aligned16(q) || !aligned16(out)) return SKV_ERR_ALIGN;
  const int g = L->n_q_heads / L->n_kv_heads;
  const int64_t tiles = ((int64_t)T + prefill_tile_tokens(g) - 1) / prefill_tile_tokens(g);
  const int64_t rows_y = (int64_t)L->batch * L->n_kv_heads * (g / heads_per_pass(g));
  if (tiles * rows_y > std::numeric_limits<int32_t>::max()) return SKV_ERR_SHAPE;
  return SKV_OK;
}

skv_status run_prefill(const skv_layer* L, bool folded, const void* q, int64_t sb, int64_t st_, int64_t sh,
                       void* out, int32_t T, int64_t n_prev, float scale, int32_t mode, void* stream,
                       const PageMap* pages = nullptr) {
  PrefillParams p;
  p.pages = pages ? *pages : PageMap{nullptr, 0, 0, 0};
  p.k_cache = static_cast<const uint16_t*>(L->k_cache);
  p.v_cache = static_cast<const uint16_t*>(L->v_cache);
  p.p_k = static_cast<const uint16_t*>(L->p_k);
  p.p_v = static_cast<const uint16_t*>(L->p_v);
  p.q = static_cast<const uint16_t*>(q);
  p.out = static_cast<float*>(out);
  p.capacity = L->capacity;
  p.p_k_head_stride = L->p_k_head_stride;
  p.p_v_head_stride = L->p_v_head_stride;
  p.q_stride_b = sb;
  p.q_stride_t = st_;
  p.q_stride_h = sh;
  p.batch = L->batch;
  p.n_q_heads = L->n_q_heads;
  p.n_kv_heads = L->n_kv_heads;
  p.group = L->n_q_heads / L->n_kv_heads;
  p.T = T;
  p.n_prev = (int32_t)n_prev;
  p.n_tiles = (T + prefill_tile_tokens(p.group) - 1) / prefill_tile_tokens(p.group);
  p.n_rows_y = L->batch * L->n_kv_heads * (p.group / heads_per_pass(p.group));
  const double sc = scale > 0.f ? (double)scale : 1.0 / std::sqrt((double)SKV_HEAD_DIM);
  p.scale_log2e = (float)(sc * 1.4426950408889634);
  p.folded = folded ? 1 : 0;
  prefill_launcher launch = pages ? paged_prefill_launcher_for(L->r_k) : prefill_launcher_for(L->r_k);
  if (!launch) return SKV_ERR_RANK;
  const int sched = (mode & SKV_PREFILL_SCHED_TOGETHER) ? 1 : (mode & SKV_PREFILL_SCHED_AHEAD) ? 2 : 0;
  if (launch(L->r_v, sched, p, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status check_q_strides(int64_t sb, int64_t st, int64_t sh) {
  if (sb < 0 || st < 0 || sh < 0) return SKV_ERR_SHAPE;
  if ((sb % 8) || (st % 8) || (sh % 8)) return SKV_ERR_ALIGN;
  return SKV_OK;
}

}  // namespace

extern "C" {

int32_t skv_prefill_tile_tokens(const skv_layer* L) {
  if (check_layer(L, false) != SKV_OK) return 0;
  return prefill_tile_tokens(L->n_q_heads / L->n_kv_heads);
}

skv_status skv_prefill_attention(const skv_layer* L, const void* q, int64_t q_stride_b,
                                 int64_t q_stride_t, int64_t q_stride_h, void* out, int32_t T,
                                 int64_t n_prev, float scale, int32_t mode, void* stream) {
  skv_status st = check_prefill(L, false, q, out, T, n_prev, scale, mode);
  if (st != SKV_OK || T == 0) return st;
  st = check_q_strides(q_stride_b, q_stride_t, q_stride_h);
  if (st != SKV_OK) return st;
  return run_prefill(L, false, q, q_stride_b, q_stride_t, q_stride_h, out, T, n_prev, scale, mode, stream);
}

skv_status skv_prefill_attention_folded(const skv_layer* L, const void* q_low, void* out_low, int32_t T,
                                        int64_t n_prev, float scale, int32_t mode, void* stream) {
  const skv_status st = check_prefill(L, true, q_low, out_low, T, n_prev, scale, mode);
  if (st != SKV_OK || T == 0) return st;
  return run_prefill(L, true, q_low, 0, 0, 0, out_low, T, n_prev, scale, mode, stream);
}

skv_status skv_prefill_step(const skv_layer* L, const void* k_new, const void* v_new, int64_t stride_b,
                            int64_t stride_t, int64_t stride_h, const void* q, int64_t q_stride_b,
                            int64_t q_stride_t, int64_t q_stride_h, void* out, int32_t T,
                            int64_t cur_len, float scale, int32_t mode, void* stream) {
  skv_status st = check_append(L, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
  if (st != SKV_OK) return st;
  st = check_prefill(L, false, q, out, T, cur_len, scale, mode);
  if (st != SKV_OK || T == 0) return st;
  st = check_q_strides(q_stride_b, q_stride_t, q_stride_h);
  if (st != SKV_OK) return st;
  AppendParams ap;
  fill_append_params(L, &ap, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
  if (launch_append(ap, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return run_prefill(L, false, q, q_stride_b, q_stride_t, q_stride_h, out, T, cur_len, scale, mode, stream);
}

}  // extern "C"

namespace {

// The quantised cache stores whole 32-bit words of a row per lane: ranks are multiples of 32 with
// 8-bit codes (one byte per channel) and of 64 with 4-bit codes (two channels per byte).
skv_status check_q_layer(const skv_q8_layer* Q, int bits) {
  if (!Q) return SKV_ERR_NULL;
  const skv_status st = check_layer(&Q->base);
  if (st != SKV_OK) return st;
  const int step = bits == 8 ? 32 : 64;
  if ((Q->base.r_k % step) || (Q->base.r_v % step)) return SKV_ERR_RANK;
  if (!Q->k_scale || !Q->k_zero || !Q->v_meta) return SKV_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(Q->k_scale) | reinterpret_cast<uintptr_t>(Q->k_zero) |
       reinterpret_cast<uintptr_t>(Q->v_meta)) & 3u)
    return SKV_ERR_ALIGN;
  return SKV_OK;
}

void fill_q_query(const skv_q8_layer* Q, DecodeParams* p, const void* q, float scale, void* workspace) {
  fill_query_params(&Q->base, p, q, scale, workspace);
  p->k_scale = Q->k_scale;
}

void fill_q_append(const skv_q8_layer* Q, int bits, AppendParams* p, const void* k_new, const void* v_new,
                   int64_t stride_b, int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len) {
  fill_append_params(&Q->base, p, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
  p->k_scale = Q->k_scale;
  p->k_zero = Q->k_zero;
  p->v_meta = static_cast<uint32_t*>(Q->v_meta);
  p->qbits = bits;
}

size_t q_cache_bytes(const skv_q8_layer* Q, int bits, int64_t n_tokens) {
  if (!Q || n_tokens < 0) return 0;
  const skv_layer* L = &Q->base;
  const size_t groups_v = (size_t)(L->r_v + 63) / 64;
  return (size_t)L->batch * L->n_kv_heads * (size_t)n_tokens *
         ((size_t)(L->r_k + L->r_v) * (size_t)bits / 8u + 4u * groups_v);
}

skv_status q_project_append(const skv_q8_layer* Q, int bits, const void* k_new, const void* v_new, int64_t stride_b,
                            int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len, void* stream,
                            const int32_t* cur_lens = nullptr, const PageMap* pages = nullptr) {
  skv_status st = check_q_layer(Q, bits);
  if (st != SKV_OK) return st;
  st = check_append(&Q->base, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
  if (st != SKV_OK || T == 0) return st;
  if (reinterpret_cast<uintptr_t>(cur_lens) & 3u) return SKV_ERR_ALIGN;
  AppendParams p;
  fill_q_append(Q, bits, &p, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
  p.cur_lens = cur_lens;
  if (pages) p.pages = *pages;
  if (launch_append(p, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;   // few rows: vector path; a chunk: matrix cores
  return SKV_OK;
}

skv_status q_decode_project_query(const skv_q8_layer* Q, int bits, const void* q, float scale, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  skv_status st = check_q_layer(Q, bits);
  if (st != SKV_OK) return st;
  st = check_query_stage(&Q->base, q, scale, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  DecodeParams p;
  fill_q_query(Q, &p, q, scale, workspace);
  if (launch_project(nullptr, &p, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return SKV_OK;
}

int32_t q_default_splits(const skv_q8_layer* Q, int bits, int64_t n_ctx) {
  if (check_q_layer(Q, bits) != SKV_OK) return 0;
  const skv_layer* L = &Q->base;
  if (n_ctx < 1 || n_ctx > L->capacity) return 0;
  int32_t s = 0;
  if (!plan_splits(L, n_ctx, 0, &s, bits)) return 0;
  return s;
}

skv_status q_decode_partial(const skv_q8_layer* Q, int bits, int64_t n_ctx, int32_t n_splits, void* workspace,
                            size_t workspace_bytes, void* stream) {
  skv_status st = check_q_layer(Q, bits);
  if (st != SKV_OK) return st;
  int32_t s = 0;
  st = check_partial_stage(&Q->base, n_ctx, n_splits, workspace, workspace_bytes, &s, bits);
  if (st != SKV_OK) return st;
  return run_partial(&Q->base, n_ctx, s, workspace, stream, Q, bits);
}

// One launch for the ranges of a quantised cache with the queries projected inside it and, when T_new > 0, the
// new rows quantised, stored and attended by extra workgroups (matrix-core kernel only).
skv_status run_partial_fused_q(const skv_q8_layer* Q, int bits, const void* q, float scale, int64_t n_ctx,
                               int32_t s_stream, const void* k_new, const void* v_new, int64_t stride_b,
                               int64_t stride_t, int64_t stride_h, int32_t T_new, void* workspace, void* stream,
                               const int32_t* seq_lens, const PageMap* pages) {
  const skv_layer* L = &Q->base;
  DecodeParams p;
  const int32_t total = s_stream + (T_new > 0 ? 1 : 0);
  fill_decode_params(L, &p, total, workspace);
  p.n_stream = s_stream;
  p.n_ctx = (int32_t)n_ctx;
  p.q = static_cast<const uint16_t*>(q);
  p.scale_log2e = scale_log2e_of(scale);
  p.k_new = static_cast<const uint16_t*>(k_new);
  p.v_new = static_cast<const uint16_t*>(v_new);
  p.stride_b = stride_b;
  p.stride_t = stride_t;
  p.stride_h = stride_h;
  p.cur_len = n_ctx;
  p.T_new = T_new;
  p.seq_lens = seq_lens;
  p.k_scale = Q->k_scale;
  p.k_zero = Q->k_zero;
  p.v_meta = static_cast<const uint32_t*>(Q->v_meta);
  p.engine = 1;
  p.stream_loads = stream_loads_for(L, n_ctx, bits);
  if (pages) p.pages = *pages;
  decode_partial_launcher launch = pages ? paged_partial_q_launcher_for(bits, L->r_k) : partial_q_launcher_for(bits, L->r_k);
  if (!launch) return SKV_ERR_RANK;
  if (launch(L->r_v, decode_heads_per_pass(L, bits, pages != nullptr), p, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SKV_ERR_HIP;
  return SKV_OK;
}

// T = 0: attention only
skv_status q_decode_step(const skv_q8_layer* Q, int bits, const void* k_new, const void* v_new, int64_t stride_b,
                         int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len, const void* q, void* out,
                         float scale, void* workspace, size_t workspace_bytes, void* stream,
                         const int32_t* cur_lens = nullptr, const PageMap* pages = nullptr) {
  skv_status st = check_q_layer(Q, bits);
  if (st != SKV_OK) return st;
  if (reinterpret_cast<uintptr_t>(cur_lens) & 3u) return SKV_ERR_ALIGN;
  const skv_layer* L = &Q->base;
  if (T > 0 || k_new || v_new) {
    st = check_append(L, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
    if (st != SKV_OK) return st;
  }
  st = check_query_stage(L, q, scale, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  const int64_t n_ctx = cur_len + T;
  int32_t s = 0;
  st = check_partial_stage(L, n_ctx, 0, workspace, workspace_bytes, &s, bits, pages != nullptr);
  if (st != SKV_OK) return st;
  st = check_combine_stage(L, out, s, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  // With the matrix-core kernel a step is two launches, as over the bf16 cache: the range kernel projects the
  // queries itself, and for a few new tokens extra workgroups quantise, store and attend them.
  const int gq = L->n_q_heads / L->n_kv_heads;
  const bool paged_codes = pages != nullptr;
  const bool matrix = engine_for(L, bits, paged_codes) == 1;
  const bool grid_ok = 2 * (int64_t)L->batch * L->n_kv_heads * (gq / decode_heads_per_pass(L, bits, paged_codes)) <= 65535;
  if (matrix && T == 0) {
    st = run_partial_fused_q(Q, bits, q, scale, n_ctx, s, nullptr, nullptr, 0, 0, 0, 0, workspace, stream, cur_lens, pages);
    if (st != SKV_OK) return st;
    return run_combine(L, out, s, workspace, stream);
  }
  if (matrix && T <= kFusedStepMaxTokens && cur_len > 0 && grid_ok) {
    int32_t s_old = 0;
    if (!plan_splits(L, cur_len, 0, &s_old, bits, paged_codes)) return SKV_ERR_SHAPE;
    leave_room_for_new_rows(L, bits, paged_codes, &s_old);
    if (s_old + 1 > SKV_MAX_SPLITS) s_old = SKV_MAX_SPLITS - 1;
    if (workspace_bytes < workspace_need(L, s_old + 1)) return SKV_ERR_WORKSPACE;   // one more partial than ranges
    st = run_partial_fused_q(Q, bits, q, scale, cur_len, s_old, k_new, v_new, stride_b, stride_t, stride_h, T, workspace,
                             stream, cur_lens, pages);
    if (st != SKV_OK) return st;
    return run_combine(L, out, s_old + 1, workspace, stream);
  }
  DecodeParams qp;
  fill_q_query(Q, &qp, q, scale, workspace);
  AppendParams ap;
  if (T > 0) {
    fill_q_append(Q, bits, &ap, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len);
    ap.cur_lens = cur_lens;
    if (pages) ap.pages = *pages;
  }
  const bool few = T > 0 && (int64_t)L->batch * T <= kVectorAppendMaxRows;
  if (T > 0 && !few && launch_append(ap, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  if (launch_project(few ? &ap : nullptr, &qp, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SKV_ERR_HIP;
  st = run_partial(L, n_ctx, s, workspace, stream, Q, bits, cur_lens, T, pages);
  if (st != SKV_OK) return st;
  return run_combine(L, out, s, workspace, stream);
}

}  // namespace

extern "C" {

size_t skv_q8_cache_bytes(const skv_q8_layer* Q, int64_t n_tokens) { return q_cache_bytes(Q, 8, n_tokens); }
size_t skv_q4_cache_bytes(const skv_q4_layer* Q, int64_t n_tokens) { return q_cache_bytes(Q, 4, n_tokens); }

skv_status skv_q8_project_append(const skv_q8_layer* Q, const void* k_new, const void* v_new, int64_t stride_b,
                                 int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len, void* stream) {
  return q_project_append(Q, 8, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len, stream);
}
skv_status skv_q4_project_append(const skv_q4_layer* Q, const void* k_new, const void* v_new, int64_t stride_b,
                                 int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len, void* stream) {
  return q_project_append(Q, 4, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len, stream);
}

skv_status skv_q8_decode_attention(const skv_q8_layer* Q, const void* q, void* out, int64_t n_ctx, float scale,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  return q_decode_step(Q, 8, nullptr, nullptr, 0, 0, 0, 0, n_ctx, q, out, scale, workspace, workspace_bytes, stream);
}
skv_status skv_q4_decode_attention(const skv_q4_layer* Q, const void* q, void* out, int64_t n_ctx, float scale,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  return q_decode_step(Q, 4, nullptr, nullptr, 0, 0, 0, 0, n_ctx, q, out, scale, workspace, workspace_bytes, stream);
}

int32_t skv_q8_decode_default_splits(const skv_q8_layer* Q, int64_t n_ctx) { return q_default_splits(Q, 8, n_ctx); }
int32_t skv_q4_decode_default_splits(const skv_q4_layer* Q, int64_t n_ctx) { return q_default_splits(Q, 4, n_ctx); }

skv_status skv_q8_decode_project_query(const skv_q8_layer* Q, const void* q, float scale, void* workspace,
                                       size_t workspace_bytes, void* stream) {
  return q_decode_project_query(Q, 8, q, scale, workspace, workspace_bytes, stream);
}
skv_status skv_q4_decode_project_query(const skv_q4_layer* Q, const void* q, float scale, void* workspace,
                                       size_t workspace_bytes, void* stream) {
  return q_decode_project_query(Q, 4, q, scale, workspace, workspace_bytes, stream);
}

skv_status skv_q8_decode_partial(const skv_q8_layer* Q, int64_t n_ctx, int32_t n_splits, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  return q_decode_partial(Q, 8, n_ctx, n_splits, workspace, workspace_bytes, stream);
}
skv_status skv_q4_decode_partial(const skv_q4_layer* Q, int64_t n_ctx, int32_t n_splits, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  return q_decode_partial(Q, 4, n_ctx, n_splits, workspace, workspace_bytes, stream);
}

skv_status skv_q8_decode_step(const skv_q8_layer* Q, const void* k_new, const void* v_new, int64_t stride_b,
                              int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len, const void* q, void* out,
                              float scale, void* workspace, size_t workspace_bytes, void* stream) {
  if (T < 0) return SKV_ERR_SHAPE;
  return q_decode_step(Q, 8, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len, q, out, scale, workspace,
                       workspace_bytes, stream);
}
skv_status skv_q4_decode_step(const skv_q4_layer* Q, const void* k_new, const void* v_new, int64_t stride_b,
                              int64_t stride_t, int64_t stride_h, int32_t T, int64_t cur_len, const void* q, void* out,
                              float scale, void* workspace, size_t workspace_bytes, void* stream) {
  if (T < 0) return SKV_ERR_SHAPE;
  return q_decode_step(Q, 4, k_new, v_new, stride_b, stride_t, stride_h, T, cur_len, q, out, scale, workspace,
                       workspace_bytes, stream);
}

}  // extern "C"

namespace {

// Folded-weights variant: the bases are not used.
skv_status check_folded_append(const skv_layer* L, const void* k_low, const void* v_low, int32_t T, int64_t cur_len) {
  const skv_status st = check_layer(L, false);
  if (st != SKV_OK) return st;
  if (T < 0) return SKV_ERR_SHAPE;
  if (cur_len < 0 || cur_len + (int64_t)T > L->capacity) return SKV_ERR_CAPACITY;
  if (T == 0) return SKV_OK;
  if (!k_low || !v_low) return SKV_ERR_NULL;
  if (!aligned16(k_low) || !aligned16(v_low)) return SKV_ERR_ALIGN;
  if ((int64_t)L->batch * T > std::numeric_limits<int32_t>::max() / 64) return SKV_ERR_SHAPE;
  return SKV_OK;
}

skv_status check_folded_decode(const skv_layer* L, const void* q_low, const void* out_low, int64_t n_ctx,
                               float scale, const void* workspace, size_t workspace_bytes, int32_t* s_out) {
  const skv_status st = check_layer(L, false);
  if (st != SKV_OK) return st;
  if (!q_low || !out_low || !workspace) return SKV_ERR_NULL;
  if (!aligned16(q_low) || !aligned16(out_low) || !aligned16(workspace)) return SKV_ERR_ALIGN;
  if (!(scale == scale) || std::isinf(scale)) return SKV_ERR_SHAPE;
  if (n_ctx < 1 || n_ctx > L->capacity) return SKV_ERR_CAPACITY;
  if (!plan_splits(L, n_ctx, 0, s_out)) return SKV_ERR_SHAPE;
  return check_decode_common(L, *s_out, workspace, workspace_bytes);
}

// Range kernel, then the merge of the ranges without the lift: out_low stays in rank-r_V coordinates.
skv_status run_folded_attention(const skv_layer* L, void* out_low, int64_t n_ctx, int32_t s, void* workspace,
                                void* stream, const int32_t* seq_lens = nullptr, int32_t len_add = 0,
                                const PageMap* pages = nullptr) {
  const skv_status st = run_partial(L, n_ctx, s, workspace, stream, nullptr, 8, seq_lens, len_add, pages);
  if (st != SKV_OK) return st;
  DecodeParams cp;
  fill_decode_params(L, &cp, s, workspace);
  cp.out = static_cast<float*>(out_low);
  cp.lift = 0;
  if (launch_decode_combine(cp, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return SKV_OK;
}

}  // namespace

namespace {

// The quantised layer a paged description with integer codes stands for (its arrays are the pools).
skv_q8_layer paged_quant_view(const skv_paged_layer* P) {
  skv_q8_layer Q;
  Q.base = P->layer;
  Q.k_scale = P->k_scale;
  Q.k_zero = P->k_zero;
  Q.v_meta = P->v_meta;
  return Q;
}

// The paged layer's checks; fills the device-side description of its page table.
skv_status check_paged(const skv_paged_layer* P, PageMap* pm, bool need_bases = true) {
  if (!P) return SKV_ERR_NULL;
  const skv_status st = check_layer(&P->layer, need_bases);
  if (st != SKV_OK) return st;
  if (!P->block_table) return SKV_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(P->block_table) & 3u) return SKV_ERR_ALIGN;
  const int32_t pt = P->page_tokens;
  if (pt < kRangeQuantum || pt > (1 << 20) || (pt & (pt - 1))) return SKV_ERR_SHAPE;   // a power of two, >= 64
  if (P->n_pages < 1 || P->max_pages_per_seq < 1) return SKV_ERR_SHAPE;
  if (P->layer.capacity != (int64_t)pt * P->max_pages_per_seq) return SKV_ERR_CAPACITY;
  if (P->code_bits != 0 && P->code_bits != 8 && P->code_bits != 4) return SKV_ERR_SHAPE;
  if (P->code_bits != 0) {
    const skv_q8_layer Q = paged_quant_view(P);
    const skv_status sq = check_q_layer(&Q, P->code_bits);
    if (sq != SKV_OK) return sq;
  }
  int shift = 0;
  while ((1 << shift) < pt) ++shift;
  *pm = PageMap{P->block_table, P->max_pages_per_seq, shift, P->n_pages};
  return SKV_OK;
}

// The calls with per-sequence lengths; lens may be null (every sequence at the host-side bound) and pages
// null (contiguous cache).
skv_status append_lens(const skv_layer* L, const void* k_new, const void* v_new, int64_t stride_b, int64_t stride_t,
                       int64_t stride_h, int32_t T, const int32_t* cur_lens, int64_t max_cur_len, void* stream,
                       const PageMap* pages) {
  const skv_status st = check_append(L, k_new, v_new, stride_b, stride_t, stride_h, T, max_cur_len);
  if (st != SKV_OK) return st;
  if (reinterpret_cast<uintptr_t>(cur_lens) & 3u) return SKV_ERR_ALIGN;
  if (T == 0) return SKV_OK;
  AppendParams p;
  fill_append_params(L, &p, k_new, v_new, stride_b, stride_t, stride_h, T, max_cur_len);
  p.cur_lens = cur_lens;
  if (pages) p.pages = *pages;
  if (launch_append(p, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status attention_lens(const skv_layer* L, const void* q, void* out, const int32_t* seq_lens, int64_t max_len,
                          float scale, void* workspace, size_t workspace_bytes, void* stream, const PageMap* pages) {
  skv_status st = check_query_stage(L, q, scale, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  if (reinterpret_cast<uintptr_t>(seq_lens) & 3u) return SKV_ERR_ALIGN;
  int32_t s = 0;
  st = check_partial_stage(L, max_len, 0, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  st = check_combine_stage(L, out, s, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  st = run_partial_fused(L, q, scale, max_len, s, nullptr, nullptr, 0, 0, 0, 0, workspace, stream, seq_lens, 0, pages);
  if (st != SKV_OK) return st;
  return run_combine(L, out, s, workspace, stream);
}

skv_status step_lens(const skv_layer* L, const void* k_new, const void* v_new, int64_t stride_b, int64_t stride_t,
                     int64_t stride_h, int32_t T, const int32_t* cur_lens, int64_t max_cur_len, const void* q,
                     void* out, float scale, void* workspace, size_t workspace_bytes, void* stream,
                     const PageMap* pages) {
  skv_status st = check_append(L, k_new, v_new, stride_b, stride_t, stride_h, T, max_cur_len);
  if (st != SKV_OK) return st;
  if (T < 1) return SKV_ERR_SHAPE;                       // a step appends at least one row per sequence
  if (reinterpret_cast<uintptr_t>(cur_lens) & 3u) return SKV_ERR_ALIGN;
  st = check_query_stage(L, q, scale, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  const int64_t n_max = max_cur_len + T;
  int32_t s = 0;
  st = check_partial_stage(L, n_max, 0, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  st = check_combine_stage(L, out, s, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  const int gq = L->n_q_heads / L->n_kv_heads;
  const bool grid_ok = 2 * (int64_t)L->batch * L->n_kv_heads * (gq / decode_heads_per_pass(L)) <= 65535;
  if (T <= kFusedStepMaxTokens && max_cur_len > 0 && grid_ok) {
    int32_t s_old = 0;
    if (!plan_splits(L, max_cur_len, 0, &s_old)) return SKV_ERR_SHAPE;
    if (s_old + 1 > SKV_MAX_SPLITS) s_old = SKV_MAX_SPLITS - 1;
    if (workspace_bytes < workspace_need(L, s_old + 1)) return SKV_ERR_WORKSPACE;   // one more partial than ranges
    st = run_partial_fused(L, q, scale, max_cur_len, s_old, k_new, v_new, stride_b, stride_t, stride_h, T, workspace,
                           stream, cur_lens, 0, pages);
    if (st != SKV_OK) return st;
    return run_combine(L, out, s_old + 1, workspace, stream);
  }
  AppendParams ap;
  fill_append_params(L, &ap, k_new, v_new, stride_b, stride_t, stride_h, T, max_cur_len);
  ap.cur_lens = cur_lens;
  if (pages) ap.pages = *pages;
  if (launch_append(ap, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  st = run_partial_fused(L, q, scale, n_max, s, nullptr, nullptr, 0, 0, 0, 0, workspace, stream, cur_lens, T, pages);
  if (st != SKV_OK) return st;
  return run_combine(L, out, s, workspace, stream);
}

}  // namespace

extern "C" {

skv_status skv_append_projected(const skv_layer* L, const void* k_low, const void* v_low, int32_t T,
                                int64_t cur_len, void* stream) {
  const skv_status st = check_folded_append(L, k_low, v_low, T, cur_len);
  if (st != SKV_OK || T == 0) return st;
  AppendParams p;
  fill_append_params(L, &p, k_low, v_low, 0, 0, 0, T, cur_len);
  if (launch_copy_projected(p, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status skv_decode_attention_folded(const skv_layer* L, const void* q_low, void* out_low,
                                       int64_t n_ctx, float scale, void* workspace,
                                       size_t workspace_bytes, void* stream) {
  int32_t s = 0;
  skv_status st = check_folded_decode(L, q_low, out_low, n_ctx, scale, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  DecodeParams qp;
  fill_query_params(L, &qp, q_low, scale, workspace);
  if (launch_scale_query(qp, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return run_folded_attention(L, out_low, n_ctx, s, workspace, stream);
}

skv_status skv_decode_step_folded(const skv_layer* L, const void* k_low, const void* v_low, int32_t T,
                                  int64_t cur_len, const void* q_low, void* out_low, float scale,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  skv_status st = check_folded_append(L, k_low, v_low, T, cur_len);
  if (st != SKV_OK) return st;
  const int64_t n_ctx = cur_len + T;
  int32_t s = 0;
  st = check_folded_decode(L, q_low, out_low, n_ctx, scale, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  DecodeParams qp;
  fill_query_params(L, &qp, q_low, scale, workspace);
  if (T > 0) {
    AppendParams ap;
    fill_append_params(L, &ap, k_low, v_low, 0, 0, 0, T, cur_len);
    if (launch_folded_prepare(ap, qp, hs) != hipSuccess) return SKV_ERR_HIP;
  } else if (launch_scale_query(qp, hs) != hipSuccess) {
    return SKV_ERR_HIP;
  }
  return run_folded_attention(L, out_low, n_ctx, s, workspace, stream);
}

skv_status skv_project_append_varlen(const skv_layer* L, const void* k_new, const void* v_new, int64_t stride_b,
                                     int64_t stride_t, int64_t stride_h, int32_t T, const int32_t* cur_lens,
                                     int64_t max_cur_len, void* stream) {
  if (!cur_lens) return SKV_ERR_NULL;
  return append_lens(L, k_new, v_new, stride_b, stride_t, stride_h, T, cur_lens, max_cur_len, stream, nullptr);
}

skv_status skv_decode_attention_varlen(const skv_layer* L, const void* q, void* out, const int32_t* seq_lens,
                                       int64_t max_len, float scale, void* workspace, size_t workspace_bytes,
                                       void* stream) {
  if (!seq_lens) return SKV_ERR_NULL;
  return attention_lens(L, q, out, seq_lens, max_len, scale, workspace, workspace_bytes, stream, nullptr);
}

skv_status skv_decode_step_varlen(const skv_layer* L, const void* k_new, const void* v_new, int64_t stride_b,
                                  int64_t stride_t, int64_t stride_h, int32_t T, const int32_t* cur_lens,
                                  int64_t max_cur_len, const void* q, void* out, float scale, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  if (!cur_lens) return SKV_ERR_NULL;
  return step_lens(L, k_new, v_new, stride_b, stride_t, stride_h, T, cur_lens, max_cur_len, q, out, scale, workspace,
                   workspace_bytes, stream, nullptr);
}

// ---- paged cache ------------------------------------------------------------------------------

size_t skv_paged_pool_bytes(const skv_paged_layer* P) {
  PageMap pm;
  if (check_paged(P, &pm) != SKV_OK) return 0;
  const size_t rows = (size_t)P->n_pages * P->layer.n_kv_heads * (size_t)P->page_tokens;
  if (P->code_bits == 0) return rows * (size_t)(P->layer.r_k + P->layer.r_v) * 2u;
  return rows * ((size_t)(P->layer.r_k + P->layer.r_v) * (size_t)P->code_bits / 8u + 4u * (size_t)((P->layer.r_v + 63) / 64));
}

int32_t skv_paged_decode_default_splits(const skv_paged_layer* P, int64_t n_ctx) {
  PageMap pm;
  if (check_paged(P, &pm) != SKV_OK) return 0;
  const skv_layer* L = &P->layer;
  if (n_ctx < 1 || n_ctx > L->capacity) return 0;
  int32_t s = 0;
  if (!plan_splits(L, n_ctx, 0, &s, P->code_bits, P->code_bits != 0)) return 0;
  return s;
}

skv_status skv_paged_project_append(const skv_paged_layer* P, const void* k_new, const void* v_new, int64_t stride_b,
                                    int64_t stride_t, int64_t stride_h, int32_t T, const int32_t* cur_lens,
                                    int64_t max_cur_len, void* stream) {
  PageMap pm;
  const skv_status st = check_paged(P, &pm);
  if (st != SKV_OK) return st;
  if (P->code_bits != 0) {
    const skv_q8_layer Q = paged_quant_view(P);
    return q_project_append(&Q, P->code_bits, k_new, v_new, stride_b, stride_t, stride_h, T, max_cur_len, stream,
                            cur_lens, &pm);
  }
  return append_lens(&P->layer, k_new, v_new, stride_b, stride_t, stride_h, T, cur_lens, max_cur_len, stream, &pm);
}

skv_status skv_paged_decode_attention(const skv_paged_layer* P, const void* q, void* out, const int32_t* seq_lens,
                                      int64_t max_len, float scale, void* workspace, size_t workspace_bytes,
                                      void* stream) {
  PageMap pm;
  const skv_status st = check_paged(P, &pm);
  if (st != SKV_OK) return st;
  if (P->code_bits != 0) {
    const skv_q8_layer Q = paged_quant_view(P);
    return q_decode_step(&Q, P->code_bits, nullptr, nullptr, 0, 0, 0, 0, max_len, q, out, scale, workspace,
                         workspace_bytes, stream, seq_lens, &pm);
  }
  return attention_lens(&P->layer, q, out, seq_lens, max_len, scale, workspace, workspace_bytes, stream, &pm);
}

skv_status skv_paged_decode_partial_q(const skv_paged_layer* P, const void* q, const int32_t* seq_lens, float scale,
                                      int64_t max_len, int32_t n_splits, void* workspace, size_t workspace_bytes,
                                      void* stream) {
  PageMap pm;
  skv_status st = check_paged(P, &pm);
  if (st != SKV_OK) return st;
  if (P->code_bits != 0) return SKV_ERR_SHAPE;             // offered over bf16 pages only
  const skv_layer* L = &P->layer;
  st = check_query_stage(L, q, scale, workspace, workspace_bytes);
  if (st != SKV_OK) return st;
  if (reinterpret_cast<uintptr_t>(seq_lens) & 3u) return SKV_ERR_ALIGN;
  int32_t s = 0;
  st = check_partial_stage(L, max_len, n_splits, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  return run_partial_fused(L, q, scale, max_len, s, nullptr, nullptr, 0, 0, 0, 0, workspace, stream, seq_lens, 0, &pm);
}

skv_status skv_paged_decode_step(const skv_paged_layer* P, const void* k_new, const void* v_new, int64_t stride_b,
                                 int64_t stride_t, int64_t stride_h, int32_t T, const int32_t* cur_lens,
                                 int64_t max_cur_len, const void* q, void* out, float scale, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  PageMap pm;
  const skv_status st = check_paged(P, &pm);
  if (st != SKV_OK) return st;
  if (P->code_bits != 0) {
    if (T < 1) return SKV_ERR_SHAPE;                     // a step appends at least one row per sequence
    const skv_q8_layer Q = paged_quant_view(P);
    return q_decode_step(&Q, P->code_bits, k_new, v_new, stride_b, stride_t, stride_h, T, max_cur_len, q, out, scale,
                         workspace, workspace_bytes, stream, cur_lens, &pm);
  }
  return step_lens(&P->layer, k_new, v_new, stride_b, stride_t, stride_h, T, cur_lens, max_cur_len, q, out, scale,
                   workspace, workspace_bytes, stream, &pm);
}

skv_status skv_paged_prefill_attention(const skv_paged_layer* P, const void* q, int64_t q_stride_b, int64_t q_stride_t,
                                       int64_t q_stride_h, void* out, int32_t T, int64_t n_prev, float scale,
                                       int32_t mode, void* stream) {
  PageMap pm;
  skv_status st = check_paged(P, &pm);
  if (st != SKV_OK) return st;
  if (P->code_bits != 0) return SKV_ERR_SHAPE;             // offered over bf16 pages only
  st = check_prefill(&P->layer, false, q, out, T, n_prev, scale, mode);
  if (st != SKV_OK || T == 0) return st;
  if (n_prev + (int64_t)T > kPagedPrefillMaxRows) return SKV_ERR_CAPACITY;   // the kernel's table of tile starts
  st = check_q_strides(q_stride_b, q_stride_t, q_stride_h);
  if (st != SKV_OK) return st;
  return run_prefill(&P->layer, false, q, q_stride_b, q_stride_t, q_stride_h, out, T, n_prev, scale, mode, stream, &pm);
}

// Folded-weights variant over bf16 pages: rows arrive projected, queries projected, outputs stay in rank-r_V
// coordinates; only where a row lives differs from the contiguous calls.
skv_status skv_paged_append_projected(const skv_paged_layer* P, const void* k_low, const void* v_low, int32_t T,
                                      const int32_t* cur_lens, int64_t max_cur_len, void* stream) {
  PageMap pm;
  skv_status st = check_paged(P, &pm, false);
  if (st != SKV_OK) return st;
  if (P->code_bits != 0) return SKV_ERR_SHAPE;             // offered over bf16 pages only
  st = check_folded_append(&P->layer, k_low, v_low, T, max_cur_len);
  if (st != SKV_OK) return st;
  if (reinterpret_cast<uintptr_t>(cur_lens) & 3u) return SKV_ERR_ALIGN;
  if (T == 0) return SKV_OK;
  AppendParams p;
  fill_append_params(&P->layer, &p, k_low, v_low, 0, 0, 0, T, max_cur_len);
  p.cur_lens = cur_lens;
  p.pages = pm;
  if (launch_copy_projected(p, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status skv_paged_decode_attention_folded(const skv_paged_layer* P, const void* q_low, void* out_low,
                                             const int32_t* seq_lens, int64_t max_len, float scale, void* workspace,
                                             size_t workspace_bytes, void* stream) {
  PageMap pm;
  skv_status st = check_paged(P, &pm, false);
  if (st != SKV_OK) return st;
  if (P->code_bits != 0) return SKV_ERR_SHAPE;
  const skv_layer* L = &P->layer;
  int32_t s = 0;
  st = check_folded_decode(L, q_low, out_low, max_len, scale, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  if (reinterpret_cast<uintptr_t>(seq_lens) & 3u) return SKV_ERR_ALIGN;
  DecodeParams qp;
  fill_query_params(L, &qp, q_low, scale, workspace);
  if (launch_scale_query(qp, static_cast<hipStream_t>(stream)) != hipSuccess) return SKV_ERR_HIP;
  return run_folded_attention(L, out_low, max_len, s, workspace, stream, seq_lens, 0, &pm);
}

skv_status skv_paged_decode_step_folded(const skv_paged_layer* P, const void* k_low, const void* v_low, int32_t T,
                                        const int32_t* cur_lens, int64_t max_cur_len, const void* q_low,
                                        void* out_low, float scale, void* workspace, size_t workspace_bytes,
                                        void* stream) {
  PageMap pm;
  skv_status st = check_paged(P, &pm, false);
  if (st != SKV_OK) return st;
  if (P->code_bits != 0) return SKV_ERR_SHAPE;
  const skv_layer* L = &P->layer;
  st = check_folded_append(L, k_low, v_low, T, max_cur_len);
  if (st != SKV_OK) return st;
  if (reinterpret_cast<uintptr_t>(cur_lens) & 3u) return SKV_ERR_ALIGN;
  const int64_t n_ctx = max_cur_len + T;
  int32_t s = 0;
  st = check_folded_decode(L, q_low, out_low, n_ctx, scale, workspace, workspace_bytes, &s);
  if (st != SKV_OK) return st;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  DecodeParams qp;
  fill_query_params(L, &qp, q_low, scale, workspace);
  if (T > 0) {
    AppendParams ap;
    fill_append_params(L, &ap, k_low, v_low, 0, 0, 0, T, max_cur_len);
    ap.cur_lens = cur_lens;
    ap.pages = pm;
    if (launch_folded_prepare(ap, qp, hs) != hipSuccess) return SKV_ERR_HIP;
  } else if (launch_scale_query(qp, hs) != hipSuccess) {
    return SKV_ERR_HIP;
  }
  return run_folded_attention(L, out_low, n_ctx, s, workspace, stream, cur_lens, T, &pm);
}

int32_t skv_padded_rank(int32_t r) {
  if (r < 1 || r > SKV_HEAD_DIM) return 0;
  return (r + 15) / 16 * 16;
}

skv_status skv_pad_basis(const void* src, int32_t n_bases, int32_t r, void* dst, void* stream) {
  if (!src || !dst) return SKV_ERR_NULL;
  if (n_bases < 1) return SKV_ERR_SHAPE;
  const int32_t r_pad = skv_padded_rank(r);
  if (r_pad == 0) return SKV_ERR_RANK;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 1u) return SKV_ERR_ALIGN;
  if (launch_pad_basis(src, dst, r, r_pad, (int64_t)n_bases * SKV_HEAD_DIM, static_cast<hipStream_t>(stream)) !=
      hipSuccess)
    return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status skv_orthonormalize(const void* a, int32_t n_bases, int32_t r, int32_t pad, void* p_out, void* stream) {
  if (!a || !p_out) return SKV_ERR_NULL;
  if (n_bases < 1) return SKV_ERR_SHAPE;
  if (r < 1 || r > SKV_HEAD_DIM) return SKV_ERR_RANK;
  if ((reinterpret_cast<uintptr_t>(a) & 3u) || (reinterpret_cast<uintptr_t>(p_out) & 1u)) return SKV_ERR_ALIGN;
  const int32_t r_out = pad ? skv_padded_rank(r) : r;
  if (launch_orthonormalize(a, p_out, n_bases, r, r_out, static_cast<hipStream_t>(stream)) != hipSuccess)
    return SKV_ERR_HIP;
  return SKV_OK;
}

skv_status skv_layer_ranks(int32_t n_layers, int32_t head_dim, double rho, const int32_t* cand_k,
                           int32_t n_k, const int32_t* cand_v, int32_t n_v, const double* delta,
                           int32_t* r_k_out, int32_t* r_v_out, double* achieved_ratio) {
  if (!cand_k || !cand_v || !delta || !r_k_out || !r_v_out) return SKV_ERR_NULL;
  if (n_layers < 1 || n_k < 1 || n_v < 1 || head_dim < 1) return SKV_ERR_SHAPE;
  if (!(rho > 0.0) || std::isinf(rho)) return SKV_ERR_SHAPE;
  for (int i = 0; i < n_k; ++i)
    if (cand_k[i] < 1 || cand_k[i] > head_dim) return SKV_ERR_SHAPE;
  for (int j = 0; j < n_v; ++j)
    if (cand_v[j] < 1 || cand_v[j] > head_dim) return SKV_ERR_SHAPE;
  const int64_t total = (int64_t)n_layers * n_k * n_v;
  for (int64_t i = 0; i < total; ++i)
    if (delta[i] != delta[i]) return SKV_ERR_SHAPE;

  // Budget carried in rank units (2 * head_dim * B_l) so that costs are integers.
  double units = 2.0 * (double)head_dim * (double)n_layers * rho;
  bool all_feasible = true;
  int64_t spent = 0;
  for (int l = 0; l < n_layers; ++l) {
    const double remaining = (double)(n_layers - l);
    const double* surf = delta + (int64_t)l * n_k * n_v;
    int bi = -1, bj = -1;
    // pass 1: affordable pairs, ordered by (delta, cost, larger r_V, position)
    for (int i = 0; i < n_k; ++i) {
      for (int j = 0; j < n_v; ++j) {
        const int cost = cand_k[i] + cand_v[j];
        if ((double)cost * remaining > units * (1.0 + 1e-12)) continue;
        bool better;
        if (bi < 0) {
          better = true;
        } else {
          const double d0 = surf[bi * n_v + bj], d1 = surf[i * n_v + j];
          const int c0 = cand_k[bi] + cand_v[bj];
          if (d1 != d0) better = d1 < d0;
          else if (cost != c0) better = cost < c0;
          else if (cand_v[j] != cand_v[bj]) better = cand_v[j] > cand_v[bj];
          else better = false;
        }
        if (better) { bi = i; bj = j; }
      }
    }
    if (bi < 0) {
      // pass 2: nothing fits -- cheapest pair, ordered by (cost, delta, larger r_V, position)
      all_feasible = false;
      for (int i = 0; i < n_k; ++i) {
        for (int j = 0; j < n_v; ++j) {
          const int cost = cand_k[i] + cand_v[j];
          bool better;
          if (bi < 0) {
            better = true;
          } else {
            const double d0 = surf[bi * n_v + bj], d1 = surf[i * n_v + j];
            const int c0 = cand_k[bi] + cand_v[bj];
            if (cost != c0) better = cost < c0;
            else if (d1 != d0) better = d1 < d0;
            else if (cand_v[j] != cand_v[bj]) better = cand_v[j] > cand_v[bj];
            else better = false;
          }
          if (better) { bi = i; bj = j; }
        }
      }
    }
    r_k_out[l] = cand_k[bi];
    r_v_out[l] = cand_v[bj];
    units -= (double)(cand_k[bi] + cand_v[bj]);
    spent += cand_k[bi] + cand_v[bj];
  }
  if (achieved_ratio) *achieved_ratio = (double)spent / (2.0 * (double)head_dim * (double)n_layers);
  return all_feasible ? SKV_OK : SKV_ERR_BUDGET;
}

}  // extern "C"
