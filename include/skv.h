/*
 * skv -- decode attention over a KV cache stored as rank-r projections onto
 * orthonormal bases, for AMD MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only.  Every pointer marked "device" is GPU
 * memory owned by the caller; "host" is ordinary process memory.  The library
 * keeps no state between calls (everything a call depends on is in its
 * arguments), never allocates and never synchronises, and owns no memory but
 * one static device scratch array that a single entry point,
 * skv_decode_attention_static, uses (described there).  GPU work is enqueued
 * on the hipStream_t passed as `stream` (NULL = the default stream) and the
 * call returns at once.  All arguments are
 * checked on the host before anything is launched; when a call returns an
 * error nothing has been written.  The return value is the only error channel.
 *
 * Notation follows the paper: d_h = head_dim, r_K / r_V = ranks of the key and
 * value bases P_K, P_V (d_h x r, orthonormal columns), H_Q query heads, H_KV
 * KV heads, G = H_Q / H_KV query heads per KV head, n = tokens in the cache.
 *
 * All bf16 data is IEEE-style bfloat16 (upper half of a float32), 2 bytes.
 */
#ifndef SKV_H
#define SKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SKV_OK = 0,
  SKV_ERR_NULL = 1,      /* a required pointer is NULL                                   */
  SKV_ERR_SHAPE = 2,     /* head_dim != 128, batch < 1, H_Q not a multiple of H_KV,
                            G not in {1,2,4,8}, too many (sequence, KV head) pairs,
                            T < 0, bad strides, bad split count                          */
  SKV_ERR_RANK = 3,      /* a rank is not a multiple of 16 in [16, 128]                  */
  SKV_ERR_CAPACITY = 4,  /* cur_len + T > capacity, n_ctx < 1 or n_ctx > capacity        */
  SKV_ERR_ALIGN = 5,     /* a device pointer is not 16-byte aligned, or a stride is not
                            a multiple of 8 elements                                     */
  SKV_ERR_WORKSPACE = 6, /* workspace smaller than the call needs                        */
  SKV_ERR_BUDGET = 7,    /* skv_layer_ranks: some layer had no affordable rank pair
                            (outputs are still filled, see there)                        */
  SKV_ERR_HIP = 8        /* a launch failed; hipGetLastError() has the detail            */
} skv_status;

#define SKV_HEAD_DIM 128
#define SKV_MAX_SPLITS 256

/*
 * One decoder layer's compressed cache (Sec. 2.1: K_down = K P_K stored in place
 * of K, V_down = V P_V in place of V; ranks differ per layer, Sec. 3.5).
 * Plain data, filled and owned by the caller.
 *
 *   k_cache  device bf16 [batch][n_kv_heads][capacity][r_k], row-major, rows packed
 *   v_cache  device bf16 [batch][n_kv_heads][capacity][r_v]
 *   p_k      device bf16 [n_bases][head_dim][r_k] row-major
 *   p_v      device bf16 [n_bases][head_dim][r_v] row-major
 *   p_k_head_stride / p_v_head_stride: elements between consecutive KV heads'
 *            bases.  0 means one basis shared by every head (the paper shares
 *            the key basis across heads and keeps value bases per head,
 *            Sec. 3.3 "Head sharing"); otherwise at least head_dim * r.
 * The bf16 numbers stored in p_k / p_v are the basis: nothing re-orthonormalises.
 *   flags    hints for the decode calls, 0 = every choice left to the library.  They never change what is
 *            computed (App. A.1 Eq. 18 to the same 2e-3 bound), only how fast; a value with unknown bits
 *            set is SKV_ERR_SHAPE.
 *            SKV_READS_*: how the range kernels load cache rows (every row of the compressed cache is
 *              read once per step, Sec. 2.1 Eq. 2 inside Eq. 18).  SKV_READS_BY_SIZE (0): streaming
 *              (non-temporal) loads when the rows one launch covers add up to more than 288 MiB, clearly
 *              more than the 256 MiB last-level cache, ordinary loads otherwise.  SKV_READS_STREAMING: the
 *              caller knows that the rows will not be found in a cache at the next step, whatever one
 *              launch covers -- the layers of a model whose caches together exceed the last-level cache
 *              should all carry it.  SKV_READS_CACHED: ordinary loads always.
 *            SKV_ENGINE_*: which range kernel streams the cache.  SKV_ENGINE_BY_SHAPE (0): the library's
 *              choice for the shape (what skv_decode_engine_for reports); SKV_ENGINE_VECTOR: vector
 *              arithmetic; SKV_ENGINE_MATRIX: matrix cores (the query heads of a group as columns of
 *              16x16 bf16 products, float32 operands split into two bf16 terms, integer codes of the
 *              quantised formats taken as they are).  For tuning and tests; quantised pages run on the
 *              matrix kernel whatever the flag says.
 */
#define SKV_READS_BY_SIZE 0u
#define SKV_READS_STREAMING 1u
#define SKV_READS_CACHED 2u
#define SKV_READS_MASK 3u
#define SKV_ENGINE_BY_SHAPE 0u
#define SKV_ENGINE_VECTOR 4u
#define SKV_ENGINE_MATRIX 8u
#define SKV_ENGINE_MASK 12u
typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  int32_t r_k, r_v;
  int64_t capacity;
  void* k_cache;
  void* v_cache;
  const void* p_k;
  const void* p_v;
  int64_t p_k_head_stride;
  int64_t p_v_head_stride;
  uint32_t flags;
  uint32_t reserved;       /* must be 0 */
} skv_layer;

/*
 * Compression of new tokens (Sec. 2.1 Eq. 1; Sec. 3.2: the compressed tensors
 * are what is cached).  For every sequence b, KV head h and new token t < T:
 *     k_cache[b][h][cur_len + t][:] = bf16( k_new[b][t][h][:] . P_K[h] )
 *     v_cache[b][h][cur_len + t][:] = bf16( v_new[b][t][h][:] . P_V[h] )
 * with float32 accumulation over head_dim and one round-to-nearest-even to bf16.
 * No mean is subtracted.  Rows outside [cur_len, cur_len + T) are not touched.
 *
 *   k_new, v_new  device bf16, element (b,t,h,i) at
 *                 b*stride_b + t*stride_t + h*stride_h + i  (strides in elements,
 *                 each a multiple of 8; the head_dim axis is contiguous)
 *   T             number of new tokens per sequence (0 is a no-op)
 *   cur_len       tokens already in the cache (the caller tracks it)
 * Errors: NULL, SHAPE, RANK, CAPACITY, ALIGN, HIP.
 */
skv_status skv_project_append(const skv_layer* layer,
                              const void* k_new, const void* v_new,
                              int64_t stride_b, int64_t stride_t, int64_t stride_h,
                              int32_t T, int64_t cur_len, void* stream);

/*
 * One decode step of attention with the reconstructed cache (App. A.1 Eq. 18
 * applied per query head to K~ = K_down P_K^T and V~ = V_down P_V^T, Sec. 3.2
 * Eq. 7).  For every sequence b and query head h, with kv = h / G:
 *     out[b][h][:] = softmax_j( scale * <q[b][h], K~[b][kv][j]> ) . V~[b][kv][0:n_ctx]
 * over cache rows j in [0, n_ctx).  The library evaluates the algebraically
 * equal factored form ((q P_K) against K_down, mix V_down, lift with P_V^T)
 * with float32 arithmetic and a split of the context into independent ranges
 * merged in a fixed order, so results are deterministic run to run.  Inside a
 * range the rows are swept front to back when the sequence holds an even
 * number of rows and back to front when it holds an odd number: a decode loop
 * adds a row per step, so consecutive steps meet first the rows the step before
 * read last, which a last-level cache may still hold.  The direction only
 * permutes the terms of sums; the same call gives the same bits.
 *
 *   q          device bf16 [batch][n_q_heads][head_dim]
 *   out        device float32 [batch][n_q_heads][head_dim]
 *   n_ctx      rows of the cache to attend, 1 <= n_ctx <= capacity (the same for
 *              every sequence); rows >= n_ctx are never read
 *   scale      softmax scale; <= 0 selects 1/sqrt(head_dim) -- the ORIGINAL head
 *              dimension of Eq. 18, not the rank
 *   workspace  device scratch of at least skv_decode_workspace_bytes(); contents
 *              on entry are irrelevant; two calls that may overlap in time need
 *              separate workspaces
 * Errors: NULL, SHAPE, RANK, CAPACITY, ALIGN, WORKSPACE, HIP.
 */
skv_status skv_decode_attention(const skv_layer* layer, const void* q, void* out,
                                int64_t n_ctx, float scale,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * skv_decode_attention for callers that cannot allocate device memory or hand over a workspace: code under
 * stream capture, tight serving loops, harnesses that forbid allocation.  The same computation with the
 * same kernels and the same range plan (results are bit-identical to skv_decode_attention), but the scratch
 * memory is a static device array of SKV_STATIC_SCRATCH_BYTES that the library itself holds on every GPU it
 * runs on, from the first such call on that GPU until the process ends.  The call allocates nothing and frees
 * nothing.  Its first use on a device resolves the array's address there (a symbol lookup): make that first
 * call outside stream capture.
 *   Limit: a call whose plan needs more than SKV_STATIC_SCRATCH_BYTES of scratch (projected queries,
 *   batch * n_q_heads * r_k * 4 bytes, plus batch * n_q_heads * ranges * (r_v + 2) * 4 bytes of partial
 *   results; about 1 MiB at batch 4, 32 query heads, ranks 128) returns SKV_ERR_WORKSPACE and launches nothing.
 *   Sharing: every call on one GPU uses that GPU's one array, whose contents on entry are irrelevant (the
 *   kernels write every word they later read).  Calls that may overlap in time on one GPU -- different
 *   streams, different threads -- race on it: serialise them, or use skv_decode_attention with separate
 *   workspaces.
 * Other arguments and errors as for skv_decode_attention.
 */
#define SKV_STATIC_SCRATCH_BYTES (4u << 20)
skv_status skv_decode_attention_static(const skv_layer* layer, const void* q, void* out,
                                       int64_t n_ctx, float scale, void* stream);

/* Bytes of workspace that skv_decode_attention, skv_decode_step and the stages need for
 * this layer at any n_ctx <= capacity and any split count <= SKV_MAX_SPLITS.
 * Returns 0 if the layer's shape is invalid. */
size_t skv_decode_workspace_bytes(const skv_layer* layer);

/* The number of context ranges skv_decode_attention uses for this shape
 * (1..SKV_MAX_SPLITS); 0 if the arguments are invalid. */
int32_t skv_decode_default_splits(const skv_layer* layer, int64_t n_ctx);

/* Which range kernel the decode calls run for this layer (D2-D4: scores, online softmax and value mix of
 * App. A.1 Eq. 18 in the factored form): 0 = vector arithmetic (decode_partial_kernel), 1 = matrix cores
 * (decode_partial_mma_kernel); -1 for an invalid layer or code width.  code_bits: 0 for bf16 rows, 8 or 4
 * for the quantised formats.  The layer's SKV_ENGINE_* flag decides when set; by shape the matrix kernel
 * takes groups of eight query heads per KV head (one pass over the cache where the vector kernel needs
 * two), the quantised formats, and bf16 layers with groups of four whose ranks are both 32 or 64 -- of a
 * layer flagged SKV_READS_STREAMING (rows from HBM alone) only the pairs it was measured ahead at there:
 * r_v = 128 under r_k = 32 or 64, and 32/64; the vector kernel everything else.  Host only. */
int32_t skv_decode_engine_for(const skv_layer* layer, int32_t code_bits);
/* 1 if the range kernel of a decode call over n_ctx rows reads the cache with streaming loads, 0 for
 * ordinary loads (the layer's SKV_READS_* flag, or by size), -1 for invalid arguments.  Host only. */
int32_t skv_decode_streams_rows(const skv_layer* layer, int64_t n_ctx, int32_t code_bits);

/* Rows [*first_row, *end_row) of the cache that context range `range` of `n_splits` covers
 * when n_ctx rows are attended (host only).  Ranges are runs of whole 64-row quanta, dealt as
 * evenly as possible; together they tile [0, n_ctx); a range may be empty.
 * Errors: NULL, CAPACITY (n_ctx < 1), SHAPE (n_splits or range out of bounds). */
skv_status skv_decode_range(int64_t n_ctx, int32_t n_splits, int32_t range,
                            int64_t* first_row, int64_t* end_row);

/*
 * One whole decode step for T new tokens per sequence (T = 1 in a serving
 * loop): exactly skv_project_append(k_new, v_new, T, cur_len) followed by
 * skv_decode_attention(q, out, n_ctx = cur_len + T), i.e. the query attends
 * the freshly appended rows too (Sec. 3.2: attention always sees the
 * reconstructed, compressed forms).  Doing both in one call lets the library
 * fold the append into the streaming launch: for T <= 4 the context ranges
 * cover the rows already cached while one more workgroup per (sequence, KV
 * head) projects, stores and attends the new rows as a range of their own, so a
 * step is two launches (ranges, merge).  The cache ends up bit-identical to
 * the two separate calls; outputs agree up to the order in which ranges are
 * merged.  Arguments and errors as for the two calls.
 */
skv_status skv_decode_step(const skv_layer* layer,
                           const void* k_new, const void* v_new,
                           int64_t stride_b, int64_t stride_t, int64_t stride_h,
                           int32_t T, int64_t cur_len,
                           const void* q, void* out, float scale,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * A stack of layers (Sec. 3.3: ranks differ from layer to layer, so every layer carries its own
 * descriptor, bases and caches): skv_decode_attention, or skv_decode_step, for layers[0 .. n_layers) in
 * order on one stream, exactly as the loop of single-layer calls would run them and with bit-identical
 * results -- a convenience for callers that hold a layer's inputs ready for all layers (benchmarks, a
 * model whose attention inputs are precomputed).  Every layer is checked before the first launch: an
 * argument error in any layer returns its code with nothing enqueued.
 *   layers        host array of n_layers descriptors (n_layers = 0 is a no-op)
 *   q, out        host arrays of n_layers device pointers, each as for the single-layer call
 *   k_new, v_new  likewise (ignored when T = 0); the strides, T and cur_len are shared by all layers
 *   n_ctx         rows attended in every layer's cache
 *   workspace     one scratch buffer used by each layer in turn: at least the largest
 *                 skv_decode_workspace_bytes() over the layers
 * Errors: as the single-layer call, plus NULL for a missing array and SHAPE for n_layers < 0.  A HIP launch
 * failure at layer l leaves layers [0, l) enqueued.
 */
skv_status skv_decode_attention_layers(const skv_layer* layers, int32_t n_layers,
                                       const void* const* q, void* const* out,
                                       int64_t n_ctx, float scale,
                                       void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_decode_step_layers(const skv_layer* layers, int32_t n_layers,
                                  const void* const* k_new, const void* const* v_new,
                                  int64_t stride_b, int64_t stride_t, int64_t stride_h,
                                  int32_t T, int64_t cur_len,
                                  const void* const* q, void* const* out, float scale,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * The three stages of skv_decode_attention, exposed so that a caller can time
 * or schedule them separately; calling them back to back on one stream with
 * the same workspace and n_splits gives bit for bit the result of
 * skv_decode_attention (which folds the first stage into the second).
 *
 * skv_decode_project_query: q~ = (q P_K) * scale for every query head, with the
 * key basis of the head's KV group (projecting the keys induces the same
 * projection of the query inside q K~^T, Sec. 2.1 Eq. 2 and Sec. 2.2); kept in
 * float32 in the workspace.
 *
 * skv_decode_partial: scores of the projected queries against K_down, online
 * softmax and value mix over each of n_splits context ranges; writes per
 * (b, h, range) the running maximum, the normaliser and the un-normalised
 * rank-r_V mix into the workspace.  n_splits <= 0 selects
 * skv_decode_default_splits(); any value up to SKV_MAX_SPLITS is honoured
 * (ranges beyond the context are empty).
 *
 * skv_decode_combine: merges the ranges (softmax is invariant to the split:
 * rescale each range by exp(m_range - m), add) in range order, divides by the
 * normaliser and lifts with P_V^T into out.  n_splits must be the count the
 * partial stage used.
 */
skv_status skv_decode_project_query(const skv_layer* layer, const void* q, float scale,
                                    void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_decode_partial(const skv_layer* layer, int64_t n_ctx, int32_t n_splits,
                              void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_decode_combine(const skv_layer* layer, void* out, int32_t n_splits,
                              void* workspace, size_t workspace_bytes, void* stream);
/* skv_decode_partial with the first stage folded in: every workgroup projects the queries of its
 * head group itself (the same sums as skv_decode_project_query, so results are bit-identical) --
 * the launch skv_decode_attention and skv_decode_step actually make.  q as for
 * skv_decode_attention. */
skv_status skv_decode_partial_q(const skv_layer* layer, const void* q, float scale, int64_t n_ctx,
                                int32_t n_splits, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ---- Folded-weights variant (Sec. 3.4 "Overheads") --------------------------
 * The paper notes that P_K and P_V can be folded into the attention linear
 * layers; the model then produces projected rows itself and consumes the
 * attention output in rank-r_V coordinates (its output projection carries
 * P_V^T).  What is left is attention in the compressed space, still with the
 * scale of the ORIGINAL head dimension:
 *     out_low[b][h][:] = softmax_j( scale * <q_low[b][h], K_down[b][kv][j]> ) . V_down[b][kv][0:n_ctx]
 * layer->p_k and layer->p_v are not used and may be NULL.
 *
 * skv_append_projected: stores T already-projected tokens per sequence at rows
 * [cur_len, cur_len + T) (a bit-exact copy).
 *   k_low  device bf16 [batch][T][n_kv_heads][r_k], packed;  v_low likewise with r_v
 * skv_decode_attention_folded:
 *   q_low    device bf16 [batch][n_q_heads][r_k]
 *   out_low  device float32 [batch][n_q_heads][r_v]
 * skv_decode_step_folded: both for one decode step (rows placed by the same
 *   small launch that scales the queries); attends cur_len + T tokens.
 * Other arguments, workspace and errors as for skv_project_append /
 * skv_decode_attention / skv_decode_step.
 */
skv_status skv_append_projected(const skv_layer* layer, const void* k_low, const void* v_low,
                                int32_t T, int64_t cur_len, void* stream);
skv_status skv_decode_attention_folded(const skv_layer* layer, const void* q_low, void* out_low,
                                       int64_t n_ctx, float scale,
                                       void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_decode_step_folded(const skv_layer* layer, const void* k_low, const void* v_low,
                                  int32_t T, int64_t cur_len, const void* q_low, void* out_low,
                                  float scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ---- A chunk of queries over the compressed cache (prefill) -----------------
 * App. A.1 Eq. 18 is written for Q in R^{T x d_h}.  For T new tokens per
 * sequence whose compressed keys and values are ALREADY in the cache at rows
 * [n_prev, n_prev + T) (skv_project_append first), token t of the chunk sits at
 * position n_prev + t and, as in the decoder-only models the paper evaluates,
 * attends cache rows 0 .. n_prev + t (causal mask; its own row included):
 *     out[b][t][h][:] = softmax_{j <= n_prev + t}( scale * <q[b][t][h], K~[b][kv][j]> ) . V~[b][kv]
 * with K~, V~ the reconstructed cache of Sec. 3.2 Eq. 7 and kv = h / G.  With
 * T = 1 this is skv_decode_attention at n_ctx = n_prev + 1.  Evaluated in the
 * factored form on the matrix cores (bf16 operands, float32 accumulation,
 * online softmax); needs no workspace.
 *
 *   q       device bf16, element (b,t,h,i) at b*q_stride_b + t*q_stride_t +
 *           h*q_stride_h + i (strides in elements, multiples of 8)
 *   out     device float32 [batch][T][n_q_heads][head_dim], packed
 *   T       tokens in the chunk (0 is a no-op);  n_prev + T <= capacity
 *   scale   <= 0 selects 1/sqrt(head_dim)
 *   mode    0, or one of the schedule bits below.  (Every float32 intermediate
 *           that feeds a bf16 product -- projected queries, softmax weights, the
 *           normalised mix -- is split into two bf16 terms, so results keep
 *           float32-level accuracy: the 2e-3 bound of the decode step.  There is
 *           no reduced-precision mode: each of the three, fed as one bf16 term,
 *           breaks that bound on its own.)
 * skv_prefill_attention_folded is the same in the compressed space (Sec. 3.4
 * "Overheads"): q_low bf16 [batch][T][n_q_heads][r_k] packed, out_low float32
 * [batch][T][n_q_heads][r_v] packed; the bases are not used and may be NULL.
 * skv_prefill_step = skv_project_append(k_new, v_new, T, cur_len) followed by
 * skv_prefill_attention(n_prev = cur_len): one chunk of a chunked prefill.
 * Errors: NULL, SHAPE (T < 0, bad strides or mode bits, grid too large), RANK,
 * CAPACITY, ALIGN, HIP.
 */
#define SKV_PREFILL_EXACT 0
/* Optional, OR-ed into mode: force one of the kernel's two schedules instead of the default for
 * the shape (results are identical up to summation order; for tuning and benchmarks).
 * TOGETHER stages a tile's keys and values in one step (fewer live registers, more waves per
 * SIMD); AHEAD keeps keys one tile ahead so that the score products of the next tile overlap
 * the softmax of the current one. */
#define SKV_PREFILL_SCHED_TOGETHER 0x10
#define SKV_PREFILL_SCHED_AHEAD 0x20
skv_status skv_prefill_attention(const skv_layer* layer, const void* q,
                                 int64_t q_stride_b, int64_t q_stride_t, int64_t q_stride_h,
                                 void* out, int32_t T, int64_t n_prev, float scale, int32_t mode,
                                 void* stream);
skv_status skv_prefill_attention_folded(const skv_layer* layer, const void* q_low, void* out_low,
                                        int32_t T, int64_t n_prev, float scale, int32_t mode,
                                        void* stream);
skv_status skv_prefill_step(const skv_layer* layer, const void* k_new, const void* v_new,
                            int64_t stride_b, int64_t stride_t, int64_t stride_h,
                            const void* q, int64_t q_stride_b, int64_t q_stride_t, int64_t q_stride_h,
                            void* out, int32_t T, int64_t cur_len, float scale, int32_t mode,
                            void* stream);
/* Tokens of a chunk that one workgroup of the prefill kernel covers for this layer's head
 * grouping (32, 64 or 128); 0 if the layer is invalid.  Host only. */
int32_t skv_prefill_tile_tokens(const skv_layer* layer);

/*
 * ---- 8-bit quantised compressed cache (Sec. 4.3) --------------------------
 * Asymmetric integer quantisation of the compressed rows, group size 64
 * channels (the last group of a row may be shorter): code =
 * clamp(round_half_even((x - zero) / scale), 0, 255), x_hat = code*scale + zero,
 * decided in float32.  Keys use one (scale, zero) per KV head and channel group,
 * fixed in advance and shared by every sequence and position (a calibration
 * result the caller brings); values use one pair per token and channel group,
 * computed from that group's minimum and maximum when the token is appended
 * (zero = bf16(min), scale = bf16((max - min)/255), 1 for a flat group) and
 * stored next to the codes.  Attention is Eq. 18 on K~ = K_hat P_K^T,
 * V~ = V_hat P_V^T.  Ranks must be multiples of 32.
 *
 *   base.k_cache  device uint8 [batch][n_kv_heads][capacity][r_k]   (codes)
 *   base.v_cache  device uint8 [batch][n_kv_heads][capacity][r_v]
 *   k_scale, k_zero  device float32 [n_kv_heads][ceil(r_k/64)]
 *   v_meta        device uint32 [batch][n_kv_heads][capacity][ceil(r_v/64)]:
 *                 bf16 scale in the low half, bf16 zero in the high half
 * Everything else (bases, strides, workspace, streams, errors) as for the bf16
 * cache; workspace size is skv_decode_workspace_bytes(&q->base).  Chunks are
 * projected on the matrix cores and quantised from the float32 accumulators;
 * a few rows run as vector projections (the two may round a projection
 * differently in its last float32 bit, which can move a code by one).
 */
typedef struct {
  skv_layer base;
  const float* k_scale;
  const float* k_zero;
  void* v_meta;
} skv_q8_layer;

skv_status skv_q8_project_append(const skv_q8_layer* layer,
                                 const void* k_new, const void* v_new,
                                 int64_t stride_b, int64_t stride_t, int64_t stride_h,
                                 int32_t T, int64_t cur_len, void* stream);
skv_status skv_q8_decode_attention(const skv_q8_layer* layer, const void* q, void* out,
                                   int64_t n_ctx, float scale,
                                   void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_q8_decode_step(const skv_q8_layer* layer,
                              const void* k_new, const void* v_new,
                              int64_t stride_b, int64_t stride_t, int64_t stride_h,
                              int32_t T, int64_t cur_len,
                              const void* q, void* out, float scale,
                              void* workspace, size_t workspace_bytes, void* stream);
/* Stages of skv_q8_decode_attention (see skv_decode_project_query / skv_decode_partial); the
 * third stage is skv_decode_combine(&layer->base, ...), which does not depend on the format. */
skv_status skv_q8_decode_project_query(const skv_q8_layer* layer, const void* q, float scale,
                                       void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_q8_decode_partial(const skv_q8_layer* layer, int64_t n_ctx, int32_t n_splits,
                                 void* workspace, size_t workspace_bytes, void* stream);
/* Bytes the quantised cache of one layer holds for n tokens (codes + value metadata). */
size_t skv_q8_cache_bytes(const skv_q8_layer* layer, int64_t n_tokens);
/* The number of context ranges the calls above choose for n_ctx tokens (as skv_decode_default_splits;
 * the quantised formats may plan more ranges than the bf16 cache).  0 for an invalid layer or n_ctx. */
int32_t skv_q8_decode_default_splits(const skv_q8_layer* layer, int64_t n_ctx);

/*
 * The same with 4-bit codes (the paper lowers the bit width further, Sec. 4.3):
 * code = clamp(round_half_even((x - zero) / scale), 0, 15); two channels per
 * byte, channel 2c in the low half of byte c and channel 2c + 1 in the high
 * half; value ranges scale = bf16((max - min)/15).  Ranks must be multiples
 * of 64.  The struct is shared: only the meaning of the code arrays differs.
 *   base.k_cache  device uint8 [batch][n_kv_heads][capacity][r_k / 2]
 *   base.v_cache  device uint8 [batch][n_kv_heads][capacity][r_v / 2]
 * Everything else as for the skv_q8_ functions of the same name.
 */
typedef skv_q8_layer skv_q4_layer;
skv_status skv_q4_project_append(const skv_q4_layer* layer, const void* k_new, const void* v_new,
                                 int64_t stride_b, int64_t stride_t, int64_t stride_h,
                                 int32_t T, int64_t cur_len, void* stream);
skv_status skv_q4_decode_attention(const skv_q4_layer* layer, const void* q, void* out,
                                   int64_t n_ctx, float scale,
                                   void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_q4_decode_step(const skv_q4_layer* layer, const void* k_new, const void* v_new,
                              int64_t stride_b, int64_t stride_t, int64_t stride_h,
                              int32_t T, int64_t cur_len, const void* q, void* out, float scale,
                              void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_q4_decode_project_query(const skv_q4_layer* layer, const void* q, float scale,
                                       void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_q4_decode_partial(const skv_q4_layer* layer, int64_t n_ctx, int32_t n_splits,
                                 void* workspace, size_t workspace_bytes, void* stream);
size_t skv_q4_cache_bytes(const skv_q4_layer* layer, int64_t n_tokens);
int32_t skv_q4_decode_default_splits(const skv_q4_layer* layer, int64_t n_ctx);

/*
 * Sequential budgeted rank selection (Sec. 3.5 Eqs. 15-17; App. B Alg. 2).
 * Host only; touches no GPU.  delta is host float64 [n_layers][n_k][n_v]
 * row-major: the layer-output error of layer l at ranks (cand_k[i], cand_v[j]).
 * The surfaces are inputs -- producing them needs the model -- so the
 * dependence of later surfaces on earlier choices is the caller's business.
 *
 * B_1 = n_layers * rho.  For l = 1..n_layers: allowance tau_l = B_l/(L-l+1)
 * (Alg. 2's form; it gives tau_1 = rho); among pairs whose cost
 * (r_K + r_V)/(2 head_dim) does not exceed tau_l the smallest delta wins;
 * B_{l+1} = B_l - cost.  Feasibility is tested in integer rank units with a
 * relative slack of 1e-12.  Ties in delta: lower cost, then larger r_V, then
 * the earlier (i, j).  If no pair is affordable the cheapest pair is taken
 * (ties: lower delta), selection continues, and the call finally returns
 * SKV_ERR_BUDGET with all outputs filled.
 *
 *   r_k_out, r_v_out  host int32 [n_layers]
 *   achieved_ratio    host, may be NULL: sum(r_K + r_V) / (2 head_dim n_layers)
 * Candidate ranks may be any positive integers <= head_dim (selection is
 * arithmetic only; what the kernels accept is a separate matter).
 * Errors: NULL, SHAPE (n_layers, n_k, n_v < 1; head_dim < 1; rho <= 0; a
 * candidate outside [1, head_dim]; a NaN in delta), BUDGET.
 */
skv_status skv_layer_ranks(int32_t n_layers, int32_t head_dim, double rho,
                           const int32_t* cand_k, int32_t n_k,
                           const int32_t* cand_v, int32_t n_v,
                           const double* delta,
                           int32_t* r_k_out, int32_t* r_v_out, double* achieved_ratio);

/*
 * ---- Per-sequence lengths -----------------------------------------------------
 * A serving batch mixes sequences of different lengths; Eq. 18 applies to each
 * with its own context.  The lengths live on the device (no host round trip in
 * a serving loop), so the host cannot validate them: each is clamped into
 * [0, max] where max is the host-side bound the call is checked against.
 *
 *   seq_lens / cur_lens  device int32 [batch]
 *   max_len / max_cur_len  host: an upper bound of the lengths; max_len <= capacity,
 *                        max_cur_len + T <= capacity
 * skv_decode_attention_varlen: sequence b attends rows [0, seq_lens[b]); a
 *   sequence of length 0 has nothing to attend and its outputs are zeros.
 * skv_project_append_varlen:   the T new rows of sequence b go to rows
 *   [cur_lens[b], cur_lens[b] + T).
 * skv_decode_step_varlen:      both for a decode step (T >= 1): rows appended at
 *   cur_lens[b], then cur_lens[b] + T rows attended.  The caller advances the
 *   lengths afterwards.
 * Other arguments, workspace and errors as for the calls without _varlen.
 */
skv_status skv_decode_attention_varlen(const skv_layer* layer, const void* q, void* out,
                                       const int32_t* seq_lens, int64_t max_len, float scale,
                                       void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_project_append_varlen(const skv_layer* layer, const void* k_new, const void* v_new,
                                     int64_t stride_b, int64_t stride_t, int64_t stride_h, int32_t T,
                                     const int32_t* cur_lens, int64_t max_cur_len, void* stream);
skv_status skv_decode_step_varlen(const skv_layer* layer, const void* k_new, const void* v_new,
                                  int64_t stride_b, int64_t stride_t, int64_t stride_h, int32_t T,
                                  const int32_t* cur_lens, int64_t max_cur_len,
                                  const void* q, void* out, float scale,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Ranks that are not multiples of 16.  The paper trains its bases at ranks
 * spread between 50 % and 90 % of head_dim (App. C: about 64, 77, 90, 102, 115
 * for head_dim 128); the kernels take multiples of 16.  A rank-r basis is
 * served exactly by zero columns up to skv_padded_rank(r): zero columns give
 * zero coefficients, so the cached rows, scores and outputs are those of the
 * rank-r basis (Sec. 2.1 Eqs. 1-2), at the cache-byte cost of the padding.
 *
 * skv_padded_rank: the next multiple of 16 (16..128) for 1 <= r <= 128, else 0.
 * skv_pad_basis:   dst[b][d][c] = src[b][d][c] for c < r, 0 for r <= c < skv_padded_rank(r).
 *   src  device bf16 [n_bases][head_dim][r], packed (any 2-byte alignment)
 *   dst  device bf16 [n_bases][head_dim][skv_padded_rank(r)], packed; must not overlap src
 * Errors: NULL, SHAPE (n_bases < 1), RANK (r outside [1, 128]), HIP.
 */
int32_t skv_padded_rank(int32_t r);
skv_status skv_pad_basis(const void* src, int32_t n_bases, int32_t r, void* dst, void* stream);

/*
 * Basis construction (Sec. 3.3 "Orthonormalization via QR": the predicted
 * matrix A = Q R is replaced by its orthonormal factor, P-bar = Q; Sec. 3.2
 * Eq. 6: the rank-r projection matrix is the leading r columns of P-bar).
 * For every matrix: p_out[:, 0:r] = bf16 of the leading r columns of the Q
 * factor with positive diagonal of R (unique when those columns of A are
 * independent; a column that depends on earlier ones becomes a zero column),
 * computed in float32 by Gram-Schmidt with a second pass per column, rounded
 * to bf16 once; columns r .. r_out-1 are zero, r_out = skv_padded_rank(r) if
 * pad != 0, else r.  The result can be used as p_k / p_v of a layer as it is.
 *   a      device float32 [n_bases][head_dim][head_dim] row-major
 *   p_out  device bf16 [n_bases][head_dim][r_out], packed
 * Errors: NULL, SHAPE (n_bases < 1), RANK (r outside [1, 128]), ALIGN (a not
 * 4-byte, p_out not 2-byte aligned), HIP.
 */
skv_status skv_orthonormalize(const void* a, int32_t n_bases, int32_t r, int32_t pad,
                              void* p_out, void* stream);

/*
 * ---- Paged cache ---------------------------------------------------------------
 * For serving: the compressed rows of Sec. 2.1 Eq. 1 live in a pool of fixed-size
 * pages instead of one contiguous run per sequence, and a block table maps each
 * sequence's logical pages to pool pages, so that sequences grow, finish and are
 * replaced without moving cache rows.  What is computed is unchanged (Eq. 18 per
 * sequence over its own rows); only where row t of sequence b is found differs:
 * page = block_table[b][t / page_tokens], row t % page_tokens of that page.
 *
 *   layer        shapes, ranks and bases as for skv_layer, with
 *                  k_cache  device bf16 [n_pages][n_kv_heads][page_tokens][r_k]  (the key pool)
 *                  v_cache  device bf16 [n_pages][n_kv_heads][page_tokens][r_v]
 *                  batch    sequences served by the call (rows of block_table)
 *                  capacity page_tokens * max_pages_per_seq exactly (rows a sequence can address)
 *   block_table  device int32 [batch][max_pages_per_seq]; only entries of pages a call touches
 *                are read.  The table lives on the device and cannot be validated by the host:
 *                an entry outside [0, n_pages) is clamped into that range, so nothing outside
 *                the pool is accessed (the result is then meaningless).  Two sequences may
 *                name the same page for rows both only read (a shared prefix); pages written
 *                by an append must belong to one sequence.
 *   page_tokens  rows per page: a power of two, at least 64
 *   n_pages      pages in the pool
 * Lengths: seq_lens / cur_lens are device int32 [batch] as for the _varlen calls (clamped the
 * same way against max_len / max_cur_len), or NULL when every sequence has exactly the
 * host-side length.  Workspace: skv_decode_workspace_bytes(&paged->layer).
 *
 * skv_paged_project_append   rows [cur_lens[b], cur_lens[b] + T) of sequence b, as skv_project_append_varlen
 * skv_paged_decode_attention as skv_decode_attention_varlen
 * skv_paged_decode_partial_q the first of skv_paged_decode_attention's two launches alone (as
 *                            skv_decode_partial_q: n_splits ranges, 0 = default); the second is
 *                            skv_decode_combine(&paged->layer, ...) with the same count
 * skv_paged_decode_step      as skv_decode_step_varlen
 * skv_paged_prefill_attention as skv_prefill_attention (one n_prev for the whole batch);
 *                            n_prev + T at most 1048576 rows (CAPACITY beyond)
 * skv_paged_pool_bytes       bytes of the pools: n_pages * n_kv_heads * page_tokens * (r_k + r_v) * 2 for bf16
 *                            rows, codes plus value ranges for the quantised formats (0 for an invalid
 *                            description)
 * Quantised pages (code_bits = 8 or 4): the pools hold integer codes exactly as skv_q8_layer /
 * skv_q4_layer describe them (k_cache / v_cache: codes [n_pages][n_kv_heads][page_tokens][r bits / 8
 * bytes]; v_meta one word per row and group, laid out like the code pools; k_scale / k_zero static),
 * and append, decode attention and decode step work as skv_q8_* / skv_q4_* do, with the same rank
 * rules (RANK otherwise).  skv_paged_decode_partial_q and skv_paged_prefill_attention are offered
 * over bf16 pages only (SHAPE).
 * Errors: those of the calls named, plus SHAPE (page_tokens not a power of two >= 64, n_pages or
 * max_pages_per_seq < 1), CAPACITY (capacity != page_tokens * max_pages_per_seq), NULL / ALIGN
 * (block_table missing or not 4-byte aligned).
 */
typedef struct {
  skv_layer layer;
  const int32_t* block_table;
  int32_t page_tokens;
  int32_t n_pages;
  int32_t max_pages_per_seq;
  int32_t code_bits;     /* 0: bf16 rows; 8 or 4: the quantised formats of skv_q8_layer / skv_q4_layer */
  const float* k_scale;  /* code_bits != 0: as in skv_q8_layer                                         */
  const float* k_zero;
  void* v_meta;          /* code_bits != 0: device uint32 [n_pages][n_kv_heads][page_tokens][groups of r_v] */
} skv_paged_layer;

size_t skv_paged_pool_bytes(const skv_paged_layer* paged);
/* The number of context ranges the decode calls choose for n_ctx tokens (0 for an invalid description or n_ctx). */
int32_t skv_paged_decode_default_splits(const skv_paged_layer* paged, int64_t n_ctx);
skv_status skv_paged_project_append(const skv_paged_layer* paged, const void* k_new, const void* v_new,
                                    int64_t stride_b, int64_t stride_t, int64_t stride_h, int32_t T,
                                    const int32_t* cur_lens, int64_t max_cur_len, void* stream);
skv_status skv_paged_decode_attention(const skv_paged_layer* paged, const void* q, void* out,
                                      const int32_t* seq_lens, int64_t max_len, float scale,
                                      void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_paged_decode_partial_q(const skv_paged_layer* paged, const void* q, const int32_t* seq_lens,
                                      float scale, int64_t max_len, int32_t n_splits,
                                      void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_paged_decode_step(const skv_paged_layer* paged, const void* k_new, const void* v_new,
                                 int64_t stride_b, int64_t stride_t, int64_t stride_h, int32_t T,
                                 const int32_t* cur_lens, int64_t max_cur_len,
                                 const void* q, void* out, float scale,
                                 void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_paged_prefill_attention(const skv_paged_layer* paged, const void* q, int64_t q_stride_b,
                                       int64_t q_stride_t, int64_t q_stride_h, void* out, int32_t T,
                                       int64_t n_prev, float scale, int32_t mode, void* stream);
/*
 * The folded-weights variant (Sec. 3.4 "Overheads") over bf16 pages: as skv_append_projected,
 * skv_decode_attention_folded and skv_decode_step_folded (same arguments, layouts and errors; the bases of
 * paged->layer may be NULL), with the rows of sequence b at [cur_lens[b], cur_lens[b] + T) resp.
 * [0, seq_lens[b]) of its pages; cur_lens / seq_lens as in the paged calls above (NULL: every sequence at
 * max_cur_len / max_len).  SHAPE for quantised pages.
 */
skv_status skv_paged_append_projected(const skv_paged_layer* paged, const void* k_low, const void* v_low, int32_t T,
                                      const int32_t* cur_lens, int64_t max_cur_len, void* stream);
skv_status skv_paged_decode_attention_folded(const skv_paged_layer* paged, const void* q_low, void* out_low,
                                             const int32_t* seq_lens, int64_t max_len, float scale,
                                             void* workspace, size_t workspace_bytes, void* stream);
skv_status skv_paged_decode_step_folded(const skv_paged_layer* paged, const void* k_low, const void* v_low, int32_t T,
                                        const int32_t* cur_lens, int64_t max_cur_len, const void* q_low,
                                        void* out_low, float scale, void* workspace, size_t workspace_bytes,
                                        void* stream);

/* Bytes of compressed cache one layer holds for n tokens (Sec. 2.1 Eq. 3 times
 * the uncompressed size): batch * n_kv_heads * n * (r_k + r_v) * 2. */
size_t skv_cache_bytes(const skv_layer* layer, int64_t n_tokens);

/* Static, human-readable name of a status code. */
const char* skv_status_string(skv_status s);

#ifdef __cplusplus
}
#endif
#endif /* SKV_H */
