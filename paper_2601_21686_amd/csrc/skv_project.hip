// Projections of a few rows onto a basis, on the vector ALUs:
//   * new keys / values when only a few tokens are appended
//     (Sec. 2.1 Eq. 1: k_down = k P_K, v_down = v P_V), stored as bf16 or, for
//     the quantised cache of Sec. 4.3, as 8- or 4-bit codes;
//   * the decode query, q~ = (q P_K) * scale * log2(e), for all query heads
//     (projecting the keys induces the same projection of the query inside
//     q K~^T = (q P_K) K_down^T, Sec. 2.1 Eq. 2 and Sec. 2.2).
// A decode step appends one token per sequence and projects one query per
// head: matrix-vector products, not contractions worth the matrix cores.  One
// launch serves both kinds of task, so a decode step needs a single small
// kernel ahead of the streaming kernel.
//   blocks [0, n_append)             (sequence, token, KV head, key-or-value)
//   blocks [n_append, n_append + nq) (sequence, KV head, pass): HEADS query heads of one group
#include "skv_device_util.h"
#include "skv_internal.h"

namespace skv {
namespace {

constexpr int D = SKV_HEAD_DIM;

template <int HEADS>
__global__ __launch_bounds__(kProjectThreads) void project_kernel(const AppendParams ap, const int n_append,
                                                                   const DecodeParams dp) {
  __shared__ float x_s[HEADS * D];
  __shared__ float part_s[kProjectThreads * HEADS * 8];
  __shared__ float y_s[HEADS * D];
  const int tid = threadIdx.x;

  if ((int)blockIdx.x < n_append) {
    const int which = blockIdx.x & 1;              // 0: keys, 1: values
    const int idx = blockIdx.x >> 1;               // (b * T + t) * H_KV + h
    const int h = idx % ap.n_kv_heads;
    const int bt = idx / ap.n_kv_heads;
    const int t = bt % ap.T;
    const int b = bt / ap.T;
    const int64_t src = (int64_t)b * ap.stride_b + (int64_t)t * ap.stride_t + (int64_t)h * ap.stride_h;
    const int r = which ? ap.r_v : ap.r_k;
    const uint16_t* basis = which ? ap.p_v + (int64_t)h * ap.p_v_head_stride
                                  : ap.p_k + (int64_t)h * ap.p_k_head_stride;
    ProjectPieces pp;
    project_rows_issue(basis, r, pp);
    if (tid < D) x_s[tid] = bf16_to_f32((which ? ap.v_new : ap.k_new)[src + tid]);
    __syncthreads();
    project_rows_finish<1>(pp, r, x_s, part_s, y_s);
    const int64_t row = cache_row(ap.pages, ap.capacity, ap.n_kv_heads, b, h, clamped_len(ap.cur_lens, b, ap.cur_len) + t);
    if (ap.v_meta == nullptr) {                    // bf16 cache
      uint16_t* cache = which ? ap.v_cache : ap.k_cache;
      if (tid < r) cache[row * r + tid] = (uint16_t)f32_to_bf16_bits(y_s[tid]);
      return;
    }
    // Quantised cache (Sec. 4.3): code = clamp(rne((y - zero) / scale), 0, 2^bits - 1) per 64-channel
    // group.  Thread c holds channel c; group g is wave g.
    const float top = (float)((1 << ap.qbits) - 1);
    const int ng = (r + 63) >> 6;
    const int g = tid >> 6;
    const bool live = tid < r;
    const float y = live ? y_s[tid] : 0.f;
    float scale, zero;
    if (which == 0) {                              // keys: static range of this KV head and group
      scale = live ? ap.k_scale[h * ng + g] : 1.f;
      zero = live ? ap.k_zero[h * ng + g] : 0.f;
    } else {                                       // values: range of this token's group, kept as bf16
      float lo = live ? y : 3.0e38f, hi = live ? y : -3.0e38f;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
      }
      uint32_t sb = f32_to_bf16_bits(__fdiv_rn(hi - lo, top));
      if ((sb & 0x7fffu) == 0) sb = 0x3F80u;       // flat group: scale 1
      const uint32_t zb = f32_to_bf16_bits(lo);
      scale = __uint_as_float(sb << 16);
      zero = __uint_as_float(zb << 16);
      if (live && (tid & 63) == 0) ap.v_meta[row * ng + g] = sb | (zb << 16);
    }
    const uint32_t code = live ? (uint32_t)fminf(fmaxf(rintf(__fdiv_rn(y - zero, scale)), 0.f), top) : 0u;
    uint8_t* cache = reinterpret_cast<uint8_t*>(which ? ap.v_cache : ap.k_cache);
    if (ap.qbits == 8) {
      if (live) cache[row * r + tid] = (uint8_t)code;
    } else {                                       // 4 bits: channel 2c in the low half of byte c, 2c + 1 in the high half
      const uint32_t next = __shfl_down(code, 1);
      if (live && (tid & 1) == 0) cache[(row * r + tid) >> 1] = (uint8_t)(code | (next << 4));
    }
    return;
  }

  const int passes = dp.group / HEADS;
  const int col = blockIdx.x - n_append;           // (b * H_KV + kv) * passes + pass
  const int pass = col % passes;
  const int bkv = col / passes;
  const int kv = bkv % dp.n_kv_heads;
  const int b = bkv / dp.n_kv_heads;
  const int hq0 = kv * dp.group + pass * HEADS;
  ProjectPieces pp;
  project_rows_issue(dp.p_k + (int64_t)kv * dp.p_k_head_stride, dp.r_k, pp);
  const uint16_t* qptr = dp.q + ((int64_t)b * dp.n_q_heads + hq0) * D;
  for (int i = tid; i < HEADS * D; i += kProjectThreads) x_s[i] = bf16_to_f32(qptr[i]);
  __syncthreads();
  project_rows_finish<HEADS>(pp, dp.r_k, x_s, part_s, y_s);
  float* dst = dp.qt + ((int64_t)b * dp.n_q_heads + hq0) * dp.r_k;
  const int ngk = (dp.r_k + 63) >> 6;
  for (int i = tid; i < HEADS * dp.r_k; i += kProjectThreads) {
    float v = y_s[i] * dp.scale_log2e;
    // quantised keys: <q~, code * scale + zero> = <q~ * scale, code> + const; the constant drops out of the softmax
    if (dp.k_scale != nullptr) v *= dp.k_scale[kv * ngk + ((i % dp.r_k) >> 6)];
    dst[i] = v;
  }
}

}  // namespace

// ap may be null (no append tasks); dp may be null (no query tasks).
hipError_t launch_project(const AppendParams* ap, const DecodeParams* dp, hipStream_t stream) {
  AppendParams a{};
  DecodeParams d{};
  int n_append = 0, n_query = 0, heads = 1;
  if (ap) {
    a = *ap;
    n_append = (int)((int64_t)a.batch * a.T * a.n_kv_heads * 2);
  }
  if (dp) {
    d = *dp;
    heads = heads_per_pass(d.group);
    n_query = d.batch * d.n_kv_heads * (d.group / heads);
  }
  if (n_append + n_query == 0) return hipSuccess;
  const dim3 grid((unsigned)(n_append + n_query)), block(kProjectThreads);
  switch (heads) {
    case 1: hipLaunchKernelGGL(project_kernel<1>, grid, block, 0, stream, a, n_append, d); break;
    case 2: hipLaunchKernelGGL(project_kernel<2>, grid, block, 0, stream, a, n_append, d); break;
    case 4: hipLaunchKernelGGL(project_kernel<4>, grid, block, 0, stream, a, n_append, d); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace skv
