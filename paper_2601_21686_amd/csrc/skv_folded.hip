// Folded-weights variant (Sec. 3.4 "Overheads": P_K and P_V folded into the attention
// linear layers).  The model hands over rows that are already projected, so what is
// left of the append is placing them in the cache, and what is left of the query
// projection is the softmax scale.
#include "skv_device_util.h"
#include "skv_internal.h"

namespace skv {
namespace {

// Tasks of one launch, chosen by blockIdx.y + first_task: 0 places key rows, 1 places value
// rows, 2 scales the projected queries.
//   0, 1: one 16-byte piece per thread, rows [b][t][h][r] packed -> cache [b][h][cur_len + t][r]
//         (or the page the block table names for that row)
//   2:    q~ = q_low * scale * log2(e), float32, into the workspace
__global__ __launch_bounds__(256) void folded_kernel(const AppendParams p, const DecodeParams dp, const int first_task) {
  const int task = (int)blockIdx.y + first_task;
  const int64_t stride = (int64_t)gridDim.x * 256;
  const int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (task == 2) {
    const int64_t total = (int64_t)dp.batch * dp.n_q_heads * dp.r_k;
    for (int64_t i = i0; i < total; i += stride) dp.qt[i] = bf16_to_f32(dp.q[i]) * dp.scale_log2e;
    return;
  }
  const int r = task ? p.r_v : p.r_k;
  const int pieces = r >> 3;                     // 16-byte pieces per row
  const int64_t total = (int64_t)p.batch * p.T * p.n_kv_heads * pieces;
  const uint4* src = reinterpret_cast<const uint4*>(task ? p.v_new : p.k_new);
  uint4* dst = reinterpret_cast<uint4*>(task ? p.v_cache : p.k_cache);
  for (int64_t i = i0; i < total; i += stride) {
    const int piece = (int)(i % pieces);
    const int64_t row = i / pieces;              // (b * T + t) * H_KV + h
    const int h = (int)(row % p.n_kv_heads);
    const int64_t bt = row / p.n_kv_heads;
    const int t = (int)(bt % p.T);
    const int64_t b = bt / p.T;
    const int64_t drow = cache_row(p.pages, p.capacity, p.n_kv_heads, (int)b, h, clamped_len(p.cur_lens, (int)b, p.cur_len) + t);
    dst[drow * pieces + piece] = src[i];
  }
}

unsigned blocks_for(int64_t items, int64_t most) {
  int64_t blocks = (items + 255) / 256;
  if (blocks > most) blocks = most;
  return (unsigned)(blocks < 1 ? 1 : blocks);
}

int64_t copy_pieces(const AppendParams& p) {
  return (int64_t)p.batch * p.T * p.n_kv_heads * ((p.r_k > p.r_v ? p.r_k : p.r_v) >> 3);
}

}  // namespace

hipError_t launch_copy_projected(const AppendParams& p, hipStream_t stream) {
  hipLaunchKernelGGL(folded_kernel, dim3(blocks_for(copy_pieces(p), 4096), 2u), dim3(256), 0, stream, p,
                     DecodeParams{}, 0);
  return hipGetLastError();
}

hipError_t launch_scale_query(const DecodeParams& p, hipStream_t stream) {
  const int64_t total = (int64_t)p.batch * p.n_q_heads * p.r_k;
  hipLaunchKernelGGL(folded_kernel, dim3(blocks_for(total, 1024), 1u), dim3(256), 0, stream, AppendParams{}, p, 2);
  return hipGetLastError();
}

hipError_t launch_folded_prepare(const AppendParams& ap, const DecodeParams& dp, hipStream_t stream) {
  const int64_t total = (int64_t)dp.batch * dp.n_q_heads * dp.r_k;
  const int64_t items = total > copy_pieces(ap) ? total : copy_pieces(ap);
  hipLaunchKernelGGL(folded_kernel, dim3(blocks_for(items, 1024), 3u), dim3(256), 0, stream, ap, dp, 0);
  return hipGetLastError();
}

}  // namespace skv
