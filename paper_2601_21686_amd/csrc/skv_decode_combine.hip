// Merge of the per-range partial results of decode attention, normalisation
// and lift back to head_dim with P_V^T.
//
// Softmax over the whole context equals the merge of softmaxes over disjoint
// ranges: with m = max_s m_s,  l = sum_s l_s 2^(m_s - m),  a = sum_s a_s 2^(m_s - m)
// the attention output in rank-r_V coordinates is a / l, and the output in
// head_dim is (a / l) P_V^T  (Sec. 3.2 Eq. 7: V~ = V_down P_V^T, so
// softmax(.) V~ = (softmax(.) V_down) P_V^T).  Sums run in range order, so the
// result does not depend on scheduling.
#include "skv_internal.h"

namespace skv {
namespace {

constexpr int kCombineThreads = SKV_HEAD_DIM;   // one thread per output channel

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

__global__ __launch_bounds__(kCombineThreads) void decode_combine_kernel(const DecodeParams p) {
  __shared__ float w_s[SKV_MAX_SPLITS];          // 2^(m_s - m)
  __shared__ float l_s[SKV_MAX_SPLITS];
  __shared__ float a_s[SKV_HEAD_DIM];            // a / l, rank-r_V coordinates
  __shared__ float red_s[kCombineThreads / 64];

  const int tid = threadIdx.x;
  const int bh = blockIdx.x;                     // b * H_Q + h
  const int h = bh % p.n_q_heads;
  const int kv = h / p.group;
  const int S = p.n_splits;
  const int RV = p.r_v;
  const float* ml = p.part_ml + (int64_t)bh * S * 2;
  const float* pa = p.part_acc + (int64_t)bh * S * RV;

  float mloc = -3.0e38f;
  for (int s = tid; s < S; s += kCombineThreads) {
    const float ms = ml[2 * s];
    w_s[s] = ms;
    l_s[s] = ml[2 * s + 1];
    mloc = fmaxf(mloc, ms);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, off));
  if ((tid & 63) == 0) red_s[tid >> 6] = mloc;
  __syncthreads();
  float m = red_s[0];
#pragma unroll
  for (int w = 1; w < kCombineThreads / 64; ++w) m = fmaxf(m, red_s[w]);
  for (int s = tid; s < S; s += kCombineThreads) w_s[s] = __builtin_amdgcn_exp2f(w_s[s] - m);
  __syncthreads();

  float l = 0.f;
  for (int s = 0; s < S; ++s) l = fmaf(l_s[s], w_s[s], l);
  if (tid < RV) {
    float a = 0.f;
    for (int s = 0; s < S; ++s) a = fmaf(pa[(int64_t)s * RV + tid], w_s[s], a);
    a_s[tid] = a / l;
  }
  __syncthreads();

  // out[d] = sum_c a[c] * P_V[kv][d][c]
  const uint4* prow = reinterpret_cast<const uint4*>(p.p_v + (int64_t)kv * p.p_v_head_stride + (int64_t)tid * RV);
  float o = 0.f;
  for (int c8 = 0; c8 < RV / 8; ++c8) {
    const uint4 v = prow[c8];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o = fmaf(a_s[c8 * 8 + 2 * i], __uint_as_float(w[i] << 16), o);
      o = fmaf(a_s[c8 * 8 + 2 * i + 1], __uint_as_float(w[i] & 0xffff0000u), o);
    }
  }
  p.out[(int64_t)bh * SKV_HEAD_DIM + tid] = o;
}

}  // namespace

hipError_t launch_decode_combine(const DecodeParams& p, hipStream_t stream) {
  const dim3 grid((unsigned)(p.batch * p.n_q_heads));
  hipLaunchKernelGGL(decode_combine_kernel, grid, dim3(kCombineThreads), 0, stream, p);
  return hipGetLastError();
}

}  // namespace skv
