// Merge of the per-range partial results of decode attention, normalisation
// and lift back to head_dim with P_V^T.
//
// Softmax over the whole context equals the merge of softmaxes over disjoint
// ranges: with m = max_s m_s,  l = sum_s l_s 2^(m_s - m),  a = sum_s a_s 2^(m_s - m)
// the attention output in rank-r_V coordinates is a / l, and the output in
// head_dim is (a / l) P_V^T  (Sec. 3.2 Eq. 7: V~ = V_down P_V^T, so
// softmax(.) V~ = (softmax(.) V_down) P_V^T).  Every sum runs in a fixed order,
// so the result does not depend on scheduling.
//
// The kernel is a chain of small dependent steps, so its time is latency: every
// global load it will need (its row of P_V, the range maxima, its share of the
// partial mixes) is requested at the top, before the first wait.
#include "skv_device_util.h"
#include "skv_internal.h"

namespace skv {
namespace {

constexpr int kCombineThreads = SKV_HEAD_DIM;   // one thread per output channel

// The maximum over a wave with vector instructions only (rotations inside a row of 16 lanes, then the swaps of
// odd and even rows and of the two halves): the kernel is a chain of dependent steps, and six exchanges through
// the LDS pipeline were a tenth of it.  Every lane receives the maximum.
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_f32<0x128>(x));               // row_ror:8
  x = fmaxf(x, dpp_f32<0x124>(x));               // row_ror:4
  x = fmaxf(x, dpp_f32<0x122>(x));               // row_ror:2
  x = fmaxf(x, dpp_f32<0x121>(x));               // row_ror:1
  const u32x2_t a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(a.x), __uint_as_float(a.y));
  const u32x2_t b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
}
constexpr int kPreload = 8;                     // partial-mix values per thread requested up front
constexpr int kMlPerThread = SKV_MAX_SPLITS / kCombineThreads;

__global__ __launch_bounds__(kCombineThreads) void decode_combine_kernel(const DecodeParams p) {
  __shared__ float w_s[SKV_MAX_SPLITS];          // 2^(m_s - m)
  __shared__ float lw_s[SKV_MAX_SPLITS];         // l_s 2^(m_s - m)
  __shared__ float part_s[kCombineThreads];      // [range group][channel]
  __shared__ float a_s[SKV_HEAD_DIM];            // a / l, rank-r_V coordinates
  __shared__ float red_s[kCombineThreads / 64];

  const int tid = threadIdx.x;
  const int bh = blockIdx.x;                     // b * H_Q + h
  const int h = bh % p.n_q_heads;
  const int kv = h / p.group;
  const int S = p.n_splits;
  const int RV = p.r_v;
  const float2* ml = reinterpret_cast<const float2*>(p.part_ml) + (int64_t)bh * S;
  const float* pa = p.part_acc + (int64_t)bh * S * RV;

  // ---- every request first -----------------------------------------------------------------
  const bool lift = p.lift != 0;                 // folded-weights callers take the rank-r_V result as it is
  const uint4* prow = reinterpret_cast<const uint4*>(p.p_v + (int64_t)kv * p.p_v_head_stride + (int64_t)tid * RV);
  const int nc8 = RV >> 3;
  uint4 pv[SKV_HEAD_DIM / 8];
#pragma unroll
  for (int k = 0; k < SKV_HEAD_DIM / 8; ++k)
    if (lift && k < nc8) pv[k] = prow[k];
  float2 mlr[kMlPerThread];
#pragma unroll
  for (int k = 0; k < kMlPerThread; ++k) {
    const int s = tid + k * kCombineThreads;
    mlr[k] = s < S ? ml[s] : make_float2(-3.0e38f, 0.f);
  }
  // thread -> (channel c, range group sg): group sg sums ranges sg, sg + NG, ...
  const int ng = kCombineThreads / RV;
  const int c = tid % RV;
  const int sg = tid / RV;
  const bool active = sg < ng;
  float av[kPreload];
#pragma unroll
  for (int k = 0; k < kPreload; ++k) {
    const int s = sg + k * ng;
    av[k] = (active && s < S) ? pa[(int64_t)s * RV + c] : 0.f;
  }

  // ---- m = max_s m_s; weights ------------------------------------------------------------
  float mloc = mlr[0].x;
#pragma unroll
  for (int k = 1; k < kMlPerThread; ++k) mloc = fmaxf(mloc, mlr[k].x);
  mloc = wave_max(mloc);
  if ((tid & 63) == 0) red_s[tid >> 6] = mloc;
  __syncthreads();
  float m = red_s[0];
#pragma unroll
  for (int w = 1; w < kCombineThreads / 64; ++w) m = fmaxf(m, red_s[w]);
#pragma unroll
  for (int k = 0; k < kMlPerThread; ++k) {
    const int s = tid + k * kCombineThreads;
    if (s < S) {
      const float w = __builtin_amdgcn_exp2f(mlr[k].x - m);
      w_s[s] = w;
      lw_s[s] = mlr[k].y * w;
    }
  }
  __syncthreads();

  // ---- a[c] = sum_s a_s[c] w_s: per range group, then over groups; l = sum_s l_s w_s -----------
  float a = 0.f;
#pragma unroll
  for (int k = 0; k < kPreload; ++k) {
    const int s = sg + k * ng;
    if (active && s < S) a = fmaf(av[k], w_s[s], a);
  }
  // more ranges than were requested up front (a schedule for unequal lengths can have up to 255): the rest
  // in batches of kPreload loads in flight, same order of summation
  for (int s0 = sg + kPreload * ng; s0 < S; s0 += kPreload * ng) {
    float more[kPreload];
#pragma unroll
    for (int k = 0; k < kPreload; ++k) {
      const int s = s0 + k * ng;
      more[k] = (active && s < S) ? pa[(int64_t)s * RV + c] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < kPreload; ++k) {
      const int s = s0 + k * ng;
      if (active && s < S) a = fmaf(more[k], w_s[s], a);
    }
  }
  if (active) part_s[sg * RV + c] = a;
  float l = 0.f;
  for (int s = 0; s < S; ++s) l += lw_s[s];
  __syncthreads();
  if (tid < RV) {
    float t = part_s[tid];
    for (int g = 1; g < ng; ++g) t += part_s[g * RV + tid];
    a_s[tid] = l > 0.f ? t / l : 0.f;            // a sequence with no rows (per-sequence lengths) gives zeros
  }
  __syncthreads();
  if (!lift) {
    if (tid < RV) p.out[(int64_t)bh * RV + tid] = a_s[tid];
    return;
  }

  // ---- out[d] = sum_c a[c] * P_V[kv][d][c] --------------------------------------------------
  float o = 0.f;
#pragma unroll
  for (int k = 0; k < SKV_HEAD_DIM / 8; ++k) {
    if (k < nc8) {
      const uint32_t w[4] = {pv[k].x, pv[k].y, pv[k].z, pv[k].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        o = fmaf(a_s[k * 8 + 2 * i], bf16_lo(w[i]), o);
        o = fmaf(a_s[k * 8 + 2 * i + 1], bf16_hi(w[i]), o);
      }
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
