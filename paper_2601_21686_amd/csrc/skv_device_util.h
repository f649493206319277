// Small device-side helpers shared by the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skv.h"

namespace skv {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// float32 -> bf16, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

constexpr int kProjectThreads = 256;
constexpr int kProjectMaxPieces = 8;   // 16-byte basis pieces per thread: 128 / (256 / (r/8)) <= 8

// Matrix-vector projection of ROWS rows onto one basis by a 256-thread workgroup:
//   y[g][c] = sum_d x[g][d] * basis[d][c],  g < ROWS, c < r,  basis bf16 [128][r] row-major.
// The time of such a small product is the latency of fetching the basis, so every
// thread requests all of its 16-byte pieces first and computes afterwards; partial
// sums meet in LDS and are added in a fixed order (deterministic).
//   x_s    LDS [ROWS][128], filled and synchronised by the caller
//   part_s LDS scratch, 256 * ROWS * 8 floats
//   y_s    LDS [ROWS][r], result; synchronised on return
// Thread t owns channel octet t % (r/8) and the basis rows d = dg, dg + ND, ... with
// dg = t / (r/8), ND = 256 / (r/8).  The two halves can be called apart so that other
// memory requests are issued between them.
struct ProjectPieces {
  uint4 w[kProjectMaxPieces];
};

// First half: request this thread's pieces of the basis (no waiting).
__device__ __forceinline__ void project_rows_issue(const uint16_t* __restrict__ basis, int r,
                                                   ProjectPieces& pp) {
  constexpr int D = SKV_HEAD_DIM;
  const int tid = threadIdx.x;
  const int nc8 = r >> 3;
  const int nd = kProjectThreads / nc8;
  const int c8 = tid % nc8;
  const int dg = tid / nc8;
#pragma unroll
  for (int k = 0; k < kProjectMaxPieces; ++k) {
    const int d = dg + k * nd;
    if (dg < nd && d < D) pp.w[k] = *reinterpret_cast<const uint4*>(basis + d * r + c8 * 8);
  }
}

// Second half: multiply, meet in LDS, add in fixed order.
template <int ROWS>
__device__ __forceinline__ void project_rows_finish(const ProjectPieces& pp, int r, const float* x_s,
                                                    float* part_s, float* y_s) {
  constexpr int D = SKV_HEAD_DIM;
  const int tid = threadIdx.x;
  const int nc8 = r >> 3;
  const int nd = kProjectThreads / nc8;
  const int c8 = tid % nc8;
  const int dg = tid / nc8;
  const bool active = dg < nd;

  float a[ROWS][8];
#pragma unroll
  for (int g = 0; g < ROWS; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) a[g][e] = 0.f;
#pragma unroll
  for (int k = 0; k < kProjectMaxPieces; ++k) {
    const int d = dg + k * nd;
    if (active && d < D) {
      const uint32_t ww[4] = {pp.w[k].x, pp.w[k].y, pp.w[k].z, pp.w[k].w};
#pragma unroll
      for (int g = 0; g < ROWS; ++g) {
        const float xv = x_s[g * D + d];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a[g][2 * e] = fmaf(xv, bf16_lo(ww[e]), a[g][2 * e]);
          a[g][2 * e + 1] = fmaf(xv, bf16_hi(ww[e]), a[g][2 * e + 1]);
        }
      }
    }
  }
  if (active) {
#pragma unroll
    for (int g = 0; g < ROWS; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) part_s[(dg * ROWS + g) * r + c8 * 8 + e] = a[g][e];
  }
  __syncthreads();
  for (int i = tid; i < ROWS * r; i += kProjectThreads) {
    const int g = i / r, c = i % r;
    float s = 0.f;
#pragma unroll 8
    for (int k = 0; k < nd; ++k) s += part_s[(k * ROWS + g) * r + c];
    y_s[i] = s;
  }
  __syncthreads();
}

template <int ROWS>
__device__ __forceinline__ void project_rows(const uint16_t* __restrict__ basis, int r,
                                             const float* x_s, float* part_s, float* y_s) {
  ProjectPieces pp;
  project_rows_issue(basis, r, pp);
  project_rows_finish<ROWS>(pp, r, x_s, part_s, y_s);
}

}  // namespace skv
