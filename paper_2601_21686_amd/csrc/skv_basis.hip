// Preparation of projection bases (not on the per-token path).
//
// Ranks the kernels do not take natively.  The paper trains bases at ranks
// spread between 50 % and 90 % of d_h (App. C; for d_h = 128 that is about 64,
// 77, 90, 102, 115) while the kernels here take multiples of 16.  A basis of
// rank r is served exactly by appending zero columns up to the next multiple
// of 16: a zero column of P_K gives a zero key coefficient and a zero query
// coefficient, a zero column of P_V a zero value coefficient that the lift
// multiplies by zero, so compression (Sec. 2.1 Eq. 1), scores and outputs are
// those of the rank-r basis; the price is the cache bytes of the padding.
#include "skv_device_util.h"
#include "skv_internal.h"

namespace skv {
namespace {

__global__ __launch_bounds__(256) void pad_basis_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst,
                                                        int r, int r_pad, int64_t rows) {
  const int64_t total = rows * r_pad;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = i / r_pad;
    const int c = (int)(i % r_pad);
    dst[i] = c < r ? src[row * r + c] : (uint16_t)0;
  }
}

}  // namespace

hipError_t launch_pad_basis(const void* src, void* dst, int r, int r_pad, int64_t rows, hipStream_t stream) {
  const int64_t total = rows * r_pad;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(pad_basis_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                     static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), r, r_pad, rows);
  return hipGetLastError();
}

}  // namespace skv

// ---------------------------------------------------------------------------
// Orthonormalisation of a predicted matrix (Sec. 3.3: A = Q R, the basis is the
// orthonormal factor, P-bar = Q; Sec. 3.2 Eq. 6: the rank-r projection is its leading
// r columns).  The leading r columns of Q depend on the leading r columns of A only
// and are what Gram-Schmidt produces, with R_jj = |v_j| > 0 -- the factorisation with a
// positive diagonal, which is unique for full column rank.  Classical Gram-Schmidt with
// a second pass per column ("twice is enough") keeps Q^T Q - I at float32 rounding level.
//
// One workgroup per matrix.  q_s holds the finished columns, column-major with an odd
// pitch; per column: coefficients c_i = <q_i, v> (thread i), v -= sum_i c_i q_i (thread d),
// twice, then the norm.
// ---------------------------------------------------------------------------
namespace skv {
namespace {

constexpr int kQrThreads = 256;
constexpr int kQrPitch = SKV_HEAD_DIM + 1;

__global__ __launch_bounds__(kQrThreads) void orthonormalize_kernel(const float* __restrict__ a, uint16_t* __restrict__ out,
                                                                    int r, int r_out) {
  constexpr int D = SKV_HEAD_DIM;
  extern __shared__ float lds[];
  float* q_s = lds;                              // [r][kQrPitch]: column i at q_s + i * kQrPitch
  float* v_s = q_s + (size_t)r * kQrPitch;       // [D]
  float* c_s = v_s + D;                          // [D]
  float* red_s = c_s + D;                        // [4]
  const int tid = threadIdx.x;
  const float* am = a + (size_t)blockIdx.x * D * D;
  uint16_t* om = out + (size_t)blockIdx.x * D * r_out;

  for (int j = 0; j < r; ++j) {
    if (tid < D) v_s[tid] = am[(size_t)tid * D + j];
    __syncthreads();
    for (int pass = 0; pass < 2; ++pass) {
      if (tid < j) {
        const float* qi = q_s + (size_t)tid * kQrPitch;
        float c = 0.f;
        for (int d = 0; d < D; ++d) c = fmaf(qi[d], v_s[d], c);
        c_s[tid] = c;
      }
      __syncthreads();
      if (tid < D) {
        float v = v_s[tid];
        for (int i = 0; i < j; ++i) v = fmaf(-c_s[i], q_s[(size_t)i * kQrPitch + tid], v);
        v_s[tid] = v;
      }
      __syncthreads();
    }
    // |v|^2 in a fixed order: lanes, then the two waves that hold data
    float sq = tid < D ? v_s[tid] * v_s[tid] : 0.f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sq += __shfl_xor(sq, off);
    if ((tid & 63) == 0) red_s[tid >> 6] = sq;
    __syncthreads();
    const float nrm2 = red_s[0] + red_s[1];
    // a column that depends on the earlier ones has no direction left: it becomes a zero column
    const float inv = nrm2 > 1e-30f ? 1.0f / sqrtf(nrm2) : 0.f;
    if (tid < D) q_s[(size_t)j * kQrPitch + tid] = v_s[tid] * inv;
    __syncthreads();
  }
  for (int i = tid; i < D * r_out; i += kQrThreads) {
    const int d = i / r_out, c = i % r_out;
    om[i] = c < r ? (uint16_t)f32_to_bf16_bits(q_s[(size_t)c * kQrPitch + d]) : (uint16_t)0;
  }
}

}  // namespace

hipError_t launch_orthonormalize(const void* a, void* out, int n, int r, int r_out, hipStream_t stream) {
  const size_t lds = ((size_t)r * kQrPitch + 2 * SKV_HEAD_DIM + 4) * sizeof(float);
  static bool attr_set = false;                  // more than the default 64 KB of dynamic LDS at large r
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(orthonormalize_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(orthonormalize_kernel, dim3((unsigned)n), dim3(kQrThreads), lds, stream,
                     static_cast<const float*>(a), static_cast<uint16_t*>(out), r, r_out);
  return hipGetLastError();
}

}  // namespace skv
