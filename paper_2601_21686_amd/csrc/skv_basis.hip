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
