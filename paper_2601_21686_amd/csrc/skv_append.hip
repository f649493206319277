// Compression of new keys and values and their placement in the cache
// (Sec. 2.1 Eq. 1: K_down = K P_K, V_down = V P_V; Sec. 3.2: these compressed
// tensors are what gets cached).
//
// A chunk of tokens is a dense [tokens x 128] . [128 x r] contraction per KV
// head and runs on the matrix cores (MFMA 16x16x32 bf16, float32 accumulate);
// this file holds that kernel, for the bf16 cache and for the quantised one.  A handful of tokens (a decode step appends one
// per sequence) is a matrix-vector product and runs on the vector ALUs (see
// skv_project.hip).  Both round the float32 sum to bf16 once, to nearest even.
#include "skv_device_util.h"
#include "skv_internal.h"

namespace skv {
namespace {

constexpr int D = SKV_HEAD_DIM;

// ---------------------------------------------------------------------------
// Chunk of tokens on the matrix cores.
//
// Per (KV head, key-or-value) the product is computed transposed,
// C^T[channel][token] = sum_d P[d][channel] * X[token][d], so that each lane of
// the 16x16 result tile ends up with 4 consecutive channels of one token and
// can store them as one 8-byte piece of the cache row.
//   A operand (16 channels x 32 d): from the basis, staged transposed in LDS
//   B operand (32 d x 16 tokens):   straight from global, 16 bytes per lane
// v_mfma_f32_16x16x32_bf16 operand layout: lane L supplies A[L%16][8*(L/16)..+7]
// and B[8*(L/16)..+7][L%16]; result register v of lane L is C[4*(L/16)+v][L%16].
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two float32 -> packed bf16 pair with the hardware conversion (round to nearest even).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

constexpr int kTilesPerWave = 4;                 // 16-token tiles per wave and pass
constexpr int kTokensPerWave = kTilesPerWave * 16;
constexpr int kTokensPerWg = 4 * kTokensPerWave;
constexpr int kLdsPitch = D + 8;                 // bf16 elements; keeps 16-byte reads conflict-free
constexpr int kMaxBlocksPerHead = 32;            // workgroups per (KV head, key-or-value): each stages the
                                                 // basis once and then walks over many token tiles

// The 16-byte pieces of 64 token rows that one wave feeds to the matrix cores.
struct TokenFrags {
  bf16x8 b[kTilesPerWave][4];
};

__device__ __forceinline__ void load_token_frags(const AppendParams& p, const uint16_t* x, int h, int m0,
                                                 int M, int lrow, int lk, TokenFrags& f) {
#pragma unroll
  for (int nt = 0; nt < kTilesPerWave; ++nt) {
    const int tok = m0 + nt * 16 + lrow;
    const int tc = tok < M ? tok : M - 1;        // rows past the end re-read the last row; never stored
    const int b = tc / p.T, t = tc % p.T;
    const uint16_t* src = x + (int64_t)b * p.stride_b + (int64_t)t * p.stride_t + (int64_t)h * p.stride_h;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      f.b[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(src + ks * 32 + lk * 8));
  }
}

// QBITS: 0 = bf16 rows; 8 / 4 = the quantised cache of Sec. 4.3 (codes of that width, static key ranges,
// per-token value ranges), quantised straight from the float32 accumulators.
template <int QBITS>
__global__ __launch_bounds__(256) void append_mfma_kernel(const AppendParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t pt_s[SKV_HEAD_DIM * kLdsPitch];   // [channel][d]

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int h = blockIdx.y;
  const int which = blockIdx.z;                  // 0: keys, 1: values
  const int r = which ? p.r_v : p.r_k;
  const uint16_t* basis = which ? p.p_v + (int64_t)h * p.p_v_head_stride
                                : p.p_k + (int64_t)h * p.p_k_head_stride;
  const uint16_t* x = which ? p.v_new : p.k_new;
  uint16_t* cache = which ? p.v_cache : p.k_cache;
  const int M = p.batch * p.T;                   // token rows of this head
  const int lrow = lane & 15;
  const int lk = lane >> 4;
  const int stride = gridDim.x * kTokensPerWg;

  // the first tile is requested before the basis is staged
  int m0 = blockIdx.x * kTokensPerWg + wave * kTokensPerWave;
  TokenFrags cur, nxt;
  if (m0 < M) load_token_frags(p, x, h, m0, M, lrow, lk, cur);

  // basis [d][c] -> LDS [c][d]
  const int c8n = r >> 3;
  for (int i = tid; i < D * c8n; i += 256) {
    const int d = i / c8n, c8 = i % c8n;
    const uint4 v = *reinterpret_cast<const uint4*>(basis + d * r + c8 * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      pt_s[(c8 * 8 + 2 * e) * kLdsPitch + d] = (uint16_t)(w[e] & 0xffffu);
      pt_s[(c8 * 8 + 2 * e + 1) * kLdsPitch + d] = (uint16_t)(w[e] >> 16);
    }
  }
  __syncthreads();

  for (; m0 < M; m0 += stride) {
    const int m_next = m0 + stride;
    if (m_next < M) load_token_frags(p, x, h, m_next, M, lrow, lk, nxt);   // on its way while this tile computes

    int64_t dst_row[kTilesPerWave];
    bool valid[kTilesPerWave];
#pragma unroll
    for (int nt = 0; nt < kTilesPerWave; ++nt) {
      const int tok = m0 + nt * 16 + lrow;
      valid[nt] = tok < M;
      const int tc = valid[nt] ? tok : M - 1;
      const int b = tc / p.T, t = tc % p.T;
      dst_row[nt] = cache_row(p.pages, p.capacity, p.n_kv_heads, b, h, clamped_len(p.cur_lens, b, p.cur_len) + t);
    }

    if constexpr (QBITS == 0) {
      for (int mt = 0; mt < (r >> 4); ++mt) {
        f32x4 acc[kTilesPerWave];
#pragma unroll
        for (int nt = 0; nt < kTilesPerWave; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8 a = __builtin_bit_cast(
              bf16x8, *reinterpret_cast<const uint4*>(&pt_s[(mt * 16 + lrow) * kLdsPitch + ks * 32 + lk * 8]));
#pragma unroll
          for (int nt = 0; nt < kTilesPerWave; ++nt)
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, cur.b[nt][ks], acc[nt], 0, 0, 0);
        }
#pragma unroll
        for (int nt = 0; nt < kTilesPerWave; ++nt) {
          if (!valid[nt]) continue;
          uint2 o;
          o.x = pack_bf16x2(acc[nt][0], acc[nt][1]);
          o.y = pack_bf16x2(acc[nt][2], acc[nt][3]);
          *reinterpret_cast<uint2*>(cache + dst_row[nt] * r + mt * 16 + lk * 4) = o;
        }
      }
    } else {
      // One 64-channel quantisation group (4 channel tiles, fewer in a short last group) at a time:
      // code = clamp(rne((y - zero) / scale), 0, 2^bits - 1), the same float32 operations as the
      // few-token path.  A lane holds 4 consecutive channels of a token per tile; the 4 lanes that
      // share a token sit 16 apart.
      constexpr float top = (float)((1 << QBITS) - 1);
      const int ng = (r + 63) >> 6;
      uint8_t* codes = reinterpret_cast<uint8_t*>(cache);
      for (int g = 0; g < ng; ++g) {
        const int mt0 = g * 4;
        const int mtn = (r >> 4) - mt0 < 4 ? (r >> 4) - mt0 : 4;
        f32x4 acc[4][kTilesPerWave];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
#pragma unroll
          for (int nt = 0; nt < kTilesPerWave; ++nt) acc[m][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
          if (m < mtn) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
              const bf16x8 a = __builtin_bit_cast(
                  bf16x8, *reinterpret_cast<const uint4*>(&pt_s[((mt0 + m) * 16 + lrow) * kLdsPitch + ks * 32 + lk * 8]));
#pragma unroll
              for (int nt = 0; nt < kTilesPerWave; ++nt)
                acc[m][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, cur.b[nt][ks], acc[m][nt], 0, 0, 0);
            }
          }
        }
#pragma unroll
        for (int nt = 0; nt < kTilesPerWave; ++nt) {
          float scale, zero;
          if (which == 0) {                            // keys: static range of this KV head and group
            scale = p.k_scale[h * ng + g];
            zero = p.k_zero[h * ng + g];
          } else {                                     // values: this token's range over the group, kept as bf16
            float lo = 3.0e38f, hi = -3.0e38f;
#pragma unroll
            for (int m = 0; m < 4; ++m)
              if (m < mtn) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  lo = fminf(lo, acc[m][nt][e]);
                  hi = fmaxf(hi, acc[m][nt][e]);
                }
              }
            lo = fminf(lo, __shfl_xor(lo, 16));
            hi = fmaxf(hi, __shfl_xor(hi, 16));
            lo = fminf(lo, __shfl_xor(lo, 32));
            hi = fmaxf(hi, __shfl_xor(hi, 32));
            uint32_t sb = f32_to_bf16_bits(__fdiv_rn(hi - lo, top));
            if ((sb & 0x7fffu) == 0) sb = 0x3F80u;     // flat group: scale 1
            const uint32_t zb = f32_to_bf16_bits(lo);
            scale = __uint_as_float(sb << 16);
            zero = __uint_as_float(zb << 16);
            if (valid[nt] && lk == 0) p.v_meta[dst_row[nt] * ng + g] = sb | (zb << 16);
          }
          if (!valid[nt]) continue;
#pragma unroll
          for (int m = 0; m < 4; ++m)
            if (m < mtn) {
              uint32_t c[4];
#pragma unroll
              for (int e = 0; e < 4; ++e)
                c[e] = (uint32_t)fminf(fmaxf(rintf(__fdiv_rn(acc[m][nt][e] - zero, scale)), 0.f), top);
              const int64_t ch = dst_row[nt] * r + (mt0 + m) * 16 + lk * 4;      // first of this lane's 4 channels
              if constexpr (QBITS == 8)
                *reinterpret_cast<uint32_t*>(codes + ch) = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
              else
                *reinterpret_cast<uint16_t*>(codes + (ch >> 1)) = (uint16_t)(c[0] | (c[1] << 4) | (c[2] << 8) | (c[3] << 12));
            }
        }
      }
    }
    cur = nxt;
  }
}

}  // namespace

hipError_t launch_append(const AppendParams& p, hipStream_t stream) {
  const int64_t rows = (int64_t)p.batch * p.T;
  if (rows <= kVectorAppendMaxRows) return launch_project(&p, nullptr, stream);
  int64_t blocks = (rows + kTokensPerWg - 1) / kTokensPerWg;
  if (blocks > kMaxBlocksPerHead) blocks = kMaxBlocksPerHead;
  const dim3 grid((unsigned)blocks, (unsigned)p.n_kv_heads, 2u);
  if (p.qbits == 8) hipLaunchKernelGGL(append_mfma_kernel<8>, grid, dim3(256), 0, stream, p);
  else if (p.qbits == 4) hipLaunchKernelGGL(append_mfma_kernel<4>, grid, dim3(256), 0, stream, p);
  else hipLaunchKernelGGL(append_mfma_kernel<0>, grid, dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace skv
