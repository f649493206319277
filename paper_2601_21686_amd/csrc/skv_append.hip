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
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two float32 -> packed bf16 pair with the hardware conversion (round to nearest even).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 16-token tiles per wave and pass: 4 for bf16 rows; 2 for the quantised caches, whose 64-channel
// groups keep four result tiles per token tile alive (4 would leave one wave per SIMD)
__host__ __device__ constexpr int tiles_per_wave(int qbits) { return qbits ? 2 : 4; }
constexpr int kLdsPitch = D + 8;                 // bf16 elements; keeps 16-byte reads conflict-free
constexpr int kMaxBlocksPerHead = 64;            // workgroups per (KV head, key-or-value): each stages the
                                                 // basis once and then walks over many token tiles

// The 16-byte pieces of 64 token rows that one wave feeds to the matrix cores.
template <int NT>
struct TokenFrags {
  bf16x8 b[NT][4];
};

// STREAM: non-temporal loads, for a chunk too large to be found in a cache (see launch_append).
template <bool STREAM, int NT>
__device__ __forceinline__ void load_token_frags(const AppendParams& p, const uint16_t* x, int h, int m0,
                                                 int M, int lrow, int lk, TokenFrags<NT>& f) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int tok = m0 + nt * 16 + lrow;
    const int tc = tok < M ? tok : M - 1;        // rows past the end re-read the last row; never stored
    const int b = tc / p.T, t = tc % p.T;
    const uint16_t* src = x + (int64_t)b * p.stride_b + (int64_t)t * p.stride_t + (int64_t)h * p.stride_h;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      if constexpr (STREAM) f.b[nt][ks] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(src + ks * 32 + lk * 8));
      else f.b[nt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(src + ks * 32 + lk * 8));
  }
}

// Output rows leave through a per-wave LDS stage so that a store instruction writes 1 KB of
// consecutive cache bytes (whole rows of consecutive tokens) instead of a 32-byte piece per token.
// The channel tiles of a row are staged in one group when there are at most 5 of them, else in two.
constexpr int kMaxGroupTiles = 5;
__host__ __device__ constexpr int group_tiles(int n_mt) { return n_mt <= kMaxGroupTiles ? n_mt : (n_mt + 1) >> 1; }
// bytes between staged token rows: the group's bytes plus 16 keeps both the 8-byte writes of a
// result tile (16 tokens at once) and the 16-byte reads of the flush spread over the banks
__host__ __device__ constexpr int stage_pitch(int n_mt) { return group_tiles(n_mt) * 32 + 16; }
__host__ __device__ constexpr int append_lds_bytes(int r, int tokens_per_wave) {
  return r * (kLdsPitch * 2) + 4 * (tokens_per_wave * stage_pitch(r >> 4) + tokens_per_wave * 8);
}

// QBITS: 0 = bf16 rows; 8 / 4 = the quantised cache of Sec. 4.3 (codes of that width, static key ranges,
// per-token value ranges), quantised straight from the float32 accumulators.
template <int QBITS, bool STREAM>
__global__ __launch_bounds__(256) void append_mfma_kernel(const AppendParams p) {
  constexpr int kTilesPerWave = tiles_per_wave(QBITS);
  constexpr int kTokensPerWave = kTilesPerWave * 16;
  constexpr int kTokensPerWg = 4 * kTokensPerWave;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
  uint16_t* pt_s = reinterpret_cast<uint16_t*>(lds_raw);                             // [channel][d], r rows

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // a scalar: the tile loop below branches as a wave
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
  // per-wave output stage: the 64 token rows of one channel group, then their destination rows
  const int n_mt = r >> 4;
  const int g_first = group_tiles(n_mt);
  const int pitch = stage_pitch(n_mt);
  uint8_t* stage = lds_raw + r * (kLdsPitch * 2) + wave * (kTokensPerWave * pitch + kTokensPerWave * 8);
  int64_t* row_s = reinterpret_cast<int64_t*>(stage + kTokensPerWave * pitch);

  int m0 = blockIdx.x * kTokensPerWg + wave * kTokensPerWave;
  TokenFrags<kTilesPerWave> fa, fb;

  // basis [d][c] -> LDS [c][d]
  // Thread = (row d of the basis, one of two 8-channel pieces per round); all pieces are requested
  // before the first is written.  Consecutive lanes write consecutive 2-byte slots of one LDS row.
  {
    const int d = tid & (D - 1);
    const int rounds = r >> 4;
    uint4 v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k < rounds) v[k] = *reinterpret_cast<const uint4*>(basis + d * r + (2 * k + (tid >> 7)) * 8);
    // The wave's first two tiles are requested behind the basis and without a condition (rows past the end
    // re-read the last row): requests return in order and a wait counts the requests made since, so the
    // basis is staged while the token rows are on their way.  Requested ahead of the basis, or under a
    // condition, the staging waited for every token row (5-6 us into the launch).
    load_token_frags<STREAM>(p, x, h, m0, M, lrow, lk, fa);
    load_token_frags<STREAM>(p, x, h, m0 + stride, M, lrow, lk, fb);
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k < rounds) {
        const int c0 = (2 * k + (tid >> 7)) * 8;
        const uint32_t w[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          pt_s[(c0 + 2 * e) * kLdsPitch + d] = (uint16_t)(w[e] & 0xffffu);
          pt_s[(c0 + 2 * e + 1) * kLdsPitch + d] = (uint16_t)(w[e] >> 16);
        }
      }
  }
  __syncthreads();

  // Two register sets of token fragments take turns: a set is requested again, two tiles ahead,
  // right after the rows computed from it have been sent off, so requests of this wave are
  // outstanding all the time.
  // Where the wave's token rows [m, m + kTokensPerWave) go (-1: past the end).  With per-sequence lengths or
  // pages this reads a table, under a condition; it is called where no request of token rows has been made
  // since the last wait, because a request under a condition makes every later wait a wait for everything.
  auto plan_rows = [&](const int m) {
    const int tok = m + lane;
    int64_t row = -1;
    if (lane < kTokensPerWave && tok < M) {
      const int b = tok / p.T, t = tok % p.T;
      row = cache_row(p.pages, p.capacity, p.n_kv_heads, b, h, clamped_len(p.cur_lens, b, p.cur_len) + t);
    }
    if (lane < kTokensPerWave) row_s[lane] = row;
  };
  auto process = [&](TokenFrags<kTilesPerWave>& cur, const int m0) {
    // Sends `ppr` 16-byte pieces of every staged row to the cache, 1 KB of consecutive bytes per
    // store instruction when the tokens are consecutive rows.  Streaming stores: the rows are not
    // read again here and should not displace the chunk being read in the caches.
    auto flush = [&](uint8_t* dst, const int64_t row_bytes, const int ppr) {
      __builtin_amdgcn_wave_barrier();             // the stage is this wave's own: its LDS accesses stay in order
      for (int q = lane; q < kTokensPerWave * ppr; q += 64) {
        const int tok = q / ppr, piece = q - tok * ppr;
        const int64_t row = row_s[tok];
        const uint4 v = *reinterpret_cast<const uint4*>(stage + tok * pitch + piece * 16);
        if (row >= 0)
          __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w},
                                      reinterpret_cast<u32x4*>(dst + row * row_bytes + piece * 16));
      }
      __builtin_amdgcn_wave_barrier();
    };
    if constexpr (QBITS == 0) {
      for (int mt0 = 0; mt0 < n_mt; mt0 += g_first) {
        const int gt = n_mt - mt0 < g_first ? n_mt - mt0 : g_first;
        for (int m = 0; m < gt; ++m) {
          f32x4 acc[kTilesPerWave];
#pragma unroll
          for (int nt = 0; nt < kTilesPerWave; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 a = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const uint4*>(&pt_s[((mt0 + m) * 16 + lrow) * kLdsPitch + ks * 32 + lk * 8]));
#pragma unroll
            for (int nt = 0; nt < kTilesPerWave; ++nt)
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, cur.b[nt][ks], acc[nt], 0, 0, 0);
          }
#pragma unroll
          for (int nt = 0; nt < kTilesPerWave; ++nt) {
            uint2 o;
            o.x = pack_bf16x2(acc[nt][0], acc[nt][1]);
            o.y = pack_bf16x2(acc[nt][2], acc[nt][3]);
            *reinterpret_cast<uint2*>(stage + (nt * 16 + lrow) * pitch + m * 32 + lk * 8) = o;
          }
        }
        flush(reinterpret_cast<uint8_t*>(cache) + mt0 * 32, (int64_t)r * 2, gt * 2);
      }
    } else {
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
      // One 64-channel quantisation group (4 channel tiles, fewer in a short last group) at a time:
      // code = clamp(rne((y - zero) / scale), 0, 2^bits - 1), the same float32 operations as the
      // few-token path.  A lane holds 4 consecutive channels of a token per tile; the 4 lanes that
      // share a token sit 16 apart.
      constexpr float top = (float)((1 << QBITS) - 1);
      const int ng = (r + 63) >> 6;
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
#pragma unroll
          for (int m = 0; m < 4; ++m)
            if (m < mtn) {
              uint32_t c[4];
#pragma unroll
              for (int e = 0; e < 4; ++e)
                c[e] = (uint32_t)fminf(fmaxf(rintf(__fdiv_rn(acc[m][nt][e] - zero, scale)), 0.f), top);
              const int ch = (mt0 + m) * 16 + lk * 4;                            // first of this lane's 4 channels
              uint8_t* srow = stage + (nt * 16 + lrow) * pitch;                  // the whole row of codes is staged
              if constexpr (QBITS == 8)
                *reinterpret_cast<uint32_t*>(srow + ch) = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
              else
                *reinterpret_cast<uint16_t*>(srow + (ch >> 1)) = (uint16_t)(c[0] | (c[1] << 4) | (c[2] << 8) | (c[3] << 12));
            }
        }
      }
      const int row_bytes = QBITS == 8 ? r : r >> 1;
      flush(reinterpret_cast<uint8_t*>(cache), row_bytes, row_bytes >> 4);
    }
    // The next tile's destination rows (the last flush has read this tile's), then this set's next token
    // rows, as the last thing, so that they stay on their way while the other set is worked on.  (Requested
    // without a condition they cost more than the exact waits gain: a wave of a 4096-token chunk has two tiles
    // and would request four.)
    plan_rows(m0 + stride);
    if (m0 + 2 * stride < M) load_token_frags<STREAM>(p, x, h, m0 + 2 * stride, M, lrow, lk, cur);
  };
  if (m0 >= M) return;                           // no barrier below this point
  plan_rows(m0);
  // Two tiles per turn and one way out: with a way out between the two, the paths that meet at the top of
  // the loop differ in what they have requested last, and the wait there becomes a wait for everything.  A
  // second tile past the end computes on re-read rows and stores nothing (its destination rows are all -1).
  while (true) {
    process(fa, m0);
    m0 += stride;
    process(fb, m0);
    m0 += stride;
    if (m0 >= M) break;
  }
}

}  // namespace

hipError_t launch_append(const AppendParams& p, hipStream_t stream) {
  const int64_t rows = (int64_t)p.batch * p.T;
  if (rows <= kVectorAppendMaxRows) return launch_project(&p, nullptr, stream);
  const int tokens_per_wave = tiles_per_wave(p.qbits) * 16;
  int64_t blocks = (rows + 4 * tokens_per_wave - 1) / (4 * tokens_per_wave);
  if (blocks > kMaxBlocksPerHead) blocks = kMaxBlocksPerHead;
  const dim3 grid((unsigned)blocks, (unsigned)p.n_kv_heads, 2u);
  const int lds_k = append_lds_bytes(p.r_k, tokens_per_wave), lds_v = append_lds_bytes(p.r_v, tokens_per_wave);
  const size_t lds = (size_t)(lds_k > lds_v ? lds_k : lds_v);
  auto launch = [&](auto kernel) -> hipError_t {
    if (lds > 48 * 1024) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, grid, dim3(256), lds, stream, p);
    return hipGetLastError();
  };
  // A chunk that is clearly larger than the 256 MiB last-level cache is read with streaming loads (5 % faster
  // at 0.5 GB); a smaller one has usually just been written and is found in the caches (streaming loads: 25 %
  // slower at 134 MB).
  const bool stream_in = 2 * rows * p.n_kv_heads * SKV_HEAD_DIM * (int64_t)sizeof(uint16_t) > (288ll << 20);
  if (p.qbits == 8) return stream_in ? launch(append_mfma_kernel<8, true>) : launch(append_mfma_kernel<8, false>);
  if (p.qbits == 4) return stream_in ? launch(append_mfma_kernel<4, true>) : launch(append_mfma_kernel<4, false>);
  return stream_in ? launch(append_mfma_kernel<0, true>) : launch(append_mfma_kernel<0, false>);
}

}  // namespace skv
