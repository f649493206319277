// Split-context decode attention over the compressed cache: query projection,
// scores, online softmax and value mix for one context range of one KV head.
//
// This file is compiled once per key rank (-DSKV_RK=16,32,...,128); each
// object holds the kernels for that r_K and every r_V in {16,...,128} and
// 1, 2 or 4 query heads per workgroup.
//
// What is computed (App. A.1 Eq. 18 on the reconstructed cache of Sec. 3.2
// Eq. 7, in the factored form q K~^T = (q P_K) K_down^T,
// softmax(.) V~ = (softmax(.) V_down) P_V^T):
//   q~[g]   = (q[g] . P_K) * scale * log2(e)               per query head g of the group
//   s[g][j] = <q~[g], K_down[j]>                            j in this range
//   m, l, a = running max, normaliser and sum_j 2^(s_j - m) V_down[j]
// written per (sequence, query head, range) for the combine kernel.
//
// Mapping.  The (b, kv-head) stream K_down[0:n][r_K] is one contiguous span, so
// any run of rows is a coalesced segment whatever the rank.  Eight lanes (an
// "octet") share one cache row: lane j of the octet owns the j-th eighth of
// the first 128 bytes of the row and the j-th eighth of the rest, which keeps
// every load a 4..16-byte piece that is contiguous across the octet.  A
// 64-lane wave therefore covers 8 consecutive rows per load, U loads deep.
// Scores are reduced across the octet with DPP adds (no LDS); each octet runs
// its own online-softmax stream and streams are merged once at the end.
#include "skv_internal.h"

#ifndef SKV_RK
#error "compile with -DSKV_RK=<key rank>"
#endif

namespace skv {
namespace {

constexpr float kNegBig = -1.0e30f;   // "no score seen yet"; finite so that differences stay finite

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// How the r channels of a row are dealt to the 8 lanes of an octet.
template <int R>
struct RowMap {
  static constexpr int NA = R < 64 ? R : 64;   // channels in the first segment (<= 128 bytes)
  static constexpr int NB = R - NA;            // channels in the second segment
  static constexpr int CA = NA / 8;            // channels per lane, first segment: 2,4,6,8
  static constexpr int CB = NB / 8;            // second segment: 0,2,4,6,8
  static constexpr int DA = CA / 2;            // dwords per lane
  static constexpr int DB = CB / 2;
  static constexpr int CPL = CA + CB;          // channels per lane
  static constexpr int DPL = DA + DB;          // dwords per lane
  static constexpr int ROW_DW = R / 2;         // dwords per row
  // channel held in slot i of lane j
  __device__ static constexpr int chan(int j, int i) {
    return i < CA ? j * CA + i : NA + j * CB + (i - CA);
  }
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int N>
__device__ __forceinline__ void load_dwords(const uint32_t* p, uint32_t* w) {
  if constexpr (N == 1) {
    w[0] = __builtin_nontemporal_load(p);
  } else if constexpr (N == 2) {
    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
    w[0] = v.x; w[1] = v.y;
  } else if constexpr (N == 3) {
    w[0] = __builtin_nontemporal_load(p);
    w[1] = __builtin_nontemporal_load(p + 1);
    w[2] = __builtin_nontemporal_load(p + 2);
  } else if constexpr (N == 4) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  }
}

template <int R>
__device__ __forceinline__ void load_row(const uint32_t* row, int j, uint32_t (&w)[RowMap<R>::DPL]) {
  using M = RowMap<R>;
  load_dwords<M::DA>(row + j * M::DA, &w[0]);
  if constexpr (M::DB > 0) load_dwords<M::DB>(row + 32 + j * M::DB, &w[M::DA]);
}

template <int R>
__device__ __forceinline__ void unpack_row(const uint32_t (&w)[RowMap<R>::DPL], float (&f)[RowMap<R>::CPL]) {
#pragma unroll
  for (int i = 0; i < RowMap<R>::DPL; ++i) {
    f[2 * i] = bf16_lo(w[i]);
    f[2 * i + 1] = bf16_hi(w[i]);
  }
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Sum over the 8 lanes of an octet; every lane receives the same bits.
__device__ __forceinline__ float octet_sum(float x) {
  x += dpp_f32<0x141>(x);   // row_half_mirror: lane i <-> 7-i
  x += dpp_f32<0xB1>(x);    // quad_perm [1,0,3,2]
  x += dpp_f32<0x4E>(x);    // quad_perm [2,3,0,1]
  return x;
}

// Rows in flight per lane: about 16 dwords of keys and of values.
template <int RK, int RV>
struct Depth {
  static constexpr int kMaxDw = RowMap<RK>::DPL > RowMap<RV>::DPL ? RowMap<RK>::DPL : RowMap<RV>::DPL;
  static constexpr int U = kMaxDw <= 2 ? 8 : (kMaxDw <= 4 ? 4 : 2);
};

// One pass over 8*U rows of a wave.  row0 is this lane's first row; the lane's
// rows are row0 + 8u.  With MASKED, rows >= t_end are ignored (their loads are
// redirected to row t_end-1 so that nothing outside [0, n_ctx) is ever read).
template <int RK, int RV, int GT, int U, bool MASKED>
__device__ __forceinline__ void process_rows(const uint32_t* __restrict__ kbase,
                                             const uint32_t* __restrict__ vbase, int row0, int t_end,
                                             int j, const float (&qreg)[GT][RowMap<RK>::CPL],
                                             float (&m)[GT], float (&l)[GT],
                                             float (&acc)[GT][RowMap<RV>::CPL]) {
  using KM = RowMap<RK>;
  using VM = RowMap<RV>;
  uint32_t kw[U][KM::DPL];
  uint32_t vw[U][VM::DPL];
  bool valid[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int row = row0 + 8 * u;
    valid[u] = true;
    if constexpr (MASKED) {
      valid[u] = row < t_end;
      row = valid[u] ? row : t_end - 1;
    }
    load_row<RK>(kbase + (int64_t)row * KM::ROW_DW, j, kw[u]);
    load_row<RV>(vbase + (int64_t)row * VM::ROW_DW, j, vw[u]);
  }

  float s[U][GT];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float kf[KM::CPL];
    unpack_row<RK>(kw[u], kf);
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float d = 0.f;
#pragma unroll
      for (int i = 0; i < KM::CPL; ++i) d = fmaf(qreg[g][i], kf[i], d);
      s[u][g] = d;
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float t = octet_sum(s[u][g]);
      if constexpr (MASKED) t = valid[u] ? t : kNegBig;
      s[u][g] = t;
    }
  }

  float pw[U][GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    float mx = s[0][g];
#pragma unroll
    for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u][g]);
    if (mx > m[g]) {                       // rare once the stream has warmed up
      const float c = fast_exp2(m[g] - mx);
      l[g] *= c;
#pragma unroll
      for (int i = 0; i < VM::CPL; ++i) acc[g][i] *= c;
      m[g] = mx;
    }
    float lsum = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float pv = fast_exp2(s[u][g] - m[g]);
      if constexpr (MASKED) pv = valid[u] ? pv : 0.f;
      pw[u][g] = pv;
      lsum += pv;
    }
    l[g] += lsum;
  }

#pragma unroll
  for (int u = 0; u < U; ++u) {
    float vf[VM::CPL];
    unpack_row<RV>(vw[u], vf);
#pragma unroll
    for (int g = 0; g < GT; ++g) {
#pragma unroll
      for (int i = 0; i < VM::CPL; ++i) acc[g][i] = fmaf(pw[u][g], vf[i], acc[g][i]);
    }
  }
}

template <int RK, int RV, int GT>
__global__ __launch_bounds__(kDecodeThreads) void decode_partial_kernel(const DecodeParams p) {
  using KM = RowMap<RK>;
  using VM = RowMap<RV>;
  constexpr int U = Depth<RK, RV>::U;
  constexpr int ROWS_PER_WAVE = 8 * U;
  constexpr int ROWS_PER_WG = 4 * ROWS_PER_WAVE;
  constexpr int D = SKV_HEAD_DIM;
  constexpr int DSLICES = 8;                     // head_dim split 8 ways for the query projection

  // LDS: query projection scratch, later reused for the cross-wave merge.
  constexpr int kProjFloats = GT * D + DSLICES * GT * RK + GT * RK;
  constexpr int kMergeFloats = 4 * GT * (RV + 2);
  constexpr int kLdsFloats = kProjFloats > kMergeFloats ? kProjFloats : kMergeFloats;
  __shared__ float lds[kLdsFloats];

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int oct = lane >> 3;
  const int j = lane & 7;

  const int split = blockIdx.x;
  const int passes = p.group / GT;
  const int col = blockIdx.y;                    // ((b * H_KV + kv) * passes + pass)
  const int pass = col % passes;
  const int bkv = col / passes;
  const int kv = bkv % p.n_kv_heads;
  const int b = bkv / p.n_kv_heads;
  const int hq0 = kv * p.group + pass * GT;      // first query head of this pass

  const int t0 = split * p.chunk;
  const int t1 = min(t0 + p.chunk, p.n_ctx);

  float* out_acc = p.part_acc + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + split) * RV;
  float* out_ml = p.part_ml + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + split) * 2;
  const int64_t head_step_acc = (int64_t)p.n_splits * RV;
  const int64_t head_step_ml = (int64_t)p.n_splits * 2;

  if (t0 >= p.n_ctx) {
    // Empty range: the neutral element of the merge.
    for (int i = tid; i < GT * RV; i += kDecodeThreads) out_acc[(i / RV) * head_step_acc + (i % RV)] = 0.f;
    if (tid < GT) { out_ml[tid * head_step_ml] = kNegBig; out_ml[tid * head_step_ml + 1] = 0.f; }
    return;
  }

  // ---- q~ = (q . P_K) * scale * log2(e) --------------------------------------------------
  float* q_s = lds;                              // [GT][D]
  float* part_s = lds + GT * D;                  // [DSLICES][GT][RK]
  float* qt_s = part_s + DSLICES * GT * RK;      // [GT][RK]
  const uint16_t* qptr = p.q + ((int64_t)b * p.n_q_heads + hq0) * D;
  for (int i = tid; i < GT * D; i += kDecodeThreads) q_s[i] = bf16_to_f32(qptr[i]);
  __syncthreads();
  const uint16_t* pk = p.p_k + (int64_t)kv * p.p_k_head_stride;
  for (int item = tid; item < RK * DSLICES; item += kDecodeThreads) {
    const int c = item % RK;
    const int ds = item / RK;
    float a[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g) a[g] = 0.f;
#pragma unroll 4
    for (int dd = 0; dd < D / DSLICES; ++dd) {
      const int d = ds * (D / DSLICES) + dd;
      const float w = bf16_to_f32(pk[d * RK + c]);
#pragma unroll
      for (int g = 0; g < GT; ++g) a[g] = fmaf(q_s[g * D + d], w, a[g]);
    }
#pragma unroll
    for (int g = 0; g < GT; ++g) part_s[(ds * GT + g) * RK + c] = a[g];
  }
  __syncthreads();
  for (int i = tid; i < GT * RK; i += kDecodeThreads) {
    const int g = i / RK, c = i % RK;
    float a = 0.f;
#pragma unroll
    for (int ds = 0; ds < DSLICES; ++ds) a += part_s[(ds * GT + g) * RK + c];
    qt_s[i] = a * p.scale_log2e;
  }
  __syncthreads();
  float qreg[GT][KM::CPL];
#pragma unroll
  for (int g = 0; g < GT; ++g)
#pragma unroll
    for (int i = 0; i < KM::CPL; ++i) qreg[g][i] = qt_s[g * RK + KM::chan(j, i)];

  // ---- stream the range ---------------------------------------------------------------
  const uint32_t* kbase = p.k_cache + ((int64_t)b * p.n_kv_heads + kv) * p.capacity * KM::ROW_DW;
  const uint32_t* vbase = p.v_cache + ((int64_t)b * p.n_kv_heads + kv) * p.capacity * VM::ROW_DW;

  float m[GT], l[GT], acc[GT][VM::CPL];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    m[g] = kNegBig;
    l[g] = 0.f;
#pragma unroll
    for (int i = 0; i < VM::CPL; ++i) acc[g][i] = 0.f;
  }

  int base = t0;
  for (; base + ROWS_PER_WG <= t1; base += ROWS_PER_WG)
    process_rows<RK, RV, GT, U, false>(kbase, vbase, base + wave * ROWS_PER_WAVE + oct, t1, j, qreg, m, l, acc);
  if (base < t1)
    process_rows<RK, RV, GT, U, true>(kbase, vbase, base + wave * ROWS_PER_WAVE + oct, t1, j, qreg, m, l, acc);

  // ---- merge the 8 octet streams of the wave (lanes 8, 16, 32 apart) ---------------------
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    float mw = m[g];
    mw = fmaxf(mw, __shfl_xor(mw, 8));
    mw = fmaxf(mw, __shfl_xor(mw, 16));
    mw = fmaxf(mw, __shfl_xor(mw, 32));
    const float f = fast_exp2(m[g] - mw);
    float lg = l[g] * f;
    lg += __shfl_xor(lg, 8);
    lg += __shfl_xor(lg, 16);
    lg += __shfl_xor(lg, 32);
    l[g] = lg;
    m[g] = mw;
#pragma unroll
    for (int i = 0; i < VM::CPL; ++i) {
      float a = acc[g][i] * f;
      a += __shfl_xor(a, 8);
      a += __shfl_xor(a, 16);
      a += __shfl_xor(a, 32);
      acc[g][i] = a;
    }
  }

  // ---- merge the 4 waves through LDS, in wave order -----------------------------------
  __syncthreads();                               // projection scratch no longer needed
  float* red = lds;                              // [4][GT][RV + 2]
  if (oct == 0) {
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float* r = red + (wave * GT + g) * (RV + 2);
#pragma unroll
      for (int i = 0; i < VM::CPL; ++i) r[VM::chan(j, i)] = acc[g][i];
      if (j == 0) { r[RV] = m[g]; r[RV + 1] = l[g]; }
    }
  }
  __syncthreads();
  for (int i = tid; i < GT * (RV + 2); i += kDecodeThreads) {
    const int g = i / (RV + 2), c = i % (RV + 2);
    float mt = red[(0 * GT + g) * (RV + 2) + RV];
#pragma unroll
    for (int w = 1; w < 4; ++w) mt = fmaxf(mt, red[(w * GT + g) * (RV + 2) + RV]);
    if (c == RV) {
      out_ml[g * head_step_ml] = mt;
    } else {
      const int src = c == RV + 1 ? RV + 1 : c;
      float a = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float* r = red + (w * GT + g) * (RV + 2);
        a += r[src] * fast_exp2(r[RV] - mt);
      }
      if (c == RV + 1) out_ml[g * head_step_ml + 1] = a;
      else out_acc[g * head_step_acc + c] = a;
    }
  }
}

template <int RK, int RV>
hipError_t launch_rv(int heads, const DecodeParams& p, hipStream_t stream) {
  const int passes = p.group / heads;
  const dim3 grid((unsigned)p.n_splits, (unsigned)(p.batch * p.n_kv_heads * passes));
  const dim3 block(kDecodeThreads);
  switch (heads) {
    case 1: hipLaunchKernelGGL((decode_partial_kernel<RK, RV, 1>), grid, block, 0, stream, p); break;
    case 2: hipLaunchKernelGGL((decode_partial_kernel<RK, RV, 2>), grid, block, 0, stream, p); break;
    case 4: hipLaunchKernelGGL((decode_partial_kernel<RK, RV, 4>), grid, block, 0, stream, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int RK>
hipError_t launch_rk(int r_v, int heads, const DecodeParams& p, hipStream_t stream) {
  switch (r_v) {
    case 16: return launch_rv<RK, 16>(heads, p, stream);
    case 32: return launch_rv<RK, 32>(heads, p, stream);
    case 48: return launch_rv<RK, 48>(heads, p, stream);
    case 64: return launch_rv<RK, 64>(heads, p, stream);
    case 80: return launch_rv<RK, 80>(heads, p, stream);
    case 96: return launch_rv<RK, 96>(heads, p, stream);
    case 112: return launch_rv<RK, 112>(heads, p, stream);
    case 128: return launch_rv<RK, 128>(heads, p, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace

#define SKV_CAT2(a, b) a##b
#define SKV_CAT(a, b) SKV_CAT2(a, b)
hipError_t SKV_CAT(launch_decode_partial_rk, SKV_RK)(int r_v, int heads, const DecodeParams& p,
                                                      hipStream_t stream) {
  return launch_rk<SKV_RK>(r_v, heads, p, stream);
}

}  // namespace skv
