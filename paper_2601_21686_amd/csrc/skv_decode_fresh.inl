// The extra workgroups of a fused decode step: the rows the step appends, projected (and, for a quantised
// cache, quantised), stored and attended, as one more partial result beside those of the context ranges.
// Included by skv_decode_partial.hip inside its namespaces; uses its constants and helpers.

// The projection of a pass's GT query rows.  The scratch of project_rows_finish grows with the row count; it
// is sized for four rows, so eight go in two halves (the basis pieces are held in registers across both).
template <int GT>
__device__ __forceinline__ void project_query_rows(const ProjectPieces& pp, int r, const float* x_s, float* part_s,
                                                   float* y_s) {
  if constexpr (GT <= 4) {
    project_rows_finish<GT>(pp, r, x_s, part_s, y_s);
  } else {
    static_assert(GT == 8, "one, two, four or eight query heads per pass");
    project_rows_finish<4>(pp, r, x_s, part_s, y_s);
    project_rows_finish<4>(pp, r, x_s + 4 * SKV_HEAD_DIM, part_s, y_s + 4 * r);
  }
}

// Everything a new-rows workgroup reads from global memory, requested at once before the first wait: the
// workgroup runs beside a chip full of streaming ones, where a round trip takes 3-5 us, and as a chain of
// request, wait, compute (queries, then per new token keys, then values) it lived 20-30 us -- as long as a whole
// range launch over a quantised cache.  Held in registers: the pieces of both bases (the key basis serves the
// queries and every new key), the raw queries, and the raw new rows of up to kFusedStepMaxTokens tokens (one
// element per thread and token).
template <int GT>
struct NewRowInputs {
  static constexpr int kQPerLane = (GT * SKV_HEAD_DIM + kDecodeThreads - 1) / kDecodeThreads;
  ProjectPieces ppk, ppv;
  uint32_t qraw[kQPerLane];
  uint32_t knew[kFusedStepMaxTokens], vnew[kFusedStepMaxTokens];
};
template <int RK, int RV, int GT>
__device__ __forceinline__ void request_new_row_inputs(const DecodeParams& p, int b, int kv, int hq0, NewRowInputs<GT>& in) {
  constexpr int D = SKV_HEAD_DIM;
  const int tid = threadIdx.x;
  project_rows_issue(p.p_k + (int64_t)kv * p.p_k_head_stride, RK, in.ppk);
  const uint16_t* qptr = p.q + ((int64_t)b * p.n_q_heads + hq0) * D;
#pragma unroll
  for (int k = 0; k < NewRowInputs<GT>::kQPerLane; ++k) in.qraw[k] = qptr[(tid + k * kDecodeThreads) % (GT * D)];
#pragma unroll
  for (int t = 0; t < kFusedStepMaxTokens; ++t) {
    in.knew[t] = 0u;
    in.vnew[t] = 0u;
    if (t < p.T_new && tid < D) {
      const int64_t src = (int64_t)b * p.stride_b + (int64_t)t * p.stride_t + (int64_t)kv * p.stride_h;
      in.knew[t] = p.k_new[src + tid];
      in.vnew[t] = p.v_new[src + tid];
    }
  }
  project_rows_issue(p.p_v + (int64_t)kv * p.p_v_head_stride, RV, in.ppv);
}
// the raw queries into x_s (synchronised), ready for project_query_rows
template <int GT>
__device__ __forceinline__ void stage_queries(const NewRowInputs<GT>& in, float* x_s) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int k = 0; k < NewRowInputs<GT>::kQPerLane; ++k)
    if (tid + k * kDecodeThreads < GT * SKV_HEAD_DIM) x_s[tid + k * kDecodeThreads] = bf16_to_f32((uint16_t)in.qraw[k]);
  __syncthreads();
}

#if !SKV_Q8
// The rows a decode step appends (Sec. 2.1 Eq. 1: k_down = k P_K, v_down = v P_V, rounded to bf16 and
// cached, Sec. 3.2) and their share of the attention, for one (sequence, KV head, pass): projects the
// T_new new keys and values exactly as the few-token append does (same sums, same rounding), stores
// them at rows [cur_len, cur_len + T_new), and attends them with the group's projected queries.  The
// result is one more partial (m, l, a~) for the combine kernel, so the streaming workgroups never
// have to wait for these rows to land in the cache.
template <int RK, int RV, int GT>
__device__ __forceinline__ void fresh_rows_block(const DecodeParams& p, int b, int kv, int pass, int hq0,
                                                 float* x_s, float* part_s, float* y_s) {
  constexpr int D = SKV_HEAD_DIM;
  __shared__ float qt_s[GT * RK];
  __shared__ float kd_s[RK];
  __shared__ float vd_s[RV];
  __shared__ float w_s[GT][2];                   // per head: factor of the sums so far, weight of the new row
  const int tid = threadIdx.x;
  NewRowInputs<GT> in;
  request_new_row_inputs<RK, RV, GT>(p, b, kv, hq0, in);
  stage_queries<GT>(in, x_s);
  project_query_rows<GT>(in.ppk, RK, x_s, part_s, y_s);
  for (int i = tid; i < GT * RK; i += kDecodeThreads) qt_s[i] = y_s[i] * p.scale_log2e;
  float m = kNegBig, l = 0.f;                    // thread g < GT: softmax state of head g
  float acc[GT];                                 // thread c < RV: channel c of every head's mix
#pragma unroll
  for (int g = 0; g < GT; ++g) acc[g] = 0.f;
#pragma unroll
  for (int t = 0; t < kFusedStepMaxTokens; ++t) {
    if (t >= p.T_new) break;
    const int64_t row = cache_row(p.pages, p.capacity, p.n_kv_heads, b, kv, clamped_len(p.seq_lens, b, p.cur_len) + t);
    {
      if (tid < D) x_s[tid] = bf16_to_f32((uint16_t)in.knew[t]);
      __syncthreads();
      project_rows_finish<1>(in.ppk, RK, x_s, part_s, y_s);
      if (tid < RK) {
        const uint32_t bits = f32_to_bf16_bits(y_s[tid]);
        if (pass == 0) p.k_cache_w[row * RK + tid] = (uint16_t)bits;
        kd_s[tid] = bf16_to_f32((uint16_t)bits);
      }
    }
    {
      if (tid < D) x_s[tid] = bf16_to_f32((uint16_t)in.vnew[t]);
      __syncthreads();
      project_rows_finish<1>(in.ppv, RV, x_s, part_s, y_s);
      if (tid < RV) {
        const uint32_t bits = f32_to_bf16_bits(y_s[tid]);
        if (pass == 0) p.v_cache_w[row * RV + tid] = (uint16_t)bits;
        vd_s[tid] = bf16_to_f32((uint16_t)bits);
      }
    }
    __syncthreads();
    if (tid < GT) {
      float sc = 0.f;
      for (int c = 0; c < RK; ++c) sc = fmaf(qt_s[tid * RK + c], kd_s[c], sc);
      const float mn = fmaxf(m, sc);
      const float alpha = fast_exp2(m - mn);
      const float pw = fast_exp2(sc - mn);
      l = l * alpha + pw;
      m = mn;
      w_s[tid][0] = alpha;
      w_s[tid][1] = pw;
    }
    __syncthreads();
    if (tid < RV) {
#pragma unroll
      for (int g = 0; g < GT; ++g) acc[g] = acc[g] * w_s[g][0] + w_s[g][1] * vd_s[tid];
    }
    __syncthreads();
  }
  float* out_acc = p.part_acc + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + p.n_stream) * RV;
  float* out_ml = p.part_ml + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + p.n_stream) * 2;
  if (tid < RV) {
#pragma unroll
    for (int g = 0; g < GT; ++g) out_acc[(int64_t)g * p.n_splits * RV + tid] = acc[g];
  }
  if (tid < GT) {
    out_ml[(int64_t)tid * p.n_splits * 2] = m;
    out_ml[(int64_t)tid * p.n_splits * 2 + 1] = l;
  }
}
#endif

#if SKV_Q8
// The rows a decode step appends to a QUANTISED cache, and their share of the attention, for one (sequence,
// KV head, pass): projected like the few-token append, quantised with the same float32 arithmetic (keys on the
// static range of their head and group, values on the row's own range per group, kept as bf16), stored, and
// attended as the range kernel will see them from the next step on.  Scores are taken in the range kernel's
// convention -- the folded queries against the integer codes, i.e. shifted by a constant per query, the same
// in every partial of the launch -- and the mix uses the dequantised values scale * code + zero.
template <int RK, int RV, int GT>
__device__ __forceinline__ void fresh_rows_block_q(const DecodeParams& p, int b, int kv, int pass, int hq0,
                                                   float* x_s, float* part_s, float* y_s) {
  constexpr int D = SKV_HEAD_DIM;
  constexpr int NGK = (RK + 63) / 64, NGV = (RV + 63) / 64;
  __shared__ float qt_s[GT * RK];
  __shared__ float kc_s[RK];
  __shared__ float vd_s[RV];
  __shared__ float w_s[GT][2];
  const int tid = threadIdx.x;
  const float top = (float)((1 << SKV_QBITS) - 1);
  NewRowInputs<GT> in;
  request_new_row_inputs<RK, RV, GT>(p, b, kv, hq0, in);
  uint8_t* k_codes = reinterpret_cast<uint8_t*>(p.k_cache_w);
  uint8_t* v_codes = reinterpret_cast<uint8_t*>(p.v_cache_w);
  uint32_t* v_meta = const_cast<uint32_t*>(p.v_meta);
  stage_queries<GT>(in, x_s);
  project_query_rows<GT>(in.ppk, RK, x_s, part_s, y_s);
  for (int i = tid; i < GT * RK; i += kDecodeThreads)
    qt_s[i] = y_s[i] * p.scale_log2e * p.k_scale[kv * NGK + ((i % RK) >> 6)];
  // code = clamp(rne((y - zero) / scale), 0, 2^bits - 1), stored 8 bits: one byte per channel; 4 bits: channel 2c in
  // the low half of byte c.  Thread c holds channel c; 64-channel group g is wave g.
  auto store_code = [&](uint8_t* codes, int64_t row, int r, uint32_t code, bool live) {
    if (SKV_QBITS == 8) {
      if (live && pass == 0) codes[row * r + tid] = (uint8_t)code;
    } else {
      const uint32_t next = __shfl_down(code, 1);
      if (live && pass == 0 && (tid & 1) == 0) codes[(row * r + tid) >> 1] = (uint8_t)(code | (next << 4));
    }
  };
  float m = kNegBig, l = 0.f;
  float acc[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) acc[g] = 0.f;
#pragma unroll
  for (int t = 0; t < kFusedStepMaxTokens; ++t) {
    if (t >= p.T_new) break;
    const int64_t row = cache_row(p.pages, p.capacity, p.n_kv_heads, b, kv, clamped_len(p.seq_lens, b, p.cur_len) + t);
    {
      if (tid < D) x_s[tid] = bf16_to_f32((uint16_t)in.knew[t]);
      __syncthreads();
      project_rows_finish<1>(in.ppk, RK, x_s, part_s, y_s);
      const bool live = tid < RK;
      const float y = live ? y_s[tid] : 0.f;
      const float scale = live ? p.k_scale[kv * NGK + (tid >> 6)] : 1.f;
      const float zero = live ? p.k_zero[kv * NGK + (tid >> 6)] : 0.f;
      const uint32_t code = live ? (uint32_t)fminf(fmaxf(rintf(__fdiv_rn(y - zero, scale)), 0.f), top) : 0u;
      store_code(k_codes, row, RK, code, live);
      if (live) kc_s[tid] = (float)code;
    }
    {
      if (tid < D) x_s[tid] = bf16_to_f32((uint16_t)in.vnew[t]);
      __syncthreads();
      project_rows_finish<1>(in.ppv, RV, x_s, part_s, y_s);
      const bool live = tid < RV;
      const float y = live ? y_s[tid] : 0.f;
      float lo = live ? y : 3.0e38f, hi = live ? y : -3.0e38f;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
      }
      uint32_t sb = f32_to_bf16_bits(__fdiv_rn(hi - lo, top));
      if ((sb & 0x7fffu) == 0) sb = 0x3F80u;       // flat group: scale 1
      const uint32_t zb = f32_to_bf16_bits(lo);
      const float scale = __uint_as_float(sb << 16), zero = __uint_as_float(zb << 16);
      if (live && pass == 0 && (tid & 63) == 0) v_meta[row * NGV + (tid >> 6)] = sb | (zb << 16);
      const uint32_t code = live ? (uint32_t)fminf(fmaxf(rintf(__fdiv_rn(y - zero, scale)), 0.f), top) : 0u;
      store_code(v_codes, row, RV, code, live);
      if (live) vd_s[tid] = fmaf((float)code, scale, zero);
    }
    __syncthreads();
    if (tid < GT) {
      float sc = 0.f;
      for (int c = 0; c < RK; ++c) sc = fmaf(qt_s[tid * RK + c], kc_s[c], sc);
      const float mn = fmaxf(m, sc);
      const float alpha = fast_exp2(m - mn);
      const float pw = fast_exp2(sc - mn);
      l = l * alpha + pw;
      m = mn;
      w_s[tid][0] = alpha;
      w_s[tid][1] = pw;
    }
    __syncthreads();
    if (tid < RV) {
#pragma unroll
      for (int g = 0; g < GT; ++g) acc[g] = acc[g] * w_s[g][0] + w_s[g][1] * vd_s[tid];
    }
    __syncthreads();
  }
  float* out_acc = p.part_acc + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + p.n_stream) * RV;
  float* out_ml = p.part_ml + (((int64_t)b * p.n_q_heads + hq0) * p.n_splits + p.n_stream) * 2;
  if (tid < RV) {
#pragma unroll
    for (int g = 0; g < GT; ++g) out_acc[(int64_t)g * p.n_splits * RV + tid] = acc[g];
  }
  if (tid < GT) {
    out_ml[(int64_t)tid * p.n_splits * 2] = m;
    out_ml[(int64_t)tid * p.n_splits * 2 + 1] = l;
  }
}
#endif  // SKV_Q8
