// Causal grouped-query attention on the vector ALUs (fp32 accumulation), for fp32 models and as the
// shape-agnostic fallback of the MFMA kernel.  One wave per (64 query rows, head, sample): each lane owns
// one query row (q and the output accumulator live in registers), K/V tiles of 32 keys are staged in LDS
// and read as broadcasts, softmax is the usual running (max, sum) recurrence per tile.  The lane that owns
// a sample's last row also emits that row's scaled logits and final (max, sum): the side output Eq. 4 is
// finalised from.
#include "common.hpp"

namespace fastav {

template <typename T, int DH>
__global__ __launch_bounds__(64) void k_attn_generic(const T* __restrict__ q, int64_t q_stride,
                                                     const T* __restrict__ k, const T* __restrict__ v,
                                                     int64_t kv_stride, T* __restrict__ o, int64_t o_stride,
                                                     const int32_t* __restrict__ cu, int Hq, int Hkv, float scale,
                                                     int64_t T_total, float* __restrict__ last_logits,
                                                     float* __restrict__ last_ml) {
  constexpr int KT = 32;
  __shared__ float Ks[KT][DH];
  __shared__ float Vs[KT][DH];
  const int b = blockIdx.z, h = blockIdx.y;
  const int row0 = cu[b], n = cu[b + 1] - row0;
  const int i0 = blockIdx.x * 64;
  if (i0 >= n) return;
  const int tid = threadIdx.x;
  const int i = i0 + tid;
  const bool active = i < n;
  const int g = h / (Hq / Hkv);
  const bool emit = active && (i == n - 1) && (last_logits != nullptr);

  float qr[DH], acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    qr[c] = active ? to_f32(q[(int64_t)(row0 + i) * q_stride + h * DH + c]) : 0.f;
    acc[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int last_key = (i0 + 64 < n ? i0 + 64 : n) - 1;
  for (int j0 = 0; j0 <= last_key; j0 += KT) {
    __syncthreads();
    for (int e = tid; e < KT * DH; e += 64) {
      const int jj = e / DH, c = e % DH;
      const int j = j0 + jj;
      const bool ok = j < n;
      Ks[jj][c] = ok ? to_f32(k[(int64_t)(row0 + j) * kv_stride + g * DH + c]) : 0.f;
      Vs[jj][c] = ok ? to_f32(v[(int64_t)(row0 + j) * kv_stride + g * DH + c]) : 0.f;
    }
    __syncthreads();
    float s[KT];
    float tmax = -INFINITY;
#pragma unroll
    for (int jj = 0; jj < KT; ++jj) {
      float d = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) d = fmaf(qr[c], Ks[jj][c], d);
      d *= scale;
      const int j = j0 + jj;
      const bool vis = active && j <= i;
      s[jj] = vis ? d : -INFINITY;
      tmax = fmaxf(tmax, s[jj]);
      if (emit && vis) last_logits[(int64_t)h * T_total + row0 + j] = d;
    }
    const float m_new = fmaxf(m, tmax);
    if (m_new > -INFINITY) {
      const float corr = expf(m - m_new);                    // m = -inf -> 0
      l *= corr;
#pragma unroll
      for (int c = 0; c < DH; ++c) acc[c] *= corr;
#pragma unroll
      for (int jj = 0; jj < KT; ++jj) {
        const float p = expf(s[jj] - m_new);                 // masked -> 0
        l += p;
#pragma unroll
        for (int c = 0; c < DH; ++c) acc[c] = fmaf(p, Vs[jj][c], acc[c]);
      }
    }
    m = m_new;
  }
  if (active) {
    const float inv = 1.0f / l;
#pragma unroll
    for (int c = 0; c < DH; ++c) o[(int64_t)(row0 + i) * o_stride + h * DH + c] = from_f32<T>(acc[c] * inv);
    if (emit && last_ml) {
      last_ml[((int64_t)b * Hq + h) * 2] = m;
      last_ml[((int64_t)b * Hq + h) * 2 + 1] = l;
    }
  }
}

fastav_status_t launch_attention_generic(const void* q, int64_t q_stride, const void* k, const void* v,
                                         int64_t kv_stride, void* o, int64_t o_stride, const int32_t* cu, int batch,
                                         int64_t T, int max_seqlen, int Hq, int Hkv, int dh, float* last_logits,
                                         float* last_ml, int dtype, hipStream_t s) {
  if (batch == 0 || max_seqlen == 0) return FASTAV_OK;
  dim3 grid((unsigned)ceil_div(max_seqlen, 64), (unsigned)Hq, (unsigned)batch);
  const float scale = 1.0f / sqrtf((float)dh);
#define FASTAV_ATTN_CASE(TT, DHH)                                                                                \
  hipLaunchKernelGGL((k_attn_generic<TT, DHH>), grid, dim3(64), 0, s, (const TT*)q, q_stride, (const TT*)k,     \
                     (const TT*)v, kv_stride, (TT*)o, o_stride, cu, Hq, Hkv, scale, T, last_logits, last_ml)
  if (dtype == FASTAV_BF16) { if (dh == 128) FASTAV_ATTN_CASE(bf16_t, 128); else FASTAV_ATTN_CASE(bf16_t, 64); }
  else { if (dh == 128) FASTAV_ATTN_CASE(float, 128); else FASTAV_ATTN_CASE(float, 64); }
#undef FASTAV_ATTN_CASE
  return check_launch("attention_generic");
}

}  // namespace fastav
