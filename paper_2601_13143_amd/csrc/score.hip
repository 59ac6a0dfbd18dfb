// Eq. 4 of the paper: s = mean over heads of softmax(Q_last K^T), computed without the attention map.
//
//   k_score_logits   streams K once (coalesced 16-byte loads, fp32 FMA on the vector ALUs — the work is
//                    ~4-7 flop per byte, far below the MFMA ridge, so it is laid out for bandwidth, not
//                    for the matrix cores) and writes the scaled logits of the last query row(s) plus a
//                    per-chunk (max, sum-exp) partial for every head.
//   k_score_finalize merges the partials into each head's (max, sum) and writes
//                    s_j = 1/(Hq*rows) * sum_{row,h} exp(L[row,h,j] - m[row,h]) / l[row,h].
//                    The flash-attention kernel can hand it (m, l) directly (its side output).
#include "common.hpp"

namespace fastav {

constexpr int kScoreChunk = 128;   // keys per workgroup

template <typename T> struct Vec16;
template <> struct Vec16<bf16_t> { typedef bf16x8_t type; static constexpr int n = 8; };
template <> struct Vec16<float> { typedef f32x4_t type; static constexpr int n = 4; };

// Sum over the LPR adjacent lanes that share one K row (LPR is a power of two <= 32).
template <int LPR> __device__ __forceinline__ float sub_sum(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// G_T > 0: the Hq/Hkv query heads of this lane's KV head are held in registers (needs n_sub >= Hkv).
// G_T == 0: generic path, q fragments are re-read from LDS for whatever KV head the row belongs to.
template <typename T, int DH, int G_T>
__global__ __launch_bounds__(256) void k_score_logits(const T* __restrict__ q, int64_t q_stride,
                                                      const T* __restrict__ k, int64_t k_stride,
                                                      const int32_t* __restrict__ cu, int Hq, int Hkv, int n_last,
                                                      float scale, int64_t T_total, int64_t n_chunk_slots,
                                                      float* __restrict__ logits, float* __restrict__ partials) {
  typedef typename Vec16<T>::type vec_t;
  constexpr int VEC = Vec16<T>::n;
  constexpr int LPR = DH / VEC;              // lanes per (key, kv-head) row
  constexpr int NSUB = 256 / LPR;            // sub-groups per workgroup
  extern __shared__ float smem[];
  float* qs = smem;                          // [Hq][DH] fp32: the current query row
  float* outs = smem + Hq * DH;              // [Hq][kScoreChunk] staged logits

  const int b = blockIdx.y;
  const int row0 = cu[b], n = cu[b + 1] - row0;
  const int j0 = blockIdx.x * kScoreChunk;
  if (j0 >= n) return;
  const int n_rows = n_last < n ? n_last : n;
  const int G = Hq / Hkv;
  const int sub = threadIdx.x / LPR, lis = threadIdx.x % LPR;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;

  for (int rl = 0; rl < n_rows; ++rl) {
    const int r = n - n_rows + rl;                         // query row; it sees keys 0..r
    __syncthreads();
    for (int i = threadIdx.x; i < Hq * DH; i += 256) qs[i] = to_f32(q[(int64_t)(row0 + r) * q_stride + i]);
    for (int i = threadIdx.x; i < Hq * kScoreChunk; i += 256) outs[i] = -INFINITY;
    __syncthreads();

    if (G_T > 0) {
      const int per_pass = NSUB / Hkv;                     // keys handled per pass
      if (sub < per_pass * Hkv) {
        const int g = sub % Hkv;
        float qr[(G_T > 0 ? G_T : 1)][VEC];
#pragma unroll
        for (int i = 0; i < G_T; ++i)
#pragma unroll
          for (int c = 0; c < VEC; ++c) qr[i][c] = qs[(g * G_T + i) * DH + lis * VEC + c];
        for (int jj = sub / Hkv; jj < kScoreChunk; jj += per_pass) {
          const int j = j0 + jj;
          if (j > r) break;                                // keys beyond the query row are invisible (and j <= r < n)
          const vec_t kv = *(const vec_t*)(k + (int64_t)(row0 + j) * k_stride + g * DH + lis * VEC);
          float acc[(G_T > 0 ? G_T : 1)];
#pragma unroll
          for (int i = 0; i < G_T; ++i) acc[i] = 0.f;
#pragma unroll
          for (int c = 0; c < VEC; ++c) {
            const float kc = to_f32(kv[c]);
#pragma unroll
            for (int i = 0; i < G_T; ++i) acc[i] = fmaf(qr[i][c], kc, acc[i]);
          }
#pragma unroll
          for (int i = 0; i < G_T; ++i) {
            const float tot = sub_sum<LPR>(acc[i]);
            if (lis == 0) outs[(g * G_T + i) * kScoreChunk + jj] = tot * scale;
          }
        }
      }
    } else {
      const int n_rows_kv = kScoreChunk * Hkv;
      for (int rho = sub; rho < n_rows_kv; rho += NSUB) {
        const int jj = rho / Hkv, g = rho % Hkv;
        const int j = j0 + jj;
        if (j > r) break;
        const vec_t kv = *(const vec_t*)(k + (int64_t)(row0 + j) * k_stride + g * DH + lis * VEC);
        float kf[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) kf[c] = to_f32(kv[c]);
        for (int i = 0; i < G; ++i) {
          const float* qp = qs + (g * G + i) * DH + lis * VEC;
          float acc = 0.f;
#pragma unroll
          for (int c = 0; c < VEC; ++c) acc = fmaf(qp[c], kf[c], acc);
          const float tot = sub_sum<LPR>(acc);
          if (lis == 0) outs[(g * G + i) * kScoreChunk + jj] = tot * scale;
        }
      }
    }
    __syncthreads();

    // per-head (max, sum-exp) of this chunk + coalesced store of the logits
    for (int h = wave; h < Hq; h += 4) {
      const float a0 = outs[h * kScoreChunk + lane], a1 = outs[h * kScoreChunk + 64 + lane];
      const float m = wave_max(fmaxf(a0, a1));
      float e = 0.f;
      if (m > -INFINITY) e = expf(a0 - m) + expf(a1 - m);
      e = wave_sum(e);
      float* lg = logits + ((int64_t)rl * Hq + h) * T_total + row0 + j0;
      if (j0 + lane < n) lg[lane] = a0;
      if (j0 + 64 + lane < n) lg[64 + lane] = a1;
      if (lane == 0) {
        // chunk slot of (sample b, chunk c): row0/chunk + b + c  (sum of earlier samples' chunk counts <= row0/chunk + b)
        float* p = partials + (((int64_t)rl * Hq + h) * n_chunk_slots + row0 / kScoreChunk + b + blockIdx.x) * 2;
        p[0] = m; p[1] = e;
      }
    }
  }
}

// ml_in != nullptr: per-head (m, l) given as [batch, n_last, Hq, 2]; else merged here from partials.
__global__ __launch_bounds__(256) void k_score_finalize(const float* __restrict__ logits,
                                                        const float* __restrict__ ml_in,
                                                        const float* __restrict__ partials, int64_t n_chunk_slots,
                                                        const int32_t* __restrict__ cu, int Hq, int n_last,
                                                        int64_t T_total, float* __restrict__ scores) {
  extern __shared__ float mls[];                           // [n_rows*Hq][2] : (m, 1/l)
  const int b = blockIdx.y;
  const int row0 = cu[b], n = cu[b + 1] - row0;
  if ((int)(blockIdx.x * 256) >= n) return;
  const int n_rows = n_last < n ? n_last : n;
  for (int idx = threadIdx.x; idx < n_rows * Hq; idx += 256) {
    const int rl = idx / Hq, h = idx % Hq;
    float m, l;
    if (ml_in) {
      const float* p = ml_in + (((int64_t)b * n_last + rl) * Hq + h) * 2;
      m = p[0]; l = p[1];
    } else {
      const float* p = partials + (((int64_t)rl * Hq + h) * n_chunk_slots + row0 / kScoreChunk + b) * 2;
      const int nc = (n + kScoreChunk - 1) / kScoreChunk;
      m = -INFINITY;
      for (int c = 0; c < nc; ++c) m = fmaxf(m, p[2 * c]);
      l = 0.f;
      for (int c = 0; c < nc; ++c) { const float mc = p[2 * c]; if (mc > -INFINITY) l += p[2 * c + 1] * expf(mc - m); }
    }
    mls[2 * idx] = m; mls[2 * idx + 1] = 1.0f / l;
  }
  __syncthreads();
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  float s = 0.f;
  for (int idx = 0; idx < n_rows * Hq; ++idx) {
    const float L = logits[(int64_t)idx * T_total + row0 + j];   // idx = rl*Hq + h
    s += expf(L - mls[2 * idx]) * mls[2 * idx + 1];
  }
  scores[row0 + j] = s / (float)(n_rows * Hq);
}

// Chunk slots of the whole packed batch: sample b's chunks start at slot cu[b]/chunk + b.
static int64_t chunk_slots(int64_t T, int batch) { return T / kScoreChunk + batch + 1; }

size_t score_partials_bytes(int Hq, int64_t T, int batch, int n_last) {
  return (size_t)n_last * Hq * chunk_slots(T, batch) * 2 * sizeof(float);
}

template <typename T, int DH>
static void dispatch_logits(int G, bool reg_ok, dim3 grid, size_t shmem, hipStream_t s, const T* q, int64_t qs,
                            const T* k, int64_t ks, const int32_t* cu, int Hq, int Hkv, int n_last, float scale,
                            int64_t Tt, int64_t ncm, float* logits, float* partials) {
#define FASTAV_SCORE_CASE(GT)                                                                                 \
  hipLaunchKernelGGL((k_score_logits<T, DH, GT>), grid, dim3(256), shmem, s, q, qs, k, ks, cu, Hq, Hkv, n_last, \
                     scale, Tt, ncm, logits, partials)
  if (reg_ok && G == 1) FASTAV_SCORE_CASE(1);
  else if (reg_ok && G == 2) FASTAV_SCORE_CASE(2);
  else if (reg_ok && G == 4) FASTAV_SCORE_CASE(4);
  else if (reg_ok && G == 7) FASTAV_SCORE_CASE(7);
  else if (reg_ok && G == 8) FASTAV_SCORE_CASE(8);
  else FASTAV_SCORE_CASE(0);
#undef FASTAV_SCORE_CASE
}

fastav_status_t launch_score_logits(const void* q, int64_t q_stride, const void* k, int64_t k_stride,
                                    const int32_t* cu, int batch, int64_t T, int max_seqlen, int Hq, int Hkv, int dh,
                                    int n_last, float* logits, float* partials, int dtype, hipStream_t s) {
  if (batch == 0 || max_seqlen == 0) return FASTAV_OK;
  ProfScope prof(FASTAV_PROF_SCORE, (double)T * Hkv * dh * (dtype == FASTAV_BF16 ? 2.0 : 4.0) + 4.0 * n_last * Hq * T, s);
  const int64_t ncm = chunk_slots(T, batch);
  dim3 grid((unsigned)ceil_div(max_seqlen, kScoreChunk), (unsigned)batch);
  const size_t shmem = (size_t)Hq * (dh + kScoreChunk) * sizeof(float);
  const float scale = 1.0f / sqrtf((float)dh);
  const int G = Hq / Hkv;
  const int vec = dtype == FASTAV_BF16 ? 8 : 4;
  const int nsub = 256 / (dh / vec);
  const bool reg_ok = nsub >= Hkv;
  if (shmem > 64 * 1024) return fail(FASTAV_EUNSUPPORTED, "score: n_q_heads*(head_dim+128)*4 bytes must fit 64 KB of LDS");
  if (dtype == FASTAV_BF16) {
    if (dh == 128) dispatch_logits<bf16_t, 128>(G, reg_ok, grid, shmem, s, (const bf16_t*)q, q_stride, (const bf16_t*)k, k_stride, cu, Hq, Hkv, n_last, scale, T, ncm, logits, partials);
    else dispatch_logits<bf16_t, 64>(G, reg_ok, grid, shmem, s, (const bf16_t*)q, q_stride, (const bf16_t*)k, k_stride, cu, Hq, Hkv, n_last, scale, T, ncm, logits, partials);
  } else {
    if (dh == 128) dispatch_logits<float, 128>(G, reg_ok, grid, shmem, s, (const float*)q, q_stride, (const float*)k, k_stride, cu, Hq, Hkv, n_last, scale, T, ncm, logits, partials);
    else dispatch_logits<float, 64>(G, reg_ok, grid, shmem, s, (const float*)q, q_stride, (const float*)k, k_stride, cu, Hq, Hkv, n_last, scale, T, ncm, logits, partials);
  }
  return check_launch("score_logits");
}

fastav_status_t launch_score_finalize(const float* logits, const float* ml, const float* partials, const int32_t* cu,
                                      int batch, int64_t T, int max_seqlen, int Hq, int n_last, float* scores,
                                      hipStream_t s) {
  if (batch == 0 || max_seqlen == 0) return FASTAV_OK;
  ProfScope prof(FASTAV_PROF_SCORE, 4.0 * n_last * Hq * T + 4.0 * T, s);
  dim3 grid((unsigned)ceil_div(max_seqlen, 256), (unsigned)batch);
  const size_t shmem = (size_t)n_last * Hq * 2 * sizeof(float);
  hipLaunchKernelGGL(k_score_finalize, grid, dim3(256), shmem, s, logits, ml, partials, chunk_slots(T, batch), cu, Hq,
                     n_last, T, scores);
  return check_launch("score_finalize");
}

}  // namespace fastav
