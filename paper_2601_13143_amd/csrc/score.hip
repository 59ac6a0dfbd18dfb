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
constexpr int kFinalizeKeys = 1024; // keys per workgroup of the finalize kernel (a multiple of 256)
constexpr int kFinalizeBatch = 8;   // 16-byte logits loads in flight per lane

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

// bf16 variant on the matrix cores.  The contraction q . k over head_dim is dense, so it goes through
// v_mfma_f32_16x16x32_bf16 with 16 keys as the M side and the query rows (heads of one KV group x last
// rows, padded to 16) as the N side; K fragments are loaded from HBM straight into the MFMA operand layout
// (lane = key, 16 bytes of head_dim each: every byte of K is fetched once, by one lane, and used once), so
// there is no LDS staging, no cross-lane reduction and no workgroup barrier.  In the result a lane owns ONE
// query row and four consecutive keys: it scales, masks, stores them and keeps a running (max, sum-exp)
// for its row.  The matrix cores run mostly on padding here (4 of 16 columns at GQA 4:1); that costs
// nothing next to the HBM stream this kernel is bound by.
// Wave w of workgroup (x, b, z) handles KV head w + W z over kScoreChunk keys of sample b, W = waves per
// workgroup (up to 8): with all KV heads of a key chunk in one workgroup the chunk is one contiguous run of
// whole K rows.
template <int DH, int NBMAX>
__global__ __launch_bounds__(512) void k_score_logits_mfma(const bf16_t* __restrict__ q, int64_t q_stride,
                                                           const bf16_t* __restrict__ k, int64_t k_stride,
                                                           const int32_t* __restrict__ cu, int Hq, int Hkv, int n_last,
                                                           float scale, int64_t T_total, int64_t n_chunk_slots,
                                                           float* __restrict__ logits, float* __restrict__ partials) {
  constexpr int NSTEP = DH / 32;             // MFMA k-steps of 32
  constexpr int KG = kScoreChunk / 16;       // key groups of 16 per chunk
  // NBMAX: query-row batches of 16 this instantiation can hold (G * n_rows <= 16 * NBMAX)
  const int b = blockIdx.y;
  const int row0 = cu[b], n = cu[b + 1] - row0;
  const int j0 = blockIdx.x * kScoreChunk;
  if (j0 >= n) return;
  const int g = threadIdx.x / 64 + (int)(blockDim.x / 64) * (int)blockIdx.z;
  if (g >= Hkv) return;                      // no barriers below, so a wave may simply leave
  const int n_rows = n_last < n ? n_last : n;
  const int G = Hq / Hkv;
  const int R = G * n_rows;                  // query rows per KV head: index m = rl * G + hq
  const int NB = (R + 15) / 16;
  const int lane = threadIdx.x & 63;
  const int l16 = lane & 15, l4 = lane >> 4;
  const bool full_chunk = j0 + kScoreChunk <= n;
  const bool vec_ok = full_chunk && ((row0 & 3) == 0) && ((T_total & 3) == 0);   // 16-byte aligned rows of 4 keys

  // B operands: lane holds query row m = rb*16 + l16, head_dim chunk l4 of every k-step.  The same lane
  // receives that query row's column of the result.
  bf16x8_t qb[NBMAX][NSTEP];
  int rr[NBMAX];                             // in-sample position of the query row, -1 for padding
  float* dst[NBMAX];                         // &logits[rl][head][row0]
  float mrun[NBMAX], lrun[NBMAX];
#pragma unroll
  for (int rb = 0; rb < NBMAX; ++rb) {
    const int mrow = rb * 16 + l16;
    const bool ok = (NBMAX == 1 || rb < NB) && mrow < R;
    const int rl = ok ? mrow / G : 0, hq = ok ? mrow % G : 0;
    rr[rb] = ok ? n - n_rows + rl : -1;
    dst[rb] = logits + ((int64_t)rl * Hq + g * G + hq) * T_total + row0;
    mrun[rb] = -INFINITY; lrun[rb] = 0.f;
    const bf16_t* qp = q + (int64_t)(row0 + n - n_rows + rl) * q_stride + (g * G + hq) * DH + l4 * 8;
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) {
      bf16x8_t v = *(const bf16x8_t*)(qp + st * 32);
      if (!ok) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (bf16_t)0.f;
      }
      qb[rb][st] = v;
    }
  }

  // A operands of the whole chunk are requested up front (KG * NSTEP 16-byte loads per lane in flight): the
  // kernel is a pure HBM stream and this is what keeps the memory system busy.  lane = key l16 of a group,
  // head_dim chunk l4.
  bf16x8_t ka_all[KG][NSTEP];
#pragma unroll
  for (int kg = 0; kg < KG; ++kg) {
    const int akey = j0 + kg * 16 + l16;
    const int kr = akey < n ? akey : n - 1;
    const bf16_t* kp = k + (int64_t)(row0 + kr) * k_stride + g * DH + l4 * 8;
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) ka_all[kg][st] = *(const bf16x8_t*)(kp + st * 32);
  }
#pragma unroll
  for (int kg = 0; kg < KG; ++kg) {
    const bf16x8_t (&ka)[NSTEP] = ka_all[kg];
    const int key0 = j0 + kg * 16 + l4 * 4;  // result rows of this lane: keys key0 .. key0+3
#pragma unroll
    for (int rb = 0; rb < NBMAX; ++rb) {
      if (NBMAX == 1 || rb < NB) {
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[st], qb[rb][st], acc, 0, 0, 0);
        float x[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = (key0 + r <= rr[rb]) ? acc[r] * scale : -INFINITY;   // visible: key <= row < n
        if (rr[rb] >= 0) {
          if (vec_ok) {
            f32x4_t xv = {x[0], x[1], x[2], x[3]};
            *(f32x4_t*)(dst[rb] + key0) = xv;
          } else if (full_chunk) {
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[rb][key0 + r] = x[r];
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) if (key0 + r < n) dst[rb][key0 + r] = x[r];
          }
        }
        const float mn = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), mrun[rb]);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        lrun[rb] = lrun[rb] * __expf(mrun[rb] - ms) + (__expf(x[0] - ms) + __expf(x[1] - ms)) + (__expf(x[2] - ms) + __expf(x[3] - ms));
        mrun[rb] = mn;
      }
    }
  }
  // merge the four lanes that hold the same query row (different keys); lanes 0..15 write the chunk partial
#pragma unroll
  for (int rb = 0; rb < NBMAX; ++rb) {
    float m1 = mrun[rb], l1 = lrun[rb];
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
      const float m2 = __shfl_xor(m1, o, kWave), l2 = __shfl_xor(l1, o, kWave);
      const float mn = fmaxf(m1, m2);
      const float ms = (mn == -INFINITY) ? 0.f : mn;
      l1 = l1 * __expf(m1 - ms) + l2 * __expf(m2 - ms);
      m1 = mn;
    }
    const int mrow = rb * 16 + l16;
    if (l4 == 0 && rr[rb] >= 0) {
      const int rl = mrow / G, hq = mrow % G;
      float* p = partials + (((int64_t)rl * Hq + g * G + hq) * n_chunk_slots + row0 / kScoreChunk + b + blockIdx.x) * 2;
      p[0] = m1; p[1] = l1;
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
  if ((int)(blockIdx.x * kFinalizeKeys) >= n + 3) return;
  const int n_rows = n_last < n ? n_last : n;
  const int P = n_rows * Hq;
  // vector path: a thread owns four consecutive positions of the packed token axis, aligned to 16 bytes there (a
  // sample may start anywhere, so the quad may hang over the sample's ends: those lanes of it are dropped).  The
  // first kFinalizeBatch planes are requested before the (max, sum) merge below, which does not depend on them.
  const bool vec = (T_total & 3) == 0;
  const int64_t q0 = (int64_t)(row0 & ~3) + (int64_t)blockIdx.x * kFinalizeKeys + threadIdx.x * 4;
  const bool mine = vec && q0 < row0 + n;
  f32x4_t L[kFinalizeBatch];
  if (mine) {
#pragma unroll
    for (int u = 0; u < kFinalizeBatch; ++u)
      if (u < P) L[u] = *(const f32x4_t*)(logits + q0 + (int64_t)u * T_total);
  }
  if (ml_in) {
    for (int idx = threadIdx.x; idx < n_rows * Hq; idx += 256) {
      const int rl = idx / Hq, h = idx % Hq;
      const float* p = ml_in + (((int64_t)b * n_last + rl) * Hq + h) * 2;
      mls[2 * idx] = p[0]; mls[2 * idx + 1] = 1.0f / p[1];
    }
  } else {
    // merge the per-chunk (max, sum-exp) partials: eight lanes per (row, head) pair, strided over the chunks,
    // 32 pairs per pass of the workgroup.  Every workgroup of a sample repeats this small merge, so it is laid
    // out for few dependent steps: eight independent 8-byte loads per lane and round, merged online, then one
    // 8-lane butterfly.
    const int nc = (n + kScoreChunk - 1) / kScoreChunk;
    const int sub = threadIdx.x & 7;
    for (int base = 0; base < n_rows * Hq; base += 32) {
      const int idx = base + (threadIdx.x >> 3);
      const bool live = idx < n_rows * Hq;
      const int rl = live ? idx / Hq : 0, h = live ? idx % Hq : 0;
      const float2* p = (const float2*)(partials + (((int64_t)rl * Hq + h) * n_chunk_slots + row0 / kScoreChunk + b) * 2);
      float m = -INFINITY, l = 0.f;
      for (int c0 = 0; c0 < nc; c0 += 64) {
        float2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int c = c0 + sub + 8 * u;
          v[u] = (live && c < nc) ? p[c] : make_float2(-INFINITY, 0.f);
        }
        float mb = m;
#pragma unroll
        for (int u = 0; u < 8; ++u) mb = fmaxf(mb, v[u].x);
        if (mb > -INFINITY) {
          l *= expf(m - mb);
#pragma unroll
          for (int u = 0; u < 8; ++u) if (v[u].x > -INFINITY) l += v[u].y * expf(v[u].x - mb);
          m = mb;
        }
      }
#pragma unroll
      for (int o = 1; o < 8; o <<= 1) {
        const float m2 = __shfl_xor(m, o, kWave), l2 = __shfl_xor(l, o, kWave);
        const float mn = fmaxf(m, m2);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        l = l * expf(m - ms) + l2 * expf(m2 - ms);
        m = mn;
      }
      if (live && sub == 0) { mls[2 * idx] = m; mls[2 * idx + 1] = 1.0f / l; }
    }
  }
  __syncthreads();
  if (vec) {
    if (!mine) return;
    const float* lp = logits + q0;                                // idx = rl*Hq + h selects the plane
    f32x4_t s = {0.f, 0.f, 0.f, 0.f};                             // the terms are added in index order
    for (int idx = 0; idx < P; idx += kFinalizeBatch) {
      if (idx > 0) {
#pragma unroll
        for (int u = 0; u < kFinalizeBatch; ++u)
          if (idx + u < P) L[u] = *(const f32x4_t*)(lp + (int64_t)(idx + u) * T_total);
      }
#pragma unroll
      for (int u = 0; u < kFinalizeBatch; ++u) {
        if (idx + u < P) {
          const float m = mls[2 * (idx + u)], il = mls[2 * (idx + u) + 1];
#pragma unroll
          for (int e = 0; e < 4; ++e) s[e] = fmaf(expf(L[u][e] - m), il, s[e]);
        }
      }
    }
    if (q0 >= row0 && q0 + 3 < row0 + n && ((uintptr_t)scores & 15) == 0) {
      *(f32x4_t*)(scores + q0) = s / (float)P;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (q0 + e >= row0 && q0 + e < row0 + n) scores[q0 + e] = s[e] / (float)P;
    }
    return;
  }
  for (int it = 0; it < kFinalizeKeys / 256; ++it) {
    const int j = blockIdx.x * kFinalizeKeys + it * 256 + threadIdx.x;
    if (j >= n) return;
    const float* lp = logits + row0 + j;
    float s = 0.f;
    for (int idx = 0; idx < P; ++idx) s = fmaf(expf(lp[(int64_t)idx * T_total] - mls[2 * idx]), mls[2 * idx + 1], s);
    scores[row0 + j] = s / (float)P;
  }
}

// Chunk slots of the whole packed batch: sample b's chunks start at slot cu[b]/chunk + b.
static int64_t chunk_slots(int64_t T, int batch) { return T / kScoreChunk + batch + 1; }

// logits [n_last][Hq][T]
size_t score_logits_bytes(int Hq, int64_t T, int n_last) { return (size_t)n_last * Hq * T * sizeof(float); }

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
  if (dtype == FASTAV_BF16 && G * n_last <= 64 && q_stride % 8 == 0 && k_stride % 8 == 0 &&
      (((uintptr_t)q | (uintptr_t)k) % 16) == 0) {
    const int wpg = Hkv < 8 ? Hkv : 8;                            // waves (KV heads) per workgroup
    // one 128-key chunk per workgroup, chunks in launch order: neighbouring workgroups stream neighbouring
    // memory (letting a workgroup walk chunks a stride apart measured 10 % slower)
    const dim3 grid_m(grid.x, grid.y, (unsigned)((Hkv + wpg - 1) / wpg));
#define FASTAV_SCORE_MFMA(DHH, NBB)                                                                                      \
  hipLaunchKernelGGL((k_score_logits_mfma<DHH, NBB>), grid_m, dim3(64 * wpg), 0, s, (const bf16_t*)q, q_stride, (const bf16_t*)k, \
                     k_stride, cu, Hq, Hkv, n_last, scale, T, ncm, logits, partials)
    const bool one = G * n_last <= 16;
    if (dh == 128) { if (one) FASTAV_SCORE_MFMA(128, 1); else FASTAV_SCORE_MFMA(128, 4); }
    else { if (one) FASTAV_SCORE_MFMA(64, 1); else FASTAV_SCORE_MFMA(64, 4); }
#undef FASTAV_SCORE_MFMA
    return check_launch("score_logits_mfma");
  }
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
  // + 3: a sample that starts off a 16-byte boundary needs up to three more positions
  dim3 grid((unsigned)ceil_div(max_seqlen + 3, kFinalizeKeys), (unsigned)batch);
  const size_t shmem = (size_t)n_last * Hq * 2 * sizeof(float);
  hipLaunchKernelGGL(k_score_finalize, grid, dim3(256), shmem, s, logits, ml, partials, chunk_slots(T, batch), cu, Hq,
                     n_last, T, scores);
  return check_launch("score_finalize");
}

}  // namespace fastav
