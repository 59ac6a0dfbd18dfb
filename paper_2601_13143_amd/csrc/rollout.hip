// Attention rollout (Eq. 2-3 of the paper): the offline analysis that tells FastAV where to prune globally.
//
//   A^l  = mean over heads of the causal attention weights of layer l        (k_attn_rowstats + k_attn_map)
//   R^l  = (alpha A^l + (1 - alpha) I) R^{l-1}                               (one GEMM + two elementwise passes)
//
// The head-mean map is formed without ever holding a per-head n x n map: a first pass computes every query
// row's softmax (max, sum) per head by streaming K through the matrix cores (S^T = K Q^T tiles, running
// max / sum per lane, like the prefill attention but with no values), a second pass recomputes each 128 x 64
// tile of logits for every head, turns it into probabilities with those (max, sum) and accumulates the mean
// in registers, so A is written exactly once (bf16, the operand type of the GEMM that consumes it).  Both
// passes read Q and K straight from global memory in MFMA operand layout (they are served by L2: a tile of
// one head is a few KB and is reused by the neighbouring workgroups); no LDS, no barriers.
//
// The rollout is kept transposed, RT = (R^l)^T, because the library's GEMM multiplies by a row-major [out, in]
// matrix: RT_new = RT (alpha A + (1 - alpha) I)^T = alpha (RT A^T) + (1 - alpha) RT, and C[i][j] =
// sum_k RT[i][k] A[j][k] is exactly launch_linear(a = RT, w = A).  RT is carried in fp32 with a bf16 copy as
// the GEMM operand.
#include "common.hpp"

namespace fastav {

struct MapArgs {
  const bf16_t* q; const bf16_t* k;
  int64_t qs, ks;               // row strides in elements
  int n, Hq, Hkv;
  float scale_log2;             // log2(e) / sqrt(head_dim)
  float* stats;                 // [n, Hq, 2]: running max (log2 domain) and sum of exp2
  bf16_t* a_out;                // [n, n]
};

// Q operand (B of S^T = K Q^T): lane = query l32, k-chunk hf of k-step s.  K operand (A): lane = key l32.
template <int DH>
__device__ __forceinline__ void load_q_frags(const MapArgs& a, int qrow, int h, int hf, bf16x8_t (&qf)[DH / 16]) {
  const bf16_t* qp = a.q + (int64_t)qrow * a.qs + h * DH + hf * 8;
#pragma unroll
  for (int s = 0; s < DH / 16; ++s) qf[s] = *(const bf16x8_t*)(qp + 16 * s);
}
template <int DH>
__device__ __forceinline__ void load_k_frags(const MapArgs& a, int krow, int g, int hf, bf16x8_t (&kf)[DH / 16]) {
  const bf16_t* kp = a.k + (int64_t)krow * a.ks + g * DH + hf * 8;
#pragma unroll
  for (int s = 0; s < DH / 16; ++s) kf[s] = *(const bf16x8_t*)(kp + 16 * s);
}

// grid (query tiles of 128, Hq); wave w owns 32 query rows; every row's (max, sum) over its visible keys.
template <int DH>
__global__ __launch_bounds__(256) void k_attn_rowstats(MapArgs a) {
  constexpr int NS = DH / 16;
  const int h = blockIdx.y, g = h / (a.Hq / a.Hkv);
  const int lane = threadIdx.x & 63, l32 = lane & 31, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int qw0 = blockIdx.x * 128 + 32 * wave;
  if (qw0 >= a.n) return;
  const int qi = qw0 + l32;
  bf16x8_t qf[NS];
  load_q_frags<DH>(a, qi < a.n ? qi : a.n - 1, h, hf, qf);
  const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;
  const int n_blocks = (((qw0 + 32 < a.n) ? qw0 + 32 : a.n) + 31) / 32;     // key blocks this wave can see
  for (int kb = 0; kb < n_blocks; ++kb) {
    const int key = kb * 32 + l32;
    bf16x8_t kf[NS];
    load_k_frags<DH>(a, key < a.n ? key : a.n - 1, g, hf, kf);
    f32x16_t s = zero16;
#pragma unroll
    for (int st = 0; st < NS; ++st) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st], qf[st], s, 0, 0, 0);
    // s[r] = (key kb*32 + (r/4)*8 + hf*4 + r%4, query qi)
    float x[16], mx = m;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kk = kb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
      x[r] = (kk <= qi && kk < a.n) ? s[r] * a.scale_log2 : -INFINITY;
      mx = fmaxf(mx, x[r]);
    }
    const float ms = (mx == -INFINITY) ? 0.f : mx;
    float add = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) add += __builtin_amdgcn_exp2f(x[r] - ms);
    l = l * __builtin_amdgcn_exp2f(m - ms) + add;
    m = mx;
  }
  // the lane 32 away holds the other half of this query's keys
  const float m2 = __shfl_xor(m, 32, kWave), l2 = __shfl_xor(l, 32, kWave);
  const float mt = fmaxf(m, m2);
  const float lt = l * __builtin_amdgcn_exp2f(m - mt) + l2 * __builtin_amdgcn_exp2f(m2 - mt);   // key 0 is always visible: mt is finite
  if (hf == 0 && qi < a.n) {
    a.stats[((int64_t)qi * a.Hq + h) * 2] = mt;
    a.stats[((int64_t)qi * a.Hq + h) * 2 + 1] = lt;
  }
}

// grid (query tiles of 128, key tiles of 64); A tile = mean over heads of exp2(logit - max) / sum.
template <int DH>
__global__ __launch_bounds__(256) void k_attn_map(MapArgs a) {
  constexpr int NS = DH / 16;
  const int lane = threadIdx.x & 63, l32 = lane & 31, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int qw0 = blockIdx.x * 128 + 32 * wave;
  const int j0 = blockIdx.y * 64;
  if (qw0 >= a.n) return;
  const int qi = qw0 + l32;
  const int G = a.Hq / a.Hkv;
  float acc[2][16];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[kb][r] = 0.f;
  if (j0 <= qw0 + 31) {                                 // else the tile lies above the diagonal: zeros
    const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int qr = qi < a.n ? qi : a.n - 1;
    for (int g = 0; g < a.Hkv; ++g) {
      bf16x8_t kf[2][NS];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const int key = j0 + kb * 32 + l32;
        load_k_frags<DH>(a, key < a.n ? key : a.n - 1, g, hf, kf[kb]);
      }
      for (int hq = 0; hq < G; ++hq) {
        const int h = g * G + hq;
        bf16x8_t qf[NS];
        load_q_frags<DH>(a, qr, h, hf, qf);
        const float m = a.stats[((int64_t)qr * a.Hq + h) * 2];
        const float inv_l = 1.0f / a.stats[((int64_t)qr * a.Hq + h) * 2 + 1];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          f32x16_t s = zero16;
#pragma unroll
          for (int st = 0; st < NS; ++st) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][st], qf[st], s, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[kb][r] += __builtin_amdgcn_exp2f(fmaf(s[r], a.scale_log2, -m)) * inv_l;
        }
      }
    }
  }
  if (qi >= a.n) return;
  const float inv_h = 1.0f / (float)a.Hq;
  bf16_t* orow = a.a_out + (int64_t)qi * a.n;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int key0 = j0 + kb * 32 + r4 * 8 + hf * 4;
      bf16x4_t w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (bf16_t)((key0 + e <= qi) ? acc[kb][4 * r4 + e] * inv_h : 0.f);
      if (key0 + 3 < a.n) *(bf16x4_t*)(orow + key0) = w;
      else
        for (int e = 0; e < 4; ++e) if (key0 + e < a.n) orow[key0 + e] = w[e];
    }
}

size_t attention_map_stats_bytes(int n, int Hq) { return align_up((size_t)n * Hq * 2 * sizeof(float), 256); }

fastav_status_t launch_attention_map(const void* q, int64_t q_stride, const void* k, int64_t k_stride, int n, int Hq,
                                     int Hkv, int dh, float* stats, void* a_out, hipStream_t s) {
  if (n == 0) return FASTAV_OK;
  if (dh != 64 && dh != 128) return fail(FASTAV_EUNSUPPORTED, "attention map: head_dim must be 64 or 128");
  if (q_stride % 8 || k_stride % 8 || (((uintptr_t)q | (uintptr_t)k) % 16) || n % 4 || ((uintptr_t)a_out % 8))
    return fail(FASTAV_EINVAL, "attention map: q, k must be 16-byte aligned with strides of 8 elements, n a multiple of 4");
  MapArgs a;
  a.q = (const bf16_t*)q; a.k = (const bf16_t*)k; a.qs = q_stride; a.ks = k_stride; a.n = n; a.Hq = Hq; a.Hkv = Hkv;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)dh);
  a.stats = stats; a.a_out = (bf16_t*)a_out;
  // 3 passes of the causal Q K^T products: one for the statistics, one for the map (plus masked halves)
  ProfScope prof(FASTAV_PROF_ATTENTION, 2.0 * 2.0 * Hq * dh * (double)n * ((double)n + 1.0) * 0.5, s);
  const dim3 g1((unsigned)ceil_div(n, 128), (unsigned)Hq), g2((unsigned)ceil_div(n, 128), (unsigned)ceil_div(n, 64));
  if (dh == 128) {
    hipLaunchKernelGGL(k_attn_rowstats<128>, g1, dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_attn_map<128>, g2, dim3(256), 0, s, a);
  } else {
    hipLaunchKernelGGL(k_attn_rowstats<64>, g1, dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_attn_map<64>, g2, dim3(256), 0, s, a);
  }
  return check_launch("attention_map");
}

// ---------------------------------------------------------------------------------------- rollout step
__global__ void k_rollout_init(float* __restrict__ rt, bf16_t* __restrict__ rt16, int n) {
  const int64_t total = (int64_t)n * n;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const float v = (i / n == i % n) ? 1.f : 0.f;
    rt[i] = v; rt16[i] = (bf16_t)v;
  }
}
// c = beta * rt   (the residual term, pre-divided by alpha so the GEMM can accumulate onto it)
__global__ void k_rollout_prefill(float* __restrict__ c, const float* __restrict__ rt, float beta, int64_t total4) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total4; i += (int64_t)gridDim.x * blockDim.x) {
    const f32x4_t v = ((const f32x4_t*)rt)[i];
    ((f32x4_t*)c)[i] = v * beta;
  }
}
// rt = alpha * c, and its bf16 copy
__global__ void k_rollout_finish(const float* __restrict__ c, float alpha, float* __restrict__ rt,
                                 bf16_t* __restrict__ rt16, int64_t total4) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total4; i += (int64_t)gridDim.x * blockDim.x) {
    const f32x4_t v = ((const f32x4_t*)c)[i] * alpha;
    ((f32x4_t*)rt)[i] = v;
    bf16x4_t w;
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (bf16_t)v[e];
    ((bf16x4_t*)rt16)[i] = w;
  }
}

__global__ void k_iota(int32_t* __restrict__ p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i;
}
fastav_status_t launch_iota(int32_t* p, int n, hipStream_t s) {
  if (n == 0) return FASTAV_OK;
  hipLaunchKernelGGL(k_iota, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, p, n);
  return check_launch("iota");
}

fastav_status_t launch_rollout_init(float* rt, void* rt16, int n, hipStream_t s) {
  if (n == 0) return FASTAV_OK;
  hipLaunchKernelGGL(k_rollout_init, dim3(2048), dim3(256), 0, s, rt, (bf16_t*)rt16, n);
  return check_launch("rollout_init");
}

// RT <- alpha (RT A^T) + (1 - alpha) RT.  c: fp32 [n, n] scratch; linear_ws: optional split-K workspace.
fastav_status_t launch_rollout_step(float* rt, void* rt16, const void* a16, float* c, int n, float alpha,
                                    void* linear_ws, size_t linear_ws_bytes, hipStream_t s) {
  if (n == 0 || alpha == 0.f) return FASTAV_OK;       // alpha = 0: every factor is the identity
  if (n % 4) return fail(FASTAV_EINVAL, "rollout: n must be a multiple of 4");
  const int64_t total4 = (int64_t)n * n / 4;
  hipLaunchKernelGGL(k_rollout_prefill, dim3(2048), dim3(256), 0, s, c, (const float*)rt, (1.0f - alpha) / alpha, total4);
  fastav_status_t st = launch_linear(rt16, a16, nullptr, c, n, n, n, FASTAV_EPI_RESADD, FASTAV_BF16, linear_ws, linear_ws_bytes, s);
  if (st != FASTAV_OK) return st;
  hipLaunchKernelGGL(k_rollout_finish, dim3(2048), dim3(256), 0, s, (const float*)c, alpha, rt, (bf16_t*)rt16, total4);
  return check_launch("rollout_step");
}

// ---- rollout threshold -> cut-off position (Section 2.2, Global pruning) -------------------------------------
// influence[j] = (1/n) sum_i R[i][j]: the mean of row j of the transposed product.  One wave per row.
__global__ __launch_bounds__(256) void k_rollout_influence(const float* __restrict__ rt, int n, float* __restrict__ influence) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n) return;
  const f32x4_t* p = (const f32x4_t*)(rt + (int64_t)row * n);
  float s0 = 0.f, s1 = 0.f;
  int i = lane;
  for (; i + 64 < n / 4; i += 128) {
    const f32x4_t a = p[i], b = p[i + 64];
    s0 += (a[0] + a[1]) + (a[2] + a[3]);
    s1 += (b[0] + b[1]) + (b[2] + b[3]);
  }
  if (i < n / 4) { const f32x4_t a = p[i]; s0 += (a[0] + a[1]) + (a[2] + a[3]); }
  float t = s0 + s1;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o, kWave);
  if (lane == 0) influence[row] = t / (float)n;
}
// cutoff = 1 + the last unprotected position whose influence reaches `threshold` uniform shares (influence * n >=
// threshold, in fp32), 0 if there is none.  One workgroup.
__global__ __launch_bounds__(1024) void k_rollout_cutoff(const float* __restrict__ influence, const uint8_t* __restrict__ prot,
                                                         int n, float threshold, int32_t* __restrict__ cutoff) {
  __shared__ int wave_best[16];
  int best = 0;
  for (int j = threadIdx.x; j < n; j += 1024)
    if (!prot[j] && influence[j] * (float)n >= threshold) best = j + 1;     // j ascends: the last hit stays
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { const int t = __shfl_xor(best, o, kWave); best = t > best ? t : best; }
  if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = best;
  __syncthreads();
  if (threadIdx.x == 0) {
    int b = 0;
    for (int w = 0; w < 16; ++w) b = wave_best[w] > b ? wave_best[w] : b;
    cutoff[0] = b;
  }
}
fastav_status_t launch_rollout_cutoff(const float* rt, int n, const uint8_t* prot, float threshold, float* influence,
                                      int32_t* cutoff, hipStream_t s) {
  if (n % 4) return fail(FASTAV_EINVAL, "rollout: n must be a multiple of 4");
  if (n > 0) hipLaunchKernelGGL(k_rollout_influence, dim3((unsigned)ceil_div(n, 4)), dim3(256), 0, s, rt, n, influence);
  hipLaunchKernelGGL(k_rollout_cutoff, dim3(1), dim3(1024), 0, s, (const float*)influence, prot, n, threshold, cutoff);
  return check_launch("rollout_cutoff");
}

}  // namespace fastav
