// One decode step on the per-layer K/V caches a pruned prefill leaves behind (Section 3.1: the paper's
// latency is the time to generate a single token, its memory saving the compacted caches).
//
// A decode step for a handful of samples is bound by streaming the weights (7B: 13 GB per step) and, far
// behind, the caches.  Two kernel families:
//
//   k_skinny_linear  Y[b, n] = sum_k X[b, k] W[n, k] for b < 16.  A workgroup owns 16 output features; its
//                    four or eight waves walk K interleaved in steps of 32 and feed v_mfma_f32_16x16x32_bf16
//                    with the weights as the A operand straight from global memory in operand layout (lane =
//                    feature row x 16-byte k-chunk: a wave instruction reads 16 rows x 64 contiguous bytes,
//                    the waves together 256 or 512 contiguous bytes per row) and the padded batch as the B
//                    operand, 8-16 loads in flight per lane.  The matrix cores run on 16 - B rows of padding,
//                    which is free next to the HBM stream.  The partial tiles are summed through LDS in wave
//                    order, then the epilogue (store, fp32 residual add, or SiLU(gate) * up with two weight
//                    streams) runs once.  Plain (cached) loads measured faster than non-temporal ones.
//
//   k_decode_attn    single-query grouped-query attention over [cache prefix | generated so far | the new
//                    token itself] for one (sample, KV head, key split): K and V chunks of 64 keys are staged
//                    in LDS with coalesced 16-byte loads; one wave per query head of the group computes its 64
//                    logits (lane = key), updates the running (max, sum) with wave reductions and accumulates
//                    P V with lane = two output dims.  k_decode_merge combines the splits' (max, sum, o).
#include "common.hpp"

namespace fastav {

typedef float f32x4v __attribute__((ext_vector_type(4)));

// Workgroup barrier that orders LDS traffic only: global loads already issued stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---------------------------------------------------------------------------------------- skinny linear
struct SkinnyArgs {
  const bf16_t* x;            // [B, K] bf16
  const bf16_t* w[3];         // up to three [rows, K] matrices stacked along the output dimension (Q | K | V)
  int seg_end[3];             // exclusive end row of each segment
  const bf16_t* w2;           // "up" matrix (SwiGLU only), same shape as w[0]
  void* y;                    // store / SwiGLU: bf16 [B, ldy]; residual: fp32 [B, ldy]
  int64_t ldy;
  int B, N, K;
  // NORM kernels: the input is the fp32 residual stream, RMS-normalised by every workgroup for itself into
  // LDS, X = bf16(xres * r * g), which saves the separate one-row norm launches of a decode step
  const float* xres;          // [B, K] fp32
  const bf16_t* g;            // [K] gain
  float eps;
};

template <int EPI, int NW, bool NORM>
__global__ __launch_bounds__(64 * NW) void k_skinny_linear(SkinnyArgs a) {
  __shared__ f32x4v red[2][NW][64];
  __shared__ float rs[16];                                      // NORM: 1 / rms of every batch row
  extern __shared__ __attribute__((aligned(16))) bf16_t xs[];   // NORM: [B][K] normalised input
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n0 = blockIdx.x * 16;
  // segment of this row block (segments are multiples of 16 rows)
  const bf16_t* wbase = a.w[0];
  int seg0 = 0;
  if (EPI != FASTAV_EPI_SWIGLU) {
    if (n0 >= a.seg_end[0]) { wbase = a.w[1]; seg0 = a.seg_end[0]; }
    if (n0 >= a.seg_end[1]) { wbase = a.w[2]; seg0 = a.seg_end[1]; }
  }
  const int r16 = lane & 15, kc = (lane >> 4) * 8;            // operand row and k offset inside a 32-k step
  const int64_t wrow = (int64_t)(n0 - seg0 + r16) * a.K;
  const bf16x8_t* wp = (const bf16x8_t*)(wbase + wrow + kc);
  const bf16x8_t* w2p = (EPI == FASTAV_EPI_SWIGLU) ? (const bf16x8_t*)(a.w2 + wrow + kc) : nullptr;
  const int xb = r16 < a.B ? r16 : a.B - 1;                   // padded batch rows re-read the last real one
  const bf16x8_t* xp = NORM ? (const bf16x8_t*)(xs + xb * a.K + kc) : (const bf16x8_t*)(a.x + (int64_t)xb * a.K + kc);
  f32x4v acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};
  const int steps = a.K / 32;                                  // K % (32 NW) == 0: every wave gets steps / NW
  constexpr int U = (EPI == FASTAV_EPI_SWIGLU) ? 8 : 16;       // 16-byte loads in flight per lane and weight stream
  int s = wave;
  bf16x8_t wf[U], w2f[U];
  // NORM: the first batch of weight loads is issued before the norm prologue and stays in flight across its
  // barriers (they wait on LDS traffic only), so the prologue costs no bandwidth time
  bool preloaded = false;
  if (NORM && s + NW * (U - 1) < steps) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      wf[u] = wp[(s + NW * u) * 4];
      if (EPI == FASTAV_EPI_SWIGLU) w2f[u] = w2p[(s + NW * u) * 4];
    }
    preloaded = true;
  }
  if (NORM) {
    // wave w reduces the rows w, w + NW, ...; then all threads write the normalised rows, rounded the way
    // k_rmsnorm rounds them
    for (int b = wave; b < a.B; b += NW) {
      const f32x4v* xr = (const f32x4v*)(a.xres + (int64_t)b * a.K);
      float ss = 0.f;
      for (int i = lane; i < a.K / 4; i += 64) {
        const f32x4v v = xr[i];
        ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
      }
      ss = wave_sum(ss);
      if (lane == 0) rs[b] = 1.0f / sqrtf(ss / (float)a.K + a.eps);
    }
    lds_barrier();
    const int per_row = a.K / 4;
    for (int i = tid; i < a.B * per_row; i += 64 * NW) {
      const int b = i / per_row, c = i % per_row;
      const f32x4v v = ((const f32x4v*)(a.xres + (int64_t)b * a.K))[c];
      const bf16x4_t gv = ((const bf16x4_t*)a.g)[c];
      const float r = rs[b];
      bf16x4_t o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(v[e] * r * (float)gv[e]);
      ((bf16x4_t*)(xs + b * a.K))[c] = o;
    }
    lds_barrier();
  }

  for (; s + NW * (U - 1) < steps; s += NW * U) {
    bf16x8_t xf[U];
    if (!(NORM && preloaded)) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        wf[u] = wp[(s + NW * u) * 4];
        if (EPI == FASTAV_EPI_SWIGLU) w2f[u] = w2p[(s + NW * u) * 4];
      }
    }
    preloaded = false;
#pragma unroll
    for (int u = 0; u < U; ++u) xf[u] = xp[(s + NW * u) * 4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[u], xf[u], acc, 0, 0, 0);
      if (EPI == FASTAV_EPI_SWIGLU) acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w2f[u], xf[u], acc2, 0, 0, 0);
    }
  }
  for (; s < steps; s += NW) {
    const bf16x8_t wf = wp[s * 4], xf = xp[s * 4];
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf, acc, 0, 0, 0);
    if (EPI == FASTAV_EPI_SWIGLU) acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w2p[s * 4], xf, acc2, 0, 0, 0);
  }
  red[0][wave][lane] = acc;
  if (EPI == FASTAV_EPI_SWIGLU) red[1][wave][lane] = acc2;
  __syncthreads();
  if (wave != 0) return;
  // accumulator element r of lane l: feature n0 + (l / 16) * 4 + r, batch row l % 16; partials in wave order
  acc = red[0][0][lane];
#pragma unroll
  for (int w = 1; w < NW; ++w) acc = acc + red[0][w][lane];
  if (EPI == FASTAV_EPI_SWIGLU) {
    acc2 = red[1][0][lane];
#pragma unroll
    for (int w = 1; w < NW; ++w) acc2 = acc2 + red[1][w][lane];
  }
  const int b = lane & 15, n = n0 + (lane >> 4) * 4;
  if (b >= a.B) return;
  if (EPI == FASTAV_EPI_RESADD) {
    f32x4v* yp = (f32x4v*)((float*)a.y + (int64_t)b * a.ldy + n);
    *yp = *yp + acc;
  } else {
    bf16x4_t o;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = (EPI == FASTAV_EPI_SWIGLU) ? acc[r] / (1.0f + __expf(-acc[r])) * acc2[r] : acc[r];
      o[r] = (bf16_t)v;
    }
    *(bf16x4_t*)((bf16_t*)a.y + (int64_t)b * a.ldy + n) = o;
  }
}

bool skinny_linear_supported(int64_t m, int n, int k, int dtype, int64_t ldy) {
  return dtype == FASTAV_BF16 && m >= 1 && m <= 16 && n % 16 == 0 && k % 128 == 0 && ldy % 4 == 0;
}

// norm_x != nullptr: the input is rmsnorm(norm_x [B,k] fp32; gain norm_g, norm_eps) and x is ignored (needs
// B * k <= 32768 so that the normalised rows fit 64 KB of LDS; not with the residual epilogue)
bool skinny_norm_supported(int B, int k) { return (int64_t)B * k <= 32768; }

fastav_status_t launch_skinny_linear(const void* x, const void* const* w_seg, const int* seg_rows, int n_seg,
                                     const void* w2, void* y, int64_t ldy, int B, int n, int k, int epilogue,
                                     hipStream_t s, const float* norm_x, const void* norm_g, float norm_eps) {
  if (B == 0 || n == 0) return FASTAV_OK;
  if (!skinny_linear_supported(B, n, k, FASTAV_BF16, ldy)) return fail(FASTAV_EUNSUPPORTED, "skinny linear: unsupported shape");
  if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)norm_x | (uintptr_t)norm_g) % 16)
    return fail(FASTAV_EINVAL, "skinny linear: x, y and the norm inputs must be 16-byte aligned");
  if (norm_x && (!norm_g || epilogue == FASTAV_EPI_RESADD || !skinny_norm_supported(B, k)))
    return fail(FASTAV_EINVAL, "skinny linear: bad fused-norm arguments");
  SkinnyArgs a;
  a.xres = norm_x; a.g = (const bf16_t*)norm_g; a.eps = norm_eps;
  a.x = (const bf16_t*)x; a.w2 = (const bf16_t*)w2; a.y = y; a.ldy = ldy; a.B = B; a.N = n; a.K = k;
  int end = 0;
  for (int i = 0; i < 3; ++i) {
    if (i < n_seg) {
      if (seg_rows[i] % 16 || ((uintptr_t)w_seg[i] % 16)) return fail(FASTAV_EINVAL, "skinny linear: segments must be 16-row, 16-byte aligned");
      end += seg_rows[i];
      a.w[i] = (const bf16_t*)w_seg[i];
    } else {
      a.w[i] = a.w[0];
    }
    a.seg_end[i] = i < n_seg ? end : 0x7FFFFFFF;
  }
  if (end != n) return fail(FASTAV_EINVAL, "skinny linear: segments do not add up to n");
  const int kind = epilogue == FASTAV_EPI_SWIGLU ? FASTAV_PROF_LINEAR_SWIGLU
                   : (epilogue == FASTAV_EPI_RESADD ? FASTAV_PROF_LINEAR_RESADD : FASTAV_PROF_LINEAR_STORE);
  // the work figure of a decode GEMV is its weight bytes (HBM-bound), not flops
  ProfScope prof(kind, (double)n * k * 2.0 * (epilogue == FASTAV_EPI_SWIGLU ? 2.0 : 1.0), s);
  // few row blocks (narrow outputs): eight waves split K, which doubles the loads in flight per CU
  const bool wide = (n / 16 < 3 * 256) && (k % 256 == 0);
  const dim3 grid((unsigned)(n / 16));
  if (epilogue == FASTAV_EPI_SWIGLU && (!w2 || ((uintptr_t)w2 % 16)))
    return fail(FASTAV_EINVAL, "skinny linear: SwiGLU needs a 16-byte aligned up matrix");
  const size_t shmem = norm_x ? (size_t)B * k * 2 : 0;
#define FASTAV_SKINNY(EPI, NORM)                                                                          \
  do {                                                                                                    \
    if (wide) hipLaunchKernelGGL((k_skinny_linear<EPI, 8, NORM>), grid, dim3(512), shmem, s, a);          \
    else hipLaunchKernelGGL((k_skinny_linear<EPI, 4, NORM>), grid, dim3(256), shmem, s, a);               \
  } while (0)
  if (epilogue == FASTAV_EPI_SWIGLU) { if (norm_x) FASTAV_SKINNY(FASTAV_EPI_SWIGLU, true); else FASTAV_SKINNY(FASTAV_EPI_SWIGLU, false); }
  else if (epilogue == FASTAV_EPI_RESADD) FASTAV_SKINNY(FASTAV_EPI_RESADD, false);
  else { if (norm_x) FASTAV_SKINNY(FASTAV_EPI_STORE, true); else FASTAV_SKINNY(FASTAV_EPI_STORE, false); }
#undef FASTAV_SKINNY
  return check_launch("skinny_linear");
}

// ---------------------------------------------------------------------------------------- decode attention
struct DecodeAttnArgs {
  const bf16_t* q;            // [B, q_stride]: the new token's rotated queries
  const bf16_t* k_self;       // [B, q_stride]: its own rotated key ...
  const bf16_t* v_self;       // ... and value (all three live in the step's QKV row)
  int64_t q_stride;
  const bf16_t* k_prefix;     // [T_l, kd] packed per sample (cu_prefix), the prefill's cache of this layer
  const bf16_t* v_prefix;
  const int32_t* cu_prefix;   // [B + 1]
  const bf16_t* k_gen;        // [B, gen_cap, kd] tokens generated before this step (gen_len of them), or null
  const bf16_t* v_gen;
  int gen_len, gen_cap;
  int Hq, Hkv, splits, chunk; // chunk = keys per split (multiple of 64)
  float scale;
  float* part;                // [B, Hq, splits, DH + 2] fp32: o (unnormalised), max, sum
};

template <int DH>
__global__ __launch_bounds__(256) void k_decode_attn(DecodeAttnArgs a) {
  constexpr int CK = 64;                              // keys per staged chunk
  constexpr int KROW = DH + 8;                        // padded K row (elements): 16-byte reads of 16 rows spread over the banks
  __shared__ __attribute__((aligned(16))) bf16_t ks[CK * KROW];
  __shared__ __attribute__((aligned(16))) bf16_t vs[CK * DH];
  __shared__ float qs[8][DH];
  __shared__ float ps[8][CK];
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int G = a.Hq / a.Hkv;                         // <= 8 (checked by the launcher)
  const int kd = a.Hkv * DH;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int p0 = a.cu_prefix[b], n_pre = a.cu_prefix[b + 1] - p0;
  const int n_tot = n_pre + a.gen_len + 1;
  const int j_begin = split * a.chunk;
  const int j_end = (j_begin + a.chunk < n_tot) ? j_begin + a.chunk : n_tot;

  for (int i = tid; i < G * DH; i += 256) qs[i / DH][i % DH] = (float)a.q[(int64_t)b * a.q_stride + (g * G) * DH + i];

  // row j of the unified key list: prefix, then generated, then the token itself
  auto krow = [&](int j) -> const bf16_t* {
    if (j < n_pre) return a.k_prefix + (int64_t)(p0 + j) * kd + g * DH;
    if (j < n_pre + a.gen_len) return a.k_gen + ((int64_t)b * a.gen_cap + (j - n_pre)) * kd + g * DH;
    return a.k_self + (int64_t)b * a.q_stride + g * DH;
  };
  auto vrow = [&](int j) -> const bf16_t* {
    if (j < n_pre) return a.v_prefix + (int64_t)(p0 + j) * kd + g * DH;
    if (j < n_pre + a.gen_len) return a.v_gen + ((int64_t)b * a.gen_cap + (j - n_pre)) * kd + g * DH;
    return a.v_self + (int64_t)b * a.q_stride + g * DH;
  };

  constexpr int NP = 2;                               // head passes: waves 0..3 serve heads 0..3, then 4..7
  constexpr int DPL = DH / 64;                        // output dims per lane
  float m_run[NP], l_run[NP], o[NP][DPL];
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    m_run[p] = -INFINITY; l_run[p] = 0.f;
#pragma unroll
    for (int d = 0; d < DPL; ++d) o[p][d] = 0.f;
  }

  for (int j0 = j_begin; j0 < j_end; j0 += CK) {
    __syncthreads();                                  // previous chunk fully consumed (and qs written)
    constexpr int VPR = DH / 8;                       // 16-byte vectors per row
    for (int i = tid; i < CK * VPR; i += 256) {
      const int r = i / VPR, c = i % VPR;
      const int j = (j0 + r < j_end) ? j0 + r : j_end - 1;       // tail rows repeat the last key (masked below)
      *(bf16x8_t*)(ks + r * KROW + c * 8) = *(const bf16x8_t*)(krow(j) + c * 8);
      *(bf16x8_t*)(vs + r * DH + c * 8) = *(const bf16x8_t*)(vrow(j) + c * 8);
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int hs = p * 4 + wave;                    // head inside the group (wave-uniform)
      if (hs < G) {
        // logits: lane = key
        float z = 0.f;
        const bf16_t* kr = ks + lane * KROW;
#pragma unroll
        for (int c = 0; c < VPR; ++c) {
          const bf16x8_t kv = *(const bf16x8_t*)(kr + c * 8);
#pragma unroll
          for (int e = 0; e < 8; ++e) z = fmaf(qs[hs][c * 8 + e], (float)kv[e], z);
        }
        z = (j0 + lane < j_end) ? z * a.scale : -INFINITY;
        const float m_new = fmaxf(m_run[p], wave_max(z));         // finite: every chunk holds at least one key
        const float alpha = __expf(m_run[p] - m_new);
        const float pr = __expf(z - m_new);
        l_run[p] = l_run[p] * alpha + wave_sum(pr);
        m_run[p] = m_new;
        ps[hs][lane] = pr;
        // P V: lane = DPL consecutive output dims; a wave's own writes to ps are visible to it after the
        // LDS counter wait the compiler places before the reads
        __builtin_amdgcn_wave_barrier();
        float acc[DPL];
#pragma unroll
        for (int d = 0; d < DPL; ++d) acc[d] = 0.f;
        for (int jj = 0; jj < CK; ++jj) {
          const float pj = ps[hs][jj];
#pragma unroll
          for (int d = 0; d < DPL; ++d) acc[d] = fmaf(pj, (float)vs[jj * DH + lane * DPL + d], acc[d]);
        }
#pragma unroll
        for (int d = 0; d < DPL; ++d) o[p][d] = o[p][d] * alpha + acc[d];
      }
    }
  }
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const int hs = p * 4 + wave;
    if (hs < G) {
      float* out = a.part + (((int64_t)b * a.Hq + g * G + hs) * a.splits + split) * (DH + 2);
#pragma unroll
      for (int d = 0; d < DPL; ++d) out[lane * DPL + d] = o[p][d];
      if (lane == 0) { out[DH] = m_run[p]; out[DH + 1] = l_run[p]; }
    }
  }
}

// One wave per (sample, head).  Lane s first holds split s's (max, sum): the global max and every split's
// weight come from two wave reductions; then the lanes turn to the output dims and add the splits' partial
// outputs in split order (independent, coalesced loads).  splits <= 64.
template <int DH>
__global__ __launch_bounds__(64) void k_decode_merge(const float* __restrict__ part, int splits, int Hq,
                                                     bf16_t* __restrict__ out, int64_t out_stride) {
  constexpr int DPL = DH / 64;
  const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  const float* p = part + ((int64_t)b * Hq + h) * splits * (DH + 2);
  const float ms = lane < splits ? p[lane * (DH + 2) + DH] : -INFINITY;      // -inf: a split past this sample's keys
  const float ls = lane < splits ? p[lane * (DH + 2) + DH + 1] : 0.f;
  const float m = wave_max(ms);
  const float wgt = (ms == -INFINITY) ? 0.f : __expf(ms - m);
  const float inv = 1.0f / wave_sum(wgt * ls);
  float o[DPL];
#pragma unroll
  for (int d = 0; d < DPL; ++d) o[d] = 0.f;
  for (int s = 0; s < splits; ++s) {
    const float w = __shfl(wgt, s, kWave);
#pragma unroll
    for (int d = 0; d < DPL; ++d) o[d] = fmaf(w, p[s * (DH + 2) + lane * DPL + d], o[d]);
  }
#pragma unroll
  for (int d = 0; d < DPL; ++d) out[(int64_t)b * out_stride + h * DH + lane * DPL + d] = (bf16_t)(o[d] * inv);
}

size_t decode_attn_workspace_bytes(int batch, int Hq, int dh, int max_splits) {
  return align_up((size_t)batch * Hq * max_splits * (dh + 2) * sizeof(float), 256);
}

int decode_attn_splits(int batch, int Hkv, int max_keys) {
  int chunks = (max_keys + 63) / 64;
  int want = (1024 + batch * Hkv - 1) / (batch * Hkv);          // about four workgroups per CU
  int s = want < chunks ? want : chunks;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  return s;
}

fastav_status_t launch_decode_attention(const void* q, const void* k_self, const void* v_self, int64_t q_stride,
                                        const void* k_prefix, const void* v_prefix, const int32_t* cu_prefix,
                                        int max_prefix, const void* k_gen, const void* v_gen, int gen_len,
                                        int gen_cap, int batch, int Hq, int Hkv, int dh, float* part,
                                        size_t part_bytes, void* out, int64_t out_stride, double bytes_hint,
                                        hipStream_t s) {
  if (batch == 0) return FASTAV_OK;
  if (dh != 64 && dh != 128) return fail(FASTAV_EUNSUPPORTED, "decode attention: head_dim must be 64 or 128");
  if (Hq % Hkv || Hq / Hkv > 8) return fail(FASTAV_EUNSUPPORTED, "decode attention: at most 8 query heads per KV head");
  if (gen_len > 0 && (!k_gen || !v_gen)) return fail(FASTAV_EINVAL, "decode attention: gen_len > 0 needs the generated-token caches");
  if (q_stride % 8 || ((uintptr_t)q | (uintptr_t)k_self | (uintptr_t)v_self | (uintptr_t)k_prefix | (uintptr_t)v_prefix |
                        (uintptr_t)k_gen | (uintptr_t)v_gen) % 16)
    return fail(FASTAV_EINVAL, "decode attention: operands must be 16-byte aligned");
  DecodeAttnArgs a;
  a.q = (const bf16_t*)q; a.k_self = (const bf16_t*)k_self; a.v_self = (const bf16_t*)v_self; a.q_stride = q_stride;
  a.k_prefix = (const bf16_t*)k_prefix; a.v_prefix = (const bf16_t*)v_prefix; a.cu_prefix = cu_prefix;
  a.k_gen = (const bf16_t*)k_gen; a.v_gen = (const bf16_t*)v_gen; a.gen_len = gen_len; a.gen_cap = gen_cap;
  a.Hq = Hq; a.Hkv = Hkv;
  const int max_keys = max_prefix + gen_len + 1;
  a.splits = decode_attn_splits(batch, Hkv, max_keys);
  a.chunk = (int)(ceil_div(ceil_div(max_keys, a.splits), 64) * 64);
  a.scale = 1.0f / sqrtf((float)dh);
  a.part = part;
  if (decode_attn_workspace_bytes(batch, Hq, dh, a.splits) > part_bytes)
    return fail(FASTAV_EINVAL, "decode attention: workspace too small");
  ProfScope prof(FASTAV_PROF_ATTENTION, bytes_hint, s);
  const dim3 grid((unsigned)a.splits, (unsigned)Hkv, (unsigned)batch);
  if (dh == 128) {
    hipLaunchKernelGGL(k_decode_attn<128>, grid, dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_decode_merge<128>, dim3((unsigned)Hq, (unsigned)batch), dim3(64), 0, s, part, a.splits, Hq, (bf16_t*)out, out_stride);
  } else {
    hipLaunchKernelGGL(k_decode_attn<64>, grid, dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_decode_merge<64>, dim3((unsigned)Hq, (unsigned)batch), dim3(64), 0, s, part, a.splits, Hq, (bf16_t*)out, out_stride);
  }
  return check_launch("decode_attention");
}

}  // namespace fastav
