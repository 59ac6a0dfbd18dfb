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
//                    token itself] for one (sample, KV head, key split): logits of all heads of the group on
//                    the matrix cores with the keys read from global memory in operand layout, P V on the
//                    vector units straight from the V rows.  k_decode_merge combines the splits' (max, sum, o).
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
  // ROPE kernels (one-row GEMV, store epilogue): output features below rope_rows are heads of dh features each,
  // rotated at position pos[0] (rotate-half pairs (i, i + dh/2), angle pos * base^(-2i/dh)) before they are stored
  const int32_t* pos;
  int rope_rows, dh;
  double rope_coef;           // -log2(base) * 2 / dh
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
    constexpr int NT = 64 * NW, R1 = 4;                         // one row in registers: up to R1 quads per thread
    const int per_row = a.K / 4;
    if (a.B == 1 && per_row <= R1 * NT) {
      // a single row: every thread keeps its quads, the row is read once
      __shared__ float wsum[NW];
      f32x4v v[R1];
      bf16x4_t gv[R1];
      float ss = 0.f;
#pragma unroll
      for (int it = 0; it < R1; ++it) {
        const int i = tid + it * NT;
        if (i < per_row) {
          v[it] = ((const f32x4v*)a.xres)[i];
          gv[it] = ((const bf16x4_t*)a.g)[i];
        }
      }
#pragma unroll
      for (int it = 0; it < R1; ++it)
        if (tid + it * NT < per_row) ss += v[it][0] * v[it][0] + v[it][1] * v[it][1] + v[it][2] * v[it][2] + v[it][3] * v[it][3];
      ss = wave_sum(ss);
      if (lane == 0) wsum[wave] = ss;
      lds_barrier();
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) tot += wsum[w];              // fixed order: the same value in every thread
      const float r = 1.0f / sqrtf(tot / (float)a.K + a.eps);
#pragma unroll
      for (int it = 0; it < R1; ++it) {
        const int i = tid + it * NT;
        if (i < per_row) {
          bf16x4_t o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(v[it][e] * r * (float)gv[it][e]);
          ((bf16x4_t*)xs)[i] = o;
        }
      }
      lds_barrier();
    } else {
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
      for (int i = tid; i < a.B * per_row; i += NT) {
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

// ---------------------------------------------------------------------------------------- one-row GEMV
// Y[n] = sum_k X[k] W[n, k] for a single input row (the paper's latency case: one sample generates one token).
// With one row there is nothing for the matrix cores to reuse, so the kernel is laid out purely for the weight
// stream: a wave owns two consecutive weight rows and reads them as whole 1 KB runs (lane = 16-byte chunk), eight
// to sixteen loads in flight per lane; a workgroup's eight waves cover 16 rows = one contiguous slab.  The input
// row sits in LDS as bf16 (normalised there when NORM, exactly as k_skinny_linear does it), each 16-byte chunk of
// it is read once per pair of rows and multiplied with v_dot2_f32_bf16 into fp32 sums, which the wave reduces at
// the end.  K % 512 == 0.
__device__ __forceinline__ float dot8(bf16x8_t w, bf16x8_t x, float acc) {
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(w, w, 0, 1), __builtin_shufflevector(x, x, 0, 1), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(w, w, 2, 3), __builtin_shufflevector(x, x, 2, 3), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(w, w, 4, 5), __builtin_shufflevector(x, x, 4, 5), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(w, w, 6, 7), __builtin_shufflevector(x, x, 6, 7), acc, false);
  return acc;
}

template <int EPI, bool NORM, bool ROPE>
__global__ __launch_bounds__(512) void k_gemv_rows(SkinnyArgs a) {
  constexpr int NW = 8, NT = 64 * NW;
  constexpr int UB = 4;                                         // chunks per row and batch: 8 or 16 (SwiGLU) loads in flight per lane
  extern __shared__ __attribute__((aligned(16))) bf16_t xs[];   // [K] the input row
  __shared__ float wsum[NW];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n0 = blockIdx.x * 16;
  // this wave's two output features: neighbours, or - where the rotation is fused - the pair (i, i + dh/2) of a
  // head, so that the wave holds both halves of the rotation (a workgroup then covers 8 + 8 features of one head)
  const bool rot = ROPE && n0 < a.rope_rows;
  int n_lo = n0 + 2 * wave, dn = 1;
  if (rot) {
    const int wph = a.dh / 16;                                  // workgroups per head
    n_lo = (blockIdx.x / wph) * a.dh + (blockIdx.x % wph) * 8 + wave;
    dn = a.dh / 2;
  }
  const bf16_t* wbase = a.w[0];
  int seg0 = 0;
  if (EPI != FASTAV_EPI_SWIGLU) {                               // both features lie in one segment (whole heads)
    if (n_lo >= a.seg_end[0]) { wbase = a.w[1]; seg0 = a.seg_end[0]; }
    if (n_lo >= a.seg_end[1]) { wbase = a.w[2]; seg0 = a.seg_end[1]; }
  }
  const int cpr = a.K / 8;                                      // 16-byte chunks per row
  const int per_lane = cpr / 64;
  const int64_t row = (int64_t)(n_lo - seg0);                   // this wave's rows: row, row + dn
  const int64_t cdn = (int64_t)dn * cpr;
  const bf16x8_t* w0 = (const bf16x8_t*)(wbase + row * a.K) + lane;
  const bf16x8_t* u0 = (EPI == FASTAV_EPI_SWIGLU) ? (const bf16x8_t*)(a.w2 + row * a.K) + lane : nullptr;
  bf16x8_t f0[UB], f1[UB], g0[UB], g1[UB];
  auto load_batch = [&](int c) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      if (c + u < per_lane) {                                   // uniform
        f0[u] = w0[(c + u) * 64];
        f1[u] = w0[(c + u) * 64 + cdn];
        if (EPI == FASTAV_EPI_SWIGLU) { g0[u] = u0[(c + u) * 64]; g1[u] = u0[(c + u) * 64 + cdn]; }
      }
    }
  };
  load_batch(0);                                                // in flight across the prologue (its barriers wait on LDS only)
  float rc = 1.f, rs_ = 0.f;
  if (rot) {                                                    // angle in fp64, as the stand-alone rotation evaluates it
    const double ang = (double)a.pos[0] * exp2((double)(n_lo % a.dh) * a.rope_coef);
    double sd, cd;
    sincos(ang, &sd, &cd);
    rc = (float)cd; rs_ = (float)sd;
  }
  if (NORM) {
    // every thread keeps its quads of the row in registers: the row is read once
    constexpr int R1 = 4;                                       // K <= 4 * R1 * NT = 8192
    const int per_row = a.K / 4;
    f32x4v v[R1];
    bf16x4_t gv[R1];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < R1; ++it) {
      const int i = tid + it * NT;
      if (i < per_row) { v[it] = ((const f32x4v*)a.xres)[i]; gv[it] = ((const bf16x4_t*)a.g)[i]; }
    }
#pragma unroll
    for (int it = 0; it < R1; ++it)
      if (tid + it * NT < per_row) ss += v[it][0] * v[it][0] + v[it][1] * v[it][1] + v[it][2] * v[it][2] + v[it][3] * v[it][3];
    ss = wave_sum(ss);
    if (lane == 0) wsum[wave] = ss;
    lds_barrier();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) tot += wsum[w];                // fixed order: the same value in every thread
    const float r = 1.0f / sqrtf(tot / (float)a.K + a.eps);
#pragma unroll
    for (int it = 0; it < R1; ++it) {
      const int i = tid + it * NT;
      if (i < per_row) {
        bf16x4_t o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(v[it][e] * r * (float)gv[it][e]);
        ((bf16x4_t*)xs)[i] = o;
      }
    }
  } else {
    for (int i = tid; i < cpr; i += NT) ((bf16x8_t*)xs)[i] = ((const bf16x8_t*)a.x)[i];
  }
  lds_barrier();

  float acc0 = 0.f, acc1 = 0.f, acc0u = 0.f, acc1u = 0.f;
  for (int c = 0; c < per_lane; c += UB) {
    if (c > 0) load_batch(c);
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      if (c + u < per_lane) {
        const bf16x8_t xv = ((const bf16x8_t*)xs)[(c + u) * 64 + lane];
        acc0 = dot8(f0[u], xv, acc0);
        acc1 = dot8(f1[u], xv, acc1);
        if (EPI == FASTAV_EPI_SWIGLU) { acc0u = dot8(g0[u], xv, acc0u); acc1u = dot8(g1[u], xv, acc1u); }
      }
    }
  }
  acc0 = wave_sum(acc0);
  acc1 = wave_sum(acc1);
  if (EPI == FASTAV_EPI_SWIGLU) { acc0u = wave_sum(acc0u); acc1u = wave_sum(acc1u); }
  if (lane != 0) return;
  if (EPI == FASTAV_EPI_RESADD) {
    float2* yp = (float2*)((float*)a.y + n_lo);
    float2 y = *yp;
    y.x += acc0; y.y += acc1;
    *yp = y;
  } else if (rot) {
    ((bf16_t*)a.y)[n_lo] = (bf16_t)(acc0 * rc - acc1 * rs_);
    ((bf16_t*)a.y)[n_lo + dn] = (bf16_t)(acc1 * rc + acc0 * rs_);
  } else {
    if (EPI == FASTAV_EPI_SWIGLU) {
      acc0 = acc0 / (1.0f + __expf(-acc0)) * acc0u;
      acc1 = acc1 / (1.0f + __expf(-acc1)) * acc1u;
    }
    bf16x2_t o;
    o[0] = (bf16_t)acc0; o[1] = (bf16_t)acc1;
    *(bf16x2_t*)((bf16_t*)a.y + n_lo) = o;
  }
}

bool gemv_rows_supported(int B, int n, int k, bool norm) {
  return B == 1 && n % 16 == 0 && k % 512 == 0 && k <= 32768 && (!norm || k <= 8192);
}
// The one-row GEMV can rotate the heads it produces (see SkinnyArgs): the caller then skips the rope launch.
bool gemv_rows_fuses_rope(int B, int n, int k, bool norm, int rope_rows, int dh) {
  return gemv_rows_supported(B, n, k, norm) && dh % 16 == 0 && rope_rows % dh == 0 && rope_rows <= n;
}

bool skinny_linear_supported(int64_t m, int n, int k, int dtype, int64_t ldy) {
  return dtype == FASTAV_BF16 && m >= 1 && m <= 16 && n % 16 == 0 && k % 128 == 0 && ldy % 4 == 0;
}

// norm_x != nullptr: the input is rmsnorm(norm_x [B,k] fp32; gain norm_g, norm_eps) and x is ignored (needs
// B * k <= 32768 so that the normalised rows fit 64 KB of LDS; not with the residual epilogue)
bool skinny_norm_supported(int B, int k) { return (int64_t)B * k <= 32768; }

fastav_status_t launch_skinny_linear(const void* x, const void* const* w_seg, const int* seg_rows, int n_seg,
                                     const void* w2, void* y, int64_t ldy, int B, int n, int k, int epilogue,
                                     hipStream_t s, const float* norm_x, const void* norm_g, float norm_eps,
                                     const int32_t* rope_pos, int rope_rows, int rope_dh, float rope_base) {
  if (B == 0 || n == 0) return FASTAV_OK;
  if (rope_pos && (epilogue != FASTAV_EPI_STORE || !gemv_rows_fuses_rope(B, n, k, norm_x != nullptr, rope_rows, rope_dh)))
    return fail(FASTAV_EINVAL, "skinny linear: the fused rotation needs the one-row store kernel and whole heads");
  if (!skinny_linear_supported(B, n, k, FASTAV_BF16, ldy)) return fail(FASTAV_EUNSUPPORTED, "skinny linear: unsupported shape");
  if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)norm_x | (uintptr_t)norm_g) % 16)
    return fail(FASTAV_EINVAL, "skinny linear: x, y and the norm inputs must be 16-byte aligned");
  if (norm_x && (!norm_g || epilogue == FASTAV_EPI_RESADD || !skinny_norm_supported(B, k)))
    return fail(FASTAV_EINVAL, "skinny linear: bad fused-norm arguments");
  SkinnyArgs a;
  a.xres = norm_x; a.g = (const bf16_t*)norm_g; a.eps = norm_eps;
  a.pos = rope_pos; a.rope_rows = rope_pos ? rope_rows : 0; a.dh = rope_pos ? rope_dh : 16;
  a.rope_coef = rope_pos ? -log2((double)rope_base) * 2.0 / (double)rope_dh : 0.0;
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
  if (epilogue == FASTAV_EPI_SWIGLU && (!w2 || ((uintptr_t)w2 % 16)))
    return fail(FASTAV_EINVAL, "skinny linear: SwiGLU needs a 16-byte aligned up matrix");
  const int kind = epilogue == FASTAV_EPI_SWIGLU ? FASTAV_PROF_LINEAR_SWIGLU
                   : (epilogue == FASTAV_EPI_RESADD ? FASTAV_PROF_LINEAR_RESADD : FASTAV_PROF_LINEAR_STORE);
  // the work figure of a decode GEMV is its weight bytes (HBM-bound), not flops
  ProfScope prof(kind, (double)n * k * 2.0 * (epilogue == FASTAV_EPI_SWIGLU ? 2.0 : 1.0), s);
  if (gemv_rows_supported(B, n, k, norm_x != nullptr)) {
    const size_t lds = (size_t)k * 2;
#define FASTAV_GEMV(EPI, NORM, ROPE)                                                                            \
  do {                                                                                                          \
    if (lds > 32 * 1024) {                                                                                      \
      hipError_t e = hipFuncSetAttribute((const void*)k_gemv_rows<EPI, NORM, ROPE>, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024); \
      if (e != hipSuccess) return fail(FASTAV_EHIP, "gemv: hipFuncSetAttribute: %s", hipGetErrorString(e));     \
    }                                                                                                           \
    hipLaunchKernelGGL((k_gemv_rows<EPI, NORM, ROPE>), dim3((unsigned)(n / 16)), dim3(512), lds, s, a);         \
  } while (0)
    if (epilogue == FASTAV_EPI_SWIGLU) { if (norm_x) FASTAV_GEMV(FASTAV_EPI_SWIGLU, true, false); else FASTAV_GEMV(FASTAV_EPI_SWIGLU, false, false); }
    else if (epilogue == FASTAV_EPI_RESADD) FASTAV_GEMV(FASTAV_EPI_RESADD, false, false);
    else if (rope_pos) { if (norm_x) FASTAV_GEMV(FASTAV_EPI_STORE, true, true); else FASTAV_GEMV(FASTAV_EPI_STORE, false, true); }
    else { if (norm_x) FASTAV_GEMV(FASTAV_EPI_STORE, true, false); else FASTAV_GEMV(FASTAV_EPI_STORE, false, false); }
#undef FASTAV_GEMV
    return check_launch("gemv_rows");
  }
  // eight waves split K where its length allows: twice the loads in flight per workgroup (measured faster for
  // every projection of the 7B shape, also the wide gate/up one)
  const bool wide = k % 256 == 0;
  const dim3 grid((unsigned)(n / 16));
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
  float scale_log2;           // log2(e) / sqrt(head_dim): logits live in the base-2 domain
  float* part;                // [B, Hkv, splits, G, DH + 2] fp32: o (unnormalised), max (base-2 domain), sum
};

// One workgroup per (key split, KV head, sample); its four waves take the split's 64-key chunks in turn.
// Per chunk a wave
//   * reads the 64 keys straight from global memory in matrix-core operand layout (lane = key row x 16-byte
//     dim chunk) and the query heads of the group as the other operand (heads padded to 16 columns): the
//     logits of all heads of the group come out of DH/32 v_mfma_f32_16x16x32_bf16 per 16 keys, lane = head,
//     four keys each;
//   * updates the running (max, sum) of every head (in-lane over its keys, two shuffles across the lane
//     groups), writes the 64 x G probabilities to LDS;
//   * accumulates P V with lane = (key subgroup, 8 output dims): a V row is one 16-byte load per lane, the
//     G probabilities of its key one broadcast LDS read, G x 8 FMAs.
// Nothing is staged through LDS but the probabilities, and the waves never wait for each other until the
// end, where their (max, sum, o) are combined and written as the split's partial; k_decode_merge combines the
// splits.  (Merging in the same launch by the workgroup that finishes last was measured: the device-scope
// release every workgroup then needs writes back its L2 and costs more than the second launch.)
template <int DH, int GP>
__global__ __launch_bounds__(256) void k_decode_attn(DecodeAttnArgs a) {
  constexpr int CK = 64;                              // keys per chunk
  constexpr int STEPS = DH / 32;                      // matrix instructions per 16-key tile
  constexpr int SEGS = DH / 8;                        // lanes (16-byte segments) per V row
  constexpr int KPI = 64 / SEGS;                      // keys one wave-wide V load covers
  constexpr int NIT = CK / KPI;
  constexpr int PD = DH + 2;
  __shared__ __attribute__((aligned(16))) float ps[4][CK][GP];
  __shared__ __attribute__((aligned(16))) float red_o[4][GP][DH];     // the four waves' outputs
  __shared__ float red_m[4][GP], red_l[4][GP];
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int G = a.Hq / a.Hkv;                         // <= GP (checked by the launcher)
  const int kd = a.Hkv * DH;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int p0 = a.cu_prefix[b], n_pre = a.cu_prefix[b + 1] - p0;
  const int n_tot = n_pre + a.gen_len + 1;
  const int j_begin = split * a.chunk;
  const int j_end = (j_begin + a.chunk < n_tot) ? j_begin + a.chunk : n_tot;
  const int head = lane & 15, lg = lane >> 4;         // logits: lane = (head column, lane group)
  const int seg = lane % SEGS, kq = lane / SEGS;      // P V: lane = (8 output dims, key subgroup)

  // row j of the unified key list: prefix, then generated, then the token itself
  auto krow = [&](int j) __attribute__((always_inline)) -> const bf16_t* {
    if (j < n_pre) return a.k_prefix + (int64_t)(p0 + j) * kd + g * DH;
    if (j < n_pre + a.gen_len) return a.k_gen + ((int64_t)b * a.gen_cap + (j - n_pre)) * kd + g * DH;
    return a.k_self + (int64_t)b * a.q_stride + g * DH;
  };
  auto vrow = [&](int j) __attribute__((always_inline)) -> const bf16_t* {
    if (j < n_pre) return a.v_prefix + (int64_t)(p0 + j) * kd + g * DH;
    if (j < n_pre + a.gen_len) return a.v_gen + ((int64_t)b * a.gen_cap + (j - n_pre)) * kd + g * DH;
    return a.v_self + (int64_t)b * a.q_stride + g * DH;
  };

  bf16x8_t qf[STEPS];
#pragma unroll
  for (int st = 0; st < STEPS; ++st) {
    bf16x8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
    qf[st] = head < G ? *(const bf16x8_t*)(a.q + (int64_t)b * a.q_stride + (g * G + head) * DH + lg * 8 + 32 * st) : z;
  }
  float m_run = -INFINITY, l_part = 0.f;              // per head (column): max over all lane groups, this lane's share of the sum
  float acc[GP][8];
#pragma unroll
  for (int h = 0; h < GP; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;

  for (int c0 = j_begin + wave * CK; c0 < j_end; c0 += 4 * CK) {
    bf16x8_t kf[4][STEPS], vf[NIT];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      int j = c0 + t * 16 + head;                     // here `head` is the key row of the A operand
      j = j < j_end ? j : j_end - 1;                  // rows past the end repeat the last key (masked below)
      const bf16_t* kr = krow(j) + lg * 8;
#pragma unroll
      for (int st = 0; st < STEPS; ++st) kf[t][st] = *(const bf16x8_t*)(kr + 32 * st);
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      int j = c0 + it * KPI + kq;
      j = j < j_end ? j : j_end - 1;
      vf[it] = *(const bf16x8_t*)(vrow(j) + seg * 8);
    }
    f32x4v sc[4];
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      f32x4v c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < STEPS; ++st) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][st], qf[st], c, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        c[r] = (c0 + t * 16 + lg * 4 + r < j_end) ? c[r] * a.scale_log2 : -INFINITY;
        mx = fmaxf(mx, c[r]);
      }
      sc[t] = c;
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));        // finite: key c0 exists
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);      // exp2(-inf) = 0 on the first chunk
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float pr = __builtin_amdgcn_exp2f(sc[t][r] - m_new);
        psum += pr;
        if (head < GP) ps[wave][t * 16 + lg * 4 + r][head] = pr;
      }
    l_part = l_part * alpha + psum;
    m_run = m_new;
    // the wave's own LDS writes are visible to its other lanes after the LDS counter wait below
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
#pragma unroll
    for (int h = 0; h < GP; ++h) {
      const float ah = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(alpha), h));          // lane h holds head h
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] *= ah;
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      float pv[GP];
#pragma unroll
      for (int h4 = 0; h4 < GP; h4 += 4) {
        const f32x4v t4 = *(const f32x4v*)&ps[wave][it * KPI + kq][h4];
        pv[h4] = t4[0]; pv[h4 + 1] = t4[1]; pv[h4 + 2] = t4[2]; pv[h4 + 3] = t4[3];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float v = (float)vf[it][e];
#pragma unroll
        for (int h = 0; h < GP; ++h) acc[h][e] = fmaf(pv[h], v, acc[h][e]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();                  // all reads of ps done before the next chunk rewrites it
  }

  // ---- combine inside the wave: the sum over lane groups, the outputs over key subgroups
  l_part += __shfl_xor(l_part, 16, kWave);
  l_part += __shfl_xor(l_part, 32, kWave);
#pragma unroll
  for (int h = 0; h < GP; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[h][e];
#pragma unroll
      for (int o = SEGS; o < 64; o <<= 1) v += __shfl_xor(v, o, kWave);
      acc[h][e] = v;
    }
  if (kq == 0) {
#pragma unroll
    for (int h = 0; h < GP; ++h) {
      f32x4v lo = {acc[h][0], acc[h][1], acc[h][2], acc[h][3]}, hi = {acc[h][4], acc[h][5], acc[h][6], acc[h][7]};
      *(f32x4v*)&red_o[wave][h][seg * 8] = lo;
      *(f32x4v*)&red_o[wave][h][seg * 8 + 4] = hi;
    }
  }
  if (lane < GP) { red_m[wave][lane] = m_run; red_l[wave][lane] = l_part; }
  __syncthreads();
  // ---- combine the four waves, write the split's partial: thread = (head, dim)
  float* part = a.part + (((int64_t)b * a.Hkv + g) * a.splits + split) * (int64_t)(G * PD);
  for (int i = tid; i < G * DH; i += 256) {
    const int h = i / DH, d = i % DH;
    float M = red_m[0][h];
#pragma unroll
    for (int w = 1; w < 4; ++w) M = fmaxf(M, red_m[w][h]);
    float o = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = red_m[w][h];
      const float f = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
      o = fmaf(f, red_o[w][h][d], o);
      l = fmaf(f, red_l[w][h], l);
    }
    part[h * PD + d] = o;
    if (d == 0) { part[h * PD + DH] = M; part[h * PD + DH + 1] = l; }
  }
}

// Merge of the splits' partials: one workgroup per (query head, sample), no loop-carried waits.  Every wave
// loads the splits' (max, sum) with lane = split and gets the global max and the weights from two wave
// reductions; thread = (split group, 4 output dims) has the weighted outputs of its splits in flight at the same
// time (independent 8-byte loads, out-of-range splits clamped and weighted 0), and the groups are summed through
// LDS.  splits <= 64.
template <int DH>
__global__ __launch_bounds__(256) void k_decode_merge(const float* __restrict__ part_all, int splits, int Hq, int Hkv,
                                                      bf16_t* __restrict__ out, int64_t out_stride) {
  constexpr int PD = DH + 2;
  constexpr int QUADS = DH / 4;                       // 32 or 16 column quads
  constexpr int NSG = 256 / QUADS;                    // 8 or 16 split groups
  constexpr int NK = 64 / NSG;                        // splits per thread
  __shared__ __attribute__((aligned(16))) float red_o[NSG][DH];
  const int hq = blockIdx.x, b = blockIdx.y;
  const int G = Hq / Hkv, g = hq / G, h = hq % G;
  const int tid = threadIdx.x, lane = tid & 63;
  // partial of (split sp, head h): pall + sp * G * PD
  const float* pall = part_all + (((int64_t)b * Hkv + g) * splits * G + h) * (int64_t)PD;
  const int c = tid % QUADS, sg = tid / QUADS;
  float2 lo[NK], hi[NK];
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    int sp = sg + k * NSG;
    sp = sp < splits ? sp : splits - 1;
    // rows are PD = DH + 2 floats apart: 8-byte aligned, so two 8-byte loads per quad
    lo[k] = *(const float2*)(pall + (int64_t)sp * G * PD + c * 4);
    hi[k] = *(const float2*)(pall + (int64_t)sp * G * PD + c * 4 + 2);
  }
  const float ms = lane < splits ? pall[(int64_t)lane * G * PD + DH] : -INFINITY;   // -inf: a split past this sample's keys
  const float ls = lane < splits ? pall[(int64_t)lane * G * PD + DH + 1] : 0.f;
  const float M = wave_max(ms);                       // finite: split 0 always holds a key
  const float wgt = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - M);
  const float inv = 1.0f / wave_sum(wgt * ls);
  f32x4v o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    const int sp = sg + k * NSG;                      // < 64: lane sp of this wave holds its weight (0 beyond splits)
    const float f = __shfl(wgt, sp, kWave);
    o[0] = fmaf(f, lo[k].x, o[0]); o[1] = fmaf(f, lo[k].y, o[1]);
    o[2] = fmaf(f, hi[k].x, o[2]); o[3] = fmaf(f, hi[k].y, o[3]);
  }
  *(f32x4v*)&red_o[sg][c * 4] = o;
  __syncthreads();
  if (tid < DH) {
    float t = 0.f;
#pragma unroll
    for (int q = 0; q < NSG; ++q) t += red_o[q][tid];
    out[(int64_t)b * out_stride + hq * DH + tid] = (bf16_t)(t * inv);
  }
}

// partials [B, Hkv, splits, G, dh + 2] fp32
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
                        (uintptr_t)k_gen | (uintptr_t)v_gen) % 16 || ((Hkv * dh) % 8))
    return fail(FASTAV_EINVAL, "decode attention: operands must be 16-byte aligned");
  DecodeAttnArgs a;
  a.q = (const bf16_t*)q; a.k_self = (const bf16_t*)k_self; a.v_self = (const bf16_t*)v_self; a.q_stride = q_stride;
  a.k_prefix = (const bf16_t*)k_prefix; a.v_prefix = (const bf16_t*)v_prefix; a.cu_prefix = cu_prefix;
  a.k_gen = (const bf16_t*)k_gen; a.v_gen = (const bf16_t*)v_gen; a.gen_len = gen_len; a.gen_cap = gen_cap;
  a.Hq = Hq; a.Hkv = Hkv;
  const int max_keys = max_prefix + gen_len + 1;
  a.splits = decode_attn_splits(batch, Hkv, max_keys);
  a.chunk = (int)(ceil_div(ceil_div(max_keys, a.splits), 64) * 64);
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)dh);
  a.part = part;
  if ((size_t)batch * Hq * a.splits * (dh + 2) * sizeof(float) > part_bytes)
    return fail(FASTAV_EINVAL, "decode attention: workspace too small");
  ProfScope prof(FASTAV_PROF_ATTENTION, bytes_hint, s);
  const dim3 grid((unsigned)a.splits, (unsigned)Hkv, (unsigned)batch);
  const int G = Hq / Hkv;
  const dim3 mgrid((unsigned)Hq, (unsigned)batch);
#define FASTAV_DECODE_ATTN(DH_, GP_)                                                                              \
  do {                                                                                                            \
    hipLaunchKernelGGL((k_decode_attn<DH_, GP_>), grid, dim3(256), 0, s, a);                                      \
    hipLaunchKernelGGL((k_decode_merge<DH_>), mgrid, dim3(256), 0, s, (const float*)part, a.splits, Hq, Hkv,      \
                       (bf16_t*)out, out_stride);                                                                 \
  } while (0)
  if (dh == 128 && G <= 4) FASTAV_DECODE_ATTN(128, 4);
  else if (dh == 128) FASTAV_DECODE_ATTN(128, 8);
  else if (G <= 4) FASTAV_DECODE_ATTN(64, 4);
  else FASTAV_DECODE_ATTN(64, 8);
#undef FASTAV_DECODE_ATTN
  return check_launch("decode_attention");
}

}  // namespace fastav
