// Row-wise and bookkeeping kernels of the decoder layer: small-array upload, token bookkeeping
// (original positions + protected mask), dtype conversion, RMSNorm and rotate-half RoPE.
// All of them are HBM-bound streaming kernels: one pass over the data with 16-byte accesses.
#include "common.hpp"

namespace fastav {

// ---------------------------------------------------------------------------------------- upload_small
struct SmallPayload { uint32_t w[896]; };   // 3584 B: stays under the 4 KB kernel-argument limit

__global__ void k_upload_small(uint32_t* __restrict__ dst, SmallPayload p, int n_words) {
  for (int i = threadIdx.x; i < n_words; i += blockDim.x) dst[i] = p.w[i];
}

fastav_status_t upload_small(void* dst_dev, const void* host_src, size_t bytes, hipStream_t s) {
  if (bytes == 0) return FASTAV_OK;
  if ((bytes & 3) || ((uintptr_t)dst_dev & 3)) return fail(FASTAV_EINVAL, "upload_small: size/alignment must be 4 bytes");
  const uint32_t* src = (const uint32_t*)host_src;
  size_t words = bytes / 4, done = 0;
  while (done < words) {
    SmallPayload p;
    int n = (int)((words - done) < 896 ? (words - done) : 896);
    for (int i = 0; i < n; ++i) p.w[i] = src[done + i];
    hipLaunchKernelGGL(k_upload_small, dim3(1), dim3(256), 0, s, (uint32_t*)dst_dev + done, p, n);
    done += n;
  }
  return check_launch("upload_small");
}

// ---------------------------------------------------------------------------------------- init_tokens
// pos[row] = in-sample position; prot[row] = 1 for TEXT spans and the last n_last positions
// (the tokens a prune may never remove).
__global__ void k_init_tokens(const int32_t* __restrict__ cu, const int32_t* __restrict__ span_off,
                              const fastav_span_t* __restrict__ spans, int n_last, int32_t* __restrict__ pos,
                              uint8_t* __restrict__ prot) {
  const int b = blockIdx.y;
  const int base = cu[b], n = cu[b + 1] - base;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  int is_text = 0;
  for (int si = span_off[b]; si < span_off[b + 1]; ++si) {
    const fastav_span_t sp = spans[si];
    if (j >= sp.start && j < sp.start + sp.len) { is_text = (sp.modality == FASTAV_TEXT); break; }
  }
  pos[base + j] = j;
  prot[base + j] = (uint8_t)((is_text || j >= n - n_last) ? 1 : 0);
}

fastav_status_t launch_init_tokens(const int32_t* cu, const int32_t* span_offsets, const fastav_span_t* spans,
                                   int batch, int64_t T, int max_seqlen, int n_last, int32_t* pos, uint8_t* prot,
                                   hipStream_t s) {
  (void)T;
  if (batch == 0 || max_seqlen == 0) return FASTAV_OK;
  dim3 grid((unsigned)ceil_div(max_seqlen, 256), (unsigned)batch);
  hipLaunchKernelGGL(k_init_tokens, grid, dim3(256), 0, s, cu, span_offsets, spans, n_last, pos, prot);
  return check_launch("init_tokens");
}

// ---------------------------------------------------------------------------------------- to_f32
template <typename T>
__global__ void k_to_f32(const T* __restrict__ x, float* __restrict__ y, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) y[i] = to_f32(x[i]);
}
__global__ void k_bf16x8_to_f32(const bf16x8_t* __restrict__ x, f32x4_t* __restrict__ y, int64_t n8) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n8; i += stride) {
    const bf16x8_t v = x[i];
    f32x4_t a, b;
    a[0] = (float)v[0]; a[1] = (float)v[1]; a[2] = (float)v[2]; a[3] = (float)v[3];
    b[0] = (float)v[4]; b[1] = (float)v[5]; b[2] = (float)v[6]; b[3] = (float)v[7];
    y[2 * i] = a; y[2 * i + 1] = b;
  }
}

fastav_status_t launch_to_f32(const void* x, float* y, int64_t n, int dtype, hipStream_t s) {
  if (n == 0) return FASTAV_OK;
  if (dtype == FASTAV_BF16 && (n % 8) == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)y % 16) == 0) {
    const int64_t n8 = n / 8;
    unsigned blocks = (unsigned)(ceil_div(n8, 256) < 16384 ? ceil_div(n8, 256) : 16384);
    hipLaunchKernelGGL(k_bf16x8_to_f32, dim3(blocks), dim3(256), 0, s, (const bf16x8_t*)x, (f32x4_t*)y, n8);
  } else {
    unsigned blocks = (unsigned)(ceil_div(n, 256) < 16384 ? ceil_div(n, 256) : 16384);
    if (dtype == FASTAV_BF16) hipLaunchKernelGGL(k_to_f32<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)x, y, n);
    else hipLaunchKernelGGL(k_to_f32<float>, dim3(blocks), dim3(256), 0, s, (const float*)x, y, n);
  }
  return check_launch("to_f32");
}

// ---------------------------------------------------------------------------------------- rmsnorm
// One 256-thread workgroup per row of the fp32 residual stream.  The row (<= 32 KB) is read twice; the
// second read is served by the CU's vector cache, so HBM sees 4*d bytes in and sizeof(T)*d out per row.
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm(const float* __restrict__ x, const T* __restrict__ g,
                                                 T* __restrict__ y, int d, float eps) {
  __shared__ float red[4];
  const float* xr = x + (int64_t)blockIdx.x * d;
  T* yr = y + (int64_t)blockIdx.x * d;
  float ss = 0.f;
  const bool vec = (d % 4) == 0;
  if (vec) {
    const f32x4_t* xv = (const f32x4_t*)xr;
    for (int i = threadIdx.x; i < d / 4; i += 256) {
      const f32x4_t v = xv[i];
      ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    }
  } else {
    for (int i = threadIdx.x; i < d; i += 256) ss += xr[i] * xr[i];
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = red[0] + red[1] + red[2] + red[3];
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
  if (vec) {
    const f32x4_t* xv = (const f32x4_t*)xr;
    for (int i = threadIdx.x; i < d / 4; i += 256) {
      const f32x4_t v = xv[i];
#pragma unroll
      for (int c = 0; c < 4; ++c) yr[4 * i + c] = from_f32<T>(v[c] * r * to_f32(g[4 * i + c]));
    }
  } else {
    for (int i = threadIdx.x; i < d; i += 256) yr[i] = from_f32<T>(xr[i] * r * to_f32(g[i]));
  }
}

// The same for rows of up to 1024 * NV floats with d a multiple of 4: the row is read ONCE, 16 bytes per lane and
// load, kept in registers across the reduction, and written back 4 elements per store.
// With `partial` (splits > 0) the row is first completed: x += partial[0] + partial[1] + ... (the pending split-K sums
// of the residual projection that produced it, added in split order like k_splitk_reduce adds them) and written back.
template <typename T, int NV>
__global__ __launch_bounds__(256) void k_rmsnorm_reg(float* __restrict__ x, const T* __restrict__ g,
                                                     T* __restrict__ y, int d, float eps,
                                                     const float* __restrict__ partial, int splits, int64_t split_stride) {
  __shared__ float red[4];
  f32x4_t* xv = (f32x4_t*)(x + (int64_t)blockIdx.x * d);
  T* yr = y + (int64_t)blockIdx.x * d;
  const int n4 = d >> 2;
  f32x4_t v[NV];
  float ss = 0.f;
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int i = threadIdx.x + u * 256;
    v[u] = (i < n4) ? xv[i] : f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  if (splits > 0) {
    const f32x4_t* pv = (const f32x4_t*)(partial + (int64_t)blockIdx.x * d);
    for (int sp = 0; sp < splits; ++sp) {
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const int i = threadIdx.x + u * 256;
        if (i < n4) {
          const f32x4_t q = pv[(int64_t)sp * (split_stride / 4) + i];
          v[u][0] += q[0]; v[u][1] += q[1]; v[u][2] += q[2]; v[u][3] += q[3];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int i = threadIdx.x + u * 256;
      if (i < n4) xv[i] = v[u];
    }
  }
#pragma unroll
  for (int u = 0; u < NV; ++u) ss += v[u][0] * v[u][0] + v[u][1] * v[u][1] + v[u][2] * v[u][2] + v[u][3] * v[u][3];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = red[0] + red[1] + red[2] + red[3];
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int i = threadIdx.x + u * 256;
    if (i < n4) {
      if constexpr (sizeof(T) == 2) {
        const bf16x4_t gv = *(const bf16x4_t*)(g + 4 * i);
        bf16x4_t o;
#pragma unroll
        for (int c = 0; c < 4; ++c) o[c] = (bf16_t)(v[u][c] * r * (float)gv[c]);
        *(bf16x4_t*)(yr + 4 * i) = o;
      } else {
        const f32x4_t gv = *(const f32x4_t*)(g + 4 * i);
        f32x4_t o;
#pragma unroll
        for (int c = 0; c < 4; ++c) o[c] = v[u][c] * r * gv[c];
        *(f32x4_t*)(yr + 4 * i) = o;
      }
    }
  }
}

fastav_status_t launch_rmsnorm(float* x, const void* g, void* y, int64_t rows, int d, float eps, int dtype,
                               hipStream_t s, const SplitKPending* pend) {
  if (rows == 0) return FASTAV_OK;
  ProfScope prof(FASTAV_PROF_RMSNORM, (double)rows * d * (4.0 + (dtype == FASTAV_BF16 ? 2.0 : 4.0)), s);
  const size_t es = dtype == FASTAV_BF16 ? 2 : 4;
  const bool reg = (d % 4) == 0 && d <= 8192 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)g % (4 * es)) == 0 && ((uintptr_t)y % (4 * es)) == 0;
  const float* partial = nullptr;
  int splits = 0;
  int64_t split_stride = 0;
  if (pend != nullptr && pend->splits > 0) {
    const bool fits = reg && pend->N == d && pend->M == rows && ((uintptr_t)pend->partial % 16) == 0;
    if (fits) { partial = pend->partial; splits = pend->splits; split_stride = pend->M * (int64_t)pend->N; }
    else { fastav_status_t st = launch_splitk_reduce(x, d, *pend, s); if (st != FASTAV_OK) return st; }
  }
  const dim3 grid((unsigned)rows), blk(256);
#define FASTAV_RMS_REG(TT, NVV) hipLaunchKernelGGL((k_rmsnorm_reg<TT, NVV>), grid, blk, 0, s, x, (const TT*)g, (TT*)y, d, eps, partial, splits, split_stride)
  if (reg && dtype == FASTAV_BF16) {
    if (d <= 1024) FASTAV_RMS_REG(bf16_t, 1); else if (d <= 2048) FASTAV_RMS_REG(bf16_t, 2);
    else if (d <= 4096) FASTAV_RMS_REG(bf16_t, 4); else FASTAV_RMS_REG(bf16_t, 8);
  } else if (reg) {
    if (d <= 1024) FASTAV_RMS_REG(float, 1); else if (d <= 2048) FASTAV_RMS_REG(float, 2);
    else if (d <= 4096) FASTAV_RMS_REG(float, 4); else FASTAV_RMS_REG(float, 8);
  } else if (dtype == FASTAV_BF16)
    hipLaunchKernelGGL(k_rmsnorm<bf16_t>, grid, blk, 0, s, x, (const bf16_t*)g, (bf16_t*)y, d, eps);
  else
    hipLaunchKernelGGL(k_rmsnorm<float>, grid, blk, 0, s, x, (const float*)g, (float*)y, d, eps);
#undef FASTAV_RMS_REG
  return check_launch("rmsnorm");
}

// ---------------------------------------------------------------------------------------- rope
// One workgroup per row.  Thread t < head_dim/2 owns frequency index i = t: it evaluates the angle
// pos * base^(-2i/dh) once in fp64 (positions reach 16k+, where an fp32 angle loses ~1e-3 rad) and applies
// the rotation to pair (i, i + dh/2) of every head: n_heads heads of x, then n_heads2 heads of a second tensor x2
// (K living in a cache of its own).
template <typename T>
__global__ void k_rope(T* __restrict__ x, int64_t row_stride, T* __restrict__ x2, int64_t row_stride2,
                       const int32_t* __restrict__ pos, int n_heads, int n_heads2, int head_dim,
                       double neg_log2_base_2_over_dh) {
  const int half = head_dim >> 1;
  const int i = threadIdx.x % half;
  const int h0 = threadIdx.x / half;
  const int hstep = blockDim.x / half;
  const int64_t r = blockIdx.x;
  const double inv_freq = exp2((double)i * neg_log2_base_2_over_dh);
  const double ang = (double)pos[r] * inv_freq;
  double sd, cd;
  sincos(ang, &sd, &cd);
  const float c = (float)cd, sn = (float)sd;
  T* xr = x + r * row_stride;
  T* xr2 = x2 + r * row_stride2;
  for (int h = h0; h < n_heads + n_heads2; h += hstep) {
    T* p = h < n_heads ? xr + h * head_dim : xr2 + (h - n_heads) * head_dim;
    const float a = to_f32(p[i]), b = to_f32(p[i + half]);
    p[i] = from_f32<T>(a * c - b * sn);
    p[i + half] = from_f32<T>(b * c + a * sn);
  }
}

// (cos, sin) of pos * base^(-2i/dh) for every position below n_pos and frequency index i < dh/2, angles evaluated
// in fp64 as above: computed once per prefill (a token keeps its original position through every prune), so that
// the per-layer rotation is a pure streaming pass.
__global__ void k_rope_table(float2* __restrict__ table, int n_pos, int half, double neg_log2_base_2_over_dh) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_pos * half) return;
  const int p = idx / half, i = idx % half;
  double sd, cd;
  sincos((double)p * exp2((double)i * neg_log2_base_2_over_dh), &sd, &cd);
  table[idx] = make_float2((float)cd, (float)sd);
}

// Rotation from the table, bf16, head_dim a multiple of 16: a thread owns 8 consecutive frequency indices (16-byte
// loads and stores of both halves of the pair) of every 8th head of one row, so the 64 bytes of table it needs are
// read once for several heads; the lanes of a wave cover eight neighbouring heads at a time, whole 128-byte runs.
constexpr int kRopeHeadGroups = 8;
__global__ __launch_bounds__(256) void k_rope_tab(bf16_t* __restrict__ x, int64_t row_stride, bf16_t* __restrict__ x2,
                                                  int64_t row_stride2, const int32_t* __restrict__ pos,
                                                  const float2* __restrict__ table, int n_heads, int n_heads2, int head_dim,
                                                  int64_t rows) {
  const int half = head_dim >> 1, cph = half >> 3;               // 8-index chunks per head
  const int per_row = kRopeHeadGroups * cph;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t r = idx / per_row;
  if (r >= rows) return;
  const int w = (int)(idx - r * per_row);
  const int hg = w / cph, c = w % cph;
  const float2* tr = table + (int64_t)pos[r] * half;
  const f32x4_t t0 = *(const f32x4_t*)(tr + 8 * c), t1 = *(const f32x4_t*)(tr + 8 * c + 2);
  const f32x4_t t2 = *(const f32x4_t*)(tr + 8 * c + 4), t3 = *(const f32x4_t*)(tr + 8 * c + 6);
  const float cs[8] = {t0[0], t0[2], t1[0], t1[2], t2[0], t2[2], t3[0], t3[2]};
  const float sn[8] = {t0[1], t0[3], t1[1], t1[3], t2[1], t2[3], t3[1], t3[3]};
  for (int h = hg; h < n_heads + n_heads2; h += kRopeHeadGroups) {
    bf16_t* p = (h < n_heads ? x + r * row_stride + h * head_dim : x2 + r * row_stride2 + (h - n_heads) * head_dim) + 8 * c;
    const bf16x8_t a = *(const bf16x8_t*)p, b = *(const bf16x8_t*)(p + half);
    bf16x8_t oa, ob;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float fa = (float)a[e], fb = (float)b[e];
      oa[e] = (bf16_t)(fa * cs[e] - fb * sn[e]);
      ob[e] = (bf16_t)(fb * cs[e] + fa * sn[e]);
    }
    *(bf16x8_t*)p = oa;
    *(bf16x8_t*)(p + half) = ob;
  }
}

size_t rope_table_bytes(int n_pos, int head_dim) { return (size_t)n_pos * (head_dim / 2) * sizeof(float2); }

fastav_status_t launch_rope_table(void* table, int n_pos, int head_dim, float base, hipStream_t s) {
  if (n_pos == 0) return FASTAV_OK;
  const int half = head_dim / 2;
  const double e = -log2((double)base) * 2.0 / (double)head_dim;
  hipLaunchKernelGGL(k_rope_table, dim3((unsigned)ceil_div((int64_t)n_pos * half, 256)), dim3(256), 0, s, (float2*)table, n_pos, half, e);
  return check_launch("rope_table");
}

fastav_status_t launch_rope2(void* x, int64_t row_stride, int n_heads, void* x2, int64_t row_stride2, int n_heads2,
                             const int32_t* pos, int64_t rows, int head_dim, float base, int dtype, hipStream_t s,
                             const void* table) {
  const int nh = n_heads + n_heads2;
  if (rows == 0 || nh == 0) return FASTAV_OK;
  ProfScope prof(FASTAV_PROF_ROPE, 2.0 * rows * nh * head_dim * (dtype == FASTAV_BF16 ? 2.0 : 4.0), s);
  if (table != nullptr && dtype == FASTAV_BF16 && head_dim % 16 == 0 && row_stride % 8 == 0 && row_stride2 % 8 == 0 &&
      (((uintptr_t)x | (uintptr_t)x2 | (uintptr_t)table) % 16) == 0) {
    const int64_t items = rows * kRopeHeadGroups * (head_dim / 16);
    hipLaunchKernelGGL(k_rope_tab, dim3((unsigned)ceil_div(items, 256)), dim3(256), 0, s, (bf16_t*)x, row_stride, (bf16_t*)x2, row_stride2, pos,
                       (const float2*)table, n_heads, n_heads2, head_dim, rows);
    return check_launch("rope_tab");
  }
  const int half = head_dim / 2;
  int hpb = 256 / half; if (hpb < 1) hpb = 1; if (hpb > nh) hpb = nh;
  const double e = -log2((double)base) * 2.0 / (double)head_dim;
  if (dtype == FASTAV_BF16)
    hipLaunchKernelGGL(k_rope<bf16_t>, dim3((unsigned)rows), dim3(half * hpb), 0, s, (bf16_t*)x, row_stride, (bf16_t*)x2, row_stride2,
                       pos, n_heads, n_heads2, head_dim, e);
  else
    hipLaunchKernelGGL(k_rope<float>, dim3((unsigned)rows), dim3(half * hpb), 0, s, (float*)x, row_stride, (float*)x2, row_stride2,
                       pos, n_heads, n_heads2, head_dim, e);
  return check_launch("rope");
}

fastav_status_t launch_rope(void* x, int64_t row_stride, const int32_t* pos, int64_t rows, int n_heads, int head_dim,
                            float base, int dtype, hipStream_t s, const void* table) {
  return launch_rope2(x, row_stride, n_heads, x, row_stride, 0, pos, rows, head_dim, base, dtype, s, table);
}

}  // namespace fastav
