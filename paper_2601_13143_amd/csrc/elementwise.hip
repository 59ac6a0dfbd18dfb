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

fastav_status_t launch_rmsnorm(const float* x, const void* g, void* y, int64_t rows, int d, float eps, int dtype,
                               hipStream_t s) {
  if (rows == 0) return FASTAV_OK;
  ProfScope prof(FASTAV_PROF_RMSNORM, (double)rows * d * (4.0 + (dtype == FASTAV_BF16 ? 2.0 : 4.0)), s);
  if (dtype == FASTAV_BF16)
    hipLaunchKernelGGL(k_rmsnorm<bf16_t>, dim3((unsigned)rows), dim3(256), 0, s, x, (const bf16_t*)g, (bf16_t*)y, d, eps);
  else
    hipLaunchKernelGGL(k_rmsnorm<float>, dim3((unsigned)rows), dim3(256), 0, s, x, (const float*)g, (float*)y, d, eps);
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

fastav_status_t launch_rope2(void* x, int64_t row_stride, int n_heads, void* x2, int64_t row_stride2, int n_heads2,
                             const int32_t* pos, int64_t rows, int head_dim, float base, int dtype, hipStream_t s) {
  const int nh = n_heads + n_heads2;
  if (rows == 0 || nh == 0) return FASTAV_OK;
  ProfScope prof(FASTAV_PROF_ROPE, 2.0 * rows * nh * head_dim * (dtype == FASTAV_BF16 ? 2.0 : 4.0), s);
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
                            float base, int dtype, hipStream_t s) {
  return launch_rope2(x, row_stride, n_heads, x, row_stride, 0, pos, rows, head_dim, base, dtype, s);
}

}  // namespace fastav
