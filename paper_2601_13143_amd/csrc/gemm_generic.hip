// Shape-agnostic linear layer C = A W^T (W stored [N, K]) on the vector ALUs with fp32 accumulation.
// It serves the fp32 models and any bf16 shape the MFMA kernel's tiling does not cover (K or N not a
// multiple of its tile); every access is bounds-checked.  64x64 output tile per 256-thread workgroup,
// 4x4 outputs per thread, K staged 16 at a time through LDS.
#include "common.hpp"

namespace fastav {

template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm_generic(const T* __restrict__ A, const T* __restrict__ W,
                                                      const T* __restrict__ W2, void* __restrict__ Cv, int64_t ldc,
                                                      int64_t M, int N, int K) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Ws[BK][BN + 4];
  __shared__ float W2s[EPI == FASTAV_EPI_SWIGLU ? BK : 1][BN + 4];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int64_t m0 = (int64_t)blockIdx.y * BM;
  const int n0 = blockIdx.x * BN;
  float acc[4][4] = {}, acc2[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = threadIdx.x; i < BM * BK; i += 256) {
      const int r = i / BK, c = i % BK;
      const int64_t gm = m0 + r;
      const int gk = k0 + c;
      As[c][r] = (gm < M && gk < K) ? to_f32(A[gm * K + gk]) : 0.f;
      const int gn = n0 + r;
      Ws[c][r] = (gn < N && gk < K) ? to_f32(W[(int64_t)gn * K + gk]) : 0.f;
      if (EPI == FASTAV_EPI_SWIGLU) W2s[c][r] = (gn < N && gk < K) ? to_f32(W2[(int64_t)gn * K + gk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], w[4], w2[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; w[i] = Ws[kk][tx * 4 + i]; }
      if (EPI == FASTAV_EPI_SWIGLU) {
#pragma unroll
        for (int i = 0; i < 4; ++i) w2[i] = W2s[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
          if (EPI == FASTAV_EPI_SWIGLU) acc2[i][j] = fmaf(a[i], w2[j], acc2[i][j]);
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      if (EPI == FASTAV_EPI_STORE) {
        ((T*)Cv)[gm * ldc + gn] = from_f32<T>(acc[i][j]);
      } else if (EPI == FASTAV_EPI_RESADD) {
        ((float*)Cv)[gm * ldc + gn] += acc[i][j];
      } else {
        const float g = acc[i][j];
        ((T*)Cv)[gm * ldc + gn] = from_f32<T>(g / (1.0f + expf(-g)) * acc2[i][j]);
      }
    }
  }
}

template <typename T>
static void launch_generic_t(const void* a, const void* w, const void* w2, void* c, int64_t ldc, int64_t m, int n, int k,
                             int epilogue, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(n, 64), (unsigned)ceil_div(m, 64));
  if (epilogue == FASTAV_EPI_STORE)
    hipLaunchKernelGGL((k_gemm_generic<T, FASTAV_EPI_STORE>), grid, dim3(256), 0, s, (const T*)a, (const T*)w, (const T*)w2, c, ldc, m, n, k);
  else if (epilogue == FASTAV_EPI_RESADD)
    hipLaunchKernelGGL((k_gemm_generic<T, FASTAV_EPI_RESADD>), grid, dim3(256), 0, s, (const T*)a, (const T*)w, (const T*)w2, c, ldc, m, n, k);
  else
    hipLaunchKernelGGL((k_gemm_generic<T, FASTAV_EPI_SWIGLU>), grid, dim3(256), 0, s, (const T*)a, (const T*)w, (const T*)w2, c, ldc, m, n, k);
}

fastav_status_t launch_linear_generic(const void* a, const void* w, const void* w2, void* c, int64_t ldc, int64_t m, int n, int k,
                                      int epilogue, int dtype, hipStream_t s) {
  if (m == 0 || n == 0) return FASTAV_OK;
  if (dtype == FASTAV_BF16) launch_generic_t<bf16_t>(a, w, w2, c, ldc, m, n, k, epilogue, s);
  else launch_generic_t<float>(a, w, w2, c, ldc, m, n, k, epilogue, s);
  return check_launch("linear_generic");
}

}  // namespace fastav
