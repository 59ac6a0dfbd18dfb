// bf16 linear layers on the CDNA4 matrix cores: C = A W^T with A [M, K] and W [N, K] both K-contiguous,
// fp32 accumulation in v_mfma_f32_32x32x16_bf16.
//
// Tiling: one workgroup of 4 waves (2 x 2) owns a BM x BN output tile and walks K in steps of 64.  Each
// K-step's A and B panels are fetched from HBM/L2 with 16-byte loads into registers while the previous
// step is being multiplied, then parked in one of two LDS stages (row = 64 bf16 = 128 bytes, 16-byte
// chunks XOR-swizzled with the row index so that both the row-major stores and the MFMA operand reads
// (32 rows x one chunk) spread over all banks).  A wave multiplies a (BM/2) x (BN/2) sub-tile as
// 32 x 32 MFMA blocks.
//
// B rows may come from several matrices: Q|K|V stacked along N (segments), or gate/up for the SwiGLU
// epilogue, where 32-row blocks of the B tile alternate gate, up, gate, up ... so that a lane holds
// gate[r, c] and up[r, c] in matching accumulator registers and silu(g) * u needs no exchange.
//
// Workgroup ids are first re-dealt so that each of the 8 XCDs (ids are dispatched round-robin over them)
// owns a contiguous run of tiles, then walk M fastest: the 32 CUs of an XCD share a few W panels and the
// A panels through their common L2.
#include "common.hpp"

namespace fastav {

struct GemmArgs {
  const bf16_t* A;
  const bf16_t* W[3];
  int seg_end[3];          // exclusive end column of each segment
  const bf16_t* W2;        // "up" matrix (SwiGLU only)
  void* C;
  int64_t ldc;
  int M, N, K;             // N = output columns
  int tiles_m, tiles_n;
};

__device__ __forceinline__ int swz(int row, int chunk) { return row * 8 + (chunk ^ (row & 7)); }   // in 16-byte units

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void k_gemm_mfma(GemmArgs g) {
  constexpr int BK = 64;
  constexpr int WTM = BM / 2, WTN = BN / 2;            // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;          // 32x32 blocks per wave
  constexpr int A_CH = BM * 8 / 256, B_CH = BN * 8 / 256;   // 16-byte chunks per thread per K-step
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  extern __shared__ bf16x8_t lds[];
  bf16x8_t* As = lds;                                     // [2][BM*8]
  bf16x8_t* Bs = lds + 2 * BM * 8;                        // [2][BN*8]

  // ---- tile assignment
  const int nblk = g.tiles_m * g.tiles_n;
  int pid = blockIdx.x;
  {
    const int per = nblk / 8, rem = nblk % 8, xcd = pid % 8, idx = pid / 8;
    pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int tile_m = pid % g.tiles_m, tile_n = pid / g.tiles_m;
  const int m0 = tile_m * BM;
  const int n0 = tile_n * OUT_BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int K = g.K;

  // ---- per-thread global source pointers (row clamped to stay inside the matrices)
  const int lr = tid >> 3, lc = tid & 7;               // this thread's row-in-32 and chunk
  const bf16_t* a_src[A_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    int row = m0 + lr + 32 * i;
    row = row < g.M ? row : g.M - 1;
    a_src[i] = g.A + (int64_t)row * K + lc * 8;
  }
  const bf16_t* b_src[B_CH];
  {
    const bf16_t* wbase = g.W[0];
    int seg_start = 0;
    if (EPI != FASTAV_EPI_SWIGLU) {
      if (n0 >= g.seg_end[0]) { wbase = g.W[1]; seg_start = g.seg_end[0]; }
      if (n0 >= g.seg_end[1]) { wbase = g.W[2]; seg_start = g.seg_end[1]; }
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      if (EPI == FASTAV_EPI_SWIGLU) {
        const bf16_t* wsel = (i & 1) ? g.W2 : g.W[0];  // 32-row blocks alternate gate / up
        b_src[i] = wsel + (int64_t)(n0 + (i >> 1) * 32 + lr) * K + lc * 8;
      } else {
        b_src[i] = wbase + (int64_t)(n0 - seg_start + lr + 32 * i) * K + lc * 8;
      }
    }
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8_t a_reg[A_CH], b_reg[B_CH];
  const int KT = K / BK;
#pragma unroll
  for (int i = 0; i < A_CH; ++i) a_reg[i] = *(const bf16x8_t*)(a_src[i]);
#pragma unroll
  for (int i = 0; i < B_CH; ++i) b_reg[i] = *(const bf16x8_t*)(b_src[i]);
#pragma unroll
  for (int i = 0; i < A_CH; ++i) As[swz(lr + 32 * i, lc)] = a_reg[i];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) Bs[swz(lr + 32 * i, lc)] = b_reg[i];
  __syncthreads();

  const int frow = lane & 31, fch = lane >> 5;         // operand fragment: row in block, which 8-wide k chunk
  for (int kt = 0; kt < KT; ++kt) {
    const int st = kt & 1;
    if (kt + 1 < KT) {
      const int koff = (kt + 1) * BK;
#pragma unroll
      for (int i = 0; i < A_CH; ++i) a_reg[i] = *(const bf16x8_t*)(a_src[i] + koff);
#pragma unroll
      for (int i = 0; i < B_CH; ++i) b_reg[i] = *(const bf16x8_t*)(b_src[i] + koff);
    }
    const bf16x8_t* Asb = As + st * BM * 8;
    const bf16x8_t* Bsb = Bs + st * BN * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8_t af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        af[i] = Asb[swz(wm * WTM + i * 32 + frow, kk * 2 + fch)];
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        bfr[j] = Bsb[swz(wn * WTN + j * 32 + frow, kk * 2 + fch)];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      bf16x8_t* Asn = As + (st ^ 1) * BM * 8;
      bf16x8_t* Bsn = Bs + (st ^ 1) * BN * 8;
#pragma unroll
      for (int i = 0; i < A_CH; ++i) Asn[swz(lr + 32 * i, lc)] = a_reg[i];
#pragma unroll
      for (int i = 0; i < B_CH; ++i) Bsn[swz(lr + 32 * i, lc)] = b_reg[i];
    }
    __syncthreads();
  }

  // ---- epilogue.  Accumulator register r of a 32x32 block: column = lane % 32,
  //      row = (r / 4) * 8 + (lane / 32) * 4 + r % 4.
  const int ecol = lane & 31, erow0 = (lane >> 5) * 4;
  if (EPI == FASTAV_EPI_SWIGLU) {
    bf16_t* C = (bf16_t*)g.C;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; j += 2) {
        const int col = n0 + (wn * TN / 2 + j / 2) * 32 + ecol;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm * WTM + i * 32 + (r >> 2) * 8 + erow0 + (r & 3);
          if (row < g.M) {
            const float gt = acc[i][j][r], up = acc[i][j + 1][r];
            C[(int64_t)row * g.ldc + col] = (bf16_t)(gt / (1.0f + __expf(-gt)) * up);
          }
        }
      }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * WTN + j * 32 + ecol;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm * WTM + i * 32 + (r >> 2) * 8 + erow0 + (r & 3);
          if (row < g.M) {
            if (EPI == FASTAV_EPI_STORE) ((bf16_t*)g.C)[(int64_t)row * g.ldc + col] = (bf16_t)acc[i][j][r];
            else ((float*)g.C)[(int64_t)row * g.ldc + col] += acc[i][j][r];
          }
        }
      }
  }
}

bool mfma_linear_supported(int64_t m, int n, int k, int epilogue, int dtype) {
  if (dtype != FASTAV_BF16 || m < 1 || m > 0x7FFFFFFF) return false;
  if (k % 64 != 0 || k < 64) return false;
  return epilogue == FASTAV_EPI_SWIGLU ? (n % 64 == 0) : (n % 128 == 0);
}

template <int BM, int BN, int EPI>
static fastav_status_t launch_cfg(GemmArgs& g, hipStream_t s) {
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = g.N / OUT_BN;
  const size_t shmem = (size_t)2 * (BM + BN) * 8 * sizeof(bf16x8_t);
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)k_gemm_mfma<BM, BN, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return fail(FASTAV_EHIP, "gemm: hipFuncSetAttribute: %s", hipGetErrorString(e));
  }
  hipLaunchKernelGGL((k_gemm_mfma<BM, BN, EPI>), dim3((unsigned)(g.tiles_m * g.tiles_n)), dim3(256), shmem, s, g);
  return check_launch("gemm_mfma");
}

template <int EPI>
static fastav_status_t launch_epi(GemmArgs& g, bool big_ok, hipStream_t s) {
  // 256x256 tiles when they still fill the 256 CUs, else 128x128
  const int64_t tiles_big = (int64_t)((g.M + 255) / 256) * (g.N / (EPI == FASTAV_EPI_SWIGLU ? 128 : 256));
  if (big_ok && tiles_big >= 192) return launch_cfg<256, 256, EPI>(g, s);
  return launch_cfg<128, 128, EPI>(g, s);
}

fastav_status_t launch_linear_mfma(const void* a, const void* const* w_seg, const int* seg_rows, int n_seg,
                                   const void* w2, void* c, int64_t ldc, int64_t m, int n, int k, int epilogue,
                                   hipStream_t s) {
  GemmArgs g;
  g.A = (const bf16_t*)a;
  int end = 0;
  bool big_ok = true;
  for (int i = 0; i < 3; ++i) {
    if (i < n_seg) {
      end += seg_rows[i];
      g.W[i] = (const bf16_t*)w_seg[i];
      if (seg_rows[i] % (epilogue == FASTAV_EPI_SWIGLU ? 128 : 256)) big_ok = false;
    } else {
      g.W[i] = g.W[0];
    }
    g.seg_end[i] = i < n_seg ? end : 0x7FFFFFFF;
  }
  g.W2 = (const bf16_t*)w2;
  g.C = c; g.ldc = ldc; g.M = (int)m; g.N = n; g.K = k;
  if (((uintptr_t)a | (uintptr_t)w_seg[0]) % 16) return fail(FASTAV_EINVAL, "gemm: A and W must be 16-byte aligned");
  if (epilogue == FASTAV_EPI_STORE) return launch_epi<FASTAV_EPI_STORE>(g, big_ok, s);
  if (epilogue == FASTAV_EPI_RESADD) return launch_epi<FASTAV_EPI_RESADD>(g, big_ok, s);
  return launch_epi<FASTAV_EPI_SWIGLU>(g, big_ok, s);
}

}  // namespace fastav
