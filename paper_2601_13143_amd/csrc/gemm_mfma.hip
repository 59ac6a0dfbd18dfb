// bf16 linear layers on the CDNA4 matrix cores: C = A W^T with A [M, K] and W [N, K] both K-contiguous,
// fp32 accumulation in v_mfma_f32_32x32x16_bf16.
//
// Tiling: one workgroup (2 x 4 waves for the 256 x 256 tile, so that two waves share each SIMD and one's
// MFMAs cover the other's LDS and barrier waits; 2 x 2 waves for 128 x 128) owns a BM x BN output tile
// and walks K in steps of 64.  Each
// K-step's A and B panels are fetched from HBM/L2 with 16-byte loads into registers while the previous
// step is being multiplied, then parked in one of two LDS stages (row = 64 bf16 = 128 bytes, 16-byte
// chunks XOR-swizzled with half the row index so that both the row-major stores and the MFMA operand reads
// (32 rows x one chunk) spread over all 64 banks).  A wave multiplies its (BM/WM) x (BN/WN) sub-tile as
// 32 x 32 MFMA blocks.
//
// B rows may come from several matrices: Q|K|V stacked along N (segments), or gate/up for the SwiGLU
// epilogue, where 32-row blocks of the B tile alternate gate, up, gate, up ... so that a lane holds
// gate[r, c] and up[r, c] in matching accumulator registers and silu(g) * u needs no exchange.
//
// Workgroup ids are first re-dealt so that each of the 8 XCDs (ids are dispatched round-robin over them)
// owns a contiguous run of tiles, then walk M fastest: the 32 CUs of an XCD share a few W panels and the
// A panels through their common L2.
#include <cstdlib>

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
  int pf_dist;             // K-steps ahead that lines are pulled into L2 (0 = off)
};

// LDS tile rows are 128 bytes (8 chunks of 16).  The LDS has 64 four-byte banks and serves a 16-byte-per-lane
// access 16 lanes at a time, so 16 consecutive rows reading the same logical chunk must land in 16 different
// 16-byte slots of the 256-byte bank window: two rows share a window, hence the XOR with row/2.
__device__ __forceinline__ int swz(int row, int chunk) { return row * 8 + (chunk ^ ((row >> 1) & 7)); }   // in 16-byte units

// Asynchronous 16-byte global -> LDS copy (no VGPR staging, no ds_write): lane l's data lands at
// lds_base + 16 l, so a wave fills 8 consecutive 128-byte tile rows per instruction; the XOR swizzle is
// applied on the global side (each lane fetches the chunk that belongs in its slot).  Completion is
// tracked by vmcnt; the caller waits with dma_wait() before the barrier that publishes the stage.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_byte_addr) : "memory");
}
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }
// Same path with a 4-byte payload aimed at a scratch corner of LDS: used only to pull a cache line into L2
// a few K-steps before the real copy needs it (no VGPR is written, so nothing has to stay reserved).
__device__ __forceinline__ void l2_touch(const void* gptr, uint32_t lds_scratch_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" : : "v"(gptr), "s"(lds_scratch_addr) : "memory");
}
// All copies of this K-step have landed; the one younger instruction (the L2 touch) may still be in flight.
__device__ __forceinline__ void dma_wait_keep1() { asm volatile("s_waitcnt vmcnt(1)" : : : "memory"); }

template <int BM, int BN, int WM, int WN, int EPI, bool DMA, int SCHED = 0>
__global__ __launch_bounds__(WM * WN * 64) void k_gemm_mfma(GemmArgs g) {
  constexpr int BK = 64;
  constexpr int NT = WM * WN * 64;                     // threads
  constexpr int WTM = BM / WM, WTN = BN / WN;          // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;          // 32x32 blocks per wave
  constexpr int RPP = NT / 8;                          // rows covered by one load pass of the workgroup
  constexpr int A_CH = BM / RPP, B_CH = BN / RPP;      // 16-byte chunks per thread per K-step
  static_assert(RPP % 32 == 0 && TN % 2 == 0, "tile shape");
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
  const int wm = wave / WN, wn = wave % WN;
  const int K = g.K;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int KT = K / BK;
  const int frow = lane & 31, fch = lane >> 5;         // operand fragment: row in block, which 8-wide k chunk

  // B-tile row -> source row pointer (segments for Q|K|V; gate/up interleaved per 32 rows for SwiGLU)
  const bf16_t* wbase = g.W[0];
  int seg_start = 0;
  if (EPI != FASTAV_EPI_SWIGLU) {
    if (n0 >= g.seg_end[0]) { wbase = g.W[1]; seg_start = g.seg_end[0]; }
    if (n0 >= g.seg_end[1]) { wbase = g.W[2]; seg_start = g.seg_end[1]; }
  }
  auto b_row_ptr = [&](int brow) -> const bf16_t* {
    if (EPI == FASTAV_EPI_SWIGLU) {
      const int blk = brow >> 5;
      const bf16_t* wsel = (blk & 1) ? g.W2 : g.W[0];
      return wsel + (int64_t)(n0 + (blk >> 1) * 32 + (brow & 31)) * K;
    }
    return wbase + (int64_t)(n0 - seg_start + brow) * K;
  };
  auto a_row_ptr = [&](int arow) -> const bf16_t* {
    int row = m0 + arow;
    row = row < g.M ? row : g.M - 1;                    // clamp: stay inside A, the epilogue masks the row
    return g.A + (int64_t)row * K;
  };

  // One K-step (4 MFMA k-slices of 16) on LDS stage st.  Operand fragments are double-buffered in
  // registers: the reads of slice kk+1 are issued before the MFMAs of slice kk, so LDS latency hides
  // behind matrix work instead of stalling it.
  auto mma_stage = [&](int st) {
    const bf16x8_t* Asb = As + st * BM * 8;
    const bf16x8_t* Bsb = Bs + st * BN * 8;
    bf16x8_t af[2][TM], bfr[2][TN];
    auto frags = [&](int buf, int kk) {
#pragma unroll
      for (int i = 0; i < TM; ++i) af[buf][i] = Asb[swz(wm * WTM + i * 32 + frow, kk * 2 + fch)];
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[buf][j] = Bsb[swz(wn * WTN + j * 32 + frow, kk * 2 + fch)];
    };
    frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk + 1 < 4) frags((kk + 1) & 1, kk + 1);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
    }
  };

  if constexpr (DMA) {
    // wave `wave` owns tile rows [wave*8 + 8*NW*i, +8) of A and of B for i = 0 .. *_DI-1
    constexpr int NW = WM * WN;
    constexpr int A_DI = BM / (8 * NW), B_DI = BN / (8 * NW);
    const int drow = lane >> 3, dpos = lane & 7;       // row inside the 8-row group, 16-byte slot inside the row
    const bf16_t* a_src[A_DI];
    const bf16_t* b_src[B_DI];
    uint32_t a_dst[A_DI], b_dst[B_DI];                 // LDS byte address of the 8-row group in stage 0
    const uint32_t as_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)As;
    const uint32_t bs_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)Bs;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
    for (int i = 0; i < A_DI; ++i) {
      const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
      a_src[i] = a_row_ptr(row) + ((dpos ^ ((row >> 1) & 7)) * 8);
      a_dst[i] = as_base + (uint32_t)r0 * 128u;
    }
#pragma unroll
    for (int i = 0; i < B_DI; ++i) {
      const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
      b_src[i] = b_row_ptr(row) + ((dpos ^ ((row >> 1) & 7)) * 8);
      b_dst[i] = bs_base + (uint32_t)r0 * 128u;
    }
    auto issue = [&](int kt, int st) {
      const int koff = kt * BK;
#pragma unroll
      for (int i = 0; i < A_DI; ++i) dma16(a_src[i] + koff, a_dst[i] + (uint32_t)st * (BM * 128u));
#pragma unroll
      for (int i = 0; i < B_DI; ++i) dma16(b_src[i] + koff, b_dst[i] + (uint32_t)st * (BN * 128u));
    };
    issue(0, 0);
    dma_wait();
    __syncthreads();
    if constexpr (SCHED == 0) {
      for (int kt = 0; kt < KT; ++kt) {
        const int st = kt & 1;
        if (kt + 1 < KT) issue(kt + 1, st ^ 1);        // stage st^1 was last read before the previous barrier
        mma_stage(st);
        dma_wait();
        __syncthreads();
      }
    } else {
      // Software-pipelined across the barrier: the last k-slice of a stage is multiplied AFTER the barrier
      // that publishes the next stage, while the next stage's first operand reads are already in flight.
      bf16x8_t af[2][TM], bfr[2][TN];
      auto frags = [&](int buf, int st, int kk) {
        const bf16x8_t* Asb = As + st * BM * 8;
        const bf16x8_t* Bsb = Bs + st * BN * 8;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[buf][i] = Asb[swz(wm * WTM + i * 32 + frow, kk * 2 + fch)];
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[buf][j] = Bsb[swz(wn * WTN + j * 32 + frow, kk * 2 + fch)];
        if constexpr (SCHED == 2) __builtin_amdgcn_sched_barrier(0);
      };
      auto mfmas = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bfr[buf][j], acc[i][j], 0, 0, 0);
        if constexpr (SCHED == 2) __builtin_amdgcn_sched_barrier(0);
        if constexpr (SCHED == 3 || SCHED == 4 || SCHED == 5 || SCHED == 6) {
          // interleave: one LDS read between MFMAs
#pragma unroll
          for (int q = 0; q < TM + TN; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 DS read
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
          }
          __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - (TM + TN), 0);
        }
      };
      if constexpr (SCHED == 4) {
        // As above, and the next tile's copies are spread over the K-step (one A and one B instruction per
        // k-slice) instead of being issued in one burst that backs up the memory pipeline.
        static_assert(A_DI == 4 && B_DI == 4, "spread schedule assumes 4 + 4 copies per wave and K-step");
        // Past the last tile the copy is re-aimed at the last tile (into a stage nobody reads any more):
        // keeping the loop body branch-free matters more than the two redundant copies per workgroup.
        auto dma_part = [&](int kt_next, int part) {
          const int koff = (kt_next < KT ? kt_next : KT - 1) * BK, stn = kt_next & 1;
          dma16(a_src[part] + koff, a_dst[part] + (uint32_t)stn * (BM * 128u));
          dma16(b_src[part] + koff, b_dst[part] + (uint32_t)stn * (BN * 128u));
        };
        dma_part(1, 0);
        frags(0, 0, 0);
        for (int kt = 0; kt < KT; ++kt) {
          const int st = kt & 1;
          frags(1, st, 1); dma_part(kt + 1, 1); mfmas(0);
          frags(0, st, 2); dma_part(kt + 1, 2); mfmas(1);
          frags(1, st, 3); dma_part(kt + 1, 3); mfmas(0);
          dma_wait();
          __syncthreads();
          frags(0, st ^ 1, 0);                          // (after the last tile: a harmless read of the idle stage)
          dma_part(kt + 2, 0);                          // stage st is free again after the barrier
          mfmas(1);
        }
        dma_wait();
      } else if constexpr (SCHED == 6 || SCHED == 7) {
        constexpr bool SPREAD = (SCHED == 7);
        // Four LDS stages of 32 k each (same 128 KB): copies run three stages ahead of the math, so a stage
        // has three stage-times to arrive instead of one.  Rows are 64 bytes here (4 chunks): four rows
        // share a 256-byte bank window, hence the XOR with row/4.
        constexpr int NST = 4;
        constexpr int A_D = BM / (16 * NW), B_D = BN / (16 * NW);
        static_assert(A_D >= 1 && B_D >= 1, "tile too small for the 4-stage copy pattern");
        bf16x8_t* A4 = lds;                              // [NST][BM*4]
        bf16x8_t* B4 = lds + NST * BM * 4;               // [NST][BN*4]
        auto swz4 = [](int row, int chunk) { return row * 4 + (chunk ^ ((row >> 2) & 3)); };
        const int drow4 = lane >> 2, dpos4 = lane & 3;
        const bf16_t* a4_src[A_D];
        const bf16_t* b4_src[B_D];
        uint32_t a4_dst[A_D], b4_dst[B_D];
#pragma unroll
        for (int i = 0; i < A_D; ++i) {
          const int r0 = (i * NW + wave_u) * 16, row = r0 + drow4;
          a4_src[i] = a_row_ptr(row) + ((dpos4 ^ ((row >> 2) & 3)) * 8);
          a4_dst[i] = as_base + (uint32_t)r0 * 64u;
        }
        const uint32_t b4_base = as_base + (uint32_t)NST * BM * 64u;
#pragma unroll
        for (int i = 0; i < B_D; ++i) {
          const int r0 = (i * NW + wave_u) * 16, row = r0 + drow4;
          b4_src[i] = b_row_ptr(row) + ((dpos4 ^ ((row >> 2) & 3)) * 8);
          b4_dst[i] = b4_base + (uint32_t)r0 * 64u;
        }
        const int KT4 = K / 32;
        auto issue4 = [&](int t) {
          const int koff = (t < KT4 ? t : KT4 - 1) * 32;   // past the end: a redundant copy into an idle slot
          const uint32_t slot = (uint32_t)(t & 3);
#pragma unroll
          for (int i = 0; i < A_D; ++i) dma16(a4_src[i] + koff, a4_dst[i] + slot * (BM * 64u));
#pragma unroll
          for (int i = 0; i < B_D; ++i) dma16(b4_src[i] + koff, b4_dst[i] + slot * (BN * 64u));
        };
        auto frags4 = [&](int buf, int slot, int kk) {
          const bf16x8_t* Asb = A4 + slot * BM * 4;
          const bf16x8_t* Bsb = B4 + slot * BN * 4;
#pragma unroll
          for (int i = 0; i < TM; ++i) af[buf][i] = Asb[swz4(wm * WTM + i * 32 + frow, kk * 2 + fch)];
#pragma unroll
          for (int j = 0; j < TN; ++j) bfr[buf][j] = Bsb[swz4(wn * WTN + j * 32 + frow, kk * 2 + fch)];
        };
        // waits until at most 2 stages' worth of this wave's copies are still in flight
        auto wait_keep2 = [&]() {
          static_assert(A_D + B_D == 4, "the vmcnt immediate below is 2 * (A_D + B_D)");
          asm volatile("s_waitcnt vmcnt(8)" : : : "memory");
        };
        issue4(0); issue4(1); issue4(2);
        wait_keep2();
        __syncthreads();
        frags4(0, 0, 0);
        if constexpr (SPREAD) {
          // One copy instruction at a time, fenced between halves of a k-slice's MFMAs: a burst of copies
          // at the top of a stage would sit in the memory pipeline's input queue (64 B/clk) and hold up the
          // issuing waves' matrix instructions behind it.
          static_assert(A_D == 2 && B_D == 2 && TM % 2 == 0, "spread schedule: 2 + 2 copies per wave and stage");
          auto mfma_half = [&](int buf, int half) {
#pragma unroll
            for (int i = half * (TM / 2); i < (half + 1) * (TM / 2); ++i)
#pragma unroll
              for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bfr[buf][j], acc[i][j], 0, 0, 0);
          };
          auto dma_one = [&](int t, bool is_b, int i) {
            const int koff = (t < KT4 ? t : KT4 - 1) * 32;
            const uint32_t slot = (uint32_t)(t & 3);
            __builtin_amdgcn_sched_barrier(0);
            if (is_b) dma16(b4_src[i] + koff, b4_dst[i] + slot * (BN * 64u));
            else dma16(a4_src[i] + koff, a4_dst[i] + slot * (BM * 64u));
            __builtin_amdgcn_sched_barrier(0);
          };
          for (int t = 0; t < KT4; ++t) {
            frags4(1, t & 3, 1);
            mfma_half(0, 0); dma_one(t + 3, false, 0);
            mfma_half(0, 1); dma_one(t + 3, true, 0);
            asm volatile("s_waitcnt vmcnt(6)" : : : "memory");   // stage t+1 landed; stage t+2 and two copies of t+3 may fly
            __syncthreads();
            frags4(0, (t + 1) & 3, 0);
            mfma_half(1, 0); dma_one(t + 3, false, 1);
            mfma_half(1, 1); dma_one(t + 3, true, 1);
          }
        } else {
          for (int t = 0; t < KT4; ++t) {
            issue4(t + 3);                               // its slot held stage t-1, free since the last barrier
            frags4(1, t & 3, 1); mfmas(0);
            wait_keep2();                                // stage t+1 has landed (this wave's share)
            __syncthreads();
            frags4(0, (t + 1) & 3, 0);
            mfmas(1);
          }
        }
        dma_wait();
      } else if constexpr (SCHED == 5) {
        // SCHED 3 plus an L2 warm-up: each wave touches 64 cache lines (one per lane) of the tile pf_dist
        // K-steps ahead, so that the real copies one K-step ahead hit L2 instead of paying DRAM latency.
        static_assert(NW == 8 && BM == 256 && BN == 256, "the touch pattern assumes 8 waves on a 256 x 256 tile");
        const uint32_t scratch = bs_base + 2u * BN * 128u;               // 256 bytes past the B stages
        const int prow = (wave_u & 3) * 64 + lane;
        const bf16_t* pf_src = (wave_u < 4) ? a_row_ptr(prow) : b_row_ptr(prow);
        const int pd = g.pf_dist;
        frags(0, 0, 0);
        for (int kt = 0; kt < KT; ++kt) {
          const int st = kt & 1;
          if (kt + 1 < KT) issue(kt + 1, st ^ 1);
          { const int kp = kt + pd; l2_touch(pf_src + (kp < KT ? kp : KT - 1) * BK, scratch); }
          frags(1, st, 1); mfmas(0);
          frags(0, st, 2); mfmas(1);
          frags(1, st, 3); mfmas(0);
          dma_wait_keep1();
          __syncthreads();
          if (kt + 1 < KT) frags(0, st ^ 1, 0);
          mfmas(1);
        }
        dma_wait();
      } else if constexpr (SCHED >= 100) {
        // measurement-only ablations (results are wrong): 101 no copies, 102 no barrier, 103 no operand reads
        frags(0, 0, 0);
        frags(1, 0, 1);
        for (int kt = 0; kt < KT; ++kt) {
          const int st = kt & 1;
          if (SCHED != 101 && kt + 1 < KT) issue(kt + 1, st ^ 1);
          if (SCHED != 103) frags(1, st, 1);
          mfmas(0);
          if (SCHED != 103) frags(0, st, 2);
          mfmas(1);
          if (SCHED != 103) frags(1, st, 3);
          mfmas(0);
          if (SCHED != 102) { dma_wait(); __syncthreads(); }
          if (SCHED != 103 && kt + 1 < KT) frags(0, st ^ 1, 0);
          mfmas(1);
        }
        dma_wait();
      } else {
        frags(0, 0, 0);
        for (int kt = 0; kt < KT; ++kt) {
          const int st = kt & 1;
          if (kt + 1 < KT) issue(kt + 1, st ^ 1);
          frags(1, st, 1); mfmas(0);
          frags(0, st, 2); mfmas(1);
          frags(1, st, 3); mfmas(0);
          dma_wait();
          __syncthreads();
          if (kt + 1 < KT) frags(0, st ^ 1, 0);
          mfmas(1);
        }
      }
    }
  } else {
    const int lr = tid >> 3, lc = tid & 7;             // this thread's row in a load pass and chunk
    const bf16_t* a_src[A_CH];
    const bf16_t* b_src[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) a_src[i] = a_row_ptr(lr + RPP * i) + lc * 8;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) b_src[i] = b_row_ptr(lr + RPP * i) + lc * 8;
    bf16x8_t a_reg[A_CH], b_reg[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) a_reg[i] = *(const bf16x8_t*)(a_src[i]);
#pragma unroll
    for (int i = 0; i < B_CH; ++i) b_reg[i] = *(const bf16x8_t*)(b_src[i]);
#pragma unroll
    for (int i = 0; i < A_CH; ++i) As[swz(lr + RPP * i, lc)] = a_reg[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) Bs[swz(lr + RPP * i, lc)] = b_reg[i];
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
      const int st = kt & 1;
      if (kt + 1 < KT) {
        const int koff = (kt + 1) * BK;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) a_reg[i] = *(const bf16x8_t*)(a_src[i] + koff);
#pragma unroll
        for (int i = 0; i < B_CH; ++i) b_reg[i] = *(const bf16x8_t*)(b_src[i] + koff);
      }
      mma_stage(st);
      if (kt + 1 < KT) {
        bf16x8_t* Asn = As + (st ^ 1) * BM * 8;
        bf16x8_t* Bsn = Bs + (st ^ 1) * BN * 8;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) Asn[swz(lr + RPP * i, lc)] = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) Bsn[swz(lr + RPP * i, lc)] = b_reg[i];
      }
      __syncthreads();
    }
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

template <int BM, int BN, int WM, int WN, int EPI, bool DMA, int SCHED = 0>
static fastav_status_t launch_cfg(GemmArgs& g, hipStream_t s) {
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = g.N / OUT_BN;
  const size_t shmem = (size_t)2 * (BM + BN) * 8 * sizeof(bf16x8_t) + (SCHED == 5 ? 256 : 0);
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)k_gemm_mfma<BM, BN, WM, WN, EPI, DMA, SCHED>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return fail(FASTAV_EHIP, "gemm: hipFuncSetAttribute: %s", hipGetErrorString(e));
  }
  hipLaunchKernelGGL((k_gemm_mfma<BM, BN, WM, WN, EPI, DMA, SCHED>), dim3((unsigned)(g.tiles_m * g.tiles_n)), dim3(WM * WN * 64), shmem, s, g);
  return check_launch("gemm_mfma");
}

template <int EPI>
static fastav_status_t launch_epi(GemmArgs& g, bool big_ok, hipStream_t s) {
  // 256x256 tiles when they still fill the 256 CUs, else 128x128
  const int64_t tiles_big = (int64_t)((g.M + 255) / 256) * (g.N / (EPI == FASTAV_EPI_SWIGLU ? 128 : 256));
  if (big_ok && tiles_big >= 192) {
    static const int variant = getenv("FASTAV_GEMM_VARIANT") ? atoi(getenv("FASTAV_GEMM_VARIANT")) : 0;
    if (variant == 1) return launch_cfg<256, 256, 2, 4, EPI, true, 1>(g, s);
    if (variant == 2) return launch_cfg<256, 256, 2, 4, EPI, true, 2>(g, s);
    if (variant == 3) return launch_cfg<256, 256, 2, 4, EPI, true, 3>(g, s);
    if (variant == 4) return launch_cfg<256, 256, 2, 4, EPI, true, 4>(g, s);
    if (variant == 5) { g.pf_dist = getenv("FASTAV_GEMM_PD") ? atoi(getenv("FASTAV_GEMM_PD")) : 3; return launch_cfg<256, 256, 2, 4, EPI, true, 5>(g, s); }
    if (variant == 6) return launch_cfg<256, 256, 2, 4, EPI, true, 6>(g, s);
    if (variant == 7) return launch_cfg<256, 256, 2, 4, EPI, true, 7>(g, s);
    if (variant == 101) return launch_cfg<256, 256, 2, 4, EPI, true, 101>(g, s);
    if (variant == 102) return launch_cfg<256, 256, 2, 4, EPI, true, 102>(g, s);
    if (variant == 103) return launch_cfg<256, 256, 2, 4, EPI, true, 103>(g, s);
    return launch_cfg<256, 256, 2, 4, EPI, true>(g, s);
  }
  return launch_cfg<128, 128, 2, 2, EPI, false>(g, s);
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
  g.C = c; g.ldc = ldc; g.M = (int)m; g.N = n; g.K = k; g.pf_dist = 0;
  if (((uintptr_t)a | (uintptr_t)w_seg[0]) % 16) return fail(FASTAV_EINVAL, "gemm: A and W must be 16-byte aligned");
  if (epilogue == FASTAV_EPI_STORE) return launch_epi<FASTAV_EPI_STORE>(g, big_ok, s);
  if (epilogue == FASTAV_EPI_RESADD) return launch_epi<FASTAV_EPI_RESADD>(g, big_ok, s);
  return launch_epi<FASTAV_EPI_SWIGLU>(g, big_ok, s);
}

}  // namespace fastav
