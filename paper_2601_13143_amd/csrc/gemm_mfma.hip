// bf16 linear layers on the CDNA4 matrix cores: C = A W^T with A [M, K] and W [N, K] both K-contiguous,
// fp32 accumulation in v_mfma_f32_32x32x16_bf16.
//
// One workgroup owns a BM x BN output tile; its WM x WN waves each multiply a (BM/WM) x (BN/WN) sub-tile as
// 32 x 32 MFMA blocks.  K is walked in stages of 32.  The operands of a stage travel HBM/L2 -> LDS with
// asynchronous 16-byte copies (global_load_lds_dwordx4: no VGPR staging, no ds_write) into a ring of four
// LDS stages, three stages ahead of the math.  The copies are issued one at a time between groups of MFMAs:
// the memory pipeline takes 64 B/clk per CU, and a burst of copies would queue up in front of the issuing
// waves' matrix instructions.  The last k-slice of a stage is multiplied after the barrier that publishes
// the next stage, while that stage's first operand reads are already in flight.
//
// LDS layout: a stage holds BM + BN rows of 32 bf16 = 64 bytes (4 chunks of 16).  The LDS has 64 four-byte
// banks and serves a 16-byte-per-lane read 16 lanes at a time, so the 16 rows an MFMA operand read touches
// (same logical chunk) must fall in 16 distinct 16-byte slots of the 256-byte bank window: four rows share
// a window, hence chunk ^ (row/4 & 3).  A copy instruction lands lane l at base + 16 l, i.e. it fills 16
// consecutive rows; the swizzle is applied on the global side (a lane fetches the chunk that belongs in
// its slot).
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
  int band;                // tile columns per band of the tile order (1 = column-major)
  int n_off;               // first output column of this launch (a launch may cover a range of tile columns)
  int splits;              // split-K: blockIdx.y picks a K range and writes an fp32 partial tile to `partial`
  float* partial;          // [splits][M][N] fp32 (split-K only)
  int vec_ok;              // the output (C, or `partial`) takes 16-byte accesses: base and row pitch are multiples of 16 bytes
};

constexpr int kNumCUs = 256;
constexpr int kEpiPartial = 100;   // internal epilogue: plain fp32 store of a split-K partial
constexpr int kEpiResAtomic = 101; // internal epilogue: residual update through fire-and-forget hardware adds

// Asynchronous 16-byte global -> LDS copy; lane l's data lands at lds_byte_addr + 16 l.  Completion is
// tracked by vmcnt (copies complete in issue order).
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_byte_addr) : "memory");
}
// The same with the address split into a wave-uniform base (SGPR pair) and a 32-bit lane offset: no vector
// arithmetic per copy.
__device__ __forceinline__ void dma16_sbase(const void* base, uint32_t voff, uint32_t lds_byte_addr) {
  // the base is wave-uniform by contract; say so, or the register allocator may leave it in VGPRs
  const uint64_t u = (uint64_t)(uintptr_t)base;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  const void* sbase = (const void*)(uintptr_t)(((uint64_t)hi << 32) | lo);
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(sbase), "s"(lds_byte_addr) : "memory");
}
// The same copy as a buffer load: a 128-bit resource (base, no stride, no bounds of interest) in SGPRs, a 32-bit
// lane offset and a scalar byte offset that advances along K.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t make_rsrc(const void* base) {
  const uint64_t u = (uint64_t)(uintptr_t)base;
  u32x4_t r;
  r[0] = __builtin_amdgcn_readfirstlane((uint32_t)u);
  r[1] = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32) & 0xFFFFu);
  r[2] = 0xFFFFFFFFu;                                  // num_records: the whole address range after base
  r[3] = 0x00020000u;                                  // raw buffer, 32-bit data format
  return r;
}
__device__ __forceinline__ void dma16_buf(u32x4_t rsrc, uint32_t voff, uint32_t soff, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %3\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(voff), "s"(rsrc), "s"(soff), "s"(lds_byte_addr) : "memory");
}
template <int N> __device__ __forceinline__ void dma_wait_keep() {   // until at most N copies are in flight
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

__device__ __forceinline__ int swz4(int row, int chunk) { return row * 4 + (chunk ^ ((row >> 2) & 3)); }   // 16-byte units

// Epilogue shared by the GEMM kernels.  The main loops compute the transposed product (weight fragment as the
// first MFMA operand), so accumulator register r of a 32x32 block holds row = lane % 32 and
// column = (r / 4) * 8 + (lane / 32) * 4 + r % 4: four consecutive columns of one row per register quad.  fp32
// outputs go out as 16-byte accesses; bf16 outputs first trade quads between lanes l and l + 32 so that every lane
// owns eight consecutive columns (16 bytes).  Only the hardware-add epilogue keeps the untransposed product (row
// quads per lane, one column): its adds are issued element by element and want the 32 lanes on one line.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2_t t = {(bf16_t)a, (bf16_t)b};
  return __builtin_bit_cast(uint32_t, t);
}
constexpr bool gemm_transposed(int epi) { return epi != kEpiResAtomic; }

// One 32x32 block (SwiGLU: the gate block `b0` and the up block `b1` of one output block) of a wave's tile.
// row0 / col0: the block's first output row / column.
template <int EPI>
__device__ __forceinline__ void gemm_epilogue_block(const GemmArgs& g, const f32x16_t& b0, const f32x16_t& b1, int row0, int col0, int lane) {
  if constexpr (EPI == kEpiResAtomic) {
    const int col = col0 + (lane & 31), erow0 = row0 + (lane >> 5) * 4;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = erow0 + (r >> 2) * 8 + (r & 3);
      // Residual update as a fire-and-forget hardware add at the L2: no read round trip holds the
      // wave, so the main loop that follows on this CU overlaps the drain.  Each element receives
      // exactly one addend per launch, so the result is that of a read-modify-write.
      if (row < g.M) unsafeAtomicAdd(&((float*)g.C)[(int64_t)row * g.ldc + col], b0[r]);
    }
  } else {
    const int row = row0 + (lane & 31), hf = lane >> 5;
    const bool ok = row < g.M;
    const bool vec = g.vec_ok != 0;
    float v[16];                                         // v[4q + e]: column 8q + 4 hf + e of the block
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if constexpr (EPI == FASTAV_EPI_SWIGLU) v[r] = b0[r] / (1.0f + __expf(-b0[r])) * b1[r];
      else v[r] = b0[r];
    }
    if constexpr (EPI == FASTAV_EPI_STORE || EPI == FASTAV_EPI_SWIGLU) {
      bf16_t* C = (bf16_t*)g.C + (int64_t)row * g.ldc + col0;
      if (vec) {
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {                 // quads (2 pr, 2 pr + 1): columns 16 pr .. 16 pr + 15
          const uint32_t x0 = pack_bf16(v[8 * pr + 0], v[8 * pr + 1]), x1 = pack_bf16(v[8 * pr + 2], v[8 * pr + 3]);
          const uint32_t y0 = pack_bf16(v[8 * pr + 4], v[8 * pr + 5]), y1 = pack_bf16(v[8 * pr + 6], v[8 * pr + 7]);
          // upper half of x <-> lower half of y: lanes 0-31 end up with columns 0-7, lanes 32-63 with 8-15
          const auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
          const auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
          const u32x4_t out = {s0[0], s1[0], s0[1], s1[1]};
          if (ok) *(u32x4_t*)(C + pr * 16 + hf * 8) = out;
        }
      } else if (ok) {
#pragma unroll
        for (int r = 0; r < 16; ++r) C[(r >> 2) * 8 + hf * 4 + (r & 3)] = (bf16_t)v[r];
      }
    } else {
      float* C = (EPI == kEpiPartial) ? g.partial + ((int64_t)blockIdx.y * g.M + row) * g.N + col0 + hf * 4
                                      : (float*)g.C + (int64_t)row * g.ldc + col0 + hf * 4;
      if (ok) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (vec) {
            f32x4_t t = {v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
            if constexpr (EPI == FASTAV_EPI_RESADD) {
              const f32x4_t o = *(const f32x4_t*)(C + 8 * q);
              t[0] += o[0]; t[1] += o[1]; t[2] += o[2]; t[3] += o[3];
            }
            *(f32x4_t*)(C + 8 * q) = t;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if constexpr (EPI == FASTAV_EPI_RESADD) C[8 * q + e] += v[4 * q + e];
              else C[8 * q + e] = v[4 * q + e];
            }
          }
        }
      }
    }
  }
}

// Epilogue of a wave's tile.  `stage` is LDS the wave may use as it likes (the caller has made sure that no copy
// is still in flight and no other wave reads it): 2 x 32 rows of the wave's output width in bf16.  An aligned bf16
// output goes through it - the lanes' 16-byte pieces are laid down row by row and read back so that a store
// instruction covers whole rows of the wave's tile (full 128-byte lines, a quarter of the L2 write requests of
// storing the pieces as the accumulators hold them).
template <int EPI, int TM, int TN, int WTM, int WTN, bool USE_F32_STAGE = true>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, f32x16_t (&acc)[TM][TN], int m0, int n0, int wm, int wn, int lane,
                                              bf16x8_t* stage) {
  constexpr int JS = (EPI == FASTAV_EPI_SWIGLU) ? 2 : 1;
  constexpr int NB = TN / JS;                            // output blocks per block row
  constexpr int NCHK = NB * 4;                           // 16-byte chunks per output row of the wave
  constexpr int RPI = 64 / NCHK;                         // rows a 64-lane access covers
  if constexpr (EPI == FASTAV_EPI_STORE || EPI == FASTAV_EPI_SWIGLU) {
    // (measured: worth 1.5-3 % for the plain store; the gate/up output is half as wide and comes out 1 % slower
    // this way than with the pieces stored directly, so it keeps the direct path)
    if (EPI == FASTAV_EPI_STORE && g.vec_ok) {
      static_assert(NCHK == 4 || NCHK == 8 || NCHK == 16, "wave tile width");
      constexpr int SWM = NCHK >= 8 ? 7 : NCHK - 1;          // chunk swizzle: spreads a column of pieces over the banks
      const int m = lane & 31, hf = lane >> 5;
      const int rr = lane / NCHK, cc = lane % NCHK;
      const int colw = (EPI == FASTAV_EPI_SWIGLU) ? n0 + wn * (WTN / 2) : n0 + wn * WTN;
      bf16_t* C = (bf16_t*)g.C + colw + cc * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        bf16x8_t* st = stage + (i & 1) * 32 * NCHK;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
          float v[16];                                   // v[4q + e]: column 8q + 4 hf + e of the block
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            if constexpr (EPI == FASTAV_EPI_SWIGLU) {
              const float gt = acc[i][2 * jb][r], up = acc[i][2 * jb + 1][r];
              v[r] = gt / (1.0f + __expf(-gt)) * up;
            } else {
              v[r] = acc[i][jb][r];
            }
          }
#pragma unroll
          for (int pr = 0; pr < 2; ++pr) {               // quads (2 pr, 2 pr + 1): columns 16 pr .. 16 pr + 15
            const uint32_t x0 = pack_bf16(v[8 * pr + 0], v[8 * pr + 1]), x1 = pack_bf16(v[8 * pr + 2], v[8 * pr + 3]);
            const uint32_t y0 = pack_bf16(v[8 * pr + 4], v[8 * pr + 5]), y1 = pack_bf16(v[8 * pr + 6], v[8 * pr + 7]);
            // upper half of x <-> lower half of y: lanes 0-31 end up with columns 0-7, lanes 32-63 with 8-15
            const auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
            const auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
            const u32x4_t out = {s0[0], s1[0], s0[1], s1[1]};
            const int c = jb * 4 + pr * 2 + hf;
            *(u32x4_t*)&st[m * NCHK + (c ^ (m & SWM))] = out;
          }
        }
        // the wave's own LDS accesses execute in order: no wait between the writes above and the reads below
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
          const int r = it * RPI + rr;
          const u32x4_t val = *(const u32x4_t*)&st[r * NCHK + (cc ^ (r & SWM))];
          const int row = m0 + wm * WTM + i * 32 + r;
          if (row < g.M) *(u32x4_t*)(C + (int64_t)row * g.ldc) = val;
        }
      }
      return;
    }
  }
  if constexpr (EPI == FASTAV_EPI_RESADD || EPI == kEpiPartial) {
    // fp32 outputs the same way: 16-byte pieces of four columns, 8 TN of them per output row of the wave
    if (g.vec_ok && USE_F32_STAGE) {
      constexpr int NC = TN * 8, RP = 64 / NC;           // chunks per row, rows per 64-lane access
      static_assert(NC == 16 || NC == 32, "wave tile width");
      const int m = lane & 31, hf = lane >> 5;
      const int rr = lane / NC, cc = lane % NC;
      float* C = (EPI == kEpiPartial) ? g.partial + (int64_t)blockIdx.y * g.M * g.N + n0 + wn * WTN + cc * 4
                                      : (float*)g.C + n0 + wn * WTN + cc * 4;
      const int64_t pitch = (EPI == kEpiPartial) ? g.N : g.ldc;
      f32x4_t* stf = (f32x4_t*)stage;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        f32x4_t* st = stf + (i & 1) * 32 * NC;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4_t t = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            const int c = j * 8 + q * 2 + hf;
            st[m * NC + (c ^ (m & 7))] = t;
          }
        f32x4_t old[32 / RP];
        if constexpr (EPI == FASTAV_EPI_RESADD) {
#pragma unroll
          for (int it = 0; it < 32 / RP; ++it) {
            const int row = m0 + wm * WTM + i * 32 + it * RP + rr;
            old[it] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            if (row < g.M) old[it] = *(const f32x4_t*)(C + (int64_t)row * pitch);
          }
        }
#pragma unroll
        for (int it = 0; it < 32 / RP; ++it) {
          const int r = it * RP + rr;
          f32x4_t val = st[r * NC + (cc ^ (r & 7))];
          if constexpr (EPI == FASTAV_EPI_RESADD) { val[0] += old[it][0]; val[1] += old[it][1]; val[2] += old[it][2]; val[3] += old[it][3]; }
          const int row = m0 + wm * WTM + i * 32 + r;
          if (row < g.M) *(f32x4_t*)(C + (int64_t)row * pitch) = val;
        }
      }
      return;
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; j += JS) {
      const int col0 = (EPI == FASTAV_EPI_SWIGLU) ? n0 + (wn * TN / 2 + j / 2) * 32 : n0 + wn * WTN + j * 32;
      gemm_epilogue_block<EPI>(g, acc[i][j], acc[i][JS == 2 ? j + 1 : j], m0 + wm * WTM + i * 32, col0, lane);
    }
}

// NST = LDS ring depth in stages of 32 k (copies run NST-1 stages ahead).  A 256 x 128 tile with 4 waves and
// NST = 3 lets two workgroups share a CU (one computes while the other sits in its prologue, epilogue or at a
// barrier); it measured 15 % slower than one 8-wave 256 x 256 workgroup with NST = 4 on every shape of the 7B
// model (half again as many copy bytes per flop, copies only two stages ahead), so nothing launches it.
template <int BM, int BN, int WM, int WN, int EPI, int NST = 4>
__global__ __launch_bounds__(WM * WN * 64, (WM * WN == 4 && NST == 3) ? 2 : 1) void k_gemm_mfma(GemmArgs g) {
  constexpr int NW = WM * WN;                          // waves
  constexpr int WTM = BM / WM, WTN = BN / WN;          // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;          // 32x32 blocks per wave
  constexpr int A_D = BM / (16 * NW), B_D = BN / (16 * NW);   // copy instructions per wave and stage
  constexpr int D = A_D + B_D;
  constexpr int NMF = TM * TN;                         // MFMAs per k-slice
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  static_assert(A_D >= 1 && B_D >= 1 && D % 2 == 0 && NMF >= D / 2 && TN % 2 == 0 && NST >= 3, "tile shape");
  extern __shared__ bf16x8_t lds[];
  bf16x8_t* A4 = lds;                                  // [NST][BM*4]
  bf16x8_t* B4 = lds + NST * BM * 4;                   // [NST][BN*4]

  // ---- tile assignment
  const int nblk = g.tiles_m * g.tiles_n;
  int pid = blockIdx.x;
  {
    const int per = nblk / 8, rem = nblk % 8, xcd = pid % 8, idx = pid / 8;
    pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  // Tile order: bands of `band` tile columns, swept row by row.  With several rounds of tiles per launch the
  // ~32 tiles an XCD works on at one time then form a block of about 8 x 4 tiles instead of 2 whole columns,
  // which cuts the operand panels it streams through its L2 per round by a third or more.  A launch of a
  // single round keeps whole columns (band = 1), which measured faster there.
  const int kb = g.band;
  const int band = pid / (kb * g.tiles_m);
  const int bw = (g.tiles_n - band * kb < kb) ? g.tiles_n - band * kb : kb;   // columns in this band
  const int inb = pid - band * kb * g.tiles_m;
  const int tile_m = inb / bw, tile_n = band * kb + inb % bw;
  const int m0 = tile_m * BM;
  const int n0 = g.n_off + tile_n * OUT_BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave / WN, wn = wave % WN;
  const int K = g.K;
  // stages of 32 k owned by this workgroup (all of them unless split-K)
  const int kt_all = K / 32;
  const int kt0 = (int)((int64_t)kt_all * blockIdx.y / g.splits);
  const int KT = (int)((int64_t)kt_all * (blockIdx.y + 1) / g.splits) - kt0;

  // B-tile row -> source row (segments for Q|K|V; gate/up interleaved per 32 rows for SwiGLU)
  const bf16_t* wbase = g.W[0];
  int seg_start = 0;
  if (EPI != FASTAV_EPI_SWIGLU) {
    if (n0 >= g.seg_end[0]) { wbase = g.W[1]; seg_start = g.seg_end[0]; }
    if (n0 >= g.seg_end[1]) { wbase = g.W[2]; seg_start = g.seg_end[1]; }
  }

  // ---- this wave's copies: instruction i covers tile rows [(i*NW + wave)*16, +16).  The vector ALU also issues
  // the matrix instructions, so the main loop is written to need none: a copy's address is a wave-uniform base in
  // SGPRs (advanced along K with scalar adds) plus one constant 32-bit lane offset, and an operand fragment's LDS
  // address is one constant lane offset plus an immediate (the ring slot is a compile-time constant: the stage
  // loop is unrolled over the ring).
  const int drow = lane >> 2, dpos = lane & 3;          // row inside the 16-row group, 16-byte slot inside the row
  const bf16_t* a_sb = g.A + (int64_t)m0 * K + kt0 * 32;
  const bf16_t* b_sb[B_D];
  uint32_t a_vo[A_D], b_vo[B_D];                        // lane offsets in bytes (at most 255 rows of K elements)
  uint32_t a_dst[A_D], b_dst[B_D];                      // LDS byte address of the 16-row group in stage 0
  const uint32_t a_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)A4;
  const uint32_t b_base = a_base + (uint32_t)NST * BM * 64u;
#pragma unroll
  for (int i = 0; i < A_D; ++i) {
    const int r0 = (i * NW + wave_u) * 16, row = r0 + drow;
    int grow = m0 + row;
    grow = grow < g.M ? grow : g.M - 1;                 // clamp: stay inside A, the epilogue masks the row
    a_vo[i] = (uint32_t)(((int64_t)(grow - m0) * K + (dpos ^ ((row >> 2) & 3)) * 8) * 2);
    a_dst[i] = a_base + (uint32_t)r0 * 64u;
  }
#pragma unroll
  for (int i = 0; i < B_D; ++i) {
    const int r0 = (i * NW + wave_u) * 16, row = r0 + drow;
    if (EPI == FASTAV_EPI_SWIGLU) {
      const int blk = r0 >> 5;                          // the 16 rows of a copy lie inside one 32-row block
      b_sb[i] = ((blk & 1) ? g.W2 : g.W[0]) + (int64_t)(n0 + (blk >> 1) * 32) * K + kt0 * 32;
      b_vo[i] = (uint32_t)(((int64_t)(row & 31) * K + (dpos ^ ((row >> 2) & 3)) * 8) * 2);
    } else {
      b_sb[i] = wbase + (int64_t)(n0 - seg_start) * K + kt0 * 32;
      b_vo[i] = (uint32_t)(((int64_t)row * K + (dpos ^ ((row >> 2) & 3)) * 8) * 2);
    }
    b_dst[i] = b_base + (uint32_t)r0 * 64u;
  }
  // copy number c (0 .. D-1: A's first) of stage t into ring slot dslot.  Past the last stage the copy is re-aimed
  // at the last stage (into a ring slot nobody reads any more): a branch-free loop body matters more than the few
  // redundant copies per workgroup.
  auto dma_one = [&](int t, int c, uint32_t dslot) __attribute__((always_inline)) {
    const int koff = (t < KT ? t : KT - 1) * 32;
    if (c < A_D) dma16_sbase(a_sb + koff, a_vo[c < A_D ? c : 0], a_dst[c < A_D ? c : 0] + dslot * (BM * 64u));
    else dma16_sbase(b_sb[c >= A_D ? c - A_D : 0] + koff, b_vo[c >= A_D ? c - A_D : 0], b_dst[c >= A_D ? c - A_D : 0] + dslot * (BN * 64u));
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frow = lane & 31, fch = lane >> 5;          // operand fragment: row in block, which 8-wide k chunk
  bf16x8_t af[2][TM], bfr[2][TN];                       // operand fragments of two k-slices
  // this lane's fragment positions inside a ring slot (16-byte units) for the two k-halves of a stage; block i of
  // the wave tile adds 32 rows = 128 units (the swizzle term depends on row bits 2-3 only)
  int a_fu[2], b_fu[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    a_fu[kk] = swz4(wm * WTM + frow, kk * 2 + fch);
    b_fu[kk] = NST * BM * 4 + swz4(wn * WTN + frow, kk * 2 + fch);
  }
  // One k-slice: NMF MFMAs in D/2 groups, one copy of stage t_copy fenced in after each group.  The operand
  // fragments of the NEXT k-slice (ring slot nslot, half nkk) are read into the other register buffer one at a
  // time, each right after an MFMA of this slice: the LDS reads are spread evenly over the slice instead of
  // arriving in a burst, and a wave never stands between its reads and its first MFMA.
  auto slice = [&](int buf, int t_copy, int c0, uint32_t dslot, uint32_t nslot, int nkk) __attribute__((always_inline)) {
#pragma unroll
    for (int grp = 0; grp < D / 2; ++grp) {
#pragma unroll
      for (int q = grp * NMF / (D / 2); q < (grp + 1) * NMF / (D / 2); ++q) {     // MFMAs between two copies
        const int i = q / TN, j = q % TN;
        acc[i][j] = gemm_transposed(EPI) ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[buf][j], af[buf][i], acc[i][j], 0, 0, 0)
                                         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bfr[buf][j], acc[i][j], 0, 0, 0);
        if (q < TM) af[buf ^ 1][q] = lds[a_fu[nkk] + (int)nslot * BM * 4 + q * 128];
        else if (q < TM + TN) bfr[buf ^ 1][q - TM] = lds[b_fu[nkk] + (int)nslot * BN * 4 + (q - TM) * 128];
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // one MFMA ...
        if (q < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);       // ... then one LDS read
      }
      __builtin_amdgcn_sched_barrier(0);
      dma_one(t_copy, c0 + grp, dslot);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  static_assert(NMF >= TM + TN, "a slice has fewer MFMAs than the next slice has fragments");
  // stage t lives in ring slot `slot`; the copies issued meanwhile (stage t+NST-1) go to the slot before it
  auto stage = [&](int t, uint32_t slot) __attribute__((always_inline)) {
    const uint32_t dslot = (slot + NST - 1) % NST, nslot = (slot + 1) % NST;
    // the ring slot of stage t+NST-1 held stage t-1, which nobody reads after the previous barrier
    slice(0, t + NST - 1, 0, dslot, slot, 1);
    dma_wait_keep<(NST - 3) * D + D / 2>();              // stage t+1 has landed (this wave's share)
    __syncthreads();
    slice(1, t + NST - 1, D / 2, dslot, nslot, 0);       // (after the last stage: a harmless read of an idle slot)
  };

  // ---- prologue: NST-1 stages in flight, the first one landed and published
#pragma unroll
  for (int t = 0; t < NST - 1; ++t)
#pragma unroll
    for (int c = 0; c < D; ++c) dma_one(t, c, (uint32_t)t);
  dma_wait_keep<(NST - 2) * D>();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i) af[0][i] = lds[a_fu[0] + i * 128];
#pragma unroll
  for (int j = 0; j < TN; ++j) bfr[0][j] = lds[b_fu[0] + j * 128];

  int t = 0;
  for (; t + NST <= KT; t += NST) {                      // t is a multiple of NST here: slots are literals
#pragma unroll
    for (int u = 0; u < NST; ++u) stage(t + u, (uint32_t)u);
  }
  for (; t < KT; ++t) stage(t, (uint32_t)t % (uint32_t)NST);
  dma_wait_keep<0>();

  __syncthreads();                                     // every wave's copies have landed: LDS is free for the epilogue
  gemm_epilogue<EPI, TM, TN, WTM, WTN>(g, acc, m0, n0, wm, wn, lane,
                                       lds + wave * (2 * 32 * 8 * TN));
}

// The same GEMM with stages of 64 k in a double buffer.  What changes is the shape of a copy: a wave instruction
// now reads 8 rows x 128 contiguous bytes (whole L2 lines) instead of 16 rows x 64, half as many address segments
// per byte - the vector-memory path, not the matrix cores, is what the 32-k kernel runs out of first.  A stage is
// (BM + BN) x 128 bytes, so only two fit in LDS; the copies of stage t+2 start as soon as the last fragments of
// stage t have been read (one barrier per stage, placed before the stage's last k-slice) and have a full stage of
// matrix work to land.  LDS row = 8 chunks of 16 bytes, chunk c of row r stored at position c ^ ((r >> 1) & 7):
// the 16 lanes of a fragment read then hit 16 different bank groups.
__device__ __forceinline__ int swz8(int row, int chunk) { return row * 8 + (chunk ^ ((row >> 1) & 7)); }   // 16-byte units

template <int BM, int BN, int WM, int WN, int EPI, int LATE = 0>
__global__ __launch_bounds__(WM * WN * 64, (BM + BN) * 256 <= 80 * 1024 ? 2 : 1) void k_gemm_mfma_k64(GemmArgs g) {
  constexpr int NW = WM * WN;                          // waves
  constexpr int WTM = BM / WM, WTN = BN / WN;          // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;          // 32x32 blocks per wave
  constexpr int A_D = BM / (8 * NW), B_D = BN / (8 * NW);     // copy instructions per wave and stage (8 rows each)
  constexpr int D = A_D + B_D;
  constexpr int NMF = TM * TN;                         // MFMAs per k-slice
  constexpr int KS = 4;                                // k-slices of 16 per stage
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  static_assert(A_D >= 1 && B_D >= 1 && D % 2 == 0 && NMF >= D / 2 && NMF >= TM + TN && TN % 2 == 0, "tile shape");
  extern __shared__ bf16x8_t lds[];                    // [2][BM*8] A, then [2][BN*8] B

  // ---- tile assignment (as in k_gemm_mfma)
  const int nblk = g.tiles_m * g.tiles_n;
  int pid = blockIdx.x;
  {
    const int per = nblk / 8, rem = nblk % 8, xcd = pid % 8, idx = pid / 8;
    pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int kb = g.band;
  const int band = pid / (kb * g.tiles_m);
  const int bw = (g.tiles_n - band * kb < kb) ? g.tiles_n - band * kb : kb;   // columns in this band
  const int inb = pid - band * kb * g.tiles_m;
  const int tile_m = inb / bw, tile_n = band * kb + inb % bw;
  const int m0 = tile_m * BM;
  const int n0 = g.n_off + tile_n * OUT_BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave / WN, wn = wave % WN;
  const int K = g.K;
  // stages of 64 k owned by this workgroup (all of them unless split-K)
  const int kt_all = K / 64;
  const int kt0 = (int)((int64_t)kt_all * blockIdx.y / g.splits);
  const int KT = (int)((int64_t)kt_all * (blockIdx.y + 1) / g.splits) - kt0;

  const bf16_t* wbase = g.W[0];
  int seg_start = 0;
  if (EPI != FASTAV_EPI_SWIGLU) {
    if (n0 >= g.seg_end[0]) { wbase = g.W[1]; seg_start = g.seg_end[0]; }
    if (n0 >= g.seg_end[1]) { wbase = g.W[2]; seg_start = g.seg_end[1]; }
  }

  // ---- this wave's copies: instruction i covers tile rows [(i*NW + wave)*8, +8), lane = (row, 16-byte chunk)
  const int drow = lane >> 3, dpos = lane & 7;
  const bf16_t* a_sb = g.A + (int64_t)m0 * K + kt0 * 64;
  const bf16_t* b_sb[B_D];
  uint32_t a_vo[A_D], b_vo[B_D];                        // lane offsets in bytes
  uint32_t a_dst[A_D], b_dst[B_D];                      // LDS byte address of the 8-row group in slot 0
  const uint32_t a_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  const uint32_t b_base = a_base + 2u * BM * 128u;
#pragma unroll
  for (int i = 0; i < A_D; ++i) {
    const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
    int grow = m0 + row;
    grow = grow < g.M ? grow : g.M - 1;                 // clamp: stay inside A, the epilogue masks the row
    a_vo[i] = (uint32_t)(((int64_t)(grow - m0) * K + (dpos ^ ((row >> 1) & 7)) * 8) * 2);
    a_dst[i] = a_base + (uint32_t)r0 * 128u;
  }
#pragma unroll
  for (int i = 0; i < B_D; ++i) {
    const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
    if (EPI == FASTAV_EPI_SWIGLU) {
      const int blk = r0 >> 5;                          // the 8 rows of a copy lie inside one 32-row block
      b_sb[i] = ((blk & 1) ? g.W2 : g.W[0]) + (int64_t)(n0 + (blk >> 1) * 32) * K + kt0 * 64;
      b_vo[i] = (uint32_t)(((int64_t)(row & 31) * K + (dpos ^ ((row >> 1) & 7)) * 8) * 2);
    } else {
      b_sb[i] = wbase + (int64_t)(n0 - seg_start) * K + kt0 * 64;
      b_vo[i] = (uint32_t)(((int64_t)row * K + (dpos ^ ((row >> 1) & 7)) * 8) * 2);
    }
    b_dst[i] = b_base + (uint32_t)r0 * 128u;
  }
  // copy number c (0 .. D-1: A's first) of stage t into slot t & 1; past the last stage the copy is re-aimed at
  // the last stage (it lands in a slot nobody reads any more)
  const u32x4_t a_rs = make_rsrc(a_sb);
  u32x4_t b_rs[B_D];
#pragma unroll
  for (int i = 0; i < B_D; ++i) b_rs[i] = make_rsrc(b_sb[i]);
  auto dma_one = [&](int t, int c) __attribute__((always_inline)) {
    const uint32_t koff = (uint32_t)((t < KT ? t : KT - 1) * 128);            // bytes along K
    const uint32_t slot = (uint32_t)t & 1u;
    if (c < A_D) dma16_buf(a_rs, a_vo[c < A_D ? c : 0], koff, a_dst[c < A_D ? c : 0] + slot * (BM * 128u));
    else dma16_buf(b_rs[c >= A_D ? c - A_D : 0], b_vo[c >= A_D ? c - A_D : 0], koff, b_dst[c >= A_D ? c - A_D : 0] + slot * (BN * 128u));
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frow = lane & 31, fch = lane >> 5;          // operand fragment: row in block, which 8-wide k chunk
  bf16x8_t af[2][TM], bfr[2][TN];                       // operand fragments of two k-slices
  int a_fu[KS], b_fu[KS];                               // fragment positions inside a slot (16-byte units) per k-slice
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    a_fu[kk] = swz8(wm * WTM + frow, kk * 2 + fch);
    b_fu[kk] = 2 * BM * 8 + swz8(wn * WTN + frow, kk * 2 + fch);
  }
  // One k-slice: NMF MFMAs; after each of the first TM + TN of them one fragment of the next slice (slot nslot,
  // k-slice nkk; nkk < 0: none) is read into the other register buffer; `ncopy` copies of stage t_copy, numbers
  // c0 .. c0 + ncopy - 1, are issued evenly between the MFMAs.
  auto slice = [&](int buf, int t_copy, int c0, int ncopy, uint32_t nslot, int nkk) __attribute__((always_inline)) {
    const int groups = ncopy > 0 ? ncopy : 1;
#pragma unroll
    for (int grp = 0; grp < groups; ++grp) {
#pragma unroll
      for (int q = grp * NMF / groups; q < (grp + 1) * NMF / groups; ++q) {
        const int i = q / TN, j = q % TN;
        acc[i][j] = gemm_transposed(EPI) ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[buf][j], af[buf][i], acc[i][j], 0, 0, 0)
                                         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bfr[buf][j], acc[i][j], 0, 0, 0);
        if (nkk >= 0) {
          // fragments in the order the next slice's MFMAs first need them: A block 0, all B blocks, the other A blocks
          if (q == 0) af[buf ^ 1][0] = lds[a_fu[nkk < 0 ? 0 : nkk] + (int)nslot * BM * 8];
          else if (q <= TN) bfr[buf ^ 1][q - 1] = lds[b_fu[nkk < 0 ? 0 : nkk] + (int)nslot * BN * 8 + (q - 1) * 256];
          else if (q < TM + TN) af[buf ^ 1][q - TN] = lds[a_fu[nkk < 0 ? 0 : nkk] + (int)nslot * BM * 8 + (q - TN) * 256];
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // one MFMA ...
        if (nkk >= 0 && q < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // ... then one LDS read
      }
      if (ncopy > 0) {
        __builtin_amdgcn_sched_barrier(0);
        dma_one(t_copy, c0 + grp);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // stage t in slot `slot`: three slices read the rest of the stage, then - all of this stage's fragments are in
  // registers, stage t+1 has landed - the barrier, and the last slice reads the first fragments of stage t+1
  // while all copies of stage t+2 go out into the slot just freed: they have a whole stage of matrix work to land.
  auto stage = [&](int t, uint32_t slot) __attribute__((always_inline)) {
    slice(0, t + 1, D - LATE, LATE, slot, 1);            // the last LATE copies of stage t+1
    slice(1, 0, 0, 0, slot, 2);
    slice(0, 0, 0, 0, slot, 3);
    dma_wait_keep<0>();                                  // stage t+1 has landed (this wave's share)
    asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory"); // this wave's reads of the slot are complete
    __syncthreads();
    slice(1, t + 2, 0, D - LATE, slot ^ 1u, 0);
  };
  static_assert(NMF >= D - LATE && NMF >= LATE, "a slice has fewer MFMAs than it has copies to issue");

  // ---- prologue: stages 0 and 1 in flight, stage 0 landed and published
#pragma unroll
  for (int c = 0; c < D; ++c) dma_one(0, c);
#pragma unroll
  for (int c = 0; c < D - LATE; ++c) dma_one(1, c);
  dma_wait_keep<D - LATE>();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i) af[0][i] = lds[a_fu[0] + i * 256];
#pragma unroll
  for (int j = 0; j < TN; ++j) bfr[0][j] = lds[b_fu[0] + j * 256];

  int t = 0;
  for (; t + 2 <= KT; t += 2) {                          // t is even here: slots are literals
    stage(t, 0u);
    stage(t + 1, 1u);
  }
  if (t < KT) stage(t, (uint32_t)t & 1u);
  dma_wait_keep<0>();
  __syncthreads();                                     // every wave's copies have landed: LDS is free for the epilogue
  gemm_epilogue<EPI, TM, TN, WTM, WTN>(g, acc, m0, n0, wm, wn, lane,
                                       lds + wave * (2 * 32 * 8 * TN));
}

// Launches tile columns [col0, col0 + ncols) of the GEMM with the 64-k kernel.
template <int BM, int BN, int WM, int WN, int EPI, int LATE = 0>
static fastav_status_t launch_cfg_k64(GemmArgs g, int col0, int ncols, int splits, hipStream_t s) {
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = ncols;
  g.n_off = col0 * OUT_BN;
  g.splits = splits;
  g.band = (g.tiles_m * g.tiles_n > kNumCUs) ? 4 : 1;
  const size_t shmem = (size_t)2 * (BM + BN) * 8 * sizeof(bf16x8_t);
  hipError_t e = hipFuncSetAttribute((const void*)k_gemm_mfma_k64<BM, BN, WM, WN, EPI, LATE>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return fail(FASTAV_EHIP, "gemm: hipFuncSetAttribute: %s", hipGetErrorString(e));
  hipLaunchKernelGGL((k_gemm_mfma_k64<BM, BN, WM, WN, EPI, LATE>), dim3((unsigned)(g.tiles_m * g.tiles_n), (unsigned)splits),
                     dim3(WM * WN * 64), shmem, s, g);
  return check_launch("gemm_mfma_k64");
}

// The 64-k loop with three slots for A and two for B (160 KB for a 256 x 256 tile: all of a CU's LDS).  With two
// slots each, every copy of stage t+2 has to go out inside stage t's last k-slice, and that burst asks the CU's
// vector-memory path for twice what it moves per clock: in-kernel timestamps show that slice taking about three
// times as long as a slice without copies.  The third A slot is free one stage earlier, so A's copies of stage
// t+2 are spread over stage t's first three slices and only B's are left for the last one - the request rate
// stays at or under what the path sustains, and every copy still has at least three slices to land.
template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM * WN * 64, 1) void k_gemm_mfma_k64a3(GemmArgs g) {
  constexpr int NW = WM * WN;                          // waves
  constexpr int WTM = BM / WM, WTN = BN / WN;          // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;          // 32x32 blocks per wave
  constexpr int A_D = BM / (8 * NW), B_D = BN / (8 * NW);     // copy instructions per wave and stage (8 rows each)
  constexpr int D = A_D + B_D;
  constexpr int NMF = TM * TN;                         // MFMAs per k-slice
  constexpr int KS = 4;                                // k-slices of 16 per stage
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  static_assert(A_D >= 1 && B_D >= 1 && D % 2 == 0 && NMF >= D / 2 && NMF >= TM + TN && TN % 2 == 0, "tile shape");
  extern __shared__ bf16x8_t lds[];                    // [3][BM*8] A, then [2][BN*8] B

  // ---- tile assignment (as in k_gemm_mfma)
  const int nblk = g.tiles_m * g.tiles_n;
  int pid = blockIdx.x;
  {
    const int per = nblk / 8, rem = nblk % 8, xcd = pid % 8, idx = pid / 8;
    pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int kb = g.band;
  const int band = pid / (kb * g.tiles_m);
  const int bw = (g.tiles_n - band * kb < kb) ? g.tiles_n - band * kb : kb;   // columns in this band
  const int inb = pid - band * kb * g.tiles_m;
  const int tile_m = inb / bw, tile_n = band * kb + inb % bw;
  const int m0 = tile_m * BM;
  const int n0 = g.n_off + tile_n * OUT_BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave / WN, wn = wave % WN;
  const int K = g.K;
  // stages of 64 k owned by this workgroup (all of them unless split-K)
  const int kt_all = K / 64;
  const int kt0 = (int)((int64_t)kt_all * blockIdx.y / g.splits);
  const int KT = (int)((int64_t)kt_all * (blockIdx.y + 1) / g.splits) - kt0;

  const bf16_t* wbase = g.W[0];
  int seg_start = 0;
  if (EPI != FASTAV_EPI_SWIGLU) {
    if (n0 >= g.seg_end[0]) { wbase = g.W[1]; seg_start = g.seg_end[0]; }
    if (n0 >= g.seg_end[1]) { wbase = g.W[2]; seg_start = g.seg_end[1]; }
  }

  // ---- this wave's copies: instruction i covers tile rows [(i*NW + wave)*8, +8), lane = (row, 16-byte chunk)
  const int drow = lane >> 3, dpos = lane & 7;
  const bf16_t* a_sb = g.A + (int64_t)m0 * K + kt0 * 64;
  const bf16_t* b_sb[B_D];
  uint32_t a_vo[A_D], b_vo[B_D];                        // lane offsets in bytes
  uint32_t a_dst[A_D], b_dst[B_D];                      // LDS byte address of the 8-row group in slot 0
  const uint32_t a_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  const uint32_t b_base = a_base + 3u * BM * 128u;
#pragma unroll
  for (int i = 0; i < A_D; ++i) {
    const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
    int grow = m0 + row;
    grow = grow < g.M ? grow : g.M - 1;                 // clamp: stay inside A, the epilogue masks the row
    a_vo[i] = (uint32_t)(((int64_t)(grow - m0) * K + (dpos ^ ((row >> 1) & 7)) * 8) * 2);
    a_dst[i] = a_base + (uint32_t)r0 * 128u;
  }
#pragma unroll
  for (int i = 0; i < B_D; ++i) {
    const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
    if (EPI == FASTAV_EPI_SWIGLU) {
      const int blk = r0 >> 5;                          // the 8 rows of a copy lie inside one 32-row block
      b_sb[i] = ((blk & 1) ? g.W2 : g.W[0]) + (int64_t)(n0 + (blk >> 1) * 32) * K + kt0 * 64;
      b_vo[i] = (uint32_t)(((int64_t)(row & 31) * K + (dpos ^ ((row >> 1) & 7)) * 8) * 2);
    } else {
      b_sb[i] = wbase + (int64_t)(n0 - seg_start) * K + kt0 * 64;
      b_vo[i] = (uint32_t)(((int64_t)row * K + (dpos ^ ((row >> 1) & 7)) * 8) * 2);
    }
    b_dst[i] = b_base + (uint32_t)r0 * 128u;
  }
  // copy number c (0 .. D-1: A's first) of stage t into slot t & 1; past the last stage the copy is re-aimed at
  // the last stage (it lands in a slot nobody reads any more)
  const u32x4_t a_rs = make_rsrc(a_sb);
  u32x4_t b_rs[B_D];
#pragma unroll
  for (int i = 0; i < B_D; ++i) b_rs[i] = make_rsrc(b_sb[i]);
  auto dma_one = [&](int t, int c, uint32_t aslot, uint32_t bslot) __attribute__((always_inline)) {
    const uint32_t koff = (uint32_t)((t < KT ? t : KT - 1) * 128);            // bytes along K
    if (c < A_D) dma16_buf(a_rs, a_vo[c < A_D ? c : 0], koff, a_dst[c < A_D ? c : 0] + aslot * (BM * 128u));
    else dma16_buf(b_rs[c >= A_D ? c - A_D : 0], b_vo[c >= A_D ? c - A_D : 0], koff, b_dst[c >= A_D ? c - A_D : 0] + bslot * (BN * 128u));
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frow = lane & 31, fch = lane >> 5;          // operand fragment: row in block, which 8-wide k chunk
  bf16x8_t af[2][TM], bfr[2][TN];                       // operand fragments of two k-slices
  int a_fu[KS], b_fu[KS];                               // fragment positions inside a slot (16-byte units) per k-slice
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    a_fu[kk] = swz8(wm * WTM + frow, kk * 2 + fch);
    b_fu[kk] = 3 * BM * 8 + swz8(wn * WTN + frow, kk * 2 + fch);
  }
  // One k-slice: NMF MFMAs; after each of the first TM + TN of them one fragment of the next slice (slot nslot,
  // k-slice nkk; nkk < 0: none) is read into the other register buffer; `ncopy` copies of stage t_copy, numbers
  // c0 .. c0 + ncopy - 1, are issued evenly between the MFMAs.
  auto slice = [&](int buf, int t_copy, int c0, int ncopy, uint32_t cas, uint32_t cbs, uint32_t ras, uint32_t rbs, int nkk) __attribute__((always_inline)) {
    const int groups = ncopy > 0 ? ncopy : 1;
#pragma unroll
    for (int grp = 0; grp < groups; ++grp) {
#pragma unroll
      for (int q = grp * NMF / groups; q < (grp + 1) * NMF / groups; ++q) {
        const int i = q / TN, j = q % TN;
        acc[i][j] = gemm_transposed(EPI) ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[buf][j], af[buf][i], acc[i][j], 0, 0, 0)
                                         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bfr[buf][j], acc[i][j], 0, 0, 0);
        if (nkk >= 0) {
          if (q == 0) af[buf ^ 1][0] = lds[a_fu[nkk < 0 ? 0 : nkk] + (int)ras * BM * 8];
          else if (q <= TN) bfr[buf ^ 1][q - 1] = lds[b_fu[nkk < 0 ? 0 : nkk] + (int)rbs * BN * 8 + (q - 1) * 256];
          else if (q < TM + TN) af[buf ^ 1][q - TN] = lds[a_fu[nkk < 0 ? 0 : nkk] + (int)ras * BM * 8 + (q - TN) * 256];
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (nkk >= 0 && q < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      if (ncopy > 0) {
        __builtin_amdgcn_sched_barrier(0);
        dma_one(t_copy, c0 + grp, cas, cbs);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // stage t reads A slot `as` (t mod 3) and B slot `bs` (t mod 2).  A's copies of stage t+2 go out during the
  // first three slices into the A slot freed by the previous stage's barrier; B's copies of stage t+2 go out in
  // the last slice, after this stage's barrier, into the B slot this stage has just finished reading.
  constexpr int A0 = A_D / 3, A1 = (2 * A_D) / 3 - A0, A2 = A_D - A0 - A1;
  auto stage = [&](int t, uint32_t as, uint32_t bs) __attribute__((always_inline)) {
    const uint32_t as2 = as >= 1u ? as - 1u : 2u;        // (t + 2) mod 3
    const uint32_t as1 = as == 2u ? 0u : as + 1u;        // (t + 1) mod 3
    slice(0, t + 2, 0, A0, as2, 0u, as, bs, 1);
    slice(1, t + 2, A0, A1, as2, 0u, as, bs, 2);
    slice(0, t + 2, A0 + A1, A2, as2, 0u, as, bs, 3);
    dma_wait_keep<A_D>();                                // stage t+1 has landed; only A of stage t+2 may be in flight
    asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
    __syncthreads();
    slice(1, t + 2, A_D, B_D, 0u, bs, as1, bs ^ 1u, 0);
  };
  static_assert(NMF >= B_D && NMF >= A2, "a slice has fewer MFMAs than it has copies to issue");

  // ---- prologue: stages 0 and 1 in flight, stage 0 landed and published
#pragma unroll
  for (int c = 0; c < D; ++c) dma_one(0, c, 0u, 0u);
#pragma unroll
  for (int c = 0; c < D; ++c) dma_one(1, c, 1u, 1u);
  dma_wait_keep<D>();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i) af[0][i] = lds[a_fu[0] + i * 256];
#pragma unroll
  for (int j = 0; j < TN; ++j) bfr[0][j] = lds[b_fu[0] + j * 256];

  int t = 0;
  for (; t + 6 <= KT; t += 6) {                          // t is a multiple of 6 here: slots are literals
#pragma unroll
    for (int u = 0; u < 6; ++u) stage(t + u, (uint32_t)(u % 3), (uint32_t)(u % 2));
  }
#pragma unroll 1
  for (; t < KT; ++t) stage(t, (uint32_t)t % 3u, (uint32_t)t & 1u);
  dma_wait_keep<0>();
  __syncthreads();                                     // every wave's copies have landed: LDS is free for the epilogue
  gemm_epilogue<EPI, TM, TN, WTM, WTN>(g, acc, m0, n0, wm, wn, lane,
                                       lds + wave * (2 * 32 * 8 * TN));
}


// Launches tile columns [col0, col0 + ncols) of the GEMM with the 64-k kernel with three A slots.
template <int BM, int BN, int WM, int WN, int EPI>
static fastav_status_t launch_cfg_k64a3(GemmArgs g, int col0, int ncols, int splits, hipStream_t s) {
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = ncols;
  g.n_off = col0 * OUT_BN;
  g.splits = splits;
  g.band = (g.tiles_m * g.tiles_n > kNumCUs) ? 4 : 1;
  const size_t shmem = (size_t)(3 * BM + 2 * BN) * 8 * sizeof(bf16x8_t);
  hipError_t e = hipFuncSetAttribute((const void*)k_gemm_mfma_k64a3<BM, BN, WM, WN, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return fail(FASTAV_EHIP, "gemm: hipFuncSetAttribute: %s", hipGetErrorString(e));
  hipLaunchKernelGGL((k_gemm_mfma_k64a3<BM, BN, WM, WN, EPI>), dim3((unsigned)(g.tiles_m * g.tiles_n), (unsigned)splits),
                     dim3(WM * WN * 64), shmem, s, g);
  return check_launch("gemm_mfma_k64a3");
}

// ------------------------------------------------------------------------------------------------------------
// The 256 x 256 kernel on v_mfma_f32_16x16x32_bf16.  Under these GEMMs the chip is power-limited, and this shape
// reads and writes half as many accumulator registers per flop as 32x32x16: a loop of nothing but matrix
// instructions sustains 2.05 GHz with it against 1.76 GHz (both at full issue rate).  Same LDS plan as
// k_gemm_mfma_k64a3 (64-k stages, three A slots, two B slots, 8-row x 128-byte copies, chunk swizzle).
//
// A stage is two k-steps of 32; a k-step is TM x TN matrix instructions, A block outer, B block inner.  Fragment
// registers: one 16-row A fragment per A block (reloaded for the next k-step as soon as the block's instructions
// are done), B fragments double-buffered by k-step.  So every read of a stage's own data has been issued when
// its second k-step starts; the stage's barrier sits after that k-step's second A block, and everything read
// after it belongs to the next stage.  B's copies of stage t+2 follow the barrier, A's go out during the first
// k-step into the slot the previous stage freed.
//
// Accumulators hold the transposed product (weight fragment first): register quad = 4 consecutive output columns
// of row lane % 16, columns (lane / 16) * 4.. of the 16 x 16 block.  The hardware-add epilogue keeps the
// untransposed product (column lane % 16, rows (lane / 16) * 4..).
// scheduling hint "then n LDS reads" for an n known after unrolling (the builtin wants literals)
__device__ __forceinline__ void sched_ds_reads(int n) {
  if (n == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  else if (n == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
  else if (n == 3) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
  else if (n == 4) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
  else if (n == 5) __builtin_amdgcn_sched_group_barrier(0x100, 5, 0);
}

template <int EPI, int TM, int TN, int WTM, int WTN>
__device__ __forceinline__ void gemm16_epilogue(const GemmArgs& g, f32x4_t (&acc)[TM][TN], int m0, int n0, int wm, int wn, int lane,
                                                bf16x8_t* stage) {
  const int mr = lane & 15, gq = lane >> 4;
  if constexpr (EPI == kEpiResAtomic) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * WTN + j * 16 + mr;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = m0 + wm * WTM + i * 16 + gq * 4 + r;
          // fire-and-forget hardware add at the L2; each element receives exactly one addend per launch
          if (row < g.M) unsafeAtomicAdd(&((float*)g.C)[(int64_t)row * g.ldc + col], acc[i][j][r]);
        }
      }
  } else if constexpr (EPI == FASTAV_EPI_STORE || EPI == FASTAV_EPI_SWIGLU) {
    // bf16 output.  SwiGLU: B rows come in groups of 64 = 32 gate rows, then 32 up rows -> of four 16-blocks
    // j = 4u .. 4u + 3 the output blocks are (gate 4u, up 4u + 2) and (gate 4u + 1, up 4u + 3).
    constexpr int NB = (EPI == FASTAV_EPI_SWIGLU) ? TN / 2 : TN;     // output blocks (16 columns) per row of the wave
    constexpr int NCH = NB * 2;                                      // 16-byte chunks per output row
    constexpr int RPI = 64 / NCH;                                    // rows per 64-lane access
    constexpr int SWM = NCH >= 8 ? 7 : NCH - 1;
    static_assert(NCH == 4 || NCH == 8 || NCH == 16, "wave tile width");
    const int colw = (EPI == FASTAV_EPI_SWIGLU) ? n0 + wn * (WTN / 2) : n0 + wn * WTN;
    const bool vec = g.vec_ok != 0;
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int jb = 0; jb < NB; ++jb) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if constexpr (EPI == FASTAV_EPI_SWIGLU) {
            const int jg = (jb / 2) * 4 + (jb & 1);
            const float gt = acc[i][jg][r], up = acc[i][jg + 2][r];
            v[r] = gt / (1.0f + __expf(-gt)) * up;
          } else {
            v[r] = acc[i][jb][r];
          }
        }
        if (vec) {
          // 8-byte piece: columns jb * 16 + gq * 4 .. + 3 of row mr -> chunk jb * 2 + gq / 2, half gq & 1
          const u32x2_t pc = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
          const int c = jb * 2 + (gq >> 1);
          *(u32x2_t*)((char*)&stage[mr * NCH + (c ^ ((mr >> 1) & SWM))] + (gq & 1) * 8) = pc;
        } else {
          const int row = m0 + wm * WTM + i * 16 + mr;
          if (row < g.M) {
            bf16_t* C = (bf16_t*)g.C + (int64_t)row * g.ldc + colw + jb * 16 + gq * 4;
#pragma unroll
            for (int r = 0; r < 4; ++r) C[r] = (bf16_t)v[r];
          }
        }
      }
      if (vec) {
        // the wave's own LDS accesses execute in order: rows are read back whole, 16 bytes per lane
        const int rr = lane / NCH, cc = lane % NCH;
#pragma unroll
        for (int it = 0; it < 16 / RPI; ++it) {
          const int r = it * RPI + rr;
          const u32x4_t val = *(const u32x4_t*)&stage[r * NCH + (cc ^ ((r >> 1) & SWM))];
          const int row = m0 + wm * WTM + i * 16 + r;
          if (row < g.M) *(u32x4_t*)((bf16_t*)g.C + (int64_t)row * g.ldc + colw + cc * 8) = val;
        }
      }
    }
  } else {
    // fp32 output (residual read-modify-write, split-K partial): 16-byte pieces, TN * 4 of them per row
    constexpr int NC = TN * 4, RP = 64 / NC;
    static_assert(NC == 16 || NC == 32, "wave tile width");
    const bool vec = g.vec_ok != 0;
    float* Cb = (EPI == kEpiPartial) ? g.partial + (int64_t)blockIdx.y * g.M * g.N + n0 + wn * WTN : (float*)g.C + n0 + wn * WTN;
    const int64_t pitch = (EPI == kEpiPartial) ? g.N : g.ldc;
    f32x4_t* st = (f32x4_t*)stage;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if (vec) {
#pragma unroll
        for (int j = 0; j < TN; ++j) st[mr * NC + ((j * 4 + gq) ^ (mr & 7))] = acc[i][j];
        const int rr = lane / NC, cc = lane % NC;
        f32x4_t old[16 / RP];
        if constexpr (EPI == FASTAV_EPI_RESADD) {
#pragma unroll
          for (int it = 0; it < 16 / RP; ++it) {
            const int row = m0 + wm * WTM + i * 16 + it * RP + rr;
            old[it] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            if (row < g.M) old[it] = *(const f32x4_t*)(Cb + (int64_t)row * pitch + cc * 4);
          }
        }
#pragma unroll
        for (int it = 0; it < 16 / RP; ++it) {
          const int r = it * RP + rr;
          f32x4_t val = st[r * NC + (cc ^ (r & 7))];
          if constexpr (EPI == FASTAV_EPI_RESADD) { val[0] += old[it][0]; val[1] += old[it][1]; val[2] += old[it][2]; val[3] += old[it][3]; }
          const int row = m0 + wm * WTM + i * 16 + r;
          if (row < g.M) *(f32x4_t*)(Cb + (int64_t)row * pitch + cc * 4) = val;
        }
      } else {
        const int row = m0 + wm * WTM + i * 16 + mr;
        if (row < g.M) {
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              float* C = Cb + (int64_t)row * pitch + j * 16 + gq * 4 + r;
              if constexpr (EPI == FASTAV_EPI_RESADD) *C += acc[i][j][r];
              else *C = acc[i][j][r];
            }
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM * WN * 64, 1) void k_gemm_mfma16(GemmArgs g) {
  constexpr int NW = WM * WN;                          // waves
  constexpr int WTM = BM / WM, WTN = BN / WN;          // wave tile
  constexpr int TM = WTM / 16, TN = WTN / 16;          // 16x16 blocks per wave
  constexpr int A_D = BM / (8 * NW), B_D = BN / (8 * NW);     // copy instructions per wave and stage (8 rows each)
  constexpr int D = A_D + B_D;
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  static_assert(A_D >= 1 && B_D >= 1 && TM >= 4 && TN >= 4 && TN % 4 == 0, "tile shape");
  extern __shared__ bf16x8_t lds[];                    // [3][BM*8] A, then [2][BN*8] B

  // ---- tile assignment (as in k_gemm_mfma)
  const int nblk = g.tiles_m * g.tiles_n;
  int pid = blockIdx.x;
  {
    const int per = nblk / 8, rem = nblk % 8, xcd = pid % 8, idx = pid / 8;
    pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int kb = g.band;
  const int band = pid / (kb * g.tiles_m);
  const int bw = (g.tiles_n - band * kb < kb) ? g.tiles_n - band * kb : kb;   // columns in this band
  const int inb = pid - band * kb * g.tiles_m;
  const int tile_m = inb / bw, tile_n = band * kb + inb % bw;
  const int m0 = tile_m * BM;
  const int n0 = g.n_off + tile_n * OUT_BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave / WN, wn = wave % WN;
  const int K = g.K;
  const int kt_all = K / 64;
  const int kt0 = (int)((int64_t)kt_all * blockIdx.y / g.splits);
  const int KT = (int)((int64_t)kt_all * (blockIdx.y + 1) / g.splits) - kt0;

  const bf16_t* wbase = g.W[0];
  int seg_start = 0;
  if (EPI != FASTAV_EPI_SWIGLU) {
    if (n0 >= g.seg_end[0]) { wbase = g.W[1]; seg_start = g.seg_end[0]; }
    if (n0 >= g.seg_end[1]) { wbase = g.W[2]; seg_start = g.seg_end[1]; }
  }

  // ---- this wave's copies: instruction i covers tile rows [(i*NW + wave)*8, +8), lane = (row, 16-byte chunk)
  const int drow = lane >> 3, dpos = lane & 7;
  uint32_t a_vo[A_D], b_vo[B_D];                        // lane offsets in bytes
  uint32_t a_dst[A_D], b_dst[B_D];                      // LDS byte address of the 8-row group in slot 0
  u32x4_t a_rs, b_rs[B_D];
  const uint32_t a_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  const uint32_t b_base = a_base + 3u * BM * 128u;
  a_rs = make_rsrc(g.A + (int64_t)m0 * K + kt0 * 64);
#pragma unroll
  for (int i = 0; i < A_D; ++i) {
    const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
    int grow = m0 + row;
    grow = grow < g.M ? grow : g.M - 1;                 // clamp: stay inside A, the epilogue masks the row
    a_vo[i] = ((uint32_t)(grow - m0) * (uint32_t)K + (uint32_t)(dpos ^ ((row >> 1) & 7)) * 8u) * 2u;
    a_dst[i] = a_base + (uint32_t)r0 * 128u;
  }
#pragma unroll
  for (int i = 0; i < B_D; ++i) {
    const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
    if (EPI == FASTAV_EPI_SWIGLU) {
      const int blk = r0 >> 5;                          // the 8 rows of a copy lie inside one 32-row block
      b_rs[i] = make_rsrc(((blk & 1) ? g.W2 : g.W[0]) + (int64_t)(n0 + (blk >> 1) * 32) * K + kt0 * 64);
      b_vo[i] = ((uint32_t)(row & 31) * (uint32_t)K + (uint32_t)(dpos ^ ((row >> 1) & 7)) * 8u) * 2u;
    } else {
      b_rs[i] = make_rsrc(wbase + (int64_t)(n0 - seg_start) * K + kt0 * 64);
      b_vo[i] = ((uint32_t)row * (uint32_t)K + (uint32_t)(dpos ^ ((row >> 1) & 7)) * 8u) * 2u;
    }
    b_dst[i] = b_base + (uint32_t)r0 * 128u;
  }
  // copy number c of A (B) for stage t; past the last stage it is re-aimed at the last stage (nobody reads it)
  auto dma_a = [&](int t, int c, uint32_t slot) __attribute__((always_inline)) {
    dma16_buf(a_rs, a_vo[c], (uint32_t)((t < KT ? t : KT - 1) * 128), a_dst[c] + slot * (BM * 128u));
  };
  auto dma_b = [&](int t, int c, uint32_t slot) __attribute__((always_inline)) {
    dma16_buf(b_rs[c], b_vo[c], (uint32_t)((t < KT ? t : KT - 1) * 128), b_dst[c] + slot * (BN * 128u));
  };

  f32x4_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // operand fragment of a 16-row block for k-step s: row lane % 16, 16-byte chunk s * 4 + lane / 16
  const int frow = lane & 15, fch = lane >> 4;
  bf16x8_t af[TM], bfr[2][TN];
  int a_fu[2], b_fu[2];                                 // fragment positions inside a slot (16-byte units) per k-step
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    a_fu[ks] = swz8(wm * WTM + frow, ks * 4 + fch);
    b_fu[ks] = 3 * BM * 8 + swz8(wn * WTN + frow, ks * 4 + fch);
  }
  auto mfma_block = [&](int i, int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      acc[i][j] = gemm_transposed(EPI) ? __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[ks][j], af[i], acc[i][j], 0, 0, 0)
                                       : __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[ks][j], acc[i][j], 0, 0, 0);
    }
  };
  // One stage.  `as`, `bs`: this stage's slots (t mod 3, t mod 2).
  constexpr int PB = (TN + TM / 2 - 1) / (TM / 2);       // B fragments read behind one A block (first half of a k-step)
  constexpr int PA = (A_D + TM - 2) / (TM - 1);          // A copies issued behind one A block of the first k-step
  constexpr int PC = (B_D + TM - 3) / (TM - 2);          // B copies issued behind one A block after the barrier
  auto stage = [&](int t, uint32_t as, uint32_t bs) __attribute__((always_inline)) {
    const uint32_t as2 = as >= 1u ? as - 1u : 2u;        // (t + 2) mod 3
    const uint32_t as1 = as == 2u ? 0u : as + 1u;        // (t + 1) mod 3
    // k-step 0: after A block i is done its register takes the block's k-step-1 fragment; B's k-step-1 fragments
    // are read behind the first blocks; A's copies of stage t+2 go out behind blocks 1, 2, ...
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      mfma_block(i, 0);
      af[i] = lds[a_fu[1] + (int)as * BM * 8 + i * 128];
      int nrd = 1;
#pragma unroll
      for (int j = i * PB; j < (i + 1) * PB && j < TN; ++j) { bfr[1][j] = lds[b_fu[1] + (int)bs * BN * 8 + j * 128]; ++nrd; }
      __builtin_amdgcn_sched_group_barrier(0x008, TN, 0);
      sched_ds_reads(nrd);
      if (i >= 1 && (i - 1) * PA < A_D) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = (i - 1) * PA; c < i * PA && c < A_D; ++c) dma_a(t + 2, c, as2);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // k-step 1: two blocks, then - every fragment of this stage is in registers, stage t+1 has landed - the
    // barrier; from there on the freed registers take the next stage's k-step-0 fragments and B's copies of
    // stage t+2 go out into the slot this stage has finished with
    mfma_block(0, 1);
    mfma_block(1, 1);
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * TN, 0);
    __builtin_amdgcn_sched_barrier(0);
    dma_wait_keep<A_D>();                                // stage t+1 has landed; only A of stage t+2 may be in flight
    asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
    __syncthreads();
    af[0] = lds[a_fu[0] + (int)as1 * BM * 8];
    af[1] = lds[a_fu[0] + (int)as1 * BM * 8 + 128];
#pragma unroll
    for (int i = 2; i < TM; ++i) {
      mfma_block(i, 1);
      af[i] = lds[a_fu[0] + (int)as1 * BM * 8 + i * 128];
      int nrd = (i == 2) ? 3 : 1;
#pragma unroll
      for (int j = (i - 2) * PB; j < (i - 1) * PB && j < TN; ++j) { bfr[0][j] = lds[b_fu[0] + (int)(bs ^ 1u) * BN * 8 + j * 128]; ++nrd; }
      __builtin_amdgcn_sched_group_barrier(0x008, TN, 0);
      sched_ds_reads(nrd);
      if ((i - 2) * PC < B_D) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = (i - 2) * PC; c < (i - 1) * PC && c < B_D; ++c) dma_b(t + 2, c, bs);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  static_assert(PB * (TM / 2) >= TN && PB * (TM - 2) >= TN && PA * (TM - 1) >= A_D && PC * (TM - 2) >= B_D, "schedule");

  // ---- prologue: stages 0 and 1 in flight, stage 0 landed and published
#pragma unroll
  for (int c = 0; c < A_D; ++c) dma_a(0, c, 0u);
#pragma unroll
  for (int c = 0; c < B_D; ++c) dma_b(0, c, 0u);
#pragma unroll
  for (int c = 0; c < A_D; ++c) dma_a(1, c, 1u);
#pragma unroll
  for (int c = 0; c < B_D; ++c) dma_b(1, c, 1u);
  dma_wait_keep<D>();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i) af[i] = lds[a_fu[0] + i * 128];
#pragma unroll
  for (int j = 0; j < TN; ++j) bfr[0][j] = lds[b_fu[0] + j * 128];

  int t = 0;
  for (; t + 6 <= KT; t += 6) {                          // t is a multiple of 6 here: slots are literals
#pragma unroll
    for (int u = 0; u < 6; ++u) stage(t + u, (uint32_t)(u % 3), (uint32_t)(u % 2));
  }
#pragma unroll 1
  for (; t < KT; ++t) stage(t, (uint32_t)t % 3u, (uint32_t)t & 1u);
  dma_wait_keep<0>();
  __syncthreads();                                     // every wave's copies have landed: LDS is free for the epilogue
  gemm16_epilogue<EPI, TM, TN, WTM, WTN>(g, acc, m0, n0, wm, wn, lane, lds + wave * (16 * 4 * TN));
}

template <int BM, int BN, int WM, int WN, int EPI>
static fastav_status_t launch_cfg_16(GemmArgs g, int col0, int ncols, int splits, hipStream_t s) {
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = ncols;
  g.n_off = col0 * OUT_BN;
  g.splits = splits;
  g.band = (g.tiles_m * g.tiles_n > kNumCUs) ? 4 : 1;
  const size_t shmem = (size_t)(3 * BM + 2 * BN) * 8 * sizeof(bf16x8_t);
  hipError_t e = hipFuncSetAttribute((const void*)k_gemm_mfma16<BM, BN, WM, WN, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return fail(FASTAV_EHIP, "gemm: hipFuncSetAttribute: %s", hipGetErrorString(e));
  hipLaunchKernelGGL((k_gemm_mfma16<BM, BN, WM, WN, EPI>), dim3((unsigned)(g.tiles_m * g.tiles_n), (unsigned)splits),
                     dim3(WM * WN * 64), shmem, s, g);
  return check_launch("gemm_mfma16");
}

bool mfma_linear_supported(int64_t m, int n, int k, int epilogue, int dtype) {
  if (dtype != FASTAV_BF16 || m < 1 || m > 0x7FFFFFFF) return false;
  if (k % 64 != 0 || k < 128) return false;            // >= 4 stages of 32
  return epilogue == FASTAV_EPI_SWIGLU ? (n % 64 == 0) : (n % 128 == 0);
}

// R[m][n] += sum over splits of partial[s][m][n], splits added in index order (deterministic).
__global__ __launch_bounds__(256) void k_splitk_reduce(float* __restrict__ R, int64_t ldc, const float* __restrict__ partial,
                                                       int M, int N, int splits) {
  const int64_t n4 = N / 4;
  const int64_t total = (int64_t)M * n4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / n4, c4 = i % n4;
    f32x4_t acc = *(const f32x4_t*)(R + row * ldc + c4 * 4);
    for (int s = 0; s < splits; ++s) {
      const f32x4_t p = *(const f32x4_t*)(partial + ((int64_t)s * M + row) * N + c4 * 4);
      acc[0] += p[0]; acc[1] += p[1]; acc[2] += p[2]; acc[3] += p[3];
    }
    *(f32x4_t*)(R + row * ldc + c4 * 4) = acc;
  }
}

// Launches tile columns [col0, col0 + ncols) (in units of the tile's output width) of the GEMM.
template <int BM, int BN, int WM, int WN, int EPI, int NST = 4>
static fastav_status_t launch_cfg(GemmArgs g, int col0, int ncols, int splits, hipStream_t s) {
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = ncols;
  g.n_off = col0 * OUT_BN;
  g.splits = splits;
  g.band = (g.tiles_m * g.tiles_n > kNumCUs) ? 4 : 1;
  const size_t shmem = (size_t)NST * (BM + BN) * 4 * sizeof(bf16x8_t);
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)k_gemm_mfma<BM, BN, WM, WN, EPI, NST>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return fail(FASTAV_EHIP, "gemm: hipFuncSetAttribute: %s", hipGetErrorString(e));
  }
  hipLaunchKernelGGL((k_gemm_mfma<BM, BN, WM, WN, EPI, NST>), dim3((unsigned)(g.tiles_m * g.tiles_n), (unsigned)splits),
                     dim3(WM * WN * 64), shmem, s, g);
  return check_launch("gemm_mfma");
}

constexpr int kCUs = kNumCUs;

// 256 x 256 tiles.  A residual epilogue over several rounds of tiles uses the hardware-add form (it overlaps
// with the next round); within a single round the plain read-modify-write drains sooner.
template <int EPI>
static fastav_status_t launch_big(const GemmArgs& g, int col0, int ncols, int64_t tiles, hipStream_t s) {
  if constexpr (EPI == FASTAV_EPI_RESADD) {
    if (tiles >= 2 * kCUs) return launch_cfg_16<256, 256, 2, 4, kEpiResAtomic>(g, col0, ncols, 1, s);
  }
  return launch_cfg_16<256, 256, 2, 4, EPI>(g, col0, ncols, 1, s);
}

constexpr size_t kSplitKScratchBytes = (size_t)2 * kCUs * 256 * 256 * sizeof(float);   // <= 512 partial tiles

size_t mfma_linear_scratch_bytes() { return kSplitKScratchBytes; }

template <int EPI>
static fastav_status_t launch_epi(GemmArgs& g, bool big_ok, void* scratch, size_t scratch_bytes, hipStream_t s) {
  constexpr int OUT_BIG = (EPI == FASTAV_EPI_SWIGLU) ? 128 : 256, OUT_SMALL = OUT_BIG / 2;
  const int tm = (g.M + 255) / 256;
  const int tn = g.N / OUT_BIG;                         // tile columns of the 256 x 256 tiling (valid if big_ok)
  const int64_t tiles_big = (int64_t)tm * tn;
  if (!big_ok) return launch_cfg_k64<128, 128, 2, 2, EPI, 4>(g, 0, g.N / OUT_SMALL, 1, s);

  // Less than one round of 256 x 256 tiles and a linear epilogue: split K so that about one tile per CU
  // is in flight; partial tiles go to scratch and are added to the residual in split order.
  if (EPI == FASTAV_EPI_RESADD && tiles_big < (kCUs * 9) / 10 && scratch != nullptr && g.ldc % 4 == 0 &&
      ((uintptr_t)g.C % 16) == 0) {
    int best = 1;
    double best_eff = (double)tiles_big / kCUs;
    for (int sp = 2; sp <= 8; ++sp) {
      if (tiles_big * sp > 2 * kCUs || (g.K / 32) / sp < 16) break;
      if ((size_t)sp * g.M * g.N * sizeof(float) > scratch_bytes) break;
      const double rounds = (double)((tiles_big * sp + kCUs - 1) / kCUs);
      const double eff = (double)tiles_big * sp / (rounds * kCUs);
      if (eff > best_eff + 0.05) { best_eff = eff; best = sp; }
    }
    if (best > 1) {
      GemmArgs gp = g;
      gp.partial = (float*)scratch;
      gp.vec_ok = ((uintptr_t)scratch % 16 == 0) ? 1 : 0;   // partial rows are N floats, N a multiple of 128
      // long K ranges: the 64-k kernel; short ones (an O projection cut in three) start and drain faster with
      // the 32-k ring, whose prologue is half as large
      fastav_status_t st = (g.K / best >= 2048) ? launch_cfg_16<256, 256, 2, 4, kEpiPartial>(gp, 0, tn, best, s)
                                                : launch_cfg<256, 256, 2, 4, kEpiPartial>(gp, 0, tn, best, s);
      if (st != FASTAV_OK) return st;
      const int64_t total = (int64_t)g.M * (g.N / 4);
      const unsigned blocks = (unsigned)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
      hipLaunchKernelGGL(k_splitk_reduce, dim3(blocks), dim3(256), 0, s, (float*)g.C, g.ldc, (const float*)scratch, g.M, g.N, best);
      return check_launch("splitk_reduce");
    }
  }
  // small launches: 128 x 128 tiles, two workgroups per CU, through the 64-k loop (copies split over two slices:
  // a 64 x 64 wave tile has four MFMAs per slice); +10-20 % over the 32-k ring on the pruned layers' QKV
  if (tiles_big < 192) return launch_cfg_k64<128, 128, 2, 2, EPI, 4>(g, 0, g.N / OUT_SMALL, 1, s);

  // Whole rounds of big tiles, then the leftover tile columns with 128 x 128 tiles (two workgroups per CU)
  // when the last round would leave three quarters of the CUs idle.
  const int64_t rem = tiles_big % kCUs;
  if (tiles_big > kCUs && rem != 0 && rem <= kCUs / 4) {
    const int cols_full = (int)((tiles_big - rem) / tm);          // whole tile columns inside the full rounds
    if (cols_full > 0 && cols_full < tn) {
      fastav_status_t st = launch_big<EPI>(g, 0, cols_full, tiles_big - rem, s);
      if (st != FASTAV_OK) return st;
      return launch_cfg<128, 128, 2, 2, EPI>(g, cols_full * 2, (tn - cols_full) * 2, 1, s);
    }
  }
  return launch_big<EPI>(g, 0, tn, tiles_big, s);
}

fastav_status_t launch_linear_mfma(const void* a, const void* const* w_seg, const int* seg_rows, int n_seg,
                                   const void* w2, void* c, int64_t ldc, int64_t m, int n, int k, int epilogue,
                                   void* scratch, size_t scratch_bytes, hipStream_t s) {
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
  g.C = c; g.ldc = ldc; g.M = (int)m; g.N = n; g.K = k; g.n_off = 0; g.splits = 1; g.partial = nullptr;
  g.vec_ok = ((uintptr_t)c % 16 == 0 && ldc % (epilogue == FASTAV_EPI_RESADD ? 4 : 8) == 0) ? 1 : 0;
  if (((uintptr_t)a | (uintptr_t)w_seg[0]) % 16) return fail(FASTAV_EINVAL, "gemm: A and W must be 16-byte aligned");
  if (epilogue == FASTAV_EPI_STORE) return launch_epi<FASTAV_EPI_STORE>(g, big_ok, scratch, scratch_bytes, s);
  if (epilogue == FASTAV_EPI_RESADD) return launch_epi<FASTAV_EPI_RESADD>(g, big_ok, scratch, scratch_bytes, s);
  return launch_epi<FASTAV_EPI_SWIGLU>(g, big_ok, scratch, scratch_bytes, s);
}

}  // namespace fastav
