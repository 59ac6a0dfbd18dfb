// bf16 linear layers on the CDNA4 matrix cores: C = A W^T with A [M, K] and W [N, K] both K-contiguous,
// fp32 accumulation in v_mfma_f32_16x16x32_bf16.
//
// One workgroup owns a BM x BN output tile (256 x 256 with 8 waves, or 128 x 128 with 4 waves and two workgroups
// per CU); its WM x WN waves each multiply a (BM/WM) x (BN/WN) sub-tile as 16 x 16 MFMA blocks.  K is walked in
// stages of 64.  The operands of a stage travel L2 -> LDS with asynchronous 16-byte-per-lane copies
// (buffer_load_dwordx4 ... lds: no VGPR staging, no ds_write); one copy instruction moves 8 rows x 128
// contiguous bytes, whole L2 lines.  LDS holds three stage slots for A and two for B.  The copies are issued one
// or two at a time between groups of MFMAs: the vector-memory path takes 64 B/clk per CU, and a burst of copies
// would queue up in front of the issuing waves' matrix instructions.
//
// Why this MFMA shape: under these GEMMs the chip is power-limited, and 16x16x32 reads and writes half as many
// accumulator registers per flop as 32x32x16.  A loop of nothing but matrix instructions sustains 2.05 GHz with
// it against 1.76 GHz (both at full issue rate); the GEMM gained 5-8 % from the switch alone.
//
// LDS layout: a slot holds BM (or BN) rows of 64 bf16 = 128 bytes (8 chunks of 16), chunk c of row r stored at
// position c ^ ((r >> 1) & 7).  The LDS has 64 four-byte banks and serves a 16-byte-per-lane read 16 lanes at a
// time: the 16 rows an MFMA operand read touches (same logical chunk) then fall in 16 distinct 16-byte slots of
// the 256-byte bank window.  A copy instruction lands lane l at base + 16 l, i.e. it fills 8 consecutive rows;
// the swizzle is applied on the global side (a lane fetches the chunk that belongs in its slot).
//
// B rows may come from several matrices: Q|K|V stacked along N (segments), or gate/up for the SwiGLU
// epilogue, where 32-row blocks of the B tile alternate gate, up, gate, up ... so that a lane holds
// gate[r, c] and up[r, c] in matching accumulator registers and silu(g) * u needs no exchange.
//
// Workgroup ids are first re-dealt so that each of the 8 XCDs (ids are dispatched round-robin over them)
// owns a contiguous run of tiles; in launches of more than one round the tiles are ordered in bands of four
// tile columns swept row by row, so the tiles an XCD runs at one time form a compact block and share operand
// panels through their common L2.
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
  void* Cs[3];             // plain-store epilogue with seg_out: segment i of the output columns goes to its own matrix
  int64_t ldcs[3];         //   Cs[i] (row pitch ldcs[i] elements) instead of columns of C
  int seg_out;
  int vec_ok;              // the output (C, or `partial`) takes 16-byte accesses: base and row pitch are multiples of 16 bytes
  // plain-store epilogue, optional: rotate-half RoPE on the output columns of the first `rope_segs` segments (whole
  // heads of rope_dh = 64 or 128 columns) before the one rounding to bf16: row r is rotated by the angles of position
  // rope_pos[r], taken from rope_tab [position][rope_dh / 2] = (cos, sin)
  const int32_t* rope_pos;
  const float2* rope_tab;
  int rope_dh, rope_segs;
  // optional: output row r is computed from row a_rows[r] of A (a row gather folded into the operand copies)
  const int32_t* a_rows;
};

constexpr int kNumCUs = 256;
constexpr int kEpiPartial = 100;   // internal epilogue: plain fp32 store of a split-K partial
constexpr int kEpiResAtomic = 101; // internal epilogue: residual update through fire-and-forget hardware adds

// Asynchronous 16-byte-per-lane global -> LDS copy as a buffer load: a 128-bit resource (base, no stride, no bounds
// of interest) in SGPRs, a 32-bit lane offset and a scalar byte offset that advances along K; lane l's data lands
// at lds_byte_addr + 16 l.  Completion is tracked by vmcnt (copies complete in issue order).
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

__device__ __forceinline__ int swz8(int row, int chunk) { return row * 8 + (chunk ^ ((row >> 1) & 7)); }   // 16-byte units

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2_t t = {(bf16_t)a, (bf16_t)b};
  return __builtin_bit_cast(uint32_t, t);
}
constexpr bool gemm_transposed(int epi) { return epi != kEpiResAtomic; }

// A stage is two k-steps of 32; a k-step is TM x TN matrix instructions, A block outer, B block inner.  Fragment
// registers: one 16-row A fragment per A block (reloaded for the next k-step as soon as the block's instructions
// are done), B fragments double-buffered by k-step.  So every read of a stage's own data has been issued when
// its second k-step starts; the stage's one barrier sits after that k-step's second A block, and everything read
// after it belongs to the next stage.  B's copies of stage t+2 follow the barrier (into the slot the stage has
// finished with), A's go out during the first k-step into the slot the previous stage freed: with two slots for
// both operands every copy would have to go out in the quarter of a stage behind the barrier, twice what the
// vector-memory path moves per clock (in-kernel timestamps showed that part taking three times as long).
//
// Accumulators hold the transposed product (weight fragment first): register quad = 4 consecutive output columns
// of row lane % 16, columns (lane / 16) * 4.. of the 16 x 16 block.  The hardware-add epilogue keeps the
// untransposed product (column lane % 16, rows (lane / 16) * 4..): its element-wise adds then cover 64 contiguous
// bytes per row.
//
// Epilogue: `stage` is LDS the wave may use as it likes (the caller has made sure that no copy is still in flight
// and no other wave reads it): 16 rows of the wave's output width.  Aligned outputs pass through it - the lanes'
// pieces are laid down row by row and read back so that a global access covers whole rows of the wave's tile
// (full 128-byte lines: a quarter of the L2 requests of storing the pieces as the accumulators hold them).
// Scheduling hint for one A block: its `nmfma` matrix instructions with `nrd` LDS reads behind the first ones,
// one read per matrix instruction (+1-2 % over all reads after the block).  Counts are known after unrolling;
// the builtin wants literals.
__device__ __forceinline__ void sched_block(int nmfma, int nrd) {
#pragma unroll
  for (int r = 0; r < 8; ++r)
    if (r < nrd && r < nmfma) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
  const int rest = nmfma - nrd;
  if (rest == 1) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
  else if (rest == 2) __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
  else if (rest == 3) __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
  else if (rest == 4) __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
  else if (rest == 5) __builtin_amdgcn_sched_group_barrier(0x008, 5, 0);
  else if (rest == 6) __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
  else if (rest >= 7) __builtin_amdgcn_sched_group_barrier(0x008, 7, 0);
  if (nrd > nmfma) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
}

// RoPE in the plain-store epilogue.  The tile's weight rows were fetched in a permuted order (see the copy addresses
// in the kernel): inside every head of 128 columns the 32-column blocks arrive as 0, 2, 1, 3, so that the wave that
// owns tile columns [64 w, 64 w + 64) holds head columns 32 (w & 1) + [0, 32) in its 16-column blocks 0, 1 and their
// rotation partners, 64 columns further on, in blocks 2, 3 - the same registers of the same lane, as with the
// gate / up pairs of the SwiGLU epilogue.  A head of 64 columns is one wave's width and needs no permutation.
// -> first column, relative to the segment's output, of the wave's 8-column chunk cc (0..7)
__device__ __forceinline__ int rope_chunk_col(int n0, int wn, int cc, int dh) {
  if (dh == 128) return n0 + ((wn * 64) & ~127) + 32 * (wn & 1) + ((cc & 4) ? 64 : 0) + 8 * (cc & 3);
  return n0 + wn * 64 + 8 * cc;
}

template <int EPI, int TM, int TN, int WTM, int WTN>
__device__ __forceinline__ void gemm16_epilogue(const GemmArgs& g, void* c_out, int64_t c_ld, f32x4_t (&acc)[TM][TN], int m0, int n0,
                                                int wm, int wn, int lane, bf16x8_t* stage, bool rope = false) {
  const int mr = lane & 15, gq = lane >> 4;
  if constexpr (EPI == FASTAV_EPI_STORE && TN == 4) {
    if (rope) {
      // frequency index of this lane's first column in blocks 0 and 1; its four columns are consecutive
      const int half = g.rope_dh >> 1;
      const int f0 = (g.rope_dh == 128 ? 32 * (wn & 1) : 0) + gq * 4;
      const bool vec = g.vec_ok != 0;
      typedef uint32_t u32x2r_t __attribute__((ext_vector_type(2)));
      // all position ids first (one round trip for the whole tile), then the table rows they select
      int pos_i[TM];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row_l = m0 + wm * WTM + i * 16 + mr;
        pos_i[i] = g.rope_pos[row_l < g.M ? row_l : g.M - 1];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row_l = m0 + wm * WTM + i * 16 + mr;
        const float2* tr = g.rope_tab + (int64_t)pos_i[i] * half + f0;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
          const f32x4_t t01 = *(const f32x4_t*)(tr + jb * 16), t23 = *(const f32x4_t*)(tr + jb * 16 + 2);
          const float cs[4] = {t01[0], t01[2], t23[0], t23[2]}, sn[4] = {t01[1], t01[3], t23[1], t23[3]};
          float v1[4], v2[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float x1 = acc[i][jb][r], x2 = acc[i][jb + 2][r];
            v1[r] = x1 * cs[r] - x2 * sn[r];
            v2[r] = x2 * cs[r] + x1 * sn[r];
          }
          if (vec) {
            const u32x2r_t p1 = {pack_bf16(v1[0], v1[1]), pack_bf16(v1[2], v1[3])};
            const u32x2r_t p2 = {pack_bf16(v2[0], v2[1]), pack_bf16(v2[2], v2[3])};
            const int c1 = jb * 2 + (gq >> 1), c2 = (jb + 2) * 2 + (gq >> 1);
            *(u32x2r_t*)((char*)&stage[mr * 8 + (c1 ^ ((mr >> 1) & 7))] + (gq & 1) * 8) = p1;
            *(u32x2r_t*)((char*)&stage[mr * 8 + (c2 ^ ((mr >> 1) & 7))] + (gq & 1) * 8) = p2;
          } else if (row_l < g.M) {
            bf16_t* C1 = (bf16_t*)c_out + (int64_t)row_l * c_ld + rope_chunk_col(n0, wn, jb * 2 + (gq >> 1), g.rope_dh) + (gq & 1) * 4;
            bf16_t* C2 = (bf16_t*)c_out + (int64_t)row_l * c_ld + rope_chunk_col(n0, wn, (jb + 2) * 2 + (gq >> 1), g.rope_dh) + (gq & 1) * 4;
#pragma unroll
            for (int r = 0; r < 4; ++r) { C1[r] = (bf16_t)v1[r]; C2[r] = (bf16_t)v2[r]; }
          }
        }
        if (vec) {
          const int rr = lane >> 3, cc = lane & 7;
          const int col = rope_chunk_col(n0, wn, cc, g.rope_dh);
#pragma unroll
          for (int it = 0; it < 2; ++it) {
            const int r = it * 8 + rr;
            const u32x4_t val = *(const u32x4_t*)&stage[r * 8 + (cc ^ ((r >> 1) & 7))];
            const int row = m0 + wm * WTM + i * 16 + r;
            if (row < g.M) *(u32x4_t*)((bf16_t*)c_out + (int64_t)row * c_ld + col) = val;
          }
        }
      }
      return;
    }
  }
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
          if (row < g.M) unsafeAtomicAdd(&((float*)c_out)[(int64_t)row * c_ld + col], acc[i][j][r]);
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
            bf16_t* C = (bf16_t*)c_out + (int64_t)row * c_ld + colw + jb * 16 + gq * 4;
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
          if (row < g.M) *(u32x4_t*)((bf16_t*)c_out + (int64_t)row * c_ld + colw + cc * 8) = val;
        }
      }
    }
  } else {
    // fp32 output (residual read-modify-write, split-K partial): 16-byte pieces, TN * 4 of them per row
    constexpr int NC = TN * 4, RP = 64 / NC;
    static_assert(NC == 16 || NC == 32, "wave tile width");
    const bool vec = g.vec_ok != 0;
    float* Cb = (EPI == kEpiPartial) ? g.partial + (int64_t)blockIdx.y * g.M * g.N + n0 + wn * WTN : (float*)c_out + n0 + wn * WTN;
    const int64_t pitch = (EPI == kEpiPartial) ? g.N : c_ld;
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

template <int BM, int BN, int WM, int WN, int EPI, bool W3 = true>
__global__ __launch_bounds__(WM * WN * 64, ((W3 ? 2 : 3) * BM + (W3 ? 3 : 2) * BN) * 128 <= 80 * 1024 ? 2 : 1) void k_gemm_mfma16(GemmArgs g) {
  // W3: the weights (B) get the three slots and the early copies, the activations (A) the two slots and the copies
  // behind the barrier.  In a model's forward pass the weights always come from HBM (they are far larger than the
  // memory-side cache) and need the longer lead; the activations were written by the previous kernel.
  constexpr int NSA = W3 ? 2 : 3, NSB = W3 ? 3 : 2;    // LDS slots per operand
  constexpr int NW = WM * WN;                          // waves
  constexpr int WTM = BM / WM, WTN = BN / WN;          // wave tile
  constexpr int TM = WTM / 16, TN = WTN / 16;          // 16x16 blocks per wave
  constexpr int A_D = BM / (8 * NW), B_D = BN / (8 * NW);     // copy instructions per wave and stage (8 rows each)
  constexpr int D = A_D + B_D;
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  static_assert(A_D >= 1 && B_D >= 1 && TM >= 4 && TN >= 4 && TN % 4 == 0, "tile shape");
  extern __shared__ bf16x8_t lds[];                    // [NSA][BM*8] A, then [NSB][BN*8] B

  // ---- tile assignment: XCD-contiguous, banded
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
  int seg_start = 0, seg = 0;
  if (EPI != FASTAV_EPI_SWIGLU) {
    if (n0 >= g.seg_end[0]) { wbase = g.W[1]; seg_start = g.seg_end[0]; seg = 1; }
    if (n0 >= g.seg_end[1]) { wbase = g.W[2]; seg_start = g.seg_end[1]; seg = 2; }
  }

  // ---- this wave's copies: instruction i covers tile rows [(i*NW + wave)*8, +8), lane = (row, 16-byte chunk)
  const int drow = lane >> 3, dpos = lane & 7;
  uint32_t a_vo[A_D], b_vo[B_D];                        // lane offsets in bytes
  uint32_t a_dst[A_D], b_dst[B_D];                      // LDS byte address of the 8-row group in slot 0
  u32x4_t a_rs, b_rs[B_D];
  const uint32_t a_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  const uint32_t b_base = a_base + (uint32_t)NSA * BM * 128u;
  a_rs = make_rsrc(g.A + (g.a_rows ? (int64_t)0 : (int64_t)m0 * K) + kt0 * 64);
#pragma unroll
  for (int i = 0; i < A_D; ++i) {
    const int r0 = (i * NW + wave_u) * 8, row = r0 + drow;
    int grow = m0 + row;
    grow = grow < g.M ? grow : g.M - 1;                 // clamp: stay inside A, the epilogue masks the row
    // with a row list the lane offset addresses the source row from the start of A (the launcher checks that all of A
    // lies within the 32-bit offset range)
    const uint32_t arow = g.a_rows ? (uint32_t)g.a_rows[grow] : (uint32_t)(grow - m0);
    a_vo[i] = (arow * (uint32_t)K + (uint32_t)(dpos ^ ((row >> 1) & 7)) * 8u) * 2u;
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
      // RoPE epilogue on heads of 128 columns: 32-row blocks of every head are fetched in the order 0, 2, 1, 3
      int grow_b = row;
      if (EPI == FASTAV_EPI_STORE && g.rope_tab != nullptr && seg < g.rope_segs && g.rope_dh == 128) {
        const int q = row >> 5, q4 = q & 3;
        grow_b = (((q & ~3) | (q4 == 1 ? 2 : q4 == 2 ? 1 : q4)) << 5) | (row & 31);
      }
      b_vo[i] = ((uint32_t)grow_b * (uint32_t)K + (uint32_t)(dpos ^ ((row >> 1) & 7)) * 8u) * 2u;
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
    b_fu[ks] = NSA * BM * 8 + swz8(wn * WTN + frow, ks * 4 + fch);
  }
  auto mfma_block = [&](int i, int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      acc[i][j] = gemm_transposed(EPI) ? __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[ks][j], af[i], acc[i][j], 0, 0, 0)
                                       : __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[ks][j], acc[i][j], 0, 0, 0);
    }
  };
  // One stage.  `as`, `bs`: this stage's slots (t mod NSA, t mod NSB).  The operand with three slots ("early") has
  // its copies of stage t+2 issued during the first k-step, into the slot the previous stage freed; the operand
  // with two slots ("late") behind the barrier, into the slot this stage has just finished with.
  constexpr int PB = (TN + TM / 2 - 1) / (TM / 2);       // B fragments read behind one A block (first half of a k-step)
  constexpr int E_D = W3 ? B_D : A_D, L_D = W3 ? A_D : B_D;
  constexpr int PE = (E_D + TM - 2) / (TM - 1);          // early copies issued behind one A block of the first k-step
  constexpr int PL = (L_D + TM - 3) / (TM - 2);          // late copies issued behind one A block after the barrier
  auto stage = [&](int t, uint32_t as, uint32_t bs) __attribute__((always_inline)) {
    const uint32_t as1 = (as + 1u) % (uint32_t)NSA, bs1 = (bs + 1u) % (uint32_t)NSB;   // next stage's slots
    const uint32_t es2 = ((W3 ? bs : as) + 2u) % 3u;     // early operand's slot of stage t+2
    // k-step 0: after A block i is done its register takes the block's k-step-1 fragment; B's k-step-1 fragments
    // are read behind the first blocks; the early copies go out behind blocks 1, 2, ...
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      mfma_block(i, 0);
      af[i] = lds[a_fu[1] + (int)as * BM * 8 + i * 128];
      int nrd = 1;
#pragma unroll
      for (int j = i * PB; j < (i + 1) * PB && j < TN; ++j) { bfr[1][j] = lds[b_fu[1] + (int)bs * BN * 8 + j * 128]; ++nrd; }
      sched_block(TN, nrd);
      if (i >= 1 && (i - 1) * PE < E_D) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = (i - 1) * PE; c < i * PE && c < E_D; ++c) {
          if (W3) dma_b(t + 2, c < B_D ? c : 0, es2);
          else dma_a(t + 2, c < A_D ? c : 0, es2);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // k-step 1: two blocks, then - every fragment of this stage is in registers, stage t+1 has landed - the
    // barrier; from there on the freed registers take the next stage's k-step-0 fragments and the late copies of
    // stage t+2 go out
    mfma_block(0, 1);
    mfma_block(1, 1);
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * TN, 0);
    __builtin_amdgcn_sched_barrier(0);
    dma_wait_keep<E_D>();                                // stage t+1 has landed; only the early copies of stage t+2 may be in flight
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
      for (int j = (i - 2) * PB; j < (i - 1) * PB && j < TN; ++j) { bfr[0][j] = lds[b_fu[0] + (int)bs1 * BN * 8 + j * 128]; ++nrd; }
      sched_block(TN, nrd);
      if ((i - 2) * PL < L_D) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = (i - 2) * PL; c < (i - 1) * PL && c < L_D; ++c) {
          if (W3) dma_a(t + 2, c < A_D ? c : 0, as);
          else dma_b(t + 2, c < B_D ? c : 0, bs);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  static_assert(PB * (TM / 2) >= TN && PB * (TM - 2) >= TN && PE * (TM - 1) >= E_D && PL * (TM - 2) >= L_D, "schedule");

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
    for (int u = 0; u < 6; ++u) stage(t + u, (uint32_t)(u % NSA), (uint32_t)(u % NSB));
  }
#pragma unroll 1
  for (; t < KT; ++t) stage(t, (uint32_t)t % (uint32_t)NSA, (uint32_t)t % (uint32_t)NSB);
  dma_wait_keep<0>();
  __syncthreads();                                     // every wave's copies have landed: LDS is free for the epilogue
  void* c_out = g.C;
  int64_t c_ld = g.ldc;
  int n0e = n0;
  if (EPI == FASTAV_EPI_STORE && g.seg_out) { c_out = g.Cs[seg]; c_ld = g.ldcs[seg]; n0e = n0 - seg_start; }
  const bool rope = EPI == FASTAV_EPI_STORE && g.rope_tab != nullptr && seg < g.rope_segs;
  gemm16_epilogue<EPI, TM, TN, WTM, WTN>(g, c_out, c_ld, acc, m0, n0e, wm, wn, lane, lds + wave * (16 * 4 * TN), rope);
}

template <int BM, int BN, int WM, int WN, int EPI, bool W3 = true>
static fastav_status_t launch_cfg_16(GemmArgs g, int col0, int ncols, int splits, hipStream_t s) {
  constexpr int OUT_BN = (EPI == FASTAV_EPI_SWIGLU) ? BN / 2 : BN;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = ncols;
  g.n_off = col0 * OUT_BN;
  g.splits = splits;
  g.band = (g.tiles_m * g.tiles_n > kNumCUs) ? 4 : 1;
  const size_t shmem = (size_t)((W3 ? 2 : 3) * BM + (W3 ? 3 : 2) * BN) * 8 * sizeof(bf16x8_t);
  hipError_t e = hipFuncSetAttribute((const void*)k_gemm_mfma16<BM, BN, WM, WN, EPI, W3>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return fail(FASTAV_EHIP, "gemm: hipFuncSetAttribute: %s", hipGetErrorString(e));
  hipLaunchKernelGGL((k_gemm_mfma16<BM, BN, WM, WN, EPI, W3>), dim3((unsigned)(g.tiles_m * g.tiles_n), (unsigned)splits),
                     dim3(WM * WN * 64), shmem, s, g);
  return check_launch("gemm_mfma16");
}

bool mfma_linear_supported(int64_t m, int n, int k, int epilogue, int dtype) {
  if (dtype != FASTAV_BF16 || m < 1 || m > 0x7FFFFFFF) return false;
  if (k % 64 != 0 || k < 128) return false;            // whole stages of 64, at least two
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

fastav_status_t launch_splitk_reduce(float* r, int64_t ldc, const SplitKPending& p, hipStream_t s) {
  if (p.splits <= 0 || p.M == 0) return FASTAV_OK;
  const int64_t total = p.M * (p.N / 4);
  const unsigned blocks = (unsigned)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
  hipLaunchKernelGGL(k_splitk_reduce, dim3(blocks), dim3(256), 0, s, r, ldc, p.partial, (int)p.M, p.N, p.splits);
  return check_launch("splitk_reduce");
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
static fastav_status_t launch_epi(GemmArgs& g, bool big_ok, void* scratch, size_t scratch_bytes, hipStream_t s, SplitKPending* pend) {
  constexpr int OUT_BIG = (EPI == FASTAV_EPI_SWIGLU) ? 128 : 256, OUT_SMALL = OUT_BIG / 2;
  const int tm = (g.M + 255) / 256;
  const int tn = g.N / OUT_BIG;                         // tile columns of the 256 x 256 tiling (valid if big_ok)
  const int64_t tiles_big = (int64_t)tm * tn;
  if (!big_ok) return launch_cfg_16<128, 128, 2, 2, EPI>(g, 0, g.N / OUT_SMALL, 1, s);

  // Less than 3/4 of a round of 256 x 256 tiles: 192-row tiles if they fill the round better
  // (2458 rows x 4096 columns: 208 tiles instead of 160; O projection 106 -> 76 us, down projection 268 -> 223 us;
  // Q/K/V projection of 1721 rows: 216 tiles in one round instead of 672 small ones in 1.3)
  if ((EPI == FASTAV_EPI_RESADD || EPI == FASTAV_EPI_STORE) && tiles_big < (kCUs * 3) / 4) {
    const int64_t t192 = (int64_t)((g.M + 191) / 192) * tn;
    if (t192 <= kCUs && t192 >= (kCUs * 3) / 4) return launch_cfg_16<192, 256, 2, 4, EPI>(g, 0, tn, 1, s);
  }
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
      fastav_status_t st = launch_cfg_16<256, 256, 2, 4, kEpiPartial>(gp, 0, tn, best, s);
      if (st != FASTAV_OK) return st;
      if (pend != nullptr && g.ldc == g.N) {                 // the consumer adds the partial sums
        pend->partial = (const float*)scratch; pend->splits = best; pend->M = g.M; pend->N = g.N;
        return FASTAV_OK;
      }
      const int64_t total = (int64_t)g.M * (g.N / 4);
      const unsigned blocks = (unsigned)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
      hipLaunchKernelGGL(k_splitk_reduce, dim3(blocks), dim3(256), 0, s, (float*)g.C, g.ldc, (const float*)scratch, g.M, g.N, best);
      return check_launch("splitk_reduce");
    }
  }
  // small launches: 128 x 128 tiles, two workgroups per CU
  if (tiles_big < 192) return launch_cfg_16<128, 128, 2, 2, EPI>(g, 0, g.N / OUT_SMALL, 1, s);

  // Whole rounds of big tiles, then the leftover tile columns with 128 x 128 tiles (two workgroups per CU)
  // when the last round would leave half of the CUs or more idle: up to 512 small tiles still are one round, and
  // that round takes about 0.6 of a big one (QKV at 4096 tokens: 384 big tiles = 1 + 0.5 rounds, 175 -> ? us).
  const int64_t rem = tiles_big % kCUs;
  if (tiles_big > kCUs && rem != 0 && rem <= kCUs / 2) {
    const int cols_full = (int)((tiles_big - rem) / tm);          // whole tile columns inside the full rounds
    if (cols_full > 0 && cols_full < tn) {
      fastav_status_t st = launch_big<EPI>(g, 0, cols_full, tiles_big - rem, s);
      if (st != FASTAV_OK) return st;
      return launch_cfg_16<128, 128, 2, 2, EPI>(g, cols_full * 2, (tn - cols_full) * 2, 1, s);
    }
  }
  return launch_big<EPI>(g, 0, tn, tiles_big, s);
}

// Whether the plain-store epilogue can apply RoPE to the leading segments of this product: whole heads per wave
// tile, and only the tile shapes whose waves are 64 columns wide.
// A row list is addressed through the copies' 32-bit lane offsets from the start of A.
bool mfma_linear_takes_rows(int k, int64_t n_src) { return n_src > 0 && (n_src + 8) * (int64_t)k * 2 < ((int64_t)1 << 32); }

bool mfma_linear_fuses_rope(int64_t m, const int* seg_rows, int n_seg, int rope_segs, int k, int dh, int dtype) {
  if ((dh != 64 && dh != 128) || rope_segs < 1 || rope_segs > n_seg) return false;
  int n = 0;
  for (int i = 0; i < n_seg; ++i) {
    if (!mfma_linear_supported(m, seg_rows[i], k, FASTAV_EPI_STORE, dtype)) return false;
    if (seg_rows[i] % 128) return false;
    n += seg_rows[i];
  }
  return mfma_linear_supported(m, n, k, FASTAV_EPI_STORE, dtype);
}

fastav_status_t launch_linear_mfma(const void* a, const void* const* w_seg, const int* seg_rows, int n_seg,
                                   const void* w2, void* c, int64_t ldc, void* const* c_seg, const int64_t* ldc_seg,
                                   int64_t m, int n, int k, int epilogue, void* scratch, size_t scratch_bytes, hipStream_t s,
                                   const RopeFuse* rope, SplitKPending* pend, RowGather rows) {
  GemmArgs g;
  if (pend != nullptr) *pend = SplitKPending();
  g.a_rows = nullptr;
  if (rows.idx != nullptr) {
    if (!mfma_linear_takes_rows(k, rows.n_src)) return fail(FASTAV_EINVAL, "gemm: the row list needs all of A within 4 GB");
    g.a_rows = rows.idx;
  }
  g.rope_pos = nullptr; g.rope_tab = nullptr; g.rope_dh = 0; g.rope_segs = 0;
  if (rope != nullptr && rope->table != nullptr) {
    if (epilogue != FASTAV_EPI_STORE || !mfma_linear_fuses_rope(m, seg_rows, n_seg, rope->n_segs, k, rope->head_dim, FASTAV_BF16))
      return fail(FASTAV_EINVAL, "gemm: this product cannot take the RoPE epilogue");
    g.rope_pos = rope->pos; g.rope_tab = (const float2*)rope->table; g.rope_dh = rope->head_dim; g.rope_segs = rope->n_segs;
  }
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
  g.seg_out = 0;
  for (int i = 0; i < 3; ++i) { g.Cs[i] = c; g.ldcs[i] = ldc; }
  if (c_seg != nullptr) {
    if (epilogue != FASTAV_EPI_STORE) return fail(FASTAV_EINVAL, "gemm: per-segment outputs need the plain-store epilogue");
    g.seg_out = 1;
    g.vec_ok = 1;
    for (int i = 0; i < n_seg; ++i) {
      g.Cs[i] = c_seg[i]; g.ldcs[i] = ldc_seg[i];
      if ((uintptr_t)c_seg[i] % 16 != 0 || ldc_seg[i] % 8 != 0) g.vec_ok = 0;
    }
  }
  if (((uintptr_t)a | (uintptr_t)w_seg[0]) % 16) return fail(FASTAV_EINVAL, "gemm: A and W must be 16-byte aligned");
  if (epilogue == FASTAV_EPI_STORE) return launch_epi<FASTAV_EPI_STORE>(g, big_ok, scratch, scratch_bytes, s, nullptr);
  if (epilogue == FASTAV_EPI_RESADD) return launch_epi<FASTAV_EPI_RESADD>(g, big_ok, scratch, scratch_bytes, s, pend);
  return launch_epi<FASTAV_EPI_SWIGLU>(g, big_ok, scratch, scratch_bytes, s, nullptr);
}

}  // namespace fastav
