// Causal grouped-query flash attention for prefill on the CDNA4 matrix cores (bf16 in, fp32 accumulate),
// with the last-query logits of Eq. 4 as a side output.
//
// One workgroup = 128 query rows of one head of one sample; each of its 4 waves owns 32 rows.  K/V tiles
// of 64 keys are copied HBM/L2 -> LDS asynchronously (global_load_lds_dwordx4) one tile ahead of the math
// into one of two LDS stages, both row-major [key][d] and XOR-swizzled so that the operand reads spread over all 64
// LDS banks (K: 32 keys x one 16-byte chunk per MFMA operand; V: 4 keys x 32 bytes per 16 lanes of the
// transposing read below).  The products are formed transposed,
//     S^T = K Q^T   and   O^T = V^T P^T   (v_mfma_f32_32x32x16_bf16),
// so that in every accumulator a lane's column is ONE query row: the running max / sum of the softmax
// recurrence are per-lane scalars (one exchange per tile with the lane 32 away, which holds the other half
// of the keys), the rescale of O^T is a per-lane multiply, and exp2(S^T - m) converts in place into the B
// operand of the second product.  V^T operands come straight out of the row-major V tile through
// ds_read_b64_tr_b16: per 16 lanes it reads 4 keys x 16 dims and hands lane i the 4 keys of dim i.  The
// key order inside an MFMA k-step is the order the S^T accumulator holds them in; a sum does not care.
//
// The lane whose query is the last row of a sample also writes that row's scaled logits for every key
// and its final (max, sum): the fine-prune score is finalised from those without a second pass over K.
//
// A workgroup processes query tiles i and last - i one after the other, which gives every workgroup of a
// sample the same number of key tiles.  Workgroup ids are re-dealt so that the query heads that share a KV
// head run on one XCD and share its L2.
#include "common.hpp"

namespace fastav {

struct AttnArgs {
  const bf16_t* q; const bf16_t* k; const bf16_t* v; bf16_t* o;
  int64_t qs, kvs, os;                 // row strides in elements
  const int32_t* cu;
  int Hq, Hkv, n_qtiles, n_pairs;
  float scale, scale_log2;             // 1/sqrt(dh) and the same times log2(e)
  int64_t T;
  float* last_logits; float* last_ml;
};

typedef __attribute__((address_space(3))) bf16x4_t* lds_bf16x4_ptr;

// Asynchronous 16-byte global -> LDS copies (no VGPR staging, no ds_write); lane l's data lands at
// lds_byte_addr + 16 l.  Completion is tracked by vmcnt.  First form: per-lane 64-bit address.  Second form:
// wave-uniform base in SGPRs plus a per-lane 32-bit byte offset, which keeps the address arithmetic of a
// streaming copy on the scalar unit.
__device__ __forceinline__ void attn_dma16(const void* gptr, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_byte_addr) : "memory");
}
__device__ __forceinline__ void attn_dma16_sbase(const void* base, uint32_t voff, uint32_t lds_byte_addr) {
  // the base is wave-uniform by contract; say so, or the register allocator may leave it in VGPRs
  const uint64_t u = (uint64_t)(uintptr_t)base;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  const void* sbase = (const void*)(uintptr_t)(((uint64_t)hi << 32) | lo);
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(sbase), "s"(lds_byte_addr) : "memory");
}

// The vector ALU's issue port is what this kernel runs out of first (it also issues the matrix
// instructions), so the softmax recurrence is written to spend as few vector instructions per logit as it
// can: one fma + one exp2 per logit, one packed conversion and one packed dot product (the row sum) per two,
// one three-way max per two, and a rescale of the accumulators only when a row's max has moved by more than
// 2^8 since the last rescale (probabilities then stay below 256, exact in fp32 and harmless in bf16).
template <int DH>
__global__ __launch_bounds__(256, 2) void k_attn_mfma(AttnArgs a) {
  constexpr int BQ = 128, BKV = 64;
  constexpr int DCH = DH / 8;                       // 16-byte chunks per row
  constexpr int NS = DH / 16;                       // MFMA k-steps over the head dimension
  constexpr int NDB = DH / 32;                      // 32-row blocks of O^T
  // Swizzles (64 LDS banks of 4 bytes; a 16-byte access is served 16 lanes at a time, an 8-byte access 32):
  //   K: 16 consecutive keys reading the same logical chunk must hit 16 distinct 16-byte slots of the 256-byte
  //      bank window -> XOR the chunk with the key (rows of 256 B) or with key/2 (rows of 128 B).
  //   V: a transposing read touches, per 32 lanes, 4 keys x two 32-byte granules -> XOR the granule so the
  //      eight pieces fall in eight distinct 32-byte slots.
  auto kswz = [](int key, int c) { return DH == 128 ? (c ^ (key & 15)) : (c ^ ((key >> 1) & 7)); };
  auto vswz = [](int key, int c) { return DH == 128 ? (c ^ ((key & 3) << 2)) : (c ^ ((key & 2) << 1)); };
  extern __shared__ bf16x8_t attn_lds[];            // K stages then V stages: [2][BKV*DCH] each
  constexpr int TILE = BKV * DCH;                   // 16-byte chunks per tile

  // Work item = one (sample, head) pair x one PAIR of query tiles (i, last - i): under the causal mask tile i
  // sees i + 1 tiles' worth of keys, so every item of a sample carries the same amount of work and a launch
  // has no long tail.  When the KV groups divide evenly over the 8 XCDs (block id % 8 is the XCD), the query
  // heads of one KV head are placed on one XCD and share its L2.
  const int v = blockIdx.x;
  int pair, item;
  const int G = a.Hq / a.Hkv, n_groups = a.n_pairs / G;
  if (n_groups % 8 == 0) {
    // KV groups are dealt round-robin over the XCDs, so a batch of samples of different lengths loads them
    // evenly; the G query heads of a group stay together
    const int per = (n_groups / 8) * G, xcd = v % 8, idx = v / 8;
    const int pl = idx % per;
    pair = (xcd + 8 * (pl / G)) * G + pl % G;
    item = idx / per;
  } else {
    pair = v % a.n_pairs;
    item = v / a.n_pairs;
  }
  const int h = pair % a.Hq;
  const int b = pair / a.Hq;
  const int row0 = __builtin_amdgcn_readfirstlane(a.cu[b]);      // wave-uniform by construction: keep them in SGPRs
  const int n = __builtin_amdgcn_readfirstlane(a.cu[b + 1]) - row0;
  const int nq = (n + BQ - 1) / BQ;                               // this sample's query tiles
  if (item >= (nq + 1) / 2) return;
  const int g = h / G;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, so control flow stays scalar
  const int l32 = lane & 31, hf = lane >> 5;
  // first K / V row of this sample and KV head; rows are then addressed with 32-bit byte offsets (the
  // launcher checks that a sample's K/V rows span less than 2 GB)
  const char* kbase = (const char*)(a.k + (int64_t)row0 * a.kvs + g * DH);
  const char* vbase = (const char*)(a.v + (int64_t)row0 * a.kvs + g * DH);
  const uint32_t row_bytes = (uint32_t)a.kvs * 2u;

  // Tile copies.  A copy instruction fills 1 KB of LDS = RPI consecutive rows; wave w issues the row groups
  // w, w+4, ...  The XOR swizzles are applied on the global side: the lane that fills slot p of a row fetches
  // the logical chunk that belongs there (the swizzles are involutions in the chunk index).  The row group
  // goes into the scalar base; what is left per lane is one constant offset for K and one for V, because the
  // swizzles only look at key bits that the group index does not touch.
  constexpr int RPI = 64 / DCH;                      // rows per copy instruction
  constexpr int NCP = BKV / RPI / 4;                 // copy instructions per wave, per tile, for K and for V each
  const uint32_t k_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)attn_lds;
  const uint32_t v_lds = k_lds + 2u * TILE * 16u;
  const int cp_row = lane / DCH, cp_pos = lane % DCH;
  const uint32_t k_voff = (uint32_t)cp_row * row_bytes + (uint32_t)kswz(wave * RPI + cp_row, cp_pos) * 16u;
  const uint32_t v_voff = (uint32_t)cp_row * row_bytes + (uint32_t)vswz(cp_row, cp_pos) * 16u;
  // Rows past the sample are clamped to its last row (their probabilities are exactly 0 after masking, so
  // they only need to be finite); only the last tile of a sample takes that slower path.
  auto fetch = [&](int t, int st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NCP; ++i) {
      const int r0 = (i * 4 + wave) * RPI;
      const uint32_t dst = (uint32_t)(st * TILE + r0 * DCH) * 16u;
      if (t * BKV + BKV <= n) {
        const uint32_t off = (uint32_t)(t * BKV + r0) * row_bytes;
        attn_dma16_sbase(kbase + off, k_voff, k_lds + dst);
        attn_dma16_sbase(vbase + off, v_voff, v_lds + dst);
      } else {
        const int key = r0 + cp_row;
        const int jr = (t * BKV + key < n) ? t * BKV + key : n - 1;
        attn_dma16(kbase + (uint32_t)jr * row_bytes + kswz(key, cp_pos) * 16, k_lds + dst);
        attn_dma16(vbase + (uint32_t)jr * row_bytes + vswz(key, cp_pos) * 16, v_lds + dst);
      }
    }
  };
  auto fetch_wait = [&]() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); };

  // this lane's part of a transposing V read: 16 lanes cover 4 keys x 16 dims (two chunks)
  const int tr_krow = (lane & 15) >> 2;                          // which of the 4 keys this lane addresses
  const int tr_c0 = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);   // chunk inside the 32-dim block
  const int tr_e = (lane & 1) * 4;                               // element inside the chunk
  const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const bf16x2_t ones2 = {(bf16_t)1.0f, (bf16_t)1.0f};
  constexpr float kRescaleStep = 8.0f;              // log2 units a row's max may drift before O^T is rescaled

  // K operand of S^T = K Q^T: the 32 keys of half kb of the tile in stage st, k-step sI over the head dimension
  auto k_frag = [&](int st, int kb, int sI) __attribute__((always_inline)) -> bf16x8_t {
    const int key = kb * 32 + l32;
    return attn_lds[st * TILE + key * DCH + kswz(key, 2 * sI + hf)];
  };
  // V^T operand of O^T += V^T P^T for 16 keys (half kb, quarter sp) and 32 dims (block d):
  // slot e holds key 32kb + 16sp + (e/4)*8 + hf*4 + e%4
  auto v_frag = [&](int st, int kb, int sp, int d) __attribute__((always_inline)) -> bf16x8_t {
    const bf16_t* vtile = (const bf16_t*)(attn_lds + (2 + st) * TILE);
    bf16x8_t vf;
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2) {
      const int key = kb * 32 + sp * 16 + r2 * 8 + hf * 4 + tr_krow;      // key & 3 == tr_krow
      const int c = vswz(tr_krow, d * 4 + tr_c0);
      const bf16x4_t got = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(vtile + key * DH + c * 8 + tr_e));
      vf[4 * r2 + 0] = got[0]; vf[4 * r2 + 1] = got[1]; vf[4 * r2 + 2] = got[2]; vf[4 * r2 + 3] = got[3];
    }
    return vf;
  };

#pragma nounroll
  for (int part = 0; part < 2; ++part) {
  const int qt = part == 0 ? nq - 1 - item : item;                // the long tile first
  if (part == 1 && qt == nq - 1 - item) break;                    // odd count: the middle tile stands alone
  const int q0 = qt * BQ;
  const int qw0 = q0 + 32 * wave;
  const int qi = qw0 + l32;                                       // this lane's query row (in-sample)
  const bool wave_live = qw0 < n;

  bf16x8_t qf[NS];
  {
    const int qr = qi < n ? qi : n - 1;
    const bf16_t* qp = a.q + (int64_t)(row0 + qr) * a.qs + h * DH + hf * 8;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s] = *(const bf16x8_t*)(qp + 16 * s);
  }
  f32x16_t o[NDB];
#pragma unroll
  for (int d = 0; d < NDB; ++d) o[d] = zero16;
  // m: running max (log2 domain); m_ref: the value the stored probabilities and sums are relative to
  float m = -INFINITY, m_ref = -INFINITY, l = 0.f;
  const bool emit = (a.last_logits != nullptr) && (qi == n - 1);
  const bool emit_wave = __ballot(emit) != 0;                    // wave-uniform: some lane owns the sample's last row

  const int kv_end = (q0 + BQ < n) ? q0 + BQ : n;                // keys this workgroup can see
  const int n_tiles = (kv_end + BKV - 1) / BKV;
  // tiles this wave can see: those that start at or before its last query row, inside the sample
  const int my_tiles = wave_live ? (((qw0 + 32 < n) ? qw0 + 32 : n) + BKV - 1) / BKV : 0;

  // One tile for one wave; st is a literal at both call sites, so every LDS address below is a constant
  // offset from a loop-invariant register.
  auto tile_math = [&](int t, int st) __attribute__((always_inline)) {
    const int j0 = t * BKV;
    // ---- S^T = K Q^T : s[kb][r] is (key j0 + 32kb + (r/4)*8 + hf*4 + r%4, query qi); operand reads run two
    // matrix instructions ahead
    f32x16_t s[2];
    bf16x8_t fr[4];
    fr[0] = k_frag(st, 0, 0);
    fr[1] = k_frag(st, 1, 0);
#pragma unroll
    for (int i = 0; i < 2 * NS; ++i) {
      if (i + 2 < 2 * NS) fr[(i + 2) % 3] = k_frag(st, (i + 2) & 1, (i + 2) >> 1);
      s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % 3], qf[i >> 1], i < 2 ? zero16 : s[i & 1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // The vector phase runs at raised wave priority: the SIMD's other wave is then mostly in a matrix phase, whose
    // instructions each keep the matrix pipe busy for 32 clocks and lose nothing by issuing a few clocks later, while
    // every issue slot this phase loses to them is time nobody gets back (measured: 169 -> 157 us at 4096 tokens,
    // 2.04 -> 1.95 ms at 16384; raising the matrix phases instead gains nothing).
    __builtin_amdgcn_s_setprio(1);
    // first V operands: their latency hides behind the softmax arithmetic
    constexpr int NPV = 4 * NDB;
    constexpr int PD = 3;
#pragma unroll
    for (int i = 0; i < PD; ++i) fr[i] = v_frag(st, i / (2 * NDB), (i / NDB) & 1, i % NDB);
    if (emit_wave) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + kb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
          if (emit && key <= qi) a.last_logits[(int64_t)h * a.T + row0 + key] = s[kb][r] * a.scale;
        }
    }
    if ((j0 + BKV - 1 > qw0) || (j0 + BKV > n)) {                 // diagonal or ragged tile: mask (wave-uniform test)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + kb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
          if (!(key <= qi && key < n)) s[kb][r] = -INFINITY;
        }
    }
    // max over the raw products (the scale is positive): a tree of three-way maxima, then the other half of
    // the keys from the lane 32 away
    float mx;
    {
      // four chains of three-way maxima (v_max3_f32), two new logits per instruction
      float c4[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        c4[c] = fmaxf(fmaxf(s[c >> 1][8 * (c & 1)], s[c >> 1][8 * (c & 1) + 1]), s[c >> 1][8 * (c & 1) + 2]);
        c4[c] = fmaxf(fmaxf(c4[c], s[c >> 1][8 * (c & 1) + 3]), s[c >> 1][8 * (c & 1) + 4]);
        c4[c] = fmaxf(fmaxf(c4[c], s[c >> 1][8 * (c & 1) + 5]), s[c >> 1][8 * (c & 1) + 6]);
        c4[c] = fmaxf(c4[c], s[c >> 1][8 * (c & 1) + 7]);
      }
      mx = fmaxf(fmaxf(fmaxf(c4[0], c4[1]), c4[2]), c4[3]);
      const unsigned bits = __float_as_uint(mx);
      const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
      mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    m = fmaxf(m, mx * a.scale_log2);
    if (__ballot(m > m_ref + kRescaleStep) != 0) {                 // also taken on the first tile (m_ref = -inf)
      const float m_to = (m > m_ref + kRescaleStep) ? m : m_ref;
      const float alpha = __builtin_amdgcn_exp2f(m_ref - m_to);    // 1 for the rows that stay
      m_ref = m_to;
      l *= alpha;
#pragma unroll
      for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
    }
    bf16x8_t pb[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        bf16x2_t pr;                                               // exp2(-inf) = 0 for masked keys
        pr[0] = (bf16_t)__builtin_amdgcn_exp2f(fmaf(s[kb][r], a.scale_log2, -m_ref));
        pr[1] = (bf16_t)__builtin_amdgcn_exp2f(fmaf(s[kb][r + 1], a.scale_log2, -m_ref));
        l = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, l, false);  // row sum of the rounded probabilities
        pb[kb][r >> 3][r & 7] = pr[0];
        pb[kb][r >> 3][(r & 7) + 1] = pr[1];
      }
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    // ---- O^T += V^T P^T over the k-steps (kb, sp); operand reads run three matrix instructions ahead
#pragma unroll
    for (int i = 0; i < NPV; ++i) {
      const int j = i + PD;
      if (j < NPV) fr[j % 4] = v_frag(st, j / (2 * NDB), (j / NDB) & 1, j % NDB);
      o[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % 4], pb[i / (2 * NDB)][(i / NDB) & 1], o[i % NDB], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto tile_step = [&](int t, int st) __attribute__((always_inline)) {
    if (t + 1 < n_tiles) fetch(t + 1, st ^ 1);                   // stage st^1 was last read before the previous barrier
    if (t < my_tiles) tile_math(t, st);
    fetch_wait();
    __syncthreads();
  };

  fetch(0, 0);
  fetch_wait();
  __syncthreads();
  for (int t = 0; t < n_tiles; t += 2) {
    tile_step(t, 0);
    if (t + 1 < n_tiles) tile_step(t + 1, 1);
  }

  // ---- normalise and store.  o[d][r] is (dim 32d + (r/4)*8 + hf*4 + r%4, query qi).
  const auto lsw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l), __float_as_uint(l), false, false);
  const float l_tot = __uint_as_float(lsw[0]) + __uint_as_float(lsw[1]);
  if (qi < n) {
    const float inv = 1.0f / l_tot;
    bf16_t* op = a.o + (int64_t)(row0 + qi) * a.os + h * DH + hf * 4;
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4_t w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (bf16_t)(o[d][4 * r4 + e] * inv);
        *(bf16x4_t*)(op + d * 32 + r4 * 8) = w;
      }
    if (emit && hf == 0 && a.last_ml) {
      // (max, sum of exp relative to the max), back from the log2 domain
      a.last_ml[((int64_t)b * a.Hq + h) * 2] = m * 0.6931471805599453f;
      a.last_ml[((int64_t)b * a.Hq + h) * 2 + 1] = l_tot * __builtin_amdgcn_exp2f(m_ref - m);
    }
  }
  __syncthreads();                                               // the next part's first copy reuses stage 0
  }  // part
}

bool mfma_attention_supported(int dh, int dtype, int64_t q_stride, int64_t kv_stride, int64_t o_stride, int max_seqlen) {
  // the tile copies address a sample's K / V rows with 32-bit byte offsets
  return dtype == FASTAV_BF16 && (dh == 64 || dh == 128) && q_stride % 8 == 0 && kv_stride % 8 == 0 && o_stride % 4 == 0 &&
         ((int64_t)max_seqlen + 64) * kv_stride * 2 < ((int64_t)1 << 31);
}

fastav_status_t launch_attention_mfma(const void* q, int64_t q_stride, const void* k, const void* v,
                                      int64_t kv_stride, void* o, int64_t o_stride, const int32_t* cu, int batch,
                                      int64_t T, int max_seqlen, int Hq, int Hkv, int dh, float* last_logits,
                                      float* last_ml, hipStream_t s) {
  if (batch == 0 || max_seqlen == 0) return FASTAV_OK;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v) % 16 || ((uintptr_t)o % 8))
    return fail(FASTAV_EINVAL, "attention: q, k, v must be 16-byte aligned and o 8-byte aligned");
  AttnArgs a;
  a.q = (const bf16_t*)q; a.k = (const bf16_t*)k; a.v = (const bf16_t*)v; a.o = (bf16_t*)o;
  a.qs = q_stride; a.kvs = kv_stride; a.os = o_stride; a.cu = cu; a.Hq = Hq; a.Hkv = Hkv;
  a.n_qtiles = (max_seqlen + 127) / 128;
  a.n_pairs = Hq * batch;
  const int64_t blocks = (int64_t)((a.n_qtiles + 1) / 2) * a.n_pairs;       // balanced pairs of query tiles
  if (blocks > 0x7FFFFFFF) return fail(FASTAV_EUNSUPPORTED, "attention: too many workgroups");
  a.scale = 1.0f / sqrtf((float)dh);
  a.scale_log2 = a.scale * 1.4426950408889634f;
  a.T = T; a.last_logits = last_logits; a.last_ml = last_ml;
  // two stages of a 64-key K tile and V tile
  if (dh == 128) hipLaunchKernelGGL(k_attn_mfma<128>, dim3((unsigned)blocks), dim3(256), 4 * 64 * 128 * 2, s, a);
  else hipLaunchKernelGGL(k_attn_mfma<64>, dim3((unsigned)blocks), dim3(256), 4 * 64 * 64 * 2, s, a);
  return check_launch("attention_mfma");
}

}  // namespace fastav
