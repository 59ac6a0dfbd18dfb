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
// sample the same number of key tiles.  Workgroup ids are re-dealt so that each XCD owns a contiguous run of
// heads: the query heads that share a KV head then share an L2.
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

// Asynchronous 16-byte global -> LDS copy (no VGPR staging, no ds_write); lane l's data lands at
// lds_byte_addr + 16 l.  Completion is tracked by vmcnt.
__device__ __forceinline__ void attn_dma16(const void* gptr, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_byte_addr) : "memory");
}

template <int DH>
__global__ __launch_bounds__(256, 2) void k_attn_mfma(AttnArgs a) {
  constexpr int BQ = 128, BKV = 64;
  constexpr int DCH = DH / 8;                       // 16-byte chunks per row
  constexpr int NS = DH / 16;                       // MFMA k-steps over the head dimension
  constexpr int NDB = DH / 32;                      // 32-row blocks of O^T
  constexpr int NLD = BKV * DCH / 256;              // 16-byte chunks per thread per tile (K and V each)
  // Swizzles (64 LDS banks of 4 bytes; a 16-byte access is served 16 lanes at a time, an 8-byte access 32):
  //   K: 16 consecutive keys reading the same logical chunk must hit 16 distinct 16-byte slots of the 256-byte
  //      bank window -> XOR the chunk with the key (rows of 256 B) or with key/2 (rows of 128 B).
  //   V: a transposing read touches, per 32 lanes, 4 keys x two 32-byte granules -> XOR the granule so the
  //      eight pieces fall in eight distinct 32-byte slots.
  auto kswz = [](int key, int c) { return DH == 128 ? (c ^ (key & 15)) : (c ^ ((key >> 1) & 7)); };
  auto vswz = [](int key, int c) { return DH == 128 ? (c ^ ((key & 3) << 2)) : (c ^ ((key & 2) << 1)); };
  extern __shared__ bf16x8_t attn_lds[];            // K stages then V stages: [2][BKV*DCH] each
  bf16x8_t (*Ks)[BKV * DCH] = (bf16x8_t (*)[BKV * DCH])attn_lds;
  bf16x8_t (*Vs)[BKV * DCH] = (bf16x8_t (*)[BKV * DCH])(attn_lds + 2 * BKV * DCH);

  // Work item = one (sample, head) pair x one PAIR of query tiles (i, last - i): under the causal mask tile i
  // sees i + 1 tiles' worth of keys, so every item of a sample carries the same amount of work and a launch
  // has no long tail.  When the (sample, head) pairs divide evenly over the 8 XCDs (block id % 8 is the XCD),
  // each XCD owns a contiguous run of them: the query heads of one KV head share an L2.
  const int v = blockIdx.x;
  int pair, item;
  if (a.n_pairs % 8 == 0) {
    const int per = a.n_pairs / 8, xcd = v % 8, idx = v / 8;
    pair = xcd * per + idx % per;
    item = idx / per;
  } else {
    pair = v % a.n_pairs;
    item = v / a.n_pairs;
  }
  const int h = pair % a.Hq;
  const int b = pair / a.Hq;
  const int row0 = a.cu[b], n = a.cu[b + 1] - row0;
  const int nq = (n + BQ - 1) / BQ;                               // this sample's query tiles
  if (item >= (nq + 1) / 2) return;
  const int g = h / (a.Hq / a.Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
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
  for (int d = 0; d < NDB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m = -INFINITY, l = 0.f;
  const bool emit = (a.last_logits != nullptr) && (qi == n - 1);
  const bool emit_wave = __ballot(emit) != 0;                    // wave-uniform: some lane owns the sample's last row

  const int kv_end = (q0 + BQ < n) ? q0 + BQ : n;                // keys this workgroup can see
  const int n_tiles = (kv_end + BKV - 1) / BKV;
  const bf16_t* kbase = a.k + (int64_t)row0 * a.kvs + g * DH;
  const bf16_t* vbase = a.v + (int64_t)row0 * a.kvs + g * DH;

  // Tile copies: a copy instruction fills 1 KB of LDS = RPI consecutive tile rows; wave w issues the groups
  // w, w+4, ...  The XOR swizzles are applied on the global side: the lane that fills slot p of row `key`
  // fetches the logical chunk that belongs there.  Rows past the sample are clamped to its last row (their
  // probabilities are exactly 0 after masking, so they only need to be finite).
  constexpr int RPI = 64 / DCH;                      // tile rows per copy instruction
  constexpr int NCP = BKV / RPI / 4;                 // copy instructions per wave, per tile, for K and for V each
  const uint32_t k_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)attn_lds;
  const uint32_t v_lds = k_lds + 2u * BKV * DCH * 16u;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int cp_row = lane / DCH, cp_pos = lane % DCH;
  auto fetch = [&](int j0, int st) {
#pragma unroll
    for (int i = 0; i < NCP; ++i) {
      const int r0 = (i * 4 + wave_u) * RPI;
      const int key = r0 + cp_row;
      const int jr = (j0 + key < n) ? j0 + key : n - 1;
      const uint32_t dst = (uint32_t)(st * BKV * DCH + r0 * DCH) * 16u;
      // kswz / vswz are involutions in the chunk index
      attn_dma16(kbase + (int64_t)jr * a.kvs + kswz(key, cp_pos) * 8, k_lds + dst);
      attn_dma16(vbase + (int64_t)jr * a.kvs + vswz(key, cp_pos) * 8, v_lds + dst);
    }
  };
  auto fetch_wait = [&]() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); };
  fetch(0, 0);
  fetch_wait();
  __syncthreads();

  // this lane's part of a transposing V read: 16 lanes cover 4 keys x 16 dims (two chunks)
  const int tr_krow = (lane & 15) >> 2;                          // which of the 4 keys this lane addresses
  const int tr_c0 = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);   // chunk inside the 32-dim block
  const int tr_e = (lane & 1) * 4;                               // element inside the chunk

  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = t * BKV;
    const int st = t & 1;
    if (t + 1 < n_tiles) fetch(j0 + BKV, st ^ 1);           // stage st^1 was last read before the previous barrier

    if (wave_live && j0 <= qw0 + 31) {                            // else nothing visible to this wave in this tile
      // ---- S^T = K Q^T : s[kb][r] is (key j0 + 32kb + (r/4)*8 + hf*4 + r%4, query qi)
      f32x16_t s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
      }
#pragma unroll
      for (int sI = 0; sI < NS; ++sI) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const int key = kb * 32 + l32;
          const bf16x8_t kf = Ks[st][key * DCH + kswz(key, 2 * sI + hf)];
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[sI], s[kb], 0, 0, 0);
        }
      }
      if (emit_wave) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = j0 + kb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
            if (emit && key <= qi) a.last_logits[(int64_t)h * a.T + row0 + key] = s[kb][r] * a.scale;
          }
      }
      // max over the raw products (the scale is positive); masked entries become -inf
      float mx = -INFINITY;
      if ((j0 + BKV - 1 > qw0) || (j0 + BKV > n)) {                // diagonal or ragged tile: mask (wave-uniform test)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = j0 + kb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
            if (!(key <= qi && key < n)) s[kb][r] = -INFINITY;
            mx = fmaxf(mx, s[kb][r]);
          }
      } else {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      const float m_new = fmaxf(m, mx * a.scale_log2);            // running max in the log2 domain
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      if (__ballot(m_new > m) != 0) {                              // rescale only when some row's max moved
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);
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
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[kb][r], a.scale_log2, -m_use));   // exp2(-inf) = 0 for masked keys
          l += p;
          pb[kb][r >> 3][r & 7] = (bf16_t)p;
        }
      m = m_new;

      // ---- O^T += V^T P^T : k-step (kb, sp), slot e holds key 32kb + 16sp + (e/4)*8 + hf*4 + e%4
      const bf16_t* vtile = (const bf16_t*)Vs[st];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
#pragma unroll
          for (int d = 0; d < NDB; ++d) {
            bf16x8_t vf;
#pragma unroll
            for (int r2 = 0; r2 < 2; ++r2) {
              const int key = kb * 32 + sp * 16 + r2 * 8 + hf * 4 + tr_krow;      // key & 3 == tr_krow
              const int c = vswz(tr_krow, d * 4 + tr_c0);
              const bf16x4_t got = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                  (lds_bf16x4_ptr)(vtile + key * DH + c * 8 + tr_e));
              vf[4 * r2 + 0] = got[0]; vf[4 * r2 + 1] = got[1]; vf[4 * r2 + 2] = got[2]; vf[4 * r2 + 3] = got[3];
            }
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[kb][sp], o[d], 0, 0, 0);
          }
        }
    }

    fetch_wait();
    __syncthreads();
  }

  // ---- normalise and store.  o[d][r] is (dim 32d + (r/4)*8 + hf*4 + r%4, query qi).
  const float l_tot = l + __shfl_xor(l, 32, kWave);
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
      a.last_ml[((int64_t)b * a.Hq + h) * 2] = m * 0.6931471805599453f;     // back from the log2 domain
      a.last_ml[((int64_t)b * a.Hq + h) * 2 + 1] = l_tot;
    }
  }
  }  // part
}

bool mfma_attention_supported(int dh, int dtype, int64_t q_stride, int64_t kv_stride, int64_t o_stride) {
  return dtype == FASTAV_BF16 && (dh == 64 || dh == 128) && q_stride % 8 == 0 && kv_stride % 8 == 0 && o_stride % 4 == 0;
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
