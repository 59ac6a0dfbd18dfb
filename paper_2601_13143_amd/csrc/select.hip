// Top-k selection and compaction for the prune step (Section 2.2, "Fine pruning" / Eq. 4: the lowest-scoring
// share P of the tokens goes; global pruning keeps the earliest positions instead; the other strategies of
// Tables 2-3 - top attentive, top informative, random - are further orders of the same kernel).
//
//   k_select  one 1024-thread workgroup per sample.  The sample's order-preserving 32-bit keys live in LDS;
//             four 8-bit MSB-first radix passes (per-wave LDS histograms, so that the narrow exponent range
//             of softmax scores does not serialise on one counter) find the k-th largest key; ties at
//             the threshold go to the lowest indices; one workgroup scan (two where the keys do not fit in
//             LDS) turns the keep flags into the ascending list of kept rows.  The positional orders need no
//             radix pass: all candidates tie, and the tie rule by rank in row order is the selection.
//             Integer work only, so the result is exact.
//   k_gather  dst[r] = src[keep_idx[r]] for several tensors in one launch, 16 bytes per lane.
#include "common.hpp"

namespace fastav {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelLdsKeys = 32768;          // samples up to this length keep their keys in LDS (128 KB)
constexpr int kSelMaxHeads = 128;           // most query heads the fused Eq. 4 finish holds (max, 1/sum) for

// fp32 -> unsigned key, larger key = better.  NaN ranks as -inf; -0.0 equals +0.0.
__device__ __forceinline__ uint32_t score_key(float s) {
  if (s != s) s = -INFINITY;
  if (s == 0.0f) s = 0.0f;
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_tot, int& total) {
  // inclusive scan inside the wave
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += t;
  }
  __syncthreads();                          // wave_tot may still be read from a previous scan
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = wave_tot[w];
    if (w < wave) base += t;
    tot += t;
  }
  total = tot;
  return base + inc - v;
}

// 32-bit avalanche mix (xor-shift 16, multiply, xor-shift 13, multiply, xor-shift 16): the finishing step of the
// published MurmurHash3 hash, a bijection on 32-bit words.
__host__ __device__ __forceinline__ uint32_t mix32(uint32_t h) {
  h ^= h >> 16; h *= 0x85EBCA6Bu;
  h ^= h >> 13; h *= 0xC2B2AE35u;
  h ^= h >> 16;
  return h;
}
constexpr uint32_t kGolden = 0x9E3779B9u;

uint32_t select_random_key(uint32_t seed, int layer) { return mix32(seed + kGolden * (uint32_t)(layer + 1)); }

// Key of candidate j (unprotected row) of sample b under the rule's order; never 0.
// Random order: the draw is the top 24 bits of mix32(mix32(key + G (b + 1)) + position id) as a fraction in
// [0, 1), ranked like a score, so that a token's draw does not depend on what was pruned before it.
__device__ __forceinline__ uint32_t cand_key_of(const SelectRule& r, float score, uint32_t sample_key, int row0, int n, int j) {
  switch (r.order) {
    case kSelHighScore: return score_key(score);
    case kSelLowScore: return score_key(-score);
    case kSelEarliest:
    case kSelLatest: return 1u;                                         // positional orders: decided by candidate rank, below
    default: {
      const uint32_t p = r.pos ? (uint32_t)r.pos[row0 + j] : (uint32_t)j;
      return score_key((float)(mix32(sample_key + p) >> 8) * 0x1p-24f);
    }
  }
}
__device__ __forceinline__ uint32_t cand_key(const SelectRule& r, const float* scores, uint32_t sample_key, int row0,
                                             int n, int j) {
  const bool by_score = r.order == kSelHighScore || r.order == kSelLowScore;
  return cand_key_of(r, by_score ? scores[row0 + j] : 0.f, sample_key, row0, n, j);
}

template <bool KEYS_IN_LDS>
__global__ __launch_bounds__(kSelThreads) void k_select(const float* __restrict__ scores,
                                                        const uint8_t* __restrict__ prot,
                                                        const int32_t* __restrict__ cu,
                                                        const int32_t* __restrict__ cu_out,
                                                        int32_t* __restrict__ keep_idx, SelectRule rule) {
  extern __shared__ __align__(16) uint32_t keys[];                      // [n] when KEYS_IN_LDS; key 0 = protected (never a candidate)
  __shared__ int hist[kSelWaves][256];
  __shared__ int wave_tot[kSelWaves];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_need;

  const int b = blockIdx.x;
  const int row0 = cu[b], n = cu[b + 1] - row0;
  const int out0 = cu_out[b], k_keep = cu_out[b + 1] - out0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (n <= 0) return;
  const uint32_t sample_key = mix32(rule.key + kGolden * (uint32_t)(b + 1));

  // ---- load keys, count protected rows.  With the attention side output at hand (rule.logits: the last query
  // row's scaled logits per head, rule.ml: that row's (max, sum of exp) per head) Eq. 4 is finished right here -
  // s_j = 1/Hq sum_h exp(L[h][j] - m_h) / l_h, the terms added in head order exactly as k_score_finalize adds them
  // - and goes straight into the key array (and to rule.scores_out for the caller), which saves a launch per prune.
  int my_prot = 0;
  if (KEYS_IN_LDS && rule.logits != nullptr) {
    __shared__ float sh_ml[2 * kSelMaxHeads];
    for (int h = tid; h < rule.n_heads; h += kSelThreads) {
      const float* pm = rule.ml + ((int64_t)b * rule.n_heads + h) * 2;
      sh_ml[2 * h] = pm[0]; sh_ml[2 * h + 1] = 1.0f / pm[1];
    }
    __syncthreads();
    // Two rows per round and sixteen heads per batch: 32 independent loads in flight per thread (the planes of the
    // heads are T floats apart, so every load is a trip to L2 or beyond, and one workgroup has to cover the whole
    // sample).  A row's terms are still added in head order.
    for (int j = tid; j < n; j += 2 * kSelThreads) {
      const int j1 = j + kSelThreads;
      const bool two = j1 < n;
      const float* lp0 = rule.logits + row0 + j;
      const float* lp1 = rule.logits + row0 + (two ? j1 : j);
      float sc0 = 0.f, sc1 = 0.f;
      for (int h0 = 0; h0 < rule.n_heads; h0 += 16) {
        float g0[16], g1[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          const int h = (h0 + u < rule.n_heads) ? h0 + u : rule.n_heads - 1;
          g0[u] = lp0[(int64_t)h * rule.T];
          g1[u] = lp1[(int64_t)h * rule.T];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          if (h0 + u < rule.n_heads) {
            sc0 = fmaf(expf(g0[u] - sh_ml[2 * (h0 + u)]), sh_ml[2 * (h0 + u) + 1], sc0);
            sc1 = fmaf(expf(g1[u] - sh_ml[2 * (h0 + u)]), sh_ml[2 * (h0 + u) + 1], sc1);
          }
        }
      }
      sc0 = sc0 / (float)rule.n_heads;
      sc1 = sc1 / (float)rule.n_heads;
      {
        const bool p = prot[row0 + j] != 0;
        my_prot += p ? 1 : 0;
        if (rule.scores_out) rule.scores_out[row0 + j] = sc0;
        keys[j] = p ? 0u : cand_key_of(rule, sc0, sample_key, row0, n, j);
      }
      if (two) {
        const bool p = prot[row0 + j1] != 0;
        my_prot += p ? 1 : 0;
        if (rule.scores_out) rule.scores_out[row0 + j1] = sc1;
        keys[j1] = p ? 0u : cand_key_of(rule, sc1, sample_key, row0, n, j1);
      }
    }
  } else {
    for (int j = tid; j < n; j += kSelThreads) {
      const bool p = prot[row0 + j] != 0;
      my_prot += p ? 1 : 0;
      if (KEYS_IN_LDS) keys[j] = p ? 0u : cand_key(rule, scores, sample_key, row0, n, j);
    }
  }
  int n_prot;
  block_exclusive_scan(my_prot, wave_tot, n_prot);
  int need = k_keep - n_prot;                             // candidates to keep
  if (need < 0) need = 0;
  const int n_cand = n - n_prot;
  if (need > n_cand) need = n_cand;

  // ---- radix select: largest `need` candidate keys.  After the passes: threshold key `prefix`,
  //      `need_eq` = how many candidates equal to the threshold are kept (lowest indices first).
  uint32_t prefix = 0, mask = 0;
  int need_eq = need;
  int eq_lo = 0;                                          // candidates equal to the threshold are kept from this rank on
  const bool positional = rule.order == kSelEarliest || rule.order == kSelLatest;
  if (positional && need > 0 && need < n_cand) {
    // every candidate carries the same key: the first (earliest) or the last (latest) `need` of them in row order are
    // kept by the rank rule alone, no pass over the keys is needed
    prefix = 1u; mask = 0xFFFFFFFFu;
    eq_lo = rule.order == kSelLatest ? n_cand - need : 0;
  } else if (need > 0 && need < n_cand) {
    for (int shift = 24; shift >= 0; shift -= 8) {
      for (int i = tid; i < kSelWaves * 256; i += kSelThreads) (&hist[0][0])[i] = 0;
      __syncthreads();
      for (int j = tid; j < n; j += kSelThreads) {
        uint32_t key;
        if (KEYS_IN_LDS) key = keys[j];
        else key = prot[row0 + j] ? 0u : cand_key(rule, scores, sample_key, row0, n, j);
        if (key != 0u && (key & mask) == prefix) atomicAdd(&hist[wave][(key >> shift) & 255u], 1);
      }
      __syncthreads();
      if (wave == 0) {
        // lane owns digits 4*lane .. 4*lane+3; walk from the top digit down until `need_eq` is covered
        int c[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          int t = 0;
          for (int w = 0; w < kSelWaves; ++w) t += hist[w][4 * lane + d];
          c[d] = t;
        }
        const int mine = c[0] + c[1] + c[2] + c[3];
        // suffix sum over lanes: above = total count of digits owned by higher lanes
        int suf = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int t = __shfl_down(suf, o, kWave);
          if (lane + o < 64) suf += t;
        }
        int above = suf - mine;
        // the lane whose range crosses need_eq finds the digit
        if (above < need_eq && need_eq <= suf) {
          int d = 3;
          for (; d >= 0; --d) {
            if (above + c[d] >= need_eq) break;
            above += c[d];
          }
          sh_prefix = prefix | ((uint32_t)(4 * lane + d) << shift);
          sh_need = need_eq - above;                     // still to take among keys with this digit
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      need_eq = sh_need;
      mask |= 255u << shift;
      __syncthreads();
    }
  } else if (need == 0) {
    prefix = 0xFFFFFFFFu; mask = 0xFFFFFFFFu; need_eq = 0;   // no candidate passes (keys never reach 0xFFFFFFFF+)
  } else {
    prefix = 0; mask = 0xFFFFFFFFu; need_eq = 0;             // need == n_cand: every candidate key (> 0) passes
  }
  // keep candidate j  <=>  key > prefix, or key == prefix and it is among the first need_eq such rows.
  const bool take_all = (need == n_cand), take_none = (need == 0);

  // ---- flags and ordered output.  Thread t owns the contiguous rows [t*per, (t+1)*per).
  auto keeps = [&](uint32_t key, int& e) __attribute__((always_inline)) -> bool {
    if (key == 0u) return true;                            // protected
    if (take_all) return true;
    if (take_none) return false;
    if (key > prefix) return true;
    if (key == prefix) { const bool kp = e >= eq_lo && e < eq_lo + need_eq; ++e; return kp; }
    return false;
  };
  if constexpr (KEYS_IN_LDS) {
    // The thread's rows come out of LDS once, 16 bytes per read (`per` is rounded up to a multiple of four, so every
    // thread starts on a 16-byte boundary; word-by-word reads at a stride of `per` words would pile a wave's lanes
    // on a few banks).  One scan carries both running counts: the rows kept for sure (protected, or above the
    // threshold) in the low half and the rows equal to the threshold in the high half - either total is at most
    // kSelLdsKeys = 2^15, so the halves do not run into each other.
    constexpr int kMaxPer = kSelLdsKeys / kSelThreads;
    static_assert(kMaxPer % 4 == 0 && kSelLdsKeys <= 32768, "packed scan");
    const int per = ((n + kSelThreads - 1) / kSelThreads + 3) & ~3;
    const int j_lo = tid * per;
    uint32_t kr[kMaxPer];
#pragma unroll
    for (int i = 0; i < kMaxPer; i += 4) {
      if (i < per) {
        const int j = j_lo + i;
        if (j + 3 < n) {
          const uint4 v = *(const uint4*)(keys + j);
          kr[i] = v.x; kr[i + 1] = v.y; kr[i + 2] = v.z; kr[i + 3] = v.w;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) kr[i + e] = (j + e < n) ? keys[j + e] : 0u;
        }
      }
    }
    int sure = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < kMaxPer; ++i) {
      if (i < per && j_lo + i < n) {
        const uint32_t key = kr[i];
        const bool cand = key != 0u;
        eq += (cand && !take_all && !take_none && key == prefix) ? 1 : 0;
        sure += (!cand || take_all || (!take_none && key > prefix)) ? 1 : 0;
      }
    }
    int dummy;
    const uint32_t before = (uint32_t)block_exclusive_scan((int)(((uint32_t)eq << 16) | (uint32_t)sure), wave_tot, dummy);
    const int eq_before = (int)(before >> 16), sure_before = (int)(before & 0xFFFFu);
    const int eq_kept_before = eq_before - eq_lo < 0 ? 0 : (eq_before - eq_lo < need_eq ? eq_before - eq_lo : need_eq);
    int e = eq_before, o = sure_before + eq_kept_before;
#pragma unroll
    for (int i = 0; i < kMaxPer; ++i) {
      if (i < per && j_lo + i < n) {
        if (keeps(kr[i], e)) {
          if (o < k_keep) keep_idx[out0 + o] = row0 + j_lo + i;   // o < k_keep always unless k_keep < #protected
          ++o;
        }
      }
    }
  } else {
    const int per = (n + kSelThreads - 1) / kSelThreads;
    const int j_lo = tid * per, j_hi = (j_lo + per < n) ? j_lo + per : n;
    auto key_at = [&](int j) __attribute__((always_inline)) -> uint32_t {
      return prot[row0 + j] ? 0u : cand_key(rule, scores, sample_key, row0, n, j);
    };
    int eq_cnt = 0;
    for (int j = j_lo; j < j_hi; ++j) {
      const uint32_t key = key_at(j);
      eq_cnt += (key != 0u && key == prefix) ? 1 : 0;
    }
    int dummy;
    const int eq_before = block_exclusive_scan(eq_cnt, wave_tot, dummy);
    int keep_cnt = 0;
    {
      int e = eq_before;
      for (int j = j_lo; j < j_hi; ++j) keep_cnt += keeps(key_at(j), e) ? 1 : 0;
    }
    const int keep_before = block_exclusive_scan(keep_cnt, wave_tot, dummy);
    int e = eq_before, o = keep_before;
    for (int j = j_lo; j < j_hi; ++j) {
      if (keeps(key_at(j), e)) {
        if (o < k_keep) keep_idx[out0 + o] = row0 + j;     // o < k_keep always unless k_keep < #protected
        ++o;
      }
    }
  }
}

bool select_fuses_score(int max_seqlen, int n_heads) { return max_seqlen <= kSelLdsKeys && n_heads >= 1 && n_heads <= kSelMaxHeads; }

fastav_status_t launch_select(const float* scores, const uint8_t* prot, const int32_t* cu, const int32_t* cu_out,
                              int batch, int max_seqlen, int32_t* keep_idx, double bytes_hint, hipStream_t s,
                              SelectRule rule) {
  if (batch == 0 || max_seqlen == 0) return FASTAV_OK;
  if ((rule.order == kSelHighScore || rule.order == kSelLowScore) && !scores && !rule.logits) return fail(FASTAV_EINVAL, "select: this order needs scores");
  if (rule.logits && (max_seqlen > kSelLdsKeys || rule.n_heads > kSelMaxHeads || rule.n_heads < 1 || !rule.ml))
    return fail(FASTAV_EUNSUPPORTED, "select: the fused score finish needs samples of at most %d rows and at most %d heads", kSelLdsKeys, kSelMaxHeads);
  ProfScope prof(FASTAV_PROF_SELECT, bytes_hint, s);
  if (max_seqlen <= kSelLdsKeys) {
    const size_t shmem = (size_t)max_seqlen * sizeof(uint32_t);
    if (shmem > 32 * 1024) {   // beyond the default dynamic-LDS limit: opt in (per device, so set on every such launch)
      hipError_t e = hipFuncSetAttribute((const void*)k_select<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         kSelLdsKeys * (int)sizeof(uint32_t));
      if (e != hipSuccess) return fail(FASTAV_EHIP, "select: hipFuncSetAttribute: %s", hipGetErrorString(e));
    }
    hipLaunchKernelGGL(k_select<true>, dim3((unsigned)batch), dim3(kSelThreads), shmem, s, scores, prot, cu, cu_out, keep_idx, rule);
  } else {
    hipLaunchKernelGGL(k_select<false>, dim3((unsigned)batch), dim3(kSelThreads), 0, s, scores, prot, cu, cu_out, keep_idx, rule);
  }
  return check_launch("select");
}

// ---------------------------------------------------------------------------------------- gather
struct GatherArgs {
  const char* src[FASTAV_MAX_GATHER_TENSORS];
  char* dst[FASTAV_MAX_GATHER_TENSORS];
  int64_t row_bytes[FASTAV_MAX_GATHER_TENSORS];
  int64_t src_stride[FASTAV_MAX_GATHER_TENSORS];
  int64_t dst_stride[FASTAV_MAX_GATHER_TENSORS];   // bytes between destination rows (row_bytes when packed)
};

// grid (row groups, tensor).  Rows whose size and addresses are multiples of 16 bytes move as uint4 with
// the workgroup's lanes laid along the row; anything else moves bytewise.  idx == nullptr copies rows in
// place order (a strided copy).
__global__ __launch_bounds__(256) void k_gather(GatherArgs a, const int32_t* __restrict__ idx, int64_t n_rows,
                                                int rows_per_block) {
  const int t = blockIdx.y;
  const int64_t rb = a.row_bytes[t];
  const int64_t ss = a.src_stride[t], ds = a.dst_stride[t];
  const char* src = a.src[t];
  char* dst = a.dst[t];
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const bool vec = ((rb | ss | ds) % 16 == 0) && (((uintptr_t)src | (uintptr_t)dst) % 16 == 0);
  if (vec) {
    const int64_t v_per_row = rb / 16;
    const int64_t total = v_per_row * rows_per_block;
    for (int64_t i = threadIdx.x; i < total; i += 256) {
      const int64_t r = r0 + i / v_per_row, c = i % v_per_row;
      if (r >= n_rows) break;
      const int64_t sr = idx ? (int64_t)idx[r] : r;
      ((uint4*)(dst + r * ds))[c] = ((const uint4*)(src + sr * ss))[c];
    }
  } else {
    const int64_t total = rb * rows_per_block;
    for (int64_t i = threadIdx.x; i < total; i += 256) {
      const int64_t r = r0 + i / rb, c = i % rb;
      if (r >= n_rows) break;
      const int64_t sr = idx ? (int64_t)idx[r] : r;
      dst[r * ds + c] = src[sr * ss + c];
    }
  }
}

static fastav_status_t gather_impl(const GatherArgs& a, int n_tensors, const int32_t* keep_idx, int64_t n_rows,
                                   int prof_kind, hipStream_t s) {
  if (n_rows == 0 || n_tensors == 0) return FASTAV_OK;
  double bytes = keep_idx ? 4.0 * n_rows : 0.0;
  for (int i = 0; i < n_tensors; ++i) bytes += 2.0 * a.row_bytes[i] * n_rows;
  ProfScope prof(prof_kind, bytes, s);
  // aim at >= 4 KB of payload per workgroup, judged by the widest tensor
  int64_t widest = 1;
  for (int i = 0; i < n_tensors; ++i) widest = a.row_bytes[i] > widest ? a.row_bytes[i] : widest;
  int rows_per_block = (int)(4096 / widest);
  if (rows_per_block < 1) rows_per_block = 1;
  if (rows_per_block > 64) rows_per_block = 64;
  dim3 grid((unsigned)ceil_div(n_rows, rows_per_block), (unsigned)n_tensors);
  hipLaunchKernelGGL(k_gather, grid, dim3(256), 0, s, a, keep_idx, n_rows, rows_per_block);
  return check_launch("gather");
}

fastav_status_t launch_gather(const GatherTensor* t, int n_tensors, const int32_t* keep_idx, int64_t n_rows,
                              hipStream_t s) {
  if (n_tensors > FASTAV_MAX_GATHER_TENSORS) return fail(FASTAV_EINVAL, "gather: too many tensors");
  GatherArgs a;
  int m = 0;
  for (int i = 0; i < n_tensors; ++i) {
    if (t[i].row_bytes == 0) continue;
    a.src[m] = (const char*)t[i].src; a.dst[m] = (char*)t[i].dst;
    a.row_bytes[m] = t[i].row_bytes; a.src_stride[m] = t[i].src_stride_bytes ? t[i].src_stride_bytes : t[i].row_bytes;
    a.dst_stride[m] = t[i].row_bytes; ++m;
  }
  for (int i = m; i < FASTAV_MAX_GATHER_TENSORS; ++i) { a.src[i] = nullptr; a.dst[i] = nullptr; a.row_bytes[i] = 0; a.src_stride[i] = 0; a.dst_stride[i] = 0; }
  // without an index this is a plain copy (KV-cache write), timed apart from the prune-step gathers
  return gather_impl(a, m, keep_idx, n_rows, keep_idx ? FASTAV_PROF_GATHER : FASTAV_PROF_OTHER, s);
}

fastav_status_t launch_copy_rows(const void* src, int64_t src_row_bytes_stride, void* dst, int64_t row_bytes,
                                 int64_t rows, const int32_t* idx, hipStream_t s, int64_t dst_row_bytes_stride) {
  GatherArgs a;
  for (int i = 0; i < FASTAV_MAX_GATHER_TENSORS; ++i) { a.src[i] = nullptr; a.dst[i] = nullptr; a.row_bytes[i] = 0; a.src_stride[i] = 0; a.dst_stride[i] = 0; }
  a.src[0] = (const char*)src; a.dst[0] = (char*)dst; a.row_bytes[0] = row_bytes; a.src_stride[0] = src_row_bytes_stride;
  a.dst_stride[0] = dst_row_bytes_stride ? dst_row_bytes_stride : row_bytes;
  // plain row copies (KV-cache writes, outputs) are not part of a prune step: they are timed as "other"
  return gather_impl(a, 1, idx, rows, idx ? FASTAV_PROF_GATHER : FASTAV_PROF_OTHER, s);
}

}  // namespace fastav
