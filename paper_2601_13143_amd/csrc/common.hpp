// Shared declarations of the FastAV HIP library (gfx950 only): types, launch helpers and the internal
// kernel-launch functions the C ABI in api.hip strings together.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/fastav.h"

namespace fastav {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE (v_cvt_pk_bf16_f32)

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// Records the message returned by fastav_last_error() and passes the status through.
fastav_status_t fail(fastav_status_t st, const char* fmt, ...);
fastav_status_t check_launch(const char* what);

// Times the launches issued while it is alive when profiling of `kind` is on (see fastav_profile_enable).
class ProfScope {
 public:
  ProfScope(int kind, double work, hipStream_t s);
  ~ProfScope();
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;
 private:
  void* rec_;
  hipStream_t stream_;
};

// ---- launchers (every pointer is a device pointer unless named host_*) ------------------------------

// Copies a small host array into device memory through kernel arguments (no memcpy, no pinned memory,
// stream-ordered, legal under graph capture).
fastav_status_t upload_small(void* dst_dev, const void* host_src, size_t bytes, hipStream_t s);

fastav_status_t launch_init_tokens(const int32_t* cu, const int32_t* span_offsets, const fastav_span_t* spans,
                                   int batch, int64_t T, int max_seqlen, int n_last, int32_t* pos, uint8_t* prot,
                                   hipStream_t s);
fastav_status_t launch_to_f32(const void* x, float* y, int64_t n, int dtype, hipStream_t s);
// dst_row_bytes_stride == 0: destination rows are packed
fastav_status_t launch_copy_rows(const void* src, int64_t src_row_bytes_stride, void* dst, int64_t row_bytes,
                                 int64_t rows, const int32_t* idx, hipStream_t s, int64_t dst_row_bytes_stride = 0);
// A residual update whose split-K partial sums have not been added yet: R[M][N] += sum over splits of
// partial[s][M][N], in split order.  launch_linear fills it (splits = 0 if the product was not split) when asked to
// leave the sum to the consumer; launch_rmsnorm can take it over (it reads the residual anyway), launch_splitk_reduce
// finishes it on its own.
struct SplitKPending { const float* partial = nullptr; int splits = 0; int64_t M = 0; int N = 0; };
fastav_status_t launch_splitk_reduce(float* r, int64_t ldc, const SplitKPending& p, hipStream_t s);
// pend (optional, splits > 0): x is first completed with the pending partial sums and written back, then normalised
fastav_status_t launch_rmsnorm(float* x, const void* g, void* y, int64_t rows, int d, float eps, int dtype,
                               hipStream_t s, const SplitKPending* pend = nullptr);
// table (optional): (cos, sin) per (position, frequency index) as launch_rope_table writes it; positions in `pos`
// must be below the n_pos it was built for.  Without it every launch evaluates the angles itself.
size_t rope_table_bytes(int n_pos, int head_dim);
fastav_status_t launch_rope_table(void* table, int n_pos, int head_dim, float base, hipStream_t s);
fastav_status_t launch_rope(void* x, int64_t row_stride, const int32_t* pos, int64_t rows, int n_heads, int head_dim,
                            float base, int dtype, hipStream_t s, const void* table = nullptr);
// the same over n_heads heads of x followed by n_heads2 heads of a second tensor (one launch)
fastav_status_t launch_rope2(void* x, int64_t row_stride, int n_heads, void* x2, int64_t row_stride2, int n_heads2,
                             const int32_t* pos, int64_t rows, int head_dim, float base, int dtype, hipStream_t s,
                             const void* table = nullptr);
// scratch (optional): device memory for split-K partial tiles; without it small-M residual GEMMs are not split
// pend (optional, residual epilogue): a split-K product leaves its partial sums pending instead of reducing them
// rows (optional, rows.idx != nullptr): row r of the product reads row rows.idx[r] of `a` instead of row r - a row
// gather folded into the operand copies; rows.n_src = number of rows `a` holds.  Only where linear_takes_rows says so.
struct RowGather { const int32_t* idx = nullptr; int64_t n_src = 0; };
bool linear_takes_rows(int64_t m, int n, int k, int epilogue, int dtype, int64_t n_src);
fastav_status_t launch_linear(const void* a, const void* w, const void* w2, void* c, int64_t m, int n, int k,
                              int epilogue, int dtype, void* scratch, size_t scratch_bytes, hipStream_t s,
                              SplitKPending* pend = nullptr, RowGather rows = RowGather());
fastav_status_t launch_attention(const void* q, int64_t q_stride, const void* k, const void* v, int64_t kv_stride,
                                 void* o, int64_t o_stride, const int32_t* cu, int batch, int64_t T, int max_seqlen,
                                 int Hq, int Hkv, int dh, float* last_logits, float* last_ml, int dtype,
                                 double flops_hint, hipStream_t s);

// RoPE folded into the plain-store epilogue of a projection: rows are rotated by pos[row] with the (cos, sin) table
// launch_rope_table wrote; the first n_segs weight segments (whole heads of head_dim columns) are rotated.
struct RopeFuse { const int32_t* pos; const void* table; int head_dim; int n_segs; };

// Eq. 4.  logits [n_last, Hq, T] fp32, ml [batch, n_last, Hq, 2] fp32.
size_t score_partials_bytes(int Hq, int64_t T, int batch, int n_last);
size_t score_logits_bytes(int Hq, int64_t T, int n_last);   // logits buffer handed to launch_score_logits
fastav_status_t launch_score_logits(const void* q, int64_t q_stride, const void* k, int64_t k_stride,
                                    const int32_t* cu, int batch, int64_t T, int max_seqlen, int Hq, int Hkv, int dh,
                                    int n_last, float* logits, float* partials, int dtype, hipStream_t s);
// exactly one of ml (per-head (max, sum-exp), e.g. the attention side output) and partials is non-null
fastav_status_t launch_score_finalize(const float* logits, const float* ml, const float* partials, const int32_t* cu,
                                      int batch, int64_t T, int max_seqlen, int Hq, int n_last, float* scores,
                                      hipStream_t s);

// How the select kernel ranks the candidates of a sample (larger rank = kept first; equal ranks -> lower index).
// The strategies compared in Tables 2-3 of the paper are these five orders.
enum SelectOrder {
  kSelHighScore = 0,   // by score, highest first (removes the low-attentive tokens: the fine rule)
  kSelLowScore = 1,    // by negated score (removes the top-attentive tokens)
  kSelEarliest = 2,    // by position, earliest first (removes the latest tokens: the global rule)
  kSelLatest = 3,      // by position, latest first
  kSelRandom = 4       // by a counter-based uniform draw per (key, sample, position id)
};
struct SelectRule {
  int order;
  uint32_t key;        // kSelRandom: mix32(seed + G * (layer + 1)), prepared on the host
  const int32_t* pos;  // kSelRandom: position id of every packed row (nullptr -> index inside the sample)
  // score orders, optional: finish Eq. 4 inside the select kernel from the attention side output instead of reading
  // `scores` - logits [n_heads][T] fp32, ml [batch][n_heads][2] = (max, sum of exp); scores_out (optional) [T]
  const float* logits = nullptr;
  const float* ml = nullptr;
  int n_heads = 0;
  int64_t T = 0;
  float* scores_out = nullptr;
};
bool select_fuses_score(int max_seqlen, int n_heads);   // limits of the fused path
uint32_t select_random_key(uint32_t seed, int layer);

// Selection + compaction.  keep_idx/cu_out as in fastav_select_gather; scores are read by the two score orders only.
fastav_status_t launch_select(const float* scores, const uint8_t* prot, const int32_t* cu, const int32_t* cu_out,
                              int batch, int max_seqlen, int32_t* keep_idx, double bytes_hint, hipStream_t s,
                              SelectRule rule);
// src_stride_bytes == 0 means rows are packed (stride = row_bytes); row_bytes == 0 skips the tensor.
struct GatherTensor { const void* src; void* dst; int64_t row_bytes; int64_t src_stride_bytes; };
fastav_status_t launch_gather(const GatherTensor* t, int n_tensors, const int32_t* keep_idx, int64_t n_rows,
                              hipStream_t s);

}  // namespace fastav
