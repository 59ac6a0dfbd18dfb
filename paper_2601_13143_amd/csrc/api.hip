// C ABI of the FastAV pruned-prefill library: argument validation, the host-side token schedule, workspace
// carving and the per-layer launch sequence.  Token counts after every prune depend only on the sequence
// lengths and keep ratios, so the whole schedule is computed on the host up front and the stream is never
// synchronised.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "common.hpp"

namespace fastav {

static thread_local char g_err[512] = "";
int g_options[FASTAV_OPT_COUNT] = {1, 1, 1, 1};

fastav_status_t fail(fastav_status_t st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

fastav_status_t check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FASTAV_EHIP, "%s: %s", what, hipGetErrorString(e));
  return FASTAV_OK;
}

fastav_status_t launch_linear_generic(const void* a, const void* w, const void* w2, void* c, int64_t ldc, int64_t m,
                                      int n, int k, int epilogue, int dtype, hipStream_t s);
bool mfma_linear_supported(int64_t m, int n, int k, int epilogue, int dtype);
fastav_status_t launch_linear_mfma(const void* a, const void* const* w_seg, const int* seg_rows, int n_seg,
                                   const void* w2, void* c, int64_t ldc, void* const* c_seg, const int64_t* ldc_seg,
                                   int64_t m, int n, int k, int epilogue, void* scratch, size_t scratch_bytes, hipStream_t s,
                                   const RopeFuse* rope = nullptr, SplitKPending* pend = nullptr, RowGather rows = RowGather());
bool mfma_linear_takes_rows(int k, int64_t n_src);
bool mfma_linear_fuses_rope(int64_t m, const int* seg_rows, int n_seg, int rope_segs, int k, int dh, int dtype);
size_t mfma_linear_scratch_bytes();
fastav_status_t launch_attention_generic(const void* q, int64_t q_stride, const void* k, const void* v,
                                         int64_t kv_stride, void* o, int64_t o_stride, const int32_t* cu, int batch,
                                         int64_t T, int max_seqlen, int Hq, int Hkv, int dh, float* last_logits,
                                         float* last_ml, int dtype, hipStream_t s);
bool mfma_attention_supported(int dh, int dtype, int64_t q_stride, int64_t kv_stride, int64_t o_stride, int max_seqlen);
fastav_status_t launch_attention_mfma(const void* q, int64_t q_stride, const void* k, const void* v,
                                      int64_t kv_stride, void* o, int64_t o_stride, const int32_t* cu, int batch,
                                      int64_t T, int max_seqlen, int Hq, int Hkv, int dh, float* last_logits,
                                      float* last_ml, hipStream_t s);

bool skinny_linear_supported(int64_t m, int n, int k, int dtype, int64_t ldy);
bool skinny_norm_supported(int B, int k);
fastav_status_t launch_skinny_linear(const void* x, const void* const* w_seg, const int* seg_rows, int n_seg,
                                     const void* w2, void* y, int64_t ldy, int B, int n, int k, int epilogue,
                                     hipStream_t s, const float* norm_x = nullptr, const void* norm_g = nullptr,
                                     float norm_eps = 0.f, const int32_t* rope_pos = nullptr, int rope_rows = 0,
                                     int rope_dh = 0, float rope_base = 0.f);
bool gemv_rows_fuses_rope(int B, int n, int k, bool norm, int rope_rows, int dh);
size_t decode_attn_workspace_bytes(int batch, int Hq, int dh, int max_splits);
fastav_status_t launch_decode_attention(const void* q, const void* k_self, const void* v_self, int64_t q_stride,
                                        const void* k_prefix, const void* v_prefix, const int32_t* cu_prefix,
                                        int max_prefix, const void* k_gen, const void* v_gen, int gen_len,
                                        int gen_cap, int batch, int Hq, int Hkv, int dh, float* part,
                                        size_t part_bytes, void* out, int64_t out_stride, double bytes_hint,
                                        hipStream_t s);

size_t attention_map_stats_bytes(int n, int Hq);
fastav_status_t launch_attention_map(const void* q, int64_t q_stride, const void* k, int64_t k_stride, int n, int Hq,
                                     int Hkv, int dh, float* stats, void* a_out, hipStream_t s);
fastav_status_t launch_iota(int32_t* p, int n, hipStream_t s);
fastav_status_t launch_rollout_init(float* rt, void* rt16, int n, hipStream_t s);
fastav_status_t launch_rollout_cutoff(const float* rt, int n, const uint8_t* prot, float threshold, float* influence,
                                      int32_t* cutoff, hipStream_t s);
fastav_status_t launch_rollout_step(float* rt, void* rt16, const void* a16, float* c, int n, float alpha,
                                    void* linear_ws, size_t linear_ws_bytes, hipStream_t s);

// One linear layer whose weight rows may come from up to three matrices stacked along N (Q|K|V).  With c_seg the
// output columns of segment i go to their own matrix c_seg[i] (row pitch ldc_seg[i] elements) instead of columns
// of c (plain-store epilogue only).
static fastav_status_t linear_segments(const void* a, const void* const* w_seg, const int* seg_rows, int n_seg,
                                       const void* w2, void* c, int64_t ldc, int64_t m, int k, int epilogue, int dtype,
                                       void* scratch, size_t scratch_bytes, hipStream_t s,
                                       void* const* c_seg = nullptr, const int64_t* ldc_seg = nullptr,
                                       const RopeFuse* rope = nullptr, SplitKPending* pend = nullptr, RowGather rows = RowGather()) {
  if (pend != nullptr) *pend = SplitKPending();
  int n = 0;
  for (int i = 0; i < n_seg; ++i) n += seg_rows[i];
  if (m == 0 || n == 0) return FASTAV_OK;
  // a handful of rows (a decode step): stream the weights through the skinny kernel, which times itself
  if (c_seg != nullptr && epilogue != FASTAV_EPI_STORE) return fail(FASTAV_EINVAL, "per-segment outputs need the plain-store epilogue");
  if (rows.idx != nullptr && !linear_takes_rows(m, n, k, epilogue, dtype, rows.n_src)) return fail(FASTAV_EINVAL, "linear: this product cannot take a row list");
  if (rows.idx == nullptr && rope == nullptr && c_seg == nullptr && m <= FASTAV_MAX_DECODE_BATCH && skinny_linear_supported(m, n, k, dtype, ldc)) {
    bool sk = (((uintptr_t)a | (uintptr_t)c) % 16) == 0;
    for (int i = 0; i < n_seg && sk; ++i) sk = seg_rows[i] % 16 == 0;
    if (sk) return launch_skinny_linear(a, w_seg, seg_rows, n_seg, w2, c, ldc, (int)m, n, k, epilogue, s);
  }
  const int kind = epilogue == FASTAV_EPI_STORE ? FASTAV_PROF_LINEAR_STORE
                   : epilogue == FASTAV_EPI_RESADD ? FASTAV_PROF_LINEAR_RESADD : FASTAV_PROF_LINEAR_SWIGLU;
  ProfScope prof(kind, 2.0 * (double)m * n * k * (epilogue == FASTAV_EPI_SWIGLU ? 2.0 : 1.0), s);
  bool ok = mfma_linear_supported(m, n, k, epilogue, dtype);
  for (int i = 0; i < n_seg && ok; ++i) ok = mfma_linear_supported(m, seg_rows[i], k, epilogue, dtype);
  if (ok) return launch_linear_mfma(a, w_seg, seg_rows, n_seg, w2, c, ldc, c_seg, ldc_seg, m, n, k, epilogue, scratch, scratch_bytes, s, rope, pend, rows);
  if (rows.idx != nullptr) return fail(FASTAV_EINVAL, "linear: the row list needs the matrix-core kernel");
  if (rope != nullptr) return fail(FASTAV_EINVAL, "linear: the RoPE epilogue needs the matrix-core kernel");
  const size_t es = dtype == FASTAV_BF16 ? 2 : 4;
  int col = 0;
  for (int i = 0; i < n_seg; ++i) {
    void* ci = c_seg ? c_seg[i] : epilogue == FASTAV_EPI_RESADD ? (void*)((float*)c + col) : (void*)((char*)c + (size_t)col * es);
    fastav_status_t st = launch_linear_generic(a, w_seg[i], w2, ci, c_seg ? ldc_seg[i] : ldc, m, seg_rows[i], k, epilogue, dtype, s);
    if (st != FASTAV_OK) return st;
    col += seg_rows[i];
  }
  return FASTAV_OK;
}

// The matrix-core kernel is the one that can read its A rows through a list; a handful of rows go to the skinny kernel.
bool linear_takes_rows(int64_t m, int n, int k, int epilogue, int dtype, int64_t n_src) {
  return m > FASTAV_MAX_DECODE_BATCH && mfma_linear_supported(m, n, k, epilogue, dtype) && mfma_linear_takes_rows(k, n_src);
}

fastav_status_t launch_linear(const void* a, const void* w, const void* w2, void* c, int64_t m, int n, int k,
                              int epilogue, int dtype, void* scratch, size_t scratch_bytes, hipStream_t s,
                              SplitKPending* pend, RowGather rows) {
  const void* seg[1] = {w};
  int seg_rows[1] = {n};
  return linear_segments(a, seg, seg_rows, 1, w2, c, n, m, k, epilogue, dtype, scratch, scratch_bytes, s, nullptr, nullptr, nullptr, pend, rows);
}

fastav_status_t launch_attention(const void* q, int64_t q_stride, const void* k, const void* v, int64_t kv_stride,
                                 void* o, int64_t o_stride, const int32_t* cu, int batch, int64_t T, int max_seqlen,
                                 int Hq, int Hkv, int dh, float* last_logits, float* last_ml, int dtype,
                                 double flops_hint, hipStream_t s) {
  ProfScope prof(FASTAV_PROF_ATTENTION, flops_hint, s);
  if (mfma_attention_supported(dh, dtype, q_stride, kv_stride, o_stride, max_seqlen))
    return launch_attention_mfma(q, q_stride, k, v, kv_stride, o, o_stride, cu, batch, T, max_seqlen, Hq, Hkv, dh,
                                 last_logits, last_ml, s);
  return launch_attention_generic(q, q_stride, k, v, kv_stride, o, o_stride, cu, batch, T, max_seqlen, Hq, Hkv, dh,
                                  last_logits, last_ml, dtype, s);
}

// ------------------------------------------------------------------------------------------ validation
static int64_t keep_count(int64_t n, double r, int64_t n_prot) {
  int64_t k = (int64_t)std::ceil(r * (double)n - 1e-9);
  if (k < n_prot) k = n_prot;
  if (k > n) k = n;
  return k;
}

static fastav_status_t check_model(const fastav_model_t* m) {
  if (!m) return fail(FASTAV_EINVAL, "model is NULL");
  if (m->n_layers < 1 || m->hidden < 1 || m->n_q_heads < 1 || m->n_kv_heads < 1 || m->mlp_dim < 1 || m->head_dim < 1)
    return fail(FASTAV_EINVAL, "model dimensions must be positive");
  if (m->n_q_heads % m->n_kv_heads) return fail(FASTAV_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
  if (m->dtype != FASTAV_BF16 && m->dtype != FASTAV_F32) return fail(FASTAV_EINVAL, "dtype must be FASTAV_BF16 or FASTAV_F32");
  if (!(m->rope_base > 1.0f) || !(m->rms_eps >= 0.0f)) return fail(FASTAV_EINVAL, "rope_base must exceed 1 and rms_eps be >= 0");
  if (m->head_dim != 64 && m->head_dim != 128) return fail(FASTAV_EUNSUPPORTED, "head_dim must be 64 or 128");
  if ((int64_t)m->n_q_heads * (m->head_dim + 128) * 4 > 64 * 1024)
    return fail(FASTAV_EUNSUPPORTED, "n_q_heads*(head_dim+128)*4 bytes must fit 64 KB of LDS");
  return FASTAV_OK;
}

static fastav_status_t check_batch(const fastav_batch_t* in, bool need_x, int64_t* T_out, int* max_len_out) {
  if (!in) return fail(FASTAV_EINVAL, "batch descriptor is NULL");
  if (in->batch < 1) return fail(FASTAV_EINVAL, "batch must be >= 1");
  if (!in->cu_seqlens || !in->spans || !in->span_offsets) return fail(FASTAV_EINVAL, "cu_seqlens/spans/span_offsets is NULL");
  if (need_x && !in->x) return fail(FASTAV_EINVAL, "x is NULL");
  if (in->cu_seqlens[0] != 0 || in->span_offsets[0] != 0) return fail(FASTAV_EINVAL, "cu_seqlens[0] and span_offsets[0] must be 0");
  int max_len = 0;
  for (int b = 0; b < in->batch; ++b) {
    const int64_t n = (int64_t)in->cu_seqlens[b + 1] - in->cu_seqlens[b];
    if (n < 1) return fail(FASTAV_EINVAL, "cu_seqlens must be strictly increasing (sample %d)", b);
    if (in->span_offsets[b + 1] <= in->span_offsets[b]) return fail(FASTAV_EINVAL, "sample %d has no spans", b);
    int64_t at = 0;
    for (int si = in->span_offsets[b]; si < in->span_offsets[b + 1]; ++si) {
      const fastav_span_t& sp = in->spans[si];
      if (sp.len < 1 || sp.start != at) return fail(FASTAV_EINVAL, "spans of sample %d must be sorted, disjoint and cover [0,n)", b);
      if (sp.modality < FASTAV_TEXT || sp.modality > FASTAV_AUDIO) return fail(FASTAV_EINVAL, "bad modality in sample %d", b);
      at += sp.len;
    }
    if (at != n) return fail(FASTAV_EINVAL, "spans of sample %d cover %lld of %lld tokens", b, (long long)at, (long long)n);
    if (n > max_len) max_len = (int)n;
  }
  *T_out = in->cu_seqlens[in->batch];
  *max_len_out = max_len;
  return FASTAV_OK;
}

static fastav_status_t check_prunes(const fastav_prune_t* prunes, int n_prunes, int n_layers, int n_last) {
  if (n_prunes < 0 || n_prunes > FASTAV_MAX_PRUNES) return fail(FASTAV_EINVAL, "n_prunes must be in [0, %d]", FASTAV_MAX_PRUNES);
  if (n_prunes > 0 && !prunes) return fail(FASTAV_EINVAL, "prunes is NULL");
  if (n_last < 1 || n_last > FASTAV_MAX_N_LAST) return fail(FASTAV_EINVAL, "n_last must be in [1, %d]", FASTAV_MAX_N_LAST);
  for (int i = 0; i < n_prunes; ++i) {
    const fastav_prune_t& p = prunes[i];
    if (p.layer < 0 || p.layer >= n_layers) return fail(FASTAV_EINVAL, "prune %d: layer %d out of range", i, p.layer);
    if (p.kind != FASTAV_GLOBAL && p.kind != FASTAV_FINE) return fail(FASTAV_EINVAL, "prune %d: bad kind", i);
    if (p.selector < FASTAV_SEL_DEFAULT || p.selector > FASTAV_SEL_RANDOM) return fail(FASTAV_EINVAL, "prune %d: bad selector", i);
    if (p.kind == FASTAV_GLOBAL && (p.selector == FASTAV_SEL_LOW_ATTENTIVE || p.selector == FASTAV_SEL_TOP_ATTENTIVE))
      return fail(FASTAV_EINVAL, "prune %d: attentive selectors need the layer's own attention (FINE steps only)", i);
    if (p.kind == FASTAV_FINE && (p.selector == FASTAV_SEL_LOW_INFORMATIVE || p.selector == FASTAV_SEL_TOP_INFORMATIVE))
      return fail(FASTAV_EINVAL, "prune %d: positional selectors belong to GLOBAL steps", i);
    if (!(p.keep_ratio > 0.0 && p.keep_ratio <= 1.0)) return fail(FASTAV_EINVAL, "prune %d: keep_ratio must be in (0,1]", i);
    if (i > 0) {
      const fastav_prune_t& q = prunes[i - 1];
      if (q.layer > p.layer || (q.layer == p.layer && q.kind >= p.kind))
        return fail(FASTAV_EINVAL, "prunes must be sorted by (layer, kind) without duplicates");
    }
  }
  return FASTAV_OK;
}

// Number of tokens of sample b a prune may never remove: TEXT spans plus the last n_last positions.
static int64_t protected_count(const fastav_batch_t* in, int b, int n_last) {
  const int64_t n = (int64_t)in->cu_seqlens[b + 1] - in->cu_seqlens[b];
  const int64_t tail0 = n - n_last > 0 ? n - n_last : 0;
  int64_t cnt = 0;
  for (int si = in->span_offsets[b]; si < in->span_offsets[b + 1]; ++si) {
    const fastav_span_t& sp = in->spans[si];
    const int64_t lo = sp.start, hi = (int64_t)sp.start + sp.len;
    if (sp.modality == FASTAV_TEXT) cnt += sp.len;
    else if (hi > tail0) cnt += hi - (lo > tail0 ? lo : tail0);
  }
  return cnt;
}

// lens[stage][b]: stage 0 = input, stage i+1 = after prune i.
static void build_schedule(const fastav_batch_t* in, const fastav_prune_t* prunes, int n_prunes, int n_last,
                           std::vector<std::vector<int32_t>>& lens) {
  lens.assign(n_prunes + 1, std::vector<int32_t>(in->batch));
  for (int b = 0; b < in->batch; ++b) {
    const int64_t n_prot = protected_count(in, b, n_last);
    int64_t cur = (int64_t)in->cu_seqlens[b + 1] - in->cu_seqlens[b];
    lens[0][b] = (int32_t)cur;
    for (int i = 0; i < n_prunes; ++i) {
      cur = keep_count(cur, (double)prunes[i].keep_ratio, n_prot);
      lens[i + 1][b] = (int32_t)cur;
    }
  }
}

// ------------------------------------------------------------------------------------------ workspace
struct Workspace {
  size_t resid[2], hn, qkv, attn[2], hmlp, logits, ml, partials, scores, pos[2], prot[2], keep_idx, cu, span_off,
      spans, gemm_scratch, gemm_scratch_bytes, rope_table, total;
};

static Workspace carve(const fastav_model_t& m, int64_t T, int B) {
  Workspace w;
  size_t at = 0;
  auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes, 256); return o; };
  const size_t es = m.dtype == FASTAV_BF16 ? 2 : 4;
  const size_t qd = (size_t)m.n_q_heads * m.head_dim, kd = (size_t)m.n_kv_heads * m.head_dim;
  w.resid[0] = take((size_t)T * m.hidden * 4);
  w.resid[1] = take((size_t)T * m.hidden * 4);
  w.hn = take((size_t)T * m.hidden * es);
  w.qkv = take((size_t)T * (qd + 2 * kd) * es);
  w.attn[0] = take((size_t)T * qd * es);
  w.attn[1] = take((size_t)T * qd * es);
  w.hmlp = take((size_t)T * m.mlp_dim * es);
  w.logits = take(score_logits_bytes(m.n_q_heads, T, FASTAV_MAX_N_LAST));
  w.ml = take((size_t)B * FASTAV_MAX_N_LAST * m.n_q_heads * 2 * 4);
  w.partials = take(score_partials_bytes(m.n_q_heads, T, B, FASTAV_MAX_N_LAST));
  w.scores = take((size_t)T * 4);
  w.pos[0] = take((size_t)T * 4);
  w.pos[1] = take((size_t)T * 4);
  w.prot[0] = take((size_t)T);
  w.prot[1] = take((size_t)T);
  w.keep_idx = take((size_t)T * 4);
  w.cu = take((size_t)(FASTAV_MAX_PRUNES + 1) * (B + 1) * 4);
  w.span_off = take((size_t)(B + 1) * 4);
  w.spans = take((size_t)T * sizeof(fastav_span_t));       // a span holds >= 1 token
  w.gemm_scratch_bytes = m.dtype == FASTAV_BF16 ? mfma_linear_scratch_bytes() : 0;   // split-K partial tiles
  w.gemm_scratch = take(w.gemm_scratch_bytes);
  w.rope_table = take(rope_table_bytes((int)(T < 0x7FFFFFFF ? T : 0x7FFFFFFF), m.head_dim));   // a sample is at most T tokens long
  w.total = at;
  return w;
}

}  // namespace fastav

using namespace fastav;

struct fastav_ctx {
  fastav_model_t m;
  std::vector<fastav_layer_weights_t> w;
  std::vector<char> has_w;
};

extern "C" {

const char* fastav_last_error(void) { return g_err; }

fastav_status_t fastav_set_option(int32_t option, int32_t value) {
  if (option < 0 || option >= FASTAV_OPT_COUNT) return fail(FASTAV_EINVAL, "unknown option %d", option);
  g_options[option] = value;
  return FASTAV_OK;
}

int64_t fastav_keep_count(int64_t n, double keep_ratio, int64_t n_protected) {
  if (n < 0 || !(keep_ratio > 0.0 && keep_ratio <= 1.0) || n_protected < 0 || n_protected > n) return -1;
  return keep_count(n, keep_ratio, n_protected);
}

fastav_status_t fastav_schedule(const fastav_batch_t* in, const fastav_prune_t* prunes, int32_t n_prunes,
                                int32_t n_last, int32_t n_layers, int64_t* tokens_in_out, int64_t* tokens_out_out,
                                int32_t* final_lens_out) {
  int64_t T; int max_len;
  fastav_status_t st = check_batch(in, false, &T, &max_len);
  if (st != FASTAV_OK) return st;
  if (n_layers < 1) return fail(FASTAV_EINVAL, "n_layers must be >= 1");
  st = check_prunes(prunes, n_prunes, n_layers, n_last);
  if (st != FASTAV_OK) return st;
  std::vector<std::vector<int32_t>> lens;
  build_schedule(in, prunes, n_prunes, n_last, lens);
  std::vector<int64_t> tot(n_prunes + 1, 0);
  for (int i = 0; i <= n_prunes; ++i) for (int b = 0; b < in->batch; ++b) tot[i] += lens[i][b];
  int stage = 0, pi = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (pi < n_prunes && prunes[pi].layer == l && prunes[pi].kind == FASTAV_GLOBAL) { ++stage; ++pi; }
    if (tokens_in_out) tokens_in_out[l] = tot[stage];
    if (pi < n_prunes && prunes[pi].layer == l && prunes[pi].kind == FASTAV_FINE) { ++stage; ++pi; }
    if (tokens_out_out) tokens_out_out[l] = tot[stage];
  }
  if (final_lens_out) for (int b = 0; b < in->batch; ++b) final_lens_out[b] = lens[n_prunes][b];
  return FASTAV_OK;
}

fastav_status_t fastav_schedule_lens(const fastav_batch_t* in, const fastav_prune_t* prunes, int32_t n_prunes,
                                     int32_t n_last, int32_t n_layers, int32_t* lens_out) {
  int64_t T; int max_len;
  fastav_status_t st = check_batch(in, false, &T, &max_len);
  if (st != FASTAV_OK) return st;
  if (n_layers < 1 || !lens_out) return fail(FASTAV_EINVAL, "n_layers must be >= 1 and lens_out non-NULL");
  st = check_prunes(prunes, n_prunes, n_layers, n_last);
  if (st != FASTAV_OK) return st;
  std::vector<std::vector<int32_t>> lens;
  build_schedule(in, prunes, n_prunes, n_last, lens);
  int stage = 0, pi = 0;
  for (int l = 0; l < n_layers; ++l) {
    while (pi < n_prunes && prunes[pi].layer == l) { ++stage; ++pi; }     // global, then fine, of this layer
    for (int b = 0; b < in->batch; ++b) lens_out[(size_t)l * in->batch + b] = lens[stage][b];
  }
  return FASTAV_OK;
}

fastav_status_t fastav_create(const fastav_model_t* model, fastav_handle_t* out) {
  if (!out) return fail(FASTAV_EINVAL, "out is NULL");
  *out = nullptr;
  fastav_status_t st = check_model(model);
  if (st != FASTAV_OK) return st;
  fastav_ctx* c = new (std::nothrow) fastav_ctx();
  if (!c) return fail(FASTAV_EINVAL, "out of host memory");
  c->m = *model;
  c->w.resize(model->n_layers);
  c->has_w.assign(model->n_layers, 0);
  *out = c;
  return FASTAV_OK;
}

void fastav_destroy(fastav_handle_t h) { delete h; }

fastav_status_t fastav_set_weights(fastav_handle_t h, int32_t layer, const fastav_layer_weights_t* w) {
  if (!h || !w) return fail(FASTAV_EINVAL, "handle or weights is NULL");
  if (layer < 0 || layer >= h->m.n_layers) return fail(FASTAV_EINVAL, "layer %d out of range", layer);
  if (!w->g_attn || !w->wq || !w->wk || !w->wv || !w->wo || !w->g_mlp || !w->w_gate || !w->w_up || !w->w_down)
    return fail(FASTAV_EINVAL, "a weight pointer of layer %d is NULL", layer);
  const uintptr_t all = (uintptr_t)w->g_attn | (uintptr_t)w->wq | (uintptr_t)w->wk | (uintptr_t)w->wv | (uintptr_t)w->wo |
                        (uintptr_t)w->g_mlp | (uintptr_t)w->w_gate | (uintptr_t)w->w_up | (uintptr_t)w->w_down;
  if (all % 16) return fail(FASTAV_EINVAL, "weight pointers must be 16-byte aligned");
  h->w[layer] = *w;
  h->has_w[layer] = 1;
  return FASTAV_OK;
}

fastav_status_t fastav_workspace_bytes(fastav_handle_t h, int64_t max_total_tokens, int32_t max_batch, size_t* out) {
  if (!h || !out) return fail(FASTAV_EINVAL, "handle or out is NULL");
  if (max_total_tokens < 1 || max_batch < 1 || max_total_tokens > 0x7FFFFFFF)
    return fail(FASTAV_EINVAL, "max_total_tokens must be in [1, 2^31) and max_batch >= 1");
  *out = carve(h->m, max_total_tokens, max_batch).total;
  return FASTAV_OK;
}

#define FASTAV_TRY(expr) do { fastav_status_t st__ = (expr); if (st__ != FASTAV_OK) return st__; } while (0)

fastav_status_t fastav_prefill(fastav_handle_t h, const fastav_batch_t* in, const fastav_prune_t* prunes,
                               int32_t n_prunes, int32_t n_last, void* workspace, size_t workspace_bytes,
                               const fastav_prefill_out_t* out, void* stream) {
  if (!h) return fail(FASTAV_EINVAL, "handle is NULL");
  const fastav_model_t& m = h->m;
  int64_t T0; int max_len0;
  FASTAV_TRY(check_batch(in, true, &T0, &max_len0));
  FASTAV_TRY(check_prunes(prunes, n_prunes, m.n_layers, n_last));
  if (!out || !out->x_out || !out->cu_seqlens_out || !out->kept_pos_out)
    return fail(FASTAV_EINVAL, "out, x_out, cu_seqlens_out and kept_pos_out must be non-NULL");
  if (!workspace || ((uintptr_t)workspace % 256)) return fail(FASTAV_EINVAL, "workspace must be non-NULL and 256-byte aligned");
  if (((uintptr_t)in->x % 16) || ((uintptr_t)out->x_out % 16)) return fail(FASTAV_EINVAL, "x and x_out must be 16-byte aligned");
  for (int l = 0; l < m.n_layers; ++l)
    if (!h->has_w[l]) return fail(FASTAV_EINVAL, "weights of layer %d were never set", l);
  // a layer without a fine prune computes on K and V in the caller's cache: the kernels read them 16 bytes at a time
  if (out->kv_out)
    for (int i = 0; i < 2 * m.n_layers; ++i)
      if ((uintptr_t)out->kv_out[i] % 16) return fail(FASTAV_EINVAL, "kv_out[%d] must be 16-byte aligned", i);
  const int B = in->batch;
  const Workspace ws = carve(m, T0, B);
  if (workspace_bytes < ws.total)
    return fail(FASTAV_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, ws.total);
  if ((size_t)in->span_offsets[B] > (size_t)T0) return fail(FASTAV_EINVAL, "more spans than tokens");

  // ---- host schedule: per-stage lengths, prefix sums, totals, longest sample
  std::vector<std::vector<int32_t>> lens;
  build_schedule(in, prunes, n_prunes, n_last, lens);
  const int n_stages = n_prunes + 1;
  std::vector<int32_t> cu_host((size_t)n_stages * (B + 1));
  std::vector<int64_t> T_stage(n_stages);
  std::vector<int> maxlen_stage(n_stages);
  for (int i = 0; i < n_stages; ++i) {
    int32_t* cu = &cu_host[(size_t)i * (B + 1)];
    cu[0] = 0;
    int mx = 0;
    for (int b = 0; b < B; ++b) { cu[b + 1] = cu[b] + lens[i][b]; if (lens[i][b] > mx) mx = lens[i][b]; }
    T_stage[i] = cu[B];
    maxlen_stage[i] = mx;
  }

  // causal attention work per stage: 2 Hq dh n (n + 1) per sample
  std::vector<double> attn_flops(n_stages, 0.0);
  for (int i = 0; i < n_stages; ++i)
    for (int b = 0; b < B; ++b)
      attn_flops[i] += 2.0 * m.n_q_heads * m.head_dim * (double)lens[i][b] * ((double)lens[i][b] + 1.0);

  hipStream_t s = (hipStream_t)stream;
  char* base = (char*)workspace;
  float* resid[2] = {(float*)(base + ws.resid[0]), (float*)(base + ws.resid[1])};
  void* hn = base + ws.hn;
  char* qkv = base + ws.qkv;
  void* attn[2] = {base + ws.attn[0], base + ws.attn[1]};
  void* hmlp = base + ws.hmlp;
  float* logits = (float*)(base + ws.logits);
  float* ml = (float*)(base + ws.ml);
  float* partials = (float*)(base + ws.partials);
  float* scores_ws = (float*)(base + ws.scores);
  int32_t* pos[2] = {(int32_t*)(base + ws.pos[0]), (int32_t*)(base + ws.pos[1])};
  uint8_t* prot[2] = {(uint8_t*)(base + ws.prot[0]), (uint8_t*)(base + ws.prot[1])};
  int32_t* keep_idx_ws = (int32_t*)(base + ws.keep_idx);
  int32_t* cu_dev = (int32_t*)(base + ws.cu);
  int32_t* span_off_dev = (int32_t*)(base + ws.span_off);
  fastav_span_t* spans_dev = (fastav_span_t*)(base + ws.spans);
  void* gscr = ws.gemm_scratch_bytes ? (void*)(base + ws.gemm_scratch) : nullptr;

  FASTAV_TRY(upload_small(cu_dev, cu_host.data(), cu_host.size() * 4, s));
  FASTAV_TRY(upload_small(span_off_dev, in->span_offsets, (size_t)(B + 1) * 4, s));
  FASTAV_TRY(upload_small(spans_dev, in->spans, (size_t)in->span_offsets[B] * sizeof(fastav_span_t), s));
  FASTAV_TRY(launch_init_tokens(cu_dev, span_off_dev, spans_dev, B, T0, max_len0, n_last, pos[0], prot[0], s));
  FASTAV_TRY(launch_to_f32(in->x, resid[0], T0 * m.hidden, m.dtype, s));
  // rotary (cos, sin) of every original position, once: tokens keep their positions through every prune
  void* rope_tab = m.dtype == FASTAV_BF16 ? (void*)(base + ws.rope_table) : nullptr;
  if (rope_tab) FASTAV_TRY(launch_rope_table(rope_tab, max_len0, m.head_dim, m.rope_base, s));

  const size_t es = m.dtype == FASTAV_BF16 ? 2 : 4;
  const int qd = m.n_q_heads * m.head_dim, kd = m.n_kv_heads * m.head_dim;
  const int64_t qkv_stride = qd + 2 * kd;                     // elements per row of the fused Q|K|V buffer
  int cur = 0, stage = 0, pi = 0;
  SplitKPending pend_down;
  for (int l = 0; l < m.n_layers; ++l) {
    const fastav_layer_weights_t& W = h->w[l];
    // ---- GLOBAL prune on the layer input: positional selection, then compaction of the residual stream
    if (pi < n_prunes && prunes[pi].layer == l && prunes[pi].kind == FASTAV_GLOBAL) {
      const int32_t* cu_in = cu_dev + (size_t)stage * (B + 1);
      const int32_t* cu_nx = cu_dev + (size_t)(stage + 1) * (B + 1);
      int32_t* kidx = (out->prune_keep_idx_out && out->prune_keep_idx_out[pi]) ? out->prune_keep_idx_out[pi] : keep_idx_ws;
      const fastav_prune_t& pr = prunes[pi];
      const SelectRule rule = pr.selector == FASTAV_SEL_RANDOM ? SelectRule{kSelRandom, select_random_key(pr.seed, l), pos[cur]}
                            : pr.selector == FASTAV_SEL_TOP_INFORMATIVE ? SelectRule{kSelLatest, 0, nullptr}
                                                                        : SelectRule{kSelEarliest, 0, nullptr};
      FASTAV_TRY(launch_select(nullptr, prot[cur], cu_in, cu_nx, B, maxlen_stage[stage], kidx,
                               (rule.order == kSelRandom ? 5.0 : 1.0) * T_stage[stage] + 4.0 * T_stage[stage + 1], s, rule));
      GatherTensor g[3] = {{resid[cur], resid[cur ^ 1], (int64_t)m.hidden * 4, 0},
                           {pos[cur], pos[cur ^ 1], 4, 0},
                           {prot[cur], prot[cur ^ 1], 1, 0}};
      FASTAV_TRY(launch_gather(g, 3, kidx, T_stage[stage + 1], s));
      cur ^= 1; ++stage; ++pi;
    }
    const int64_t Tl = T_stage[stage];
    const int32_t* cu_l = cu_dev + (size_t)stage * (B + 1);
    const bool fine = pi < n_prunes && prunes[pi].layer == l && prunes[pi].kind == FASTAV_FINE;
    const bool fine_scored = fine && prunes[pi].selector != FASTAV_SEL_RANDOM;   // Eq. 4 is needed
    const bool side = fine_scored && n_last == 1;

    // the previous layer's down projection may have left its split-K partial sums to this normalisation
    FASTAV_TRY(launch_rmsnorm(resid[cur], W.g_attn, hn, Tl, m.hidden, m.rms_eps, m.dtype, s, &pend_down));
    pend_down = SplitKPending();
    void* const k_out = out->kv_out ? out->kv_out[2 * l] : nullptr;
    void* const v_out = out->kv_out ? out->kv_out[2 * l + 1] : nullptr;
    // A layer that keeps all its tokens writes K and V straight into the caller's cache (the projection stores
    // them there, RoPE and attention work on them there); a fine-prune layer keeps them in the workspace, from
    // which only the surviving rows go to the cache.
    const bool kv_direct = !fine && k_out != nullptr && v_out != nullptr && Tl > FASTAV_MAX_DECODE_BATCH;
    const char* kptr = kv_direct ? (const char*)k_out : qkv + (size_t)qd * es;
    const char* vptr = kv_direct ? (const char*)v_out : qkv + (size_t)(qd + kd) * es;
    const int64_t kv_stride = kv_direct ? (int64_t)kd : qkv_stride;
    bool rope_fused = false;
    {
      const void* seg[3] = {W.wq, W.wk, W.wv};
      int rows[3] = {qd, kd, kd};
      void* cs[3] = {qkv, k_out, v_out};
      const int64_t lds_[3] = {qkv_stride, (int64_t)kd, (int64_t)kd};
      // RoPE rides in the projection's epilogue (Q and K segments, one rounding) where the matrix-core kernel runs
      rope_fused = rope_tab != nullptr && g_options[FASTAV_OPT_FUSED_ROPE] && Tl > FASTAV_MAX_DECODE_BATCH &&
                   mfma_linear_fuses_rope(Tl, rows, 3, 2, m.hidden, m.head_dim, m.dtype);
      const RopeFuse rf = {pos[cur], rope_tab, m.head_dim, 2};
      FASTAV_TRY(linear_segments(hn, seg, rows, 3, nullptr, qkv, qkv_stride, Tl, m.hidden, FASTAV_EPI_STORE, m.dtype, nullptr, 0, s,
                                 kv_direct ? cs : nullptr, kv_direct ? lds_ : nullptr, rope_fused ? &rf : nullptr));
    }
    if (rope_fused) {
      // nothing left to do
    } else if (kv_direct) {
      FASTAV_TRY(launch_rope2(qkv, qkv_stride, m.n_q_heads, k_out, kd, m.n_kv_heads, pos[cur], Tl, m.head_dim, m.rope_base, m.dtype, s, rope_tab));
    } else {
      FASTAV_TRY(launch_rope(qkv, qkv_stride, pos[cur], Tl, m.n_q_heads + m.n_kv_heads, m.head_dim, m.rope_base, m.dtype, s, rope_tab));
    }
    FASTAV_TRY(launch_attention(qkv, qkv_stride, kptr, vptr, kv_stride, attn[0], qd, cu_l, B, Tl, maxlen_stage[stage],
                                m.n_q_heads, m.n_kv_heads, m.head_dim, side ? logits : nullptr, side ? ml : nullptr,
                                m.dtype, attn_flops[stage], s));
    void* attn_cur = attn[0];
    RowGather o_rows;
    if (fine) {
      // ---- FINE prune: Eq. 4 scores of the last query row(s), top-k, compaction of everything later work reads
      float* sc = (out->prune_scores_out && out->prune_scores_out[pi]) ? out->prune_scores_out[pi] : scores_ws;
      const fastav_prune_t& pr = prunes[pi];
      SelectRule rule = pr.selector == FASTAV_SEL_RANDOM ? SelectRule{kSelRandom, select_random_key(pr.seed, l), pos[cur]}
                      : pr.selector == FASTAV_SEL_TOP_ATTENTIVE ? SelectRule{kSelLowScore, 0, nullptr}
                                                                : SelectRule{kSelHighScore, 0, nullptr};
      if (!fine_scored) {
        // random strategy: no scores
      } else if (side && g_options[FASTAV_OPT_FUSED_SCORE_SELECT] && select_fuses_score(maxlen_stage[stage], m.n_q_heads)) {
        // Eq. 4 is finished inside the select kernel, straight from the attention side output
        rule.logits = logits; rule.ml = ml; rule.n_heads = m.n_q_heads; rule.T = Tl; rule.scores_out = sc;
      } else if (side) {
        FASTAV_TRY(launch_score_finalize(logits, ml, nullptr, cu_l, B, Tl, maxlen_stage[stage], m.n_q_heads, 1, sc, s));
      } else {
        FASTAV_TRY(launch_score_logits(qkv, qkv_stride, kptr, qkv_stride, cu_l, B, Tl, maxlen_stage[stage], m.n_q_heads,
                                       m.n_kv_heads, m.head_dim, n_last, logits, partials, m.dtype, s));
        FASTAV_TRY(launch_score_finalize(logits, nullptr, partials, cu_l, B, Tl, maxlen_stage[stage], m.n_q_heads, n_last, sc, s));
      }
      const int32_t* cu_nx = cu_dev + (size_t)(stage + 1) * (B + 1);
      int32_t* kidx = (out->prune_keep_idx_out && out->prune_keep_idx_out[pi]) ? out->prune_keep_idx_out[pi] : keep_idx_ws;
      FASTAV_TRY(launch_select(sc, prot[cur], cu_l, cu_nx, B, maxlen_stage[stage], kidx,
                               5.0 * Tl + 4.0 * T_stage[stage + 1], s, rule));
      // The attention output is not compacted where the O projection can read its rows through the keep list (one
      // tensor less to move here; the projection's operand copies fetch the same bytes either way).
      if (g_options[FASTAV_OPT_FUSED_GATHER_OPROJ] && linear_takes_rows(T_stage[stage + 1], m.hidden, qd, FASTAV_EPI_RESADD, m.dtype, Tl)) {
        o_rows.idx = kidx; o_rows.n_src = Tl;
      }
      GatherTensor g[6] = {{resid[cur], resid[cur ^ 1], (int64_t)m.hidden * 4, 0},
                           {pos[cur], pos[cur ^ 1], 4, 0},
                           {prot[cur], prot[cur ^ 1], 1, 0},
                           {kptr, k_out, k_out ? (int64_t)kd * (int64_t)es : 0, qkv_stride * (int64_t)es},
                           {vptr, v_out, v_out ? (int64_t)kd * (int64_t)es : 0, qkv_stride * (int64_t)es},
                           {attn[0], attn[1], (int64_t)qd * (int64_t)es, 0}};
      FASTAV_TRY(launch_gather(g, o_rows.idx ? 5 : 6, kidx, T_stage[stage + 1], s));
      cur ^= 1; ++stage; ++pi;
      attn_cur = o_rows.idx ? attn[0] : attn[1];
    } else {
      // this layer's K and V rows go to the caller's cache in one launch, unless they were produced there
      GatherTensor kvc[2] = {{kptr, k_out, k_out ? (int64_t)kd * (int64_t)es : 0, qkv_stride * (int64_t)es},
                             {vptr, v_out, v_out ? (int64_t)kd * (int64_t)es : 0, qkv_stride * (int64_t)es}};
      if (!kv_direct && (k_out || v_out)) FASTAV_TRY(launch_gather(kvc, 2, nullptr, Tl, s));
    }
    const int64_t To = T_stage[stage];
    // A split-K residual product leaves its ordered sum of partial tiles to the RMSNorm that follows, which reads
    // the residual anyway (same additions in the same order as the separate reduction kernel, one launch less).
    const bool defer = g_options[FASTAV_OPT_FUSED_SPLITK_NORM] != 0;
    SplitKPending pend_o;
    FASTAV_TRY(launch_linear(attn_cur, W.wo, nullptr, resid[cur], To, m.hidden, qd, FASTAV_EPI_RESADD, m.dtype, gscr, ws.gemm_scratch_bytes, s,
                             defer ? &pend_o : nullptr, o_rows));
    FASTAV_TRY(launch_rmsnorm(resid[cur], W.g_mlp, hn, To, m.hidden, m.rms_eps, m.dtype, s, &pend_o));
    FASTAV_TRY(launch_linear(hn, W.w_gate, W.w_up, hmlp, To, m.mlp_dim, m.hidden, FASTAV_EPI_SWIGLU, m.dtype, nullptr, 0, s));
    // the down projection's sum can wait for the next layer's first RMSNorm unless something reads the residual first:
    // the last layer's output, a per-layer output, or a GLOBAL prune at the next layer's input
    const bool next_reads_resid = l + 1 == m.n_layers || (out->layer_x_out && out->layer_x_out[l]) ||
                                  (pi < n_prunes && prunes[pi].layer == l + 1 && prunes[pi].kind == FASTAV_GLOBAL);
    FASTAV_TRY(launch_linear(hmlp, W.w_down, nullptr, resid[cur], To, m.hidden, m.mlp_dim, FASTAV_EPI_RESADD, m.dtype, gscr, ws.gemm_scratch_bytes, s,
                             defer && !next_reads_resid ? &pend_down : nullptr));
    if (out->layer_x_out && out->layer_x_out[l])
      FASTAV_TRY(launch_copy_rows(resid[cur], (int64_t)m.hidden * 4, out->layer_x_out[l], (int64_t)m.hidden * 4, To, nullptr, s));
  }
  const int64_t Tf = T_stage[stage];
  FASTAV_TRY(launch_copy_rows(resid[cur], (int64_t)m.hidden * 4, out->x_out, (int64_t)m.hidden * 4, Tf, nullptr, s));
  FASTAV_TRY(launch_copy_rows(pos[cur], 4, out->kept_pos_out, 4, Tf, nullptr, s));
  FASTAV_TRY(launch_copy_rows(cu_dev + (size_t)stage * (B + 1), 4, out->cu_seqlens_out, 4, B + 1, nullptr, s));
  return FASTAV_OK;
}

size_t fastav_score_workspace_bytes(int32_t n_q_heads, int64_t total_tokens, int32_t batch, int32_t n_last) {
  if (n_q_heads < 1 || total_tokens < 0 || batch < 1 || n_last < 1) return 0;
  return align_up(score_logits_bytes(n_q_heads, total_tokens, n_last), 256) +
         align_up(score_partials_bytes(n_q_heads, total_tokens, batch, n_last), 256);
}

fastav_status_t fastav_score(const fastav_model_t* model, const void* q, int64_t q_row_stride, const void* k,
                             int64_t k_row_stride, const int32_t* cu_seqlens_dev, int32_t batch, int64_t total_tokens,
                             int32_t max_seqlen, int32_t n_last, float* scores_out, void* workspace,
                             size_t workspace_bytes, void* stream) {
  FASTAV_TRY(check_model(model));
  if (!q || !k || !cu_seqlens_dev || !scores_out || !workspace) return fail(FASTAV_EINVAL, "a pointer argument is NULL");
  if (batch < 1 || total_tokens < 0 || max_seqlen < 0 || max_seqlen > total_tokens) return fail(FASTAV_EINVAL, "bad batch/total_tokens/max_seqlen");
  if (n_last < 1 || n_last > FASTAV_MAX_N_LAST) return fail(FASTAV_EINVAL, "n_last must be in [1, %d]", FASTAV_MAX_N_LAST);
  const int64_t qd = (int64_t)model->n_q_heads * model->head_dim, kd = (int64_t)model->n_kv_heads * model->head_dim;
  if (q_row_stride < qd || k_row_stride < kd) return fail(FASTAV_EINVAL, "row strides are smaller than a row");
  const size_t es = model->dtype == FASTAV_BF16 ? 2 : 4;
  if (((uintptr_t)q % 16) || ((uintptr_t)k % 16) || (q_row_stride * es) % 16 || (k_row_stride * es) % 16 || ((uintptr_t)workspace % 256))
    return fail(FASTAV_EINVAL, "q, k and their row strides must be 16-byte aligned, workspace 256-byte aligned");
  const size_t need = fastav_score_workspace_bytes(model->n_q_heads, total_tokens, batch, n_last);
  if (workspace_bytes < need) return fail(FASTAV_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  float* logits = (float*)workspace;
  float* partials = (float*)((char*)workspace + align_up(score_logits_bytes(model->n_q_heads, total_tokens, n_last), 256));
  hipStream_t s = (hipStream_t)stream;
  FASTAV_TRY(launch_score_logits(q, q_row_stride, k, k_row_stride, cu_seqlens_dev, batch, total_tokens, max_seqlen,
                                 model->n_q_heads, model->n_kv_heads, model->head_dim, n_last, logits, partials,
                                 model->dtype, s));
  return launch_score_finalize(logits, nullptr, partials, cu_seqlens_dev, batch, total_tokens, max_seqlen,
                               model->n_q_heads, n_last, scores_out, s);
}

// ---- Eq. 4 without a workspace argument: the scratch of the score kernels (last-row logits and the per-chunk
// (max, sum) partials) lives in a fixed array inside the library's code object.  Every GPU holds its own copy at its
// own address; the address is looked up once per device and only that pointer is ever handed to a kernel (the
// array's name is a host-side stand-in, not a device address).
static __device__ __align__(256) unsigned char g_score_scratch[FASTAV_SCORE_STATIC_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of g_score_scratch on the current device (looked up on the first call there).
fastav_status_t score_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(FASTAV_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(FASTAV_EUNSUPPORTED, "device index %d is beyond the %d this library tracks", dev, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_score_scratch));
    if (e != hipSuccess || !p) return fail(FASTAV_EHIP, "hipGetSymbolAddress(score scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return FASTAV_OK;
}
}  // namespace

fastav_status_t fastav_score_static(const fastav_model_t* model, const void* q, int64_t q_row_stride, const void* k,
                                    int64_t k_row_stride, const int32_t* cu_seqlens_dev, int32_t batch,
                                    int64_t total_tokens, int32_t max_seqlen, int32_t n_last, float* scores_out,
                                    void* stream) {
  FASTAV_TRY(check_model(model));
  if (batch < 1 || total_tokens < 0 || n_last < 1 || n_last > FASTAV_MAX_N_LAST)
    return fail(FASTAV_EINVAL, "bad batch/total_tokens/n_last");
  const size_t need = fastav_score_workspace_bytes(model->n_q_heads, total_tokens, batch, n_last);
  if (need > (size_t)FASTAV_SCORE_STATIC_BYTES)
    return fail(FASTAV_EWORKSPACE, "fastav_score_static: this problem needs %zu bytes of scratch, the built-in buffer holds %zu "
                "(n_last * n_q_heads * total_tokens * 4 bytes plus the chunk partials); use fastav_score with a workspace",
                need, (size_t)FASTAV_SCORE_STATIC_BYTES);
  void* scratch = nullptr;
  FASTAV_TRY(score_scratch(&scratch));
  // every position of the scratch that the finalize pass reads is written by the logits pass of the same call,
  // so nothing has to be cleared between calls
  return fastav_score(model, q, q_row_stride, k, k_row_stride, cu_seqlens_dev, batch, total_tokens, max_seqlen, n_last,
                      scores_out, scratch, (size_t)FASTAV_SCORE_STATIC_BYTES, stream);
}

size_t fastav_select_workspace_bytes(int32_t batch) {
  if (batch < 1) return 0;
  return align_up((size_t)(batch + 1) * 4, 256);
}

fastav_status_t fastav_select_gather(const float* scores, const uint8_t* protected_mask, const int32_t* cu_seqlens,
                                     const int32_t* keep_counts, int32_t batch, int32_t n_tensors,
                                     const void* const* src, void* const* dst, const int64_t* row_bytes,
                                     int32_t* keep_idx_out, int32_t* cu_seqlens_out, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  if (!protected_mask || !cu_seqlens || !keep_counts || !keep_idx_out || !cu_seqlens_out || !workspace)
    return fail(FASTAV_EINVAL, "a pointer argument is NULL");
  if (batch < 1) return fail(FASTAV_EINVAL, "batch must be >= 1");
  if (n_tensors < 0 || n_tensors > FASTAV_MAX_GATHER_TENSORS) return fail(FASTAV_EINVAL, "n_tensors must be in [0, %d]", FASTAV_MAX_GATHER_TENSORS);
  if (n_tensors > 0 && (!src || !dst || !row_bytes)) return fail(FASTAV_EINVAL, "src/dst/row_bytes is NULL");
  if (workspace_bytes < fastav_select_workspace_bytes(batch) || ((uintptr_t)workspace % 4))
    return fail(FASTAV_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, fastav_select_workspace_bytes(batch));
  if (cu_seqlens[0] != 0) return fail(FASTAV_EINVAL, "cu_seqlens[0] must be 0");
  std::vector<int32_t> cu_out(batch + 1);
  cu_out[0] = 0;
  int max_len = 0;
  for (int b = 0; b < batch; ++b) {
    const int64_t n = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
    if (n < 0) return fail(FASTAV_EINVAL, "cu_seqlens must be non-decreasing");
    if (keep_counts[b] < 0 || keep_counts[b] > n) return fail(FASTAV_EINVAL, "keep_counts[%d] = %d exceeds the sample's %lld rows", b, keep_counts[b], (long long)n);
    cu_out[b + 1] = cu_out[b] + keep_counts[b];
    if (n > max_len) max_len = (int)n;
  }
  GatherTensor g[FASTAV_MAX_GATHER_TENSORS];
  for (int i = 0; i < n_tensors; ++i) {
    if (row_bytes[i] < 0) return fail(FASTAV_EINVAL, "row_bytes[%d] is negative", i);
    if (row_bytes[i] > 0 && (!src[i] || !dst[i])) return fail(FASTAV_EINVAL, "src[%d] or dst[%d] is NULL", i, i);
    g[i] = GatherTensor{src[i], dst[i], row_bytes[i], 0};
  }
  hipStream_t s = (hipStream_t)stream;
  int32_t* cu_dev = (int32_t*)workspace;
  FASTAV_TRY(upload_small(cu_dev, cu_seqlens, (size_t)(batch + 1) * 4, s));
  FASTAV_TRY(upload_small(cu_seqlens_out, cu_out.data(), (size_t)(batch + 1) * 4, s));
  FASTAV_TRY(launch_select(scores, protected_mask, cu_dev, cu_seqlens_out, batch, max_len, keep_idx_out,
                           (scores ? 5.0 : 1.0) * cu_seqlens[batch] + 4.0 * cu_out[batch], s,
                           SelectRule{scores ? kSelHighScore : kSelEarliest, 0, nullptr}));
  return launch_gather(g, n_tensors, keep_idx_out, cu_out[batch], s);
}

fastav_status_t fastav_rmsnorm(const float* x, const void* g, void* y, int64_t rows, int32_t d, float eps,
                               int32_t dtype, void* stream) {
  if (!x || !g || !y) return fail(FASTAV_EINVAL, "a pointer argument is NULL");
  if (rows < 0 || d < 1 || (dtype != FASTAV_BF16 && dtype != FASTAV_F32)) return fail(FASTAV_EINVAL, "bad rows/d/dtype");
  if ((d % 4 == 0) && ((uintptr_t)x % 16)) return fail(FASTAV_EINVAL, "x must be 16-byte aligned");
  return launch_rmsnorm(const_cast<float*>(x), g, y, rows, d, eps, dtype, (hipStream_t)stream);
}

fastav_status_t fastav_rope(void* x, int64_t row_stride, const int32_t* pos, int64_t rows, int32_t n_heads,
                            int32_t head_dim, float base, int32_t dtype, void* stream) {
  if (!x || !pos) return fail(FASTAV_EINVAL, "a pointer argument is NULL");
  if (rows < 0 || n_heads < 0 || head_dim < 2 || (head_dim & 1) || head_dim > 512 || row_stride < (int64_t)n_heads * head_dim ||
      (dtype != FASTAV_BF16 && dtype != FASTAV_F32) || !(base > 1.0f))
    return fail(FASTAV_EINVAL, "bad rows/n_heads/head_dim/row_stride/dtype/base");
  return launch_rope(x, row_stride, pos, rows, n_heads, head_dim, base, dtype, (hipStream_t)stream);
}

size_t fastav_linear_workspace_bytes(void) { return mfma_linear_scratch_bytes(); }

fastav_status_t fastav_linear(const void* a, const void* w, const void* w2, void* c, int64_t m, int32_t n, int32_t k,
                              int32_t epilogue, int32_t dtype, void* workspace, size_t workspace_bytes, void* stream) {
  if (workspace && ((uintptr_t)workspace % 256)) return fail(FASTAV_EINVAL, "workspace must be 256-byte aligned");
  if (!a || !w || !c) return fail(FASTAV_EINVAL, "a pointer argument is NULL");
  if (m < 0 || n < 1 || k < 1 || (dtype != FASTAV_BF16 && dtype != FASTAV_F32)) return fail(FASTAV_EINVAL, "bad m/n/k/dtype");
  if (epilogue < FASTAV_EPI_STORE || epilogue > FASTAV_EPI_SWIGLU) return fail(FASTAV_EINVAL, "bad epilogue");
  if (epilogue == FASTAV_EPI_SWIGLU && !w2) return fail(FASTAV_EINVAL, "w2 is NULL for the SwiGLU epilogue");
  return launch_linear(a, w, w2, c, m, n, k, epilogue, dtype, workspace, workspace ? workspace_bytes : 0, (hipStream_t)stream);
}

fastav_status_t fastav_attention(const fastav_model_t* model, const void* q, int64_t q_row_stride, const void* k,
                                 const void* v, int64_t kv_row_stride, void* o, int64_t o_row_stride,
                                 const int32_t* cu_seqlens_dev, int32_t batch, int64_t total_tokens,
                                 int32_t max_seqlen, float* last_logits, float* last_ml, void* stream) {
  FASTAV_TRY(check_model(model));
  if (!q || !k || !v || !o || !cu_seqlens_dev) return fail(FASTAV_EINVAL, "a pointer argument is NULL");
  if ((last_logits == nullptr) != (last_ml == nullptr)) return fail(FASTAV_EINVAL, "last_logits and last_ml go together");
  if (batch < 1 || total_tokens < 0 || max_seqlen < 0 || max_seqlen > total_tokens) return fail(FASTAV_EINVAL, "bad batch/total_tokens/max_seqlen");
  const int64_t qd = (int64_t)model->n_q_heads * model->head_dim, kd = (int64_t)model->n_kv_heads * model->head_dim;
  if (q_row_stride < qd || o_row_stride < qd || kv_row_stride < kd) return fail(FASTAV_EINVAL, "row strides are smaller than a row");
  return launch_attention(q, q_row_stride, k, v, kv_row_stride, o, o_row_stride, cu_seqlens_dev, batch, total_tokens,
                          max_seqlen, model->n_q_heads, model->n_kv_heads, model->head_dim, last_logits, last_ml,
                          model->dtype, 0.0, (hipStream_t)stream);
}

// ---- decode step ------------------------------------------------------------------------------------
struct DecodeWs { size_t x, hn, qkv, attn, hmlp, part, part_bytes, total; };

static DecodeWs carve_decode(const fastav_model_t& m, int B) {
  DecodeWs w;
  size_t at = 0;
  auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes, 256); return o; };
  const size_t qd = (size_t)m.n_q_heads * m.head_dim, kd = (size_t)m.n_kv_heads * m.head_dim;
  w.x = take((size_t)B * m.hidden * 4);
  w.hn = take((size_t)B * m.hidden * 2);
  w.qkv = take((size_t)B * (qd + 2 * kd) * 2);
  w.attn = take((size_t)B * qd * 2);
  w.hmlp = take((size_t)B * m.mlp_dim * 2);
  w.part_bytes = decode_attn_workspace_bytes(B, m.n_q_heads, m.head_dim, 64);
  w.part = take(w.part_bytes);
  w.total = at;
  return w;
}

fastav_status_t fastav_decode_workspace_bytes(fastav_handle_t h, int32_t max_batch, size_t* out) {
  if (!h || !out) return fail(FASTAV_EINVAL, "handle or out is NULL");
  if (max_batch < 1 || max_batch > FASTAV_MAX_DECODE_BATCH) return fail(FASTAV_EINVAL, "max_batch must be in [1, %d]", FASTAV_MAX_DECODE_BATCH);
  *out = carve_decode(h->m, max_batch).total;
  return FASTAV_OK;
}

fastav_status_t fastav_decode_step(fastav_handle_t h, const fastav_decode_in_t* in, float* x_out, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  if (!h || !in || !x_out) return fail(FASTAV_EINVAL, "handle, in or x_out is NULL");
  const fastav_model_t& m = h->m;
  hipStream_t s = (hipStream_t)stream;
  const int B = in->batch;
  if (B < 1 || B > FASTAV_MAX_DECODE_BATCH) return fail(FASTAV_EINVAL, "batch must be in [1, %d]", FASTAV_MAX_DECODE_BATCH);
  if (m.dtype != FASTAV_BF16) return fail(FASTAV_EUNSUPPORTED, "the decode step is built for bf16 models");
  if (!in->x_new || !in->pos_new || !in->k_prefix || !in->v_prefix || !in->cu_prefix || !in->max_prefix)
    return fail(FASTAV_EINVAL, "x_new, pos_new, k_prefix, v_prefix, cu_prefix and max_prefix must be non-NULL");
  if (in->gen_len < 0 || in->gen_cap < 0 || in->gen_len > in->gen_cap) return fail(FASTAV_EINVAL, "need 0 <= gen_len <= gen_cap");
  if ((in->k_gen == nullptr) != (in->v_gen == nullptr)) return fail(FASTAV_EINVAL, "k_gen and v_gen go together");
  if (in->gen_len > 0 && !in->k_gen) return fail(FASTAV_EINVAL, "gen_len > 0 needs k_gen / v_gen");
  if (in->k_gen && in->gen_len >= in->gen_cap) return fail(FASTAV_EINVAL, "the generated-token caches are full (gen_len == gen_cap)");
  if (!workspace || ((uintptr_t)workspace % 256)) return fail(FASTAV_EINVAL, "workspace must be non-NULL and 256-byte aligned");
  if (((uintptr_t)in->x_new % 16) || ((uintptr_t)x_out % 16)) return fail(FASTAV_EINVAL, "x_new and x_out must be 16-byte aligned");
  const DecodeWs ws = carve_decode(m, B);
  if (workspace_bytes < ws.total) return fail(FASTAV_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, ws.total);
  const int qd = m.n_q_heads * m.head_dim, kd = m.n_kv_heads * m.head_dim, qkvd = qd + 2 * kd;
  if (!skinny_linear_supported(B, qd, m.hidden, m.dtype, qkvd) || !skinny_linear_supported(B, kd, m.hidden, m.dtype, qkvd) ||
      !skinny_linear_supported(B, m.hidden, qd, m.dtype, m.hidden) || !skinny_linear_supported(B, m.mlp_dim, m.hidden, m.dtype, m.mlp_dim) ||
      !skinny_linear_supported(B, m.hidden, m.mlp_dim, m.dtype, m.hidden))
    return fail(FASTAV_EUNSUPPORTED, "decode step: hidden, heads*head_dim and mlp_dim must be multiples of 128");
  for (int l = 0; l < m.n_layers; ++l) {
    if (!h->has_w[l]) return fail(FASTAV_EINVAL, "weights of layer %d were never set", l);
    if (!in->k_prefix[l] || !in->v_prefix[l] || !in->cu_prefix[l]) return fail(FASTAV_EINVAL, "a cache pointer of layer %d is NULL", l);
    if (in->max_prefix[l] < 0) return fail(FASTAV_EINVAL, "max_prefix[%d] is negative", l);
    if (in->k_gen && (!in->k_gen[l] || !in->v_gen[l])) return fail(FASTAV_EINVAL, "a generated-token cache pointer of layer %d is NULL", l);
  }
  char* base = (char*)workspace;
  float* x = (float*)(base + ws.x);
  void* hn = base + ws.hn;
  char* qkv = base + ws.qkv;
  void* attn = base + ws.attn;
  void* hmlp = base + ws.hmlp;

  FASTAV_TRY(launch_to_f32(in->x_new, x, (int64_t)B * m.hidden, m.dtype, s));
  for (int l = 0; l < m.n_layers; ++l) {
    const fastav_layer_weights_t& W = h->w[l];
    // for a few rows RMSNorm is folded into the projection that consumes it (every workgroup normalises the
    // rows into its LDS): one launch less per norm
    const bool fuse_norm = skinny_norm_supported(B, m.hidden);
    if (!fuse_norm) FASTAV_TRY(launch_rmsnorm(x, W.g_attn, hn, B, m.hidden, m.rms_eps, m.dtype, s));
    const void* seg[3] = {W.wq, W.wk, W.wv};
    const int rows[3] = {qd, kd, kd};
    // a single sample: the projection kernel rotates the query and key heads itself (they lead the row)
    const bool fuse_rope = gemv_rows_fuses_rope(B, qkvd, m.hidden, fuse_norm, qd + kd, m.head_dim);
    FASTAV_TRY(launch_skinny_linear(hn, seg, rows, 3, nullptr, qkv, qkvd, B, qkvd, m.hidden, FASTAV_EPI_STORE, s,
                                    fuse_norm ? x : nullptr, W.g_attn, m.rms_eps, fuse_rope ? in->pos_new : nullptr,
                                    qd + kd, m.head_dim, m.rope_base));
    // the key heads follow the query heads in the row: one launch rotates both
    if (!fuse_rope)
      FASTAV_TRY(launch_rope(qkv, qkvd, in->pos_new, B, m.n_q_heads + m.n_kv_heads, m.head_dim, m.rope_base, m.dtype, s));
    const void* kg = in->k_gen ? in->k_gen[l] : nullptr;
    const void* vg = in->v_gen ? in->v_gen[l] : nullptr;
    // bytes the attention step has to move: the caches once (upper bound: the longest sample for all)
    const double abytes = 2.0 * B * ((double)in->max_prefix[l] + in->gen_len + 1) * kd * 2.0;
    FASTAV_TRY(launch_decode_attention(qkv, qkv + (size_t)qd * 2, qkv + (size_t)(qd + kd) * 2, qkvd, in->k_prefix[l],
                                       in->v_prefix[l], in->cu_prefix[l], in->max_prefix[l], kg, vg, in->gen_len,
                                       in->gen_cap, B, m.n_q_heads, m.n_kv_heads, m.head_dim, (float*)(base + ws.part),
                                       ws.part_bytes, attn, qd, abytes, s));
    if (in->k_gen) {
      // append the token's own key / value: slot gen_len of [B, gen_cap, kd]
      FASTAV_TRY(launch_copy_rows(qkv + (size_t)qd * 2, (int64_t)qkvd * 2, (char*)in->k_gen[l] + (size_t)in->gen_len * kd * 2,
                                  (int64_t)kd * 2, B, nullptr, s, (int64_t)in->gen_cap * kd * 2));
      FASTAV_TRY(launch_copy_rows(qkv + (size_t)(qd + kd) * 2, (int64_t)qkvd * 2, (char*)in->v_gen[l] + (size_t)in->gen_len * kd * 2,
                                  (int64_t)kd * 2, B, nullptr, s, (int64_t)in->gen_cap * kd * 2));
    }
    const void* so[1] = {W.wo};
    const int ro[1] = {m.hidden};
    FASTAV_TRY(launch_skinny_linear(attn, so, ro, 1, nullptr, x, m.hidden, B, m.hidden, qd, FASTAV_EPI_RESADD, s));
    if (!fuse_norm) FASTAV_TRY(launch_rmsnorm(x, W.g_mlp, hn, B, m.hidden, m.rms_eps, m.dtype, s));
    const void* sg[1] = {W.w_gate};
    const int rg[1] = {m.mlp_dim};
    FASTAV_TRY(launch_skinny_linear(hn, sg, rg, 1, W.w_up, hmlp, m.mlp_dim, B, m.mlp_dim, m.hidden, FASTAV_EPI_SWIGLU, s,
                                    fuse_norm ? x : nullptr, W.g_mlp, m.rms_eps));
    const void* sd[1] = {W.w_down};
    FASTAV_TRY(launch_skinny_linear(hmlp, sd, ro, 1, nullptr, x, m.hidden, B, m.hidden, m.mlp_dim, FASTAV_EPI_RESADD, s));
  }
  FASTAV_TRY(launch_copy_rows(x, (int64_t)m.hidden * 4, x_out, (int64_t)m.hidden * 4, B, nullptr, s));
  return FASTAV_OK;
}

// ---- attention rollout (Eq. 2-3) ----------------------------------------------------------------------
size_t fastav_attention_map_workspace_bytes(int32_t n, int32_t n_q_heads) {
  if (n < 0 || n_q_heads < 1) return 0;
  return attention_map_stats_bytes(n, n_q_heads);
}

fastav_status_t fastav_attention_map(const fastav_model_t* model, const void* q, int64_t q_row_stride, const void* k,
                                     int64_t k_row_stride, int32_t n, void* a_out, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  FASTAV_TRY(check_model(model));
  if (!q || !k || !a_out || !workspace) return fail(FASTAV_EINVAL, "a pointer argument is NULL");
  if (model->dtype != FASTAV_BF16) return fail(FASTAV_EUNSUPPORTED, "the attention map is built for bf16 inputs");
  if (n < 1 || n % 4) return fail(FASTAV_EINVAL, "n must be a positive multiple of 4");
  if (((uintptr_t)workspace % 256) || workspace_bytes < attention_map_stats_bytes(n, model->n_q_heads))
    return fail(FASTAV_EWORKSPACE, "workspace must be 256-byte aligned and hold fastav_attention_map_workspace_bytes()");
  if (q_row_stride < (int64_t)model->n_q_heads * model->head_dim || k_row_stride < (int64_t)model->n_kv_heads * model->head_dim)
    return fail(FASTAV_EINVAL, "row strides are smaller than a row");
  return launch_attention_map(q, q_row_stride, k, k_row_stride, n, model->n_q_heads, model->n_kv_heads, model->head_dim,
                              (float*)workspace, a_out, (hipStream_t)stream);
}

struct RolloutWs { size_t resid, hn, qkv, attn, hmlp, pos, cu, stats, a16, c, rt16, gemm, gemm_bytes, total; };

static RolloutWs carve_rollout(const fastav_model_t& m, int64_t n) {
  RolloutWs w;
  size_t at = 0;
  auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes, 256); return o; };
  const size_t qd = (size_t)m.n_q_heads * m.head_dim, kd = (size_t)m.n_kv_heads * m.head_dim;
  w.resid = take((size_t)n * m.hidden * 4);
  w.hn = take((size_t)n * m.hidden * 2);
  w.qkv = take((size_t)n * (qd + 2 * kd) * 2);
  w.attn = take((size_t)n * qd * 2);
  w.hmlp = take((size_t)n * m.mlp_dim * 2);
  w.pos = take((size_t)n * 4);
  w.cu = take(256);
  w.stats = take(attention_map_stats_bytes((int)n, m.n_q_heads));
  w.a16 = take((size_t)n * n * 2);
  w.c = take((size_t)n * n * 4);
  w.rt16 = take((size_t)n * n * 2);
  w.gemm_bytes = mfma_linear_scratch_bytes();
  w.gemm = take(w.gemm_bytes);
  w.total = at;
  return w;
}

fastav_status_t fastav_rollout_workspace_bytes(fastav_handle_t h, int32_t n, size_t* out) {
  if (!h || !out) return fail(FASTAV_EINVAL, "handle or out is NULL");
  if (n < 1 || n % 4) return fail(FASTAV_EINVAL, "n must be a positive multiple of 4");
  *out = carve_rollout(h->m, n).total;
  return FASTAV_OK;
}

fastav_status_t fastav_rollout(fastav_handle_t h, const void* x, int32_t n, float alpha, int32_t upto_layers,
                               float* rt_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!h || !x || !rt_out) return fail(FASTAV_EINVAL, "handle, x or rt_out is NULL");
  const fastav_model_t& m = h->m;
  hipStream_t s = (hipStream_t)stream;
  if (m.dtype != FASTAV_BF16) return fail(FASTAV_EUNSUPPORTED, "the rollout is built for bf16 models");
  if (n < 1 || n % 4) return fail(FASTAV_EINVAL, "n must be a positive multiple of 4");
  if (!(alpha >= 0.f && alpha <= 1.f)) return fail(FASTAV_EINVAL, "alpha must lie in [0, 1]");
  if (upto_layers < 1 || upto_layers > m.n_layers) return fail(FASTAV_EINVAL, "upto_layers must be in [1, n_layers]");
  if (!workspace || ((uintptr_t)workspace % 256)) return fail(FASTAV_EINVAL, "workspace must be non-NULL and 256-byte aligned");
  if (((uintptr_t)x % 16) || ((uintptr_t)rt_out % 16)) return fail(FASTAV_EINVAL, "x and rt_out must be 16-byte aligned");
  const RolloutWs ws = carve_rollout(m, n);
  if (workspace_bytes < ws.total) return fail(FASTAV_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, ws.total);
  for (int l = 0; l < upto_layers; ++l)
    if (!h->has_w[l]) return fail(FASTAV_EINVAL, "weights of layer %d were never set", l);
  char* base = (char*)workspace;
  float* resid = (float*)(base + ws.resid);
  void* hn = base + ws.hn;
  char* qkv = base + ws.qkv;
  void* attn = base + ws.attn;
  void* hmlp = base + ws.hmlp;
  int32_t* pos = (int32_t*)(base + ws.pos);
  int32_t* cu = (int32_t*)(base + ws.cu);
  const int qd = m.n_q_heads * m.head_dim, kd = m.n_kv_heads * m.head_dim, qkvd = qd + 2 * kd;
  const int32_t cu_host[2] = {0, n};
  FASTAV_TRY(upload_small(cu, cu_host, sizeof(cu_host), s));
  FASTAV_TRY(launch_iota(pos, n, s));
  FASTAV_TRY(launch_to_f32(x, resid, (int64_t)n * m.hidden, m.dtype, s));
  FASTAV_TRY(launch_rollout_init(rt_out, base + ws.rt16, n, s));
  for (int l = 0; l < upto_layers; ++l) {
    const fastav_layer_weights_t& W = h->w[l];
    FASTAV_TRY(launch_rmsnorm(resid, W.g_attn, hn, n, m.hidden, m.rms_eps, m.dtype, s));
    const void* seg[3] = {W.wq, W.wk, W.wv};
    const int rows[3] = {qd, kd, kd};
    FASTAV_TRY(linear_segments(hn, seg, rows, 3, nullptr, qkv, qkvd, n, m.hidden, FASTAV_EPI_STORE, m.dtype, nullptr, 0, s));
    FASTAV_TRY(launch_rope(qkv, qkvd, pos, n, m.n_q_heads + m.n_kv_heads, m.head_dim, m.rope_base, m.dtype, s));
    FASTAV_TRY(launch_attention_map(qkv, qkvd, qkv + (size_t)qd * 2, qkvd, n, m.n_q_heads, m.n_kv_heads, m.head_dim,
                                    (float*)(base + ws.stats), base + ws.a16, s));
    FASTAV_TRY(launch_rollout_step(rt_out, base + ws.rt16, base + ws.a16, (float*)(base + ws.c), n, alpha,
                                   base + ws.gemm, ws.gemm_bytes, s));
    if (l + 1 == upto_layers) break;                   // the hidden state past the last requested layer is not needed
    FASTAV_TRY(launch_attention(qkv, qkvd, qkv + (size_t)qd * 2, qkv + (size_t)(qd + kd) * 2, qkvd, attn, qd, cu, 1, n, n,
                                m.n_q_heads, m.n_kv_heads, m.head_dim, nullptr, nullptr, m.dtype,
                                2.0 * m.n_q_heads * m.head_dim * (double)n * ((double)n + 1.0), s));
    FASTAV_TRY(launch_linear(attn, W.wo, nullptr, resid, n, m.hidden, qd, FASTAV_EPI_RESADD, m.dtype, base + ws.gemm, ws.gemm_bytes, s));
    FASTAV_TRY(launch_rmsnorm(resid, W.g_mlp, hn, n, m.hidden, m.rms_eps, m.dtype, s));
    FASTAV_TRY(launch_linear(hn, W.w_gate, W.w_up, hmlp, n, m.mlp_dim, m.hidden, FASTAV_EPI_SWIGLU, m.dtype, nullptr, 0, s));
    FASTAV_TRY(launch_linear(hmlp, W.w_down, nullptr, resid, n, m.hidden, m.mlp_dim, FASTAV_EPI_RESADD, m.dtype, base + ws.gemm, ws.gemm_bytes, s));
  }
  return FASTAV_OK;
}

fastav_status_t fastav_rollout_cutoff(const float* rt, int32_t n, const uint8_t* protected_mask, float threshold,
                                      float* influence_out, int32_t* cutoff_out, void* stream) {
  if (!rt || !protected_mask || !influence_out || !cutoff_out) return fail(FASTAV_EINVAL, "a pointer argument is NULL");
  if (n < 4 || n % 4) return fail(FASTAV_EINVAL, "n must be a positive multiple of 4");
  if (!(threshold >= 0.f)) return fail(FASTAV_EINVAL, "threshold must be >= 0");
  if ((uintptr_t)rt % 16) return fail(FASTAV_EINVAL, "rt must be 16-byte aligned");
  return launch_rollout_cutoff(rt, n, protected_mask, threshold, influence_out, cutoff_out, (hipStream_t)stream);
}

}  // extern "C"
