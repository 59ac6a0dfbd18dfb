/*
 * fastav.h — C ABI of the MI355X (gfx950) FastAV pruned-prefill library.
 *
 * The library runs the prefill forward of a pre-norm decoder stack (RMSNorm, QKV projection, rotate-half
 * RoPE, causal grouped-query attention, output projection, SwiGLU MLP) over a packed batch of audio-visual
 * token sequences, and applies FastAV's two-stage token pruning on the way (paper Section 2.2, Fig. 3):
 *
 *   GLOBAL prune  (Section 2.2 "Global pruning"): at a middle layer, video/audio tokens in later
 *                 positions are dropped; no scores are involved.
 *   FINE prune    (Section 2.2 "Fine pruning", Eq. 4): s = mean over heads of softmax(Q_last K^T); the
 *                 lowest-scoring tokens are dropped at the layer, and every later layer sees the
 *                 survivors only.  The full attention map is never formed.
 *
 * Conventions for every entry point
 *   - "dev" pointers are device (HBM) addresses on the current HIP device, "host" pointers are ordinary
 *     host memory.  The caller owns every buffer.  Nothing here allocates or frees device memory, and
 *     nothing synchronises: all work is enqueued on the caller's stream (a hipStream_t passed as void*,
 *     NULL = the default stream) and host arrays may be reused as soon as the call returns.
 *   - Every argument error is detected on the host before the first launch; the return code is the only
 *     error channel and fastav_last_error() gives a thread-local description.  Inputs are never written.
 *   - Matrices are row-major.  Weight matrices are stored [out_features, in_features].
 *   - Activations/weights are in the model dtype (bf16 or fp32); scores, the residual stream handed back
 *     in x_out and all index arrays are fp32 / int32.
 *   - Sequences are packed: sample b owns rows cu_seqlens[b] .. cu_seqlens[b+1]-1.
 *   - Tie rule of every selection: higher score wins; equal scores go to the lower index; NaN ranks as
 *     -inf and -0.0 equals +0.0; kept indices are returned ascending.
 */
#ifndef FASTAV_H
#define FASTAV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FASTAV_OK = 0,
  FASTAV_EINVAL = 1,       /* bad argument (null pointer, k > n, unsorted cu_seqlens, ...) */
  FASTAV_EUNSUPPORTED = 2, /* valid request the kernels do not cover (e.g. head_dim not 64/128) */
  FASTAV_EWORKSPACE = 3,   /* workspace too small; see fastav_workspace_bytes */
  FASTAV_EHIP = 4          /* a HIP launch failed; fastav_last_error() holds hipGetErrorString */
} fastav_status_t;

typedef enum { FASTAV_TEXT = 0, FASTAV_VIDEO = 1, FASTAV_AUDIO = 2 } fastav_modality_t; /* TEXT is never pruned */
typedef enum { FASTAV_GLOBAL = 0, FASTAV_FINE = 1 } fastav_prune_kind_t;
typedef enum { FASTAV_BF16 = 0, FASTAV_F32 = 1 } fastav_dtype_t;
/* Which tokens a prune step removes: the strategies compared in Tables 2 and 3 (Section 3.2, "Global pruning
 * strategy", "Fine pruning strategy").  Protected tokens stay under every strategy and the kept count depends on
 * keep_ratio alone, so all strategies of a schedule cost the same FLOPs.
 *   DEFAULT          the paper's own rule for the step's kind: GLOBAL -> LOW_INFORMATIVE, FINE -> LOW_ATTENTIVE
 *   LOW_ATTENTIVE    lowest Eq. 4 scores go (FINE steps only: a GLOBAL step acts before the layer's attention)
 *   TOP_ATTENTIVE    highest Eq. 4 scores go (FINE steps only); equal scores: the lower index stays
 *   LOW_INFORMATIVE  latest positions go, the rollout-guided rule (GLOBAL steps only)
 *   TOP_INFORMATIVE  earliest positions go, its mirror image (GLOBAL steps only)
 *   RANDOM           candidates with the lowest draw go; the draw of a token is the top 24 bits, as a fraction in
 *                    [0, 1), of mix(mix(mix(seed + G (layer + 1)) + G (sample + 1)) + position id), G = 0x9E3779B9,
 *                    mix = the 32-bit finishing mix of MurmurHash3 (h ^= h >> 16; h *= 0x85EBCA6B; h ^= h >> 13;
 *                    h *= 0xC2B2AE35; h ^= h >> 16); position id = the token's position in the original sample */
typedef enum {
  FASTAV_SEL_DEFAULT = 0, FASTAV_SEL_LOW_ATTENTIVE = 1, FASTAV_SEL_TOP_ATTENTIVE = 2, FASTAV_SEL_LOW_INFORMATIVE = 3,
  FASTAV_SEL_TOP_INFORMATIVE = 4, FASTAV_SEL_RANDOM = 5
} fastav_selector_t;

#define FASTAV_MAX_N_LAST 8     /* most last-query rows Eq. 4 may be averaged over */
#define FASTAV_MAX_PRUNES 128
#define FASTAV_MAX_GATHER_TENSORS 8
#define FASTAV_MAX_DECODE_BATCH 16 /* most samples one decode step serves (one matrix-instruction tile of rows) */

/* One modality span of a sample (Section 2.1: X = [X^vis, X^aud, X^lang]).  start is relative to the
 * sample; the spans of a sample are sorted, disjoint and cover [0, n). */
typedef struct { int32_t start, len, modality; } fastav_span_t;

/* One prune step.  layer is 0-based.  GLOBAL acts on the input of that layer; FINE uses that layer's own
 * attention and shrinks the sequence from its output projection on.  keep_ratio = 1 - P in (0, 1].
 * The array passed to fastav_prefill is sorted by (layer, kind); at most one of each kind per layer.
 * selector: a fastav_selector_t (0 = the paper's rule); seed: keys the draws of FASTAV_SEL_RANDOM.  A selector
 * that does not fit the kind is FASTAV_EINVAL. */
typedef struct { int32_t layer, kind; double keep_ratio; int32_t selector; uint32_t seed; } fastav_prune_t;

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, mlp_dim;
  float rope_base, rms_eps;
  int32_t dtype; /* fastav_dtype_t */
} fastav_model_t;

/* Device pointers in the model dtype, borrowed for the handle's lifetime.
 * g_attn,g_mlp [hidden]; wq [Hq*dh, hidden]; wk,wv [Hkv*dh, hidden]; wo [hidden, Hq*dh];
 * w_gate,w_up [mlp, hidden]; w_down [hidden, mlp]. */
typedef struct {
  const void *g_attn, *wq, *wk, *wv, *wo, *g_mlp, *w_gate, *w_up, *w_down;
} fastav_layer_weights_t;

typedef struct fastav_ctx* fastav_handle_t;

/* The packed input batch (Section 2.1). */
typedef struct {
  const void* x;               /* dev  [T, hidden] token embeddings, model dtype */
  const int32_t* cu_seqlens;   /* host [batch+1], cu_seqlens[0] = 0, strictly increasing */
  int32_t batch;
  const fastav_span_t* spans;  /* host, all samples' spans concatenated */
  const int32_t* span_offsets; /* host [batch+1]: sample b owns spans[span_offsets[b] .. span_offsets[b+1]) */
} fastav_batch_t;

/* Outputs of fastav_prefill.  T_final and the per-layer token counts are known on the host beforehand
 * from fastav_schedule.  Optional members may be NULL. */
typedef struct {
  float* x_out;                /* dev [T_final, hidden] fp32 hidden state after the last layer */
  int32_t* cu_seqlens_out;     /* dev [batch+1] */
  int32_t* kept_pos_out;       /* dev [T_final] original in-sample position of every survivor */
  void* const* kv_out;         /* optional host array [2*n_layers] of dev pointers K_0,V_0,K_1,V_1,...:
                                  post-RoPE K and V of layer l, [T_l, Hkv, head_dim] in the model dtype, where
                                  T_l counts the tokens that survive layer l (a FINE layer's K/V are
                                  compacted).  Entries may be NULL. */
  float* const* prune_scores_out;   /* optional host array [n_prunes] of dev pointers (entries may be NULL):
                                       for a FINE prune with an attentive selector, the Eq. 4 scores of the tokens
                                       entering it, packed (other prunes leave the buffer untouched) */
  int32_t* const* prune_keep_idx_out; /* optional host array [n_prunes] of dev pointers (entries may be NULL):
                                       packed row indices (into the layout entering the prune) that survive */
  float* const* layer_x_out;   /* optional host array [n_layers] of dev pointers (entries may be NULL):
                                  fp32 hidden state [T_l, hidden] leaving layer l */
} fastav_prefill_out_t;

/* ---- host helpers (no GPU work) ------------------------------------------------------------------ */

/* The keep-count rule: k = min(n, max(n_protected, ceil(keep_ratio*n - 1e-9))) in double precision
 * (Section 2.2, "Fine pruning": the share P of lowest-scoring tokens goes; keep_ratio = 1 - P).  Returns -1 on a
 * bad argument (n < 0, ratio outside (0,1], n_protected outside [0,n]). */
int64_t fastav_keep_count(int64_t n, double keep_ratio, int64_t n_protected);

/* Token counts of the whole prefill, from shapes alone (they never depend on data).
 * tokens_in_out  [n_layers] (optional): total packed tokens that enter attention at each layer;
 * tokens_out_out [n_layers] (optional): total packed tokens that leave each layer (= T_l of kv_out);
 * final_lens_out [batch]    (optional): surviving tokens per sample after the last layer.
 * Protected tokens = TEXT spans plus the last n_last positions of each sample. */
fastav_status_t fastav_schedule(const fastav_batch_t* in, const fastav_prune_t* prunes, int32_t n_prunes,
                                int32_t n_last, int32_t n_layers, int64_t* tokens_in_out,
                                int64_t* tokens_out_out, int32_t* final_lens_out);

/* Tokens per sample that LEAVE each layer (= rows per sample of that layer's K/V cache in kv_out), from
 * shapes alone: lens_out [n_layers * batch], entry [l * batch + b].  A decode step needs these to find each
 * sample's rows in a pruned layer's cache. */
fastav_status_t fastav_schedule_lens(const fastav_batch_t* in, const fastav_prune_t* prunes, int32_t n_prunes,
                                     int32_t n_last, int32_t n_layers, int32_t* lens_out);

const char* fastav_last_error(void);

/* Process-wide switches between equivalent forms of a step (the forms give the same results, bit for bit unless said otherwise; the
 * switches exist so that this can be tested, and for measurements).  Not synchronised with calls in flight on other threads.
 *   FASTAV_OPT_FUSED_SCORE_SELECT (default 1): a FINE prune with n_last = 1 finishes Eq. 4 inside the selection
 *       kernel, straight from the attention kernel's last-row side output; 0 runs the separate finishing kernel.
 *   FASTAV_OPT_FUSED_ROPE (default 1): bf16 prefill rotates Q and K inside the epilogue of the Q/K/V projection
 *       (one rounding to bf16 instead of two); 0 runs the separate RoPE kernel after the projection.  The two
 *       forms agree to bf16 rounding, not bit for bit.
 *   FASTAV_OPT_FUSED_SPLITK_NORM (default 1): in the prefill, a residual projection that splits K over workgroups
 *       (few output tiles: the pruned layers) leaves the ordered sum of its partial tiles to the RMSNorm that reads
 *       the residual next; 0 runs the separate reduction kernel.  Same additions in the same order.
 *   FASTAV_OPT_FUSED_GATHER_OPROJ (default 1): after a FINE prune the O projection (bf16) reads the surviving rows
 *       of the attention output through the keep list in its operand copies; 0 compacts the attention output with
 *       the other tensors first.  Same values into the same arithmetic. */
typedef enum { FASTAV_OPT_FUSED_SCORE_SELECT = 0, FASTAV_OPT_FUSED_ROPE = 1, FASTAV_OPT_FUSED_SPLITK_NORM = 2,
               FASTAV_OPT_FUSED_GATHER_OPROJ = 3, FASTAV_OPT_COUNT = 4 } fastav_option_t;
fastav_status_t fastav_set_option(int32_t option, int32_t value);

/* ---- the decoder handle --------------------------------------------------------------------------- */

fastav_status_t fastav_create(const fastav_model_t* model, fastav_handle_t* out);
void fastav_destroy(fastav_handle_t h);
fastav_status_t fastav_set_weights(fastav_handle_t h, int32_t layer, const fastav_layer_weights_t* w);
/* Bytes of device workspace fastav_prefill needs for at most max_total_tokens packed tokens in at most
 * max_batch samples.  The workspace must be 256-byte aligned; its contents are scratch. */
fastav_status_t fastav_workspace_bytes(fastav_handle_t h, int64_t max_total_tokens, int32_t max_batch, size_t* out);

/* ---- the hot path ---------------------------------------------------------------------------------- */

/* Pruned prefill (Fig. 3): runs every layer on the packed batch and applies the prune schedule.
 * n_last >= 1 is the number of last query rows Eq. 4 averages (the paper uses 1).  With no prunes, or
 * keep_ratio 1.0 everywhere, the result is the plain prefill.  All weights must have been set. */
fastav_status_t fastav_prefill(fastav_handle_t h, const fastav_batch_t* in, const fastav_prune_t* prunes,
                               int32_t n_prunes, int32_t n_last, void* workspace, size_t workspace_bytes,
                               const fastav_prefill_out_t* out, void* stream);

/* Eq. 4 on its own: scores_out[j] = mean over the Hq heads (and the last n_last rows r of the sample,
 * row r seeing keys 0..r) of softmax_j(q_r,h . k_j,g(h) / sqrt(head_dim)), g(h) = h / (Hq/Hkv).
 * q [T, Hq, head_dim] and k [T, Hkv, head_dim] are post-RoPE features with the given row strides (in
 * elements); only the last n_last rows of each sample are read from q.  K is streamed once.
 * workspace: dev, at least fastav_score_workspace_bytes(...) bytes. */
size_t fastav_score_workspace_bytes(int32_t n_q_heads, int64_t total_tokens, int32_t batch, int32_t n_last);
fastav_status_t fastav_score(const fastav_model_t* model, const void* q, int64_t q_row_stride, const void* k,
                             int64_t k_row_stride, const int32_t* cu_seqlens_dev, int32_t batch,
                             int64_t total_tokens, int32_t max_seqlen, int32_t n_last, float* scores_out,
                             void* workspace, size_t workspace_bytes, void* stream);

/* fastav_score for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same result as
 * fastav_score, but the scratch (last-row logits and per-chunk partial sums) is a fixed FASTAV_SCORE_STATIC_BYTES
 * array that is part of the library image: every GPU the library runs on holds its own copy until the process
 * ends.  The call allocates and frees nothing.  Problems that need more scratch than that
 * (fastav_score_workspace_bytes(...) > FASTAV_SCORE_STATIC_BYTES; at 32 query heads and n_last = 1 that is beyond
 * roughly 65 000 packed tokens) are rejected with FASTAV_EWORKSPACE before any launch.  All calls on one GPU share
 * that GPU's array: calls that overlap there (different streams or threads) race; calls on one stream do not. */
#define FASTAV_SCORE_STATIC_BYTES (8u << 20)
fastav_status_t fastav_score_static(const fastav_model_t* model, const void* q, int64_t q_row_stride, const void* k,
                                    int64_t k_row_stride, const int32_t* cu_seqlens_dev, int32_t batch,
                                    int64_t total_tokens, int32_t max_seqlen, int32_t n_last, float* scores_out,
                                    void* stream);

/* Top-k selection per sample plus stable compaction (Section 2.2, "Fine pruning" / Eq. 4, and "Global
 * pruning" for the positional form).  For sample b, keeps every row whose protected_mask byte is non-zero and the
 * keep_counts[b] - (#protected) highest-scoring other rows (tie rule above); writes the kept packed row
 * indices, ascending, to keep_idx_out[cu_seqlens_out[b] ..], writes cu_seqlens_out (prefix sums of
 * keep_counts), and copies rows: dst[i][r] = src[i][keep_idx_out[r]] for each of the n_tensors tensors of
 * row_bytes[i] bytes per row (src/dst/row_bytes are host arrays of dev pointers / sizes; src and dst must
 * not overlap).  keep_counts (host, [batch]) must satisfy #protected_b <= keep_counts[b] <= n_b; the lower
 * bound cannot be checked on the host and a violation keeps all protected rows first, in index order.
 * scores == NULL selects by position instead (earliest rows win: the GLOBAL rule).
 * workspace: dev, at least fastav_select_workspace_bytes(batch) bytes. */
size_t fastav_select_workspace_bytes(int32_t batch);
fastav_status_t fastav_select_gather(const float* scores, const uint8_t* protected_mask,
                                     const int32_t* cu_seqlens /* host [batch+1] */,
                                     const int32_t* keep_counts /* host [batch] */, int32_t batch,
                                     int32_t n_tensors, const void* const* src, void* const* dst,
                                     const int64_t* row_bytes, int32_t* keep_idx_out, int32_t* cu_seqlens_out,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* ---- building blocks of one decoder layer (also used by fastav_prefill) --------------------------- */

/* y[r,:] = x[r,:] * rsqrt(mean(x[r,:]^2) + eps) * g.  x fp32 [rows, d] (the residual stream), g and y in
 * dtype. */
fastav_status_t fastav_rmsnorm(const float* x, const void* g, void* y, int64_t rows, int32_t d, float eps,
                               int32_t dtype, void* stream);

/* Rotate-half RoPE in place on the first n_heads heads of each row of x [rows, row_stride] (dtype):
 * pair (i, i + head_dim/2) of every head is rotated by pos[r] * base^(-2i/head_dim). */
fastav_status_t fastav_rope(void* x, int64_t row_stride, const int32_t* pos, int64_t rows, int32_t n_heads,
                            int32_t head_dim, float base, int32_t dtype, void* stream);

/* Linear layers, W stored [N, K] (out, in), A [M, K] in dtype:
 *   FASTAV_EPI_STORE   : C[M,N] (dtype)  = A W^T
 *   FASTAV_EPI_RESADD  : R[M,N] (fp32)  += A W^T                       (residual update, C = R)
 *   FASTAV_EPI_SWIGLU  : C[M,N] (dtype)  = silu(A W^T) * (A W2^T)      (W2 [N, K] is the "up" matrix) */
typedef enum { FASTAV_EPI_STORE = 0, FASTAV_EPI_RESADD = 1, FASTAV_EPI_SWIGLU = 2 } fastav_epilogue_t;
/* workspace (optional, dev, 256-byte aligned, fastav_linear_workspace_bytes() bytes): lets a residual update
 * with few output tiles split K across more compute units; the partial tiles are summed in a fixed order, so
 * results do not depend on scheduling.  NULL is allowed (no splitting). */
size_t fastav_linear_workspace_bytes(void);
fastav_status_t fastav_linear(const void* a, const void* w, const void* w2, void* c, int64_t m, int32_t n,
                              int32_t k, int32_t epilogue, int32_t dtype, void* workspace, size_t workspace_bytes,
                              void* stream);

/* Causal grouped-query attention over a packed batch: o = softmax(q k^T / sqrt(head_dim) + causal) v.
 * q,k,v,o are dev pointers in dtype with row strides in elements (q and o hold Hq heads, k and v Hkv).
 * last_logits (optional, dev fp32 [Hq, T]) and last_ml (optional, dev fp32 [batch, Hq, 2]) receive, for
 * the last query row of each sample, the scaled logits against every key of the sample and that row's
 * (max, sum of exp) — the side output from which Eq. 4 is finalised without a second pass over K. */
fastav_status_t fastav_attention(const fastav_model_t* model, const void* q, int64_t q_row_stride,
                                 const void* k, const void* v, int64_t kv_row_stride, void* o,
                                 int64_t o_row_stride, const int32_t* cu_seqlens_dev, int32_t batch,
                                 int64_t total_tokens, int32_t max_seqlen, float* last_logits, float* last_ml,
                                 void* stream);

/* ---- one decode step on the pruned caches ------------------------------------------------------------
 * Section 3.1 measures latency as the time to generate a single token, and the memory FastAV saves is the
 * per-layer K/V cache of the surviving tokens.  This is that forward for ONE new token per sample (bf16
 * models; at most FASTAV_MAX_DECODE_BATCH samples): every layer runs RMSNorm, the Q/K/V projections, RoPE at
 * pos_new, single-query grouped-query attention over
 *     [ that layer's prefill cache | tokens generated before this step | the new token itself ],
 * the output projection, and the SwiGLU MLP, with fp32 residuals.  After a pruned prefill the layers hold
 * different numbers of keys per sample; keys carry their original rotary positions, so a cache is a set.
 *
 * All pointers inside are DEVICE pointers unless stated; the pointer ARRAYS (k_prefix ...) live on the host.
 * The library reads the caches, never frees or reallocates anything; if k_gen / v_gen are given it writes
 * the new token's key / value into slot gen_len of every layer's generated-token cache (the caller then
 * passes gen_len + 1 on the next step). */
typedef struct {
  int32_t batch;
  const void* x_new;                /* [batch, hidden], model dtype: the new token's input embedding */
  const int32_t* pos_new;           /* [batch] rotary position of the new token (original length + generated) */
  const void* const* k_prefix;      /* host array [n_layers]: [T_l, n_kv_heads*head_dim] packed per sample */
  const void* const* v_prefix;      /* host array [n_layers] */
  const int32_t* const* cu_prefix;  /* host array [n_layers] of device int32 [batch + 1] prefix sums of the
                                       per-sample rows of that layer's cache */
  const int32_t* max_prefix;        /* HOST [n_layers]: the longest sample's rows in that layer's cache */
  void* const* k_gen;               /* host array [n_layers] of [batch, gen_cap, n_kv_heads*head_dim], or NULL */
  void* const* v_gen;               /* host array [n_layers], or NULL (both or neither) */
  int32_t gen_len;                  /* generated tokens already in k_gen / v_gen (the same for every sample) */
  int32_t gen_cap;
} fastav_decode_in_t;

/* Bytes of device workspace (256-byte aligned, scratch) one decode step needs for at most max_batch samples. */
fastav_status_t fastav_decode_workspace_bytes(fastav_handle_t h, int32_t max_batch, size_t* out);
/* x_out: device [batch, hidden] fp32, the hidden state leaving the last layer (before the final norm and
 * the vocabulary projection, like fastav_prefill).  Errors: FASTAV_EINVAL on bad arguments,
 * FASTAV_EUNSUPPORTED for fp32 models or dimensions that are not multiples of 128, FASTAV_EWORKSPACE. */
fastav_status_t fastav_decode_step(fastav_handle_t h, const fastav_decode_in_t* in, float* x_out, void* workspace,
                                   size_t workspace_bytes, void* stream);

/* ---- attention rollout (Section 2.2, Eq. 2-3): the analysis behind the global-pruning decision -------------
 * A^l = causal attention weights of layer l averaged over the query heads; A~^l = alpha A^l + (1 - alpha) I;
 * R^l = A~^l A~^(l-1) ... A~^1.  Entry [i][j] of R^l is the influence of input token j on token i after l layers.
 *
 * fastav_attention_map: q [n, >= Hq*dh], k [n, >= Hkv*dh] (device, bf16, post-RoPE, ONE sample, explicit row
 * strides in elements) -> a_out: device bf16 [n, n], row i = token i's head-mean attention over tokens 0..i
 * (zeros right of the diagonal).  n must be a multiple of 4.  workspace: device, 256-byte aligned,
 * fastav_attention_map_workspace_bytes(n, Hq) bytes of scratch. */
size_t fastav_attention_map_workspace_bytes(int32_t n, int32_t n_q_heads);
fastav_status_t fastav_attention_map(const fastav_model_t* model, const void* q, int64_t q_row_stride, const void* k,
                                     int64_t k_row_stride, int32_t n, void* a_out, void* workspace,
                                     size_t workspace_bytes, void* stream);
/* fastav_rollout: runs ONE sample x [n, hidden] (device, model dtype, bf16 models) through the first
 * upto_layers layers of the UNPRUNED decoder and accumulates Eq. 3 with the given alpha in [0, 1].
 * rt_out: device fp32 [n, n] receives the TRANSPOSE of R^upto_layers (rt_out[j][i] = R[i][j]: the library's
 * GEMM multiplies by row-major [out, in] matrices, so the product is carried transposed).  The map of every
 * layer is rounded to bf16 and the running product is fed to the GEMM as bf16 (fp32 master copy).
 * Errors: FASTAV_EINVAL (arguments), FASTAV_EUNSUPPORTED (fp32 model), FASTAV_EWORKSPACE. */
fastav_status_t fastav_rollout_workspace_bytes(fastav_handle_t h, int32_t n, size_t* out);
fastav_status_t fastav_rollout(fastav_handle_t h, const void* x, int32_t n, float alpha, int32_t upto_layers,
                               float* rt_out, void* workspace, size_t workspace_bytes, void* stream);
/* fastav_rollout_cutoff: the threshold step of the analysis (Section 2.2, "Global pruning": a rollout threshold
 * at the middle layer marks the less influential video/audio tokens, those beyond some position).
 * rt: device fp32 [n, n], the transposed rollout as fastav_rollout writes it (16-byte aligned, n a multiple of 4).
 * protected_mask: device uint8 [n], nonzero = never a candidate (text tokens, the last query positions).
 * influence_out: device fp32 [n] receives the influence of every input token = the mean over all n rows i of
 * R[i][j]; the influences sum to 1, so 1/n is the uniform share.  cutoff_out: device int32 [1] receives one past
 * the last candidate position j with influence_out[j] * n >= threshold (compared in fp32), 0 if there is none:
 * positional global pruning with that many leading positions keeps every candidate the threshold passes.
 * The statistic over a set of samples (the paper looks at 100) is the caller's mean or median of the cut-offs.
 * Errors: FASTAV_EINVAL (NULL pointer, n not a positive multiple of 4, negative or NaN threshold). */
fastav_status_t fastav_rollout_cutoff(const float* rt, int32_t n, const uint8_t* protected_mask, float threshold,
                                      float* influence_out, int32_t* cutoff_out, void* stream);

/* ---- measurement aid (benchmarks only) -------------------------------------------------------------- */

/* Kernel kinds whose launches can be timed with HIP events on the launch stream.  "work" is the
 * algorithmic work of a launch: flops for LINEAR_* (2 M N K; SwiGLU counts both matrices) and ATTENTION
 * (2 Hq dh n(n+1) per sample, the causal half only), bytes for the others (what the step must read and
 * write once). */
typedef enum {
  FASTAV_PROF_LINEAR_STORE = 0, FASTAV_PROF_LINEAR_RESADD = 1, FASTAV_PROF_LINEAR_SWIGLU = 2,
  FASTAV_PROF_ATTENTION = 3, FASTAV_PROF_SCORE = 4, FASTAV_PROF_SELECT = 5, FASTAV_PROF_GATHER = 6,
  FASTAV_PROF_RMSNORM = 7, FASTAV_PROF_ROPE = 8, FASTAV_PROF_OTHER = 9, FASTAV_PROF_KIND_COUNT = 10
} fastav_prof_kind_t;

/* Times every later launch whose kind bit (1u << kind) is set; 0 switches timing off (the default).
 * While on, launches create and record HIP events, so do not enable it under graph capture. */
fastav_status_t fastav_profile_enable(uint32_t kind_mask);
/* Waits for the recorded launches, folds them into the running totals and returns the totals of one
 * kind: summed event-to-event milliseconds, number of launches, summed work.  Outputs may be NULL. */
fastav_status_t fastav_profile_collect(int32_t kind, double* total_ms, int64_t* launches, double* total_work);
fastav_status_t fastav_profile_reset(void);

/* "Achievable peak" probes, reported by the benchmark next to the datasheet peaks.
 * fastav_probe_mfma: every CU runs `iters` rounds of 32 independent v_mfma_f32_16x16x32_bf16 per wave (2 waves per
 * SIMD, no memory traffic inside the loop); *flops_out (host, optional) receives the flops of the launch.
 * operands: dev, optional: 64 KB of bf16 (16-byte aligned) that fill the operand registers - values drawn like the
 * model's activations give the ceiling under realistic switching activity; NULL = small integer constants.
 * sink: dev, >= 2 MB, never written in practice.
 * fastav_probe_read: one streaming pass over src (dev, 16-byte aligned, `bytes` >= 16 KB; the tail beyond a multiple
 * of 16 KB per workgroup step may be skipped), 16 bytes per lane and load.  sink: dev, >= 256 KB.
 * Both only enqueue the kernel; the caller times it with events on the same stream. */
fastav_status_t fastav_probe_mfma(int32_t iters, const void* operands, float* sink, double* flops_out, void* stream);
fastav_status_t fastav_probe_read(const void* src, size_t bytes, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTAV_H */
