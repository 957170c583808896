/*
 * libsan -- shared-attention (SAN) Transformer decoding on one MI355X (gfx950).
 *
 * The library runs the cached auto-regressive Transformer decoder step in which
 * the decoder layers are grouped into blocks by a sharing policy {pi_1..pi_N}
 * (Sec. 3.3 of "Sharing Attention Weights for Fast Transformer"): inside a
 * block only the first layer computes the attention weights
 * S = Softmax(Q K^T / sqrt(d_k)) (Eq. 1, Eq. 3); the other layers of the block
 * reuse them (Eq. 4, self-attention, each layer with its own V) or reuse the
 * attended state A = S V itself (Eq. 5, encoder-decoder attention).
 *
 * General conventions
 *   - Plain C ABI.  Every pointer parameter says whether it is HOST or DEVICE
 *     memory.  DEVICE buffers are owned by the caller, must live on the device
 *     that was current at san_init and must stay valid until the work queued by
 *     the call has finished.
 *   - All device work is queued on the stream given to san_init and is
 *     asynchronous with respect to the host; no call synchronises the device
 *     except san_init and san_free.  Calls on one context must not overlap.
 *   - Every function returns a san_status (0 = ok) and never aborts; a text for
 *     the last failure of a context is available from san_last_error.
 *   - Rows: decoder row r = sentence * beam + beam_index, rows = batch * beam.
 *   - Linear maps are stored [out_features][in_features], y = x W^T + b.
 */
#ifndef SAN_H
#define SAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct san_ctx san_ctx; /* opaque, owned by the library */

#if defined(__GNUC__)
#define SAN_API __attribute__((visibility("default")))
#else
#define SAN_API
#endif

typedef enum {
  SAN_OK = 0,
  SAN_EINVAL = 1,    /* bad argument or unsupported configuration           */
  SAN_EPOLICY = 2,   /* policy does not partition the decoder layers        */
  SAN_ESTATE = 3,    /* call out of order (e.g. decode before encode)       */
  SAN_ECAPACITY = 4, /* exceeds max_batch / max_src_len / max_tgt_len       */
  SAN_EHIP = 5,      /* a HIP runtime call failed                           */
  SAN_ENOMEM = 6     /* device or host allocation failed                    */
} san_status;

enum { SAN_F32 = 0, SAN_BF16 = 1 };          /* storage type of weights, activations, caches;
                                                accumulation, softmax and LayerNorm statistics are fp32 */
enum { SAN_SELF_DOT = 0, SAN_SELF_AAN = 1 }; /* decoder self sub-layer: dot-product attention (Eq. 1-2)
                                                or the average attention network (Tab. 6 rows "+AAN") */
enum { SAN_SHARE_A = 0, SAN_SHARE_S = 1 };   /* enc-dec blocks: reuse A = S V (Eq. 5) or reuse S with a
                                                per-layer V (Tab. 4, row "shared V: no")              */

/* which tensor san_debug_get copies out */
enum { SAN_DBG_S_SELF = 0, SAN_DBG_A_SELF = 1, SAN_DBG_S_CTX = 2, SAN_DBG_A_CTX = 3, SAN_DBG_HIDDEN = 4,
       SAN_DBG_ENC_OUT = 5, SAN_DBG_MEM = 6 };

typedef struct {
  int32_t n_enc_layers, n_dec_layers;
  int32_t d_model, n_heads, d_ff, vocab; /* d_model % 64 == 0, d_ff % 64 == 0,
                                            d_model / n_heads in {16,32,64,128}        */
  int32_t max_batch;   /* sentences per san_encode call                               */
  int32_t beam;        /* hypotheses per sentence (1 = greedy), 1..32                 */
  int32_t max_src_len; /* source positions per sentence, <= 1024                     */
  int32_t max_tgt_len; /* decode steps per sentence (self cache capacity), <= 1024   */
  int32_t dtype;       /* SAN_F32 | SAN_BF16                                          */
  int32_t self_kind;   /* SAN_SELF_DOT | SAN_SELF_AAN                                 */
  int32_t encdec_share;/* SAN_SHARE_A | SAN_SHARE_S                                   */
  int32_t use_cache;   /* 1: key/value cache (Sec. 4.1 baseline); 0: recompute every
                          target position at every step (Tab. 6 row "-Cache"), with
                          either self_kind                                            */
  int32_t pad_id, bos_id, eos_id; /* word ids in [0, vocab); eos_id < 0 switches EOS handling
                                     off in san_topk                                          */
  int32_t debug;       /* sum of: 1 keep per-layer S / A / hidden copies for san_debug_get;
                          2 run only the general-purpose attention kernel (no matrix-core
                          kernel for the encoder memory): a cross-check, slower            */
  float ln_eps;        /* LayerNorm epsilon                                           */
} san_config;

/* Sharing policy (Sec. 3.3): block sizes bottom-up; each list must sum to
 * n_dec_layers and hold only sizes >= 1.  With SAN_SELF_AAN self_pi is ignored.
 * enc_pi (optional: n_enc = 0 or NULL means every encoder layer on its own) shares
 * the encoder self-attention weights the same way (Tab. 5, "encoder-side SAN") and
 * must sum to n_enc_layers. */
typedef struct {
  int32_t n_self;
  const int32_t* self_pi; /* HOST */
  int32_t n_encdec;
  const int32_t* encdec_pi; /* HOST */
  int32_t n_enc;
  const int32_t* enc_pi; /* HOST, may be NULL */
} san_policy;

/* Size in bytes of the weight blob san_init expects for this configuration
 * (0 if the configuration is invalid).  Blob = these tensors back to back, in
 * the storage type `dtype` (bf16 = upper 16 bits of the fp32 pattern):
 *   src_emb[V][d], tgt_emb[V][d],
 *   per encoder layer: attn {wq,bq,wk,bk,wv,bv,wo,bo}, ln1 {g,b},
 *                      ffn {w1[F][d],b1,w2[d][F],b2}, ln2 {g,b}
 *   per decoder layer: self {wq,bq,wk,bk,wv,bv,wo,bo}          (SAN_SELF_DOT)
 *                      or aan {w1,b1,w2,b2,wg[2d][2d],bg[2d]}  (SAN_SELF_AAN),
 *                      ln1 {g,b}, ctx {wq,bq,wk,bk,wv,bv,wo,bo}, ln2 {g,b},
 *                      ffn {w1,b1,w2,b2}, ln3 {g,b}
 *   w_out[V][d]
 * The blob is always the full standard-Transformer tensor set; the tensors a
 * policy makes unnecessary (Q/K projections of non-head self layers, Q/K/V of
 * non-head enc-dec layers; Sec. 3.2) are simply not uploaded. */
SAN_API size_t san_weight_bytes(const san_config* cfg);

/* Build a context: validate cfg + policy, upload the needed weights from the
 * HOST blob, allocate caches and workspaces on the current device.
 * hip_stream: a hipStream_t (may be NULL = default stream) on which every later
 * call queues its work.  *out receives the context (NULL on failure).
 * Errors: SAN_EINVAL (shape/dtype/blob size), SAN_EPOLICY, SAN_ENOMEM, SAN_EHIP. */
SAN_API int san_init(const san_config* cfg, const void* weights_host, size_t weight_bytes,
             const san_policy* policy, void* hip_stream, san_ctx** out);

/* Run the encoder stack on a padded source batch and precompute the
 * encoder-decoder keys/values of every decoder layer that needs them (block
 * heads; with SAN_SHARE_S also each follower's V).  Keys beyond src_len[b] are
 * never attended; src_len[b] = 0 gives a zero context vector.  Resets the
 * decoder state (step 0, empty cache).
 *   src_ids_dev DEVICE int32 [batch][max_src], src_len_dev DEVICE int32 [batch].
 * Errors: SAN_EINVAL (null, batch < 1, max_src < 1), SAN_ECAPACITY. */
SAN_API int san_encode(san_ctx* ctx, const int32_t* src_ids_dev, const int32_t* src_len_dev,
               int32_t batch, int32_t max_src);

/* Rewind the decoder to step 0 for the batch already encoded (keeps the
 * encoder-decoder keys/values; sentences dropped by san_compact are back).
 * Errors: SAN_ESTATE before san_encode. */
SAN_API int san_rewind(san_ctx* ctx);

/* One auto-regressive decoder step (Sec. 1: one target word at a time) for all
 * batch*beam rows: embeds tokens at the current position, runs every decoder
 * layer under the sharing policy, appends this position's keys/values to the
 * cache and writes the output-layer logits.
 *   tokens_dev DEVICE int32 [batch*beam] (ids outside [0,vocab) are clamped),
 *   logits_dev DEVICE fp32 [batch*beam][vocab].
 * Errors: SAN_ESTATE (no san_encode yet), SAN_ECAPACITY (step == max_tgt_len). */
SAN_API int san_decode_step(san_ctx* ctx, const int32_t* tokens_dev, float* logits_dev);

/* Beam step (Sec. 4.1: beam search over a batch).  Candidate (row r, word v)
 * scores cum_score[r] + log_softmax(logits[r])[v]; per sentence the k best of
 * the beam*vocab candidates are written in order of decreasing score, ties by
 * the lower flat index beam_index*vocab + v.  When eos_id >= 0, a row whose
 * last decoded input token was eos_id can only be extended by eos_id at cost 0.
 *   logits_dev DEVICE fp32 [batch*beam][vocab], 16-byte aligned, cum_score_dev
 *   DEVICE fp32 [batch*beam] (-inf marks a dead row), 1 <= k <= min(32, vocab);
 *   out_token_dev / out_parent_dev DEVICE int32 [batch][k] (parent = global row
 *   index), out_score_dev DEVICE fp32 [batch][k].
 * Errors: SAN_ESTATE, SAN_EINVAL. */
SAN_API int san_topk(san_ctx* ctx, const float* logits_dev, const float* cum_score_dev, int32_t k,
             int32_t* out_token_dev, int32_t* out_parent_dev, float* out_score_dev);

/* san_topk for callers that cannot allocate device memory or have the library hold
 * call-time buffers for them: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results (bit for bit) and
 * same errors as san_topk, but the per-row candidates (k (log-probability, word) pairs
 * per row, produced by the first kernel and merged per sentence by the second) live
 * in a fixed 256 KiB array in the library's device image instead of a buffer of the
 * context.  The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine) and synchronises nothing.
 *   Limit: batch*beam*k <= 32768 candidates (e.g. 1024 rows x 32); beyond that
 *   SAN_ECAPACITY and nothing is queued.
 *   Each GPU holds one copy of the array from the first san_init on it until the
 *   process ends, shared by every context on that GPU: calls of san_topk_noalloc that
 *   overlap on one GPU (different streams or threads) race on it.  The array keeps the
 *   previous call's contents; every entry a call reads it has written itself first.
 * Errors: as san_topk, plus SAN_ECAPACITY (above), SAN_ESTATE while san_profile is on. */
SAN_API int san_topk_noalloc(san_ctx* ctx, const float* logits_dev, const float* cum_score_dev, int32_t k,
                             int32_t* out_token_dev, int32_t* out_parent_dev, float* out_score_dev);

/* After a beam step: row r continues the hypothesis that was row parent[r].
 * Every per-row decoder state (self-attention key/value history, AAN running
 * sums, un-cached token history) follows; encoder-decoder keys/values are per
 * sentence and do not move.  parent[r] must lie in r's own sentence
 * (rows sentence*beam .. sentence*beam+beam-1); other values leave row r as is.
 *   parent_idx_dev DEVICE int32 [batch*beam].
 * Errors: SAN_ESTATE, SAN_EINVAL. */
SAN_API int san_beam_reorder(san_ctx* ctx, const int32_t* parent_idx_dev);

/* Copy a tensor of the most recent decode step to dst_dev (DEVICE, cap bytes).
 * Needs cfg.debug = 1 and use_cache = 1.
 *   SAN_DBG_S_SELF: fp32 [rows][heads][n], n = steps done (weights the layer used)
 *   SAN_DBG_S_CTX : fp32 [rows][heads][max_src] (entries >= src_len are 0)
 *   SAN_DBG_A_SELF / A_CTX / HIDDEN: fp32 [rows][d_model] (with SAN_SELF_AAN, A_SELF is
 *     the output of the whole average-attention sub-layer)
 * and of the last san_encode (available before the first decode step):
 *   SAN_DBG_ENC_OUT: fp32 [batch][max_src][d_model], the encoder output (`layer` ignored
 *     but must be valid)
 *   SAN_DBG_MEM    : fp32 [batch][max_src][2 d_model] = [K | V], the encoder-decoder
 *     keys/values of a block head (Sec. 3.2), or [batch][max_src][d_model] = V of a
 *     follower with SAN_SHARE_S; SAN_EINVAL for a layer that keeps none (Eq. 5 followers)
 * Errors: SAN_ESTATE, SAN_EINVAL (layer, what, cap too small). */
SAN_API int san_debug_get(san_ctx* ctx, int32_t what, int32_t layer, void* dst_dev, size_t cap);

/* n consecutive beam-search steps without returning to the host (Sec. 1: the
 * decoder produces one word at a time until the end): each step is
 * san_decode_step + san_topk with k = beam + san_beam_reorder, the chosen tokens
 * and scores feeding the next step.  With EOS handling on (eos_id >= 0),
 * finished hypotheses keep extending with EOS at no cost, and the call returns
 * early once every sentence of the batch is finished: the count of finished
 * sentences is read back every 8 steps (one stream synchronisation each), so up
 * to 7 further all-EOS steps may have run.  san_step tells how many steps were
 * done; rows of the out_* arrays past that are not written.  With eos_id < 0
 * the call always runs n steps and never synchronises.
 *   tokens_dev      DEVICE int32 [rows]     input tokens of the first step
 *   cum_io_dev      DEVICE fp32  [rows]     cumulative scores, in: before, out: after
 *   out_tokens_dev  DEVICE int32 [n][rows]  token chosen for every row at every step
 *   out_parents_dev DEVICE int32 [n][rows]  parent row of every row at every step
 *   logits_work_dev DEVICE fp32  [rows][vocab] scratch, 16-byte aligned; with use_cache = 1
 *                                           it is only written under SAN_LOOP_LOGITS
 * flags (SAN_LOOP_*, or-ed):
 *   SAN_LOOP_GRAPH: pairs of steps are replayed from a captured HIP graph (needs a
 *     stream other than the NULL stream and use_cache = 1; the graph is
 *     re-captured when the output/scratch pointers or the batch change).
 *   SAN_LOOP_COMPACT (needs use_cache = 1; no effect with eos_id < 0): at those
 *     8-step checks, once at least a quarter of the batch is finished and 16 or
 *     more steps remain, the finished sentences leave the batch (san_compact) and
 *     the remaining steps run on the smaller batch.  The caller's arrays keep the
 *     numbering of the batch at entry: in out_* a sentence that left keeps
 *     extending with EOS in place (token eos_id, parent = the row itself, as it
 *     would have), cum_io_dev holds its final scores.  Tokens are the same as
 *     without the flag except where two candidates' scores are within rounding
 *     (a smaller batch may run other GEMM tiles).  On return the context's batch
 *     is the sentences still unfinished (san_active); san_rewind restores it.
 *   SAN_LOOP_LOGITS: every step stores its logits in logits_work_dev (on return it
 *     holds the last step's) and the search reads them back, as the separate calls do.
 *     Without it (use_cache = 1, beam <= 8, at most 5120 / (2 beam) column tiles of the
 *     output layer) the output layer hands the search, per row and column tile, the
 *     tile's maximum, sum of exponentials and largest entries instead: the same tokens
 *     and parents, scores equal up to the rounding of the log-sum-exp, and neither the
 *     write nor the read of rows x vocab logits.
 * Allocates its ping-pong buffers (and that candidate workspace) on first use.
 * Errors: SAN_ESTATE, SAN_ECAPACITY (step + n > max_tgt_len), SAN_EINVAL. */
enum { SAN_LOOP_GRAPH = 1, SAN_LOOP_COMPACT = 2, SAN_LOOP_LOGITS = 4 };
SAN_API int san_decode_n(san_ctx* ctx, int32_t n, const int32_t* tokens_dev, float* cum_io_dev,
                         int32_t* out_tokens_dev, int32_t* out_parents_dev, float* logits_work_dev,
                         int32_t flags);

/* Number of sentences of the current batch that are finished: every hypothesis
 * kept by the last beam step (san_topk with k == beam, or a step of
 * san_decode_n) ends in eos_id.  Always 0 with eos_id < 0.  Synchronises the
 * context's stream.  count_out HOST.  Errors: SAN_EINVAL, SAN_ESTATE. */
SAN_API int san_finished(san_ctx* ctx, int32_t* count_out);

/* Per-sentence finished flags of the current batch (1 = finished in the sense of
 * san_finished).  flags_out HOST int32 [current batch].  Synchronises the stream.
 * Errors: SAN_EINVAL, SAN_ESTATE. */
SAN_API int san_done_flags(san_ctx* ctx, int32_t* flags_out);

/* Drop sentences from the running batch (decoding stops per sentence at its end
 * symbol, Sec. 1; a finished sentence otherwise keeps costing a full share of
 * every step).  keep HOST int32 [n_keep]: strictly increasing indices into the
 * CURRENT batch of the sentences that stay.  Afterwards the batch has n_keep
 * sentences; row i*beam + h of every later call is what row keep[i]*beam + h was,
 * and the caller permutes its own per-row arrays (tokens, cumulative scores) the
 * same way.  The state of the dropped sentences is discarded; the key/value
 * caches are not moved (they keep the row stride of the encoded batch).
 * san_rewind and san_encode restore / replace the full batch.  Synchronises the
 * stream; allocates a staging buffer on first use.  n_keep == batch is a no-op.
 * Errors: SAN_EINVAL (null, n_keep outside [1, batch], indices not increasing or
 * out of range), SAN_ESTATE (before san_encode, use_cache = 0, profiling on). */
SAN_API int san_compact(san_ctx* ctx, const int32_t* keep, int32_t n_keep);

/* The sentences of the current batch as indices into the batch given to
 * san_encode.  sentences_out HOST int32 [current batch] (may be null), n_out HOST.
 * Errors: SAN_EINVAL, SAN_ESTATE. */
SAN_API int san_active(san_ctx* ctx, int32_t* sentences_out, int32_t* n_out);

/* ---- Learning a sharing policy (Sec. 3.3) ----
 * san_policy_accumulate: after a decode step of a context with cfg.debug = 1 (every
 * layer's weights are kept), adds the Jensen-Shannon divergence (natural log)
 * between the weights of every pair of decoder layers, for every row and head of
 * that step, to running sums -- separately for self-attention (keys = the cached
 * positions) and encoder-decoder attention (keys = the source positions).  Layers
 * of one sharing block use the same weights and diverge by 0.
 * san_policy_read: the [L][L] matrix (HOST, doubles) of mean divergences "per
 * head, then averaged" (Sec. 3.1) and the number of (row, head) samples; which =
 * 0 self-attention, 1 enc-dec.  Synchronises the stream.
 * san_policy_search: host only.  Similarity mu(i,j) = ln 2 - JS(i,j); block
 * similarity sim(m,n) = mean of mu over the ordered pairs i != j of layers m..n
 * (Eq. 6); from layer 1 upwards take the biggest block with sim >= theta (a single
 * layer always qualifies).  Writes the block sizes bottom-up to pi_out (HOST,
 * room for n_layers) and their number to n_blocks_out.
 * Errors: SAN_ESTATE (no debug copies / no step yet), SAN_EINVAL. */
SAN_API int san_policy_accumulate(san_ctx* ctx);
SAN_API int san_policy_read(san_ctx* ctx, int32_t which, double* js_out, int64_t* count_out, int32_t reset);
SAN_API int san_policy_search(const double* js, int32_t n_layers, double theta, int32_t* pi_out,
                              int32_t* n_blocks_out);

/* Measurement aid: queue one plain streaming read of `bytes` bytes (rounded
 * down to a multiple of 16) of DEVICE memory at src_dev on the context's stream
 * and discard the data.  Timed by the caller, it gives the read bandwidth this
 * GPU reaches on a working set of that size -- the practical ceiling the
 * HBM-bound attention kernels are compared with.  Errors: SAN_EINVAL (null). */
SAN_API int san_stream_read(san_ctx* ctx, const void* src_dev, size_t bytes);

/* Number of decode steps done since the last san_encode / san_rewind (-1 if
 * nothing is encoded). */
SAN_API int32_t san_step(const san_ctx* ctx);

/* Device bytes held by the context (weights uploaded / caches+workspaces):
 * shows the parameter and cache saving of a policy (Sec. 3.2). */
SAN_API size_t san_device_bytes(const san_ctx* ctx, int32_t which /* 0 = weights, 1 = state */);

/* Kernel classes for san_profile_read. */
enum {
  SAN_K_MISC = 0,            /* embedding, bookkeeping, encoder                          */
  SAN_K_PROJ = 1,            /* q/k/v projections (+ cache append), enc-dec q projection  */
  SAN_K_ATTN_SELF = 2,       /* self-attention of a block head: S and A (Eq. 1-3)         */
  SAN_K_ATTN_APPLY = 3,      /* self-attention of a follower: A = S^m V (Eq. 4)           */
  SAN_K_OUT = 4,             /* attention output projections                              */
  SAN_K_LN = 5,              /* split-K reduce + bias + residual + LayerNorm              */
  SAN_K_ATTN_CTX = 6,        /* enc-dec attention of a block head (Eq. 5)                 */
  SAN_K_ATTN_CTX_APPLY = 7,  /* enc-dec follower with its own V (SAN_SHARE_S)             */
  SAN_K_FFN = 8,             /* feed-forward GEMMs                                        */
  SAN_K_LOGITS = 9,          /* output layer                                              */
  SAN_K_TOPK = 10,           /* san_topk                                                  */
  SAN_K_REORDER = 11,        /* san_beam_reorder                                          */
  SAN_K_AAN = 12,            /* average-attention self layer (all of its kernels)         */
  SAN_K_COUNT = 13
};

/* Per-kernel-class timing for benchmarks.  While enabled, every kernel the
 * context queues is bracketed by a pair of HIP events on the context's stream and
 * each API call ends with a stream synchronisation (so: not for production
 * loops).  san_profile_read adds up, per class, the elapsed milliseconds and
 * the number of launches since the last reset.  The markers themselves cost
 * about 2 us per bracketed launch, included in the figures.
 *   ms_out HOST double[SAN_K_COUNT], launches_out HOST int64[SAN_K_COUNT]
 *   (either may be NULL). */
SAN_API int san_profile(san_ctx* ctx, int32_t enable);
SAN_API int san_profile_read(san_ctx* ctx, double* ms_out, int64_t* launches_out, int32_t reset);

/* Number of kernels the last san_decode_step queued. */
SAN_API int32_t san_last_launch_count(const san_ctx* ctx);

/* Message of the last failed call on this context ("" if none).  With ctx ==
 * NULL: message of the last failed san_init on this thread. */
SAN_API const char* san_last_error(const san_ctx* ctx);

/* Waits for the stream, frees everything san_init allocated. NULL is allowed. */
SAN_API void san_free(san_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* SAN_H */
