// Host-side launchers of the gfx950 kernels.  Every launcher only queues work on
// `stream`; `dtype` selects the storage type of T-typed buffers (0 fp32, 1 bf16).
// Launchers return hipSuccess or the launch error.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace san {

// ---------------------------------------------------------------- projections
// out[m][n] = sum_k A[m][k] * W[n][k] (+ bias[n]) (ReLU) on MFMA tiles.
// The N columns are cut into segments of seg_w columns; segment s goes to
// out[s] + (*t_dev) * tstride[s] + m * ldo[s] + (n - s*seg_w).
//   out_kind 0: store as T;  1: store fp32;  2: fp32 split-K partials
//   [ksplit][M][N] at out[0] (no bias, no ReLU; the consumer reduces them).
//   ksplit > 1 is only allowed with out_kind 2.
//   out_kind 3: nothing of the product is stored.  The N columns are cut into
//   cand_tiles tiles of gemm_cand_tile_n() columns; for every row m and tile x the
//   kernel writes the tile's maximum and sum of exp(value - maximum) to
//   cand_ms[m][x][2], and to the 2 * cand_k slots cand_v / cand_i [m][x][2 * cand_k]
//   a set of (value, column) entries, in no particular order, that contains the tile's
//   cand_k largest (higher value first, then lower column); unused slots hold
//   (-inf, INT_MAX).  The bias is added; no ReLU, no segments.
//   bump: if not null, *bump is incremented once by the kernel (step counter).
struct GemmParams {
  const void* A; int lda;
  const void* W;              // [N][K]
  const void* bias;           // T [N] or nullptr
  void* out[3]; int ldo[3]; long long tstride[3];
  int seg_w;
  const int* t_dev;           // nullptr: no step offset
  int* bump;
  int M, N, K;                // K % (128 / sizeof(T)) == 0
  int relu, out_kind, ksplit;
  int xcd_rows, cps;           // set by the launcher (tile-to-XCD mapping, k chunks per split), callers leave them alone
  int cand_k, cand_tiles;      // out_kind 3
  float* cand_ms; float* cand_v; int* cand_i;
};
constexpr int kGemmCandMaxK = 8;
hipError_t launch_gemm(int dtype, const GemmParams& p, hipStream_t stream);
// split factor that fills the chip for an M x N x K product (1 when the tiles
// alone already do)
int gemm_pick_ksplit(int M, int N, int K, int dtype);
int gemm_cand_tile_n(int M, int N, int K, int dtype);

// ------------------------------------------------------------------ attention
// One kernel for every attention in the model.  A wave owns one head of one
// key/value stream and NQ queries that share the stream.
//  self (cached decoding): stream = history of decoder row r, key j lives in
//     slot j*rows + anc[r*ld_anc + j], n = *t_dev + 1 keys, one query.  rpg > 1:
//     rows come in groups of rpg (the hypotheses of a sentence) that share most
//     cache rows; a group's workgroups are placed on one XCD.
//  grouped: stream = group g (a sentence's encoder memory, or the positions of
//     one hypothesis when nothing is cached), key j in slot g*slot_stride + j;
//     the group's rpg query rows are g*rpg .. g*rpg+rpg-1; n = len[g] or, when
//     causal, query i (its index inside the group modulo causal_mod) sees
//     keys 0..i.
//  apply = 0: S = softmax(q K^T * scale) (Eq. 1), out = S V (Eq. 2); S is also
//     written to S_buf when emit != 0.   apply = 1: S is read from S_buf (the
//     block head's weights, Eq. 4) and only out = S V runs.
struct AttnParams {
  const void* q; int ldq;           // T [rows][ldq]
  const void* K; long long ldk;     // T, slot stride in elements (unused when apply)
  const void* V; long long ldv;
  const void* kv_packed; int kv_blocks;   // grouped, optional: the memory once more in fragment order (launch_pack_memory)
  float* S_buf; int ldS;            // fp32 [rows][H][ldS]
  void* out; int ldo;               // T [rows][ldo]
  const int* anc; int ld_anc;       // self mode
  const int* t_dev;                 // self mode
  const int* len;                   // grouped, non-causal: keys per group (nullptr: n_fixed)
  int n_fixed;
  int self_mode, rows, groups, rpg, slot_stride, causal;
  int grid3;                        // set by the launcher: the block index is spread over a 3-D grid
  int slot_rows;                    // self mode: rows of one cache position (0: same as rows)
  const int* group_map;             // grouped: memory of group g is slot group_map[g] (nullptr: g)
  int H, dh;
  int apply, emit, zero_tail;
  int lmax;                         // capacity of one score row (>= any n)
  float scale;
};
hipError_t launch_attention(int dtype, const AttnParams& p, hipStream_t stream);
// Block-head attention over a sentence's memory on the bf16 matrix cores (one wave per sentence
// and head, every query of the sentence at once).  Needs bf16, dh == 64, grouped non-causal mode,
// !apply, rpg <= 32 and kv_packed; launch_attention takes this route whenever it fits.
bool attention_ctx_mfma_fits(int dtype, const AttnParams& p);
hipError_t launch_attention_ctx_mfma(const AttnParams& p, hipStream_t stream);
// The memory keys / values of `groups` sentences (row (g * n_pos + pos), 64-wide heads, bf16) in the order
// that kernel reads its fragments: kv_blocks chunks of 8 KB per (sentence, head), one per 32 positions
// (zeros past n_pos); out holds groups * H * kv_blocks chunks.
hipError_t launch_pack_memory(const void* k, long long ldk, const void* v, long long ldv, int groups, int n_pos, int H,
                              void* out, int kv_blocks, hipStream_t stream);
// the same attention with each stream split over `waves` (1, 2, 4 or 8) waves of a workgroup; one_query:
// grouped mode, one query per workgroup instead of four.  launch_attention picks between the two.
hipError_t launch_attention_split(int dtype, const AttnParams& p, int waves, bool one_query, hipStream_t stream);

// ------------------------------------------------------------------ row-wise
// Optional extra outputs of the kernel that produces a decoder layer's input x when that layer is
// an average-attention layer (cached decoding): the running sum of the layer inputs over the
// positions so far (fp32 state, reset at step 0), its mean, and x as the left half of the gate's
// input [x ; g], without a launch of their own.
struct AanFuse {
  float* sum;          // [rows][d], nullptr: off
  void* avg;           // T [rows][d]
  void* cat;           // T [rows][2 d]
  const int* t_dev;
};

// x[r] = emb[clamp(tok)] * scale + pe[pos]; row r = hyp*rpg + i reads token
// tok[hyp*tok_stride + i]; pos = *t_dev when t_dev != nullptr, else i.
// With last_tok / anc given (cached decoding, rpg == 1) the kernel also does the
// step's bookkeeping: last_tok[r] = tok[r], anc[r*ld_anc + t] = r.
hipError_t launch_embed(int dtype, const int* tok, int tok_stride, int rpg, const void* emb, const float* pe,
                        const int* t_dev, void* x, int rows, int d, int vocab, float scale, int* last_tok,
                        int* anc, int ld_anc, hipStream_t stream, const AanFuse* aan = nullptr);

// out[m] = LayerNorm(sum_s part[s][m] + bias + res[m]) * g + b  (row-wise over n);
// part is [nsplit][M][ldp] and may point at a column offset of a wider buffer
// stage2 (optional): a second update + LayerNorm applied to the first one's output
// in the same launch: out = LN2(LN1(...) + sum_s part2[s][m] + bias2)
struct LnStage2 {
  const float* part; int nsplit, ldp;
  const void *bias, *gamma, *beta;
};
hipError_t launch_ln_reduce(int dtype, const float* part, int nsplit, int ldp, const void* bias, const void* res, int ldr,
                            const void* gamma, const void* beta, void* out, int ldo, float* out_f32, int M, int n,
                            float eps, hipStream_t stream, const LnStage2* stage2 = nullptr,
                            const AanFuse* aan = nullptr);

// start of a decode step: last_tok[r] = tok[r]; anc[r][t] = r; hist[r][t] = tok[r]
hipError_t launch_step_begin(const int* tok, int* last_tok, int* anc, int* hist, int ld, const int* t_dev, int rows,
                             hipStream_t stream);
hipError_t launch_to_f32(int dtype, const void* src, int lds, float* dst, int rows, int cols, hipStream_t stream);
// dst[r][h][0..n) = src[r][h][0..n) with source row stride ldS
hipError_t launch_compact_S(const float* src, int ldS, float* dst, int rows_h, int n, hipStream_t stream);

// ------------------------------------------------------------------- AAN layer
// un-cached decoding: x is [hyps][np][d]; avg[h][i] = mean of x[h][0..i], cat[h*np + i][0..d) = x[h][i]
hipError_t launch_aan_prefix_mean(int dtype, const void* x, void* avg, void* cat, int hyps, int np, int d,
                                  hipStream_t stream);
// x = LN(x + sigmoid(zi) * x + sigmoid(zf) * g), z = gate pre-activations (fp32, bias not yet added)
hipError_t launch_aan_post(int dtype, const float* z, const void* bg, const void* cat, const void* gamma,
                           const void* beta, void* x, float* out_f32, int rows, int d, float eps,
                           hipStream_t stream);

// ---------------------------------------------------------------------- search
// hist (optional): also append the picks to tok/par[step][batch*k], step =
// *t_dev - 1 - *t0_dev (the decode step just finished, relative to the call's first)
// row_map (optional, needs k == beam): the batch was compacted; row r of the current batch is row
// row_map[r] of the caller's arrays, whose steps are ld entries apart; parents are translated too
struct TopkHistory {
  int* tok; int* par;
  const int* t_dev; const int* t0_dev;
  const int* row_map; int ld;
};
// tail (optional, needs k == beam <= 32): the per-sentence merge runs inside a wider kernel that then
// applies the beam step's consequences for that sentence, so that a multi-step loop needs no further
// launch before the next step's first projection:
//   - the rows of the ancestry table (anc, columns < *t_dev) or of the AAN running sums
//     (aan_sum [layers][layer_stride]) are permuted by the chosen parents, in place;
//   - emb != nullptr: the next step's input is embedded for the sentence's rows,
//     x[r] = emb[token] * scale + pe[*t_dev], last_tok[r] = token, anc[r][*t_dev] = r
//     (skipped when *t_dev == max_t: there is no next position).
// *t_dev must already count the step whose logits are being searched.
struct BeamTail {
  int* anc; int ld_anc; int max_t; const int* t_dev;
  float* aan_sum; size_t layer_stride; int layers;
  const void* emb; const float* pe; void* x; int d; float scale; int dtype;
};
// done (optional, eos_id >= 0): int[batch]; done[b] becomes 1 once every pick of sentence b is EOS,
// *done_count counts such sentences
hipError_t launch_topk(const float* logits, const float* cum, const int* last_tok, int eos_id, int batch, int beam,
                       int vocab, int k, float* cand_lp, int* cand_idx, int* out_tok, int* out_parent,
                       float* out_score, hipStream_t stream, const TopkHistory* hist = nullptr, int* done = nullptr,
                       int* done_count = nullptr, const BeamTail* tail = nullptr, int* last_tok_out = nullptr);
// The same search fed by the output layer's per-tile candidates (GemmParams out_kind 3 with
// cand_k == k) instead of the logits: ms [rows][ntiles][2], cv / ci [rows][ntiles][2 k].
// topk_cands_fit: whether ntiles * 2 k candidate slots per row are within what the kernel holds.
bool topk_cands_fit(int ntiles, int k);
hipError_t launch_topk_cands(const float* ms, const float* cv, const int* ci, int ntiles, const float* cum,
                             const int* last_tok, int eos_id, int batch, int beam, int vocab, int k, float* cand_lp,
                             int* cand_idx, int* out_tok, int* out_parent, float* out_score, hipStream_t stream,
                             const TopkHistory* hist = nullptr, int* done = nullptr, int* done_count = nullptr,
                             const BeamTail* tail = nullptr, int* last_tok_out = nullptr);
// per sentence, in place: tab[r][j] = tab[parent[r]][j] for j < *t_dev
hipError_t launch_reorder_table(int* tab, int ld, const int* parent, const int* t_dev, int batch, int beam,
                                int max_t, hipStream_t stream);
// per sentence, in place: st[l][r][c] = st[l][parent[r]][c]; layer l starts at st + l*layer_stride
hipError_t launch_reorder_rows(float* st, size_t layer_stride, const int* parent, int layers, int batch, int beam,
                               int d, hipStream_t stream);

// ------------------------------------------------------------- policy learning
constexpr int kMaxPolicyLayers = 32;
struct JsParams {
  const float* S[kMaxPolicyLayers];   // per layer: weights [rows][H][ld]
  int L, rows, H, ld;
  const int* len; int rows_per_len;   // keys per row = len[row / rows_per_len] (nullptr: n_fixed)
  int n_fixed;
  float* part;                        // [pairs][rows*H]
};
// adds, for every layer pair, the sum over (row, head) of the JS divergence to acc[L][L]
hipError_t launch_js_accumulate(const JsParams& p, double* acc, hipStream_t stream);
// host: block sizes of the greedy search with threshold theta on a [L][L] JS matrix
int policy_search(const double* js, int L, double theta, int32_t* pi, int32_t* n_blocks);

// Dropping sentences from a running batch.  dst[(g*rpg + i)*w + c] = src[(keep[g]*rpg + i)*w + c] for
// g < groups, i < rpg, c < w (4-byte words; dst and src must not overlap)
hipError_t launch_gather_groups(void* dst, const void* src, const int* keep, int rpg, int groups, int w,
                                hipStream_t stream);
// *count = number of non-zero flags[0..n)
hipError_t launch_count_flags(const int* flags, int n, int* count, hipStream_t stream);
// tok[s][r] = eos, par[s][r] = r for the rows r of every sentence b with 0 <= from[b] and the steps
// from[b] <= s < steps ([step][rows] arrays): a dropped sentence keeps extending with EOS in place
hipError_t launch_fill_finished(int* tok, int* par, const int* from, int batch, int beam, int steps, int eos,
                                hipStream_t stream);
// dst[map[r]] = src[r] for r < n (4-byte words)
hipError_t launch_scatter_words(void* dst, const void* src, const int* map, int n, hipStream_t stream);

// reads `bytes` (multiple of 16) of device memory once and discards them; sink: 4 writable device bytes
hipError_t launch_stream_read(const void* src, size_t bytes, unsigned* sink, hipStream_t stream);

}  // namespace san
