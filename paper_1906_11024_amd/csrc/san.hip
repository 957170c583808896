// libsan: host side of the C ABI declared in include/san.h.  It validates the
// configuration and the sharing policy, uploads only the tensors the policy needs,
// owns the key/value caches and workspaces, and queues the kernels of each call on
// the caller's stream.  No arithmetic of the method happens on the host.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/san.h"
#include "kernels.h"

using namespace san;

// Candidate scratch of san_topk_noalloc: the beam step's per-row partial results
// ((log-probability, word) pairs, k per row) live in this fixed array instead of a
// buffer owned by a context, so that the call can be made where nothing may be
// allocated.  Every GPU the library runs on holds its own copy until the process ends.
// The name below is only the host-side handle of the symbol: host code uses the
// per-device address that hipGetSymbolAddress returns (scratch_address), never the name.
// No `used` attribute here: the compiler turns a file-local device variable into a symbol
// the runtime can find by name because host code refers to it; marked `used` it was kept
// as it stood, a local symbol of the device image, and the look-up aborted the process.
constexpr size_t kScratchCands = 32768;   // rows * k of one call, e.g. 1024 rows x 32
static __device__ __align__(256) unsigned char scratch[kScratchCands * 8];

// Device address of `scratch` on the current device, resolved once per device.
namespace san {
hipError_t scratch_address(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr_of[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    ptr_of[dev] = ptr;
  }
  *out = ptr_of[dev];
  return hipSuccess;
}
}  // namespace san

namespace {

thread_local std::string g_init_error;

struct EncLayer {
  // wqkv: block head [3d][d] (q;k;v); follower of an encoder-side sharing block: [d][d] (v only)
  void *wqkv, *bqkv, *wo, *bo, *ln1g, *ln1b, *w1, *b1, *w2, *b2, *ln2g, *ln2b;
  int head = 0;              // first layer of this layer's block
  float* S = nullptr;        // block head with followers: weights [batch*max_src][H][max_src]
};

struct DecLayer {
  // self sub-layer
  int self_head = 0;          // first layer of this layer's self-attention block
  void *w_self = nullptr, *b_self = nullptr;  // head: [3d][d] (q;k;v), follower: [d][d] (v)
  void *wo = nullptr, *bo = nullptr, *ln1g = nullptr, *ln1b = nullptr;
  void *aw1 = nullptr, *ab1 = nullptr, *aw2 = nullptr, *ab2 = nullptr, *awg = nullptr, *abg = nullptr;
  void *Kc = nullptr, *Vc = nullptr;          // [max_tgt][rows][d]
  float* S_self = nullptr;                    // block head only: [rows*][H][max_tgt]
  float* aan_sum = nullptr;
  // encoder-decoder sub-layer
  int ctx_head = 0;
  void *wq_c = nullptr, *bq_c = nullptr;      // head only
  void *wkv_c = nullptr, *bkv_c = nullptr;    // head: [2d][d] (k;v); follower in mode S: [d][d] (v)
  void *wo_c = nullptr, *bo_c = nullptr, *ln2g = nullptr, *ln2b = nullptr;
  void* mem = nullptr;                        // head: [batch*max_src][2d]; follower (mode S): [..][d]
  void* mem_packed = nullptr;                 // head, bf16 with 64-wide heads: K and V again, in MFMA fragment order
  float* S_ctx = nullptr;                     // head only
  void* A_ctx = nullptr;                      // head only: T [rows*][d]
  // Eq. 5 blocks, cached decoding: the followers' output projections of the shared A are
  // computed together with the head's (one GEMM over the stacked W_O of the block)
  void* wo_blk = nullptr;                     // head only: [pi*d][d]
  float* y_blk = nullptr;                     // head only: partials [ks][rows][pi*d]
  size_t y_elems = 0;
  int y_ks = 1, blk_size = 1;
  // feed-forward sub-layer
  void *w1 = nullptr, *b1 = nullptr, *w2 = nullptr, *b2 = nullptr, *ln3g = nullptr, *ln3b = nullptr;
  float *dbg_A_self = nullptr, *dbg_A_ctx = nullptr, *dbg_hidden = nullptr;
};

}  // namespace

struct san_ctx {
  san_config cfg;
  hipStream_t stream = nullptr;
  int dt = 0, esz = 4;
  int d = 0, H = 0, dh = 0, F = 0, V = 0, rows_max = 0, rows_src_max = 0;
  int src_pad = 0;             // max_src_len rounded up to 32 (DecLayer::mem_packed holds src_pad / 32 blocks per head)
  std::vector<EncLayer> enc;
  std::vector<DecLayer> dec;
  void *src_emb = nullptr, *tgt_emb = nullptr, *w_out = nullptr;
  float* pe = nullptr;
  // workspaces
  void *x = nullptr, *qkv = nullptr, *ab = nullptr, *hb = nullptr, *cat = nullptr;
  float* part = nullptr;
  size_t part_elems = 0;
  float* aan_all = nullptr;   // AAN running sums [layer][rows_max][d]
  float* dbg_enc = nullptr;   // debug copy of the encoder output [batch*max_src][d]
  // policy learning: running JS sums [2][L][L] (self, enc-dec), per-pair scratch, sample counts
  double* js_acc = nullptr;
  float* js_part = nullptr;
  long long js_count[2] = {0, 0};
  // multi-step decoding (san_decode_n): ping-pong token / score buffers, parents, first-step counter,
  // and the captured two-step graph with the pointers it was captured for
  int* pp_tok[2] = {nullptr, nullptr};
  float* pp_cum[2] = {nullptr, nullptr};
  int* pp_par = nullptr;
  int* t0_dev = nullptr;
  hipGraphExec_t graph2 = nullptr;
  const void* graph_key[3] = {nullptr, nullptr, nullptr};
  int graph_rows = 0, graph_entry_rows = 0;
  int graph_fused = 0;         // loop mode of the captured steps (see loop_step)
  int* row_map = nullptr;      // san_decode_n after a compaction: current row -> row of the caller's arrays
  float* cum_final = nullptr;  // scores in the caller's numbering
  int* drop_dev = nullptr;     // [max_batch] step at which each of the caller's sentences left the batch
  int *t_dev = nullptr, *anc = nullptr, *hist = nullptr, *last_tok = nullptr, *src_len = nullptr;
  int* done_dev = nullptr;     // [max_batch] finished flags, then the count of finished sentences
  int* done_host = nullptr;    // pinned, 2 * max_batch + 16 ints (count or flags read back; keep list going up)
  // dropping finished sentences (san_compact): the caches keep the row stride of the encoded batch
  int batch_enc = 0;           // sentences given to san_encode
  int* src_len0 = nullptr;     // their lengths (src_len holds those of the current batch)
  int* group_map = nullptr;    // [max_batch] encode-time index of each current sentence
  int* iota_dev = nullptr;     // 0, 1, 2, ... [max(rows_max, max_batch)]
  int* keep_dev = nullptr;     // [max_batch]
  void* cmp_tmp = nullptr;     // gather staging
  size_t cmp_tmp_bytes = 0;
  std::vector<int> active;     // host copy of group_map
  float* cand_lp = nullptr;
  int* cand_idx = nullptr;
  // san_decode_n: the output layer hands the beam step per-tile candidates instead of logits
  float* part_ms = nullptr;    // [rows][tiles][2]
  float* part_cv = nullptr;    // [rows][tiles][2 beam]
  int* part_ci = nullptr;
  int cand_tiles = 0;          // > 0 while a step of the loop runs in that mode: tiles per row
  // state
  int batch = 0, max_src = 0, t = -1;
  size_t weight_bytes = 0, state_bytes = 0;
  int launches = 0;
  // per-kernel-class timing (off unless san_profile switched it on)
  bool prof_on = false;
  int kind = SAN_K_MISC;
  std::vector<hipEvent_t> events;
  size_t events_used = 0;
  struct Pending { int kind; size_t e0, e1; };
  std::vector<Pending> pending;
  double prof_ms[SAN_K_COUNT] = {0};
  long long prof_n[SAN_K_COUNT] = {0};
  std::vector<void*> allocs;
  std::string err;
};

namespace {

int fail(san_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_init_error = msg;
  return code;
}

#define HIP_TRY(c, expr)                                                                        \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return fail((c), e_ == hipErrorOutOfMemory ? SAN_ENOMEM : SAN_EHIP,                       \
                  std::string(#expr) + ": " + hipGetErrorString(e_));                           \
  } while (0)

// With profiling on, a pair of events brackets every launch on the stream.
long prof_mark(san_ctx* c) {
  if (!c->prof_on) return -1;
  if (c->events_used == c->events.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return -1;
    c->events.push_back(e);
  }
  const size_t i = c->events_used++;
  if (hipEventRecord(c->events[i], c->stream) != hipSuccess) return -1;
  return (long)i;
}
void prof_close(san_ctx* c, long e0) {
  if (e0 < 0) return;
  const long e1 = prof_mark(c);
  if (e1 >= 0) c->pending.push_back({c->kind, (size_t)e0, (size_t)e1});
}
int prof_flush(san_ctx* c) {
  if (!c->prof_on) return SAN_OK;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return SAN_EHIP;
  for (const auto& p : c->pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->events[p.e0], c->events[p.e1]) == hipSuccess) {
      c->prof_ms[p.kind] += ms;
      c->prof_n[p.kind] += 1;
    }
  }
  c->pending.clear();
  c->events_used = 0;
  return SAN_OK;
}

#define LAUNCH(c, expr)              \
  do {                               \
    const long pm_ = prof_mark(c);   \
    HIP_TRY((c), (expr));            \
    prof_close((c), pm_);            \
    ++(c)->launches;                 \
  } while (0)

// ---- blob layout: element offsets of every tensor, in the order san.h documents
struct Blob {
  size_t src_emb, tgt_emb, w_out, total;
  struct Attn { size_t wq, bq, wk, bk, wv, bv, wo, bo; };
  struct Ffn { size_t w1, b1, w2, b2; };
  struct Ln { size_t g, b; };
  struct Enc { Attn attn; Ln ln1; Ffn ffn; Ln ln2; };
  struct Dec { Attn self; Ffn aan; size_t wg, bg; Ln ln1; Attn ctx; Ln ln2; Ffn ffn; Ln ln3; };
  std::vector<Enc> enc;
  std::vector<Dec> dec;
};

Blob layout(const san_config& c) {
  Blob b;
  size_t o = 0;
  const size_t d = c.d_model, F = c.d_ff, V = c.vocab;
  auto take = [&](size_t n) { size_t r = o; o += n; return r; };
  auto attn = [&]() { Blob::Attn a; a.wq = take(d * d); a.bq = take(d); a.wk = take(d * d); a.bk = take(d);
                      a.wv = take(d * d); a.bv = take(d); a.wo = take(d * d); a.bo = take(d); return a; };
  auto ffn = [&]() { Blob::Ffn f; f.w1 = take(F * d); f.b1 = take(F); f.w2 = take(d * F); f.b2 = take(d); return f; };
  auto ln = [&]() { Blob::Ln l; l.g = take(d); l.b = take(d); return l; };
  b.src_emb = take(V * d);
  b.tgt_emb = take(V * d);
  for (int i = 0; i < c.n_enc_layers; ++i) {
    Blob::Enc e; e.attn = attn(); e.ln1 = ln(); e.ffn = ffn(); e.ln2 = ln();
    b.enc.push_back(e);
  }
  for (int i = 0; i < c.n_dec_layers; ++i) {
    Blob::Dec e{};
    if (c.self_kind == SAN_SELF_AAN) { e.aan = ffn(); e.wg = take(4 * d * d); e.bg = take(2 * d); }
    else e.self = attn();
    e.ln1 = ln(); e.ctx = attn(); e.ln2 = ln(); e.ffn = ffn(); e.ln3 = ln();
    b.dec.push_back(e);
  }
  b.w_out = take(V * d);
  b.total = o;
  return b;
}

const char* check_config(const san_config& c) {
  if (c.n_enc_layers < 1 || c.n_dec_layers < 1) return "layer counts must be >= 1";
  if (c.d_model < 64 || c.d_model % 64 || c.d_model > 2048) return "d_model must be a multiple of 64 in [64, 2048]";
  if (c.d_ff < 64 || c.d_ff % 64) return "d_ff must be a multiple of 64";
  if (c.n_heads < 1 || c.d_model % c.n_heads) return "d_model must be divisible by n_heads";
  const int dh = c.d_model / c.n_heads;
  if (dh != 16 && dh != 32 && dh != 64 && dh != 128) return "head width must be 16, 32, 64 or 128";
  if (c.vocab < 4 || c.vocab % 4) return "vocab must be a positive multiple of 4";
  if (c.max_batch < 1 || c.max_src_len < 1 || c.max_tgt_len < 1) return "max_batch/max_src_len/max_tgt_len must be >= 1";
  if (c.max_src_len > 1024 || c.max_tgt_len > 1024) return "max_src_len and max_tgt_len must be <= 1024";
  if (c.beam < 1 || c.beam > 32) return "beam must be in [1, 32]";
  if (c.dtype != SAN_F32 && c.dtype != SAN_BF16) return "dtype must be SAN_F32 or SAN_BF16";
  if (c.self_kind != SAN_SELF_DOT && c.self_kind != SAN_SELF_AAN) return "bad self_kind";
  if (c.encdec_share != SAN_SHARE_A && c.encdec_share != SAN_SHARE_S) return "bad encdec_share";
  if (c.use_cache != 0 && c.use_cache != 1) return "use_cache must be 0 or 1";
  if (c.debug < 0 || c.debug > 3) return "debug must be a sum of 1 (per-layer copies) and 2 (general-purpose kernels only)";
  if (!c.use_cache && (c.debug & 1)) return "debug copies need use_cache = 1";
  if (!(c.ln_eps > 0.f)) return "ln_eps must be > 0";
  if (c.pad_id < 0 || c.pad_id >= c.vocab || c.bos_id < 0 || c.bos_id >= c.vocab)
    return "pad_id and bos_id must be word ids in [0, vocab)";
  if (c.eos_id >= c.vocab) return "eos_id must be below vocab (negative: EOS handling off)";
  if ((long long)c.max_batch * c.beam * (long long)c.max_tgt_len > (1ll << 30)) return "batch*beam*max_tgt_len too large";
  return nullptr;
}

bool policy_heads(int n, const int32_t* pi, int layers, std::vector<int>& head) {
  head.clear();
  if (n < 1 || !pi) return false;
  int start = 0;
  for (int i = 0; i < n; ++i) {
    if (pi[i] < 1 || start + pi[i] > layers) return false;
    for (int j = 0; j < pi[i]; ++j) head.push_back(start);
    start += pi[i];
  }
  return start == layers;
}

int dalloc(san_ctx* c, void** p, size_t bytes, bool is_weight) {
  *p = nullptr;
  if (bytes == 0) bytes = 256;
  HIP_TRY(c, hipMalloc(p, bytes));
  c->allocs.push_back(*p);
  (is_weight ? c->weight_bytes : c->state_bytes) += bytes;
  return SAN_OK;
}

// upload `n` elements of the blob starting at element `off` to dst + dst_off elements
int upload(san_ctx* c, void* dst, size_t dst_off, const void* blob, size_t off, size_t n) {
  HIP_TRY(c, hipMemcpy((char*)dst + dst_off * c->esz, (const char*)blob + off * c->esz, n * c->esz,
                       hipMemcpyHostToDevice));
  return SAN_OK;
}

int wtensor(san_ctx* c, void** dst, const void* blob, size_t off, size_t n) {
  int rc = dalloc(c, dst, n * c->esz, true);
  if (rc) return rc;
  return upload(c, *dst, 0, blob, off, n);
}

// ------------------------------------------------------------ kernel plumbing
int gemm(san_ctx* c, const void* A, int lda, const void* W, const void* bias, int M, int N, int K, int relu,
         int out_kind, void* o0, int ld0, long long ts0 = 0, void* o1 = nullptr, int ld1 = 0, long long ts1 = 0,
         void* o2 = nullptr, int ld2 = 0, long long ts2 = 0, int seg_w = 0, bool use_t = false, int ksplit = 0,
         bool bump = false) {
  GemmParams p{};
  p.A = A; p.lda = lda; p.W = W; p.bias = bias;
  p.out[0] = o0; p.out[1] = o1; p.out[2] = o2;
  p.ldo[0] = ld0; p.ldo[1] = ld1; p.ldo[2] = ld2;
  p.tstride[0] = ts0; p.tstride[1] = ts1; p.tstride[2] = ts2;
  p.seg_w = seg_w > 0 ? seg_w : (1 << 30);
  p.t_dev = use_t ? c->t_dev : nullptr;
  p.bump = bump ? c->t_dev : nullptr;
  p.M = M; p.N = N; p.K = K; p.relu = relu; p.out_kind = out_kind;
  if (ksplit == 0) ksplit = 1;
  p.ksplit = ksplit;
  LAUNCH(c, launch_gemm(c->dt, p, c->stream));
  return SAN_OK;
}

// x_out = LayerNorm(res + A W^T + bias): split-K GEMM into fp32 partials, reduced
// by the LayerNorm kernel.
int gemm_ln(san_ctx* c, const void* A, int lda, const void* W, const void* bias, int M, int K, const void* res,
            const void* g, const void* b, void* out, float* dbg, int* defer_ks = nullptr, const AanFuse* aan = nullptr) {
  const int N = c->d;
  int ks = gemm_pick_ksplit(M, N, K, c->dt);
  while (ks > 1 && (size_t)ks * M * N > c->part_elems) ks /= 2;
  if ((size_t)ks * M * N > c->part_elems) return fail(c, SAN_ECAPACITY, "split-K workspace too small");
  int rc = gemm(c, A, lda, W, nullptr, M, N, K, 0, 2, c->part, N, 0, nullptr, 0, 0, nullptr, 0, 0, 0, false, ks);
  if (rc) return rc;
  if (defer_ks) {   // the caller folds this LayerNorm into the next one
    *defer_ks = ks;
    return SAN_OK;
  }
  const int k0 = c->kind;
  c->kind = SAN_K_LN;
  LAUNCH(c, launch_ln_reduce(c->dt, c->part, ks, N, bias, res, N, g, b, out, N, dbg, M, N, c->cfg.ln_eps, c->stream,
                             nullptr, aan));
  c->kind = k0;
  return SAN_OK;
}

// next_aan: the layer that consumes this block's output is an average-attention layer of a
// cached decode; its running sum / mean / gate input are produced by the LayerNorm launch
int ffn_block(san_ctx* c, const DecLayer* L, const EncLayer* E, int M, float* dbg, const AanFuse* next_aan = nullptr) {
  const void* w1 = L ? L->w1 : E->w1; const void* b1 = L ? L->b1 : E->b1;
  const void* w2 = L ? L->w2 : E->w2; const void* b2 = L ? L->b2 : E->b2;
  const void* g = L ? L->ln3g : E->ln2g; const void* b = L ? L->ln3b : E->ln2b;
  if (L) c->kind = SAN_K_FFN;
  int rc = gemm(c, c->x, c->d, w1, b1, M, c->F, c->d, 1, 0, c->hb, c->F);
  if (rc) return rc;
  return gemm_ln(c, c->hb, c->F, w2, b2, M, c->F, c->x, g, b, c->x, dbg, nullptr, next_aan);
}

int dbg_copy(san_ctx* c, const void* src, int lds, float* dst, int rows) {
  if (!dst) return SAN_OK;
  c->kind = SAN_K_MISC;
  LAUNCH(c, launch_to_f32(c->dt, src, lds, dst, rows, c->d, c->stream));
  return SAN_OK;
}

}  // namespace

static int build_ctx(san_ctx* c, const Blob& bl, const void* blob, const std::vector<int>& self_head,
                     const std::vector<int>& ctx_head, const std::vector<int>& enc_head) {
  const san_config* cfg = &c->cfg;
  const int esz = cfg->dtype == SAN_BF16 ? 2 : 4;
  const int Ld = cfg->n_dec_layers;
  c->dt = cfg->dtype; c->esz = esz;
  c->d = cfg->d_model; c->H = cfg->n_heads; c->dh = c->d / c->H; c->F = cfg->d_ff; c->V = cfg->vocab;
  c->rows_max = cfg->max_batch * cfg->beam;
  c->rows_src_max = cfg->max_batch * cfg->max_src_len;
  c->src_pad = (cfg->max_src_len + 31) / 32 * 32;
  const size_t d = c->d, F = c->F, V = c->V;
  const bool aan = cfg->self_kind == SAN_SELF_AAN, shareS = cfg->encdec_share == SAN_SHARE_S;
  const bool nocache = !cfg->use_cache;
  const int T = cfg->max_tgt_len;
  // rows of the decoder-side activations: one per hypothesis, or one per
  // (hypothesis, position) when nothing is cached
  const size_t drows = nocache ? (size_t)c->rows_max * T : (size_t)c->rows_max;

#define TRY(e) do { int rc_ = (e); if (rc_) return rc_; } while (0)
    TRY(wtensor(c, &c->src_emb, blob, bl.src_emb, V * d));
    TRY(wtensor(c, &c->tgt_emb, blob, bl.tgt_emb, V * d));
    TRY(wtensor(c, &c->w_out, blob, bl.w_out, V * d));
    // sinusoidal position table, built once in double on the host
    {
      const int npos = cfg->max_src_len > T ? cfg->max_src_len : T;
      std::vector<float> pe((size_t)npos * d);
      for (int pos = 0; pos < npos; ++pos)
        for (size_t i = 0; i < d; i += 2) {
          const double ang = (double)pos / std::pow(10000.0, (double)i / (double)d);
          pe[pos * d + i] = (float)std::sin(ang);
          pe[pos * d + i + 1] = (float)std::cos(ang);
        }
      TRY(dalloc(c, (void**)&c->pe, pe.size() * 4, true));
      HIP_TRY(c, hipMemcpy(c->pe, pe.data(), pe.size() * 4, hipMemcpyHostToDevice));
    }
    c->enc.resize(cfg->n_enc_layers);
    for (int i = 0; i < cfg->n_enc_layers; ++i) {
      EncLayer& e = c->enc[i];
      const Blob::Enc& o = bl.enc[i];
      e.head = enc_head[i];
      if (e.head == i) {
        TRY(dalloc(c, &e.wqkv, 3 * d * d * esz, true));
        TRY(dalloc(c, &e.bqkv, 3 * d * esz, true));
        TRY(upload(c, e.wqkv, 0, blob, o.attn.wq, d * d));
        TRY(upload(c, e.wqkv, d * d, blob, o.attn.wk, d * d));
        TRY(upload(c, e.wqkv, 2 * d * d, blob, o.attn.wv, d * d));
        TRY(upload(c, e.bqkv, 0, blob, o.attn.bq, d));
        TRY(upload(c, e.bqkv, d, blob, o.attn.bk, d));
        TRY(upload(c, e.bqkv, 2 * d, blob, o.attn.bv, d));
        if (i + 1 < cfg->n_enc_layers && enc_head[i + 1] == i)
          TRY(dalloc(c, (void**)&e.S, (size_t)c->rows_src_max * c->H * cfg->max_src_len * 4, false));
      } else {   // encoder-side sharing (Tab. 5): a follower keeps only its value projection
        TRY(wtensor(c, &e.wqkv, blob, o.attn.wv, d * d));
        TRY(wtensor(c, &e.bqkv, blob, o.attn.bv, d));
      }
      TRY(wtensor(c, &e.wo, blob, o.attn.wo, d * d));
      TRY(wtensor(c, &e.bo, blob, o.attn.bo, d));
      TRY(wtensor(c, &e.ln1g, blob, o.ln1.g, d));
      TRY(wtensor(c, &e.ln1b, blob, o.ln1.b, d));
      TRY(wtensor(c, &e.w1, blob, o.ffn.w1, F * d));
      TRY(wtensor(c, &e.b1, blob, o.ffn.b1, F));
      TRY(wtensor(c, &e.w2, blob, o.ffn.w2, d * F));
      TRY(wtensor(c, &e.b2, blob, o.ffn.b2, d));
      TRY(wtensor(c, &e.ln2g, blob, o.ln2.g, d));
      TRY(wtensor(c, &e.ln2b, blob, o.ln2.b, d));
    }
    c->dec.resize(Ld);
    for (int n = 0; n < Ld; ++n) {
      DecLayer& L = c->dec[n];
      const Blob::Dec& o = bl.dec[n];
      L.self_head = self_head[n];
      L.ctx_head = ctx_head[n];
      const size_t cache_bytes = (size_t)T * c->rows_max * d * esz;
      if (aan) {
        TRY(wtensor(c, &L.aw1, blob, o.aan.w1, F * d));
        TRY(wtensor(c, &L.ab1, blob, o.aan.b1, F));
        TRY(wtensor(c, &L.aw2, blob, o.aan.w2, d * F));
        TRY(wtensor(c, &L.ab2, blob, o.aan.b2, d));
        TRY(wtensor(c, &L.awg, blob, o.wg, 4 * d * d));
        TRY(wtensor(c, &L.abg, blob, o.bg, 2 * d));
        if (!nocache) {   // running sums, all layers in one buffer: one reorder launch
          if (n == 0) TRY(dalloc(c, (void**)&c->aan_all, (size_t)Ld * c->rows_max * d * 4, false));
          L.aan_sum = c->aan_all + (size_t)n * c->rows_max * d;
        }
      } else {
        if (L.self_head == n) {   // block head: fused [q;k;v] projection, key and value cache, weight scratch
          TRY(dalloc(c, &L.w_self, 3 * d * d * esz, true));
          TRY(dalloc(c, &L.b_self, 3 * d * esz, true));
          TRY(upload(c, L.w_self, 0, blob, o.self.wq, d * d));
          TRY(upload(c, L.w_self, d * d, blob, o.self.wk, d * d));
          TRY(upload(c, L.w_self, 2 * d * d, blob, o.self.wv, d * d));
          TRY(upload(c, L.b_self, 0, blob, o.self.bq, d));
          TRY(upload(c, L.b_self, d, blob, o.self.bk, d));
          TRY(upload(c, L.b_self, 2 * d, blob, o.self.bv, d));
          if (!nocache) TRY(dalloc(c, &L.Kc, cache_bytes, false));
          TRY(dalloc(c, (void**)&L.S_self, drows * c->H * T * 4, false));
        } else {                  // follower: only V (Sec. 3.2: its Q/K transformations are discarded)
          TRY(wtensor(c, &L.w_self, blob, o.self.wv, d * d));
          TRY(wtensor(c, &L.b_self, blob, o.self.bv, d));
        }
        if (!nocache) TRY(dalloc(c, &L.Vc, cache_bytes, false));
        TRY(wtensor(c, &L.wo, blob, o.self.wo, d * d));
        TRY(wtensor(c, &L.bo, blob, o.self.bo, d));
      }
      TRY(wtensor(c, &L.ln1g, blob, o.ln1.g, d));
      TRY(wtensor(c, &L.ln1b, blob, o.ln1.b, d));
      if (L.ctx_head == n) {
        TRY(wtensor(c, &L.wq_c, blob, o.ctx.wq, d * d));
        TRY(wtensor(c, &L.bq_c, blob, o.ctx.bq, d));
        TRY(dalloc(c, &L.wkv_c, 2 * d * d * esz, true));
        TRY(dalloc(c, &L.bkv_c, 2 * d * esz, true));
        TRY(upload(c, L.wkv_c, 0, blob, o.ctx.wk, d * d));
        TRY(upload(c, L.wkv_c, d * d, blob, o.ctx.wv, d * d));
        TRY(upload(c, L.bkv_c, 0, blob, o.ctx.bk, d));
        TRY(upload(c, L.bkv_c, d, blob, o.ctx.bv, d));
        TRY(dalloc(c, &L.mem, (size_t)c->rows_src_max * 2 * d * esz, false));
        if (c->dt == 1 && c->dh == 64 && !(cfg->debug & 2))   // for the matrix-core enc-dec attention (attention_mfma.hip)
          TRY(dalloc(c, &L.mem_packed, (size_t)cfg->max_batch * c->H * (c->src_pad / 32) * 8192, false));
        TRY(dalloc(c, (void**)&L.S_ctx, drows * c->H * cfg->max_src_len * 4, false));
        TRY(dalloc(c, &L.A_ctx, drows * d * esz, false));
      } else if (shareS) {
        TRY(wtensor(c, &L.wkv_c, blob, o.ctx.wv, d * d));
        TRY(wtensor(c, &L.bkv_c, blob, o.ctx.bv, d));
        TRY(dalloc(c, &L.mem, (size_t)c->rows_src_max * d * esz, false));
      }
      {
        int pi = 0;   // size of this layer's enc-dec block
        for (int q = 0; q < Ld; ++q) pi += ctx_head[q] == L.ctx_head;
        const bool stacked = pi > 1 && !shareS && !nocache;
        if (stacked && L.ctx_head == n) {
          L.blk_size = pi;
          TRY(dalloc(c, &L.wo_blk, (size_t)pi * d * d * esz, true));
          for (int q = 0; q < pi; ++q) TRY(upload(c, L.wo_blk, (size_t)q * d * d, blob, bl.dec[n + q].ctx.wo, d * d));
          L.y_elems = (size_t)gemm_pick_ksplit(c->rows_max, pi * (int)d, (int)d, c->dt) * c->rows_max * pi * d;
          TRY(dalloc(c, (void**)&L.y_blk, L.y_elems * 4, false));
        }
        if (!stacked) TRY(wtensor(c, &L.wo_c, blob, o.ctx.wo, d * d));
      }
      TRY(wtensor(c, &L.bo_c, blob, o.ctx.bo, d));
      TRY(wtensor(c, &L.ln2g, blob, o.ln2.g, d));
      TRY(wtensor(c, &L.ln2b, blob, o.ln2.b, d));
      TRY(wtensor(c, &L.w1, blob, o.ffn.w1, F * d));
      TRY(wtensor(c, &L.b1, blob, o.ffn.b1, F));
      TRY(wtensor(c, &L.w2, blob, o.ffn.w2, d * F));
      TRY(wtensor(c, &L.b2, blob, o.ffn.b2, d));
      TRY(wtensor(c, &L.ln3g, blob, o.ln3.g, d));
      TRY(wtensor(c, &L.ln3b, blob, o.ln3.b, d));
      if (cfg->debug & 1) {
        TRY(dalloc(c, (void**)&L.dbg_A_self, (size_t)c->rows_max * d * 4, false));
        TRY(dalloc(c, (void**)&L.dbg_A_ctx, (size_t)c->rows_max * d * 4, false));
        TRY(dalloc(c, (void**)&L.dbg_hidden, (size_t)c->rows_max * d * 4, false));
      }
    }
    if (cfg->debug & 1) TRY(dalloc(c, (void**)&c->dbg_enc, (size_t)c->rows_src_max * d * 4, false));
    // workspaces, sized for the largest row count any call uses
    size_t mrows = drows > (size_t)c->rows_src_max ? drows : (size_t)c->rows_src_max;
    const size_t wide = F > 2 * d ? F : 2 * d;
    TRY(dalloc(c, &c->x, mrows * d * esz, false));
    TRY(dalloc(c, &c->qkv, mrows * 3 * d * esz, false));
    TRY(dalloc(c, &c->ab, mrows * d * esz, false));
    TRY(dalloc(c, &c->hb, mrows * wide * esz, false));
    if (aan) TRY(dalloc(c, &c->cat, drows * 2 * d * esz, false));
    c->part_elems = mrows * 2 * d;
    if (c->part_elems < (size_t)4 << 20) c->part_elems = (size_t)4 << 20;
    TRY(dalloc(c, (void**)&c->part, c->part_elems * 4, false));
    TRY(dalloc(c, (void**)&c->t_dev, 256, false));
    TRY(dalloc(c, (void**)&c->anc, (size_t)c->rows_max * T * 4, false));
    if (nocache) TRY(dalloc(c, (void**)&c->hist, (size_t)c->rows_max * T * 4, false));
    TRY(dalloc(c, (void**)&c->last_tok, (size_t)c->rows_max * 4, false));
    TRY(dalloc(c, (void**)&c->src_len, (size_t)cfg->max_batch * 4, false));
    TRY(dalloc(c, (void**)&c->done_dev, ((size_t)cfg->max_batch + 1) * 4, false));
    HIP_TRY(c, hipMemset(c->done_dev, 0, ((size_t)cfg->max_batch + 1) * 4));
    HIP_TRY(c, hipHostMalloc((void**)&c->done_host, ((size_t)2 * cfg->max_batch + 16) * 4, hipHostMallocDefault));
    TRY(dalloc(c, (void**)&c->src_len0, (size_t)cfg->max_batch * 4, false));
    TRY(dalloc(c, (void**)&c->group_map, (size_t)cfg->max_batch * 4, false));
    TRY(dalloc(c, (void**)&c->keep_dev, (size_t)cfg->max_batch * 4, false));
    {
      std::vector<int> iota((size_t)c->rows_max);
      for (size_t i = 0; i < iota.size(); ++i) iota[i] = (int)i;
      TRY(dalloc(c, (void**)&c->iota_dev, iota.size() * 4, false));
      HIP_TRY(c, hipMemcpy(c->iota_dev, iota.data(), iota.size() * 4, hipMemcpyHostToDevice));
    }
    TRY(dalloc(c, (void**)&c->cand_lp, (size_t)c->rows_max * 32 * 4, false));
    TRY(dalloc(c, (void**)&c->cand_idx, (size_t)c->rows_max * 32 * 4, false));
    HIP_TRY(c, hipMemset(c->t_dev, 0, 256));
    HIP_TRY(c, hipMemset(c->last_tok, 0xff, (size_t)c->rows_max * 4));
    HIP_TRY(c, hipDeviceSynchronize());
#undef TRY
  return SAN_OK;
}

// =============================================================================
extern "C" {

size_t san_weight_bytes(const san_config* cfg) {
  if (!cfg || check_config(*cfg)) return 0;
  return layout(*cfg).total * (cfg->dtype == SAN_BF16 ? 2 : 4);
}

const char* san_last_error(const san_ctx* ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

void san_free(san_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  if (ctx->graph2) (void)hipGraphExecDestroy(ctx->graph2);
  for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
  for (void* p : ctx->allocs) (void)hipFree(p);
  if (ctx->done_host) (void)hipHostFree(ctx->done_host);
  delete ctx;
}

int san_init(const san_config* cfg, const void* weights_host, size_t weight_bytes, const san_policy* policy,
             void* hip_stream, san_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !weights_host || !policy || !out) return fail(nullptr, SAN_EINVAL, "null argument");
  if (const char* m = check_config(*cfg)) return fail(nullptr, SAN_EINVAL, m);
  const Blob bl = layout(*cfg);
  const int esz = cfg->dtype == SAN_BF16 ? 2 : 4;
  if (weight_bytes != bl.total * esz) {
    char buf[128];
    snprintf(buf, sizeof buf, "weight blob is %zu bytes, expected %zu", weight_bytes, bl.total * (size_t)esz);
    return fail(nullptr, SAN_EINVAL, buf);
  }
  std::vector<int> self_head, ctx_head;
  const int Ld = cfg->n_dec_layers;
  if (cfg->self_kind == SAN_SELF_AAN) {
    for (int i = 0; i < Ld; ++i) self_head.push_back(i);
  } else if (!policy_heads(policy->n_self, policy->self_pi, Ld, self_head)) {
    return fail(nullptr, SAN_EPOLICY, "self-attention policy must be block sizes >= 1 that sum to n_dec_layers");
  }
  if (!policy_heads(policy->n_encdec, policy->encdec_pi, Ld, ctx_head))
    return fail(nullptr, SAN_EPOLICY, "enc-dec policy must be block sizes >= 1 that sum to n_dec_layers");

  std::vector<int> enc_head;
  if (policy->n_enc == 0 || !policy->enc_pi) {
    for (int i = 0; i < cfg->n_enc_layers; ++i) enc_head.push_back(i);
  } else if (!policy_heads(policy->n_enc, policy->enc_pi, cfg->n_enc_layers, enc_head)) {
    return fail(nullptr, SAN_EPOLICY, "encoder policy must be block sizes >= 1 that sum to n_enc_layers");
  }
  {
    // set-up of san_topk_noalloc's fixed scratch on this device (the context's device)
    void* ptr = nullptr;
    const hipError_t e = scratch_address(&ptr);
    if (e != hipSuccess) return fail(nullptr, SAN_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
  }
  san_ctx* c = new (std::nothrow) san_ctx();
  if (!c) return fail(nullptr, SAN_ENOMEM, "host allocation failed");
  c->cfg = *cfg;
  c->stream = (hipStream_t)hip_stream;
  const int rc = build_ctx(c, bl, weights_host, self_head, ctx_head, enc_head);
  if (rc) {
    g_init_error = c->err;
    for (void* p : c->allocs) (void)hipFree(p);
    if (c->done_host) (void)hipHostFree(c->done_host);
    delete c;
    return rc;
  }
  *out = c;
  return SAN_OK;
}

int san_encode(san_ctx* c, const int32_t* src_ids_dev, const int32_t* src_len_dev, int32_t batch, int32_t max_src) {
  if (!c) return SAN_EINVAL;
  if (!src_ids_dev || !src_len_dev || batch < 1 || max_src < 1) return fail(c, SAN_EINVAL, "san_encode: bad argument");
  if (batch > c->cfg.max_batch || max_src > c->cfg.max_src_len)
    return fail(c, SAN_ECAPACITY, "san_encode: batch or max_src exceeds the configured maximum");
  const int d = c->d, Ms = batch * max_src;
  const float scale = 1.0f / std::sqrt((float)c->dh);
  c->t = -1;
  int rc;
  c->kind = SAN_K_MISC;
  HIP_TRY(c, hipMemcpyAsync(c->src_len, src_len_dev, (size_t)batch * 4, hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(c, hipMemcpyAsync(c->src_len0, src_len_dev, (size_t)batch * 4, hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(c, hipMemcpyAsync(c->group_map, c->iota_dev, (size_t)batch * 4, hipMemcpyDeviceToDevice, c->stream));
  c->batch = batch;   // the encoder below runs on the whole batch
  c->batch_enc = batch;
  c->active.resize(batch);
  for (int i = 0; i < batch; ++i) c->active[i] = i;
  LAUNCH(c, launch_embed(c->dt, src_ids_dev, max_src, max_src, c->src_emb, c->pe, nullptr, c->x, Ms, d, c->V,
                         (float)std::sqrt((double)d), nullptr, nullptr, 0, c->stream));
  for (size_t li = 0; li < c->enc.size(); ++li) {
    const EncLayer& e = c->enc[li];
    const bool ehead = e.head == (int)li;
    if (ehead) {
      if ((rc = gemm(c, c->x, d, e.wqkv, e.bqkv, Ms, 3 * d, d, 0, 0, c->qkv, 3 * d))) return rc;
    } else {
      if ((rc = gemm(c, c->x, d, e.wqkv, e.bqkv, Ms, d, d, 0, 0, (char*)c->qkv + (size_t)2 * d * c->esz, 3 * d))) return rc;
    }
    AttnParams a{};
    a.S_buf = c->enc[e.head].S; a.ldS = c->cfg.max_src_len;
    a.apply = ehead ? 0 : 1;
    a.emit = ehead && e.S != nullptr;
    a.q = c->qkv; a.ldq = 3 * d;
    a.K = (char*)c->qkv + (size_t)d * c->esz; a.ldk = 3 * d;
    a.V = (char*)c->qkv + (size_t)2 * d * c->esz; a.ldv = 3 * d;
    a.out = c->ab; a.ldo = d;
    a.len = c->src_len; a.rows = Ms; a.groups = batch; a.rpg = max_src; a.slot_stride = max_src;
    a.H = c->H; a.dh = c->dh; a.lmax = max_src; a.scale = scale;
    LAUNCH(c, launch_attention(c->dt, a, c->stream));
    if ((rc = gemm_ln(c, c->ab, d, e.wo, e.bo, Ms, d, c->x, e.ln1g, e.ln1b, c->x, nullptr))) return rc;
    if ((rc = ffn_block(c, nullptr, &e, Ms, nullptr))) return rc;
    c->kind = SAN_K_MISC;
  }
  if (c->dbg_enc) LAUNCH(c, launch_to_f32(c->dt, c->x, d, c->dbg_enc, Ms, d, c->stream));
  // encoder-decoder keys/values: block heads get [K;V]; in mode S every follower gets its own V
  for (DecLayer& L : c->dec) {
    if (!L.mem) continue;
    const int N = L.wq_c ? 2 * d : d;
    if ((rc = gemm(c, c->x, d, L.wkv_c, L.bkv_c, Ms, N, d, 0, 0, L.mem, N))) return rc;
    if (L.mem_packed)
      LAUNCH(c, launch_pack_memory(L.mem, N, (char*)L.mem + (size_t)d * c->esz, N, batch, max_src, c->H, L.mem_packed,
                                   c->src_pad / 32, c->stream));
  }
  HIP_TRY(c, hipMemsetAsync(c->t_dev, 0, 4, c->stream));
  HIP_TRY(c, hipMemsetAsync(c->done_dev, 0, ((size_t)c->cfg.max_batch + 1) * 4, c->stream));
  c->batch = batch; c->max_src = max_src; c->t = 0;
  c->graph_rows = 0;   // a captured step graph is tied to the batch shape
  return prof_flush(c);
}

int san_rewind(san_ctx* c) {
  if (!c) return SAN_EINVAL;
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_rewind before san_encode");
  HIP_TRY(c, hipMemsetAsync(c->t_dev, 0, 4, c->stream));
  HIP_TRY(c, hipMemsetAsync(c->done_dev, 0, ((size_t)c->cfg.max_batch + 1) * 4, c->stream));
  if (c->batch != c->batch_enc) {   // sentences dropped by san_compact come back
    HIP_TRY(c, hipMemcpyAsync(c->src_len, c->src_len0, (size_t)c->batch_enc * 4, hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->group_map, c->iota_dev, (size_t)c->batch_enc * 4, hipMemcpyDeviceToDevice, c->stream));
    c->batch = c->batch_enc;
    c->active.resize(c->batch);
    for (int i = 0; i < c->batch; ++i) c->active[i] = i;
    c->graph_rows = 0;
  }
  c->t = 0;
  return SAN_OK;
}

// skip_embed: the input of this step was embedded by the previous step's beam tail (san_decode_n)
static int decode_cached(san_ctx* c, const int32_t* tokens, float* logits, bool skip_embed = false) {
  const int d = c->d, B = c->batch * c->cfg.beam, T = c->cfg.max_tgt_len;
  const float scale = 1.0f / std::sqrt((float)c->dh);
  const bool aan = c->cfg.self_kind == SAN_SELF_AAN, shareS = c->cfg.encdec_share == SAN_SHARE_S;
  const bool dbg = (c->cfg.debug & 1) != 0;
  const int cache_rows = c->batch_enc * c->cfg.beam;   // the caches keep the encoded batch's row stride
  const long long slab = (long long)cache_rows * d;    // cache elements per position
  const int* group_map = c->batch != c->batch_enc ? c->group_map : nullptr;
  int rc;
  c->kind = SAN_K_MISC;
  // an average-attention layer's running sum, mean and gate input come out of the launch that
  // writes its input x (the embedding for layer 0, the previous layer's last LayerNorm otherwise)
  auto aan_of = [&](int n) { return AanFuse{c->dec[n].aan_sum, c->ab, c->cat, c->t_dev}; };
  const AanFuse aan0 = aan ? aan_of(0) : AanFuse{};
  if (!skip_embed)
    LAUNCH(c, launch_embed(c->dt, tokens, 1, 1, c->tgt_emb, c->pe, c->t_dev, c->x, B, d, c->V,
                           (float)std::sqrt((double)d), c->last_tok, c->anc, T, c->stream, aan ? &aan0 : nullptr));
  const int Ld = (int)c->dec.size();
  for (int n = 0; n < Ld; ++n) {
    DecLayer& L = c->dec[n];
    bool fuse_ln = false;
    int ks_self = 1;
    if (aan) {
      c->kind = SAN_K_AAN;
      if ((rc = gemm(c, c->ab, d, L.aw1, L.ab1, B, c->F, d, 1, 0, c->hb, c->F))) return rc;
      // g goes to the right half of [x ; g]
      if ((rc = gemm(c, c->hb, c->F, L.aw2, L.ab2, B, d, c->F, 0, 0, (char*)c->cat + (size_t)d * c->esz, 2 * d))) return rc;
      if ((rc = gemm(c, c->cat, 2 * d, L.awg, nullptr, B, 2 * d, 2 * d, 0, 2, c->part, 2 * d, 0, nullptr, 0, 0, nullptr, 0, 0,
                     0, false, 1)))
        return rc;
      LAUNCH(c, launch_aan_post(c->dt, c->part, L.abg, c->cat, L.ln1g, L.ln1b, c->x, L.dbg_A_self, B, d,
                                c->cfg.ln_eps, c->stream));
    } else {
      const bool head = L.self_head == n;
      const bool has_followers = head && n + 1 < Ld && c->dec[n + 1].self_head == n;
      c->kind = SAN_K_PROJ;
      if (head) {   // Eq. 3: q, k, v; k and v land directly in this position's cache slot
        if ((rc = gemm(c, c->x, d, L.w_self, L.b_self, B, 3 * d, d, 0, 0, c->qkv, d, 0, L.Kc, d, slab, L.Vc, d, slab, d,
                       true)))
          return rc;
      } else {      // Eq. 4: only v
        if ((rc = gemm(c, c->x, d, L.w_self, L.b_self, B, d, d, 0, 0, L.Vc, d, slab, nullptr, 0, 0, nullptr, 0, 0, 0,
                       true)))
          return rc;
      }
      AttnParams a{};
      a.q = c->qkv; a.ldq = d;
      a.K = L.Kc; a.ldk = d; a.V = L.Vc; a.ldv = d;
      a.S_buf = c->dec[L.self_head].S_self; a.ldS = T;
      a.out = c->ab; a.ldo = d;
      a.anc = c->anc; a.ld_anc = T; a.t_dev = c->t_dev;
      a.self_mode = 1; a.rows = B; a.rpg = c->cfg.beam; a.slot_rows = cache_rows; a.H = c->H; a.dh = c->dh; a.lmax = T; a.scale = scale;
      a.apply = head ? 0 : 1;
      a.emit = head && (has_followers || dbg);
      c->kind = head ? SAN_K_ATTN_SELF : SAN_K_ATTN_APPLY;
      LAUNCH(c, launch_attention(c->dt, a, c->stream));
      if ((rc = dbg_copy(c, c->ab, d, L.dbg_A_self, B))) return rc;
      c->kind = SAN_K_OUT;
      // an enc-dec follower of an Eq. 5 block has no kernel between its two
      // LayerNorms: both run in one launch further down
      fuse_ln = c->dec[L.ctx_head].wo_blk != nullptr && L.ctx_head != n;
      if ((rc = gemm_ln(c, c->ab, d, L.wo, L.bo, B, d, c->x, L.ln1g, L.ln1b, c->x, nullptr, fuse_ln ? &ks_self : nullptr)))
        return rc;
    }
    // ---- encoder-decoder attention
    const bool chead = L.ctx_head == n;
    DecLayer& Hd = c->dec[L.ctx_head];
    const void* A = Hd.A_ctx;
    if (chead || shareS) {
      AttnParams a{};
      if (chead) {
        c->kind = SAN_K_PROJ;
        if ((rc = gemm(c, c->x, d, L.wq_c, L.bq_c, B, d, d, 0, 0, c->qkv, d))) return rc;
        a.q = c->qkv; a.ldq = d;
        a.K = L.mem; a.ldk = 2 * d;
        a.V = (char*)L.mem + (size_t)d * c->esz; a.ldv = 2 * d;
        a.kv_packed = L.mem_packed; a.kv_blocks = c->src_pad / 32;
        a.out = L.A_ctx;
        const bool has_followers = n + 1 < Ld && c->dec[n + 1].ctx_head == n;
        a.emit = (shareS && has_followers) || dbg;
        a.zero_tail = dbg;
      } else {    // mode S follower: head's weights times this layer's own V
        a.V = L.mem; a.ldv = d;
        a.out = c->ab;
        a.apply = 1;
        A = c->ab;
      }
      a.S_buf = Hd.S_ctx; a.ldS = c->cfg.max_src_len;
      a.ldo = d;
      a.len = c->src_len; a.rows = B; a.groups = c->batch; a.rpg = c->cfg.beam; a.slot_stride = c->max_src;
      a.group_map = group_map;
      a.H = c->H; a.dh = c->dh; a.lmax = c->max_src; a.scale = scale;
      c->kind = chead ? SAN_K_ATTN_CTX : SAN_K_ATTN_CTX_APPLY;
      LAUNCH(c, launch_attention(c->dt, a, c->stream));
    }
    if ((rc = dbg_copy(c, A, d, L.dbg_A_ctx, B))) return rc;
    c->kind = SAN_K_OUT;
    if (Hd.wo_blk) {
      // A^{m+i} = A^m (Eq. 5): all output projections of the block in one GEMM at the head
      const int N = Hd.blk_size * d;
      if (chead) {
        int ks = gemm_pick_ksplit(B, N, d, c->dt);
        while (ks > 1 && (size_t)ks * B * N > Hd.y_elems) ks /= 2;
        Hd.y_ks = ks;
        if ((rc = gemm(c, A, d, Hd.wo_blk, nullptr, B, N, d, 0, 2, Hd.y_blk, N, 0, nullptr, 0, 0, nullptr, 0, 0, 0, false, ks)))
          return rc;
      }
      c->kind = SAN_K_LN;
      if (fuse_ln) {
        LnStage2 s2{Hd.y_blk + (size_t)(n - L.ctx_head) * d, Hd.y_ks, N, L.bo_c, L.ln2g, L.ln2b};
        LAUNCH(c, launch_ln_reduce(c->dt, c->part, ks_self, d, L.bo, c->x, d, L.ln1g, L.ln1b, c->x, d, nullptr, B, d,
                                   c->cfg.ln_eps, c->stream, &s2));
      } else {
        LAUNCH(c, launch_ln_reduce(c->dt, Hd.y_blk + (size_t)(n - L.ctx_head) * d, Hd.y_ks, N, L.bo_c, c->x, d, L.ln2g,
                                   L.ln2b, c->x, d, nullptr, B, d, c->cfg.ln_eps, c->stream));
      }
    } else {
      if ((rc = gemm_ln(c, A, d, L.wo_c, L.bo_c, B, d, c->x, L.ln2g, L.ln2b, c->x, nullptr))) return rc;
    }
    const AanFuse nxt = (aan && n + 1 < Ld) ? aan_of(n + 1) : AanFuse{};
    if ((rc = ffn_block(c, &L, nullptr, B, L.dbg_hidden, nxt.sum ? &nxt : nullptr))) return rc;
  }
  c->kind = SAN_K_LOGITS;
  if (c->cand_tiles > 0) {
    GemmParams p{};
    p.A = c->x; p.lda = d; p.W = c->w_out;
    p.M = B; p.N = c->V; p.K = d; p.out_kind = 3; p.ksplit = 1;
    p.seg_w = 1 << 30;
    p.bump = c->t_dev;
    p.cand_k = c->cfg.beam; p.cand_tiles = c->cand_tiles;
    p.cand_ms = c->part_ms; p.cand_v = c->part_cv; p.cand_i = c->part_ci;
    LAUNCH(c, launch_gemm(c->dt, p, c->stream));
    return SAN_OK;
  }
  return gemm(c, c->x, d, c->w_out, nullptr, B, c->V, d, 0, 1, logits, c->V, 0, nullptr, 0, 0, nullptr, 0, 0, 0, false,
              0, true);
}

// Nothing cached: every position of every hypothesis is recomputed (rows =
// hypotheses x positions), with a causal mask in self-attention.
static int decode_uncached(san_ctx* c, const int32_t* tokens, float* logits) {
  const int d = c->d, B = c->batch * c->cfg.beam, T = c->cfg.max_tgt_len;
  const int np = c->t + 1, M = B * np;
  const float scale = 1.0f / std::sqrt((float)c->dh);
  const bool shareS = c->cfg.encdec_share == SAN_SHARE_S;
  int rc;
  c->kind = SAN_K_MISC;
  LAUNCH(c, launch_step_begin(tokens, c->last_tok, nullptr, c->hist, T, c->t_dev, B, c->stream));
  LAUNCH(c, launch_embed(c->dt, c->hist, T, np, c->tgt_emb, c->pe, nullptr, c->x, M, d, c->V,
                         (float)std::sqrt((double)d), nullptr, nullptr, 0, c->stream));
  const int Ld = (int)c->dec.size();
  const bool aan = c->cfg.self_kind == SAN_SELF_AAN;
  for (int n = 0; n < Ld; ++n) {
    DecLayer& L = c->dec[n];
    const bool head = L.self_head == n;
    if (aan) {
      // the average-attention layer over all positions: prefix means instead of running sums
      c->kind = SAN_K_AAN;
      LAUNCH(c, launch_aan_prefix_mean(c->dt, c->x, c->ab, c->cat, B, np, d, c->stream));
      if ((rc = gemm(c, c->ab, d, L.aw1, L.ab1, M, c->F, d, 1, 0, c->hb, c->F))) return rc;
      if ((rc = gemm(c, c->hb, c->F, L.aw2, L.ab2, M, d, c->F, 0, 0, (char*)c->cat + (size_t)d * c->esz, 2 * d))) return rc;
      if ((rc = gemm(c, c->cat, 2 * d, L.awg, nullptr, M, 2 * d, 2 * d, 0, 2, c->part, 2 * d, 0, nullptr, 0, 0, nullptr, 0, 0,
                     0, false, 1)))
        return rc;
      LAUNCH(c, launch_aan_post(c->dt, c->part, L.abg, c->cat, L.ln1g, L.ln1b, c->x, nullptr, M, d, c->cfg.ln_eps,
                                c->stream));
    } else {
    c->kind = SAN_K_PROJ;
    if (head) {
      if ((rc = gemm(c, c->x, d, L.w_self, L.b_self, M, 3 * d, d, 0, 0, c->qkv, 3 * d))) return rc;
    } else {
      if ((rc = gemm(c, c->x, d, L.w_self, L.b_self, M, d, d, 0, 0, (char*)c->qkv + (size_t)2 * d * c->esz, 3 * d)))
        return rc;
    }
    {
      AttnParams a{};
      a.q = c->qkv; a.ldq = 3 * d;
      a.K = (char*)c->qkv + (size_t)d * c->esz; a.ldk = 3 * d;
      a.V = (char*)c->qkv + (size_t)2 * d * c->esz; a.ldv = 3 * d;
      a.S_buf = c->dec[L.self_head].S_self; a.ldS = T;
      a.out = c->ab; a.ldo = d;
      a.n_fixed = np; a.rows = M; a.groups = B; a.rpg = np; a.slot_stride = np; a.causal = np;
      a.H = c->H; a.dh = c->dh; a.lmax = np; a.scale = scale;
      a.apply = head ? 0 : 1;
      a.emit = head && n + 1 < Ld && c->dec[n + 1].self_head == n;
      c->kind = head ? SAN_K_ATTN_SELF : SAN_K_ATTN_APPLY;
      LAUNCH(c, launch_attention(c->dt, a, c->stream));
    }
    c->kind = SAN_K_OUT;
    if ((rc = gemm_ln(c, c->ab, d, L.wo, L.bo, M, d, c->x, L.ln1g, L.ln1b, c->x, nullptr))) return rc;
    }
    const bool chead = L.ctx_head == n;
    DecLayer& Hd = c->dec[L.ctx_head];
    const void* A = Hd.A_ctx;
    if (chead || shareS) {
      AttnParams a{};
      if (chead) {
        c->kind = SAN_K_PROJ;
        if ((rc = gemm(c, c->x, d, L.wq_c, L.bq_c, M, d, d, 0, 0, c->qkv, d))) return rc;
        a.q = c->qkv; a.ldq = d;
        a.K = L.mem; a.ldk = 2 * d;
        a.V = (char*)L.mem + (size_t)d * c->esz; a.ldv = 2 * d;
        a.out = L.A_ctx;
        a.emit = shareS && n + 1 < Ld && c->dec[n + 1].ctx_head == n;
      } else {
        a.V = L.mem; a.ldv = d;
        a.out = c->ab;
        a.apply = 1;
        A = c->ab;
      }
      a.S_buf = Hd.S_ctx; a.ldS = c->cfg.max_src_len;
      a.ldo = d;
      a.len = c->src_len; a.rows = M; a.groups = c->batch; a.rpg = c->cfg.beam * np; a.slot_stride = c->max_src;
      a.H = c->H; a.dh = c->dh; a.lmax = c->max_src; a.scale = scale;
      c->kind = chead ? SAN_K_ATTN_CTX : SAN_K_ATTN_CTX_APPLY;
      LAUNCH(c, launch_attention(c->dt, a, c->stream));
    }
    c->kind = SAN_K_OUT;
    if ((rc = gemm_ln(c, A, d, L.wo_c, L.bo_c, M, d, c->x, L.ln2g, L.ln2b, c->x, nullptr))) return rc;
    if ((rc = ffn_block(c, &L, nullptr, M, nullptr))) return rc;
  }
  // logits of the last position of every hypothesis
  c->kind = SAN_K_LOGITS;
  return gemm(c, (char*)c->x + (size_t)(np - 1) * d * c->esz, np * d, c->w_out, nullptr, B, c->V, d, 0, 1, logits,
              c->V, 0, nullptr, 0, 0, nullptr, 0, 0, 0, false, 0, true);
}

static int decode_step_impl(san_ctx* c, const int32_t* tokens_dev, float* logits_dev, bool skip_embed) {
  if (!c) return SAN_EINVAL;
  if (!tokens_dev || !logits_dev) return fail(c, SAN_EINVAL, "san_decode_step: null argument");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_decode_step before san_encode");
  if (c->t >= c->cfg.max_tgt_len) return fail(c, SAN_ECAPACITY, "san_decode_step: max_tgt_len steps already decoded");
  c->launches = 0;
  int rc = c->cfg.use_cache ? decode_cached(c, tokens_dev, logits_dev, skip_embed) : decode_uncached(c, tokens_dev, logits_dev);
  if (rc) return rc;
  c->t += 1;   // the device-side counter was advanced by the output-layer kernel
  return prof_flush(c);
}

int san_decode_step(san_ctx* c, const int32_t* tokens_dev, float* logits_dev) {
  return decode_step_impl(c, tokens_dev, logits_dev, false);
}

int san_topk(san_ctx* c, const float* logits_dev, const float* cum_score_dev, int32_t k, int32_t* out_token_dev,
             int32_t* out_parent_dev, float* out_score_dev) {
  if (!c) return SAN_EINVAL;
  if (!logits_dev || !cum_score_dev || !out_token_dev || !out_parent_dev || !out_score_dev)
    return fail(c, SAN_EINVAL, "san_topk: null argument");
  if (k < 1 || k > 32 || k > c->V) return fail(c, SAN_EINVAL, "san_topk: k must be in [1, min(32, vocab)]");
  if (reinterpret_cast<uintptr_t>(logits_dev) % 16) return fail(c, SAN_EINVAL, "san_topk: logits must be 16-byte aligned");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_topk before san_encode");
  c->kind = SAN_K_TOPK;
  const long pm = prof_mark(c);
  HIP_TRY(c, launch_topk(logits_dev, cum_score_dev, c->last_tok, c->cfg.eos_id, c->batch, c->cfg.beam, c->V, k,
                         c->cand_lp, c->cand_idx, out_token_dev, out_parent_dev, out_score_dev, c->stream, nullptr,
                         k == c->cfg.beam ? c->done_dev : nullptr, c->done_dev + c->cfg.max_batch));
  prof_close(c, pm);
  return prof_flush(c);
}

int san_topk_noalloc(san_ctx* c, const float* logits_dev, const float* cum_score_dev, int32_t k,
                     int32_t* out_token_dev, int32_t* out_parent_dev, float* out_score_dev) {
  if (!c) return SAN_EINVAL;
  if (!logits_dev || !cum_score_dev || !out_token_dev || !out_parent_dev || !out_score_dev)
    return fail(c, SAN_EINVAL, "san_topk_noalloc: null argument");
  if (k < 1 || k > 32 || k > c->V) return fail(c, SAN_EINVAL, "san_topk_noalloc: k must be in [1, min(32, vocab)]");
  if (reinterpret_cast<uintptr_t>(logits_dev) % 16)
    return fail(c, SAN_EINVAL, "san_topk_noalloc: logits must be 16-byte aligned");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_topk_noalloc before san_encode");
  if (c->prof_on) return fail(c, SAN_ESTATE, "san_topk_noalloc: switch san_profile off first");
  const size_t cands = (size_t)c->batch * c->cfg.beam * k;
  if (cands > kScratchCands) {
    char buf[160];
    snprintf(buf, sizeof buf, "san_topk_noalloc: batch*beam*k = %zu candidates exceed the fixed scratch of %zu", cands,
             kScratchCands);
    return fail(c, SAN_ECAPACITY, buf);
  }
  void* ptr = nullptr;   // resolved in san_init on this device; a table look-up here
  const hipError_t e = scratch_address(&ptr);
  if (e != hipSuccess) return fail(c, SAN_EHIP, std::string("san_topk_noalloc: scratch address: ") + hipGetErrorString(e));
  // [cands] log-probabilities, then [cands] word ids; every entry the merge reads is
  // written by the row kernel of this same call, so nothing has to be cleared
  float* cand_lp = reinterpret_cast<float*>(ptr);
  int* cand_idx = reinterpret_cast<int*>(static_cast<unsigned char*>(ptr) + kScratchCands * 4);
  HIP_TRY(c, launch_topk(logits_dev, cum_score_dev, c->last_tok, c->cfg.eos_id, c->batch, c->cfg.beam, c->V, k, cand_lp,
                         cand_idx, out_token_dev, out_parent_dev, out_score_dev, c->stream, nullptr,
                         k == c->cfg.beam ? c->done_dev : nullptr, c->done_dev + c->cfg.max_batch));
  return SAN_OK;
}

int san_beam_reorder(san_ctx* c, const int32_t* parent_idx_dev) {
  if (!c) return SAN_EINVAL;
  if (!parent_idx_dev) return fail(c, SAN_EINVAL, "san_beam_reorder: null argument");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_beam_reorder before san_encode");
  if (c->cfg.beam == 1) return SAN_OK;   // a sentence has a single row: nothing can move
  const int T = c->cfg.max_tgt_len;
  c->kind = SAN_K_REORDER;
  const long pm = prof_mark(c);
  if (!c->cfg.use_cache) {
    HIP_TRY(c, launch_reorder_table(c->hist, T, parent_idx_dev, c->t_dev, c->batch, c->cfg.beam, T, c->stream));
  } else if (c->cfg.self_kind == SAN_SELF_AAN) {
    HIP_TRY(c, launch_reorder_rows(c->aan_all, (size_t)c->rows_max * c->d, parent_idx_dev, (int)c->dec.size(), c->batch,
                                   c->cfg.beam, c->d, c->stream));
  } else {
    // the caches stay where they are; only the per-row table of which cache row
    // holds each past position is permuted
    HIP_TRY(c, launch_reorder_table(c->anc, T, parent_idx_dev, c->t_dev, c->batch, c->cfg.beam, T, c->stream));
  }
  prof_close(c, pm);
  return prof_flush(c);
}

int san_debug_get(san_ctx* c, int32_t what, int32_t layer, void* dst_dev, size_t cap) {
  if (!c) return SAN_EINVAL;
  if (!(c->cfg.debug & 1)) return fail(c, SAN_ESTATE, "san_debug_get needs cfg.debug = 1");
  if (!dst_dev || layer < 0 || layer >= (int)c->dec.size()) return fail(c, SAN_EINVAL, "san_debug_get: bad argument");
  DecLayer& L = c->dec[layer];
  if (what == SAN_DBG_ENC_OUT || what == SAN_DBG_MEM) {   // written by san_encode
    if (c->t < 0) return fail(c, SAN_ESTATE, "san_debug_get before san_encode");
    const int Ms = c->batch_enc * c->max_src;
    const int cols = what == SAN_DBG_ENC_OUT ? c->d : (L.wq_c ? 2 * c->d : c->d);
    if (what == SAN_DBG_MEM && !L.mem) return fail(c, SAN_EINVAL, "san_debug_get: this layer keeps no encoder memory");
    if (cap < (size_t)Ms * cols * 4) return fail(c, SAN_EINVAL, "san_debug_get: destination too small");
    if (what == SAN_DBG_ENC_OUT)
      HIP_TRY(c, hipMemcpyAsync(dst_dev, c->dbg_enc, (size_t)Ms * cols * 4, hipMemcpyDeviceToDevice, c->stream));
    else
      HIP_TRY(c, launch_to_f32(c->dt, L.mem, cols, (float*)dst_dev, Ms, cols, c->stream));
    return SAN_OK;
  }
  if (c->t < 1) return fail(c, SAN_ESTATE, "san_debug_get before the first decode step");
  const int B = c->batch * c->cfg.beam;
  const float* src = nullptr;
  switch (what) {
    case SAN_DBG_S_SELF: {
      if (c->cfg.self_kind == SAN_SELF_AAN) return fail(c, SAN_EINVAL, "no self-attention weights with AAN");
      const size_t need = (size_t)B * c->H * c->t * 4;
      if (cap < need) return fail(c, SAN_EINVAL, "san_debug_get: destination too small");
      HIP_TRY(c, launch_compact_S(c->dec[L.self_head].S_self, c->cfg.max_tgt_len, (float*)dst_dev, B * c->H, c->t,
                                  c->stream));
      return SAN_OK;
    }
    case SAN_DBG_S_CTX: {
      const size_t need = (size_t)B * c->H * c->max_src * 4;
      if (cap < need) return fail(c, SAN_EINVAL, "san_debug_get: destination too small");
      HIP_TRY(c, launch_compact_S(c->dec[L.ctx_head].S_ctx, c->cfg.max_src_len, (float*)dst_dev, B * c->H, c->max_src,
                                  c->stream));
      return SAN_OK;
    }
    case SAN_DBG_A_SELF: src = L.dbg_A_self; break;
    case SAN_DBG_A_CTX: src = L.dbg_A_ctx; break;
    case SAN_DBG_HIDDEN: src = L.dbg_hidden; break;
    default: return fail(c, SAN_EINVAL, "san_debug_get: unknown tensor");
  }
  const size_t need = (size_t)B * c->d * 4;
  if (cap < need) return fail(c, SAN_EINVAL, "san_debug_get: destination too small");
  HIP_TRY(c, hipMemcpyAsync(dst_dev, src, need, hipMemcpyDeviceToDevice, c->stream));
  return SAN_OK;
}

int san_profile(san_ctx* c, int32_t enable) {
  if (!c) return SAN_EINVAL;
  int rc = prof_flush(c);
  c->prof_on = enable != 0;
  return rc;
}

int san_profile_read(san_ctx* c, double* ms_out, int64_t* launches_out, int32_t reset) {
  if (!c) return SAN_EINVAL;
  int rc = prof_flush(c);
  for (int k = 0; k < SAN_K_COUNT; ++k) {
    if (ms_out) ms_out[k] = c->prof_ms[k];
    if (launches_out) launches_out[k] = c->prof_n[k];
    if (reset) { c->prof_ms[k] = 0; c->prof_n[k] = 0; }
  }
  return rc;
}

int san_finished(san_ctx* c, int32_t* count_out) {
  if (!c || !count_out) return fail(c, SAN_EINVAL, "san_finished: null argument");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_finished before san_encode");
  HIP_TRY(c, hipMemcpyAsync(c->done_host, c->done_dev + c->cfg.max_batch, 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  *count_out = *c->done_host;
  return SAN_OK;
}

int san_done_flags(san_ctx* c, int32_t* flags_out) {
  if (!c || !flags_out) return fail(c, SAN_EINVAL, "san_done_flags: null argument");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_done_flags before san_encode");
  HIP_TRY(c, hipMemcpyAsync(c->done_host, c->done_dev, (size_t)c->batch * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int i = 0; i < c->batch; ++i) flags_out[i] = c->done_host[i];
  return SAN_OK;
}

int san_active(san_ctx* c, int32_t* sentences_out, int32_t* n_out) {
  if (!c || !n_out) return fail(c, SAN_EINVAL, "san_active: null argument");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_active before san_encode");
  *n_out = c->batch;
  if (sentences_out)
    for (int i = 0; i < c->batch; ++i) sentences_out[i] = c->active[i];
  return SAN_OK;
}

int san_compact(san_ctx* c, const int32_t* keep, int32_t n_keep) {
  if (!c || !keep) return fail(c, SAN_EINVAL, "san_compact: null argument");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_compact before san_encode");
  if (!c->cfg.use_cache) return fail(c, SAN_ESTATE, "san_compact needs use_cache = 1");
  if (c->prof_on) return fail(c, SAN_ESTATE, "san_compact: switch san_profile off first");
  if (n_keep < 1 || n_keep > c->batch) return fail(c, SAN_EINVAL, "san_compact: n_keep must be in [1, batch]");
  for (int i = 0; i < n_keep; ++i)
    if (keep[i] < 0 || keep[i] >= c->batch || (i > 0 && keep[i] <= keep[i - 1]))
      return fail(c, SAN_EINVAL, "san_compact: keep must be strictly increasing sentence indices of the current batch");
  if (n_keep == c->batch) return SAN_OK;
  const int beam = c->cfg.beam, T = c->cfg.max_tgt_len, nrows = n_keep * beam;
  const bool aan = c->cfg.self_kind == SAN_SELF_AAN;
  size_t need = (size_t)nrows * T * 4;
  if (aan && (size_t)nrows * c->d * 4 > need) need = (size_t)nrows * c->d * 4;
  if (need > c->cmp_tmp_bytes) {
    // sized once for the largest batch (the old buffer, if any, is released with the context)
    const size_t full = std::max((size_t)c->rows_max * T * 4, aan ? (size_t)c->rows_max * c->d * 4 : (size_t)0);
    int rc = dalloc(c, &c->cmp_tmp, full, false);
    if (rc) return rc;
    c->cmp_tmp_bytes = full;
  }
  // the list goes up through pinned memory; the stream is drained first so that an
  // earlier list is no longer being read
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  int* pin = c->done_host + c->cfg.max_batch + 8;
  for (int i = 0; i < n_keep; ++i) pin[i] = keep[i];
  HIP_TRY(c, hipMemcpyAsync(c->keep_dev, pin, (size_t)n_keep * 4, hipMemcpyHostToDevice, c->stream));
  // every per-row / per-sentence array: gather into the staging buffer, copy back
  auto move = [&](void* arr, int rpg, int w) -> int {
    HIP_TRY(c, launch_gather_groups(c->cmp_tmp, arr, c->keep_dev, rpg, n_keep, w, c->stream));
    HIP_TRY(c, hipMemcpyAsync(arr, c->cmp_tmp, (size_t)n_keep * rpg * w * 4, hipMemcpyDeviceToDevice, c->stream));
    return SAN_OK;
  };
  int rc;
  if (!aan && (rc = move(c->anc, beam, T))) return rc;
  if ((rc = move(c->last_tok, beam, 1))) return rc;
  if ((rc = move(c->src_len, 1, 1))) return rc;
  if ((rc = move(c->group_map, 1, 1))) return rc;
  if ((rc = move(c->done_dev, 1, 1))) return rc;
  if (aan)
    for (size_t l = 0; l < c->dec.size(); ++l)
      if ((rc = move(c->dec[l].aan_sum, beam, c->d))) return rc;
  HIP_TRY(c, launch_count_flags(c->done_dev, n_keep, c->done_dev + c->cfg.max_batch, c->stream));
  for (int i = 0; i < n_keep; ++i) c->active[i] = c->active[keep[i]];
  c->active.resize(n_keep);
  c->batch = n_keep;
  c->graph_rows = 0;   // a captured step graph is tied to the batch shape
  return SAN_OK;
}

// Column tiles per row when the loop's output layer emits candidates for `rows` rows; 0: that mode
// is off (beam too wide for the epilogue, too many candidates per row, buffers not there).
static int loop_cand_tiles(const san_ctx* c, int rows) {
  if (!c->part_ms || c->cfg.beam > kGemmCandMaxK || rows <= 0) return 0;
  const int bn = gemm_cand_tile_n(rows, c->V, c->d, c->dt);
  const int tiles = (c->V + bn - 1) / bn;
  return topk_cands_fit(tiles, c->cfg.beam) ? tiles : 0;
}

// One beam-search step on the ping-pong buffers: parity p reads set p, writes set p^1.
// entry_rows > 0: the batch was compacted during this call; the history goes to the rows
// the caller knows (row_map), entry_rows apart per step.
// mode & 1 (fused): the per-sentence merge, the reordering of the per-row state and (dot-product
// self-attention) the embedding of the next step's input run as one kernel, and this step's
// input was embedded by the previous step's (or by the call's prologue).  mode & 2: the output
// layer feeds the beam step per-tile candidates and `logits` is not written.
static int loop_step(san_ctx* c, int p, int32_t* out_tokens, int32_t* out_parents, float* logits, int entry_rows,
                     int mode) {
  const bool aan = c->cfg.self_kind == SAN_SELF_AAN, fused = (mode & 1) != 0;
  // Nobody outside the loop sees a step's logits, and the beam step needs only each row's
  // log-sum-exp and `beam` largest entries: the output layer then emits those per column tile and
  // the [rows][vocab] array is neither written nor read.
  const int tiles = (mode & 2) ? loop_cand_tiles(c, c->batch * c->cfg.beam) : 0;
  c->cand_tiles = tiles;
  int rc = decode_step_impl(c, c->pp_tok[p], logits, fused && !aan);
  c->cand_tiles = 0;
  if (rc) return rc;
  TopkHistory h{out_tokens, out_parents, c->t_dev, c->t0_dev, entry_rows > 0 ? c->row_map : nullptr, entry_rows};
  if (fused) {
    BeamTail tl{};
    tl.t_dev = c->t_dev; tl.max_t = c->cfg.max_tgt_len; tl.d = c->d; tl.dtype = c->dt;
    if (aan) {
      tl.aan_sum = c->aan_all; tl.layer_stride = (size_t)c->rows_max * c->d; tl.layers = (int)c->dec.size();
    } else {
      tl.anc = c->anc; tl.ld_anc = c->cfg.max_tgt_len;
      tl.emb = c->tgt_emb; tl.pe = c->pe; tl.x = c->x; tl.scale = (float)std::sqrt((double)c->d);
    }
    if (tiles > 0)
      HIP_TRY(c, launch_topk_cands(c->part_ms, c->part_cv, c->part_ci, tiles, c->pp_cum[p], c->last_tok, c->cfg.eos_id,
                                   c->batch, c->cfg.beam, c->V, c->cfg.beam, c->cand_lp, c->cand_idx, c->pp_tok[p ^ 1],
                                   c->pp_par, c->pp_cum[p ^ 1], c->stream, &h, c->done_dev,
                                   c->done_dev + c->cfg.max_batch, &tl, c->last_tok));
    else
      HIP_TRY(c, launch_topk(logits, c->pp_cum[p], c->last_tok, c->cfg.eos_id, c->batch, c->cfg.beam, c->V, c->cfg.beam,
                             c->cand_lp, c->cand_idx, c->pp_tok[p ^ 1], c->pp_par, c->pp_cum[p ^ 1], c->stream, &h,
                             c->done_dev, c->done_dev + c->cfg.max_batch, &tl, c->last_tok));
    return SAN_OK;
  }
  if (tiles > 0)
    HIP_TRY(c, launch_topk_cands(c->part_ms, c->part_cv, c->part_ci, tiles, c->pp_cum[p], c->last_tok, c->cfg.eos_id,
                                 c->batch, c->cfg.beam, c->V, c->cfg.beam, c->cand_lp, c->cand_idx, c->pp_tok[p ^ 1],
                                 c->pp_par, c->pp_cum[p ^ 1], c->stream, &h, c->done_dev,
                                 c->done_dev + c->cfg.max_batch));
  else
    HIP_TRY(c, launch_topk(logits, c->pp_cum[p], c->last_tok, c->cfg.eos_id, c->batch, c->cfg.beam, c->V, c->cfg.beam,
                           c->cand_lp, c->cand_idx, c->pp_tok[p ^ 1], c->pp_par, c->pp_cum[p ^ 1], c->stream, &h,
                           c->done_dev, c->done_dev + c->cfg.max_batch));
  return san_beam_reorder(c, c->pp_par);
}

int san_decode_n(san_ctx* c, int32_t n, const int32_t* tokens_dev, float* cum_io_dev, int32_t* out_tokens_dev,
                 int32_t* out_parents_dev, float* logits_work_dev, int32_t flags) {
  if (!c) return SAN_EINVAL;
  if (!tokens_dev || !cum_io_dev || !out_tokens_dev || !out_parents_dev || !logits_work_dev || n < 1)
    return fail(c, SAN_EINVAL, "san_decode_n: bad argument");
  if (flags & ~(SAN_LOOP_GRAPH | SAN_LOOP_COMPACT | SAN_LOOP_LOGITS)) return fail(c, SAN_EINVAL, "san_decode_n: unknown flag");
  if (reinterpret_cast<uintptr_t>(logits_work_dev) % 16)
    return fail(c, SAN_EINVAL, "san_decode_n: the logits scratch must be 16-byte aligned");
  if (c->t < 0) return fail(c, SAN_ESTATE, "san_decode_n before san_encode");
  if (c->t + n > c->cfg.max_tgt_len) return fail(c, SAN_ECAPACITY, "san_decode_n: would exceed max_tgt_len");
  if (c->prof_on) return fail(c, SAN_ESTATE, "san_decode_n: switch san_profile off first");
  const bool use_graph = (flags & SAN_LOOP_GRAPH) != 0;
  const bool compact = (flags & SAN_LOOP_COMPACT) != 0 && c->cfg.eos_id >= 0;
  if (use_graph && (!c->stream || !c->cfg.use_cache))
    return fail(c, SAN_EINVAL, "san_decode_n: graph replay needs a non-default stream and use_cache = 1");
  if ((flags & SAN_LOOP_COMPACT) && !c->cfg.use_cache)
    return fail(c, SAN_EINVAL, "san_decode_n: dropping finished sentences needs use_cache = 1");
  const int beam = c->cfg.beam;
  const int batch0 = c->batch, rows0 = batch0 * beam;   // the batch as the caller knows it
  int rc;
  if (!c->pp_par) {
    for (int i = 0; i < 2; ++i) {
      if ((rc = dalloc(c, (void**)&c->pp_tok[i], (size_t)c->rows_max * 4, false))) return rc;
      if ((rc = dalloc(c, (void**)&c->pp_cum[i], (size_t)c->rows_max * 4, false))) return rc;
    }
    if ((rc = dalloc(c, (void**)&c->pp_par, (size_t)c->rows_max * 4, false))) return rc;
    if ((rc = dalloc(c, (void**)&c->t0_dev, 256, false))) return rc;
    if ((rc = dalloc(c, (void**)&c->row_map, (size_t)c->rows_max * 4, false))) return rc;
    if ((rc = dalloc(c, (void**)&c->cum_final, (size_t)c->rows_max * 4, false))) return rc;
    if ((rc = dalloc(c, (void**)&c->drop_dev, (size_t)c->cfg.max_batch * 4, false))) return rc;
    if (c->cfg.use_cache && beam <= kGemmCandMaxK && topk_cands_fit((c->V + 63) / 64, beam)) {
      // sized for the narrowest column tile (64) the output layer may pick
      const size_t slots = (size_t)c->rows_max * ((c->V + 63) / 64);
      if ((rc = dalloc(c, (void**)&c->part_cv, slots * 2 * beam * 4, false))) return rc;
      if ((rc = dalloc(c, (void**)&c->part_ci, slots * 2 * beam * 4, false))) return rc;
      if ((rc = dalloc(c, (void**)&c->part_ms, slots * 2 * 4, false))) return rc;   // last: it switches the mode on
    }
  }
  HIP_TRY(c, hipMemcpyAsync(c->pp_tok[0], tokens_dev, (size_t)rows0 * 4, hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(c, hipMemcpyAsync(c->pp_cum[0], cum_io_dev, (size_t)rows0 * 4, hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(c, hipMemcpyAsync(c->t0_dev, c->t_dev, 4, hipMemcpyDeviceToDevice, c->stream));
  if (compact)
    HIP_TRY(c, hipMemcpyAsync(c->row_map, c->iota_dev, (size_t)rows0 * 4, hipMemcpyDeviceToDevice, c->stream));
  // The beam step's tail is fused (see loop_step) unless finished sentences may leave the batch
  // during this call (their state is then regathered between steps) or nothing is cached.
  const bool fused = c->cfg.use_cache && !compact && c->cfg.beam <= 32;
  const int mode = (fused ? 1 : 0) | ((c->cfg.use_cache && !(flags & SAN_LOOP_LOGITS)) ? 2 : 0);
  if (fused && c->cfg.self_kind != SAN_SELF_AAN) {
    // the first step's input; every later one is embedded by the step before it
    c->kind = SAN_K_MISC;
    LAUNCH(c, launch_embed(c->dt, c->pp_tok[0], 1, 1, c->tgt_emb, c->pe, c->t_dev, c->x, rows0, c->d, c->V,
                           (float)std::sqrt((double)c->d), c->last_tok, c->anc, c->cfg.max_tgt_len, c->stream));
  }
  // sentence i of the current batch is sentence ent[i] of the caller's; drop_from[b]: steps done
  // when the caller's sentence b left the batch (-1: still in)
  std::vector<int> ent(batch0), drop_from(batch0, -1);
  for (int i = 0; i < batch0; ++i) ent[i] = i;
  bool compacted = false;

  // With EOS handling on, the flags of finished sentences and their count are read back
  // (one stream synchronisation) every kCheckEvery steps: the loop stops once every
  // sentence is finished, and -- when asked to -- drops the finished ones from the batch
  // once they are a quarter of it and enough steps remain to pay for the new graph.
  constexpr int kCheckEvery = 8, kMinStepsLeft = 16;
  int done = 0, last_check = 0;
  bool stop = false;
  enum { kGoOn = 0, kStop = 1, kCompacted = 2 };
  auto check = [&](int& action) -> int {
    action = stop ? kStop : kGoOn;
    if (stop || c->cfg.eos_id < 0 || done - last_check < kCheckEvery) return SAN_OK;
    last_check = done;
    const int mb = c->cfg.max_batch;
    HIP_TRY(c, hipMemcpyAsync(c->done_host, c->done_dev, ((size_t)mb + 1) * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    const int cnt = c->done_host[mb];
    if (cnt >= c->batch) { stop = true; action = kStop; return SAN_OK; }
    if (!compact || cnt * 4 < c->batch || n - done < kMinStepsLeft) return SAN_OK;
    std::vector<int32_t> keep;
    for (int i = 0; i < c->batch; ++i)
      if (!c->done_host[i]) keep.push_back(i);
    if (keep.empty() || (int)keep.size() == c->batch) return SAN_OK;
    // the leaving sentences' scores are final: every current score goes to the caller's row now
    const int p = done & 1, rows = c->batch * beam;
    HIP_TRY(c, launch_scatter_words(c->cum_final, c->pp_cum[p], c->row_map, rows, c->stream));
    for (int i = 0; i < c->batch; ++i)
      if (c->done_host[i]) drop_from[ent[i]] = done;
    int r = san_compact(c, keep.data(), (int32_t)keep.size());
    if (r) return r;
    // the loop's own per-row arrays follow (san_compact left the list in keep_dev)
    const int nk = (int)keep.size();
    void* arrs[3] = {c->pp_tok[p], c->pp_cum[p], c->row_map};
    for (void* a : arrs) {
      HIP_TRY(c, launch_gather_groups(c->cmp_tmp, a, c->keep_dev, beam, nk, 1, c->stream));
      HIP_TRY(c, hipMemcpyAsync(a, c->cmp_tmp, (size_t)nk * beam * 4, hipMemcpyDeviceToDevice, c->stream));
    }
    for (int i = 0; i < nk; ++i) ent[i] = ent[keep[i]];
    ent.resize(nk);
    compacted = true;
    action = kCompacted;
    return SAN_OK;
  };

  while (done < n && !stop) {
    const int rows = c->batch * beam;
    const int entry_rows = compacted ? rows0 : 0;
    int action = kGoOn;
    if (use_graph && n - done >= 2 && (done & 1) == 0) {
      // the graph holds two steps (parity 0 then 1); it is rebuilt when the caller's
      // buffers or the batch change
      const bool stale = !c->graph2 || c->graph_key[0] != out_tokens_dev || c->graph_key[1] != out_parents_dev ||
                         c->graph_key[2] != logits_work_dev || c->graph_rows != rows ||
                         c->graph_entry_rows != entry_rows || c->graph_fused != mode;
      if (stale && n - done >= 4) {
        if (c->graph2) { (void)hipGraphExecDestroy(c->graph2); c->graph2 = nullptr; }
        // two ordinary steps first, so that one-time set-up inside the launchers
        // (per-kernel attributes) has happened before anything is captured
        for (int i = 0; i < 2; ++i, ++done)
          if ((rc = loop_step(c, done & 1, out_tokens_dev, out_parents_dev, logits_work_dev, entry_rows, mode))) return rc;
        hipGraph_t g = nullptr;
        const int t_before = c->t;
        HIP_TRY(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
        rc = loop_step(c, 0, out_tokens_dev, out_parents_dev, logits_work_dev, entry_rows, mode);
        if (!rc) rc = loop_step(c, 1, out_tokens_dev, out_parents_dev, logits_work_dev, entry_rows, mode);
        const hipError_t e = hipStreamEndCapture(c->stream, &g);
        c->t = t_before;   // capturing queued nothing
        if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
        if (e != hipSuccess) return fail(c, SAN_EHIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
        const hipError_t e2 = hipGraphInstantiate(&c->graph2, g, nullptr, nullptr, 0);
        (void)hipGraphDestroy(g);
        if (e2 != hipSuccess) return fail(c, SAN_EHIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(e2));
        c->graph_key[0] = out_tokens_dev; c->graph_key[1] = out_parents_dev; c->graph_key[2] = logits_work_dev;
        c->graph_rows = rows;
        c->graph_entry_rows = entry_rows;
        c->graph_fused = mode;
      }
      const bool fresh = c->graph2 && c->graph_rows == rows && c->graph_entry_rows == entry_rows && c->graph_fused == mode &&
                         c->graph_key[0] == out_tokens_dev && c->graph_key[1] == out_parents_dev &&
                         c->graph_key[2] == logits_work_dev;
      while (fresh && done + 2 <= n) {
        if ((rc = check(action))) return rc;
        if (action != kGoOn) break;
        HIP_TRY(c, hipGraphLaunch(c->graph2, c->stream));
        c->t += 2;
        done += 2;
      }
      if (action != kGoOn) continue;   // stopped, or the batch shrank: a new graph
    }
    // what the graph did not cover (no graph asked for, an odd tail, too few steps to capture)
    while (done < n) {
      if ((rc = check(action))) return rc;
      if (action != kGoOn) break;
      if ((rc = loop_step(c, done & 1, out_tokens_dev, out_parents_dev, logits_work_dev, entry_rows, mode))) return rc;
      ++done;
    }
  }
  if (!compacted) {
    HIP_TRY(c, hipMemcpyAsync(cum_io_dev, c->pp_cum[done & 1], (size_t)rows0 * 4, hipMemcpyDeviceToDevice, c->stream));
    return SAN_OK;
  }
  // sentences that left the batch: their rows of the history keep extending with EOS in
  // place, their scores were saved when they left
  HIP_TRY(c, launch_scatter_words(c->cum_final, c->pp_cum[done & 1], c->row_map, c->batch * beam, c->stream));
  HIP_TRY(c, hipMemcpyAsync(cum_io_dev, c->cum_final, (size_t)rows0 * 4, hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));   // the pinned staging area is free again
  int* pin = c->done_host;
  for (int b = 0; b < batch0; ++b) pin[b] = drop_from[b];
  HIP_TRY(c, hipMemcpyAsync(c->drop_dev, pin, (size_t)batch0 * 4, hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, launch_fill_finished(out_tokens_dev, out_parents_dev, c->drop_dev, batch0, beam, done, c->cfg.eos_id,
                                  c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return SAN_OK;
}

int san_policy_accumulate(san_ctx* c) {
  if (!c) return SAN_EINVAL;
  if (!(c->cfg.debug & 1) || !c->cfg.use_cache) return fail(c, SAN_ESTATE, "san_policy_accumulate needs cfg.debug = 1 and use_cache = 1");
  if (c->t < 1) return fail(c, SAN_ESTATE, "san_policy_accumulate before the first decode step");
  const int L = (int)c->dec.size(), B = c->batch * c->cfg.beam;
  if (L > kMaxPolicyLayers) return fail(c, SAN_EINVAL, "too many decoder layers for policy statistics");
  const size_t pairs = (size_t)L * (L - 1) / 2;
  if (!c->js_acc) {
    int rc = dalloc(c, (void**)&c->js_acc, 2 * (size_t)L * L * sizeof(double), false);
    if (rc) return rc;
    rc = dalloc(c, (void**)&c->js_part, (pairs ? pairs : 1) * (size_t)c->rows_max * c->H * 4, false);
    if (rc) return rc;
    HIP_TRY(c, hipMemsetAsync(c->js_acc, 0, 2 * (size_t)L * L * sizeof(double), c->stream));
  }
  JsParams p{};
  p.L = L; p.rows = B; p.H = c->H; p.part = c->js_part;
  if (c->cfg.self_kind == SAN_SELF_DOT) {
    for (int n = 0; n < L; ++n) p.S[n] = c->dec[c->dec[n].self_head].S_self;
    p.ld = c->cfg.max_tgt_len; p.len = nullptr; p.n_fixed = c->t;
    HIP_TRY(c, launch_js_accumulate(p, c->js_acc, c->stream));
    c->js_count[0] += (long long)B * c->H;
  }
  for (int n = 0; n < L; ++n) p.S[n] = c->dec[c->dec[n].ctx_head].S_ctx;
  p.ld = c->cfg.max_src_len; p.len = c->src_len; p.rows_per_len = c->cfg.beam;
  HIP_TRY(c, launch_js_accumulate(p, c->js_acc + (size_t)L * L, c->stream));
  c->js_count[1] += (long long)B * c->H;
  return SAN_OK;
}

int san_policy_read(san_ctx* c, int32_t which, double* js_out, int64_t* count_out, int32_t reset) {
  if (!c) return SAN_EINVAL;
  if (which != 0 && which != 1) return fail(c, SAN_EINVAL, "san_policy_read: which must be 0 (self) or 1 (enc-dec)");
  const int L = (int)c->dec.size();
  if (count_out) *count_out = c->js_count[which];
  if (js_out) {
    for (int i = 0; i < L * L; ++i) js_out[i] = 0.0;
    if (c->js_acc && c->js_count[which] > 0) {
      HIP_TRY(c, hipMemcpyAsync(js_out, c->js_acc + (size_t)which * L * L, (size_t)L * L * sizeof(double),
                                hipMemcpyDeviceToHost, c->stream));
      HIP_TRY(c, hipStreamSynchronize(c->stream));
      for (int i = 0; i < L * L; ++i) js_out[i] /= (double)c->js_count[which];
    }
  }
  if (reset && c->js_acc) {
    HIP_TRY(c, hipMemsetAsync(c->js_acc + (size_t)which * L * L, 0, (size_t)L * L * sizeof(double), c->stream));
    c->js_count[which] = 0;
  }
  return SAN_OK;
}

int san_policy_search(const double* js, int32_t n_layers, double theta, int32_t* pi_out, int32_t* n_blocks_out) {
  if (!js || !pi_out || !n_blocks_out || n_layers < 1) return SAN_EINVAL;
  return policy_search(js, n_layers, theta, pi_out, n_blocks_out);
}

int san_stream_read(san_ctx* c, const void* src_dev, size_t bytes) {
  if (!c || !src_dev) return fail(c, SAN_EINVAL, "null argument");
  c->kind = SAN_K_MISC;
  // t_dev is a 256-byte allocation of which only the first word is the step counter
  LAUNCH(c, launch_stream_read(src_dev, bytes, reinterpret_cast<unsigned*>(c->t_dev + 32), c->stream));
  return SAN_OK;
}

int32_t san_step(const san_ctx* c) { return c ? c->t : -1; }
size_t san_device_bytes(const san_ctx* c, int32_t which) { return !c ? 0 : (which == 0 ? c->weight_bytes : c->state_bytes); }
int32_t san_last_launch_count(const san_ctx* c) { return c ? c->launches : 0; }

}  // extern "C"
