// Beam step: per-row log-softmax statistics and k best words (one pass over the
// logits, the row is held in registers), then a per-sentence merge of the
// beam*k row candidates.  Order everywhere: higher value first, then lower index.
#include "common.h"
#include "kernels.h"

namespace san {

constexpr int kTopkThreads = 1024;
constexpr int kTopkVpt = 32;  // register-resident row: vocab <= 32 * 1024

struct Cand {
  float v;
  int i;
};
// a is better than b
__device__ __forceinline__ bool better(float av, int ai, float bv, int bi) {
  return av > bv || (av == bv && ai < bi);
}
template <int CTRL> __device__ __forceinline__ void best_step_dpp(Cand& c) {
  const float ov = dpp_mov<CTRL>(c.v);
  const int oi = dpp_mov_i<CTRL>(c.i);
  if (better(ov, oi, c.v, c.i)) { c.v = ov; c.i = oi; }
}
// best (value, index) pair of the wave, in every lane: DPP moves inside the rows
// of 16 lanes, two row swaps across rows
__device__ __forceinline__ Cand wave_best(Cand c) {
  best_step_dpp<kDppQuadSwap1>(c);
  best_step_dpp<kDppQuadSwap2>(c);
  best_step_dpp<kDppRowHalfMirror>(c);
  best_step_dpp<kDppRowMirror>(c);
  {
    const float ov = __uint_as_float(other_xor16(__float_as_uint(c.v)));
    const int oi = (int)other_xor16((unsigned)c.i);
    if (better(ov, oi, c.v, c.i)) { c.v = ov; c.i = oi; }
  }
  {
    const float ov = __uint_as_float(other_xor32(__float_as_uint(c.v)));
    const int oi = (int)other_xor32((unsigned)c.i);
    if (better(ov, oi, c.v, c.i)) { c.v = ov; c.i = oi; }
  }
  return c;
}

constexpr int kNone = 0x7fffffff;   // index of an empty candidate slot (value -inf)

// One compare-exchange stage of a bitonic network over the 64 lanes: partner is
// lane ^ J; inside blocks of K lanes that sort "best first" the lower lane of a
// pair keeps the better element, in the other blocks the worse one.
template <int K, int J> __device__ __forceinline__ void sort_stage(Cand& c, int lane) {
  const float ov = __uint_as_float(lane_xor<J>(__float_as_uint(c.v)));
  const int oi = (int)lane_xor<J>((unsigned)c.i);
  const bool lower = (lane & J) == 0;
  const bool best_first = K == kWave || (lane & K) == 0;
  const bool other_better = better(ov, oi, c.v, c.i);
  if ((lower == best_first) ? other_better : !other_better) { c.v = ov; c.i = oi; }
}
// Sorts the (value, index) pairs of each aligned group of N lanes (N = 16 or 64),
// best first: lane r of the group ends up with rank r.  Register-only stages (10
// for N = 16, 21 for N = 64); equal pairs can only be empty slots.
template <int N> __device__ __forceinline__ void wave_sort(Cand& c, int lane) {
  static_assert(N == 16 || N == kWave, "group size");
  sort_stage<2, 1>(c, lane);
  sort_stage<4, 2>(c, lane); sort_stage<4, 1>(c, lane);
  sort_stage<8, 4>(c, lane); sort_stage<8, 2>(c, lane); sort_stage<8, 1>(c, lane);
  if (N == 16) {
    // last merge of a 16-lane group: every group sorts best first
    sort_stage<kWave, 8>(c, lane); sort_stage<kWave, 4>(c, lane); sort_stage<kWave, 2>(c, lane);
    sort_stage<kWave, 1>(c, lane);
    return;
  }
  sort_stage<16, 8>(c, lane); sort_stage<16, 4>(c, lane); sort_stage<16, 2>(c, lane); sort_stage<16, 1>(c, lane);
  sort_stage<32, 16>(c, lane); sort_stage<32, 8>(c, lane); sort_stage<32, 4>(c, lane); sort_stage<32, 2>(c, lane);
  sort_stage<32, 1>(c, lane);
  sort_stage<64, 32>(c, lane); sort_stage<64, 16>(c, lane); sort_stage<64, 8>(c, lane); sort_stage<64, 4>(c, lane);
  sort_stage<64, 2>(c, lane); sort_stage<64, 1>(c, lane);
}
// The k best of the candidates load(0..nc-1), best first in lanes 0..k-1 (k <= 32).
// Up to 16 candidates: one short sort.  Otherwise 64 candidates per pass; the running
// k best ride along in lanes k..2k-1 of the next pass.
template <typename F> __device__ __forceinline__ Cand wave_topk(F load, int nc, int k, int lane) {
  Cand cur = {-INFINITY, kNone};
  if (nc <= 16) {
    if (lane < nc) cur = load(lane);
    wave_sort<16>(cur, lane);
    return cur;
  }
  for (int base = 0; base < nc; base += kWave) {
    Cand c = {-INFINITY, kNone};
    if (base + lane < nc) c = load(base + lane);
    wave_sort<kWave>(c, lane);
    if (base > 0) {
      const float mv = __shfl(cur.v, lane - k, kWave);
      const int mi = __shfl(cur.i, lane - k, kWave);
      if (lane >= k) {
        c.v = lane < 2 * k ? mv : -INFINITY;
        c.i = lane < 2 * k ? mi : kNone;
      }
      wave_sort<kWave>(c, lane);
    }
    cur = c;
  }
  return cur;
}

// (max, sum of exp(x - max)) pairs combine associatively
__device__ __forceinline__ void lse_merge(float& m, float& s, float om, float os) {
  const float M = fmaxf(m, om);
  if (M == -INFINITY) { s = 0.f; return; }
  s = s * expf(m - M) + os * expf(om - M);
  m = M;
}

constexpr int kMaxK = 32;
constexpr int kListCap = 1024;

template <bool REG>
__global__ __launch_bounds__(kTopkThreads) void topk_row_kernel(const float* logits, const int* last_tok,
                                                                int eos_id, int vocab, int k, float* cand_lp,
                                                                int* cand_idx) {
  constexpr int NW = kTopkThreads / kWave;
  __shared__ float red_m[NW], red_s[NW];
  __shared__ float wc_v[NW * kMaxK];   // every wave's k best values ...
  __shared__ int wc_i[NW * kMaxK];     // ... and their word ids
  __shared__ float list_v[kListCap];   // elements >= threshold
  __shared__ int list_i[kListCap];
  __shared__ int list_n;
  __shared__ float thresh;
  bool use_list = false;
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const float* x = logits + (size_t)row * vocab;
  const int nit = (vocab + kTopkThreads - 1) / kTopkThreads;

  // register-resident row: 16-byte loads, register `it` holds word
  // (it / 4) * 4096 + tid * 4 + it % 4 (vocab is a multiple of 4, rows are 16-byte aligned)
  float reg[REG ? kTopkVpt : 1];
  if (REG) {
#pragma unroll
    for (int q = 0; q < kTopkVpt / 4; ++q) {
      const int idx = q * 4 * kTopkThreads + tid * 4;
      float4 v = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      if (idx < vocab) v = *reinterpret_cast<const float4*>(x + idx);
      reg[4 * q] = v.x; reg[4 * q + 1] = v.y; reg[4 * q + 2] = v.z; reg[4 * q + 3] = v.w;
    }
  }
  auto index_of = [&](int it) -> int {
    return REG ? (it >> 2) * 4 * kTopkThreads + tid * 4 + (it & 3) : it * kTopkThreads + tid;
  };
  auto val = [&](int it) -> float {
    if (REG) return reg[it];
    const int idx = index_of(it);
    return idx < vocab ? x[idx] : -INFINITY;
  };

  // ---- log-sum-exp of the row: wave maximum first, then one exp per element
  float tmax = -INFINITY;
  if (REG) {
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) tmax = fmaxf(tmax, reg[it]);
  } else {
    for (int it = 0; it < nit; ++it) tmax = fmaxf(tmax, val(it));
  }
  const float m_w = wave_max(tmax);
  float s = 0.f;
  if (REG) {
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) s += (reg[it] == -INFINITY) ? 0.f : __expf(reg[it] - m_w);
  } else {
    for (int it = 0; it < nit; ++it) {
      const float v = val(it);
      s += (v == -INFINITY) ? 0.f : expf(v - m_w);
    }
  }
  s = wave_sum(s);
  if (lane == 0) { red_m[wid] = m_w; red_s[wid] = s; }

  const bool finished = eos_id >= 0 && last_tok[row] == eos_id;
  if (REG) {
    // ---- threshold pass.  Any value T with at least k elements >= T is a lower
    // bound on the k-th largest element, so every element of the row's top k is
    // >= T, and usually only a handful of elements are.  Those go to a short list in
    // LDS that wave 0 orders; a list overflow (masses of equal values) falls back to
    // the general rounds below.  T = the k-th largest wave maximum (k <= 16 waves;
    // already known from the log-sum-exp), else the k-th largest of the waves' k
    // largest thread maxima.
    const bool by_wave_max = k <= NW;
    if (!by_wave_max) {
      Cand c = {tmax, lane};
      wave_sort<kWave>(c, lane);
      if (lane < k) wc_v[wid * k + lane] = c.v;
    }
    if (tid == 0) list_n = 0;
    __syncthreads();
    if (wid == 0) {
      const Cand c = by_wave_max ? wave_topk([&](int q) { return Cand{red_m[q], q}; }, NW, k, lane)
                                 : wave_topk([&](int q) { return Cand{wc_v[q], q}; }, NW * k, k, lane);
      if (lane == k - 1) thresh = c.v;
    }
    __syncthreads();
    const float T = thresh;
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) {
      const int idx = index_of(it);
      if (idx < vocab && reg[it] >= T) {
        const int pos = atomicAdd(&list_n, 1);
        if (pos < kListCap) { list_v[pos] = reg[it]; list_i[pos] = idx; }
      }
    }
    __syncthreads();
    use_list = list_n <= kListCap;
  }
  if (!use_list) {
    // ---- general path: each wave's k best by k rounds over its elements
    float pv = INFINITY;
    int pi = -1;
    for (int round = 0; round < k; ++round) {
      Cand best = {-INFINITY, kNone};
      if (REG) {
#pragma unroll
        for (int it = 0; it < kTopkVpt; ++it) {
          const int idx = index_of(it);
          const float v = reg[it];
          const bool after = (v < pv) || (v == pv && idx > pi);
          if (idx < vocab && after && better(v, idx, best.v, best.i)) { best.v = v; best.i = idx; }
        }
      } else {
        for (int it = 0; it < nit; ++it) {
          const int idx = index_of(it);
          const float v = val(it);
          const bool after = (v < pv) || (v == pv && idx > pi);
          if (idx < vocab && after && better(v, idx, best.v, best.i)) { best.v = v; best.i = idx; }
        }
      }
      best = wave_best(best);
      if (lane == 0) { wc_v[wid * k + round] = best.v; wc_i[wid * k + round] = best.i; }
      pv = best.v;
      pi = best.i;
    }
  }
  __syncthreads();
  if (wid != 0) return;

  float m = red_m[0];
  s = red_s[0];
  for (int w = 1; w < NW; ++w) lse_merge(m, s, red_m[w], red_s[w]);   // same order in every lane
  const float lse = m + logf(s);

  // a finished hypothesis can only be extended by EOS at cost 0
  if (finished) {
    if (lane < k) {
      const int id = lane == 0 ? eos_id : (lane - 1 < eos_id ? lane - 1 : lane);
      cand_lp[(size_t)row * k + lane] = lane == 0 ? 0.f : -INFINITY;
      cand_idx[(size_t)row * k + lane] = id;
    }
    return;
  }
  // ---- wave 0 orders the candidates (the short list, or the NW * k wave candidates)
  const int nc = use_list ? list_n : NW * k;
  const float* cv = use_list ? list_v : wc_v;
  const int* ci = use_list ? list_i : wc_i;
  const Cand c = wave_topk([&](int q) { return Cand{ci[q] == kNone ? -INFINITY : cv[q], ci[q]}; }, nc, k, lane);
  if (lane < k) {
    cand_lp[(size_t)row * k + lane] = c.v - lse;
    cand_idx[(size_t)row * k + lane] = c.i;
  }
}

// The same row result from the output layer's per-tile candidates (GEMM out_kind 3) instead of
// the logits: ms[row][tile] = (max, sum of exp(x - max)) of the tile's columns, cv / ci
// [row][tile][2 k] = unordered entries that include its k largest (empty slots: id kNone).
// The row's k largest are among them; k rounds, each taking the best candidate that comes
// after the previous pick in the order (higher value, then lower word id).  CPT =
// candidate slots per thread, held in registers.
constexpr int kCombThreads = 256;
template <int CPT>
__global__ __launch_bounds__(kCombThreads) void cand_combine_kernel(const float* ms, const float* cv, const int* ci,
                                                                    int ntiles, const int* last_tok, int eos_id, int k,
                                                                    float* cand_lp, int* cand_idx) {
  constexpr int NW = kCombThreads / kWave;
  __shared__ float red_m[NW], red_s[NW];
  __shared__ float bw_v[2][NW];
  __shared__ int bw_i[2][NW];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int nc = ntiles * 2 * k;
  const float* rv = cv + (size_t)row * nc;
  const int* ri = ci + (size_t)row * nc;
  float v[CPT];
  int id[CPT];
#pragma unroll
  for (int i = 0; i < CPT; ++i) {
    // unconditional requests (clamped index), so that all of them are in flight together
    const int q = tid + i * kCombThreads, qc = min(q, nc - 1);
    const float lv = rv[qc];
    const int li = ri[qc];
    v[i] = q < nc ? lv : -INFINITY;
    id[i] = q < nc ? li : kNone;
  }
  float m = -INFINITY, s = 0.f;
  for (int x = tid; x < ntiles; x += kCombThreads) {
    const float2 t = reinterpret_cast<const float2*>(ms)[(size_t)row * ntiles + x];
    lse_merge(m, s, t.x, t.y);
  }
  {
    const float mw = wave_max(m);
    s = wave_sum(m == -INFINITY ? 0.f : s * __expf(m - mw));
    m = mw;
  }
  if (lane == 0) { red_m[wid] = m; red_s[wid] = s; }

  float pv = INFINITY;
  int pi = -1;
  float my_v = -INFINITY;
  int my_i = kNone;
  for (int round = 0; round < k; ++round) {
    Cand best = {-INFINITY, kNone};
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const bool after = (v[i] < pv) || (v[i] == pv && id[i] > pi);
      if (id[i] != kNone && after && better(v[i], id[i], best.v, best.i)) { best.v = v[i]; best.i = id[i]; }
    }
    best = wave_best(best);
    if (lane == 0) { bw_v[round & 1][wid] = best.v; bw_i[round & 1][wid] = best.i; }
    __syncthreads();   // one barrier per round: the next round writes the other pair of slots
    best = Cand{bw_v[round & 1][0], bw_i[round & 1][0]};
#pragma unroll
    for (int w = 1; w < NW; ++w)
      if (better(bw_v[round & 1][w], bw_i[round & 1][w], best.v, best.i)) best = Cand{bw_v[round & 1][w], bw_i[round & 1][w]};
    pv = best.v;
    pi = best.i;
    if (tid == round) { my_v = best.v; my_i = best.i; }
  }
  if (tid >= k) return;
  m = red_m[0];       // visible: k >= 1 barriers since they were written
  s = red_s[0];
  for (int w = 1; w < NW; ++w) lse_merge(m, s, red_m[w], red_s[w]);
  const float lse = m + logf(s);
  if (eos_id >= 0 && last_tok[row] == eos_id) {   // a finished hypothesis can only be extended by EOS at cost 0
    const int fid = tid == 0 ? eos_id : (tid - 1 < eos_id ? tid - 1 : tid);
    cand_lp[(size_t)row * k + tid] = tid == 0 ? 0.f : -INFINITY;
    cand_idx[(size_t)row * k + tid] = fid;
    return;
  }
  cand_lp[(size_t)row * k + tid] = my_i == kNone ? -INFINITY : my_v - lse;
  cand_idx[(size_t)row * k + tid] = my_i;
}

// Merge of one sentence's beam*k candidates by one wave; lanes 0..k-1 end up with the k best.
// Writes the picks, the optional history and the finished flag; returns this lane's pick.
__device__ __forceinline__ Cand merge_sentence(int b, int lane, const float* cand_lp, const int* cand_idx, const float* cum,
                                               int beam, int vocab, int k, int nsent, int* out_tok, int* out_parent,
                                               float* out_score, const TopkHistory& hist, int eos_id, int* done,
                                               int* done_count) {
  // multi-step decoding: this step's picks are also appended to the caller's
  // [step][rows] arrays; the step index comes from the device-side counters
  const long long hoff =
      hist.tok ? (long long)(*hist.t_dev - 1 - *hist.t0_dev) * (hist.row_map ? hist.ld : nsent * k) : 0;
  const Cand best = wave_topk(
      [&](int q) {
        const int bi = q / k;
        const int r = b * beam + bi;
        const int id = cand_idx[(size_t)r * k + (q % k)];
        const float sc = cum[r] + cand_lp[(size_t)r * k + (q % k)];
        // an empty row slot, or a score that is not a number, never wins
        return (id == kNone || !(sc == sc)) ? Cand{-INFINITY, kNone} : Cand{sc, bi * vocab + id};
      },
      beam * k, k, lane);
  if (lane < k) {
    const bool ok = best.i != kNone;
    const int tk = ok ? best.i % vocab : 0, pr = b * beam + (ok ? best.i / vocab : 0);
    out_tok[(size_t)b * k + lane] = tk;
    out_parent[(size_t)b * k + lane] = pr;
    out_score[(size_t)b * k + lane] = ok ? best.v : -INFINITY;
    if (hist.tok) {
      const int o = b * k + lane;
      const int oo = hist.row_map ? hist.row_map[o] : o;
      hist.tok[hoff + oo] = tk;
      hist.par[hoff + oo] = hist.row_map ? hist.row_map[pr] : pr;
    }
  }
  if (done && eos_id >= 0) {
    // the sentence is finished once every hypothesis kept ends in EOS (it stays so: such
    // a hypothesis can only be extended by EOS); counted once
    const bool open = lane < k && (best.i == kNone || best.i % vocab != eos_id);
    if (__ballot(open) == 0 && lane == 0 && done[b] == 0) {
      done[b] = 1;
      atomicAdd(done_count, 1);
    }
  }
  return best;
}

// One wave per sentence: merge the beam*k candidates, keep the k best.
__global__ __launch_bounds__(64) void topk_merge_kernel(const float* cand_lp, const int* cand_idx, const float* cum,
                                                        int beam, int vocab, int k, int* out_tok, int* out_parent,
                                                        float* out_score, TopkHistory hist, int eos_id, int* done,
                                                        int* done_count) {
  merge_sentence(blockIdx.x, threadIdx.x, cand_lp, cand_idx, cum, beam, vocab, k, (int)gridDim.x, out_tok, out_parent,
                 out_score, hist, eos_id, done, done_count);
}

// The merge, then what the beam step means for the sentence's state (see BeamTail): wave 0
// merges, all waves permute the sentence's ancestry rows (or AAN sums) by the parents and embed
// the chosen words as the next step's input.  MAXB = compile-time cap of the beam.
constexpr int kTailThreads = 256;
template <typename T, int MAXB>
__global__ __launch_bounds__(kTailThreads) void beam_tail_kernel(const float* cand_lp, const int* cand_idx,
                                                                 const float* cum, int beam, int vocab, int* out_tok,
                                                                 int* out_parent, float* out_score, TopkHistory hist,
                                                                 int eos_id, int* done, int* done_count, BeamTail tl,
                                                                 int* last_tok) {
  __shared__ int s_tok[kMaxK], s_par[kMaxK];
  const int b = blockIdx.x, tid = threadIdx.x;
  if (tid < kWave) {
    const Cand best = merge_sentence(b, tid, cand_lp, cand_idx, cum, beam, vocab, beam, (int)gridDim.x, out_tok,
                                     out_parent, out_score, hist, eos_id, done, done_count);
    if (tid < beam) {
      const bool ok = best.i != kNone;
      s_tok[tid] = ok ? best.i % vocab : 0;
      s_par[tid] = ok ? best.i / vocab : 0;     // index inside the sentence
    }
  }
  __syncthreads();
  const int t_now = *tl.t_dev;                  // steps done, this one included
  int pl[MAXB];
#pragma unroll
  for (int q = 0; q < MAXB; ++q) pl[q] = s_par[min(q, beam - 1)];
  if (tl.anc) {
    // row r of the table continues row parent[r]: a thread owns a column, reads it for every
    // old row of the sentence, then writes the permuted rows (safe in place)
    const int ncol = min(t_now, tl.max_t);
    for (int j = tid; j < ncol; j += kTailThreads) {
      int old[MAXB];
#pragma unroll
      for (int q = 0; q < MAXB; ++q) old[q] = tl.anc[(size_t)(b * beam + min(q, beam - 1)) * tl.ld_anc + j];
#pragma unroll
      for (int q = 0; q < MAXB; ++q) {
        if (q < beam && pl[q] != q) {
          int v = old[0];
#pragma unroll
          for (int s = 1; s < MAXB; ++s)
            if (s == pl[q]) v = old[s];
          tl.anc[(size_t)(b * beam + q) * tl.ld_anc + j] = v;
        }
      }
    }
  }
  if (tl.aan_sum) {
    const int d4 = tl.d / 4;
    for (int w = tid; w < tl.layers * d4; w += kTailThreads) {
      const int l = w / d4, c = (w - l * d4) * 4;
      float* base = tl.aan_sum + (size_t)l * tl.layer_stride + (size_t)b * beam * tl.d + c;
      float4 old[MAXB];
#pragma unroll
      for (int q = 0; q < MAXB; ++q) old[q] = *reinterpret_cast<const float4*>(base + (size_t)min(q, beam - 1) * tl.d);
#pragma unroll
      for (int q = 0; q < MAXB; ++q) {
        if (q < beam && pl[q] != q) {
          float4 v = old[0];
#pragma unroll
          for (int s = 1; s < MAXB; ++s)
            if (s == pl[q]) v = old[s];
          *reinterpret_cast<float4*>(base + (size_t)q * tl.d) = v;
        }
      }
    }
  }
  if (tl.emb && t_now < tl.max_t) {
    const T* emb = reinterpret_cast<const T*>(tl.emb);
    T* x = reinterpret_cast<T*>(tl.x);
    const float* pp = tl.pe + (size_t)t_now * tl.d;
    const int d4 = tl.d / 4;
    for (int w = tid; w < beam * d4; w += kTailThreads) {
      const int q = w / d4, c = (w - q * d4) * 4;
      const int id = min(max(s_tok[q], 0), vocab - 1);
      const float4 ev = load4(emb + (size_t)id * tl.d + c);
      const float4 pv = *reinterpret_cast<const float4*>(pp + c);
      store4(x + (size_t)(b * beam + q) * tl.d + c,
             make_float4(fmaf(ev.x, tl.scale, pv.x), fmaf(ev.y, tl.scale, pv.y), fmaf(ev.z, tl.scale, pv.z),
                         fmaf(ev.w, tl.scale, pv.w)));
    }
    if (tid < beam) {
      const int r = b * beam + tid;
      last_tok[r] = s_tok[tid];
      // the new position of every row is its own; written after the permutation above, which
      // only touches columns < t_now
      tl.anc[(size_t)r * tl.ld_anc + t_now] = r;
    }
  }
}

template <typename T>
static void launch_tail_t(int batch, int beam, hipStream_t stream, const float* cand_lp, const int* cand_idx,
                          const float* cum, int vocab, int* out_tok, int* out_parent, float* out_score,
                          const TopkHistory& h, int eos_id, int* done, int* done_count, const BeamTail& tl, int* last_tok) {
#define SAN_TAIL(MB)                                                                                              \
  hipLaunchKernelGGL((beam_tail_kernel<T, MB>), dim3(batch), dim3(kTailThreads), 0, stream, cand_lp, cand_idx, cum, beam, \
                     vocab, out_tok, out_parent, out_score, h, eos_id, done, done_count, tl, last_tok)
  if (beam <= 4) SAN_TAIL(4);
  else if (beam <= 8) SAN_TAIL(8);
  else if (beam <= 16) SAN_TAIL(16);
  else SAN_TAIL(32);
#undef SAN_TAIL
}

// the per-sentence stage: plain merge, or the merge inside the beam tail
static hipError_t launch_merge(const float* cum, int eos_id, int batch, int beam, int vocab, int k, float* cand_lp,
                               int* cand_idx, int* out_tok, int* out_parent, float* out_score, hipStream_t stream,
                               const TopkHistory* hist, int* done, int* done_count, const BeamTail* tail,
                               int* last_tok_out) {
  TopkHistory h{};
  if (hist) h = *hist;
  if (tail) {
    if (tail->dtype == 1)
      launch_tail_t<bf16_t>(batch, beam, stream, cand_lp, cand_idx, cum, vocab, out_tok, out_parent, out_score, h, eos_id,
                            done_count ? done : nullptr, done_count, *tail, last_tok_out);
    else
      launch_tail_t<float>(batch, beam, stream, cand_lp, cand_idx, cum, vocab, out_tok, out_parent, out_score, h, eos_id,
                           done_count ? done : nullptr, done_count, *tail, last_tok_out);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(topk_merge_kernel, dim3(batch), dim3(64), 0, stream, cand_lp, cand_idx, cum, beam, vocab, k,
                     out_tok, out_parent, out_score, h, eos_id, done_count ? done : nullptr, done_count);
  return hipGetLastError();
}

static bool tail_ok(const BeamTail* tail, int beam, int k, const int* last_tok_out) {
  return !tail || !(k != beam || beam > kMaxK || (tail->emb && (!tail->anc || !last_tok_out || tail->d % 4)));
}

hipError_t launch_topk(const float* logits, const float* cum, const int* last_tok, int eos_id, int batch, int beam,
                       int vocab, int k, float* cand_lp, int* cand_idx, int* out_tok, int* out_parent,
                       float* out_score, hipStream_t stream, const TopkHistory* hist, int* done, int* done_count,
                       const BeamTail* tail, int* last_tok_out) {
  const int rows = batch * beam;
  if (!tail_ok(tail, beam, k, last_tok_out)) return hipErrorInvalidValue;
  if (rows <= 0) return hipSuccess;
  if (vocab <= kTopkVpt * kTopkThreads)
    hipLaunchKernelGGL(topk_row_kernel<true>, dim3(rows), dim3(kTopkThreads), 0, stream, logits, last_tok, eos_id,
                       vocab, k, cand_lp, cand_idx);
  else
    hipLaunchKernelGGL(topk_row_kernel<false>, dim3(rows), dim3(kTopkThreads), 0, stream, logits, last_tok, eos_id,
                       vocab, k, cand_lp, cand_idx);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_merge(cum, eos_id, batch, beam, vocab, k, cand_lp, cand_idx, out_tok, out_parent, out_score, stream, hist,
                      done, done_count, tail, last_tok_out);
}

bool topk_cands_fit(int ntiles, int k) { return k >= 1 && ntiles >= 1 && (long)ntiles * 2 * k <= 20L * kCombThreads; }

hipError_t launch_topk_cands(const float* ms, const float* cv, const int* ci, int ntiles, const float* cum,
                             const int* last_tok, int eos_id, int batch, int beam, int vocab, int k, float* cand_lp,
                             int* cand_idx, int* out_tok, int* out_parent, float* out_score, hipStream_t stream,
                             const TopkHistory* hist, int* done, int* done_count, const BeamTail* tail,
                             int* last_tok_out) {
  const int rows = batch * beam;
  if (!tail_ok(tail, beam, k, last_tok_out) || !topk_cands_fit(ntiles, k) || k > kMaxK) return hipErrorInvalidValue;
  if (rows <= 0) return hipSuccess;
  const int nc = ntiles * 2 * k;
#define SAN_COMB(CPT)                                                                                              \
  hipLaunchKernelGGL(cand_combine_kernel<CPT>, dim3(rows), dim3(kCombThreads), 0, stream, ms, cv, ci, ntiles, last_tok, \
                     eos_id, k, cand_lp, cand_idx)
  if (nc <= 2 * kCombThreads) SAN_COMB(2);
  else if (nc <= 4 * kCombThreads) SAN_COMB(4);
  else if (nc <= 8 * kCombThreads) SAN_COMB(8);
  else SAN_COMB(20);
#undef SAN_COMB
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_merge(cum, eos_id, batch, beam, vocab, k, cand_lp, cand_idx, out_tok, out_parent, out_score, stream, hist,
                      done, done_count, tail, last_tok_out);
}

}  // namespace san
