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

// (max, sum of exp(x - max)) pairs combine associatively, so the log-sum-exp needs
// a single exchange across the block.
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

  float reg[REG ? kTopkVpt : 1];
  if (REG) {
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) {
      const int idx = it * kTopkThreads + tid;
      reg[it] = (it < nit && idx < vocab) ? x[idx] : -INFINITY;
    }
  }
  auto val = [&](int it) -> float {
    if (REG) return reg[it];
    const int idx = it * kTopkThreads + tid;
    return idx < vocab ? x[idx] : -INFINITY;
  };

  // ---- log-sum-exp of the row
  float m = -INFINITY, s = 0.f;
  if (REG) {
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) m = fmaxf(m, reg[it]);
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) s += (reg[it] == -INFINITY) ? 0.f : __expf(reg[it] - m);
  } else {
    for (int it = 0; it < nit; ++it) m = fmaxf(m, val(it));
    for (int it = 0; it < nit; ++it) {
      const float v = val(it);
      s += (v == -INFINITY) ? 0.f : expf(v - m);
    }
  }
#pragma unroll
  for (int st = 1; st < kWave; st <<= 1) {
    const float om = __shfl_xor(m, st, kWave), os = __shfl_xor(s, st, kWave);
    lse_merge(m, s, om, os);
  }
  if (lane == 0) { red_m[wid] = m; red_s[wid] = s; }

  const bool finished = eos_id >= 0 && last_tok[row] == eos_id;
  if (REG) {
    // ---- threshold pass.  The k-th largest of the per-thread maxima is a lower
    // bound T on the k-th largest element, so every element of the row's top k is
    // >= T, and usually only a handful of elements are.  Those go to a short list in
    // LDS that wave 0 orders; a list overflow (masses of equal values) falls back to
    // the general rounds below.
    float tmax = -INFINITY;
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) tmax = fmaxf(tmax, reg[it]);
    {
      // each wave's k largest thread maxima (k rounds of "largest below the previous", by value and lane)
      float pv = INFINITY;
      int pl = -1;
      for (int round = 0; round < k; ++round) {
        const bool after = (tmax < pv) || (tmax == pv && lane > pl);
        Cand best = {after ? tmax : -INFINITY, after ? lane : 0x7fffffff};
        best = wave_best(best);
        if (lane == 0) wc_v[wid * k + round] = best.v;
        pv = best.v;
        pl = best.i;
      }
    }
    if (tid == 0) list_n = 0;
    __syncthreads();
    if (wid == 0) {
      // k-th largest of the NW * k wave values (duplicates count)
      const int nc = NW * k;
      float pv = INFINITY;
      int pc = -1;
      for (int round = 0; round < k; ++round) {
        Cand best = {-INFINITY, 0x7fffffff};
        for (int c = lane; c < nc; c += kWave) {
          const float v = wc_v[c];
          const bool after = (v < pv) || (v == pv && c > pc);
          if (after && better(v, c, best.v, best.i)) { best.v = v; best.i = c; }
        }
        best = wave_best(best);
        pv = best.v;
        pc = best.i;
      }
      if (lane == 0) thresh = pv;
    }
    __syncthreads();
    const float T = thresh;
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) {
      const int idx = it * kTopkThreads + tid;
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
      Cand best = {-INFINITY, 0x7fffffff};
      if (REG) {
#pragma unroll
        for (int it = 0; it < kTopkVpt; ++it) {
          const int idx = it * kTopkThreads + tid;
          const float v = reg[it];
          const bool after = (v < pv) || (v == pv && idx > pi);
          if (idx < vocab && after && better(v, idx, best.v, best.i)) { best.v = v; best.i = idx; }
        }
      } else {
        for (int it = 0; it < nit; ++it) {
          const int idx = it * kTopkThreads + tid;
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

  m = red_m[0];
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
  float pv = INFINITY;
  int pi = -1;
  for (int round = 0; round < k; ++round) {
    Cand best = {-INFINITY, 0x7fffffff};
    for (int c = lane; c < nc; c += kWave) {
      const float v = cv[c];
      const int idx = ci[c];
      const bool after = (v < pv) || (v == pv && idx > pi);
      if (idx != 0x7fffffff && after && better(v, idx, best.v, best.i)) { best.v = v; best.i = idx; }
    }
    best = wave_best(best);
    if (lane == 0) {
      cand_lp[(size_t)row * k + round] = best.v - lse;
      cand_idx[(size_t)row * k + round] = best.i;
    }
    pv = best.v;
    pi = best.i;
  }
}

// One wave per sentence: merge the beam*k candidates, keep the k best.
__global__ __launch_bounds__(64) void topk_merge_kernel(const float* cand_lp, const int* cand_idx, const float* cum,
                                                        int beam, int vocab, int k, int* out_tok, int* out_parent,
                                                        float* out_score, TopkHistory hist) {
  const int b = blockIdx.x, lane = threadIdx.x;
  // multi-step decoding: this step's picks are also appended to the caller's
  // [step][rows] arrays; the step index comes from the device-side counters
  const long long hoff = hist.tok ? (long long)(*hist.t_dev - 1 - *hist.t0_dev) * gridDim.x * k : 0;
  const int nc = beam * k;
  float pv = INFINITY;
  int pi = -1;
  for (int round = 0; round < k; ++round) {
    Cand best = {-INFINITY, 0x7fffffff};
    for (int cidx = lane; cidx < nc; cidx += kWave) {
      const int bi = cidx / k;
      const int r = b * beam + bi;
      const float sc = cum[r] + cand_lp[(size_t)r * k + (cidx % k)];
      const int flat = bi * vocab + cand_idx[(size_t)r * k + (cidx % k)];
      const bool after = (sc < pv) || (sc == pv && flat > pi);
      if (after && better(sc, flat, best.v, best.i)) { best.v = sc; best.i = flat; }
    }
    best = wave_best(best);
    if (lane == 0) {
      const bool ok = best.i != 0x7fffffff;
      const int tk = ok ? best.i % vocab : 0, pr = b * beam + (ok ? best.i / vocab : 0);
      out_tok[(size_t)b * k + round] = tk;
      out_parent[(size_t)b * k + round] = pr;
      out_score[(size_t)b * k + round] = ok ? best.v : -INFINITY;
      if (hist.tok) {
        hist.tok[hoff + (size_t)b * k + round] = tk;
        hist.par[hoff + (size_t)b * k + round] = pr;
      }
    }
    pv = best.v;
    pi = best.i;
  }
}

hipError_t launch_topk(const float* logits, const float* cum, const int* last_tok, int eos_id, int batch, int beam,
                       int vocab, int k, float* cand_lp, int* cand_idx, int* out_tok, int* out_parent,
                       float* out_score, hipStream_t stream, const TopkHistory* hist) {
  const int rows = batch * beam;
  if (rows <= 0) return hipSuccess;
  if (vocab <= kTopkVpt * kTopkThreads)
    hipLaunchKernelGGL(topk_row_kernel<true>, dim3(rows), dim3(kTopkThreads), 0, stream, logits, last_tok, eos_id,
                       vocab, k, cand_lp, cand_idx);
  else
    hipLaunchKernelGGL(topk_row_kernel<false>, dim3(rows), dim3(kTopkThreads), 0, stream, logits, last_tok, eos_id,
                       vocab, k, cand_lp, cand_idx);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  TopkHistory h{};
  if (hist) h = *hist;
  hipLaunchKernelGGL(topk_merge_kernel, dim3(batch), dim3(64), 0, stream, cand_lp, cand_idx, cum, beam, vocab, k,
                     out_tok, out_parent, out_score, h);
  return hipGetLastError();
}

}  // namespace san
