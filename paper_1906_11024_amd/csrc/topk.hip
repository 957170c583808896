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
__device__ __forceinline__ Cand wave_best(Cand c) {
#pragma unroll
  for (int s = 1; s < kWave; s <<= 1) {
    const float ov = __shfl_xor(c.v, s, kWave);
    const int oi = __shfl_xor(c.i, s, kWave);
    if (better(ov, oi, c.v, c.i)) { c.v = ov; c.i = oi; }
  }
  return c;
}

template <bool REG>
__global__ __launch_bounds__(kTopkThreads) void topk_row_kernel(const float* logits, const int* last_tok,
                                                                int eos_id, int vocab, int k, float* cand_lp,
                                                                int* cand_idx) {
  __shared__ float red_v[kTopkThreads / kWave];
  __shared__ int red_i[kTopkThreads / kWave];
  __shared__ float bc_v;
  __shared__ int bc_i;
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const float* x = logits + (size_t)row * vocab;
  constexpr int NW = kTopkThreads / kWave;
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

  // ---- max and log-sum-exp
  float m = -INFINITY;
  if (REG) {
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) m = fmaxf(m, reg[it]);
  } else {
    for (int it = 0; it < nit; ++it) m = fmaxf(m, val(it));
  }
  m = wave_max(m);
  if (lane == 0) red_v[wid] = m;
  __syncthreads();
  m = red_v[0];
  for (int w = 1; w < NW; ++w) m = fmaxf(m, red_v[w]);
  __syncthreads();
  float s = 0.f;
  if (REG) {
#pragma unroll
    for (int it = 0; it < kTopkVpt; ++it) s += (reg[it] == -INFINITY) ? 0.f : expf(reg[it] - m);
  } else {
    for (int it = 0; it < nit; ++it) {
      const float v = val(it);
      s += (v == -INFINITY) ? 0.f : expf(v - m);
    }
  }
  s = wave_sum(s);
  if (lane == 0) red_v[wid] = s;
  __syncthreads();
  s = 0.f;
  for (int w = 0; w < NW; ++w) s += red_v[w];
  __syncthreads();
  const float lse = m + logf(s);

  // ---- a finished hypothesis can only be extended by EOS at cost 0
  if (eos_id >= 0 && last_tok[row] == eos_id) {
    if (tid < k) {
      int id = tid == 0 ? eos_id : (tid - 1 < eos_id ? tid - 1 : tid);
      cand_lp[(size_t)row * k + tid] = tid == 0 ? 0.f : -INFINITY;
      cand_idx[(size_t)row * k + tid] = id;
    }
    return;
  }

  // ---- k rounds: best element strictly after the previous pick in the order
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
    if (lane == 0) { red_v[wid] = best.v; red_i[wid] = best.i; }
    __syncthreads();
    if (wid == 0) {
      Cand c = {lane < NW ? red_v[lane] : -INFINITY, lane < NW ? red_i[lane] : 0x7fffffff};
      c = wave_best(c);
      if (lane == 0) {
        bc_v = c.v;
        bc_i = c.i;
        cand_lp[(size_t)row * k + round] = c.v - lse;
        cand_idx[(size_t)row * k + round] = c.i;
      }
    }
    __syncthreads();
    pv = bc_v;
    pi = bc_i;
    __syncthreads();
  }
}

// One wave per sentence: merge the beam*k candidates, keep the k best.
__global__ __launch_bounds__(64) void topk_merge_kernel(const float* cand_lp, const int* cand_idx, const float* cum,
                                                        int beam, int vocab, int k, int* out_tok, int* out_parent,
                                                        float* out_score) {
  const int b = blockIdx.x, lane = threadIdx.x;
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
      out_tok[(size_t)b * k + round] = ok ? best.i % vocab : 0;
      out_parent[(size_t)b * k + round] = b * beam + (ok ? best.i / vocab : 0);
      out_score[(size_t)b * k + round] = ok ? best.v : -INFINITY;
    }
    pv = best.v;
    pi = best.i;
  }
}

hipError_t launch_topk(const float* logits, const float* cum, const int* last_tok, int eos_id, int batch, int beam,
                       int vocab, int k, float* cand_lp, int* cand_idx, int* out_tok, int* out_parent,
                       float* out_score, hipStream_t stream) {
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
  hipLaunchKernelGGL(topk_merge_kernel, dim3(batch), dim3(64), 0, stream, cand_lp, cand_idx, cum, beam, vocab, k,
                     out_tok, out_parent, out_score);
  return hipGetLastError();
}

}  // namespace san
