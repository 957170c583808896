// Row-wise kernels of the decoder step: embedding, split-K reduce + bias +
// residual + LayerNorm, the average-attention (AAN) pre/post stages, beam-state
// reordering and small utilities.  All are bandwidth-trivial; they exist to keep
// the number of passes over the [rows][d] activations small.
#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace san {

// The average-attention layer's running sum, mean and gate-input copy for 4 columns of row m
// (x = the values just stored for the layer input, rounded to the storage type like a reader
// of x would see them).
template <typename T>
__device__ __forceinline__ void aan_accumulate(const AanFuse& a, int m, int c, int d, float4 x) {
  const float4 xv = make_float4(to_f32(from_f32<T>(x.x)), to_f32(from_f32<T>(x.y)), to_f32(from_f32<T>(x.z)),
                                to_f32(from_f32<T>(x.w)));
  const int t = *a.t_dev;
  float* sp = a.sum + (size_t)m * d + c;
  float4 s = (t == 0) ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4*>(sp);
  s = make_float4(s.x + xv.x, s.y + xv.y, s.z + xv.z, s.w + xv.w);
  *reinterpret_cast<float4*>(sp) = s;
  const float inv = 1.0f / (float)(t + 1);
  store4(reinterpret_cast<T*>(a.avg) + (size_t)m * d + c, make_float4(s.x * inv, s.y * inv, s.z * inv, s.w * inv));
  store4(reinterpret_cast<T*>(a.cat) + (size_t)m * 2 * d + c, xv);
}

// ---------------------------------------------------------------- embedding
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const int* tok, int tok_stride, int rpg, const T* emb,
                                                    const float* pe, const int* t_dev, T* x, int rows, int d,
                                                    int vocab, float scale, int* last_tok, int* anc, int ld_anc,
                                                    AanFuse aan) {
  const int r = blockIdx.x;
  if (r >= rows) return;
  const int hyp = r / rpg, i = r % rpg;
  int id = tok[(size_t)hyp * tok_stride + i];
  const int pos = t_dev ? *t_dev : i;
  if (threadIdx.x == 0) {
    if (last_tok) last_tok[r] = id;
    if (anc && pos < ld_anc) anc[(size_t)r * ld_anc + pos] = r;
  }
  id = min(max(id, 0), vocab - 1);
  const T* e = emb + (size_t)id * d;
  const float* pp = pe + (size_t)pos * d;
  for (int c = threadIdx.x * 4; c < d; c += blockDim.x * 4) {
    const float4 ev = load4(e + c);
    const float4 pv = *reinterpret_cast<const float4*>(pp + c);
    const float4 xv = make_float4(fmaf(ev.x, scale, pv.x), fmaf(ev.y, scale, pv.y), fmaf(ev.z, scale, pv.z),
                                  fmaf(ev.w, scale, pv.w));
    store4(x + (size_t)r * d + c, xv);
    if (aan.sum) aan_accumulate<T>(aan, r, c, d, xv);
  }
}

hipError_t launch_embed(int dtype, const int* tok, int tok_stride, int rpg, const void* emb, const float* pe,
                        const int* t_dev, void* x, int rows, int d, int vocab, float scale, int* last_tok,
                        int* anc, int ld_anc, hipStream_t stream, const AanFuse* aan) {
  if (rows <= 0) return hipSuccess;
  AanFuse af{};
  if (aan) af = *aan;
  if (af.sum && (!t_dev || rpg != 1)) return hipErrorInvalidValue;   // cached decoding only
  const int threads = d / 4 >= 256 ? 256 : (d / 4 >= 128 ? 128 : 64);
  if (dtype == 1)
    hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(rows), dim3(threads), 0, stream, tok, tok_stride, rpg,
                       (const bf16_t*)emb, pe, t_dev, (bf16_t*)x, rows, d, vocab, scale, last_tok, anc, ld_anc, af);
  else
    hipLaunchKernelGGL(embed_kernel<float>, dim3(rows), dim3(threads), 0, stream, tok, tok_stride, rpg,
                       (const float*)emb, pe, t_dev, (float*)x, rows, d, vocab, scale, last_tok, anc, ld_anc, af);
  return hipGetLastError();
}

// ------------------------------------------- reduce + bias + residual + LayerNorm
// One block per row, one 4-column group per thread (n / 4 threads, up to 8
// waves): every load of the row is issued at once, so the kernel costs a single
// memory round trip whatever the row width.  Row statistics: wave reduction, then
// the per-wave values are added in wave order through LDS (deterministic).
constexpr int kLnMaxWaves = 8;  // n <= 8 * 256 = 2048 columns

// sum of `x` over the whole block; `slot` is an LDS array of kLnMaxWaves floats used for this reduction only
__device__ __forceinline__ float block_sum(float x, float* slot, int wid, int lane, int nwaves) {
  x = wave_sum(x);
  if (lane == 0) slot[wid] = x;
  __syncthreads();
  float total = 0.f;
  for (int w = 0; w < nwaves; ++w) total += slot[w];
  return total;
}

// LayerNorm of a row held as one float4 per thread (threads past the row hold zeros and are inactive)
__device__ __forceinline__ float4 layer_norm_vec(float4 v, bool active, int n, float4 g, float4 b, float eps,
                                                 float* slots, int wid, int lane, int nwaves) {
  const float s = active ? (v.x + v.y) + (v.z + v.w) : 0.f;
  const float mean = block_sum(s, slots, wid, lane, nwaves) / (float)n;
  float q = 0.f;
  if (active) {
    const float d0 = v.x - mean, d1 = v.y - mean, d2 = v.z - mean, d3 = v.w - mean;
    q = fmaf(d0, d0, fmaf(d1, d1, fmaf(d2, d2, d3 * d3)));
  }
  const float rstd = 1.0f / sqrtf(block_sum(q, slots + kLnMaxWaves, wid, lane, nwaves) / (float)n + eps);
  return make_float4((v.x - mean) * rstd * g.x + b.x, (v.y - mean) * rstd * g.y + b.y,
                     (v.z - mean) * rstd * g.z + b.z, (v.w - mean) * rstd * g.w + b.w);
}

// bias + residual + the NS partials of one 4-column group.  Every load is
// unconditional and issued before the first use (a load behind a branch is waited
// for on the spot, and each such wait is a memory round trip): absent operands
// are read from `safe`, a valid address, and dropped by a select.
template <typename T, int NS>
__device__ __forceinline__ float4 gather_fixed(const float* part, size_t split_stride, const T* bias, const T* res,
                                               const T* safe) {
  const float4 bv = load4(bias ? bias : safe);
  const float4 rv = load4(res ? res : safe);
  float4 pv[NS];
#pragma unroll
  for (int u = 0; u < NS; ++u) pv[u] = *reinterpret_cast<const float4*>(part + (size_t)u * split_stride);
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  if (bias) a = bv;
  if (res) { a.x += rv.x; a.y += rv.y; a.z += rv.z; a.w += rv.w; }
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int u = 0; u < NS; ++u) { sum.x += pv[u].x; sum.y += pv[u].y; sum.z += pv[u].z; sum.w += pv[u].w; }
  return make_float4(sum.x + a.x, sum.y + a.y, sum.z + a.z, sum.w + a.w);
}
// the split factors the GEMM launcher produces are powers of two up to 16; anything else takes the loop
template <typename T>
__device__ __forceinline__ float4 gather_update(const float* part, int nsplit, size_t split_stride, const T* bias,
                                                const T* res, const T* safe) {
  switch (nsplit) {
    case 1: return gather_fixed<T, 1>(part, split_stride, bias, res, safe);
    case 2: return gather_fixed<T, 2>(part, split_stride, bias, res, safe);
    case 4: return gather_fixed<T, 4>(part, split_stride, bias, res, safe);
    case 8: return gather_fixed<T, 8>(part, split_stride, bias, res, safe);
    case 16: return gather_fixed<T, 16>(part, split_stride, bias, res, safe);
    default: break;
  }
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  if (bias) a = load4(bias);
  if (res) {
    const float4 rv = load4(res);
    a.x += rv.x; a.y += rv.y; a.z += rv.z; a.w += rv.w;
  }
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < nsplit; ++s) {
    const float4 pv = *reinterpret_cast<const float4*>(part + (size_t)s * split_stride);
    sum.x += pv.x; sum.y += pv.y; sum.z += pv.z; sum.w += pv.w;
  }
  return make_float4(sum.x + a.x, sum.y + a.y, sum.z + a.z, sum.w + a.w);
}

template <typename T>
__global__ __launch_bounds__(kLnMaxWaves * 64) void ln_reduce_kernel(const float* part, int nsplit, int ldp,
                                                                     const T* bias, const T* res, int ldr,
                                                                     const T* gamma, const T* beta, T* out, int ldo,
                                                                     float* out_f32, int M, int n, float eps,
                                                                     LnStage2 s2, AanFuse aan) {
  __shared__ float slots[4 * kLnMaxWaves];
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int m = blockIdx.x;
  const int c = threadIdx.x * 4;
  const bool active = c < n;
  const int cc = active ? c : 0;   // inactive threads load column 0 and drop it
  const float4 g1 = load4(gamma + cc), b1 = load4(beta + cc);
  float4 g2 = g1, b2 = b1, u2 = make_float4(0.f, 0.f, 0.f, 0.f);
  if (s2.part) {
    g2 = load4(reinterpret_cast<const T*>(s2.gamma) + cc);
    b2 = load4(reinterpret_cast<const T*>(s2.beta) + cc);
    u2 = gather_update<T>(s2.part + (size_t)m * s2.ldp + cc, s2.nsplit, (size_t)M * s2.ldp,
                          reinterpret_cast<const T*>(s2.bias) + cc, (const T*)nullptr, gamma + cc);
  }
  const float4 v = gather_update<T>(part + (size_t)m * ldp + cc, nsplit, (size_t)M * ldp, bias ? bias + cc : nullptr,
                                    res ? res + (size_t)m * ldr + cc : nullptr, gamma + cc);
  float4 y = layer_norm_vec(v, active, n, g1, b1, eps, slots, wid, lane, nwaves);
  if (s2.part) {
    // second sub-layer without a GEMM of its own in between (an enc-dec follower
    // whose projected context was computed at the block head): add the second
    // update to the first LayerNorm's output and normalise again.  That output was
    // rounded to the storage type when it was a separate launch; keep the rounding
    // so both forms give the same bits.
    const float4 y1 = make_float4(to_f32(from_f32<T>(y.x)) + u2.x, to_f32(from_f32<T>(y.y)) + u2.y,
                                  to_f32(from_f32<T>(y.z)) + u2.z, to_f32(from_f32<T>(y.w)) + u2.w);
    y = layer_norm_vec(y1, active, n, g2, b2, eps, slots + 2 * kLnMaxWaves, wid, lane, nwaves);
  }
  if (active) {
    store4(out + (size_t)m * ldo + c, y);
    if (out_f32) *reinterpret_cast<float4*>(out_f32 + (size_t)m * n + c) = y;
    if (aan.sum) aan_accumulate<T>(aan, m, c, n, y);   // the next layer is an average-attention layer
  }
}

hipError_t launch_ln_reduce(int dtype, const float* part, int nsplit, int ldp, const void* bias, const void* res, int ldr,
                            const void* gamma, const void* beta, void* out, int ldo, float* out_f32, int M, int n,
                            float eps, hipStream_t stream, const LnStage2* stage2, const AanFuse* aan) {
  if (M <= 0) return hipSuccess;
  if (n <= 0 || n > kLnMaxWaves * 256 || n % 4) return hipErrorInvalidValue;
  LnStage2 s2{};
  if (stage2) s2 = *stage2;
  AanFuse af{};
  if (aan) af = *aan;
  dim3 grid(M), block(64 * ((n / 4 + 63) / 64));
  if (dtype == 1)
    hipLaunchKernelGGL(ln_reduce_kernel<bf16_t>, grid, block, 0, stream, part, nsplit, ldp, (const bf16_t*)bias,
                       (const bf16_t*)res, ldr, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)out, ldo,
                       out_f32, M, n, eps, s2, af);
  else
    hipLaunchKernelGGL(ln_reduce_kernel<float>, grid, block, 0, stream, part, nsplit, ldp, (const float*)bias,
                       (const float*)res, ldr, (const float*)gamma, (const float*)beta, (float*)out, ldo, out_f32,
                       M, n, eps, s2, af);
  return hipGetLastError();
}

// -------------------------------------------------------------- step bookkeeping
__global__ void step_begin_kernel(const int* tok, int* last_tok, int* anc, int* hist, int ld, const int* t_dev,
                                  int rows) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  const int t = *t_dev;
  const int id = tok[r];
  last_tok[r] = id;
  if (t < ld) {
    if (anc) anc[(size_t)r * ld + t] = r;
    if (hist) hist[(size_t)r * ld + t] = id;
  }
}
hipError_t launch_step_begin(const int* tok, int* last_tok, int* anc, int* hist, int ld, const int* t_dev, int rows,
                             hipStream_t stream) {
  hipLaunchKernelGGL(step_begin_kernel, dim3((rows + 255) / 256), dim3(256), 0, stream, tok, last_tok, anc, hist,
                     ld, t_dev, rows);
  return hipGetLastError();
}

template <typename T> __global__ void to_f32_kernel(const T* src, int lds, float* dst, int rows, int cols) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)rows * cols) return;
  const int r = (int)(i / cols), c = (int)(i % cols);
  dst[i] = to_f32(src[(size_t)r * lds + c]);
}
hipError_t launch_to_f32(int dtype, const void* src, int lds, float* dst, int rows, int cols, hipStream_t stream) {
  const size_t total = (size_t)rows * cols;
  if (!total) return hipSuccess;
  dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == 1)
    hipLaunchKernelGGL(to_f32_kernel<bf16_t>, grid, dim3(256), 0, stream, (const bf16_t*)src, lds, dst, rows, cols);
  else
    hipLaunchKernelGGL(to_f32_kernel<float>, grid, dim3(256), 0, stream, (const float*)src, lds, dst, rows, cols);
  return hipGetLastError();
}

__global__ void compact_S_kernel(const float* src, int ldS, float* dst, int rows_h, int n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)rows_h * n) return;
  dst[i] = src[(i / n) * ldS + (i % n)];
}
hipError_t launch_compact_S(const float* src, int ldS, float* dst, int rows_h, int n, hipStream_t stream) {
  const size_t total = (size_t)rows_h * n;
  if (!total) return hipSuccess;
  hipLaunchKernelGGL(compact_S_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, src, ldS, dst,
                     rows_h, n);
  return hipGetLastError();
}

// ----------------------------------------------------------------- AAN stages
// (cached decoding: the running sum and mean are produced by aan_accumulate above, inside the
// launch that writes the layer input)
// Nothing cached: the mean over positions 0..i of every position i of every hypothesis
// (x is [hyps][np][d]); a thread owns 4 columns of one hypothesis and walks its positions,
// adding in the order and precision of the running sum above.
template <typename T>
__global__ __launch_bounds__(256) void aan_prefix_mean_kernel(const T* x, T* avg, T* cat, int hyps, int np, int d) {
  const size_t i4 = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i4 >= (size_t)hyps * d) return;
  const int b = (int)(i4 / d), c = (int)(i4 % d);
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int i = 0; i < np; ++i) {
    const size_t row = (size_t)b * np + i;
    const float4 xv = load4(x + row * d + c);
    s.x += xv.x; s.y += xv.y; s.z += xv.z; s.w += xv.w;
    const float inv = 1.0f / (float)(i + 1);
    store4(avg + row * d + c, make_float4(s.x * inv, s.y * inv, s.z * inv, s.w * inv));
    store4(cat + row * 2 * d + c, xv);
  }
}
hipError_t launch_aan_prefix_mean(int dtype, const void* x, void* avg, void* cat, int hyps, int np, int d,
                                  hipStream_t stream) {
  const size_t total = (size_t)hyps * d / 4;
  if (!total || np <= 0) return hipSuccess;
  dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == 1)
    hipLaunchKernelGGL(aan_prefix_mean_kernel<bf16_t>, grid, dim3(256), 0, stream, (const bf16_t*)x, (bf16_t*)avg,
                       (bf16_t*)cat, hyps, np, d);
  else
    hipLaunchKernelGGL(aan_prefix_mean_kernel<float>, grid, dim3(256), 0, stream, (const float*)x, (float*)avg,
                       (float*)cat, hyps, np, d);
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(kLnMaxWaves * 64) void aan_post_kernel(const float* z, const T* bg, const T* cat,
                                                                    const T* gamma, const T* beta, T* x,
                                                                    float* out_f32, int rows, int d, float eps) {
  // one block per row, one 4-column group per thread (as the LayerNorm kernel above)
  __shared__ float slots[2 * kLnMaxWaves];
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int m = blockIdx.x;
  const int c = threadIdx.x * 4;
  const bool active = c < d;
  const int cc = active ? c : 0;
  const float4 g = load4(gamma + cc), b = load4(beta + cc);
  const float4 zi = *reinterpret_cast<const float4*>(z + (size_t)m * 2 * d + cc);
  const float4 zf = *reinterpret_cast<const float4*>(z + (size_t)m * 2 * d + d + cc);
  const float4 bi = load4(bg + cc), bf = load4(bg + d + cc);
  const float4 xv = load4(cat + (size_t)m * 2 * d + cc);
  const float4 gv = load4(cat + (size_t)m * 2 * d + d + cc);
  const float zia[4] = {zi.x + bi.x, zi.y + bi.y, zi.z + bi.z, zi.w + bi.w};
  const float zfa[4] = {zf.x + bf.x, zf.y + bf.y, zf.z + bf.z, zf.w + bf.w};
  const float xa[4] = {xv.x, xv.y, xv.z, xv.w}, ga[4] = {gv.x, gv.y, gv.z, gv.w};
  float v[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float ig = 1.0f / (1.0f + expf(-zia[e]));
    const float fg = 1.0f / (1.0f + expf(-zfa[e]));
    v[e] = xa[e] + ig * xa[e] + fg * ga[e];
  }
  const float4 y = layer_norm_vec(make_float4(v[0], v[1], v[2], v[3]), active, d, g, b, eps, slots, wid, lane, nwaves);
  if (active) {
    store4(x + (size_t)m * d + c, y);
    if (out_f32) *reinterpret_cast<float4*>(out_f32 + (size_t)m * d + c) = y;
  }
}
hipError_t launch_aan_post(int dtype, const float* z, const void* bg, const void* cat, const void* gamma,
                           const void* beta, void* x, float* out_f32, int rows, int d, float eps,
                           hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  if (d <= 0 || d > kLnMaxWaves * 256 || d % 4) return hipErrorInvalidValue;
  dim3 grid(rows), block(64 * ((d / 4 + 63) / 64));
  if (dtype == 1)
    hipLaunchKernelGGL(aan_post_kernel<bf16_t>, grid, block, 0, stream, z, (const bf16_t*)bg,
                       (const bf16_t*)cat, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)x, out_f32, rows, d,
                       eps);
  else
    hipLaunchKernelGGL(aan_post_kernel<float>, grid, block, 0, stream, z, (const float*)bg, (const float*)cat,
                       (const float*)gamma, (const float*)beta, (float*)x, out_f32, rows, d, eps);
  return hipGetLastError();
}

// ------------------------------------------------------------ beam reordering
// A thread owns one column of one sentence: it reads that column of every old row
// of the sentence, then writes the permuted rows, so the update is safe in place.
constexpr int kMaxBeam = 32;

// MAXB = compile-time cap of the beam.  Every load (step counter, parents, the old
// entries; rows past the beam re-read the last one) goes out before anything is
// used, so the kernel costs one memory round trip.
template <int MAXB>
__global__ void reorder_table_kernel(int* tab, int ld, const int* parent, const int* t_dev, int batch, int beam,
                                     int max_t) {
  const int b = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= max_t) return;
  const int t = *t_dev;
  int pl[MAXB], old[MAXB];
#pragma unroll
  for (int k = 0; k < MAXB; ++k) pl[k] = parent[b * beam + min(k, beam - 1)] - b * beam;
#pragma unroll
  for (int k = 0; k < MAXB; ++k) old[k] = tab[(size_t)(b * beam + min(k, beam - 1)) * ld + j];
  if (j >= min(t, max_t)) return;
#pragma unroll
  for (int k = 0; k < MAXB; ++k) {
    if (k < beam && pl[k] >= 0 && pl[k] < beam && pl[k] != k) {
      int v = old[0];
#pragma unroll
      for (int q = 1; q < MAXB; ++q)
        if (q == pl[k]) v = old[q];
      tab[(size_t)(b * beam + k) * ld + j] = v;
    }
  }
}
hipError_t launch_reorder_table(int* tab, int ld, const int* parent, const int* t_dev, int batch, int beam,
                                int max_t, hipStream_t stream) {
  if (beam > kMaxBeam || beam < 1 || max_t > ld) return hipErrorInvalidValue;
  dim3 grid((max_t + 127) / 128, batch);
  if (beam <= 4)
    hipLaunchKernelGGL(reorder_table_kernel<4>, grid, dim3(128), 0, stream, tab, ld, parent, t_dev, batch, beam, max_t);
  else if (beam <= 8)
    hipLaunchKernelGGL(reorder_table_kernel<8>, grid, dim3(128), 0, stream, tab, ld, parent, t_dev, batch, beam, max_t);
  else if (beam <= 16)
    hipLaunchKernelGGL(reorder_table_kernel<16>, grid, dim3(128), 0, stream, tab, ld, parent, t_dev, batch, beam, max_t);
  else
    hipLaunchKernelGGL(reorder_table_kernel<32>, grid, dim3(128), 0, stream, tab, ld, parent, t_dev, batch, beam, max_t);
  return hipGetLastError();
}

// V = float4 (4 columns per thread) or float (1 column, for beams whose register copy would not fit otherwise)
template <int MAXB, typename V>
__global__ void reorder_rows_kernel(float* st, size_t layer_stride, const int* parent, int batch, int beam, int d) {
  constexpr int W = sizeof(V) / sizeof(float);
  const int b = blockIdx.y, l = blockIdx.z;
  const int c = (blockIdx.x * blockDim.x + threadIdx.x) * W;
  if (c >= d) return;
  float* base = st + (size_t)l * layer_stride + (size_t)b * beam * d + c;
  int pl[MAXB];
#pragma unroll
  for (int k = 0; k < MAXB; ++k)
    if (k < beam) pl[k] = parent[b * beam + k] - b * beam;
  V old[MAXB];
#pragma unroll
  for (int k = 0; k < MAXB; ++k)
    if (k < beam) old[k] = *reinterpret_cast<const V*>(base + (size_t)k * d);
#pragma unroll
  for (int k = 0; k < MAXB; ++k) {
    if (k < beam) {
      if (pl[k] >= 0 && pl[k] < beam && pl[k] != k) {
        V v = old[0];
#pragma unroll
        for (int q = 1; q < MAXB; ++q)
          if (q == pl[k]) v = old[q];
        *reinterpret_cast<V*>(base + (size_t)k * d) = v;
      }
    }
  }
}
hipError_t launch_reorder_rows(float* st, size_t layer_stride, const int* parent, int layers, int batch, int beam,
                               int d, hipStream_t stream) {
  if (beam > kMaxBeam || d % 4) return hipErrorInvalidValue;
  if (layers <= 0) return hipSuccess;
  const dim3 g4((d / 4 + 63) / 64, batch, layers), g1((d + 127) / 128, batch, layers);
  if (beam <= 4)
    hipLaunchKernelGGL((reorder_rows_kernel<4, float4>), g4, dim3(64), 0, stream, st, layer_stride, parent, batch, beam, d);
  else if (beam <= 8)
    hipLaunchKernelGGL((reorder_rows_kernel<8, float4>), g4, dim3(64), 0, stream, st, layer_stride, parent, batch, beam, d);
  else if (beam <= 16)
    hipLaunchKernelGGL((reorder_rows_kernel<16, float4>), g4, dim3(64), 0, stream, st, layer_stride, parent, batch, beam, d);
  else
    hipLaunchKernelGGL((reorder_rows_kernel<32, float>), g1, dim3(128), 0, stream, st, layer_stride, parent, batch, beam, d);
  return hipGetLastError();
}

// ---- dropping sentences from a running batch (rare, tiny: plain word copies)
__global__ __launch_bounds__(256) void gather_groups_kernel(int* __restrict__ dst, const int* __restrict__ src,
                                                            const int* __restrict__ keep, int rpg, int groups, int w) {
  const size_t per = (size_t)rpg * w, total = (size_t)groups * per;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const size_t g = i / per, rest = i - g * per;
    dst[i] = src[(size_t)keep[g] * per + rest];
  }
}
hipError_t launch_gather_groups(void* dst, const void* src, const int* keep, int rpg, int groups, int w,
                                hipStream_t stream) {
  const size_t total = (size_t)groups * rpg * w;
  if (total == 0) return hipSuccess;
  const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
  hipLaunchKernelGGL(gather_groups_kernel, dim3(blocks), dim3(256), 0, stream, reinterpret_cast<int*>(dst),
                     reinterpret_cast<const int*>(src), keep, rpg, groups, w);
  return hipGetLastError();
}

__global__ __launch_bounds__(64) void count_flags_kernel(const int* flags, int n, int* count) {
  int s = 0;
  for (int i = threadIdx.x; i < n; i += 64) s += flags[i] != 0;
  s = (int)wave_sum((float)s);   // exact: n is far below 2^24
  if (threadIdx.x == 0) *count = s;
}
hipError_t launch_count_flags(const int* flags, int n, int* count, hipStream_t stream) {
  hipLaunchKernelGGL(count_flags_kernel, dim3(1), dim3(64), 0, stream, flags, n, count);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_finished_kernel(int* tok, int* par, const int* from, int batch, int beam,
                                                            int steps, int eos) {
  const int rows = batch * beam;
  const size_t total = (size_t)steps * rows;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int s = (int)(i / rows), r = (int)(i - (size_t)s * rows);
    const int f = from[r / beam];
    if (f >= 0 && s >= f) { tok[i] = eos; par[i] = r; }
  }
}
hipError_t launch_fill_finished(int* tok, int* par, const int* from, int batch, int beam, int steps, int eos,
                                hipStream_t stream) {
  const size_t total = (size_t)steps * batch * beam;
  if (total == 0) return hipSuccess;
  const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
  hipLaunchKernelGGL(fill_finished_kernel, dim3(blocks), dim3(256), 0, stream, tok, par, from, batch, beam, steps, eos);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void scatter_words_kernel(int* dst, const int* src, const int* map, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[map[i]] = src[i];
}
hipError_t launch_scatter_words(void* dst, const void* src, const int* map, int n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(scatter_words_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, reinterpret_cast<int*>(dst),
                     reinterpret_cast<const int*>(src), map, n);
  return hipGetLastError();
}

// Plain streaming read of a buffer (16-byte loads, grid-stride, 8 in flight per
// thread): the yardstick the attention kernels' achieved bandwidth is set against.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16, unsigned* sink) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  unsigned acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const uint4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) *sink = acc;   // keeps the loads alive; practically never true
}
hipError_t launch_stream_read(const void* src, size_t bytes, unsigned* sink, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  hipLaunchKernelGGL(stream_read_kernel, dim3(2048), dim3(256), 0, stream, reinterpret_cast<const uint4*>(src), n16, sink);
  return hipGetLastError();
}

}  // namespace san
