// Learning a sharing policy (Sec. 3.3): Jensen-Shannon divergence between the
// attention weights of every pair of decoder layers, accumulated over decode
// steps on the device, and the host-side block search of Eq. 6.
#include "common.h"
#include "kernels.h"

namespace san {

// One wave per (row, head): JS(S_a[row,head,:], S_b[row,head,:]) over n keys.
__global__ __launch_bounds__(256) void js_pairs_kernel(JsParams p) {
  const int lane = threadIdx.x & 63;
  const int rh = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (rh >= p.rows * p.H) return;
  // pair index -> layers a < b
  int a = 0, rest = blockIdx.y;
  while (rest >= p.L - 1 - a) { rest -= p.L - 1 - a; ++a; }
  const int b = a + 1 + rest;
  const int row = rh / p.H;
  const int n = p.len ? max(0, min(p.len[row / p.rows_per_len], p.ld)) : min(p.n_fixed, p.ld);
  const float* pa = p.S[a] + (size_t)rh * p.ld;
  const float* pb = p.S[b] + (size_t)rh * p.ld;
  float acc = 0.f;
  if (pa != pb) {   // layers of one block share the buffer: divergence 0
    for (int j = lane; j < n; j += kWave) {
      const float x = pa[j], y = pb[j];
      const float m = 0.5f * (x + y);
      if (x > 0.f) acc += 0.5f * x * (logf(x) - logf(m));
      if (y > 0.f) acc += 0.5f * y * (logf(y) - logf(m));
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) p.part[(size_t)blockIdx.y * p.rows * p.H + rh] = acc;
}

// One block per pair: fixed-order sum of the per-(row, head) values, added to the
// running fp64 sums (both triangles of the matrix).
__global__ __launch_bounds__(256) void js_reduce_kernel(const float* part, int count, int L, double* acc) {
  __shared__ double red[256];
  const float* src = part + (size_t)blockIdx.x * count;
  double s = 0.0;
  for (int i = threadIdx.x; i < count; i += 256) s += (double)src[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    int a = 0, rest = blockIdx.x;
    while (rest >= L - 1 - a) { rest -= L - 1 - a; ++a; }
    const int b = a + 1 + rest;
    acc[a * L + b] += red[0];
    acc[b * L + a] += red[0];
  }
}

hipError_t launch_js_accumulate(const JsParams& p, double* acc, hipStream_t stream) {
  const int pairs = p.L * (p.L - 1) / 2;
  if (pairs <= 0 || p.rows <= 0) return hipSuccess;
  dim3 grid((p.rows * p.H + 3) / 4, pairs);
  hipLaunchKernelGGL(js_pairs_kernel, grid, dim3(256), 0, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(js_reduce_kernel, dim3(pairs), dim3(256), 0, stream, p.part, p.rows * p.H, p.L, acc);
  return hipGetLastError();
}

// ---- host: Eq. 6 and the greedy search
static double block_similarity(const double* js, int L, int m, int n) {
  const double ln2 = 0.69314718055994530942;
  double total = 0.0;
  for (int i = m; i <= n; ++i)
    for (int j = m; j <= n; ++j)
      if (i != j) total += ln2 - js[i * L + j];
  const int size = n - m + 1;
  return total / ((double)size * (size - 1));
}

int policy_search(const double* js, int L, double theta, int32_t* pi, int32_t* n_blocks) {
  int nb = 0, m = 0;
  while (m < L) {
    int best = m;   // a single layer always qualifies
    for (int n = m + 1; n < L; ++n)
      if (block_similarity(js, L, m, n) >= theta) best = n;
    pi[nb++] = best - m + 1;
    m = best + 1;
  }
  *n_blocks = nb;
  return 0;
}

}  // namespace san
