// Projection / FFN / output-layer GEMMs on CDNA4 matrix cores.
//
// out[m][n] = sum_k A[m][k] * W[n][k]: both operands are contiguous along k, so a
// lane's MFMA operand fragment is one 16-byte load.  A block of 4 waves (2x2)
// owns a (64*TM) x (64*TN) tile of the output; k is walked in chunks of 128 bytes
// per row, staged global -> registers -> LDS (double buffered, rows padded to 144
// bytes so that the 16-byte fragment reads of 16 neighbouring lanes hit all 64
// banks once).  The weight rows feed the MFMA "A" side and the activation rows
// the "B" side, so a lane ends up with 4 consecutive output columns of one
// output row, which makes the epilogue's bias loads and stores 16-byte wide.
#include "common.h"
#include "kernels.h"

namespace san {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kChunkBytes = 128;  // k-extent of one LDS stage, per row
constexpr int kRowBytes = 144;    // padded LDS row

template <typename T> __device__ __forceinline__ void mma_frag(f32x16& acc, const uint4& w, const uint4& x);

// fp32: a 16-byte fragment is 4 k-values -> 4 rank-2 updates (32x32x2).  Lanes
// 0-31 carry k = 0..3 of the 32-byte sub-step, lanes 32-63 carry k = 4..7; the
// pairing of k-values inside an instruction is irrelevant as both operands use it.
template <> __device__ __forceinline__ void mma_frag<float>(f32x16& acc, const uint4& w, const uint4& x) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w.x), __uint_as_float(x.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w.y), __uint_as_float(x.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w.z), __uint_as_float(x.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w.w), __uint_as_float(x.w), acc, 0, 0, 0);
}
// bf16: a 16-byte fragment is 8 k-values -> one 32x32x16 instruction.
template <> __device__ __forceinline__ void mma_frag<bf16_t>(f32x16& acc, const uint4& w, const uint4& x) {
  union U { uint4 u; bf16x8 b; };
  U a, b;
  a.u = w;
  b.u = x;
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.b, b.b, acc, 0, 0, 0);
}

template <typename T, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_kernel(GemmParams p) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int EPC = kChunkBytes / (int)sizeof(T);  // elements per chunk
  constexpr int LA = BM / 32, LB = BN / 32;          // 16-byte loads per thread per chunk
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Xs = smem;                                // [2][BM][144]
  unsigned char* Ws = smem + 2 * BM * kRowBytes;           // [2][BN][144]

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int wm = wid & 1, wn = wid >> 1;
  const int l32 = lane & 31, kh = lane >> 5;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  const int nchunks = p.K / EPC;
  const int cps = (nchunks + p.ksplit - 1) / p.ksplit;
  const int c_begin = blockIdx.z * cps;
  const int c_end = min(nchunks, c_begin + cps);

  const T* A = reinterpret_cast<const T*>(p.A);
  const T* W = reinterpret_cast<const T*>(p.W);
  const int lrow = tid >> 3, lseg = tid & 7;  // this thread's row (0..31) and 16-byte segment of a chunk

  uint4 xa[LA], wb[LB];
  auto load_global = [&](int c) {
    const size_t koff = (size_t)c * EPC + lseg * (16 / sizeof(T));
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int m = min(m0 + lrow + 32 * i, p.M - 1);
      xa[i] = *reinterpret_cast<const uint4*>(A + (size_t)m * p.lda + koff);
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int n = min(n0 + lrow + 32 * i, p.N - 1);
      wb[i] = *reinterpret_cast<const uint4*>(W + (size_t)n * p.K + koff);
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LA; ++i)
      *reinterpret_cast<uint4*>(Xs + (buf * BM + lrow + 32 * i) * kRowBytes + lseg * 16) = xa[i];
#pragma unroll
    for (int i = 0; i < LB; ++i)
      *reinterpret_cast<uint4*>(Ws + (buf * BN + lrow + 32 * i) * kRowBytes + lseg * 16) = wb[i];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (c_begin < c_end) {
    load_global(c_begin);
    store_lds(0);
  }
  __syncthreads();
  for (int c = c_begin; c < c_end; ++c) {
    const int buf = (c - c_begin) & 1;
    if (c + 1 < c_end) load_global(c + 1);
    const unsigned char* xs = Xs + (buf * BM + wm * 32 * TM + l32) * kRowBytes + kh * 16;
    const unsigned char* ws = Ws + (buf * BN + wn * 32 * TN + l32) * kRowBytes + kh * 16;
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      uint4 xf[TM], wf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) xf[i] = *reinterpret_cast<const uint4*>(xs + i * 32 * kRowBytes + sub * 32);
#pragma unroll
      for (int j = 0; j < TN; ++j) wf[j] = *reinterpret_cast<const uint4*>(ws + j * 32 * kRowBytes + sub * 32);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) mma_frag<T>(acc[i][j], wf[j], xf[i]);
    }
    if (c + 1 < c_end) store_lds(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue.  acc[i][j][v]: output row m = tile_m + l32, column
  // n = tile_n + (v/4)*8 + kh*4 + (v%4).
  const int t = p.t_dev ? *p.t_dev : 0;
  const T* bias = reinterpret_cast<const T*>(p.bias);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * 32 * TM + i * 32 + l32;
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn * 32 * TN + j * 32 + g * 8 + kh * 4;
        if (n >= p.N) continue;
        float v[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        if (p.out_kind == 2) {
          float* dst = reinterpret_cast<float*>(p.out[0]) + ((size_t)blockIdx.z * p.M + m) * p.N + n;
          if (n + 3 < p.N) {
            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            for (int e = 0; e < 4 && n + e < p.N; ++e) dst[e] = v[e];
          }
          continue;
        }
        const bool full = (n + 3 < p.N);
        if (bias) {
          for (int e = 0; e < 4; ++e)
            if (n + e < p.N) v[e] += to_f32(bias[n + e]);
        }
        if (p.relu) {
          for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
        }
        const int s = n / p.seg_w;       // segments are multiples of 4 columns wide
        const int nn = n - s * p.seg_w;
        const size_t off = (size_t)t * p.tstride[s] + (size_t)m * p.ldo[s] + nn;
        if (p.out_kind == 1) {
          float* dst = reinterpret_cast<float*>(p.out[s]) + off;
          if (full) {
            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            for (int e = 0; e < 4 && n + e < p.N; ++e) dst[e] = v[e];
          }
        } else {
          T* dst = reinterpret_cast<T*>(p.out[s]) + off;
          if (full) {
            store4(dst, make_float4(v[0], v[1], v[2], v[3]));
          } else {
            for (int e = 0; e < 4 && n + e < p.N; ++e) dst[e] = from_f32<T>(v[e]);
          }
        }
      }
    }
  }
}

template <typename T, int TM, int TN> static hipError_t launch_tile(const GemmParams& p, hipStream_t stream) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  dim3 grid((p.N + BN - 1) / BN, (p.M + BM - 1) / BM, p.ksplit);
  const size_t smem = 2 * (BM + BN) * kRowBytes;
  if (smem > 64 * 1024) {
    static bool raised = false;   // the limit is a per-function attribute; set it once
    if (!raised) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<T, TM, TN>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return e;
      raised = true;
    }
  }
  hipLaunchKernelGGL((gemm_kernel<T, TM, TN>), grid, dim3(256), smem, stream, p);
  return hipGetLastError();
}

static int pick_tile(int M, int N) {
  // 128x128 tiles only when they still give every CU at least ~2 blocks.
  const long blocks128 = (long)((M + 127) / 128) * ((N + 127) / 128);
  return blocks128 >= 512 ? 2 : 1;
}

int gemm_pick_ksplit(int M, int N, int K, int dtype) {
  const int epc = dtype == 1 ? 64 : 32;
  const int nchunks = K / epc;
  const long blocks = (long)((M + 63) / 64) * ((N + 63) / 64);
  int ks = 1;
  // aim for >= 256 blocks (one per CU), keep at least 4 chunks of k per block
  while (blocks * ks < 256 && nchunks / (ks * 2) >= 4 && ks < 16) ks *= 2;
  return ks;
}

hipError_t launch_gemm(int dtype, const GemmParams& p, hipStream_t stream) {
  if (p.M <= 0 || p.N <= 0) return hipSuccess;
  const int epc = dtype == 1 ? 64 : 32;
  if (p.K <= 0 || p.K % epc != 0 || p.ksplit < 1 || p.seg_w % 4 != 0) return hipErrorInvalidValue;
  const int tile = pick_tile(p.M, p.N);
  if (dtype == 1) {
    return tile == 2 ? launch_tile<bf16_t, 2, 2>(p, stream) : launch_tile<bf16_t, 1, 1>(p, stream);
  }
  return tile == 2 ? launch_tile<float, 2, 2>(p, stream) : launch_tile<float, 1, 1>(p, stream);
}

}  // namespace san
