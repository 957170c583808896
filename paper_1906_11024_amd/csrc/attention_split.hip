// Decode-time attention (Eq. 1-5) for long streams in launches with few of them: the
// stream is split over the waves of a workgroup.  (attention.hip holds the kernel that
// gives a stream to one wave, which is faster whenever a launch has at least about two
// waves per SIMD that way, and says which launches come here.)
//
// The work is HBM-bound (4 flops per key/value element pair) and, at decode sizes,
// latency-bound: a launch moves a few tens of MB and every wave's chain of
// dependent instructions counts.  So a key/value stream (one head of one decoder
// row's history, or of one sentence's encoder memory) is split over the NW waves of
// a workgroup: LPP lanes cover the dh elements of one position with 16-byte loads,
// a load instruction covers 64/LPP positions, and wave w takes the load slots w,
// w + NW, w + 2 NW, ...  Each wave requests its keys AND values up front (one memory
// round trip for streams of up to NW x 32 positions), keeps its scores in registers,
// and reduces them to a partial softmax (running maximum m, sum l of exp(s - m),
// weighted value sum) without ever writing a probability to LDS; the partials of the
// NW waves are combined through LDS after a single workgroup barrier:
//   M = max_w m_w,  L = sum_w l_w exp(m_w - M),  A = sum_w acc_w exp(m_w - M) / L.
// (Scores are kept in units of log 2, so every exp is the hardware's 2^x.)
// A block head of a sharing block also emits the normalised weights
// S_j = exp(s_j - M) / L once (Eq. 3); the other layers of the block (apply mode,
// Eq. 4) read them straight into the lanes that own the positions and only stream
// their own V.
#include "common.h"
#include "kernels.h"

namespace san {

constexpr int kMaxWavesPerBlock = 8;

// Scores are kept in units of log 2 (the query scale carries the factor log2 e), so that
// exp(s - m) is the hardware's 2^x, one instruction; every lane of a position group
// evaluates its group's exponentials itself, which is cheaper than passing them around.
constexpr float kLog2e = 1.4426950408889634f;
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// max / sum over the position groups of a wave, i.e. over the lanes that agree in their
// place inside the group (lane bits >= log2 LPP); all lanes of a group hold the same value
template <int LPP> __device__ __forceinline__ float groups_max(float v) {
  if (LPP <= 1) v = fmaxf(v, dpp_mov<0x121>(v));   // row_ror:1
  if (LPP <= 2) v = fmaxf(v, dpp_mov<0x122>(v));
  if (LPP <= 4) v = fmaxf(v, dpp_mov<0x124>(v));
  if (LPP <= 8) v = fmaxf(v, dpp_mov<0x128>(v));
  if (LPP <= 16) v = max_xor16(v);
  return max_xor32(v);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// 16-byte fragment -> fp32 values
static __device__ __forceinline__ void widen(const uint4& raw, float (&out)[4]) {
  out[0] = __uint_as_float(raw.x); out[1] = __uint_as_float(raw.y);
  out[2] = __uint_as_float(raw.z); out[3] = __uint_as_float(raw.w);
}
static __device__ __forceinline__ void widen(const uint4& raw, float (&out)[8]) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

// Query fragment of one lane: fp32 values, or the raw bf16 pairs for the packed dot product.
template <typename T> struct QFrag;
template <> struct QFrag<float> {
  float v[4];
  __device__ __forceinline__ void load(const float* p, float scale) {
    const float4 x = *reinterpret_cast<const float4*>(p);
    v[0] = x.x * scale; v[1] = x.y * scale; v[2] = x.z * scale; v[3] = x.w * scale;
  }
  __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0.f; }
  // this lane's part of q . k (the scale is already in q)
  __device__ __forceinline__ float dot(const uint4& k, float) const {
    float d = v[0] * __uint_as_float(k.x);
    d = fmaf(v[1], __uint_as_float(k.y), d);
    d = fmaf(v[2], __uint_as_float(k.z), d);
    return fmaf(v[3], __uint_as_float(k.w), d);
  }
};
template <> struct QFrag<bf16_t> {
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_t* p, float) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void zero() { raw = make_uint4(0u, 0u, 0u, 0u); }
  // both operands are bf16, so their products are exact in fp32: the packed dot
  // product (two products and an add per instruction) replaces unpack + multiply-add
  __device__ __forceinline__ float dot(const uint4& k, float scale) const {
    float d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, raw.x), __builtin_bit_cast(bf16x2, k.x), 0.f, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, raw.y), __builtin_bit_cast(bf16x2, k.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, raw.z), __builtin_bit_cast(bf16x2, k.z), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, raw.w), __builtin_bit_cast(bf16x2, k.w), d, false);
    return d * scale;
  }
};

// MULTI = 0: the launcher guarantees that a wave's share of the stream is at most one
// chunk (U load instructions), so there is no loop and no running rescale.
template <typename T, int LPP, int NQ, int MULTI>
__global__ __launch_bounds__(kMaxWavesPerBlock * 64) void attention_kernel_split(AttnParams p) {
  constexpr int EPL = Frag<T>::N;       // elements per lane per position
  constexpr int PPL = kWave / LPP;      // positions per load instruction
  constexpr int DH = LPP * EPL;
  // load instructions per chunk: ~32 positions for both storage types
  constexpr int U = PPL >= 8 ? 4 : 8;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, NW = blockDim.x >> 6;
  const int c = lane % LPP, g = lane / LPP;
  // LDS: raw scores [NQ][lmax] (only written when the weights are emitted), then the
  // waves' partials [NW][NQ][2 + DH] = (m, l, weighted value sum)
  float* sc = reinterpret_cast<float*>(smem);
  float* comb = sc + (p.emit ? NQ * p.lmax : 0);
  constexpr int CW = 2 + DH;

  // ---- which stream, which head, which queries, how many keys
  int h, rest, qb = 0;
  if (p.self_mode && p.rpg > 1) {
    // The hypotheses of a sentence descend from common ancestors, so their streams
    // name the same cache rows for most past positions.  Workgroups go to the 8
    // XCDs round-robin by linear index and each XCD has its own L2: the rpg rows
    // of a sentence (same head) take consecutive slots of ONE XCD, so a shared
    // cache row leaves HBM once and the other hypotheses hit in L2.
    // grid = (8 XCDs, rpg rows, rounds): linear index = xcd + 8 * (row + rpg * round)
    const int grp = blockIdx.z * 8 + blockIdx.x;          // (sentence, head)
    if (grp >= p.groups * p.H) return;                    // padding of the last round (whole block)
    const bool pow2 = (p.H & (p.H - 1)) == 0;
    const int sentence = pow2 ? grp >> __builtin_ctz(p.H) : grp / p.H;
    h = grp - sentence * p.H;
    rest = sentence * p.rpg + blockIdx.y;
  } else if (p.grid3) {
    h = blockIdx.x;            // grid = (heads, rows) or (heads, groups, query blocks)
    rest = blockIdx.y;
    qb = blockIdx.z;
  } else {
    h = blockIdx.x % p.H;
    rest = blockIdx.x / p.H;
    if (!p.self_mode) { qb = rest / p.groups; rest = rest % p.groups; }
  }

  int n = 0;                 // keys of the stream that any query of this block sees
  int qrow[NQ], nk[NQ];      // query row (-1: none) and number of keys it may see
  long long slot_base = 0;
  const int* anc_row = nullptr;
  if (p.self_mode) {
    const int r = rest;
    anc_row = p.anc + (size_t)r * p.ld_anc;
    n = min(*p.t_dev + 1, p.lmax);
    qrow[0] = r;
    nk[0] = n;
#pragma unroll
    for (int i = 1; i < NQ; ++i) { qrow[i] = -1; nk[i] = 0; }
  } else {
    const int grp = rest;
    slot_base = (long long)(p.group_map ? p.group_map[grp] : grp) * p.slot_stride;
    const int nfull = p.len ? max(0, min(p.len[grp], p.lmax)) : p.n_fixed;
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const int li = qb * NQ + i;
      if (li < p.rpg) {
        qrow[i] = grp * p.rpg + li;
        nk[i] = p.causal ? min(nfull, li % p.causal + 1) : nfull;
        n = max(n, nk[i]);
      } else {
        qrow[i] = -1;
        nk[i] = 0;
      }
    }
  }

  const T* Kp = reinterpret_cast<const T*>(p.K);
  const T* Vp = reinterpret_cast<const T*>(p.V);
  const T* Qp = reinterpret_cast<const T*>(p.q);
  T* Op = reinterpret_cast<T*>(p.out);
  const int col = h * DH + c * EPL;
  const bool self_mode = p.self_mode != 0;
  const bool apply = p.apply != 0;
  // this lane's column of the stream's first slot; per key only an offset is added
  // (the key and value caches have the same layout in self mode: one offset serves both)
  Kp += slot_base * p.ldk + col;
  Vp += slot_base * p.ldv + col;
  const unsigned ldk = (unsigned)p.ldk, ldv = (unsigned)p.ldv;   // < 2^24 (checked at launch)
  const unsigned slot_rows = (unsigned)(p.slot_rows > 0 ? p.slot_rows : p.rows);

  // Load slot s of this wave's chunk k: s = (k U + u) NW + w covers positions s PPL .. s PPL + PPL - 1.
  // Positions past n - 1 inside a slot re-read position n - 1 (never out of bounds) and are
  // ignored later; slots wholly past the end are not requested (wave-uniform test).
  auto first_pos = [&](int k, int u) { return ((k * U + u) * NW + wid) * PPL; };
  // In self mode the cache row of every position comes from the ancestry table: those
  // (dependent) loads all go out first, then the key/value loads, so that a chunk costs two
  // memory round trips and not one pair per load slot.
  auto load_chunk = [&](int k, uint4 (&kb)[U], uint4 (&vb)[U]) {
    int row[U];
    if (self_mode) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j0 = first_pos(k, u);
        row[u] = (j0 < n) ? anc_row[min(j0 + g, n - 1)] : 0;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j0 = first_pos(k, u);
      if (j0 < n) {
        const int j = min(j0 + g, n - 1);
        long long ko, vo;
        if (self_mode) {
          // position-major cache: element offset of (position j, its row)
          const unsigned slot = (unsigned)j * slot_rows + (unsigned)row[u];        // < 2^30 (checked at init)
          ko = (long long)((unsigned long long)slot * ldk);
          vo = (long long)((unsigned long long)slot * ldv);
        } else {
          ko = (long long)__umul24((unsigned)j, ldk);                              // j < 2^10
          vo = (long long)__umul24((unsigned)j, ldv);
        }
        kb[u] = apply ? make_uint4(0u, 0u, 0u, 0u) : *reinterpret_cast<const uint4*>(Kp + ko);
        vb[u] = *reinterpret_cast<const uint4*>(Vp + vo);
      } else {
        kb[u] = make_uint4(0u, 0u, 0u, 0u);
        vb[u] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
  };

  const int nslots = (n + PPL - 1) / PPL;                       // load slots of the whole stream
  const int my_slots = nslots > wid ? (nslots - wid + NW - 1) / NW : 0;
  const int nchunks = (my_slots + U - 1) / U;

  uint4 kb0[U], vb0[U];
  if (nchunks > 0) load_chunk(0, kb0, vb0);

  // queries (the scale goes into fp32 queries; bf16 ones stay packed and the score is scaled)
  QFrag<T> qf[NQ];
  if (!apply) {
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      if (qrow[i] >= 0) qf[i].load(Qp + (size_t)qrow[i] * p.ldq + col, p.scale * kLog2e);
      else qf[i].zero();
    }
  }
  const float* Sg[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i)
    Sg[i] = (p.S_buf && qrow[i] >= 0) ? p.S_buf + ((size_t)qrow[i] * p.H + h) * p.ldS : nullptr;

  float m_run[NQ], l_lane[NQ], acc[NQ][EPL];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    m_run[i] = -INFINITY;
    l_lane[i] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[i][e] = 0.f;
  }

  // One chunk: scores of the wave's positions (registers), their partial softmax, the
  // weighted value sum.
  auto consume = [&](int k, const uint4 (&kb)[U], const uint4 (&vb)[U]) {
    if (!apply) {
      float s[NQ][U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = first_pos(k, u) + g;
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
          float dot = lanes_sum<LPP>(qf[i].dot(kb[u], p.scale * kLog2e));
          dot = (j < nk[i]) ? dot : -INFINITY;
          s[i][u] = dot;
          if (p.emit && c == 0 && j < n) sc[i * p.lmax + j] = dot;
        }
      }
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        float mx = s[i][0];
#pragma unroll
        for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[i][u]);
        mx = groups_max<LPP>(mx);
        const float m_new = fmaxf(m_run[i], mx);
        if (MULTI) {
          // earlier chunks were summed relative to the old maximum
          const float r = (m_run[i] == -INFINITY) ? 0.f : exp2_fast(m_run[i] - m_new);
          l_lane[i] *= r;
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[i][e] *= r;
        }
        m_run[i] = m_new;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const float pj = (s[i][u] == -INFINITY) ? 0.f : exp2_fast(s[i][u] - m_new);
          s[i][u] = pj;
          l_lane[i] += pj;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float vf[EPL];
        widen(vb[u], vf);
#pragma unroll
        for (int i = 0; i < NQ; ++i)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[i][e] = fmaf(s[i][u], vf[e], acc[i][e]);
      }
    } else {
      // ---- shared weights: S^{m+i} = S^m (Eq. 4), read by the lanes that own the positions
      float w[NQ][U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = first_pos(k, u) + g;
#pragma unroll
        for (int i = 0; i < NQ; ++i) w[i][u] = (j < nk[i] && Sg[i]) ? Sg[i][j] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float vf[EPL];
        widen(vb[u], vf);
#pragma unroll
        for (int i = 0; i < NQ; ++i)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[i][e] = fmaf(w[i][u], vf[e], acc[i][e]);
      }
    }
  };

  if constexpr (MULTI) {
    uint4 kb1[U], vb1[U];
    for (int k = 0; k < nchunks; k += 2) {
      if (k + 1 < nchunks) load_chunk(k + 1, kb1, vb1);
      consume(k, kb0, vb0);
      if (k + 1 < nchunks) {
        if (k + 2 < nchunks) load_chunk(k + 2, kb0, vb0);
        consume(k + 1, kb1, vb1);
      }
    }
  } else if (nchunks > 0) {
    consume(0, kb0, vb0);
  }

  // ---- this wave's partial: sum over the position groups of the wave, then to LDS
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[i][e] = xor_sum<LPP, kWave>(acc[i][e]);
    float* dst = comb + (size_t)(wid * NQ + i) * CW;
    if (!apply) {
      const float l_w = xor_sum<LPP, kWave>(l_lane[i]);   // over the position groups
      if (lane == 0) { dst[0] = m_run[i]; dst[1] = l_w; }
    }
    if (g == 0) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) dst[2 + c * EPL + e] = acc[i][e];
    }
  }
  __syncthreads();

  // ---- combine the partials: one output fragment (EPL columns of one query) per thread
  for (int t = threadIdx.x; t < NQ * LPP; t += blockDim.x) {
    const int i = t / LPP, cc = t % LPP;
    int qr = qrow[0];
#pragma unroll
    for (int ii = 1; ii < NQ; ++ii)
      if (i == ii) qr = qrow[ii];
    if (qr < 0) continue;
    float o[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = 0.f;
    if (apply) {
      for (int w = 0; w < NW; ++w) {
        const float* src = comb + (size_t)(w * NQ + i) * CW + 2 + cc * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] += src[e];
      }
    } else {
      float M = -INFINITY;
      for (int w = 0; w < NW; ++w) M = fmaxf(M, comb[(size_t)(w * NQ + i) * CW]);
      float L = 0.f;
      for (int w = 0; w < NW; ++w) {
        const float* src = comb + (size_t)(w * NQ + i) * CW;
        const float r = (src[0] == -INFINITY) ? 0.f : exp2_fast(src[0] - M);
        L += src[1] * r;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] = fmaf(src[2 + cc * EPL + e], r, o[e]);
      }
      const float inv = L > 0.f ? 1.0f / L : 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] *= inv;
    }
    store_frag(Op + (size_t)qr * p.ldo + h * DH + cc * EPL, o);
  }

  // ---- the normalised weights, once per sharing block (Eq. 3): S_j = exp(s_j - M) / L
  if (p.emit && !apply) {
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      if (qrow[i] < 0) continue;
      float M = -INFINITY;
      for (int w = 0; w < NW; ++w) M = fmaxf(M, comb[(size_t)(w * NQ + i) * CW]);
      float L = 0.f;
      for (int w = 0; w < NW; ++w) {
        const float* src = comb + (size_t)(w * NQ + i) * CW;
        L += (src[0] == -INFINITY) ? 0.f : src[1] * exp2_fast(src[0] - M);
      }
      const float inv = L > 0.f ? 1.0f / L : 0.f;
      float* out_S = p.S_buf + ((size_t)qrow[i] * p.H + h) * p.ldS;
      for (int j = threadIdx.x; j < n; j += blockDim.x) {
        const float sj = sc[i * p.lmax + j];
        out_S[j] = (sj == -INFINITY) ? 0.f : exp2_fast(sj - M) * inv;
      }
      if (p.zero_tail)
        for (int j = n + threadIdx.x; j < p.ldS; j += blockDim.x) out_S[j] = 0.f;
    }
  }
}

// nw waves per stream; the kernel variant without a chunk loop is taken when a wave's share
// of the longest stream fits one chunk.
template <typename T, int LPP, int NQ>
static hipError_t launch_nq(const AttnParams& p, dim3 grid, int nw, hipStream_t stream) {
  constexpr int DH = LPP * Frag<T>::N;
  constexpr int PPL = kWave / LPP, CH = PPL * (PPL >= 8 ? 4 : 8);   // positions per chunk, as in the kernel
  const size_t smem = sizeof(float) * ((p.emit ? (size_t)NQ * p.lmax : 0) + (size_t)nw * NQ * (2 + DH));
  const bool multi = p.lmax > nw * CH;
  if (multi) hipLaunchKernelGGL((attention_kernel_split<T, LPP, NQ, 1>), grid, dim3(nw * 64), smem, stream, p);
  else hipLaunchKernelGGL((attention_kernel_split<T, LPP, NQ, 0>), grid, dim3(nw * 64), smem, stream, p);
  return hipGetLastError();
}

template <typename T, int LPP>
static hipError_t launch_split_lpp(const AttnParams& p0, int nw, bool one_query, hipStream_t stream) {
  AttnParams p = p0;
  constexpr unsigned kMaxDim = 65535;
  p.grid3 = 0;
  if (p.self_mode) {
    dim3 grid((unsigned)(p.rows * p.H));
    if (p.rpg > 1) {   // rows of a sentence on one XCD: (sentence, head) pairs padded to a multiple of 8
      if (p.rows % p.rpg) return hipErrorInvalidValue;
      p.groups = p.rows / p.rpg;
      const unsigned rounds = (unsigned)((p.groups * p.H + 7) / 8);
      if (rounds > kMaxDim || (unsigned)p.rpg > kMaxDim) return hipErrorInvalidValue;
      grid = dim3(8, (unsigned)p.rpg, rounds);
    } else if ((unsigned)p.rows <= kMaxDim) {
      p.grid3 = 1;
      grid = dim3((unsigned)p.H, (unsigned)p.rows, 1);
    }
    return launch_nq<T, LPP, 1>(p, grid, nw, stream);
  }
  // grouped: the queries of a group (the beams of a sentence, or the positions of a
  // hypothesis when nothing is cached) share the stream; a workgroup takes four of them, or
  // one when there are too few streams to fill the chip otherwise (the other queries'
  // reads of the stream hit in L2: their workgroups are a multiple of 8 apart, on one XCD)
  const int nq = (p.rpg == 1 || one_query) ? 1 : 4;
  const int nqb = (p.rpg + nq - 1) / nq;
  dim3 grid((unsigned)((size_t)p.groups * nqb * p.H));
  if ((unsigned)p.groups <= kMaxDim && (unsigned)nqb <= kMaxDim) {
    p.grid3 = 1;
    grid = dim3((unsigned)p.H, (unsigned)p.groups, (unsigned)nqb);
  }
  return nq == 1 ? launch_nq<T, LPP, 1>(p, grid, nw, stream) : launch_nq<T, LPP, 4>(p, grid, nw, stream);
}

hipError_t launch_attention_split(int dtype, const AttnParams& p, int waves, bool one_query, hipStream_t stream) {
  if (p.rows <= 0 || p.lmax <= 0) return hipSuccess;
  if (p.lmax > 1024) return hipErrorInvalidValue;   // score rows must fit the LDS budget
  if (p.ldk < 0 || p.ldv < 0 || p.ldk >= (1 << 24) || p.ldv >= (1 << 24)) return hipErrorInvalidValue;
  if (waves != 1 && waves != 2 && waves != 4 && waves != 8) return hipErrorInvalidValue;
  const int lpp = dtype == 1 ? p.dh / 8 : p.dh / 4;
  if (dtype == 1) {
    switch (lpp) {
      case 2: return launch_split_lpp<bf16_t, 2>(p, waves, one_query, stream);
      case 4: return launch_split_lpp<bf16_t, 4>(p, waves, one_query, stream);
      case 8: return launch_split_lpp<bf16_t, 8>(p, waves, one_query, stream);
      case 16: return launch_split_lpp<bf16_t, 16>(p, waves, one_query, stream);
      default: return hipErrorInvalidValue;
    }
  }
  switch (lpp) {
    case 4: return launch_split_lpp<float, 4>(p, waves, one_query, stream);
    case 8: return launch_split_lpp<float, 8>(p, waves, one_query, stream);
    case 16: return launch_split_lpp<float, 16>(p, waves, one_query, stream);
    case 32: return launch_split_lpp<float, 32>(p, waves, one_query, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace san
