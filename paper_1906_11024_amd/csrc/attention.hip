// Decode-time attention for the shared-attention decoder (Eq. 1-5).
//
// The work is HBM-bound (4 flops per key/value element pair), so the kernel is a
// streaming one: a 64-lane wave owns one head of one key/value stream; LPP lanes
// cover the dh elements of one position with 16-byte loads and 64/LPP positions
// are in flight per load instruction, several instructions deep.  Scores live in
// LDS (one row per query), the softmax max/sum are wave shuffles, and the
// normalised weights are written out once per sharing block so that the other
// layers of the block (apply mode) only stream their own V.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace san {

constexpr int kWavesPerBlock = 4;

// The LDS score rows are private to a wave: order its lanes' writes before the
// other lanes' reads without a block-wide barrier.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

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

// PIPE = 1: the variant for long streams (see stream_pass below): every request after
// a stream's first chunk is unconditional, so the waits are exact and loading overlaps
// computing.  It holds three chunks in registers where PIPE = 0 gets by with fewer,
// and wastes a few instructions on short streams, so the launcher picks it by the
// capacity of the stream (lmax).
template <typename T, int LPP, int NQ, int PIPE>
__global__ __launch_bounds__(kWavesPerBlock * 64) void attention_kernel(AttnParams p) {
  constexpr int EPL = Frag<T>::N;       // elements per lane per position
  constexpr int PPL = kWave / LPP;      // positions per load instruction
  constexpr int DH = LPP * EPL;
  // load instructions per chunk: a chunk of ~32 positions measured best for both
  // storage types (deeper chunks cost registers, hence waves; shallower ones loop more)
  constexpr int U = PPL >= 8 ? 4 : 8;
  constexpr int CH = PPL * U;           // positions per chunk
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  const int c = lane % LPP, g = lane / LPP;
  float* sc = reinterpret_cast<float*>(smem) + (size_t)wid * NQ * p.lmax;                 // [NQ][lmax]
  // self mode: element offset of key j's row inside the cache, [lmax]
  long long* slot_off = reinterpret_cast<long long*>(smem + sizeof(float) * kWavesPerBlock * NQ * p.lmax);

  // The launcher spreads the work over a 3-D grid whose linear order (x fastest) is
  // the order wanted on the XCDs, so that the block index needs no run-time
  // divisions here (four of them were ~130 scalar instructions at the head of
  // every wave).  p.grid3 == 0: plain 1-D grid (a dimension would not fit).
  const int nhg = (p.H + kWavesPerBlock - 1) / kWavesPerBlock;
  int hg, rest, qb_grid = 0;
  if (p.self_mode && p.rpg > 1) {
    // The hypotheses of a sentence descend from common ancestors, so their streams
    // name the same cache rows for most past positions.  Workgroups go to the 8
    // XCDs round-robin by linear index and each XCD has its own L2: the rpg rows
    // of a sentence (same heads) take consecutive slots of ONE XCD, so a shared
    // cache row leaves HBM once and the other hypotheses hit in L2.
    // grid = (8 XCDs, rpg rows, rounds): linear index = xcd + 8 * (row + rpg * round)
    const int grp = blockIdx.z * 8 + blockIdx.x;          // (sentence, head group)
    if (grp >= p.groups * nhg) return;                    // padding of the last round (whole block)
    const bool pow2 = (nhg & (nhg - 1)) == 0;
    const int sentence = pow2 ? grp >> __builtin_ctz(nhg) : grp / nhg;
    hg = grp - sentence * nhg;
    rest = sentence * p.rpg + blockIdx.y;
  } else if (p.grid3) {
    hg = blockIdx.x;            // grid = (head groups, rows) or (head groups, groups, query blocks)
    rest = blockIdx.y;
    qb_grid = blockIdx.z;
  } else {
    hg = blockIdx.x % nhg;
    rest = blockIdx.x / nhg;
  }
  const int h = hg * kWavesPerBlock + wid;
  const bool head_ok = h < p.H;

  // ---- which stream, which queries, how many keys
  int n = 0;                 // keys this wave walks
  int qrow[NQ], nk[NQ];      // query row (-1: none) and number of keys it may see
  long long slot_base = 0;
  if (p.self_mode) {
    const int r = rest;
    // slot of key j: position-major cache, row taken from the ancestry table.  The
    // whole table row is fetched (entries past the current step are never used),
    // so these loads do not wait for the step counter.  The 64-bit multiply by the
    // row stride is done here, once per key, not once per load (K and V caches
    // have the same layout in this mode).
    const long long ld_cache = p.apply ? p.ldv : p.ldk;
    const int slot_rows = p.slot_rows > 0 ? p.slot_rows : p.rows;
    for (int j = threadIdx.x; j < p.lmax; j += blockDim.x)
      slot_off[j] = (long long)(j * slot_rows + p.anc[(size_t)r * p.ld_anc + j]) * ld_cache;
    n = *p.t_dev + 1;
    n = min(n, p.lmax);
    qrow[0] = r;
    nk[0] = n;
#pragma unroll
    for (int i = 1; i < NQ; ++i) { qrow[i] = -1; nk[i] = 0; }
    __syncthreads();
  } else {
    // blocks of one group (= the beams of a sentence) are numbered a multiple of
    // 8 apart where possible, so that they land on the same XCD and share its L2
    const int qb = p.grid3 ? qb_grid : rest / p.groups;   // query block inside the group
    const int grp = p.grid3 ? rest : rest % p.groups;
    slot_base = (long long)(p.group_map ? p.group_map[grp] : grp) * p.slot_stride;
    const int nfull = p.len ? max(0, min(p.len[grp], p.lmax)) : p.n_fixed;
    n = 0;
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
  if (!head_ok) return;  // no block-wide barrier below this point

  const T* Kp = reinterpret_cast<const T*>(p.K);
  const T* Vp = reinterpret_cast<const T*>(p.V);
  const T* Qp = reinterpret_cast<const T*>(p.q);
  T* Op = reinterpret_cast<T*>(p.out);
  const int col = h * DH + c * EPL;
  const bool self_mode = p.self_mode != 0;
  // this lane's column of the stream's first slot; per key only an offset is added
  Kp += slot_base * p.ldk + col;
  Vp += slot_base * p.ldv + col;
  const unsigned ldk = (unsigned)p.ldk, ldv = (unsigned)p.ldv;   // < 2^24 (checked at launch)

  // One chunk = U load instructions = CH positions; inside the last instruction
  // positions past n-1 re-read position n-1 (never out of bounds) and are ignored
  // later.
  auto load_chunk = [&](const T* base, unsigned ld, int j0, uint4 (&buf)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (j0 + u * PPL < n) {   // wave-uniform: instructions wholly past the end are not issued
        const int j = min(j0 + u * PPL + g, n - 1);
        const long long off = self_mode ? slot_off[j] : (long long)__umul24((unsigned)j, ld);   // j < 2^10
        buf[u] = *reinterpret_cast<const uint4*>(base + off);
      } else {
        buf[u] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
  };

  // The same chunk with every instruction issued (positions past n-1 re-read
  // position n-1: the same cache line, so only the instruction is wasted).  Used
  // in the steady state of long streams: a request the compiler sees as
  // unconditional is one it can count, and only then does the wait for an older
  // chunk let the younger one stay in flight (behind conditional requests every
  // wait drains all loads, and loading and computing take turns instead of
  // overlapping).
  auto load_all = [&](const T* base, unsigned ld, int j0, uint4 (&buf)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = min(j0 + u * PPL + g, n - 1);
      const long long off = self_mode ? slot_off[j] : (long long)__umul24((unsigned)j, ld);
      buf[u] = *reinterpret_cast<const uint4*>(base + off);
    }
  };
  // One pass over the stream with two buffers: on entry b0 holds (a request for)
  // chunk 0 and b1 chunk 1; a buffer is refilled two chunks ahead as soon as it has
  // been consumed.  PIPE: the steady state has no branches around its requests, and
  // the last one to three chunks are written out case by case for the same reason.
  auto stream_pass = [&](auto&& consume, const T* base, unsigned ld, uint4 (&b0)[U], uint4 (&b1)[U]) {
    int j0 = 0;
    if constexpr (PIPE) {
      while (j0 + 3 * CH < n) {
        consume(j0, b0);
        load_all(base, ld, j0 + 2 * CH, b0);
        consume(j0 + CH, b1);
        load_all(base, ld, j0 + 3 * CH, b1);
        j0 += 2 * CH;
      }
      if (j0 + 2 * CH < n) {
        consume(j0, b0);
        load_all(base, ld, j0 + 2 * CH, b0);
        consume(j0 + CH, b1);
        consume(j0 + 2 * CH, b0);
      } else if (j0 + CH < n) {
        consume(j0, b0);
        consume(j0 + CH, b1);
      } else if (j0 < n) {
        consume(j0, b0);
      }
    } else {
      for (; j0 < n; j0 += 2 * CH) {
        consume(j0, b0);
        if (j0 + 2 * CH < n) load_chunk(base, ld, j0 + 2 * CH, b0);
        if (j0 + CH < n) {
          consume(j0 + CH, b1);
          if (j0 + 3 * CH < n) load_chunk(base, ld, j0 + 3 * CH, b1);
        }
      }
    }
  };
  auto load_second = [&](const T* base, unsigned ld, uint4 (&buf)[U]) {   // chunk 1, if there is one
    if (CH < n) {
      if constexpr (PIPE) load_all(base, ld, CH, buf);
      else load_chunk(base, ld, CH, buf);
    }
  };

  // The first chunks of K and V are requested before any score is computed, so a
  // short stream costs a single memory round trip.
  uint4 kb0[U], kb1[U], vb0[U], vb1[U];
  if (n > 0) {
    if (!p.apply) {
      load_chunk(Kp, ldk, 0, kb0);
      if constexpr (PIPE) load_second(Kp, ldk, kb1);
    }
    load_chunk(Vp, ldv, 0, vb0);
  }

  if (!p.apply) {
    // ---- pass 1: scores (Eq. 1, numerator)
    const float scale2 = p.scale * 1.44269504088896341f;   // scores in log2 units: the softmax is one v_exp_f32 per score
    constexpr bool kPacked = std::is_same<T, bf16_t>::value;
    // fp32: the query times the scale, as floats.  bf16: the raw pairs -- both operands are bf16, their
    // products exact in fp32, so the packed dot product (two products and an add per instruction)
    // replaces unpacking and multiply-adds; the scale is applied to the sum.
    float qf[kPacked ? 1 : NQ][EPL];
    uint4 qraw[kPacked ? NQ : 1];
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      if constexpr (kPacked) {
        qraw[i] = make_uint4(0u, 0u, 0u, 0u);
        if (qrow[i] >= 0) qraw[i] = *reinterpret_cast<const uint4*>(Qp + (size_t)qrow[i] * p.ldq + col);
      } else {
        if (qrow[i] >= 0) {
          load_frag(Qp + (size_t)qrow[i] * p.ldq + col, qf[i]);
#pragma unroll
          for (int e = 0; e < EPL; ++e) qf[i][e] *= scale2;
        } else {
#pragma unroll
          for (int e = 0; e < EPL; ++e) qf[i][e] = 0.f;
        }
      }
    }
    auto scores = [&](int j0, const uint4 (&buf)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = j0 + u * PPL + g;
        if constexpr (kPacked) {
          typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
#pragma unroll
          for (int i = 0; i < NQ; ++i) {
            float dot = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, qraw[i].x),
                                                        __builtin_bit_cast(bf16x2_t, buf[u].x), 0.f, false);
            dot = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, qraw[i].y), __builtin_bit_cast(bf16x2_t, buf[u].y), dot, false);
            dot = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, qraw[i].z), __builtin_bit_cast(bf16x2_t, buf[u].z), dot, false);
            dot = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, qraw[i].w), __builtin_bit_cast(bf16x2_t, buf[u].w), dot, false);
            dot = lanes_sum<LPP>(dot) * scale2;
            if (c == 0 && j < n) sc[i * p.lmax + j] = (j < nk[i]) ? dot : -INFINITY;
          }
        } else {
          float kf[EPL];
          widen(buf[u], kf);
#pragma unroll
          for (int i = 0; i < NQ; ++i) {
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) dot = fmaf(qf[i][e], kf[e], dot);
            dot = lanes_sum<LPP>(dot);
            if (c == 0 && j < n) sc[i * p.lmax + j] = (j < nk[i]) ? dot : -INFINITY;
          }
        }
      }
    };
    if constexpr (PIPE) {
      stream_pass(scores, Kp, ldk, kb0, kb1);
    } else {
      for (int j0 = 0; j0 < n; j0 += 2 * CH) {   // K chunks are requested one chunk ahead
        if (j0 + CH < n) load_chunk(Kp, ldk, j0 + CH, kb1);
        scores(j0, kb0);
        if (j0 + CH < n) {
          if (j0 + 2 * CH < n) load_chunk(Kp, ldk, j0 + 2 * CH, kb0);
          scores(j0 + CH, kb1);
        }
      }
    }
    wave_lds_sync();
    load_second(Vp, ldv, vb1);   // second V chunk travels during the softmax
    if (NQ == 4) {
      // ---- softmax over key positions, the four queries side by side: lanes
      // [16 i, 16 i + 16) own query i, so the maxima and sums are 16-lane row
      // reductions (DPP only) and the four rows cost one pass instead of four
      const int i = lane >> 4, l16 = lane & 15;
      int qr = qrow[0];
#pragma unroll
      for (int q = 1; q < NQ; ++q)
        if (i == q) qr = qrow[q];
      float* row = sc + i * p.lmax;
      float m = -INFINITY;
      for (int j = l16; j < n; j += 16) m = fmaxf(m, row[j]);
      m = group_max<16>(m);
      float s = 0.f;
      for (int j = l16; j < n; j += 16) {
        const float e = (row[j] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(row[j] - m);
        row[j] = e;
        s += e;
      }
      s = group_sum<16>(s);
      const float inv = s > 0.f ? 1.0f / s : 0.f;
      if (qr >= 0) {
        float* Sg = p.S_buf ? p.S_buf + ((size_t)qr * p.H + h) * p.ldS : nullptr;
        for (int j = l16; j < n; j += 16) {
          const float w = row[j] * inv;
          row[j] = w;
          if (p.emit) Sg[j] = w;
        }
        if (p.emit && p.zero_tail)
          for (int j = n + l16; j < p.ldS; j += 16) Sg[j] = 0.f;
      }
    } else {
      // ---- softmax over key positions, one query at a time
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        if (qrow[i] < 0) continue;
        float* row = sc + i * p.lmax;
        float m = -INFINITY;
        for (int j = lane; j < n; j += kWave) m = fmaxf(m, row[j]);
        m = wave_max(m);
        float s = 0.f;
        for (int j = lane; j < n; j += kWave) {
          const float e = (row[j] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(row[j] - m);
          row[j] = e;
          s += e;
        }
        s = wave_sum(s);
        const float inv = s > 0.f ? 1.0f / s : 0.f;
        float* Sg = p.S_buf ? p.S_buf + ((size_t)qrow[i] * p.H + h) * p.ldS : nullptr;
        for (int j = lane; j < n; j += kWave) {
          const float w = row[j] * inv;
          row[j] = w;
          if (p.emit) Sg[j] = w;
        }
        if (p.emit && p.zero_tail)
          for (int j = n + lane; j < p.ldS; j += kWave) Sg[j] = 0.f;
      }
    }
  } else {
    load_second(Vp, ldv, vb1);
    // ---- shared weights: S^{m+i} = S^m (Eq. 4)
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      if (qrow[i] < 0) continue;
      const float* Sg = p.S_buf + ((size_t)qrow[i] * p.H + h) * p.ldS;
      for (int j = lane; j < n; j += kWave) sc[i * p.lmax + j] = (j < nk[i]) ? Sg[j] : 0.f;
    }
  }
  wave_lds_sync();

  // ---- pass 2: A = S V (Eq. 2)
  float acc[NQ][EPL];
#pragma unroll
  for (int i = 0; i < NQ; ++i)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[i][e] = 0.f;
  auto weighted = [&](int j0, const uint4 (&buf)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = j0 + u * PPL + g;
      if (j < n) {
        float vf[EPL];
        widen(buf[u], vf);
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
          const float w = sc[i * p.lmax + j];
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[i][e] = fmaf(w, vf[e], acc[i][e]);
        }
      }
    }
  };
  stream_pass(weighted, Vp, ldv, vb0, vb1);
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[i][e] = xor_sum<LPP, kWave>(acc[i][e]);
    if (g == 0 && qrow[i] >= 0) store_frag(Op + (size_t)qrow[i] * p.ldo + col, acc[i]);
  }
}

template <typename T, int LPP> static hipError_t launch_lpp(const AttnParams& p0, hipStream_t stream) {
  AttnParams p = p0;
  const int nhg = (p.H + kWavesPerBlock - 1) / kWavesPerBlock;
  constexpr unsigned kMaxDim = 65535;
  p.grid3 = 0;
  // streams that can grow past four chunks of 32 positions take the variant whose loads overlap its arithmetic
  const bool pipe = p.lmax >= 128;
  if (p.self_mode) {
    const size_t smem = sizeof(float) * kWavesPerBlock * p.lmax + sizeof(long long) * p.lmax;
    dim3 grid((unsigned)(p.rows * nhg));
    if (p.rpg > 1) {   // rows of a sentence on one XCD: (sentence, head group) pairs padded to a multiple of 8
      if (p.rows % p.rpg) return hipErrorInvalidValue;
      p.groups = p.rows / p.rpg;
      const unsigned rounds = (unsigned)((p.groups * nhg + 7) / 8);
      if (rounds > kMaxDim || (unsigned)p.rpg > kMaxDim) return hipErrorInvalidValue;
      grid = dim3(8, (unsigned)p.rpg, rounds);
    } else if ((unsigned)p.rows <= kMaxDim) {
      p.grid3 = 1;
      grid = dim3((unsigned)nhg, (unsigned)p.rows, 1);
    }
    if (pipe) hipLaunchKernelGGL((attention_kernel<T, LPP, 1, 1>), grid, dim3(kWavesPerBlock * 64), smem, stream, p);
    else hipLaunchKernelGGL((attention_kernel<T, LPP, 1, 0>), grid, dim3(kWavesPerBlock * 64), smem, stream, p);
  } else if (p.rpg <= 32 && (long)p.groups * p.H * ((p.rpg + 3) / 4) < 1024) {
    // few queries per stream (the beams of a sentence) and few streams: one wave
    // per query keeps enough waves in flight (at least ~one per SIMD); the queries'
    // re-reads of the stream hit in L2.  With >= 1024 streams a wave takes 4 queries.
    const size_t smem = sizeof(float) * kWavesPerBlock * p.lmax;
    dim3 grid((unsigned)(p.groups * p.rpg * nhg));
    if ((unsigned)p.groups <= kMaxDim && (unsigned)p.rpg <= kMaxDim) {
      p.grid3 = 1;
      grid = dim3((unsigned)nhg, (unsigned)p.groups, (unsigned)p.rpg);
    }
    if (pipe) hipLaunchKernelGGL((attention_kernel<T, LPP, 1, 1>), grid, dim3(kWavesPerBlock * 64), smem, stream, p);
    else hipLaunchKernelGGL((attention_kernel<T, LPP, 1, 0>), grid, dim3(kWavesPerBlock * 64), smem, stream, p);
  } else {
    const int nqb = (p.rpg + 3) / 4;
    const size_t smem = sizeof(float) * kWavesPerBlock * 4 * p.lmax;
    dim3 grid((unsigned)((size_t)p.groups * nqb * nhg));
    if ((unsigned)p.groups <= kMaxDim && (unsigned)nqb <= kMaxDim) {
      p.grid3 = 1;
      grid = dim3((unsigned)nhg, (unsigned)p.groups, (unsigned)nqb);
    }
    if (pipe) hipLaunchKernelGGL((attention_kernel<T, LPP, 4, 1>), grid, dim3(kWavesPerBlock * 64), smem, stream, p);
    else hipLaunchKernelGGL((attention_kernel<T, LPP, 4, 0>), grid, dim3(kWavesPerBlock * 64), smem, stream, p);
  }
  return hipGetLastError();
}

hipError_t launch_attention(int dtype, const AttnParams& p, hipStream_t stream) {
  if (p.rows <= 0 || p.lmax <= 0) return hipSuccess;
  if (attention_ctx_mfma_fits(dtype, p)) return launch_attention_ctx_mfma(p, stream);
  // Long streams in a launch that has fewer of them than the chip has SIMDs are split over
  // several waves each (attention_split.hip); measured on the 12-layer, 256-step workload
  // (1024 streams of up to 256 cached positions, 256 sentence memories of 128 positions):
  // enc-dec head 13.4 -> 9.4 us with 4 waves per stream and one query per workgroup,
  // self-attention head 13.9 -> 13.4 us with 2 waves.  Everything else is faster with one
  // wave per stream (at 2048 streams of <= 64 positions the split kernel's extra workgroup
  // barrier and LDS combine cost more than its shorter chains save: 8.4 vs 7.7 us), and so
  // are followers (their single pass over V is short already).
  if (!p.apply) {
    const long streams = p.self_mode ? (long)p.rows * p.H : (long)p.groups * p.H * ((p.rpg + 3) / 4);
    if (p.self_mode && streams <= 1024 && p.lmax >= 128) return launch_attention_split(dtype, p, 2, false, stream);
    if (!p.self_mode && !p.causal && p.rpg > 1 && streams < 1024 && p.lmax >= 96)
      return launch_attention_split(dtype, p, 4, true, stream);
  }
  if (p.lmax > 1024) return hipErrorInvalidValue;   // score rows must fit 64 KB of LDS
  if (p.ldk < 0 || p.ldv < 0 || p.ldk >= (1 << 24) || p.ldv >= (1 << 24)) return hipErrorInvalidValue;
  if (p.self_mode && p.ldk != p.ldv && !p.apply) return hipErrorInvalidValue;   // one offset table serves both caches
  const int lpp = dtype == 1 ? p.dh / 8 : p.dh / 4;
  if (dtype == 1) {
    switch (lpp) {
      case 2: return launch_lpp<bf16_t, 2>(p, stream);
      case 4: return launch_lpp<bf16_t, 4>(p, stream);
      case 8: return launch_lpp<bf16_t, 8>(p, stream);
      case 16: return launch_lpp<bf16_t, 16>(p, stream);
      default: return hipErrorInvalidValue;
    }
  }
  switch (lpp) {
    case 4: return launch_lpp<float, 4>(p, stream);
    case 8: return launch_lpp<float, 8>(p, stream);
    case 16: return launch_lpp<float, 16>(p, stream);
    case 32: return launch_lpp<float, 32>(p, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace san
