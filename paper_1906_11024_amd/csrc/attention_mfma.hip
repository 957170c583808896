// Encoder-decoder attention of a block head on the bf16 matrix cores (Eq. 1-2 over a
// sentence's encoder memory, all hypotheses of the sentence at once).
//
// One wave owns one (sentence, head).  The memory is walked in blocks of 32 positions:
//   scores^T = K Q^T    32x32x16 MFMAs, positions as rows, the sentence's <= 32 queries as
//                       columns: a lane then holds, for ITS query (lane % 32), the scores of 16 of
//                       the block's positions (the other 16 are in lane ^ 32), so the softmax
//                       statistics are in-register reductions plus one exchange between the halves;
//   out += P V          the same registers, rounded to bf16, are the "A" operand (query rows, 8
//                       positions per lane); the "B" operand is 8 positions of one value channel
//                       per lane.
// The operand fragments of a lane are 16 (keys) or 8 (values) bytes that lie 128 or more bytes
// apart in the [position][channel] memory: read from there, every load instruction touches 32
// cache lines for 1 KB or 512 bytes.  The memory is static per batch, so it is stored a second time
// in the order the fragments are read (pack_memory_kernel, once per san_encode): 8 KB per
// (sentence, head, block), every load instruction of a wave reading consecutive bytes.
// Both products are exact in fp32 per term (bf16 x bf16); the weights enter as a sum of two
// bf16 terms (p = hi + lo, relative error 2^-17), i.e. they keep their fp32 meaning.  The
// running maximum / sum / rescaling is the usual one-pass softmax.  No LDS.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace san {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kMfmaDh = 64;       // head width this kernel is written for
constexpr int kMfmaBlock = 32;    // positions per block
constexpr int kMfmaChunk = 8192;  // bytes of one packed block: 4 KB of key fragments, 4 KB of value fragments
template <int I> using IC = std::integral_constant<int, I>;

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {   // round to nearest even, a in the low half
  bf16x2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(unsigned, v);
}
__device__ __forceinline__ float bf16_lo_f32(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi_f32(unsigned w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float lane_value(float v, int src_lane) {   // src_lane: wave-uniform
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src_lane));
}

// NB > 0: memories of at most NB blocks; every block's keys and values are requested before the
// first score is computed (one memory round trip per wave).  NB == 0: any length; one block in
// registers, refilled as soon as it has been used.
template <int NB>
__global__ __launch_bounds__(256, 2) void attention_kernel_ctx_mfma(AttnParams p) {
  const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wave >= p.groups * p.H) return;                 // whole waves; no barrier in this kernel
  const int g = wave / p.H, h = wave - g * p.H;
  const int n = p.len ? max(0, min(p.len[g], p.lmax)) : p.n_fixed;
  const size_t gs = (size_t)(p.group_map ? p.group_map[g] : g);
  // packed memory of this (sentence, head): kv_blocks chunks; inside a chunk the key fragment of
  // (MFMA step s, half, position) is 16 bytes at ((2 s + half) * 32 + position) * 16, the value
  // fragment part of (channel block cb, step ks, part, half, channel) 8 bytes at
  // 4096 + ((((2 cb + ks) * 2 + part) * 2 + half) * 32 + channel) * 8
  const unsigned char* mem = reinterpret_cast<const unsigned char*>(p.kv_packed) + (gs * p.H + h) * (size_t)p.kv_blocks * kMfmaChunk;
  const bool q_live = l32 < p.rpg;
  const int qrow = g * p.rpg + min(l32, p.rpg - 1);
  const float scale2 = p.scale * 1.44269504088896341f;   // scores in log2 units

  // this lane's query (B operand of K Q^T): channels (2 s + half) * 8 .. + 8 of MFMA step s
  u32x4 qf[4];
  {
    const bf16_t* qp = reinterpret_cast<const bf16_t*>(p.q) + (size_t)qrow * p.ldq + h * kMfmaDh + half * 8;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      qf[s] = *reinterpret_cast<const u32x4*>(qp + s * 16);
      if (!q_live) qf[s] = u32x4{0u, 0u, 0u, 0u};
    }
  }
  const int nblk = (n + kMfmaBlock - 1) / kMfmaBlock;
  // Fragments of one block.  Keys (A operand): position b * 32 + l32, the same channels as the
  // query.  Values (B operand): channel cb * 32 + l32, positions b * 32 + ks * 16 + 4 * half +
  // {0..3} and the same + 8: the positions whose weights this lane's half holds in registers
  // 8 ks .. 8 ks + 7 after K Q^T.  Positions past the memory's end are zeros in the packed copy.
  constexpr int NS = NB > 0 ? NB : 1;
  u32x4 kf[NS][4], vf[NS][2][2];
  // (lanes whose positions lie past the memory's end load nothing: those fragments are zeros)
  auto load_keys = [&](int b, auto slot) {
    const unsigned char* kp = mem + (size_t)b * kMfmaChunk + (half * 32 + l32) * 16;
    const bool live = b * kMfmaBlock + l32 < n;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      kf[slot][s] = u32x4{0u, 0u, 0u, 0u};
      if (live) kf[slot][s] = *reinterpret_cast<const u32x4*>(kp + s * 1024);
    }
  };
  auto load_values = [&](int b, auto slot) {
    const unsigned char* vp = mem + (size_t)b * kMfmaChunk + 4096 + (half * 32 + l32) * 8;
    const int p0 = b * kMfmaBlock + 4 * half;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        u32x2 a = u32x2{0u, 0u}, c = u32x2{0u, 0u};
        if (p0 + ks * 16 < n) a = *reinterpret_cast<const u32x2*>(vp + ((cb * 2 + ks) * 2 + 0) * 512);
        if (p0 + ks * 16 + 8 < n) c = *reinterpret_cast<const u32x2*>(vp + ((cb * 2 + ks) * 2 + 1) * 512);
        vf[slot][cb][ks] = u32x4{a.x, a.y, c.x, c.y};
      }
  };

  float m_run = -INFINITY, l_run = 0.f;
  f32x16 acc[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;
  float* Sg = (p.emit && q_live) ? p.S_buf + ((size_t)qrow * p.H + h) * p.ldS : nullptr;

  if (nblk > 0) {   // unconditional requests (a block index past the end re-reads the last block)
    load_keys(0, IC<0>{});
    if constexpr (NB > 1) load_keys(min(1, nblk - 1), IC<(NB > 1 ? 1 : 0)>{});
    if constexpr (NB > 2) load_keys(min(2, nblk - 1), IC<(NB > 2 ? 2 : 0)>{});
    if constexpr (NB > 3) load_keys(min(3, nblk - 1), IC<(NB > 3 ? 3 : 0)>{});
    load_values(0, IC<0>{});
    if constexpr (NB > 1) load_values(min(1, nblk - 1), IC<(NB > 1 ? 1 : 0)>{});
    if constexpr (NB > 2) load_values(min(2, nblk - 1), IC<(NB > 2 ? 2 : 0)>{});
    if constexpr (NB > 3) load_values(min(3, nblk - 1), IC<(NB > 3 ? 3 : 0)>{});
  }
  auto block = [&](int b, auto slot) {
    const int nxt = min(b + 1, nblk - 1);   // NB == 0, past the end: the last block again (loaded, not used)
    f32x16 st;
#pragma unroll
    for (int r = 0; r < 16; ++r) st[r] = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s)
      st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[slot][s]), __builtin_bit_cast(bf16x8, qf[s]),
                                                   st, 0, 0, 0);
    if constexpr (NB == 0) load_keys(nxt, slot);   // the next block's keys travel during this block's softmax and P V
    // st[r]: position b * 32 + 4 * half + 8 * (r / 4) + r % 4, query l32
    float bm = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int pos = b * kMfmaBlock + 4 * half + 8 * (r >> 2) + (r & 3);
      st[r] = pos < n ? st[r] * scale2 : -INFINITY;
      bm = fmaxf(bm, st[r]);
    }
    if (Sg) {
      float* sb = Sg + b * kMfmaBlock + 4 * half;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (b * kMfmaBlock + 4 * half + 8 * (r >> 2) + (r & 3) < n) sb[8 * (r >> 2) + (r & 3)] = st[r];   // raw; normalised below
    }
    bm = max_xor32(bm);                               // finite: the block has a position < n
    const float m_new = fmaxf(m_run, bm);
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 at the first block
    float bs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      st[r] = __builtin_amdgcn_exp2f(st[r] - m_new);  // 0 for masked positions
      bs += st[r];
    }
    bs = sum_xor32(bs);
    l_run = l_run * corr + bs;
    m_run = m_new;
    // weights as two bf16 terms, registers 8 ks .. 8 ks + 7 = the 8 k-values of MFMA step ks
    u32x4 ph[2], pl[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      unsigned hw[4], lw[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a0 = st[8 * ks + 2 * e], a1 = st[8 * ks + 2 * e + 1];
        hw[e] = pack_bf16(a0, a1);
        lw[e] = pack_bf16(a0 - bf16_lo_f32(hw[e]), a1 - bf16_hi_f32(hw[e]));
      }
      ph[ks] = u32x4{hw[0], hw[1], hw[2], hw[3]};
      pl[ks] = u32x4{lw[0], lw[1], lw[2], lw[3]};
    }
    // accumulator rows are queries 4 * half + 8 * i + j (register 4 i + j): rescale by the
    // owner lane's factor (lane = query), then add this block
    if (b > 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (8 * i >= p.rpg) break;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float c0 = lane_value(corr, 8 * i + j), c1 = lane_value(corr, 8 * i + j + 4);
          const float cr = half ? c1 : c0;
          acc[0][4 * i + j] *= cr;
          acc[1][4 * i + j] *= cr;
        }
      }
    }
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ph[ks]),
                                                          __builtin_bit_cast(bf16x8, vf[slot][cb][ks]), acc[cb], 0, 0, 0);
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pl[ks]),
                                                          __builtin_bit_cast(bf16x8, vf[slot][cb][ks]), acc[cb], 0, 0, 0);
      }
    if constexpr (NB == 0) load_values(nxt, slot);
  };
  if constexpr (NB == 0) {
    for (int b = 0; b < nblk; ++b) block(b, IC<0>{});
  } else {
    if (nblk > 0) block(0, IC<0>{});
    if constexpr (NB > 1) if (nblk > 1) block(1, IC<(NB > 1 ? 1 : 0)>{});
    if constexpr (NB > 2) if (nblk > 2) block(2, IC<(NB > 2 ? 2 : 0)>{});
    if constexpr (NB > 3) if (nblk > 3) block(3, IC<(NB > 3 ? 3 : 0)>{});
  }

  const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
  // ---- the block's weights S (Eq. 1), for the followers of a weight-sharing block / debugging
  if (Sg) {
    for (int b = 0; b < nblk; ++b) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int pos = b * kMfmaBlock + 4 * half + 8 * (r >> 2) + (r & 3);
        if (pos < n) Sg[pos] = __builtin_amdgcn_exp2f(Sg[pos] - m_run) * inv;
      }
    }
    if (p.zero_tail)
      for (int j = n + half; j < p.ldS; j += 2) Sg[j] = 0.f;
  }
  // ---- out = P V / sum: lane = channel, registers = queries
  bf16_t* Op = reinterpret_cast<bf16_t*>(p.out);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (8 * i >= p.rpg) break;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float i0 = lane_value(inv, 8 * i + j), i1 = lane_value(inv, 8 * i + j + 4);
      const float iv = half ? i1 : i0;
      const int q = 4 * half + 8 * i + j;
      if (q < p.rpg) {
        bf16_t* o = Op + (size_t)(g * p.rpg + q) * p.ldo + h * kMfmaDh + l32;
        o[0] = from_f32<bf16_t>(acc[0][4 * i + j] * iv);
        o[32] = from_f32<bf16_t>(acc[1][4 * i + j] * iv);
      }
    }
  }
}

bool attention_ctx_mfma_fits(int dtype, const AttnParams& p) {
  return dtype == 1 && p.dh == kMfmaDh && !p.self_mode && !p.causal && !p.apply && p.rpg >= 1 && p.rpg <= 32 &&
         p.kv_packed && p.lmax <= p.kv_blocks * kMfmaBlock && p.ldq % 8 == 0;
}

hipError_t launch_attention_ctx_mfma(const AttnParams& p, hipStream_t stream) {
  if (!attention_ctx_mfma_fits(1, p) || (p.emit && !p.S_buf)) return hipErrorInvalidValue;
  const long waves = (long)p.groups * p.H;
  if (waves <= 0) return hipSuccess;
  const dim3 grid((unsigned)((waves + 3) / 4)), blk(256);
  const int nb = (p.lmax + kMfmaBlock - 1) / kMfmaBlock;
  if (nb <= 1) hipLaunchKernelGGL(attention_kernel_ctx_mfma<1>, grid, blk, 0, stream, p);
  else if (nb == 2) hipLaunchKernelGGL(attention_kernel_ctx_mfma<2>, grid, blk, 0, stream, p);
  else if (nb == 3) hipLaunchKernelGGL(attention_kernel_ctx_mfma<3>, grid, blk, 0, stream, p);
  else if (nb == 4) hipLaunchKernelGGL(attention_kernel_ctx_mfma<4>, grid, blk, 0, stream, p);
  else hipLaunchKernelGGL(attention_kernel_ctx_mfma<0>, grid, blk, 0, stream, p);
  return hipGetLastError();
}

// One block of 32 positions of one (sentence, head): k / v rows (g * n_pos + pos) * ld + h * 64 -> the packed
// chunk described in attention_kernel_ctx_mfma; positions >= n_pos become zeros.
__global__ __launch_bounds__(256) void pack_memory_kernel(const bf16_t* k, long long ldk, const bf16_t* v, long long ldv,
                                                          int n_pos, int H, unsigned char* out, int kv_blocks) {
  __shared__ unsigned short tile[kMfmaDh][kMfmaBlock + 2];   // values, [channel][position]
  const int gh = blockIdx.x, g = gh / H, h = gh - g * H, b = blockIdx.y, t = threadIdx.x;
  unsigned char* chunk = out + ((size_t)gh * kv_blocks + b) * kMfmaChunk;
  const int pos_l = t >> 3, c8 = t & 7, pos = b * kMfmaBlock + pos_l;   // 8 channels c8 * 8 .. of one position
  uint4 kw = make_uint4(0u, 0u, 0u, 0u), vw = kw;
  if (pos < n_pos) {
    kw = *reinterpret_cast<const uint4*>(k + ((size_t)g * n_pos + pos) * ldk + h * kMfmaDh + c8 * 8);
    vw = *reinterpret_cast<const uint4*>(v + ((size_t)g * n_pos + pos) * ldv + h * kMfmaDh + c8 * 8);
  }
  // channels c8 * 8 .. + 8 = MFMA step c8 / 2, half c8 % 2: fragment index 2 s + half = c8
  *reinterpret_cast<uint4*>(chunk + (c8 * 32 + pos_l) * 16) = kw;
  const unsigned ws[4] = {vw.x, vw.y, vw.z, vw.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    tile[c8 * 8 + 2 * e][pos_l] = (unsigned short)(ws[e] & 0xffffu);
    tile[c8 * 8 + 2 * e + 1][pos_l] = (unsigned short)(ws[e] >> 16);
  }
  __syncthreads();
  // thread t writes the 8-byte items 2 t and 2 t + 1: item = (((2 cb + ks) * 2 + part) * 2 + half) * 32 + c
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const int item = 2 * t + w, c = item & 31, hf = (item >> 5) & 1, part = (item >> 6) & 1, ks = (item >> 7) & 1,
              cb = item >> 8;
    const int ch = cb * 32 + c, p0 = ks * 16 + part * 8 + hf * 4;
    uint2 o;
    o.x = (unsigned)tile[ch][p0] | ((unsigned)tile[ch][p0 + 1] << 16);
    o.y = (unsigned)tile[ch][p0 + 2] | ((unsigned)tile[ch][p0 + 3] << 16);
    *reinterpret_cast<uint2*>(chunk + 4096 + item * 8) = o;
  }
}

hipError_t launch_pack_memory(const void* k, long long ldk, const void* v, long long ldv, int groups, int n_pos, int H,
                              void* out, int kv_blocks, hipStream_t stream) {
  if (groups <= 0 || n_pos <= 0) return hipSuccess;
  const int nblk = (n_pos + kMfmaBlock - 1) / kMfmaBlock;
  if (nblk > kv_blocks || ldk % 8 || ldv % 8) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_memory_kernel, dim3((unsigned)(groups * H), (unsigned)nblk), dim3(256), 0, stream,
                     reinterpret_cast<const bf16_t*>(k), ldk, reinterpret_cast<const bf16_t*>(v), ldv, n_pos, H,
                     reinterpret_cast<unsigned char*>(out), kv_blocks);
  return hipGetLastError();
}

}  // namespace san
