// Projection / FFN / output-layer GEMMs on CDNA4 matrix cores.
//
// out[m][n] = sum_k A[m][k] * W[n][k]: both operands are contiguous along k, so a
// lane's MFMA operand fragment is one 16-byte load.  A block of WM x WN waves
// owns a (32*WM*TM) x (32*WN*TN) tile of the output; k is walked in chunks of 128
// (bf16: 256) bytes per row.  Decode-time GEMMs are small (M = batch*beam rows) and therefore
// latency-bound, so the kernel is built to keep many loads in flight: a queue of
// D chunks lives in registers (global loads issued D chunks ahead), each chunk is
// then staged through one of two LDS buffers (rows padded to 144 bytes so that the
// 16-byte fragment reads of 16 neighbouring lanes hit all 64 banks once), and
// GEMMs that feed a LayerNorm are split along k across blocks into fp32 partials
// which the LayerNorm kernel adds up in a fixed order (no atomics, no fences: a
// device-scope fence per block costs more than the whole GEMM on this multi-XCD
// part).  The others keep the whole k range in one block and run the epilogue
// (bias, ReLU, scatter into the q buffer / key cache / value cache) themselves.
// The activation rows feed the MFMA "A" side and the weight rows the "B" side, so
// the 32 lanes of a half-wave hold 32 consecutive output columns of one row and
// every epilogue store writes whole 128-byte row segments (16-byte stores per lane
// with the roles swapped measured slower on the wide output layer: each store
// instruction then touched 64 different cache lines).
#include <atomic>

#include "common.h"
#include "kernels.h"

namespace san {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte fragment as a first-class vector


template <typename T> __device__ __forceinline__ void mma_frag(f32x16& acc, const u32x4& w, const u32x4& x);   // acc += w-rows x x-rows^T

// fp32: a 16-byte fragment is 4 k-values -> 4 rank-2 updates (32x32x2).  Lanes
// 0-31 carry k = 0..3 of the 32-byte sub-step, lanes 32-63 carry k = 4..7; the
// pairing of k-values inside an instruction is irrelevant as both operands use it.
template <> __device__ __forceinline__ void mma_frag<float>(f32x16& acc, const u32x4& w, const u32x4& x) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w.x), __uint_as_float(x.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w.y), __uint_as_float(x.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w.z), __uint_as_float(x.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w.w), __uint_as_float(x.w), acc, 0, 0, 0);
}
// bf16: a 16-byte fragment is 8 k-values -> one 32x32x16 instruction.
template <> __device__ __forceinline__ void mma_frag<bf16_t>(f32x16& acc, const u32x4& w, const u32x4& x) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), acc, 0, 0, 0);
}

// CB = bytes of k per row in one LDS stage (128 or 256); rows are padded by 16
// bytes, which keeps the 16-byte fragment reads of 16 neighbouring lanes on
// distinct banks for both sizes.
// CAND: the tile is not stored.  Its rows go through LDS to groups of 16 lanes that
// reduce each row of BN columns to (max, sum of exp(x - max)) and a few entries that
// include its p.cand_k largest (see GemmParams::cand_*): the beam step needs nothing
// else of the output layer.
template <typename T, int WM, int WN, int TM, int TN, int KW, int D, int CB, bool CAND>
__global__ __launch_bounds__(WM* WN* KW * 64) void gemm_kernel(GemmParams p) {
  constexpr int kRowBytes = CB + 16;
  constexpr int SEGS = CB / 16;                      // 16-byte segments of a row chunk
  constexpr int NG = WM * WN * 64;                   // threads of one k-group
  constexpr int BM = 32 * WM * TM, BN = 32 * WN * TN;
  constexpr int EPC = CB / (int)sizeof(T);           // elements per chunk
  constexpr int RPP = NG / SEGS;                     // rows covered by one pass of 16-byte loads
  constexpr int LA = BM / RPP, LB = BN / RPP;        // 16-byte loads per thread per chunk
  constexpr int STAGE = 2 * (BM + BN) * kRowBytes;   // LDS bytes of one k-group (double buffered)
  static_assert(BM % RPP == 0 && BN % RPP == 0 && D % 2 == 0, "tile shape");
  static_assert(KW == 1 || (KW - 1) * (WM * WN) * TM * TN * 16 * 64 * 4 <= KW * STAGE, "reduction fits the stages");
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int kg = wid / (WM * WN), w_in = wid % (WM * WN);   // k-group, wave inside the group
  const int tg = tid % NG;
  const int wm = w_in % WM, wn = w_in / WM;
  const int l32 = lane & 31, kh = lane >> 5;
  // Tile of this block.  Workgroups go to the 8 XCDs round-robin by their linear
  // index, and every XCD has its own L2.  With the natural (x = column tile, y =
  // row tile) order the row tiles that share a weight tile land on one XCD only
  // when the number of column tiles is a multiple of 8; otherwise (the output
  // layer: 250 or 125 column tiles) the launcher asks for this mapping: XCD c takes
  // the column tiles c, c+8, ... and runs the row tiles of one column tile back to
  // back, so a weight tile leaves HBM once.
  int tile_x = blockIdx.x, tile_y = blockIdx.y;
  if (p.xcd_rows > 0) {
    const int slot = blockIdx.x >> 3;
    tile_y = slot % p.xcd_rows;
    tile_x = (slot / p.xcd_rows) * 8 + (blockIdx.x & 7);
    if (tile_x * BN >= p.N) return;
  }
  const int m0 = tile_y * BM, n0 = tile_x * BN;
  unsigned char* Xs = smem + kg * STAGE;           // [2][BM][144]
  unsigned char* Ws = Xs + 2 * BM * kRowBytes;     // [2][BN][144]

  // The step counter and the bias are requested now.  The bias goes into the
  // accumulators' start value (of k-group 0), so that no load is pending when the
  // epilogue runs: a pending load makes the compiler wait for *all* memory traffic
  // before every conditional store -- the counter it waits on also counts the
  // stores -- which serialises the 16 stores of a tile (+1.3 us on a 10 us GEMM).
  const int t_step = p.t_dev ? *p.t_dev : 0;
  float bias_v[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + (wn * TN + j) * 32 + l32;
    bias_v[j] = (p.bias && p.out_kind != 2 && kg == 0 && n < p.N) ? to_f32(reinterpret_cast<const T*>(p.bias)[n]) : 0.f;
  }
  const int nchunks = p.K / EPC;
  const int cps = p.cps;   // chunks per k-split, (nchunks + ksplit - 1) / ksplit, divided on the host
  const int c_begin = blockIdx.z * cps;
  const int c_end = min(nchunks, c_begin + cps);
  // inside the block the chunks are dealt round-robin to the KW k-groups; every
  // group runs the same number of iterations so that the barriers line up
  const int iters = (max(c_end - c_begin, 0) + KW - 1) / KW;

  const T* A = reinterpret_cast<const T*>(p.A);
  const T* W = reinterpret_cast<const T*>(p.W);
  const int lrow = tg / SEGS, lseg = tg % SEGS;  // this thread's row and 16-byte segment of a chunk
  const T* a_ptr[LA];
  const T* w_ptr[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i)
    a_ptr[i] = A + (size_t)min(m0 + lrow + RPP * i, p.M - 1) * p.lda + lseg * (16 / sizeof(T));
#pragma unroll
  for (int i = 0; i < LB; ++i)
    w_ptr[i] = W + (size_t)min(n0 + lrow + RPP * i, p.N - 1) * p.K + lseg * (16 / sizeof(T));

  // Register queue of chunks in flight (macros, not lambdas, so that every index
  // is a compile-time constant and the queue stays in registers).
  u32x4 qa[D][LA], qw[D][LB];
#define SAN_CHUNK(i_) (c_begin + kg + KW * (i_))
#define SAN_LOAD_GLOBAL(c_, s_)                                                              \
  do {                                                                                       \
    const size_t koff_ = (size_t)(c_) * EPC;                                                 \
    _Pragma("unroll") for (int i_ = 0; i_ < LA; ++i_)                                        \
        qa[s_][i_] = *reinterpret_cast<const u32x4*>(a_ptr[i_] + koff_);                     \
    _Pragma("unroll") for (int i_ = 0; i_ < LB; ++i_)                                        \
        qw[s_][i_] = *reinterpret_cast<const u32x4*>(w_ptr[i_] + koff_);                     \
  } while (0)
#define SAN_STORE_LDS(buf_, s_)                                                              \
  do {                                                                                       \
    _Pragma("unroll") for (int i_ = 0; i_ < LA; ++i_)                                        \
        *reinterpret_cast<u32x4*>(Xs + ((buf_) * BM + lrow + RPP * i_) * kRowBytes + lseg * 16) = qa[s_][i_]; \
    _Pragma("unroll") for (int i_ = 0; i_ < LB; ++i_)                                        \
        *reinterpret_cast<u32x4*>(Ws + ((buf_) * BN + lrow + RPP * i_) * kRowBytes + lseg * 16) = qw[s_][i_]; \
  } while (0)

  f32x16 acc[TM][TN];

#define SAN_MMA(buf_)                                                                                      \
  do {                                                                                                     \
    const unsigned char* xs_ = Xs + ((buf_) * BM + wm * 32 * TM + l32) * kRowBytes + kh * 16;              \
    const unsigned char* ws_ = Ws + ((buf_) * BN + wn * 32 * TN + l32) * kRowBytes + kh * 16;              \
    _Pragma("unroll") for (int sub_ = 0; sub_ < CB / 32; ++sub_) {                                         \
      u32x4 xf_[TM], wf_[TN];                                                                              \
      _Pragma("unroll") for (int i_ = 0; i_ < TM; ++i_)                                                    \
          xf_[i_] = *reinterpret_cast<const u32x4*>(xs_ + i_ * 32 * kRowBytes + sub_ * 32);                \
      _Pragma("unroll") for (int j_ = 0; j_ < TN; ++j_)                                                    \
          wf_[j_] = *reinterpret_cast<const u32x4*>(ws_ + j_ * 32 * kRowBytes + sub_ * 32);                \
      _Pragma("unroll") for (int i_ = 0; i_ < TM; ++i_)                                                    \
          _Pragma("unroll") for (int j_ = 0; j_ < TN; ++j_) mma_frag<T>(acc[i_][j_], xf_[i_], wf_[j_]);    \
    }                                                                                                      \
  } while (0)

  // The loads of the steady state are unconditional on purpose.  The hardware
  // counts outstanding loads in order, and the compiler must assume the worst
  // about loads that sit behind a branch: with a conditional refill it waited for
  // *every* load in flight before each chunk's LDS store, which cut the look-ahead
  // of the register queue from D chunks to one and made every chunk cost a full
  // memory latency.  Chunk indices past the end are clamped (the data is loaded
  // and never used) instead of skipped.
#define SAN_INIT_ACC()                                                                   \
  do {                                                                                   \
    _Pragma("unroll") for (int i_ = 0; i_ < TM; ++i_)                                    \
        _Pragma("unroll") for (int j_ = 0; j_ < TN; ++j_)                                \
            _Pragma("unroll") for (int v_ = 0; v_ < 16; ++v_) acc[i_][j_][v_] = bias_v[j_]; \
  } while (0)   /* column n of every row this lane holds */
  if (iters <= 0) {   // an empty k-slice of a split GEMM (those carry no bias): contributes zeros
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  }
  if (iters > 0) {
    const int c_last = c_end - 1;
#define SAN_CHUNK_C(i_) min(SAN_CHUNK(i_), c_last)
#pragma unroll
    for (int s = 0; s < D; ++s) SAN_LOAD_GLOBAL(SAN_CHUNK_C(s), s);
    // The accumulators start from the bias, which must not stall the loads above:
    // the asm ties the start values to this point of the program (the loads
    // cannot sink below a memory clobber, the moves cannot rise above it), where
    // waiting for the bias means waiting for the oldest load only.
#pragma unroll
    for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bias_v[j]) : : "memory");
    SAN_INIT_ACC();
    // steady state: every chunk used here exists, every iteration refills its slot
    const int iters_main = iters > D ? ((iters - D) / D) * D : 0;
    int ib = 0;
    for (; ib < iters_main; ib += D) {
#pragma unroll
      for (int s = 0; s < D; ++s) {
        SAN_STORE_LDS(s & 1, s);                   // D is even, so chunk parity == slot parity
        SAN_LOAD_GLOBAL(SAN_CHUNK_C(ib + s + D), s);
        __syncthreads();                           // one barrier per chunk: the other buffer is still being read
        SAN_MMA(s & 1);
      }
    }
    if (iters % D == 0) {
      // the last D chunks, nothing left to request: straight-line code, so the
      // waits stay exact (the last round may be short for some k-groups)
#pragma unroll
      for (int s = 0; s < D; ++s) {
        const bool live = SAN_CHUNK(ib + s) < c_end;
        if (live) SAN_STORE_LDS(s & 1, s);
        __syncthreads();
        if (live) SAN_MMA(s & 1);
      }
      ib = iters;
    }
    // any other tail: at most 2*D - 1 chunks with conditional refills (conservative waits)
    for (; ib < iters; ib += D) {
#pragma unroll
      for (int s = 0; s < D; ++s) {
        const int it = ib + s;
        if (it < iters) {
          const bool live = SAN_CHUNK(it) < c_end;
          if (live) SAN_STORE_LDS(s & 1, s);
          if (it + D < iters) SAN_LOAD_GLOBAL(SAN_CHUNK_C(it + D), s);
          __syncthreads();
          if (live) SAN_MMA(s & 1);
        }
      }
    }
#undef SAN_CHUNK_C
  }
#undef SAN_MMA
#undef SAN_INIT_ACC
#undef SAN_CHUNK
#undef SAN_LOAD_GLOBAL
#undef SAN_STORE_LDS

  if (KW > 1) {
    // ---- add up the k-groups through LDS, in group order (deterministic)
    __syncthreads();   // all stages are dead now
    float* red = reinterpret_cast<float*>(smem);   // [KW-1][waves per group][TM*TN*16][64]
    if (kg > 0) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            red[((((kg - 1) * (WM * WN) + w_in) * (TM * TN) + i * TN + j) * 16 + v) * 64 + lane] = acc[i][j][v];
    }
    __syncthreads();
    if (kg > 0) return;
#pragma unroll
    for (int g = 1; g < KW; ++g)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            acc[i][j][v] += red[((((g - 1) * (WM * WN) + w_in) * (TM * TN) + i * TN + j) * 16 + v) * 64 + lane];
  }

  if constexpr (CAND) {
    static_assert(KW == 1, "the tile is complete in every wave");
    constexpr int LDW = BN + 4;                    // fp32 words per LDS row (16-byte multiple, rows 4 banks apart)
    constexpr int PR = BM * LDW * 4 <= STAGE ? BM : (BM / 2 * LDW * 4 <= STAGE ? BM / 2 : BM / 4);   // rows per pass
    constexpr int VPL = BN / 16;                   // values of a row per lane
    constexpr int NGRP = NG / 16;                  // 16-lane groups, one row each at a time
    static_assert(PR % 32 == 0 && PR * LDW * 4 <= STAGE && PR % NGRP == 0 && VPL % 4 == 0, "candidate pass shape");
    constexpr int kNoCol = 0x7fffffff;
    float* tile = reinterpret_cast<float*>(smem);
    const int l16 = lane & 15, grp = tid >> 4;
    const int kc = p.cand_k, ntiles = p.cand_tiles, slots = 2 * p.cand_k;   // slots <= 16 lanes
    for (int pass = 0; pass < BM / PR; ++pass) {
      __syncthreads();   // the k loop's stages (or the previous pass's rows) are dead
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int rb = (wm * TM + i) * 32 - pass * PR;
        if (rb < 0 || rb >= PR) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = (wn * TN + j) * 32 + l32;
          const bool live = n0 + col < p.N;
#pragma unroll
          for (int v = 0; v < 16; ++v)
            tile[(rb + (v >> 2) * 8 + kh * 4 + (v & 3)) * LDW + col] = live ? acc[i][j][v] : -INFINITY;
        }
      }
      __syncthreads();
      for (int r = grp; r < PR; r += NGRP) {
        // lane l holds columns c*64 + 4*l .. +3 (c = 0 .. VPL/4-1): val[q] is column (q/4)*64 + 4*l + q%4,
        // ascending in q
        float val[VPL];
        const float* rp = tile + r * LDW + 4 * l16;
#pragma unroll
        for (int c = 0; c < VPL / 4; ++c) {
          const float4 q4 = *reinterpret_cast<const float4*>(rp + c * 64);
          val[4 * c] = q4.x; val[4 * c + 1] = q4.y; val[4 * c + 2] = q4.z; val[4 * c + 3] = q4.w;
        }
        float lm = val[0];
#pragma unroll
        for (int q = 1; q < VPL; ++q) lm = fmaxf(lm, val[q]);
        const float row_m = group_max<16>(lm);       // finite: a tile has at least one live column
        // Threshold: the kc-th largest distinct lane maximum.  At least kc entries of the row are >= it,
        // so the row's kc largest all are, and usually hardly any other entry is.
        float thr = row_m;
        for (int round = 1; round < kc; ++round) thr = group_max<16>(lm < thr ? lm : -INFINITY);
        float es = 0.f;
        int cnt = 0;
        const float nm2 = -row_m * 1.44269504088896341f;
#pragma unroll
        for (int q = 0; q < VPL; ++q) {
          es += __builtin_amdgcn_exp2f(fmaf(val[q], 1.44269504088896341f, nm2));   // 0 for the columns past N (-inf)
          cnt += val[q] >= thr ? 1 : 0;
        }
        const float row_s = group_sum<16>(es);
        // entries >= thr go to the tile's slots in lane order: prefix count over the 16 lanes
        int incl = cnt;
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x111, 0xF, 0xF, true);   // row_shr:1, zero shifted in
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x112, 0xF, 0xF, true);   // row_shr:2
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x114, 0xF, 0xF, true);   // row_shr:4
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x118, 0xF, 0xF, true);   // row_shr:8
        int total = cnt;
        total += dpp_mov_i<kDppQuadSwap1>(total);
        total += dpp_mov_i<kDppQuadSwap2>(total);
        total += dpp_mov_i<kDppRowHalfMirror>(total);
        total += dpp_mov_i<kDppRowMirror>(total);
        const int m = m0 + pass * PR + r;
        const bool row_live = m < p.M;
        // 32-bit slot offsets from the uniform base pointers (the launcher checks the size): one
        // add per store instead of 64-bit pointer arithmetic in every lane
        const unsigned slot = ((unsigned)min(m, p.M - 1) * (unsigned)ntiles + (unsigned)tile_x) * (unsigned)slots;
        char* const cvb = reinterpret_cast<char*>(p.cand_v);
        char* const cib = reinterpret_cast<char*>(p.cand_i);
        if (total <= slots) {
          if (row_live) {
            unsigned off = (slot + (unsigned)(incl - cnt)) * 4u;
            const int colb = n0 + 4 * l16;
#pragma unroll
            for (int q = 0; q < VPL; ++q) {
              if (val[q] >= thr) {
                *reinterpret_cast<float*>(cvb + off) = val[q];
                *reinterpret_cast<int*>(cib + off) = colb + (q >> 2) * 64 + (q & 3);
                off += 4u;
              }
            }
            if (l16 >= total && l16 < slots) {
              *reinterpret_cast<float*>(cvb + (slot + l16) * 4u) = -INFINITY;
              *reinterpret_cast<int*>(cib + (slot + l16) * 4u) = kNoCol;
            }
          }
        } else {
          // too many entries at the threshold (masses of equal values, or fewer than kc live columns):
          // kc rounds, each taking the best entry left (higher value, then lower column)
          float out_v = -INFINITY;
          int out_c = kNoCol;
          for (int round = 0; round < kc; ++round) {
            float bv = val[0];
            int bq = 0;
#pragma unroll
            for (int q = 1; q < VPL; ++q)
              if (val[q] > bv) { bv = val[q]; bq = q; }
            int bc = (bq >> 2) * 64 + 4 * l16 + (bq & 3);
#define SAN_BEST16(CTRL)                                                        \
            {                                                                    \
              const float ov_ = dpp_mov<CTRL>(bv);                               \
              const int oc_ = dpp_mov_i<CTRL>(bc);                               \
              if (ov_ > bv || (ov_ == bv && oc_ < bc)) { bv = ov_; bc = oc_; }   \
            }
            SAN_BEST16(kDppQuadSwap1) SAN_BEST16(kDppQuadSwap2) SAN_BEST16(kDppRowHalfMirror) SAN_BEST16(kDppRowMirror)
#undef SAN_BEST16
            if (l16 == round) { out_v = bv; out_c = bc; }
#pragma unroll
            for (int q = 0; q < VPL; ++q)
              if ((q >> 2) * 64 + 4 * l16 + (q & 3) == bc) val[q] = -INFINITY;
          }
          if (row_live && l16 < slots) {
            *reinterpret_cast<float*>(cvb + (slot + l16) * 4u) = out_v;
            *reinterpret_cast<int*>(cib + (slot + l16) * 4u) = out_v == -INFINITY ? kNoCol : n0 + out_c;
          }
        }
        if (row_live && l16 == 0)
          *reinterpret_cast<float2*>(p.cand_ms + ((size_t)m * ntiles + tile_x) * 2) = make_float2(row_m, row_s);
      }
    }
    if (p.bump && tile_x == 0 && tile_y == 0 && tid == 0) *p.bump = *p.bump + 1;
    return;
  }

  // acc[i][j][v]: output row m = tile_m + (v/4)*8 + kh*4 + (v%4), column n = tile_n + l32.
  // For a fixed v the 32 lanes of a half-wave hold 32 consecutive columns of one
  // row, so every store instruction writes two contiguous 128-byte (fp32) row
  // segments -- whole cache lines, which matters for the wide output layer.
  // Row offsets: one 64-bit product per 32x32 tile (its first row); the other 15
  // rows are that plus a compile-time multiple of the row stride.
  if (p.out_kind == 2) {
    // ---- fp32 partials [ksplit][M][N]; the consumer (LayerNorm kernel) adds them up in a fixed order
    float* part = reinterpret_cast<float*>(p.out[0]) + (size_t)blockIdx.z * p.M * p.N;
    const size_t ld = (size_t)p.N;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = n0 + (wn * TN + j) * 32 + l32;
        const int mrow = m0 + (wm * TM + i) * 32 + kh * 4;
        float* dst = part + (size_t)mrow * ld + n;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int dm = (v >> 2) * 8 + (v & 3);
          if (mrow + dm < p.M && n < p.N) dst[dm * ld] = acc[i][j][v];
        }
      }
    return;
  }

  // ---- epilogue: ReLU, scatter into up to three column segments (the bias is already in)
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + (wn * TN + j) * 32 + l32;
    if (n >= p.N) continue;
    const int s = ((unsigned)n >= (unsigned)p.seg_w) + ((unsigned)n >= 2u * (unsigned)p.seg_w);   // n / seg_w, at most 2
    const int nn = n - s * p.seg_w;
    void* obase = s == 0 ? p.out[0] : (s == 1 ? p.out[1] : p.out[2]);
    const size_t ld = (size_t)(s == 0 ? p.ldo[0] : (s == 1 ? p.ldo[1] : p.ldo[2]));
    const long long ts = s == 0 ? p.tstride[0] : (s == 1 ? p.tstride[1] : p.tstride[2]);
    const size_t base = (size_t)t_step * ts + nn;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int mrow = m0 + (wm * TM + i) * 32 + kh * 4;
      const size_t row0 = base + (size_t)mrow * ld;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int dm = (v >> 2) * 8 + (v & 3);
        if (mrow + dm >= p.M) continue;
        float val = acc[i][j][v];
        if (p.relu) val = fmaxf(val, 0.f);
        const size_t off = row0 + dm * ld;
        if (p.out_kind == 1) reinterpret_cast<float*>(obase)[off] = val;
        else reinterpret_cast<T*>(obase)[off] = from_f32<T>(val);
      }
    }
  }
  if (p.bump && tile_x == 0 && tile_y == 0 && tid == 0) *p.bump = *p.bump + 1;
}

template <typename T, int WM, int WN, int TM, int TN, int KW, int D, int CB = 128, bool CAND = false>
static hipError_t launch_tile(const GemmParams& p, hipStream_t stream) {
  constexpr int BM = 32 * WM * TM, BN = 32 * WN * TN;
  constexpr int kRowBytes = CB + 16;
  dim3 grid((p.N + BN - 1) / BN, (p.M + BM - 1) / BM, p.ksplit);
  const size_t smem = (size_t)KW * 2 * (BM + BN) * kRowBytes;
  if (smem > 64 * 1024) {
    // the limit is an attribute of the function on each device: set it once per device
    // (bit = device ordinal; a second thread that races here only sets it twice)
    static std::atomic<unsigned long long> raised{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (!(raised.load(std::memory_order_acquire) & bit)) {
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<T, WM, WN, TM, TN, KW, D, CB, CAND>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return e;
      raised.fetch_or(bit, std::memory_order_release);
    }
  }
  GemmParams q = p;
  q.xcd_rows = 0;
  {
    const int nchunks = p.K / (CB / (int)sizeof(T));
    q.cps = (nchunks + p.ksplit - 1) / p.ksplit;
  }
  if (grid.x % 8 != 0 && grid.y > 1 && grid.z == 1) {
    q.xcd_rows = (int)grid.y;
    grid = dim3((grid.x + 7) / 8 * 8 * grid.y, 1, 1);
  }
  hipLaunchKernelGGL((gemm_kernel<T, WM, WN, TM, TN, KW, D, CB, CAND>), grid, dim3(WM * WN * KW * 64), smem, stream, q);
  return hipGetLastError();
}

// Tile choice: 0 = 64x64 or smaller (2x2 waves and the k-group shapes below);
// 1 = 128x128 once that still gives ~one block per CU (the output layer);
// 2 = 256x256 (bf16 only) once that does; 3 = see below.  The wide output layer is bound by
// the operand traffic between L2 and the CUs, |X| * N/BN + |W| * M/BM, so the
// biggest tile that still fills the chip wins: measured on the output layer,
// fp32 M = 256: 128x128 with 16 waves 69 us (8 waves 81, 256x128 71-76, 256x256
// 132: half the CUs idle); bf16 M = 512: 256x256 with 16 waves 44-48 us (128x128
// 63, 256x128 51, 128x256 55).
// 3 = 64x128 with 8 waves and 256-byte chunks (bf16 only, K % 128 == 0): the bf16
// decode GEMMs are bound by the same operand traffic (their MFMA time is
// negligible), and this tile moves 25-30 % fewer bytes than 64x64 at the same
// block count after splitting k (Big FFN-1 11.9 -> 9.6 us, FFN-2 12.4 -> 10.7).
// can_split: the GEMM writes partials, so k may be divided over up to 4 blocks to fill the chip
int gemm_pick_tile(int M, int N, int K, int dtype, bool can_split) {
  if (dtype == 1 && M >= 256 && (long)((M + 255) / 256) * ((N + 255) / 256) >= 200) return 2;
  if (M >= 128 && (long)((M + 127) / 128) * ((N + 127) / 128) >= 200) return 1;
  if (dtype == 1 && K % 128 == 0 && (long)((M + 63) / 64) * ((N + 127) / 128) >= (can_split ? 64 : 160)) return 3;
  return 0;
}

int gemm_pick_ksplit(int M, int N, int K, int dtype) {
  const int tile = gemm_pick_tile(M, N, K, dtype, true);
  if (tile == 1 || tile == 2) return 1;
  int ks = 1;
  if (tile == 3) {
    const int nchunks = K / 128;   // 256-byte chunks
    const long blocks = (long)((M + 63) / 64) * ((N + 127) / 128);
    while (blocks * ks < 192 && nchunks / (ks * 2) >= 2 && ks < 16) ks *= 2;
    return ks;
  }
  const int epc = dtype == 1 ? 64 : 32;
  const int nchunks = K / epc;
  const long blocks = (long)((M + 63) / 64) * ((N + 63) / 64);
  // aim for >= 256 blocks (one per CU), keep at least 2 chunks of k per block
  while (blocks * ks < 256 && nchunks / (ks * 2) >= 2 && ks < 16) ks *= 2;
  return ks;
}

// width of the column tiles a GEMM with out_kind 3 cuts the N columns into
static int cand_pick_tile(int M, int N, int K, int dtype) { return gemm_pick_tile(M, N, K, dtype, false); }
int gemm_cand_tile_n(int M, int N, int K, int dtype) {
  const int tile = cand_pick_tile(M, N, K, dtype);
  if (tile == 2) return 256;
  if (tile == 1 || tile == 3) return 128;
  return 64;
}

// out_kind 3: the tiles whose k range is whole in every wave, with the candidate epilogue
static hipError_t launch_gemm_cand(int dtype, const GemmParams& p, hipStream_t stream) {
  const int bn = gemm_cand_tile_n(p.M, p.N, p.K, dtype);
  if (p.cand_k < 1 || p.cand_k > kGemmCandMaxK || !p.cand_ms || !p.cand_v || !p.cand_i || p.ksplit != 1 ||
      p.cand_tiles != (p.N + bn - 1) / bn || (size_t)p.M * p.cand_tiles * 2 * p.cand_k * 4 >= ((size_t)1 << 31))
    return hipErrorInvalidValue;
  const int tile = cand_pick_tile(p.M, p.N, p.K, dtype);
  if (dtype == 1) {
    if (tile == 2) return launch_tile<bf16_t, 4, 4, 2, 2, 1, 2, 128, true>(p, stream);
    if (tile == 3) return launch_tile<bf16_t, 2, 4, 1, 1, 1, 2, 256, true>(p, stream);
    if (tile == 1) return launch_tile<bf16_t, 4, 2, 1, 2, 1, 2, 128, true>(p, stream);
    if (p.K % 128 == 0) return launch_tile<bf16_t, 2, 2, 1, 1, 1, 2, 256, true>(p, stream);
    return launch_tile<bf16_t, 2, 2, 1, 1, 1, 4, 128, true>(p, stream);
  }
  if (tile == 1) return launch_tile<float, 4, 4, 1, 1, 1, 2, 128, true>(p, stream);
  return launch_tile<float, 2, 2, 1, 1, 1, 4, 128, true>(p, stream);
}

hipError_t launch_gemm(int dtype, const GemmParams& p, hipStream_t stream) {
  if (p.M <= 0 || p.N <= 0) return hipSuccess;
  // bf16 MFMAs retire a 128-byte chunk four times faster than fp32 ones, so bf16
  // GEMMs walk k in 256-byte chunks (half the barriers) whenever K allows it
  const bool wide = dtype == 1 && p.K % 128 == 0;
  const int epc = dtype == 1 ? 64 : 32;
  if (p.K <= 0 || p.K % epc != 0 || p.ksplit < 1) return hipErrorInvalidValue;
  if (p.ksplit > 1 && p.out_kind != 2) return hipErrorInvalidValue;   // only partial outputs may be split across blocks
  if (p.out_kind == 3) return launch_gemm_cand(dtype, p, stream);
  int tile = gemm_pick_tile(p.M, p.N, p.K, dtype, p.out_kind == 2);
  if (p.ksplit > 1 && tile != 3) tile = 0;   // only the small tiles split k across blocks
  // A wave's MFMA chain over the whole k range is what bounds a small GEMM, and
  // only waves on different SIMDs run their chains in parallel.  When 64x64 tiles
  // would leave most SIMDs idle, use smaller tiles and deal each tile's k range to
  // 2 or 4 wave groups (reduced through LDS), aiming at ~one wave per SIMD:
  //   shape 1: 64x32 tiles, 2 waves x 2 k-groups;  shape 2: 32x32 tiles, 1 wave x 4 k-groups.
  // (64x32 with 4 k-groups, 32x64 and 64x64 with 2, 32x32 with 8 all measured within 3% of these.)
  const int chunks = (p.K / (dtype == 1 ? 64 : 32) + p.ksplit - 1) / p.ksplit;   // in 128-byte units
  const long tiles64 = (long)((p.M + 63) / 64) * ((p.N + 63) / 64) * p.ksplit;
  int shape = 0;
  if (tile == 0) {
    if (tiles64 <= 64 && chunks >= 8) shape = 2;
    else if (tiles64 <= 192 && chunks >= 4) shape = 1;
  }
  if (dtype == 1) {
    if (tile == 2) return launch_tile<bf16_t, 4, 4, 2, 2, 1, 2>(p, stream);
    if (tile == 3) return launch_tile<bf16_t, 2, 4, 1, 1, 1, 2, 256>(p, stream);
    if (wide && tile != 1) {   // (the 128x128 tile with wide chunks would not fit two blocks per CU: slower)
      if (shape == 2) return launch_tile<bf16_t, 1, 1, 1, 1, 4, 2, 256>(p, stream);
      if (shape == 1) return launch_tile<bf16_t, 2, 1, 1, 1, 2, 2, 256>(p, stream);
      return launch_tile<bf16_t, 2, 2, 1, 1, 1, 2, 256>(p, stream);
    }
    if (tile == 1) return launch_tile<bf16_t, 4, 2, 1, 2, 1, 2>(p, stream);
    if (shape == 2) return launch_tile<bf16_t, 1, 1, 1, 1, 4, 4>(p, stream);
    if (shape == 1) return launch_tile<bf16_t, 2, 1, 1, 1, 2, 4>(p, stream);
    return chunks <= 3 ? launch_tile<bf16_t, 2, 2, 1, 1, 1, 2>(p, stream) : launch_tile<bf16_t, 2, 2, 1, 1, 1, 4>(p, stream);
  }
  if (tile == 1) return launch_tile<float, 4, 4, 1, 1, 1, 2>(p, stream);
  // the register queue is always filled D chunks deep (clamped re-reads when the k
  // range is shorter), so short ranges take the 2-deep variants
  const int kw = shape == 2 ? 4 : (shape == 1 ? 2 : 1);
  const bool shallow = (chunks + kw - 1) / kw <= 3;
  if (shape == 2) return shallow ? launch_tile<float, 1, 1, 1, 1, 4, 2>(p, stream) : launch_tile<float, 1, 1, 1, 1, 4, 4>(p, stream);
  if (shape == 1) return shallow ? launch_tile<float, 2, 1, 1, 1, 2, 2>(p, stream) : launch_tile<float, 2, 1, 1, 1, 2, 4>(p, stream);
  return shallow ? launch_tile<float, 2, 2, 1, 1, 1, 2>(p, stream) : launch_tile<float, 2, 2, 1, 1, 1, 4>(p, stream);
}

}  // namespace san
