// Device-side helpers shared by the gfx950 kernels: storage types, 16-byte
// fragment access, wavefront (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace san {

constexpr int kWave = 64;

// bf16 storage: the upper 16 bits of an fp32 pattern.
struct bf16_t {
  uint16_t v;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x.v) << 16); }

// round-to-nearest-even fp32 -> bf16 (NaN kept quiet): the hardware conversion of gfx950
// (v_cvt_pk_bf16_f32, two values per instruction where the compiler can pair them)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  return __builtin_bit_cast(uint16_t, (__bf16)f);
}
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_bits(float lo, float hi) {   // lo in the low half
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  bf16x2_t v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

template <typename T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) {
  bf16_t r;
  r.v = f32_to_bf16_bits(f);
  return r;
}

// Elements of T in one 16-byte fragment.
template <typename T> struct Frag;
template <> struct Frag<float> {
  static constexpr int N = 4;
};
template <> struct Frag<bf16_t> {
  static constexpr int N = 8;
};

// Load a 16-byte fragment (p must be 16-byte aligned) and widen to fp32.
__device__ __forceinline__ void load_frag(const float* p, float (&out)[4]) {
  const float4 v = *reinterpret_cast<const float4*>(p);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
__device__ __forceinline__ void load_frag(const bf16_t* p, float (&out)[8]) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ void store_frag(float* p, const float (&in)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(in[0], in[1], in[2], in[3]);
}
__device__ __forceinline__ void store_frag(bf16_t* p, const float (&in)[8]) {
  uint4 v;
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = f32x2_to_bf16x2_bits(in[2 * i], in[2 * i + 1]);
  v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3];
  *reinterpret_cast<uint4*>(p) = v;
}

// 4 consecutive elements (used by row-wise kernels; p aligned to 4 elements).
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const bf16_t* p) {
  const uint2 v = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                     __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
}
__device__ __forceinline__ void store4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void store4(bf16_t* p, float4 v) {
  uint2 o;
  o.x = f32x2_to_bf16x2_bits(v.x, v.y);
  o.y = f32x2_to_bf16x2_bits(v.z, v.w);
  *reinterpret_cast<uint2*>(p) = o;
}

// DPP moves inside a row of 16 lanes (no LDS traffic, unlike a bpermute shuffle).
template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
template <int CTRL> __device__ __forceinline__ int dpp_mov_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]: lane ^ 1
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]: lane ^ 2
constexpr int kDppRowHalfMirror = 0x141; // lane i <-> 7 - i inside each 8 lanes
constexpr int kDppRowMirror = 0x140;     // lane i <-> 15 - i inside each 16 lanes

// Sum / max over aligned groups of N lanes (N = 2, 4, 8, 16); every lane of the
// group gets the result.
template <int N> __device__ __forceinline__ float group_sum(float v) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8 || N == 16, "group size");
  if (N >= 2) v += dpp_mov<kDppQuadSwap1>(v);
  if (N >= 4) v += dpp_mov<kDppQuadSwap2>(v);
  if (N >= 8) v += dpp_mov<kDppRowHalfMirror>(v);
  if (N >= 16) v += dpp_mov<kDppRowMirror>(v);
  return v;
}
// Maxima are written as v_max_f32 instructions: for fmaxf(v, dpp(v)) the compiler emits five (a
// zeroed destination, the move, two canonicalising maxima, the maximum), for fmaxf of two swapped
// registers three.  The s_nop cover the DPP read-after-write hazards (2 wait states after a VALU
// write of the source, 5 after a VALU write of EXEC), which the compiler cannot see inside asm.
__device__ __forceinline__ float max_raw(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
template <int N> __device__ __forceinline__ float group_max(float v) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8 || N == 16, "group size");
  if (N >= 2) asm("s_nop 4\n\tv_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "+v"(v));
  if (N >= 4) asm("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "+v"(v));
  if (N >= 8) asm("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf" : "+v"(v));
  if (N >= 16) asm("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf" : "+v"(v));
  return v;
}

// Cross-row exchanges without LDS traffic: v_permlane16_swap / v_permlane32_swap
// (gfx950) swap the odd 16- (32-) lane rows of one register with the even rows of
// another.  Fed the same value twice, the two results hold, in every lane, the
// values of lane and of lane ^ 16 (lane ^ 32).
__device__ __forceinline__ float sum_xor16(float v) {
  const unsigned x = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float sum_xor32(float v) {
  const unsigned x = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float max_xor16(float v) {
  const unsigned x = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  return max_raw(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float max_xor32(float v) {
  const unsigned x = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  return max_raw(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// The value lane ^ 16 (lane ^ 32) holds.
__device__ __forceinline__ unsigned other_xor16(unsigned x) {
  const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  return (threadIdx.x & 16) ? r[0] : r[1];
}
__device__ __forceinline__ unsigned other_xor32(unsigned x) {
  const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  return (threadIdx.x & 32) ? r[0] : r[1];
}

// The value lane ^ J holds (J a power of two): DPP inside a row, row swaps across rows.
template <int J> __device__ __forceinline__ unsigned lane_xor(unsigned x) {
  static_assert(J == 1 || J == 2 || J == 4 || J == 8 || J == 16 || J == 32, "stride");
  if (J == 1) return (unsigned)dpp_mov_i<kDppQuadSwap1>((int)x);
  if (J == 2) return (unsigned)dpp_mov_i<kDppQuadSwap2>((int)x);
  if (J == 4) {
    const int up = dpp_mov_i<0x104>((int)x);    // row_shl:4: from lane + 4
    const int down = dpp_mov_i<0x114>((int)x);  // row_shr:4: from lane - 4
    return (unsigned)((threadIdx.x & 4) ? down : up);
  }
  if (J == 8) return (unsigned)dpp_mov_i<0x128>((int)x);   // row_ror:8
  if (J == 16) return other_xor16(x);
  return other_xor32(x);
}

// Sum over the lanes that agree with this one in the low log2(LO) bits of the
// lane id, inside aligned groups of HI lanes (LO, HI powers of two, HI = 64 here).
// Inside a 16-lane row the partners are reached by rotating the row by LO, 2*LO,
// ... 8 lanes (DPP row_ror), across rows by the swaps above.
template <int LO, int HI> __device__ __forceinline__ float xor_sum(float v) {
  static_assert(HI == kWave, "reduces up to the whole wave");
  if (LO <= 1) v += dpp_mov<0x121>(v);
  if (LO <= 2) v += dpp_mov<0x122>(v);
  if (LO <= 4) v += dpp_mov<0x124>(v);
  if (LO <= 8) v += dpp_mov<0x128>(v);
  if (LO <= 16) v = sum_xor16(v);
  return sum_xor32(v);
}
__device__ __forceinline__ float wave_sum(float v) { return sum_xor32(sum_xor16(group_sum<16>(v))); }
__device__ __forceinline__ float wave_max(float v) { return max_xor32(max_xor16(group_max<16>(v))); }
// sum over aligned groups of LPP lanes (LPP up to 32)
template <int LPP> __device__ __forceinline__ float lanes_sum(float v) {
  if (LPP <= 16) return group_sum<(LPP <= 16 ? LPP : 16)>(v);
  return sum_xor16(group_sum<16>(v));
}

}  // namespace san
