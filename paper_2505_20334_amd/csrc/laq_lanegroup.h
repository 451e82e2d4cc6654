// Helpers for kernels in which a group of adjacent lanes shares one row of d elements, 8 elements
// (one 16- or 32-byte piece) per lane: loads of a piece, the product of two pieces, and the sum
// over the lanes of a group.  Used by the decode-attention kernel and the generic scoring kernels.
#ifndef LAQ_LANEGROUP_H
#define LAQ_LANEGROUP_H

#include "laq_internal.h"

namespace laq {

// Eight consecutive elements of a row: raw bits as loaded, widened to fp32 at the point of use.
struct Piece8F32 { float4 a, b; };
struct Piece8BF16 { uint4 r; };

__device__ __forceinline__ void fetch8(const float* p, Piece8F32& x) {
  x.a = *reinterpret_cast<const float4*>(p);
  x.b = *reinterpret_cast<const float4*>(p + 4);
}
__device__ __forceinline__ void fetch8(const uint16_t* p, Piece8BF16& x) { x.r = *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void clear8(Piece8F32& x) { x.a = x.b = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void clear8(Piece8BF16& x) { x.r = make_uint4(0u, 0u, 0u, 0u); }

__device__ __forceinline__ void widen8(const Piece8F32& x, float (&f)[8]) {
  f[0] = x.a.x; f[1] = x.a.y; f[2] = x.a.z; f[3] = x.a.w;
  f[4] = x.b.x; f[5] = x.b.y; f[6] = x.b.z; f[7] = x.b.w;
}
__device__ __forceinline__ void widen8(const Piece8BF16& x, float (&f)[8]) {   // bf16 = the high half of fp32
  f[0] = __uint_as_float(x.r.x << 16); f[1] = __uint_as_float(x.r.x & 0xffff0000u);
  f[2] = __uint_as_float(x.r.y << 16); f[3] = __uint_as_float(x.r.y & 0xffff0000u);
  f[4] = __uint_as_float(x.r.z << 16); f[5] = __uint_as_float(x.r.z & 0xffff0000u);
  f[6] = __uint_as_float(x.r.w << 16); f[7] = __uint_as_float(x.r.w & 0xffff0000u);
}

// Sum over the PP (8, 16 or 32) adjacent lanes of a group, result in every lane.  Data-parallel
// lane permutations within a row of 16 lanes: swap neighbours, swap pairs, then mirror the 8 and
// the 16 lanes (the halves already agree, so a mirror reaches the other half's sum).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
template <int PP>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_move<0xB1>(x);                   // quad_perm [1,0,3,2]
  x += dpp_move<0x4E>(x);                   // quad_perm [2,3,0,1]
  x += dpp_move<0x141>(x);                  // row_half_mirror
  if (PP >= 16) x += dpp_move<0x140>(x);    // row_mirror
  if (PP >= 32) x += __shfl_xor(x, 16);
  return x;
}

// Product of two 8-element pieces.  bf16: four two-element dot-product instructions on the raw
// pairs (products and sums in fp32), no widening; fp32: eight fused multiply-adds.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}
__device__ __forceinline__ float dot8(const Piece8BF16& a, const Piece8BF16& b) {
  float s = dot2_bf16(a.r.x, b.r.x, 0.f);
  s = dot2_bf16(a.r.y, b.r.y, s);
  s = dot2_bf16(a.r.z, b.r.z, s);
  return dot2_bf16(a.r.w, b.r.w, s);
}
__device__ __forceinline__ float dot8(const Piece8F32& a, const Piece8F32& b) {
  float s = a.a.x * b.a.x;
  s = fmaf(a.a.y, b.a.y, s); s = fmaf(a.a.z, b.a.z, s); s = fmaf(a.a.w, b.a.w, s);
  s = fmaf(a.b.x, b.b.x, s); s = fmaf(a.b.y, b.b.y, s); s = fmaf(a.b.z, b.b.z, s);
  return fmaf(a.b.w, b.b.w, s);
}

template <typename T> struct PieceOf;
template <> struct PieceOf<float> { using type = Piece8F32; };
template <> struct PieceOf<uint16_t> { using type = Piece8BF16; };

// lanes per row: the power of two (at least 8, at most 32) that covers the row's d / 8 pieces
inline int lanes_per_row(int d) {
  int pp = 8;
  while (pp * 8 < d) pp <<= 1;
  return pp;
}

}  // namespace laq
#endif  // LAQ_LANEGROUP_H
