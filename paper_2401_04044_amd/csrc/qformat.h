// Internal: the quantised tiled weight format of the 8-bit heavy / 3-bit remainder split
// (Sec. 5.2, the setting for the LLMs) and its device-side pack / unpack helpers.
//
// A matrix [rows, K] (K-contiguous, like every packed weight here) is cut into blocks of
// 32 rows x 64 reduction elements = four 32 x 16 operand blocks of v_mfma_f32_32x32x16_bf16.
// Lane l = 32 c + r of a wavefront owns row r and, for each of the four operand blocks j,
// the eight elements 16 j + 8 c + e (e = 0..7): 32 codes, numbered t = 8 j + e.  Codes are
// stored offset-binary, u = q + 2^(bits-1).
//   8 bits  2 KiB per block: two 1 KiB halves; half h holds, at byte 16 l + 8 (j & 1) + e,
//           the code of operand block j = 2 h + (j & 1).
//   3 bits  768 bytes per block: three dwords per lane at 12 l.  The code of operand block j,
//           element e belongs to pair p = 4 j + (e >> 1) (one MFMA operand register holds a
//           pair, element 2 i in its low half) and half h = e & 1.  Dword j >> 1 has its low
//           two bits at bit 2 (p & 7) + 16 h; dword 2 has its third bit at bit
//           (p + 2 + 16 h) mod 32.  So  (lo >> 2 (p & 7)) & 0x00030003  and
//           rotr(hi, p) & 0x00040004  are both halves of the pair's register at once, and
//           or-ing 0x43004300 (0x64006400) makes it the bf16 (fp16) pair 128 + u (1024 + u).
// Blocks are ordered [row block][k block].
#pragma once
#include "common.h"

namespace ffsplit {

typedef __attribute__((ext_vector_type(4))) uint32_t q_u32x4;

// round-to-nearest symmetric code of w for scale s (fp32 decisions), offset-binary
__device__ __forceinline__ uint32_t q_code(float w, float s, int bits) {
  const float qmax = (float)((1 << (bits - 1)) - 1);
  int q = 0;
  if (s > 0.f) {
    float t = rintf(w / s);
    t = fminf(fmaxf(t, -qmax - 1.f), qmax);
    q = (int)t;
  }
  return (uint32_t)(q + (1 << (bits - 1)));
}

__device__ __forceinline__ float q_scale(float amax, int bits, uint16_t* bits_out) {
  const _Float16 h = (_Float16)(amax / (float)((1 << (bits - 1)) - 1));
  __builtin_memcpy(bits_out, &h, 2);
  return (float)h;
}

__device__ __forceinline__ float q_half(uint16_t h) {
  _Float16 x;
  __builtin_memcpy(&x, &h, 2);
  return (float)x;
}

// the lane's 32 codes of one block, still packed
template <int BITS>
struct QPacked;
template <>
struct QPacked<8> {
  q_u32x4 h[2];
};
template <>
struct QPacked<3> {
  uint32_t lo[2], hi;
};

__device__ __forceinline__ QPacked<8> q_load8(const char* block, int lane) {
  QPacked<8> p;
  p.h[0] = *(const q_u32x4*)(block + lane * 16);
  p.h[1] = *(const q_u32x4*)(block + 1024 + lane * 16);
  return p;
}
__device__ __forceinline__ QPacked<3> q_load3(const char* block, int lane) {
  QPacked<3> p;
  const uint32_t* w = (const uint32_t*)(block + lane * 12);
  p.lo[0] = w[0]; p.lo[1] = w[1]; p.hi = w[2];
  return p;
}

// code t (0..31) of the lane as a signed integer
__device__ __forceinline__ int q_get(const QPacked<8>& p, int t) {
  const int j = t >> 3, e = t & 7;
  const uint32_t w = p.h[j >> 1][2 * (j & 1) + (e >> 2)];
  return (int)((w >> (8 * (e & 3))) & 255u) - 128;
}
__device__ __forceinline__ int q_pos_lo(int t) { return 2 * ((4 * (t >> 3) + ((t & 7) >> 1)) & 7) + 16 * (t & 1); }
__device__ __forceinline__ int q_pos_hi(int t) { return (4 * (t >> 3) + ((t & 7) >> 1) + 2 + 16 * (t & 1)) & 31; }
__device__ __forceinline__ int q_get(const QPacked<3>& p, int t) {
  const uint32_t lo = (p.lo[t >> 4] >> q_pos_lo(t)) & 3u;
  const uint32_t hi = (p.hi >> q_pos_hi(t)) & 1u;
  return (int)(lo | (hi << 2)) - 4;
}

// (a & mask) | o in one instruction (the compiler's own choice, two ands and a three-input or,
// costs one more per register; the unpack is what bounds the small-batch kernels)
__device__ __forceinline__ uint32_t q_and_or(uint32_t a, uint32_t mask, uint32_t o) {
  uint32_t r;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(o));
  return r;
}

// register i (elements 2 i, 2 i + 1) of operand block j as the pair (magic + u) in both halves
__device__ __forceinline__ uint32_t q_pair(const QPacked<3>& p, int j, int i, uint32_t magic) {
  const int pr = 4 * j + i;
  const uint32_t r = q_and_or(p.lo[j >> 1] >> (2 * (pr & 7)), 0x00030003u, magic);
  return q_and_or(__builtin_amdgcn_alignbit(p.hi, p.hi, pr), 0x00040004u, r);
}
// 8 bits: bytes (2 i, 2 i + 1) of operand block j under the high byte of magic
__device__ __forceinline__ uint32_t q_pair(const QPacked<8>& p, int j, int i, uint32_t magic_bytes) {
  const uint32_t w = p.h[j >> 1][2 * (j & 1) + (i >> 1)];
  return __builtin_amdgcn_perm(magic_bytes, w, (i & 1) ? 0x04030402u : 0x04010400u);
}

}  // namespace ffsplit
