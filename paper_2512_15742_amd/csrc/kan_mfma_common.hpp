// Pieces shared by the matrix-core kernels: fp16 packing, the raw codeword of an edge and
// its dequantisation into fp16 pairs (Int8: packed-half arithmetic; fp32: multiply, round).
#pragma once

#include "kan_device.hpp"

namespace kan {

typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t pack_h2(float a, float b) {
  h16x2 v = {(_Float16)a, (_Float16)b};
  return __builtin_bit_cast(uint32_t, v);
}

// fp16 pair (g*q[p], g*q[p+1]) from bytes p, p+1 of w, where w holds q + 128 as
// unsigned bytes: 0x6400 | byte is the half 1024 + byte, so subtracting 1152 is
// exact and leaves q.
template <int P>
__device__ __forceinline__ uint32_t dq_pair(uint32_t w, h16x2 g2) {
  const uint32_t sel = 0x04000400u | ((uint32_t)(P + 1) << 16) | (uint32_t)P;
  const uint32_t m = __builtin_amdgcn_perm(0x64646464u, w, sel);
  const h16x2 off = {(_Float16)-1152.0f, (_Float16)-1152.0f};
  const h16x2 v = (__builtin_bit_cast(h16x2, m) + off) * g2;
  return __builtin_bit_cast(uint32_t, v);
}

// Both halves of a packed fp16 pair with subnormals set to zero.  The split form does this to
// its high parts itself, before it forms the low parts from what is left, so that the sum of
// the parts does not depend on how conversions and matrix instructions treat subnormals.
__device__ __forceinline__ uint32_t flush_h2(uint32_t v) {
  if ((v & 0x7c00u) == 0u) v &= 0xffff8000u;
  if ((v & 0x7c000000u) == 0u) v &= 0x8000ffffu;
  return v;
}

// Split form of the precise path: a number v travels as two fp16 parts, v = hi + lo / 2048 with
// hi = fp16(v) and lo = fp16((v - hi) * 2048): 22 significant bits; the factor keeps the low
// parts out of the fp16 subnormals.  Ten coefficients in consecutive pairs (2m, 2m + 1).
__device__ __forceinline__ void split_consecutive(const float (&c)[kG], uint32_t (&hi)[5], uint32_t (&lo)[5]) {
#pragma unroll
  for (int m = 0; m < 5; ++m) {
    hi[m] = flush_h2(pack_h2(c[2 * m], c[2 * m + 1]));
    lo[m] = flush_h2(pack_h2((c[2 * m] - half_bits_to_float(hi[m] & 0xffffu)) * 2048.0f,
                             (c[2 * m + 1] - half_bits_to_float(hi[m] >> 16)) * 2048.0f));
  }
}

// A pair of basis weights (never negative) in split form: the high parts cut to fp16 towards zero
// (so that the low parts are never negative either), no subnormal high parts.
__device__ __forceinline__ void split_weights(float wa, float wb, uint32_t& hi, uint32_t& lo) {
  const uint32_t h = pack_h2(wa, wb);
  uint32_t ha = h & 0xffffu, hb = h >> 16;
  if (half_bits_to_float(ha) > wa) ha -= 1u;                   // one fp16 step down (w > 0 there)
  if (half_bits_to_float(hb) > wb) hb -= 1u;
  if ((ha & 0x7c00u) == 0u) ha = 0u;
  if ((hb & 0x7c00u) == 0u) hb = 0u;
  hi = ha | (hb << 16);
  lo = flush_h2(pack_h2((wa - half_bits_to_float(ha)) * 2048.0f, (wb - half_bits_to_float(hb)) * 2048.0f)) & 0x7fff7fffu;
}

// Raw codeword of one edge as loaded from the codebook.
template <typename CbT> struct RawRow;
template <> struct RawRow<int8_t> { uint32_t a, b, d; };
template <> struct RawRow<__half> { uint32_t w[kG / 2]; };
template <> struct RawRow<float> { float c[kG]; };
template <> struct RawRow<bfp8_t> { uint32_t a, b, d; };           // d: mantissas 8, 9, exponent byte, zero

// One row = one to three load instructions per lane, as wide as they come: every vector-memory
// instruction of a divergent gather costs the CU's address and tag pipeline a slot per lane,
// whether it brings 2 bytes or 16.  The loads are raw buffer loads (exact widths whatever the
// alignment of the row; the resource spans the address space from the codebook's base, so no
// range check cuts a row short):
//   Int8 (10 bytes, 2-byte aligned): the three aligned dwords that hold the row, shifted into
//     place (0 or 2 bytes).  Every dword touched holds at least one byte of the row, so the load
//     never leaves the pages of the codebook, whatever its size.
//   fp16 (20 bytes, 4-byte aligned): 16 + 4.   fp32 (40 bytes, 8-byte aligned): 16 + 16 + 8.
constexpr int kRowBufferFlags = 0x00020000;       // buffer resource word 3: raw 32-bit data, no swizzle

// For Int8 rows the shift is applied when the row is used (align_row), so that a row in flight
// costs three registers and one bit: row_odd() is that bit, and callers keep the bits of the
// rows of a step in one word.
template <typename CbT>
__device__ __forceinline__ uint32_t row_odd(const CbT* cb, uint32_t id) {
  if constexpr (sizeof(CbT) == 1) return ((uint32_t)((uintptr_t)cb >> 1) + id) & 1u;    // (base + 10 id) / 2 mod 2
  else return 0u;
}

template <typename CbT>
__device__ __forceinline__ void load_row(const CbT* cb, uint32_t id, RawRow<CbT>& r) {
  typedef unsigned int bu32x2 __attribute__((ext_vector_type(2)));
  typedef unsigned int bu32x3 __attribute__((ext_vector_type(3)));
  typedef unsigned int bu32x4 __attribute__((ext_vector_type(4)));
  if constexpr (kIsBfp8<CbT>) {                                   // twelve bytes, 4-byte aligned: one load
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)cb, 0, 0x7fffffff, kRowBufferFlags);
    const bu32x3 v = __builtin_amdgcn_raw_buffer_load_b96(rs, (int)(id * 12u), 0, 0);
    r.a = v.x;
    r.b = v.y;
    r.d = v.z;
  } else if constexpr (sizeof(CbT) == 1) {
    const uint32_t mis = (uint32_t)(uintptr_t)cb & 3u;           // 0 or 2: the base within its dword
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc((void*)((uintptr_t)cb - mis), 0, 0x7fffffff, kRowBufferFlags);
    const uint32_t at = id * (uint32_t)kG + mis;                 // byte offset of the row from the aligned base
    const bu32x3 v = __builtin_amdgcn_raw_buffer_load_b96(rs, (int)(at & ~3u), 0, 0);
    r.a = v.x;                                                   // still to be shifted: align_row
    r.b = v.y;
    r.d = v.z;
  } else if constexpr (sizeof(CbT) == 2) {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)cb, 0, 0x7fffffff, kRowBufferFlags);
    const int at = (int)(id * (uint32_t)(kG * 2));
    const bu32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, at, 0, 0);
    r.w[0] = v.x;
    r.w[1] = v.y;
    r.w[2] = v.z;
    r.w[3] = v.w;
    r.w[4] = __builtin_amdgcn_raw_buffer_load_b32(rs, at, 16, 0);
  } else {
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)cb, 0, 0x7fffffff, kRowBufferFlags);
    const int at = (int)(id * (uint32_t)(kG * 4));
    const bu32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(rs, at, 0, 0);
    const bu32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(rs, at, 16, 0);
    const bu32x2 v2 = __builtin_amdgcn_raw_buffer_load_b64(rs, at, 32, 0);
    r.c[0] = __uint_as_float(v0.x); r.c[1] = __uint_as_float(v0.y); r.c[2] = __uint_as_float(v0.z); r.c[3] = __uint_as_float(v0.w);
    r.c[4] = __uint_as_float(v1.x); r.c[5] = __uint_as_float(v1.y); r.c[6] = __uint_as_float(v1.z); r.c[7] = __uint_as_float(v1.w);
    r.c[8] = __uint_as_float(v2.x); r.c[9] = __uint_as_float(v2.y);
  }
}

// The row as it lies in memory: bytes 0..3 in a, 4..7 in b, 8..9 in the low half of d (odd: the
// row starts in the upper half of its first dword).  No-op for the other row types.
template <typename CbT>
__device__ __forceinline__ void align_row(RawRow<CbT>& r, uint32_t odd) {
  if constexpr (sizeof(CbT) == 1) {
    const uint32_t sh = odd * 2u;
    const uint32_t a = __builtin_amdgcn_alignbyte(r.b, r.a, sh);
    const uint32_t b = __builtin_amdgcn_alignbyte(r.d, r.b, sh);
    const uint32_t d = __builtin_amdgcn_alignbyte(0u, r.d, sh) & 0xffffu;
    r.a = a;
    r.b = b;
    r.d = d;
  }
}

// w[0..3] = fp16 pairs of g*coef 0..7, w[4] = g*coef 8, 9.
template <typename CbT>
__device__ __forceinline__ void dequant_row(const RawRow<CbT>& r, float g, uint32_t (&w)[5]) {
  if constexpr (sizeof(CbT) == 1 || kIsBfp8<CbT>) {
    float gs = g;
    if constexpr (kIsBfp8<CbT>) gs = g * bfp8_row_scale(r.d);      // the row's own power of two goes with the gain
    const _Float16 gh = (_Float16)gs;
    const h16x2 g2 = {gh, gh};
    const uint32_t a = r.a ^ 0x80808080u, b = r.b ^ 0x80808080u, d = r.d ^ 0x00008080u;
    w[0] = dq_pair<0>(a, g2);
    w[1] = dq_pair<2>(a, g2);
    w[2] = dq_pair<0>(b, g2);
    w[3] = dq_pair<2>(b, g2);
    w[4] = dq_pair<0>(d, g2);
  } else if constexpr (sizeof(CbT) == 2) {
#pragma unroll
    for (int m = 0; m < 5; ++m)
      w[m] = pack_h2(g * half_bits_to_float(r.w[m] & 0xffffu), g * half_bits_to_float(r.w[m] >> 16));
  } else {
#pragma unroll
    for (int m = 0; m < 5; ++m) w[m] = pack_h2(g * r.c[2 * m], g * r.c[2 * m + 1]);
  }
}

// c[m] = g * coef m as fp32 (matrix-core path with fp32 operands).
template <typename CbT>
__device__ __forceinline__ void dequant_row_f32(const RawRow<CbT>& r, float g, float (&c)[kG]) {
  if constexpr (sizeof(CbT) == 1 || kIsBfp8<CbT>) {
    if constexpr (kIsBfp8<CbT>) g *= bfp8_row_scale(r.d);          // the row's own power of two goes with the gain
    const float off = -128.0f * g;
    float t[4];
    dequant4(r.a, g, off, &c[0]);
    dequant4(r.b, g, off, &c[4]);
    dequant4(r.d, g, off, t);
    c[8] = t[0];
    c[9] = t[1];
  } else if constexpr (sizeof(CbT) == 2) {
#pragma unroll
    for (int m = 0; m < kG / 2; ++m) {
      c[2 * m] = g * half_bits_to_float(r.w[m] & 0xffffu);
      c[2 * m + 1] = g * half_bits_to_float(r.w[m] >> 16);
    }
  } else {
#pragma unroll
    for (int m = 0; m < kG; ++m) c[m] = g * r.c[m];
  }
}

// Byte-permute selectors that place the four fp16 weights {w23:w01} of one input at
// half-word slots l..l+3 of its ten: entry [l][k], k = 0..4, builds slots 2k, 2k+1;
// selector byte 0x0c yields 0.  56 threads fill the 7 x 8 table.
__device__ __forceinline__ void fill_weight_selectors(uint32_t (*sel)[8], int tid) {
  if (tid < kSpans * 8) {
    const int l = tid >> 3, k = tid & 7;
    uint32_t v = 0x0c0c0c0cu;
    if (k < 5) {
      const int r0 = 2 * k - l, r1 = 2 * k + 1 - l;
      const uint32_t lo = (r0 >= 0 && r0 <= 3) ? (uint32_t)((2 * r0) | ((2 * r0 + 1) << 8)) : 0x0c0cu;
      const uint32_t hi = (r1 >= 0 && r1 <= 3) ? (uint32_t)((2 * r1) | ((2 * r1 + 1) << 8)) : 0x0c0cu;
      v = lo | (hi << 16);
    }
    sel[l][k] = v;
  }
}

// Span (0..6) and the two weight words from a packed basis word (kan_prep_basis, fp16 form).
__device__ __forceinline__ void unpack_basis(uint2 u, uint32_t& l, uint32_t& w01, uint32_t& w23) {
  l = ((u.x >> 15) & 1u) | ((u.x >> 30) & 2u) | ((u.y >> 13) & 4u);
  w01 = u.x & 0x7fff7fffu;
  w23 = u.y & 0x7fff7fffu;
}

}  // namespace kan
