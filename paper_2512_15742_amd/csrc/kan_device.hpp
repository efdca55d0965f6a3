// Device-side building blocks shared by the gfx950 kernels: the span/basis
// routine for the cubic, G = 10, [-1,1] spline family (paper App. A.1), and the
// loaders for per-edge metadata and codeword rows (paper Eq. (1), section 4.2).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kan {

constexpr int kG = 10;        // coefficients per edge
constexpr int kSpans = 7;     // uniform intervals on [-1, 1]
constexpr int kWave = 64;

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct BasisW {
  float w0, w1, w2, w3;   // weights of coefficients span .. span+3
  int span;               // 0..6
};

// Span and the four nonzero cubic weights at x (clamped to [-1,1]).
//
// The knots are the rationals (2l-7)/7.  7*x is exact in fp64 for an fp32 x, so
// "x >= knot" is decided exactly by comparing 7x with the odd integers -5..5,
// and the local coordinate u = (x - t_{l+3}) / h = (7x + 7 - 2l) / 2 is exact as
// well.  x = +1 gives l = 6, u = 1 (closed right end).  The weights are the
// uniform cubic B-spline blending polynomials, evaluated in fp64 and rounded
// once to fp32.
__device__ __forceinline__ BasisW basis_eval(float xf) {
  const float xc = fminf(fmaxf(xf, -1.0f), 1.0f);
  const double x7 = 7.0 * (double)xc;
  const int l = (int)(x7 >= -5.0) + (int)(x7 >= -3.0) + (int)(x7 >= -1.0) +
                (int)(x7 >= 1.0) + (int)(x7 >= 3.0) + (int)(x7 >= 5.0);
  const double u = (x7 + (double)(7 - 2 * l)) * 0.5;
  const double u2 = u * u, u3 = u2 * u, om = 1.0 - u;
  const double sixth = 1.0 / 6.0;
  BasisW r;
  r.w0 = (float)(om * om * om * sixth);
  r.w1 = (float)((3.0 * u3 - 6.0 * u2 + 4.0) * sixth);
  r.w2 = (float)((-3.0 * u3 + 3.0 * u2 + 3.0 * u + 1.0) * sixth);
  r.w3 = (float)(u3 * sixth);
  r.span = l;
  return r;
}

// The runtime rule of the paper's own operator (sections 4.1 and 4.3): the G = 10 entries of a
// codeword are samples at the uniform nodes n_k = -1 + 2k/9 and the edge function is the
// linear interpolation between the two neighbours of x, index floor((x + 1) / dx), dx = 2/9.
// 9x is exact in fp64, so the index is decided exactly by comparing 9x with the odd integers
// -7..7, and u = (9x + 9 - 2k) / 2 is exact; x = +1 gives k = 8, u = 1 (closed right end).
// Returned in the same form as the cubic family - a window of four consecutive entries and
// four weights - so that every kernel serves both rules: the window starts at min(k, 6) and
// the two weights 1-u, u sit at offset k - min(k, 6) inside it, the others are 0.
struct PliIndex {
  int k;        // 0..8
  double u;     // 0..1
};
__device__ __forceinline__ PliIndex pli_index(float xf) {
  const float xc = fminf(fmaxf(xf, -1.0f), 1.0f);
  const double x9 = 9.0 * (double)xc;
  PliIndex r;
  r.k = (int)(x9 >= -7.0) + (int)(x9 >= -5.0) + (int)(x9 >= -3.0) + (int)(x9 >= -1.0) +
        (int)(x9 >= 1.0) + (int)(x9 >= 3.0) + (int)(x9 >= 5.0) + (int)(x9 >= 7.0);
  r.u = (x9 + (double)(9 - 2 * r.k)) * 0.5;
  return r;
}
__device__ __forceinline__ BasisW window_of_pair(int k, float w_lo, float w_hi) {
  BasisW r;
  r.span = min(k, kSpans - 1);
  const int o = k - r.span;                    // 0, 1 or 2
  r.w0 = o == 0 ? w_lo : 0.f;
  r.w1 = o == 0 ? w_hi : (o == 1 ? w_lo : 0.f);
  r.w2 = o == 1 ? w_hi : (o == 2 ? w_lo : 0.f);
  r.w3 = o == 2 ? w_hi : 0.f;
  return r;
}
__device__ __forceinline__ BasisW basis_eval_pli(float xf) {
  const PliIndex p = pli_index(xf);
  return window_of_pair(p.k, (float)(1.0 - p.u), (float)p.u);
}

enum EdgeRule : int { kRuleBspline3 = 0, kRulePli2 = 1 };

__device__ __forceinline__ BasisW basis_eval_rule(float xf, int rule) {
  return rule == kRulePli2 ? basis_eval_pli(xf) : basis_eval(xf);
}

// The same two families with the weights evaluated in fp32 from the exact fp64 index and local
// coordinate (one fma + truncation instead of the comparisons); used where the weights are
// about to be rounded to fp16 or feed fp32 matrix-core operands.
__device__ __forceinline__ BasisW basis_fast(float xf, int rule) {
  const float xc = fminf(fmaxf(xf, -1.0f), 1.0f);
  if (rule == kRulePli2) {
    const double t = fma((double)xc, 4.5, 4.5);          // exact: (9x + 9) / 2
    const int k = min((int)t, kG - 2);
    const float u = (float)(t - (double)k);
    return window_of_pair(k, 1.0f - u, u);
  }
  // exact span: t = (7x + 7) / 2 is exact in fp64; span = min(floor(t), 6); the local
  // coordinate u = t - span is exact too and is rounded once to fp32
  const double t = fma((double)xc, 3.5, 3.5);
  BasisW r;
  r.span = min((int)t, kSpans - 1);
  const float u = (float)(t - (double)r.span);
  const float u2 = u * u, u3 = u2 * u, om = 1.0f - u;
  r.w0 = om * om * om * (1.0f / 6.0f);
  r.w3 = u3 * (1.0f / 6.0f);
  r.w1 = fmaf(0.5f, u3, fmaf(-1.0f, u2, 2.0f / 3.0f));
  r.w2 = fmaf(-0.5f, u3, fmaf(0.5f, u2, fmaf(0.5f, u, 1.0f / 6.0f)));
  return r;
}

// ---- streaming loads of N consecutive per-edge values ------------------------
// The metadata stream is read once per batch tile and never reused, so it is
// loaded non-temporally to keep it from displacing the codebook in L2.

template <int BYTES> struct RawVec;
template <> struct RawVec<1> { typedef uint8_t type; };
template <> struct RawVec<2> { typedef uint16_t type; };
template <> struct RawVec<4> { typedef uint32_t type; };
template <> struct RawVec<8> { typedef u32x2 type; };
template <> struct RawVec<16> { typedef u32x4 type; };
template <> struct RawVec<32> { struct type { u32x4 a, b; }; };

template <int BYTES>
__device__ __forceinline__ void stream_load(const void* p, void* dst) {
  if constexpr (BYTES == 32) {
    const u32x4* q = (const u32x4*)p;
    u32x4 a = __builtin_nontemporal_load(q);
    u32x4 b = __builtin_nontemporal_load(q + 1);
    ((u32x4*)dst)[0] = a;
    ((u32x4*)dst)[1] = b;
  } else {
    typedef typename RawVec<BYTES>::type V;
    V v = __builtin_nontemporal_load((const V*)p);
    *(V*)dst = v;
  }
}

template <typename IdxT, int N>
__device__ __forceinline__ void load_idx(const IdxT* p, uint32_t (&id)[N]) {
  alignas(16) IdxT raw[N];
  stream_load<sizeof(IdxT) * N>(p, raw);
#pragma unroll
  for (int n = 0; n < N; ++n) id[n] = (uint32_t)raw[n];   // zero-extends
}

// Per-edge gain and bias come as fp32, fp16, or one byte each (paper section 4.2: gains as
// logarithmic Int8, biases as linear Int8 - 16 bits per edge beside the index).  The byte
// codes mean
//     gain = 0 for code 0, else exp2(gain_log2_lo + gain_log2_step * code)   code = 1..255
//     bias = bias_scale * code                                               code = -127..127
// with the three parameters fixed per layer (the paper prints no formula; this reading keeps
// a zero code for exact zeros and spends the other 255 codes evenly on log2 of the gain).
struct Q8Params {
  float gain_log2_lo, gain_log2_step, bias_scale;
};
struct q8_t {          // element type tag of byte-coded gain/bias arrays
  uint8_t v;
};

__device__ __forceinline__ float q8_gain(uint32_t code, const Q8Params& qp) {
  const float g = exp2f(fmaf(qp.gain_log2_step, (float)code, qp.gain_log2_lo));
  return code ? g : 0.f;
}
__device__ __forceinline__ float q8_bias(uint32_t code, const Q8Params& qp) {
  return qp.bias_scale * (float)(int)(int8_t)code;
}

template <typename T, int N, bool GAIN>
__device__ __forceinline__ void load_gb_any(const T* p, const Q8Params& qp, float (&v)[N]) {
  if constexpr (sizeof(T) == 1) {
    alignas(8) uint8_t raw[N];
    stream_load<N>(p, raw);
#pragma unroll
    for (int n = 0; n < N; ++n) v[n] = GAIN ? q8_gain(raw[n], qp) : q8_bias(raw[n], qp);
  } else {
    alignas(16) T raw[N];
    stream_load<sizeof(T) * N>(p, raw);
#pragma unroll
    for (int n = 0; n < N; ++n) {
      if constexpr (sizeof(T) == 2) v[n] = __half2float(raw[n]);
      else v[n] = raw[n];
    }
  }
}
template <typename T, int N>
__device__ __forceinline__ void load_gain(const T* p, const Q8Params& qp, float (&v)[N]) {
  load_gb_any<T, N, true>(p, qp, v);
}
template <typename T, int N>
__device__ __forceinline__ void load_bias(const T* p, const Q8Params& qp, float (&v)[N]) {
  load_gb_any<T, N, false>(p, qp, v);
}

// ---- codeword rows -------------------------------------------------------------

// Block floating point with 8-bit mantissas (the BFP8 codebook row of the paper's Table 1; the
// paper names the precision but not the format, so the format is this library's): a codeword
// row is one block of twelve bytes - ten signed mantissa bytes q[0..9] in -127..127, one signed
// exponent byte e shared by the row, one zero byte - and entry m means q[m] * 2^e.
struct bfp8_t {
  int8_t q[10];
  int8_t e;
  int8_t zero;
};
static_assert(sizeof(bfp8_t) == 12, "a block-floating-point row is twelve bytes");

template <typename CbT> constexpr bool kIsBfp8 = sizeof(CbT) == 12;

// 2^e for the exponent byte held in bits 16..23 of the row's third dword.
__device__ __forceinline__ float bfp8_row_scale(uint32_t third_dword) {
  const int e = (int)(int8_t)(third_dword >> 16);
  return __uint_as_float((uint32_t)(e + 127) << 23);      // e in -126..127: a normal fp32 power of two
}

__device__ __forceinline__ float half_bits_to_float(uint32_t bits) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
}

__device__ __forceinline__ uint32_t ld_u32_any(const uint8_t* p) {
  uint32_t v;
  __builtin_memcpy(&v, p, 4);
  return v;
}
__device__ __forceinline__ uint32_t ld_u16_any(const uint8_t* p) {
  uint16_t v;
  __builtin_memcpy(&v, p, 2);
  return v;
}

// mul * q for the four signed bytes of w: q + 128 is read as an unsigned byte by
// the byte-to-float converts, and the offset is folded into one fma, so each
// coefficient costs one convert and one fma, rounded once.
__device__ __forceinline__ void dequant4(uint32_t w, float mul, float off, float* c) {
  const uint32_t b = w ^ 0x80808080u;
  c[0] = fmaf((float)(b & 0xffu), mul, off);
  c[1] = fmaf((float)((b >> 8) & 0xffu), mul, off);
  c[2] = fmaf((float)((b >> 16) & 0xffu), mul, off);
  c[3] = fmaf((float)(b >> 24), mul, off);
}

// Whole row: c[m] = mul * C[id][m], m = 0..9.
template <typename CbT>
__device__ __forceinline__ void fetch_row(const CbT* cb, uint32_t id, float mul, float (&c)[kG]) {
  if constexpr (kIsBfp8<CbT>) {
    const uint32_t* p = (const uint32_t*)(cb + id);                // 4-byte aligned rows
    const uint32_t a = p[0], b = p[1], d = p[2];
    const float m2 = mul * bfp8_row_scale(d), off = -128.0f * m2;
    float t[4];
    dequant4(a, m2, off, &c[0]);
    dequant4(b, m2, off, &c[4]);
    dequant4(d, m2, off, t);
    c[8] = t[0];
    c[9] = t[1];
  } else if constexpr (sizeof(CbT) == 1) {
    const uint8_t* p = (const uint8_t*)cb + (size_t)id * kG;       // 2-byte aligned
    const uint32_t a = ld_u32_any(p), b = ld_u32_any(p + 4), d = ld_u16_any(p + 8);
    const float off = -128.0f * mul;
    float t[4];
    dequant4(a, mul, off, &c[0]);
    dequant4(b, mul, off, &c[4]);
    dequant4(d, mul, off, t);
    c[8] = t[0];
    c[9] = t[1];
  } else if constexpr (sizeof(CbT) == 2) {
    const uint32_t* p = (const uint32_t*)((const uint16_t*)cb + (size_t)id * kG);   // fp16 rows, 4-byte aligned
#pragma unroll
    for (int m = 0; m < kG / 2; ++m) {
      const uint32_t v = p[m];
      c[2 * m] = mul * half_bits_to_float(v & 0xffffu);
      c[2 * m + 1] = mul * half_bits_to_float(v >> 16);
    }
  } else {
    const float2* p = (const float2*)(cb + (size_t)id * kG);       // 8-byte aligned
#pragma unroll
    for (int m = 0; m < kG / 2; ++m) {
      const float2 v = p[m];
      c[2 * m] = mul * v.x;
      c[2 * m + 1] = mul * v.y;
    }
  }
}

// Window of four: c[r] = mul * C[id][span + r], r = 0..3 (batch-1 path: only the
// four coefficients under the nonzero bases are fetched).  Load and dequantisation
// are separate so that many gathers can be issued before the first one is used.
template <typename CbT> struct WindowRaw;
template <> struct WindowRaw<int8_t> { typedef uint32_t type; };
template <> struct WindowRaw<__half> { typedef uint2 type; };
template <> struct WindowRaw<float> { typedef float4 type; };
template <> struct WindowRaw<bfp8_t> { typedef uint2 type; };      // four mantissa bytes, the row's third dword

template <typename CbT>
__device__ __forceinline__ typename WindowRaw<CbT>::type load_window(const CbT* cb, uint32_t id, int span) {
  if constexpr (kIsBfp8<CbT>) {
    const uint8_t* p = (const uint8_t*)(cb + id);
    return make_uint2(ld_u32_any(p + span), ((const uint32_t*)p)[2]);
  } else if constexpr (sizeof(CbT) == 1) {
    return ld_u32_any((const uint8_t*)cb + (size_t)id * kG + span);
  } else if constexpr (sizeof(CbT) == 2) {
    uint2 v;                                                       // four halves, 2-byte aligned
    __builtin_memcpy(&v, (const uint16_t*)cb + (size_t)id * kG + span, 8);
    return v;
  } else {
    float4 v;
    __builtin_memcpy(&v, cb + (size_t)id * kG + span, 16);
    return v;
  }
}

template <typename CbT>
__device__ __forceinline__ void dequant_window(typename WindowRaw<CbT>::type raw, float mul, float (&c)[4]) {
  if constexpr (kIsBfp8<CbT>) {
    const float m2 = mul * bfp8_row_scale(raw.y);
    dequant4(raw.x, m2, -128.0f * m2, c);
  } else if constexpr (sizeof(CbT) == 1) {
    dequant4(raw, mul, -128.0f * mul, c);
  } else if constexpr (sizeof(CbT) == 2) {
    c[0] = mul * half_bits_to_float(raw.x & 0xffffu);
    c[1] = mul * half_bits_to_float(raw.x >> 16);
    c[2] = mul * half_bits_to_float(raw.y & 0xffffu);
    c[3] = mul * half_bits_to_float(raw.y >> 16);
  } else {
    c[0] = mul * raw.x;
    c[1] = mul * raw.y;
    c[2] = mul * raw.z;
    c[3] = mul * raw.w;
  }
}

}  // namespace kan
