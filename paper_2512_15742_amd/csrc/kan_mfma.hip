// Matrix-core path of the VQ-KAN forward pass for gfx950 (large batch).
//
// The layer sum y[b][j] = sum_i sum_m B_m(x_bi) * c_ij[m] (paper section 3 with
// the reconstructed coefficients of section 4.2) is a contraction over
// k = (i, m), m = 0..9:
//     Y[b][j] = scale * sum_k Phi[b][k] * Chat[k][j] + sum_i bias_ij
//     Phi[b][(i,m)]  = B_m(x_bi)            (4 nonzeros per 10, App. A.1 family)
//     Chat[(i,m)][j] = gain_ij * q_ij[m]    (q = Int8 codeword, or the fp32 row)
// Both operands are fp16 (11-bit significand, same matrix-core rate as bf16); products
// accumulate in fp32 in v_smfmac_f32_32x32x32_f16.  The basis operand lies in [0, 1]; the
// coefficient operand is gain * q with q the Int8 code (|q| <= 127) or gain * C for floating
// codebooks, so |gain * q| (resp. |gain * C|) must stay below the fp16 maximum 65504, and
// magnitudes below 6.1e-5 (the fp16 normal range) lose precision: one-pass form to fp16
// subnormal spacing, split form to the 11 bits of its low part.
// The per-layer Int8 scale and the bias sum (the bases sum to one) stay in fp32
// and are applied to the accumulators at the end.
//
// Three kernels per layer:
//   kan_prep_coef   every edge once per forward: read idx/gain/bias (coalesced),
//                   gather the codeword from L2, dequantise with packed fp16 math,
//                   write Chat in the exact order the MFMA B-operand lanes read
//                   it, and write per-32-row partial bias sums.  A random 10-byte
//                   gather costs the L1 a whole cache line, so it is done once per
//                   edge here instead of once per edge and batch tile.
//   kan_prep_basis  every (sample, input) once: exact span (fp64) and the four
//                   basis weights as fp16, the span hidden in three of their
//                   (always clear) sign bits; 8 bytes per pair, stored transposed
//                   and in pairs of inputs ([input / 2][sample][input % 2]) so that
//                   the contraction kernel reads it coalesced, 16 bytes per lane.
//   kan_mfma        64 or 128 samples x 128 outputs per workgroup, 4 waves side by
//                   side along the outputs; two or three workgroups share a CU and
//                   drift apart, so one's MFMAs overlap the other's tile generation
//                   and LDS latency.  Or 128 samples x 256 outputs for one workgroup
//                   of 8 waves per CU: the same waves per SIMD and registers per wave,
//                   but one Phi tile per CU and step instead of two (half the tile
//                   generation and basis-word loads).  Per step of 16 inputs: the Phi tile (the two
//                   stored values of every group of four k-slots, plus their
//                   positions) is built in LDS (double buffered) from the packed basis
//                   words with byte permutes whose selectors come from a 7-entry
//                   table (one row per span), the Chat fragments stream from memory
//                   straight into registers a step and a half ahead, and the
//                   contraction runs on the sparse matrix instruction
//                   v_smfmac_f32_32x32x32_f16 (5 per row block and step).
//   kan_prep_start  the first two for a single head's call in one launch: the coefficient
//                   records of all its layers and the first layer's basis words.
// The precise path at batch > 64 runs the same kernels on operands split into high
// and low fp16 parts (c = hi + lo / 2048): the preparation kernels write both parts,
// the contraction kernel makes three passes over its steps (hi*lo, lo*hi, scale by
// 1/2048, hi*hi on top) and keeps fp32-grade sums.
// k order inside a step: see kan_mfma_kernel.

#include <type_traits>

#include "kan_device.hpp"
#include "kan_internal.hpp"
#include "kan_mfma_common.hpp"

namespace kan {
namespace {

constexpr int kThreads = 256;          // preparation kernels
constexpr int kMfmaThreads = 256;      // contraction kernel: 4 waves along the outputs (8 waves: 512)
constexpr int IT = 16;                 // input rows per step (160 k-slots = 40 groups of four = 5 sparse MFMAs of K = 32)
constexpr int kRowBytes = 208;         // LDS row of the Phi tile: 160 B of weights, 2 x 16 B of index words, 16 B of
                                       // padding (52 dwords: sixteen consecutive rows start in sixteen different banks)
constexpr int kIdxOffset = 160;        // index words of the row: [lane half][S = 0..4] as u16, 16 bytes per lane half
constexpr int kBufferFlags = 0x00020000;   // buffer resource word 3: raw 32-bit data format, no swizzle

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 h16x16 __attribute__((ext_vector_type(16)));

// Ten fp32 coefficients as high and low fp16 parts, in pairs (m, m + 5): c = hi + lo / 2048.
__device__ __forceinline__ void split_pairs(const float (&c)[kG], uint32_t (&hi)[5], uint32_t (&lo)[5]) {
#pragma unroll
  for (int m = 0; m < 5; ++m) {
    hi[m] = flush_h2(pack_h2(c[m], c[m + 5]));
    lo[m] = flush_h2(pack_h2((c[m] - half_bits_to_float(hi[m] & 0xffffu)) * 2048.0f,
                             (c[m + 5] - half_bits_to_float(hi[m] >> 16)) * 2048.0f));
  }
}

// ---- kan_prep_coef ------------------------------------------------------------------
// Chat as uint4 records: rec[(((step*5 + S) * 2 + h) * 2 + a) * n_out + j], step = i / 16: the
// half a (elements 8a .. 8a+7) of the B operand of lane half h in sparse MFMA S of the step,
// so that both the writer and the MFMA B-operand lanes touch 16-byte items contiguous in j.
// Input ii = i % 16 of a step puts its coefficients (0,5,1,6,2,7,3,8) into record
// (S = ii / 4, h = (ii % 4) / 2, a = ii % 2) and its coefficients (4,9) into word ii % 4 of
// record (S = 4, h = ii / 8, a = (ii % 8) / 4): see the k order at kan_mfma_kernel.
// A workgroup covers 64 output columns x 32 input rows: each of its 4 waves takes 8 rows
// (half a step; lanes along the columns), so all loads of an edge's chain (metadata, then
// codeword) are in flight at once across many small waves.
// SPLIT: fp32-grade operands for the precise path at large batch: every coefficient c (fp32) is
// written as hi = fp16(c) into cf and as lo = fp16((c - hi) * 2048) into cf_lo (hi + lo / 2048
// carries 22 bits of c; the factor keeps the low parts out of the fp16 subnormals).
// The ids, gains and biases of whole tiles are fetched with 16-byte loads - a wave's 8 rows x 64
// columns of an array of E-byte elements are 512 E bytes, E / 2 loads per lane (unit t = row
// t / (4 E), 16 / E columns from (t % (4 E)) * 16 / E) - and dealt out to the lanes that own the
// columns through a strip of LDS that only this wave touches: with two-byte elements 3
// vector-memory instructions in place of 24 (the kernel is bound by its address units).
constexpr int kPrepStripBytes = 3 * 2048;      // three arrays of at most 4-byte elements

template <int E>
__device__ __forceinline__ void prep_wide_load(const void* base, int ib, int n_in, int n_out, int col0, int lane,
                                               u32x4 (&v)[(E + 1) / 2]) {
#pragma unroll
  for (int u = 0; u < (E + 1) / 2; ++u) {
    const int t = (lane + 64 * u) & (32 * E - 1);          // (one-byte arrays: the upper half of the wave repeats the lower)
    const int r = t / (4 * E), part = t % (4 * E);
    v[u] = __builtin_nontemporal_load(
        (const u32x4*)((const char*)base + ((size_t)min(ib + r, n_in - 1) * n_out + col0) * E + part * 16));
  }
}
template <int E>
__device__ __forceinline__ void prep_wide_store(unsigned char* strip, int lane, const u32x4 (&v)[(E + 1) / 2]) {
#pragma unroll
  for (int u = 0; u < (E + 1) / 2; ++u) *(u32x4*)(strip + ((lane + 64 * u) & (32 * E - 1)) * 16) = v[u];
}

template <typename IdxT, typename GbT, typename CbT, bool SPLIT>
__device__ __forceinline__ void prep_coef_block(const LayerPtrs& hp, uint4* __restrict__ cf, uint4* __restrict__ cf_lo,
                                                float* __restrict__ bp, const int n_in, const int n_out, const int bx,
                                                const int by, float (*sb)[64], unsigned char (*strips)[kPrepStripBytes]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = bx * 64 + lane;
  const IdxT* idx = (const IdxT*)hp.idx;
  const GbT* gain = (const GbT*)hp.gain;
  const GbT* bias = (const GbT*)hp.bias;
  const Q8Params qp = {hp.gain_log2_lo, hp.gain_log2_step, hp.bias_scale};
  const CbT* cb = (const CbT*)hp.cb;
  const int ib = by * kMfmaPrepRows + wave * 8;
  float bs = 0.f;
  if (j < n_out && ib < (n_in + IT - 1) / IT * IT) {      // rows past the end of a ragged last step are written as zeros
    const long long step = ib / IT;
    const int wh = (ib / 8) & 1;                          // which half of the step these 8 rows are
    uint32_t id[8];
    float g[8];
    // (uniform: a whole tile of columns, rows that are whole 16-byte units)
    // (with 32-bit ids - large codebooks, whose gathers miss in L2 - the narrow loads were the faster ones:
    // config 5's preparation 276 against 305 us)
    const bool wide = sizeof(IdxT) == 2 && (n_out & 15) == 0 && bx * 64 + 64 <= n_out &&
                      ((((size_t)hp.idx) | ((size_t)hp.gain) | ((size_t)hp.bias)) & 15) == 0;
    if (wide) {
      constexpr int EI = (int)sizeof(IdxT), EG = (int)sizeof(GbT);
      unsigned char* strip = strips[wave];
      u32x4 vi[(EI + 1) / 2], vg[(EG + 1) / 2], vb[(EG + 1) / 2];
      prep_wide_load<EI>(idx, ib, n_in, n_out, bx * 64, lane, vi);
      prep_wide_load<EG>(gain, ib, n_in, n_out, bx * 64, lane, vg);
      prep_wide_load<EG>(bias, ib, n_in, n_out, bx * 64, lane, vb);
      prep_wide_store<EI>(strip, lane, vi);                       // [row][column] per array
      prep_wide_store<EG>(strip + 2048, lane, vg);
      prep_wide_store<EG>(strip + 4096, lane, vb);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const bool ok = ib + r < n_in;
        id[r] = (uint32_t)*(const IdxT*)(strip + (r * 64 + lane) * EI);
        const GbT gr = *(const GbT*)(strip + 2048 + (r * 64 + lane) * EG);
        const GbT br = *(const GbT*)(strip + 4096 + (r * 64 + lane) * EG);
        float gv, bv;
        if constexpr (EG == 1) {
          gv = q8_gain(gr.v, qp);
          bv = q8_bias(br.v, qp);
        } else if constexpr (EG == 2) {
          gv = __half2float(gr);
          bv = __half2float(br);
        } else {
          gv = gr;
          bv = br;
        }
        g[r] = ok ? gv : 0.f;
        bs += ok ? bv : 0.f;
      }
    }
    if (!wide) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int i = ib + r;
        const bool ok = i < n_in;
        const long long e = (long long)min(i, n_in - 1) * n_out + j;
        uint32_t idv[1];
        float gv[1], bv[1];
        load_idx<IdxT, 1>(idx + e, idv);
        load_gain<GbT, 1>(gain + e, qp, gv);
        load_bias<GbT, 1>(bias + e, qp, bv);
        id[r] = idv[0];
        g[r] = ok ? gv[0] : 0.f;
        bs += ok ? bv[0] : 0.f;
      }
    }
    RawRow<CbT> raw[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) load_row<CbT>(cb, id[r], raw[r]);
#pragma unroll
    for (int r = 0; r < 8; ++r) align_row<CbT>(raw[r], row_odd<CbT>(cb, id[r]));
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const long long S = 2 * wh + q;
      uint32_t tail[4], tail_lo[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {                       // ii = 8 wh + 4 q + t: h = t / 2, a = t % 2
        const long long rec = (((step * 5 + S) * 2 + (t >> 1)) * 2 + (t & 1)) * n_out + j;
        if constexpr (SPLIT) {
          float c[kG];
          dequant_row_f32<CbT>(raw[4 * q + t], g[4 * q + t], c);
          uint32_t hi[5], lo[5];
          split_pairs(c, hi, lo);
          cf[rec] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
          cf_lo[rec] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
          tail[t] = hi[4];
          tail_lo[t] = lo[4];
        } else {
          uint32_t w[5];
          dequant_row<CbT>(raw[4 * q + t], g[4 * q + t], w);   // (c0,c1) (c2,c3) (c4,c5) (c6,c7) (c8,c9)
          const uint32_t p0 = __builtin_amdgcn_perm(w[2], w[0], 0x07060100u);   // (c0, c5)
          const uint32_t p1 = __builtin_amdgcn_perm(w[3], w[0], 0x05040302u);   // (c1, c6)
          const uint32_t p2 = __builtin_amdgcn_perm(w[3], w[1], 0x07060100u);   // (c2, c7)
          const uint32_t p3 = __builtin_amdgcn_perm(w[4], w[1], 0x05040302u);   // (c3, c8)
          tail[t] = __builtin_amdgcn_perm(w[4], w[2], 0x07060100u);             // (c4, c9)
          cf[rec] = make_uint4(p0, p1, p2, p3);
        }
      }
      const long long trec = (((step * 5 + 4) * 2 + wh) * 2 + q) * n_out + j;
      cf[trec] = make_uint4(tail[0], tail[1], tail[2], tail[3]);
      if constexpr (SPLIT) cf_lo[trec] = make_uint4(tail_lo[0], tail_lo[1], tail_lo[2], tail_lo[3]);
    }
  }
  sb[wave][lane] = bs;
  __syncthreads();
  if (wave == 0 && j < n_out)
    bp[(long long)by * n_out + j] = (sb[0][lane] + sb[1][lane]) + (sb[2][lane] + sb[3][lane]);
}

template <typename IdxT, typename GbT, typename CbT, bool SPLIT>
__global__ __launch_bounds__(kThreads) void kan_prep_coef_kernel(const PrepCoefArgs a) {
  __shared__ float sb[4][64];
  __shared__ __attribute__((aligned(16))) unsigned char strips[4][kPrepStripBytes];
  const int head = blockIdx.z;
  prep_coef_block<IdxT, GbT, CbT, SPLIT>(a.h[head], a.cf + (long long)head * a.cf_head_stride,
                                         SPLIT ? a.cf_lo + (long long)head * a.cf_head_stride : nullptr,
                                         a.bias_partial + (long long)head * a.bp_head_stride, a.n_in, a.n_out,
                                         blockIdx.x, blockIdx.y, sb, strips);
}

// ---- kan_prep_dense -----------------------------------------------------------------
// The dense baseline at large batch: its fp32 coefficients coef[i][j][10] in the split form,
// in the record order of kan_prep_coef (same grid: 64 columns x 32 rows per workgroup, a wave
// takes 8 rows).  No bias sums: the contraction is launched without them.
__global__ __launch_bounds__(kThreads) void kan_prep_dense_kernel(const float* __restrict__ coef, uint4* __restrict__ cf,
                                                                  uint4* __restrict__ cf_lo, int n_in, int n_out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane;
  const int ib = blockIdx.y * kMfmaPrepRows + wave * 8;
  if (j >= n_out || ib >= (n_in + IT - 1) / IT * IT) return;
  const long long step = ib / IT;
  const int wh = (ib / 8) & 1;
  float2 raw[8][5];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const float2* p = (const float2*)(coef + ((long long)min(ib + r, n_in - 1) * n_out + j) * kG);
#pragma unroll
    for (int m = 0; m < 5; ++m) raw[r][m] = p[m];
  }
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const long long S = 2 * wh + q;
    uint32_t tail[4], tail_lo[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const bool ok = ib + 4 * q + t < n_in;              // rows past the end of a ragged last step are zeros
      float c[kG];
#pragma unroll
      for (int m = 0; m < 5; ++m) {
        c[2 * m] = ok ? raw[4 * q + t][m].x : 0.f;
        c[2 * m + 1] = ok ? raw[4 * q + t][m].y : 0.f;
      }
      uint32_t hi[5], lo[5];
      split_pairs(c, hi, lo);
      const long long rec = (((step * 5 + S) * 2 + (t >> 1)) * 2 + (t & 1)) * n_out + j;
      cf[rec] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
      cf_lo[rec] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
      tail[t] = hi[4];
      tail_lo[t] = lo[4];
    }
    const long long trec = (((step * 5 + 4) * 2 + wh) * 2 + q) * n_out + j;
    cf[trec] = make_uint4(tail[0], tail[1], tail[2], tail[3]);
    cf_lo[trec] = make_uint4(tail_lo[0], tail_lo[1], tail_lo[2], tail_lo[3]);
  }
}

// ---- kan_prep_basis -----------------------------------------------------------------
// An input's basis word for a sample = { half2(w0, w1), half2(w2, w3) } with span bit 0, 1, 2 in
// the sign bits of w0, w1, w2 (the weights are never negative); W[i / 2][b][i % 2], so that a
// lane of the contraction kernel fetches two inputs with one 16-byte load; rows n_in .. next
// multiple of 16 are zeros.
// The input is x itself, or (x_parts > 1) the previous layer's partial sums, added here in
// the order of the slices and squashed, so that no separate reduction pass runs in between.
__device__ __forceinline__ void prep_basis_block(const float* __restrict__ xh, const int x_parts,
                                                 const long long x_part_stride, const int x_tanh,
                                                 uint2* __restrict__ wh, uint2* __restrict__ wl, const int n_in,
                                                 const int B, const int rule, const int bx, const int by,
                                                 uint2 (*tile)[33], uint2 (*tile_lo)[33]) {
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
  const int ib = bx * 32, bb = by * 32;
  // The inputs of the thread's four elements first, every load unconditional (clamped addresses): the
  // slices of all four are in flight together instead of one element's after the other's arithmetic.
  const float* xp[4];
  float xs[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    xp[r] = xh + (long long)min(bb + ty + 8 * r, B - 1) * n_in + min(ib + tx, n_in - 1);
    xs[r] = xp[r][0];
  }
  for (int p0 = 1; p0 < x_parts; p0 += 8) {           // eight slices in flight per element, added in order
    float t[8][4];
#pragma unroll
    for (int pp = 0; pp < 8; ++pp) {
      const long long off = (long long)min(p0 + pp, x_parts - 1) * x_part_stride;
#pragma unroll
      for (int r = 0; r < 4; ++r) t[pp][r] = xp[r][off];
    }
#pragma unroll
    for (int pp = 0; pp < 8; ++pp)
#pragma unroll
      for (int r = 0; r < 4; ++r) xs[r] += p0 + pp < x_parts ? t[pp][r] : 0.f;
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int b = bb + ty + 8 * r, i = ib + tx;
    uint2 v = make_uint2(0u, 0u), vlo = make_uint2(0u, 0u);
    if (b < B && i < n_in) {
      float xv = xs[r];
      if (x_tanh) xv = tanhf(xv);
      const BasisW bw = basis_fast(xv, rule);
      const uint32_t l = (uint32_t)bw.span;
      const float w0 = bw.w0, w1 = bw.w1, w2 = bw.w2, w3 = bw.w3;
      const uint32_t sx = ((l & 1u) << 15) | ((l & 2u) << 30), sy = (l & 4u) << 13;
      uint32_t hx = pack_h2(w0, w1), hy = pack_h2(w2, w3);
      if (wl) {
        // split form: the high part is the weight cut to fp16 towards zero, so that the low
        // part (w - hi) * 2048 is never negative and its sign bits are free for the span too
        const float w[4] = {w0, w1, w2, w3};
        uint32_t hb[4];
        float rest[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          hb[k] = ((k & 1) ? ((k < 2 ? hx : hy) >> 16) : ((k < 2 ? hx : hy) & 0xffffu));
          if (half_bits_to_float(hb[k]) > w[k]) hb[k] -= 1u;       // one fp16 step down (w > 0 there)
          if ((hb[k] & 0x7c00u) == 0u) hb[k] = 0u;                 // no subnormal high parts (and no -0)
          rest[k] = (w[k] - half_bits_to_float(hb[k])) * 2048.0f;
        }
        hx = hb[0] | (hb[1] << 16);
        hy = hb[2] | (hb[3] << 16);
        vlo.x = (flush_h2(pack_h2(rest[0], rest[1])) & 0x7fff7fffu) | sx;
        vlo.y = (flush_h2(pack_h2(rest[2], rest[3])) & 0x7fff7fffu) | sy;
      }
      v.x = hx | sx;
      v.y = hy | sy;
    }
    tile[ty + 8 * r][tx] = v;
    if (wl) tile_lo[ty + 8 * r][tx] = vlo;
  }
  __syncthreads();
  // the words of a pair of inputs lie side by side: one 16-byte store per thread and pair
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int p = ty + 8 * r, i = ib + 2 * p, b = bb + tx;
    if (i < (n_in + IT - 1) / IT * IT && b < B) {    // rows up to a whole step: zeros
      const uint2 e0 = tile[tx][2 * p], e1 = tile[tx][2 * p + 1];
      ((uint4*)wh)[(long long)(i >> 1) * B + b] = make_uint4(e0.x, e0.y, e1.x, e1.y);
      if (wl) {
        const uint2 l0 = tile_lo[tx][2 * p], l1 = tile_lo[tx][2 * p + 1];
        ((uint4*)wl)[(long long)(i >> 1) * B + b] = make_uint4(l0.x, l0.y, l1.x, l1.y);
      }
    }
  }
}

__global__ __launch_bounds__(256) void kan_prep_basis_kernel(const float* __restrict__ x, long long x_head_stride,
                                                             int x_parts, long long x_part_stride, int x_tanh,
                                                             uint2* __restrict__ W, uint2* __restrict__ W_lo,
                                                             long long w_head_stride, int n_in, int B, int rule) {
  __shared__ uint2 tile[32][33];
  __shared__ uint2 tile_lo[32][33];
  const int head = blockIdx.z;
  prep_basis_block(x + (long long)head * x_head_stride, x_parts, x_part_stride, x_tanh,
                   W + (long long)head * w_head_stride, W_lo ? W_lo + (long long)head * w_head_stride : nullptr, n_in, B,
                   rule, blockIdx.x, blockIdx.y, tile, tile_lo);
}

// ---- kan_prep_start -----------------------------------------------------------------
// Everything a single head's call can prepare before its first contraction, in one launch:
// the coefficient records of its matrix-core layers (they depend on the parameters only) and
// the basis words of the first layer's input.  The small grids of the later layers and the
// basis pass fill the tail of the first layer's coefficient pass instead of running as
// launches of their own behind it.  Blocks are numbered job after job, the largest first.
template <typename IdxT, typename GbT, typename CbT, bool SPLIT>
__global__ __launch_bounds__(kThreads) void kan_prep_start_kernel(const PrepStartArgs a) {
  __shared__ float sb[4][64];
  __shared__ __attribute__((aligned(16))) unsigned char strips[4][kPrepStripBytes];
  __shared__ uint2 tile[32][33];
  __shared__ uint2 tile_lo[SPLIT ? 32 : 1][33];
  const int blk = blockIdx.x;
  int k = 0;
  while (k < a.n_jobs && blk >= a.first_block[k + 1]) ++k;
  const int rel = blk - a.first_block[k];
  if (k < a.n_jobs) {
    const PrepStartArgs::Job& job = a.job[k];
    prep_coef_block<IdxT, GbT, CbT, SPLIT>(job.h, job.cf, SPLIT ? job.cf_lo : nullptr, job.bp, job.n_in, job.n_out,
                                           rel % job.nx, rel / job.nx, sb, strips);
  } else {
    prep_basis_block(a.x, 1, 0, 0, a.W, SPLIT ? a.W_lo : nullptr, a.n_in, a.B, a.rule, rel % a.basis_nx,
                     rel / a.basis_nx, tile, SPLIT ? tile_lo : tile);
  }
}

// ---- kan_mfma ---------------------------------------------------------------------------
// The Phi operand is 60 % structural zeros: of an input's ten basis values only four
// consecutive ones (l .. l+3, l = span) are nonzero.  Coefficients m and m+5 are therefore
// never both under the window, so the k order
//     group of four k-slots = [m, m+5, m', m'+5]
// holds at most two nonzeros per group whatever the span: exactly the 2:4 structure of the
// sparse matrix instruction v_smfmac_f32_32x32x32_f16, which takes the A operand as the two
// stored values of every group plus two 2-bit positions, and runs K = 32 in the time the
// dense instruction runs K = 16.  A step of 16 inputs is 40 groups = 5 such MFMAs:
//   S = 0..3   groups (0,5,1,6) and (2,7,3,8) of inputs 4S .. 4S+3
//   S = 4      groups (4,9 of input 2g; 4,9 of input 2g+1), g = 0..7
// Operand layout of the instruction (lane = 32 * half + n): the A lane (row, half a) holds
// stored values e = 0..7, value pair t = e / 2 belonging to the group at B elements
// 8a + 4 (t % 2) .. + 3 of B lane half h = t / 2, at the positions given by bits 4t .. 4t+3 of
// the lane's 16 index bits (ABID picks the low or high half of the index register).
//
// MB = MFMA row blocks per wave (tile of 32 MB samples), NB = column blocks per wave (the
// four waves cover 128 NB outputs).  MB = 4 reads half the Chat bytes per MFMA; MB = 2 is
// for layers whose grid of 128-sample tiles would leave CUs idle (three workgroups per CU).

// Per span l: byte-permute selectors that pick, from the four fp16 weights {w23:w01} of an
// input, the stored values of its pairs (m, m+5): word 0 pairs 0 and 1, word 1 pairs 2 and 3,
// word 2 pair 4 (high half zero); word 3 the index byte of the input's two full groups
// (nibble = position of the first value | position of the second << 2) and, in bit 8, whether
// pair 4 takes coefficient 9: one 16-byte table read per input.  Selector byte 0x0c yields 0.
__device__ __forceinline__ void fill_sparse_selectors(uint32_t (*sel)[8], int tid) {
  if (tid < kSpans) {
    const int l = tid;
    uint32_t half_sel[5], hi[5];
#pragma unroll
    for (int p = 0; p < 5; ++p) {
      int k = -1;
      hi[p] = 0;
      if (p >= l && p <= l + 3) k = p - l;
      else if (p + 5 >= l && p + 5 <= l + 3) { k = p + 5 - l; hi[p] = 1; }
      half_sel[p] = k >= 0 ? (uint32_t)((2 * k) | ((2 * k + 1) << 8)) : 0x0c0cu;
    }
    sel[l][0] = half_sel[0] | (half_sel[1] << 16);
    sel[l][1] = half_sel[2] | (half_sel[3] << 16);
    sel[l][2] = half_sel[4] | 0x0c0c0000u;
    sel[l][3] = (hi[0] | ((2u + hi[1]) << 2)) | ((hi[2] | ((2u + hi[3]) << 2)) << 4) | (hi[4] << 8);
    sel[l][4] = sel[l][5] = sel[l][6] = sel[l][7] = 0;
  }
}

template <int MB, int NB, bool THREE, int NW = 4>
__global__ __launch_bounds__(64 * NW, NW == 8 ? 1 : (MB == 2 ? 3 : 2)) void kan_mfma_kernel(const MfmaArgs a) {
  constexpr int kThreadsWg = 64 * NW;  // NW waves side by side along the outputs, all reading one Phi tile
  constexpr int BM = 32 * MB;          // samples per workgroup tile (MB = MFMA row blocks per wave)
  constexpr int BN = NW * 32 * NB;     // outputs per workgroup tile
  constexpr int NSUB = BM * 4 / kThreadsWg;   // quarters of a step (inputs 4 ph .. 4 ph + 3) per thread
  constexpr int NPAIR = 4 * NSUB;      // (sample, input) pairs per thread and step
  static_assert(NSUB >= 1 && BM * 4 == kThreadsWg * NSUB && IT == 16, "threads of a sample row share out the four quarters of a step");
  // Phi tiles.  Four waves: two tiles, a barrier per step.  Eight waves (alone on their CU, so the LDS is
  // theirs): four tiles, built two steps ahead, and a barrier every second step - between two barriers the
  // waves read tiles k, k + 1 and write tiles k + 2, k + 3, and may drift apart by up to two steps.
  constexpr int kAhead = NW == 8 ? 2 : 1;
  constexpr int kTiles = 2 * kAhead;
  __shared__ __attribute__((aligned(16))) unsigned char sA[kTiles][BM * kRowBytes];
  __shared__ __attribute__((aligned(16))) uint32_t sSel[kSpans][8];
  fill_sparse_selectors(sSel, threadIdx.x);
  __syncthreads();

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int wn = wave;
  const int head = blockIdx.z;
  // Which (tile, chunk of inputs) this workgroup takes.  Workgroups go to the eight XCDs in
  // turn (linear index mod 8), and each XCD has its own L2: giving an XCD all tiles of the same
  // chunk(s) makes its L2 hold one slice of the inputs of both operands, each fetched from
  // memory once, instead of every XCD fetching the whole basis operand.
  // Within a chunk the tiles are taken in patches of 64, the workgroups an XCD runs at a time: 32
  // sample tiles x 2 output tiles where the grid allows it (they then share two slices of the
  // coefficient records, the larger operand, 32 ways; measured on 4096 x 4096 at batch 8192 against 8 x 8:
  // 2.17 against 2.25 ms, 16 x 4: 2.23, 4 x 16: 2.6-2.7, 2 x 32: 3.04), else 8 x 8.
  int chunk = blockIdx.y, seq = blockIdx.x;
  const int T = gridDim.x, njt = a.n_jt, nbt = T / njt;
  {
    const int C = gridDim.y;
    const int L = blockIdx.x + T * blockIdx.y, xcd = L & 7, m = L >> 3;
    if ((T * C) % 8 == 0) {
      if (C % 8 == 0) {
        chunk = xcd + 8 * (m / T);
        seq = m % T;
      } else if (8 % C == 0 && T % (8 / C) == 0) {      // 8 / C XCDs per chunk, a run of tiles each
        chunk = xcd % C;
        seq = (xcd / C) * (T / (8 / C)) + m;
      }
    }
  }
  int jt = seq % njt, bt = seq / njt;
  constexpr int kPatchJ = 2;        // output tiles of a patch of 64 workgroups (sample tiles: 64 / kPatchJ), else 8 x 8
  const int pj = (njt % kPatchJ == 0 && nbt % (64 / kPatchJ) == 0) ? kPatchJ : ((njt % 8 == 0 && nbt % 8 == 0) ? 8 : 0);
  if (pj) {
    const int pb = 64 / pj;
    const int patch = seq >> 6, w = seq & 63, per_row = njt / pj;
    bt = (patch / per_row) * pb + w / pj;
    jt = (patch % per_row) * pj + w % pj;
  }
  const int b0 = bt * BM, j0 = jt * BN;
  const int n_in = a.n_in, n_out = a.n_out, B = a.B;
  const int i_begin = chunk * a.rows_per_chunk;
  const int i_end = min(n_in, i_begin + a.rows_per_chunk);
  const int n_steps = (i_end - i_begin + IT - 1) / IT;
  const int step0 = i_begin / IT;
  const int last_step = (n_in + IT - 1) / IT - 1;

  // Passes over the chunk's steps.  One pass: operands (W, cf).  Three (split form): first the
  // cross products (W, cf_lo) and (W_lo, cf), whose low operands carry a factor 2048, then the
  // accumulators are scaled by 1 / 2048 (exact) and the main product (W, cf) is added on top.
  // Virtual step k = pass * n_steps + step; n1, n2 are the first steps of passes 1 and 2.
  constexpr bool three = THREE;       // (a.passes == 3; a template parameter so that the one-pass form carries none of it)
  const int total_steps = three ? 3 * n_steps : n_steps;
  const int n1 = three ? n_steps : 0x3fffffff, n2 = three ? 2 * n_steps : 0x3fffffff;
  const uint4* cf_main = a.cf + (long long)head * a.cf_head_stride;
  const uint2* W_main = a.W + (long long)head * a.w_head_stride;
  const uint4* cf_low = three ? a.cf_lo + (long long)head * a.cf_head_stride : cf_main;
  const uint2* W_low = three ? a.W_lo + (long long)head * a.w_head_stride : W_main;

  // Phi generation: this thread owns sample row pb and inputs 4 ph0 .. 4 ph0 + NPAIR - 1 of every step.
  const int pb = tid & (BM - 1);
  const int ph0 = __builtin_amdgcn_readfirstlane(tid / BM) * NSUB;      // first quarter of this thread
  // B operand: columns jc[nb]
  int jc[NB];
  bool j_ok[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int j = j0 + wn * (32 * NB) + nb * 32 + ln;
    j_ok[nb] = j < n_out;
    jc[nb] = min(j, n_out - 1);
  }

  f32x16 acc[MB][NB];
#pragma unroll
  for (int m = 0; m < MB; ++m)
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.f;

  // Every load of the main loop is a buffer load: the resource (base, size) is rebuilt on the
  // scalar unit for each step, the lane offsets never change, so a load costs no vector
  // arithmetic.  Offsets stay below 2^31 because a resource spans one step of one head.
  const uint32_t u_off = (uint32_t)min(b0 + pb, B - 1) * (uint32_t)sizeof(uint4);
  const uint32_t w_row_bytes = (uint32_t)B * (uint32_t)sizeof(uint4);       // a pair of inputs
  auto u_rsrc = [&](int kv) {                            // virtual step index
    // (the rows of a ragged last step exist and hold zeros; past the chunk: valid memory, never used)
    const int k = kv - (kv >= n2 ? n2 : (kv >= n1 ? n1 : 0));
    const char* w_bytes = (const char*)((three && kv >= n1 && kv < n2) ? W_low : W_main);
    const int i = min(step0 + k, last_step) * IT + 4 * ph0;
    const char* rows = w_bytes + (size_t)(i >> 1) * w_row_bytes;
    return __builtin_amdgcn_make_buffer_rsrc((void*)rows, 0, (int)(NPAIR / 2 * w_row_bytes), kBufferFlags);
  };
  auto load_u_one = [&](const __amdgpu_buffer_rsrc_t r, int q, uint2 (&uv)[NPAIR]) {      // pair q of the thread's inputs
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)u_off, (int)(q * w_row_bytes), 0);
    uv[2 * q] = make_uint2(v.x, v.y);
    uv[2 * q + 1] = make_uint2(v.z, v.w);
  };
  auto load_u = [&](int kv, uint2 (&uv)[NPAIR]) {
    const __amdgpu_buffer_rsrc_t r = u_rsrc(kv);
#pragma unroll
    for (int q = 0; q < NPAIR / 2; ++q) load_u_one(r, q, uv);
  };

  // Input 4 ph + q = 4 S + 2 x + a with S = ph: its four stored values go to bytes x * 8 of
  // fragment (S, a); its pair-4 value to half q of the 8 bytes that fragment (4, ph % 2)
  // keeps for inputs 4 ph .. 4 ph + 3; index bytes likewise.  (Quarter ph of the step.)
  auto gen_phi = [&](const uint2 (&uv)[NPAIR], unsigned char* tile) {
    unsigned char* rowp = tile + pb * kRowBytes;
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
      const int ph = ph0 + sub;
      uint32_t v4[4], ib[4], h4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint32_t l, w01, w23;
        unpack_basis(uv[4 * sub + q], l, w01, w23);
        const uint4 sl = *(const uint4*)&sSel[l][0];
        uint2 st;
        st.x = __builtin_amdgcn_perm(w23, w01, sl.x);
        st.y = __builtin_amdgcn_perm(w23, w01, sl.y);
        v4[q] = __builtin_amdgcn_perm(w23, w01, sl.z);
        ib[q] = sl.w & 0xffu;
        h4[q] = sl.w >> 8;            // (word 3 carries both: one table read per input)
        *(uint2*)(rowp + (ph * 2 + (q & 1)) * 16 + (q >> 1) * 8) = st;
      }
      uint2 t4;
      t4.x = v4[0] | (v4[1] << 16);
      t4.y = v4[2] | (v4[3] << 16);
      *(uint2*)(rowp + 128 + (ph & 1) * 16 + (ph >> 1) * 8) = t4;
      *(uint16_t*)(rowp + kIdxOffset + 0 * 16 + ph * 2) = (uint16_t)(ib[0] | (ib[2] << 8));
      *(uint16_t*)(rowp + kIdxOffset + 1 * 16 + ph * 2) = (uint16_t)(ib[1] | (ib[3] << 8));
      *(uint8_t*)(rowp + kIdxOffset + (ph & 1) * 16 + 8 + (ph >> 1)) =
          (uint8_t)((h4[0] | ((2u + h4[1]) << 2)) | ((h4[2] | ((2u + h4[3]) << 2)) << 4));
    }
  };

  // The same in three pieces for threads that own one quarter of a step (NSUB = 1), so that the step can place
  // them behind its MFMAs: the selector row of input q is requested (LDS), later its values are permuted and
  // stored, last the words that collect bits of all four inputs.
  struct PhiState {
    uint4 sel[4];
    uint32_t v4[4], ib[4], h4[4];
  };
  auto phi_request = [&](const uint2 (&uv)[NPAIR], int q, PhiState& ps) {
    uint32_t l, w01, w23;
    unpack_basis(uv[q], l, w01, w23);
    ps.sel[q] = *(const uint4*)&sSel[l][0];
  };
  auto phi_place = [&](const uint2 (&uv)[NPAIR], int q, PhiState& ps, unsigned char* tile) {
    unsigned char* rowp = tile + pb * kRowBytes;
    uint32_t l, w01, w23;
    unpack_basis(uv[q], l, w01, w23);
    const uint4 sl = ps.sel[q];
    uint2 st;
    st.x = __builtin_amdgcn_perm(w23, w01, sl.x);
    st.y = __builtin_amdgcn_perm(w23, w01, sl.y);
    ps.v4[q] = __builtin_amdgcn_perm(w23, w01, sl.z);
    ps.ib[q] = sl.w & 0xffu;
    ps.h4[q] = sl.w >> 8;
    *(uint2*)(rowp + (ph0 * 2 + (q & 1)) * 16 + (q >> 1) * 8) = st;
  };
  auto phi_finish = [&](const PhiState& ps, unsigned char* tile) {
    unsigned char* rowp = tile + pb * kRowBytes;
    const int ph = ph0;
    uint2 t4;
    t4.x = ps.v4[0] | (ps.v4[1] << 16);
    t4.y = ps.v4[2] | (ps.v4[3] << 16);
    *(uint2*)(rowp + 128 + (ph & 1) * 16 + (ph >> 1) * 8) = t4;
    *(uint16_t*)(rowp + kIdxOffset + 0 * 16 + ph * 2) = (uint16_t)(ps.ib[0] | (ps.ib[2] << 8));
    *(uint16_t*)(rowp + kIdxOffset + 1 * 16 + ph * 2) = (uint16_t)(ps.ib[1] | (ps.ib[3] << 8));
    *(uint8_t*)(rowp + kIdxOffset + (ph & 1) * 16 + 8 + (ph >> 1)) =
        (uint8_t)((ps.h4[0] | ((2u + ps.h4[1]) << 2)) | ((ps.h4[2] | ((2u + ps.h4[3]) << 2)) << 4));
  };

  // Chat fragments of half a step (S = 2 hs, 2 hs + 1 and half hs of S = 4): 5 uint4 per
  // column block: [0] (S0, a=0) [1] (S0, a=1) [2] (S1, a=0) [3] (S1, a=1) [4] (S = 4, a = hs),
  // all of B lane half lh.
  uint32_t b_off[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) b_off[nb] = (uint32_t)(lh * 2 * n_out + jc[nb]) * (uint32_t)sizeof(uint4);
  const uint32_t a_bytes = (uint32_t)n_out * (uint32_t)sizeof(uint4);     // from a = 0 to a = 1
  const uint32_t s_bytes = 4u * a_bytes;                                  // from S to S + 1
  auto step_rsrc = [&](int kv) {                         // virtual step index
    const int k = kv - (kv >= n2 ? n2 : (kv >= n1 ? n1 : 0));
    const char* cf_bytes = (const char*)((three && kv < n1) ? cf_low : cf_main);
    const int step = min(step0 + k, last_step);         // past the end: valid memory, never used
    const char* sb = cf_bytes + (size_t)step * (5 * s_bytes);
    return __builtin_amdgcn_make_buffer_rsrc((void*)sb, 0, (int)(5 * s_bytes), kBufferFlags);
  };
  auto load_b_main = [&](int k, auto HS, uint4 (&bf)[NB][5]) {
    constexpr int hs = decltype(HS)::value;
    const __amdgpu_buffer_rsrc_t r = step_rsrc(k);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)b_off[nb],
                                                              (int)((2 * hs + (u >> 1)) * s_bytes + (u & 1) * a_bytes), 0);
        bf[nb][u] = make_uint4(v.x, v.y, v.z, v.w);
      }
  };
  auto load_b_one = [&](const __amdgpu_buffer_rsrc_t r, auto HS, int u, uint4 (&bf)[NB][5]) {      // fragment u = 0..3 of the half step
    constexpr int hs = decltype(HS)::value;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)b_off[nb],
                                                            (int)((2 * hs + (u >> 1)) * s_bytes + (u & 1) * a_bytes), 0);
      bf[nb][u] = make_uint4(v.x, v.y, v.z, v.w);
    }
  };
  auto load_b_tail = [&](int k, auto HS, uint4 (&bf)[NB][5]) {
    constexpr int hs = decltype(HS)::value;
    const __amdgpu_buffer_rsrc_t r = step_rsrc(k);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)b_off[nb], (int)(4 * s_bytes + hs * a_bytes), 0);
      bf[nb][4] = make_uint4(v.x, v.y, v.z, v.w);
    }
  };

  // The index words and stored values of this lane's rows, then the sparse MFMAs S0, S0 + 1
  // of the step with the fragments of one half step.
  auto read_idx = [&](const unsigned char* tile, uint4 (&ix)[MB]) {
#pragma unroll
    for (int m = 0; m < MB; ++m) ix[m] = *(const uint4*)(tile + (m * 32 + ln) * kRowBytes + kIdxOffset + lh * 16);
  };
  // A fragments of MFMA group g of the step (g = 2 hs + q for the pairs, 4 for the tail): one 16-byte LDS
  // read per row block.  The groups run through two register sets: while the matrix pipe works on group g the
  // reads of group g + 2 are already on their way, so that no MFMA waits for an LDS round trip of its own
  // (the compiler, left alone, reads every fragment right in front of its MFMA and waits each time).
  auto read_a = [&](const unsigned char* tile, auto G, h16x8 (&fa)[MB]) {
    constexpr int g = decltype(G)::value;
    constexpr int off = g < 4 ? g * 32 : 128;
#pragma unroll
    for (int m = 0; m < MB; ++m)
      fa[m] = __builtin_bit_cast(h16x8, *(const uint4*)(tile + (m * 32 + ln) * kRowBytes + off + lh * 16));
  };
  // (`between(m)` runs behind the m-th MFMA of the group, pinned there: the loads it issues go out in the shadow
  // of the matrix pipe instead of in one burst at the end of the step, when every wave of the CU would queue
  // at the address unit at once and none would have an MFMA to issue)
  auto mfma_group = [&](auto G, const h16x8 (&fa)[MB], const uint4 (&ix)[MB], const uint4 (&bf0)[NB][5], const uint4 (&bf1)[NB][5],
                        auto&& between) {
    constexpr int g = decltype(G)::value;
    constexpr int hs = g >> 1, q = g & 1;
#pragma unroll
    for (int n = 0; n < NB; ++n) {
      // pairs: fragments 2 q, 2 q + 1 of the half step (bf0); tail: the S = 4 fragments of both half steps
      const uint4 two[2] = {g < 4 ? bf0[n][2 * q] : bf0[n][4], g < 4 ? bf0[n][2 * q + 1] : bf1[n][4]};
      const h16x16 fb = __builtin_bit_cast(h16x16, two);
#pragma unroll
      for (int m = 0; m < MB; ++m) {
        const int iw = g == 4 ? (int)ix[m].z : (hs == 0 ? (int)ix[m].x : (int)ix[m].y);   // S = 2 hs + q: word hs, half q
        if (g < 4 && q == 1) acc[m][n] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(fa[m], fb, acc[m][n], iw, 0, 1);
        else acc[m][n] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(fa[m], fb, acc[m][n], iw, 0, 0);
        if (n == NB - 1) {
          __builtin_amdgcn_sched_barrier(0);
          between(m);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };
  auto nothing = [](int) {};

  // ---- pipeline.  Fragments travel in half steps through a ring of three register slots
  // (half step H in slot H mod 3), basis words in whole steps through a ring of three; all
  // slots are compile-time, so the loop is unrolled by three steps.  Top of step k: Phi tiles
  // k .. k + kAhead - 1 and the fragments of half steps 2k, 2k+1 are ready, those of 2k+2 and the
  // basis words of steps k + kAhead, k + kAhead + 1 are in flight; the step requests the basis words
  // of step k + kAhead + 2 (behind MFMA group 0) and the fragments of half steps 2k+3 (behind group 2)
  // and 2k+4 (behind group 4), and builds tile k + kAhead.  The S = 4 fragment of half step 2k is
  // needed until the end of the step, so its successor (half step 2k+3) is requested in two parts.
  // The bias sums of the tile's columns are fetched ahead of everything else (thread t owns
  // column j0 + t) and parked in LDS until the epilogue, so their latency is never exposed.
  static_assert(BN <= kThreadsWg, "one bias column per thread (the others repeat the last column)");
  __shared__ float sBias[kThreadsWg];
  const float* bp = a.bias_partial + (long long)head * a.bp_head_stride + min(j0 + tid, n_out - 1);
  const int rb0 = i_begin / kMfmaPrepRows, rb1 = (i_end + kMfmaPrepRows - 1) / kMfmaPrepRows;
  float bias_v[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) bias_v[u] = bp[(long long)min(rb0 + u, rb1 - 1) * n_out];

  using HS0 = std::integral_constant<int, 0>;
  using HS1 = std::integral_constant<int, 1>;
  uint4 bfr[3][NB][5];
  uint2 uv[3][NPAIR];
  load_u(0, uv[0]);
  load_b_main(0, HS0{}, bfr[0]);
  load_b_tail(0, HS0{}, bfr[0]);
  load_b_main(0, HS1{}, bfr[1]);
  load_b_tail(0, HS1{}, bfr[1]);
  load_u(1, uv[1]);
  load_b_main(1, HS0{}, bfr[2]);
  load_b_tail(1, HS0{}, bfr[2]);
  load_u(2, uv[2]);
  {
    float bs = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) bs += rb0 + u < rb1 ? bias_v[u] : 0.f;
    for (int rb = rb0 + 8; rb < rb1; ++rb) bs += bp[(long long)rb * n_out];
    sBias[tid] = a.bias_on ? bs : 0.f;      // read after the barriers of the main loop
  }
  gen_phi(uv[0], sA[0]);
  if constexpr (kAhead == 2) {
    gen_phi(uv[1], sA[1]);
    load_u(3, uv[0]);
  }

  auto step = [&](auto T, int k) {
    constexpr int t = decltype(T)::value;          // k mod 3
    constexpr int sa = (2 * t) % 3, sb = (2 * t + 1) % 3;
    const unsigned char* tile = sA[k & (kTiles - 1)];
    // tiles k .. k + kAhead - 1 are complete; every wave is done reading the tiles before them
    if (kAhead == 1 || (k & 1) == 0) __syncthreads();
    if (three && k == n2) {       // split form: the cross products are complete
      const float f = a.lo_scale;
#pragma unroll
      for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int n = 0; n < NB; ++n)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[m][n][r] *= f;
    }
    uint4 ix[MB];
    h16x8 fa0[MB], fa1[MB];
    using G0 = std::integral_constant<int, 0>;
    using G1 = std::integral_constant<int, 1>;
    using G2 = std::integral_constant<int, 2>;
    using G3 = std::integral_constant<int, 3>;
    using G4 = std::integral_constant<int, 4>;
    // resources of the loads of this step (scalar arithmetic, ahead of the MFMA groups)
    const __amdgpu_buffer_rsrc_t ru = u_rsrc(k + 2 + kAhead), r1 = step_rsrc(k + 1), r2 = step_rsrc(k + 2);
    constexpr int kUPerMfma = (NPAIR / 2 + MB - 1) / MB, kBPerMfma = 4 / MB;     // loads behind each MFMA of a group
    read_idx(tile, ix);
    read_a(tile, G0{}, fa0);
    read_a(tile, G1{}, fa1);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(2);     // the wave that has its operands goes first at the matrix pipe (measured: 1.5-2 %)
    // basis words of step k + 2 + kAhead, into the slot whose words went into a tile a step ago
    mfma_group(G0{}, fa0, ix, bfr[sa], bfr[sa], [&](int m) {
#pragma unroll
      for (int q = m * kUPerMfma; q < (m + 1) * kUPerMfma; ++q)
        if (q < NPAIR / 2) load_u_one(ru, q, uv[(t + kAhead + 2) % 3]);
    });
    read_a(tile, G2{}, fa0);
    __builtin_amdgcn_sched_barrier(0);
    // (threads with one quarter of the step: the next tile is built behind the MFMAs of groups 1 and 3)
    constexpr bool kPhiInShadow = NSUB == 1 && MB == 4;
    PhiState phs;
    const uint2 (&uvn)[NPAIR] = uv[(t + kAhead) % 3];
    unsigned char* tile_next = sA[(k + kAhead) & (kTiles - 1)];     // basis tile of step k + kAhead
    mfma_group(G1{}, fa1, ix, bfr[sa], bfr[sa], [&](int m) {
      if constexpr (kPhiInShadow) phi_request(uvn, m, phs);
    });
    read_a(tile, G3{}, fa1);
    __builtin_amdgcn_sched_barrier(0);
    // half step 2k+3 (fragments 0..3 of this step's first half are done with; its S = 4 fragment follows below)
    mfma_group(G2{}, fa0, ix, bfr[sb], bfr[sb], [&](int m) {
#pragma unroll
      for (int u = m * kBPerMfma; u < (m + 1) * kBPerMfma; ++u) load_b_one(r1, HS1{}, u, bfr[sa]);
    });
    read_a(tile, G4{}, fa0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(G3{}, fa1, ix, bfr[sb], bfr[sb], [&](int m) {
      if constexpr (kPhiInShadow) phi_place(uvn, m, phs, tile_next);
    });
    // half step 2k+4
    mfma_group(G4{}, fa0, ix, bfr[sa], bfr[sb], [&](int m) {
#pragma unroll
      for (int u = m * kBPerMfma; u < (m + 1) * kBPerMfma; ++u) load_b_one(r2, HS0{}, u, bfr[sb]);
    });
    __builtin_amdgcn_s_setprio(0);
    load_b_tail(k + 1, HS1{}, bfr[sa]);
    load_b_tail(k + 2, HS0{}, bfr[sb]);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (kPhiInShadow) phi_finish(phs, tile_next);
    else gen_phi(uvn, tile_next);
  };
  // Whole groups of three steps run without a branch between them: a branch around a step makes
  // the compiler lose count of the loads in flight and wait for all of them.
  int k = 0;
  for (; k + 3 <= total_steps; k += 3) {
    step(std::integral_constant<int, 0>{}, k);
    step(std::integral_constant<int, 1>{}, k + 1);
    step(std::integral_constant<int, 2>{}, k + 2);
  }
  if (k < total_steps) step(std::integral_constant<int, 0>{}, k);
  if (k + 1 < total_steps) step(std::integral_constant<int, 1>{}, k + 1);

  // ---- epilogue.  D layout of the 32x32 MFMA: lane holds column (lane & 31), rows
  //      8*(r/4) + 4*(lane/32) + r%4 for r = 0..15 -------------------------------------------
  const float scale = a.scale[head];
  float* dst = a.dst + (long long)head * a.dst_head_stride + (long long)chunk * a.dst_chunk_stride;
#pragma unroll
  for (int n = 0; n < NB; ++n) {
    const float bs = sBias[wn * (32 * NB) + n * 32 + ln];
    if (j_ok[n]) {
#pragma unroll
      for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int b = b0 + m * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (b < B) {
            float v = fmaf(scale, acc[m][n][r], bs);
            if (a.apply_tanh) v = tanhf(v);
            dst[(long long)b * n_out + jc[n]] = v;
          }
        }
    }
  }
}

template <typename T>
struct TypeTag {
  using type = T;
};

// Calls launch(gain/bias type, codebook type) for the layer's storage types.
template <typename F>
hipError_t prep_types(const GatherCfg& c, F&& launch) {
  if (c.code == kCbI8) {
    if (c.gb_kind == kGbQ8) launch(TypeTag<q8_t>(), TypeTag<int8_t>());
    else if (c.gb_kind == kGbF16) launch(TypeTag<__half>(), TypeTag<int8_t>());
    else launch(TypeTag<float>(), TypeTag<int8_t>());
  } else {
    if (c.gb_kind == kGbQ8) return hipErrorInvalidValue;    // byte-coded gain/bias go with Int8 codebooks
    if (c.code == kCbBfp8) {
      if (c.gb_kind == kGbF16) launch(TypeTag<__half>(), TypeTag<bfp8_t>());
      else launch(TypeTag<float>(), TypeTag<bfp8_t>());
    } else if (c.code == kCbF16) {
      if (c.gb_kind == kGbF16) launch(TypeTag<__half>(), TypeTag<__half>());
      else launch(TypeTag<float>(), TypeTag<__half>());
    } else if (c.gb_kind == kGbF16) launch(TypeTag<__half>(), TypeTag<float>());
    else launch(TypeTag<float>(), TypeTag<float>());
  }
  return hipGetLastError();
}

template <typename IdxT, bool SPLIT>
hipError_t prep_coef_types(const GatherCfg& c, const PrepCoefArgs& a, dim3 grid, hipStream_t s) {
  return prep_types(c, [&](auto gb, auto cb) {
    hipLaunchKernelGGL((kan_prep_coef_kernel<IdxT, typename decltype(gb)::type, typename decltype(cb)::type, SPLIT>), grid,
                       dim3(kThreads), 0, s, a);
  });
}

template <typename IdxT, bool SPLIT>
hipError_t prep_start_types(const GatherCfg& c, const PrepStartArgs& a, dim3 grid, hipStream_t s) {
  return prep_types(c, [&](auto gb, auto cb) {
    hipLaunchKernelGGL((kan_prep_start_kernel<IdxT, typename decltype(gb)::type, typename decltype(cb)::type, SPLIT>), grid,
                       dim3(kThreads), 0, s, a);
  });
}

}  // namespace

hipError_t launch_prep_coef(const GatherCfg& c, const PrepCoefArgs& a, int heads, hipStream_t s) {
  if (c.code == kDense) return hipErrorInvalidValue;
  dim3 grid((a.n_out + 63) / 64, (a.n_in + kMfmaPrepRows - 1) / kMfmaPrepRows, heads);
  if (a.cf_lo) return c.idx_u32 ? prep_coef_types<uint32_t, true>(c, a, grid, s) : prep_coef_types<uint16_t, true>(c, a, grid, s);
  return c.idx_u32 ? prep_coef_types<uint32_t, false>(c, a, grid, s) : prep_coef_types<uint16_t, false>(c, a, grid, s);
}

hipError_t launch_prep_start(const GatherCfg& c, PrepStartArgs& a, bool split, hipStream_t s) {
  if (c.code == kDense || a.n_jobs < 1 || a.n_jobs > kStartJobs || !a.x || !a.W || (split && !a.W_lo)) return hipErrorInvalidValue;
  long long blocks = 0;
  for (int k = 0; k < a.n_jobs; ++k) {
    PrepStartArgs::Job& job = a.job[k];
    if (!job.cf || !job.bp || (split && !job.cf_lo)) return hipErrorInvalidValue;
    job.nx = (job.n_out + 63) / 64;
    a.first_block[k] = (int)blocks;
    blocks += (long long)job.nx * ((job.n_in + kMfmaPrepRows - 1) / kMfmaPrepRows);
  }
  a.first_block[a.n_jobs] = (int)blocks;
  a.basis_nx = (a.n_in + 31) / 32;
  blocks += (long long)a.basis_nx * ((a.B + 31) / 32);
  if (blocks != prep_start_blocks(a) || blocks > kPrepStartMaxBlocks) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks, 1, 1);
  if (split) return c.idx_u32 ? prep_start_types<uint32_t, true>(c, a, grid, s) : prep_start_types<uint16_t, true>(c, a, grid, s);
  return c.idx_u32 ? prep_start_types<uint32_t, false>(c, a, grid, s) : prep_start_types<uint16_t, false>(c, a, grid, s);
}

hipError_t launch_prep_dense(const float* coef, uint4* cf, uint4* cf_lo, int n_in, int n_out, hipStream_t s) {
  if (!coef || !cf || !cf_lo) return hipErrorInvalidValue;
  dim3 grid((n_out + 63) / 64, (n_in + kMfmaPrepRows - 1) / kMfmaPrepRows, 1);
  hipLaunchKernelGGL(kan_prep_dense_kernel, grid, dim3(kThreads), 0, s, coef, cf, cf_lo, n_in, n_out);
  return hipGetLastError();
}

hipError_t launch_prep_basis(const float* x, long long x_head_stride, int x_parts, long long x_part_stride,
                             int x_tanh, uint2* W, uint2* W_lo, long long w_head_stride, int n_in, int B, int heads,
                             int rule, hipStream_t s) {
  if (x_parts < 1) return hipErrorInvalidValue;
  dim3 grid((n_in + 31) / 32, (B + 31) / 32, heads);
  hipLaunchKernelGGL(kan_prep_basis_kernel, grid, dim3(256), 0, s, x, x_head_stride, x_parts, x_part_stride, x_tanh,
                     W, W_lo, w_head_stride, n_in, B, rule);
  return hipGetLastError();
}

hipError_t launch_mfma(const MfmaArgs& a, int tile_m, int tile_n, dim3 grid, hipStream_t s) {
  if (tile_n == 256) {          // eight waves, one workgroup per CU (128-sample tiles only: 64 x 4 threads build a 64-row tile)
    if (tile_m != 128) return hipErrorInvalidValue;
    if (a.passes != 1 && (a.passes != 3 || !a.cf_lo || !a.W_lo)) return hipErrorInvalidValue;
    if ((long long)a.n_jt * tile_n < a.n_out) return hipErrorInvalidValue;
    if ((long long)a.n_out * 20 * (long long)sizeof(uint4) > 0x7fffffffLL ||
        (long long)a.B * 8 * (long long)sizeof(uint2) > 0x7fffffffLL)
      return hipErrorInvalidValue;
    if (a.passes == 3) hipLaunchKernelGGL((kan_mfma_kernel<4, 1, true, 8>), grid, dim3(2 * kMfmaThreads), 0, s, a);
    else hipLaunchKernelGGL((kan_mfma_kernel<4, 1, false, 8>), grid, dim3(2 * kMfmaThreads), 0, s, a);
    return hipGetLastError();
  }
  if ((tile_m != 64 && tile_m != 128) || tile_n != 128) return hipErrorInvalidValue;
  if (a.passes != 1 && (a.passes != 3 || !a.cf_lo || !a.W_lo)) return hipErrorInvalidValue;
  if ((long long)a.n_jt * tile_n < a.n_out) return hipErrorInvalidValue;
  // one step of coefficient records and one row of basis words must fit a buffer resource
  if ((long long)a.n_out * 20 * (long long)sizeof(uint4) > 0x7fffffffLL ||
      (long long)a.B * 8 * (long long)sizeof(uint2) > 0x7fffffffLL)
    return hipErrorInvalidValue;
  if (a.passes == 3) {
    if (tile_m == 128) hipLaunchKernelGGL((kan_mfma_kernel<4, 1, true>), grid, dim3(kMfmaThreads), 0, s, a);
    else hipLaunchKernelGGL((kan_mfma_kernel<2, 1, true>), grid, dim3(kMfmaThreads), 0, s, a);
  } else {
    if (tile_m == 128) hipLaunchKernelGGL((kan_mfma_kernel<4, 1, false>), grid, dim3(kMfmaThreads), 0, s, a);
    else hipLaunchKernelGGL((kan_mfma_kernel<2, 1, false>), grid, dim3(kMfmaThreads), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace kan
