// Matrix-core path of the VQ-KAN forward pass for gfx950 (large batch).
//
// The layer sum y[b][j] = sum_i sum_m B_m(x_bi) * c_ij[m] (paper section 3 with
// the reconstructed coefficients of section 4.2) is a contraction over
// k = (i, m), m = 0..9:
//     Y[b][j] = scale * sum_k Phi[b][k] * Chat[k][j] + sum_i bias_ij
//     Phi[b][(i,m)]  = B_m(x_bi)            (4 nonzeros per 10, App. A.1 family)
//     Chat[(i,m)][j] = gain_ij * q_ij[m]    (q = Int8 codeword, or the fp32 row)
// Both operands are fp16 (11-bit significand, same matrix-core rate as bf16, all
// values lie in [-2, 2]); products accumulate in fp32 in v_mfma_f32_32x32x16_f16.
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
//                   ([input][sample]) so that the contraction kernel reads it
//                   coalesced.
//   kan_mfma        64 samples x 256 outputs per workgroup, 4 waves side by side
//                   along the outputs (wave tile 64 x 64); two workgroups share a
//                   CU and drift apart, so one's MFMAs overlap the other's tile
//                   generation and LDS latency.  Per step of 8 inputs:
//                   the Phi tile is built in LDS (double buffered) from the packed
//                   basis words with byte permutes whose selectors come from a
//                   7-entry table (one row per span), the Chat fragments stream
//                   from memory straight into registers one step ahead, 20
//                   MFMAs per wave.
// k order inside a step of 8 inputs (80 slots = 5 MFMA k-steps x 2 lane halves x 8):
// k-step s < 4, half h carries coefficients 0..7 of input 4h+s; k-step 4, half h
// carries coefficients 8, 9 of inputs 4h..4h+3.

#include <type_traits>

#include "kan_device.hpp"
#include "kan_internal.hpp"
#include "kan_mfma_common.hpp"

namespace kan {
namespace {

constexpr int kThreads = 256;          // preparation kernels
constexpr int kMfmaThreads = 256;      // contraction kernel: 4 waves along the outputs
constexpr int IT = 8;                  // input rows per step (80 k-slots = 5 MFMA k-steps)
constexpr int LDK = 88;                // LDS row stride in halves (176 B = 11 x 16 B)
constexpr int kBufferFlags = 0x00020000;   // buffer resource word 3: raw 32-bit data format, no swizzle

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// ---- kan_prep_coef ------------------------------------------------------------------
// Chat as uint4 records: rec[((step*5 + ks) * 2 + h) * n_out + j], step = i / 8, so that
// both the writer and the MFMA B-operand lanes touch 16-byte items contiguous in j.
// A workgroup covers 64 output columns x 32 input rows: each of its 4 waves takes one
// step of 8 rows (lanes along the columns), so all loads of an edge's chain
// (metadata, then codeword) are in flight at once across many small waves.
template <typename IdxT, typename GbT, typename CbT>
__global__ __launch_bounds__(kThreads) void kan_prep_coef_kernel(const PrepCoefArgs a) {
  __shared__ float sb[4][64];
  const int head = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane;
  const LayerPtrs hp = a.h[head];
  const IdxT* idx = (const IdxT*)hp.idx;
  const GbT* gain = (const GbT*)hp.gain;
  const GbT* bias = (const GbT*)hp.bias;
  const Q8Params qp = {hp.gain_log2_lo, hp.gain_log2_step, hp.bias_scale};
  const CbT* cb = (const CbT*)hp.cb;
  uint4* cf = a.cf + (long long)head * a.cf_head_stride;
  float* bp = a.bias_partial + (long long)head * a.bp_head_stride;
  const int n_in = a.n_in, n_out = a.n_out;
  const int ib = blockIdx.y * kMfmaPrepRows + wave * IT;
  float bs = 0.f;
  if (j < n_out && ib < n_in) {
    const long long step = ib / IT;
    uint32_t id[IT];
    float g[IT];
#pragma unroll
    for (int r = 0; r < IT; ++r) {
      const int i = ib + r;
      const bool ok = i < n_in;
      const long long e = (long long)min(i, n_in - 1) * n_out + j;
      uint32_t idv[1];
      float gv[1], bv[1];
      load_idx<IdxT, 1>(idx + e, idv);
      load_gain<GbT, 1>(gain + e, qp, gv);
      load_bias<GbT, 1>(bias + e, qp, bv);
      id[r] = idv[0];
      g[r] = ok ? gv[0] : 0.f;          // rows past the end of a ragged last step are zero
      bs += ok ? bv[0] : 0.f;
    }
    RawRow<CbT> raw[IT];
#pragma unroll
    for (int r = 0; r < IT; ++r) load_row<CbT>(cb, id[r], raw[r]);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t tail[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        uint32_t w[5];
        dequant_row<CbT>(raw[4 * h + s], g[4 * h + s], w);
        cf[((step * 5 + s) * 2 + h) * n_out + j] = make_uint4(w[0], w[1], w[2], w[3]);
        tail[s] = w[4];
      }
      cf[((step * 5 + 4) * 2 + h) * n_out + j] = make_uint4(tail[0], tail[1], tail[2], tail[3]);
    }
  }
  sb[wave][lane] = bs;
  __syncthreads();
  if (wave == 0 && j < n_out)
    bp[(long long)blockIdx.y * n_out + j] = (sb[0][lane] + sb[1][lane]) + (sb[2][lane] + sb[3][lane]);
}

// ---- kan_prep_basis -----------------------------------------------------------------
// W[i][b] = { half2(w0, w1), half2(w2, w3) } with span bit 0, 1, 2 in the sign bits of
// w0, w1, w2 (the weights are never negative).
// The input is x itself, or (x_parts > 1) the previous layer's partial sums, added here in
// the order of the slices and squashed, so that no separate reduction pass runs in between.
__global__ __launch_bounds__(256) void kan_prep_basis_kernel(const float* __restrict__ x, long long x_head_stride,
                                                             int x_parts, long long x_part_stride, int x_tanh,
                                                             uint2* __restrict__ W, long long w_head_stride,
                                                             int n_in, int B, int rule) {
  __shared__ uint2 tile[32][33];
  const int head = blockIdx.z;
  const float* xh = x + (long long)head * x_head_stride;
  uint2* wh = W + (long long)head * w_head_stride;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
  const int ib = blockIdx.x * 32, bb = blockIdx.y * 32;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int b = bb + ty + 8 * r, i = ib + tx;
    uint2 v = make_uint2(0u, 0u);
    if (b < B && i < n_in) {
      const float* xp = xh + (long long)b * n_in + i;
      float xv = xp[0];
      for (int p0 = 1; p0 < x_parts; p0 += 8) {       // eight slices in flight, added in order
        float t[8];
#pragma unroll
        for (int pp = 0; pp < 8; ++pp) t[pp] = xp[(long long)min(p0 + pp, x_parts - 1) * x_part_stride];
#pragma unroll
        for (int pp = 0; pp < 8; ++pp) xv += p0 + pp < x_parts ? t[pp] : 0.f;
      }
      if (x_tanh) xv = tanhf(xv);
      const BasisW bw = basis_fast(xv, rule);
      const uint32_t l = (uint32_t)bw.span;
      const float w0 = bw.w0, w1 = bw.w1, w2 = bw.w2, w3 = bw.w3;
      v.x = pack_h2(w0, w1) | ((l & 1u) << 15) | ((l & 2u) << 30);
      v.y = pack_h2(w2, w3) | ((l & 4u) << 13);
    }
    tile[ty + 8 * r][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int i = ib + ty + 8 * r, b = bb + tx;
    if (i < n_in && b < B) wh[(long long)i * B + b] = tile[tx][ty + 8 * r];
  }
}

// ---- kan_mfma ---------------------------------------------------------------------------
// MB = MFMA row blocks per wave: tile of 32*MB samples.  MB = 2 keeps two workgroups on a
// CU (a 128-sample tile, MB = 4, halves the fragment bytes per MFMA but leaves one wave per
// SIMD and measured no faster on configurations 3 and 5).
//
// NB = MFMA column blocks per wave: the four waves cover 128 * NB outputs.  NB = 1 is for
// layers whose grid of 256-output tiles would leave CUs idle: half the accumulators and
// fragment registers, three workgroups per CU.
template <int MB, int NB>
__global__ __launch_bounds__(kMfmaThreads, NB == 1 ? 3 : 2) void kan_mfma_kernel(const MfmaArgs a) {
  constexpr int BM = 32 * MB;
  constexpr int BN = 4 * 32 * NB;      // outputs per workgroup tile
  constexpr int NPAIR = MB;            // (sample, input) pairs per thread and step
  __shared__ __attribute__((aligned(16))) uint16_t sA[2][BM * LDK];   // Phi tiles [b][k], 2 x 22.5 KB
  // Byte-permute selectors: row l, word k builds half-word slots 2k, 2k+1 of an input whose
  // weights w0..w3 (bytes 0..7 of {w23:w01}) sit at slots l..l+3; selector byte 0x0c yields 0.
  __shared__ __attribute__((aligned(16))) uint32_t sSel[kSpans][8];
  fill_weight_selectors(sSel, threadIdx.x);
  __syncthreads();

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int wm = 0, wn = wave;
  const int head = blockIdx.z, chunk = blockIdx.y;
  const int jt = blockIdx.x % a.n_jt, bt = blockIdx.x / a.n_jt;
  const int b0 = bt * BM, j0 = jt * BN;
  const int n_in = a.n_in, n_out = a.n_out, B = a.B;
  const int i_begin = chunk * a.rows_per_chunk;
  const int i_end = min(n_in, i_begin + a.rows_per_chunk);
  const int n_steps = (i_end - i_begin + IT - 1) / IT;
  const int step0 = i_begin / IT;
  const int last_step = (n_in + IT - 1) / IT - 1;

  const uint4* cf = a.cf + (long long)head * a.cf_head_stride;
  const uint2* W = a.W + (long long)head * a.w_head_stride;

  // Phi generation: this thread owns sample row pb and inputs NPAIR*ph .. NPAIR*ph+NPAIR-1 of every step.
  const int pb = tid & (BM - 1), ph = tid / BM;
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
  static_assert(BM % 64 == 0, "a wave generates the Phi rows of one input group");
  const int ph_u = __builtin_amdgcn_readfirstlane(ph);
  const uint32_t u_off = (uint32_t)min(b0 + pb, B - 1) * (uint32_t)sizeof(uint2);
  const char* w_bytes = (const char*)W;
  const uint32_t w_row_bytes = (uint32_t)B * (uint32_t)sizeof(uint2);
  auto load_u = [&](int k, uint2 (&uv)[NPAIR]) {       // step index relative to the chunk
    const int i = i_begin + k * IT + NPAIR * ph_u;
#pragma unroll
    for (int q = 0; q < NPAIR; ++q) {
      const char* row = w_bytes + (size_t)min(i + q, n_in - 1) * w_row_bytes;
      const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)row, 0, (int)w_row_bytes, kBufferFlags);
      const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)u_off, 0, 0);
      uv[q] = make_uint2(v.x, v.y);
    }
  };

  auto gen_phi = [&](const uint2 (&uv)[NPAIR], uint16_t* tile) {
    uint16_t* rowp = tile + pb * LDK;
#pragma unroll
    for (int q = 0; q < NPAIR; ++q) {
      const int ii = NPAIR * ph + q, h = ii >> 2, s = ii & 3;     // input ii of the step: k-step s, lane half h
      uint32_t l, w01, w23;
      unpack_basis(uv[q], l, w01, w23);
      const uint4 sl = *(const uint4*)&sSel[l][0];
      const uint32_t sh = sSel[l][4];
      uint4 lo;
      lo.x = __builtin_amdgcn_perm(w23, w01, sl.x);
      lo.y = __builtin_amdgcn_perm(w23, w01, sl.y);
      lo.z = __builtin_amdgcn_perm(w23, w01, sl.z);
      lo.w = __builtin_amdgcn_perm(w23, w01, sl.w);
      const uint32_t hi = __builtin_amdgcn_perm(w23, w01, sh);
      *(uint4*)(rowp + 16 * s + 8 * h) = lo;                    // coefficients 0..7
      *(uint32_t*)(rowp + 64 + 8 * h + 2 * s) = hi;             // coefficients 8, 9: k-step 4
    }
  };

  uint32_t b_off[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) b_off[nb] = (uint32_t)(lh * n_out + jc[nb]) * (uint32_t)sizeof(uint4);
  const char* cf_bytes = (const char*)cf;
  const uint32_t ks_bytes = 2u * (uint32_t)n_out * (uint32_t)sizeof(uint4);
  auto load_b = [&](int k, uint4 (&bf)[NB][5]) {
    const int step = min(step0 + k, last_step);           // past the end: valid memory, never used
    const char* sb = cf_bytes + (size_t)step * (5 * ks_bytes);
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)sb, 0, (int)(5 * ks_bytes), kBufferFlags);
#pragma unroll
    for (int ks = 0; ks < 5; ++ks)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)b_off[nb], (int)(ks * ks_bytes), 0);
        bf[nb][ks] = make_uint4(v.x, v.y, v.z, v.w);
      }
  };

  auto mfma_step = [&](const uint16_t* tile, const uint4 (&bf)[NB][5]) {
#pragma unroll
    for (int ks = 0; ks < 5; ++ks) {
      h16x8 fa[MB];
#pragma unroll
      for (int m = 0; m < MB; ++m)
        fa[m] = __builtin_bit_cast(h16x8, *(const uint4*)(tile + (wm * 64 + m * 32 + ln) * LDK + ks * 16 + lh * 8));
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        const h16x8 fb = __builtin_bit_cast(h16x8, bf[n][ks]);
#pragma unroll
        for (int m = 0; m < MB; ++m)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[m], fb, acc[m][n], 0, 0, 0);
      }
    }
  };

  // ---- pipeline: three-slot rings indexed by compile-time slots (loop unrolled by 6) --------
  // Top of step k: Phi tile k and fragments k are ready; fragments and basis words of
  // steps k+1, k+2 are in flight.  Step k issues those of step k+3 into the slot step k
  // frees, so every load has two full steps to arrive; the second workgroup on the CU
  // covers the rest.
  // The bias sums of the tile's columns are fetched ahead of everything else (thread t owns
  // column j0 + t) and parked in LDS until the epilogue, so their latency is never exposed.
  static_assert(BN <= kMfmaThreads, "one bias column per thread (the others repeat the last column)");
  __shared__ float sBias[kMfmaThreads];
  const float* bp = a.bias_partial + (long long)head * a.bp_head_stride + min(j0 + tid, n_out - 1);
  const int rb0 = i_begin / kMfmaPrepRows, rb1 = (i_end + kMfmaPrepRows - 1) / kMfmaPrepRows;
  float bias_v[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) bias_v[u] = bp[(long long)min(rb0 + u, rb1 - 1) * n_out];

  uint4 bfr[3][NB][5];
  uint2 uv[3][NPAIR];
  load_u(0, uv[0]);
  load_b(0, bfr[0]);
  load_u(1, uv[1]);
  load_b(1, bfr[1]);
  load_u(2, uv[2]);
  load_b(2, bfr[2]);
  {
    float bs = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) bs += rb0 + u < rb1 ? bias_v[u] : 0.f;
    for (int rb = rb0 + 8; rb < rb1; ++rb) bs += bp[(long long)rb * n_out];
    sBias[tid] = bs;      // read after the barriers of the main loop
  }
  gen_phi(uv[0], sA[0]);

  auto step = [&](auto T, int k) {
    constexpr int t = decltype(T)::value;          // k mod 6
    __syncthreads();     // tile k is complete; every wave is done reading tile k-1
    mfma_step(sA[t & 1], bfr[t % 3]);
    gen_phi(uv[(t + 1) % 3], sA[(t + 1) & 1]);     // step k+1 basis tile
    load_b(k + 3, bfr[t % 3]);                     // fragments of step k have been consumed
    load_u(k + 3, uv[t % 3]);                      // basis words of step k were consumed a step ago
  };
  // Whole groups of six steps run without a branch between them: a branch around a step makes
  // the compiler lose count of the loads in flight and wait for all of them.
  int k = 0;
  for (; k + 6 <= n_steps; k += 6) {
    step(std::integral_constant<int, 0>{}, k);
    step(std::integral_constant<int, 1>{}, k + 1);
    step(std::integral_constant<int, 2>{}, k + 2);
    step(std::integral_constant<int, 3>{}, k + 3);
    step(std::integral_constant<int, 4>{}, k + 4);
    step(std::integral_constant<int, 5>{}, k + 5);
  }
  if (k < n_steps) step(std::integral_constant<int, 0>{}, k);
  if (k + 1 < n_steps) step(std::integral_constant<int, 1>{}, k + 1);
  if (k + 2 < n_steps) step(std::integral_constant<int, 2>{}, k + 2);
  if (k + 3 < n_steps) step(std::integral_constant<int, 3>{}, k + 3);
  if (k + 4 < n_steps) step(std::integral_constant<int, 4>{}, k + 4);

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
          const int b = b0 + wm * 64 + m * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (b < B) {
            float v = fmaf(scale, acc[m][n][r], bs);
            if (a.apply_tanh) v = tanhf(v);
            dst[(long long)b * n_out + jc[n]] = v;
          }
        }
    }
  }
}

template <typename IdxT>
hipError_t prep_types(const GatherCfg& c, const PrepCoefArgs& a, dim3 grid, hipStream_t s) {
  if (c.code == kCbI8) {
    if (c.gb_kind == kGbQ8)
      hipLaunchKernelGGL((kan_prep_coef_kernel<IdxT, q8_t, int8_t>), grid, dim3(kThreads), 0, s, a);
    else if (c.gb_kind == kGbF16)
      hipLaunchKernelGGL((kan_prep_coef_kernel<IdxT, __half, int8_t>), grid, dim3(kThreads), 0, s, a);
    else
      hipLaunchKernelGGL((kan_prep_coef_kernel<IdxT, float, int8_t>), grid, dim3(kThreads), 0, s, a);
  } else {
    if (c.gb_kind == kGbQ8) return hipErrorInvalidValue;    // byte-coded gain/bias go with Int8 codebooks
    if (c.code == kCbF16) {
      if (c.gb_kind == kGbF16)
        hipLaunchKernelGGL((kan_prep_coef_kernel<IdxT, __half, __half>), grid, dim3(kThreads), 0, s, a);
      else
        hipLaunchKernelGGL((kan_prep_coef_kernel<IdxT, float, __half>), grid, dim3(kThreads), 0, s, a);
    } else if (c.gb_kind == kGbF16)
      hipLaunchKernelGGL((kan_prep_coef_kernel<IdxT, __half, float>), grid, dim3(kThreads), 0, s, a);
    else
      hipLaunchKernelGGL((kan_prep_coef_kernel<IdxT, float, float>), grid, dim3(kThreads), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prep_coef(const GatherCfg& c, const PrepCoefArgs& a, int heads, hipStream_t s) {
  if (c.code == kDense) return hipErrorInvalidValue;
  dim3 grid((a.n_out + 63) / 64, (a.n_in + kMfmaPrepRows - 1) / kMfmaPrepRows, heads);
  return c.idx_u32 ? prep_types<uint32_t>(c, a, grid, s) : prep_types<uint16_t>(c, a, grid, s);
}

hipError_t launch_prep_basis(const float* x, long long x_head_stride, int x_parts, long long x_part_stride,
                             int x_tanh, uint2* W, long long w_head_stride, int n_in, int B, int heads, int rule,
                             hipStream_t s) {
  if (x_parts < 1) return hipErrorInvalidValue;
  dim3 grid((n_in + 31) / 32, (B + 31) / 32, heads);
  hipLaunchKernelGGL(kan_prep_basis_kernel, grid, dim3(256), 0, s, x, x_head_stride, x_parts, x_part_stride, x_tanh,
                     W, w_head_stride, n_in, B, rule);
  return hipGetLastError();
}

hipError_t launch_mfma(const MfmaArgs& a, int tile_m, int tile_n, dim3 grid, hipStream_t s) {
  if (tile_m != 64 || (tile_n != 128 && tile_n != 256)) return hipErrorInvalidValue;
  if ((long long)a.n_jt * tile_n < a.n_out) return hipErrorInvalidValue;
  // one step of coefficient records and one row of basis words must fit a buffer resource
  if ((long long)a.n_out * 10 * (long long)sizeof(uint4) > 0x7fffffffLL ||
      (long long)a.B * (long long)sizeof(uint2) > 0x7fffffffLL)
    return hipErrorInvalidValue;
  if (tile_n == 128) hipLaunchKernelGGL((kan_mfma_kernel<2, 1>), grid, dim3(kMfmaThreads), 0, s, a);
  else hipLaunchKernelGGL((kan_mfma_kernel<2, 2>), grid, dim3(kMfmaThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace kan
