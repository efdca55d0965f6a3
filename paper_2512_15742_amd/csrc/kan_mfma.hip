// Matrix-core path of the VQ-KAN forward pass for gfx950 (large batch).
//
// The layer sum y[b][j] = sum_i sum_m B_m(x_bi) * c_ij[m] (paper section 3 with
// the reconstructed coefficients of section 4.2) is a contraction over
// k = (i, m), m = 0..9:
//     Y[b][j] = sum_k Phi[b][k] * Chat[k][j] + sum_i bias_ij
//     Phi[b][i*10+m]  = B_m(x_bi)                (4 nonzeros per 10, App. A.1 family)
//     Chat[i*10+m][j] = gain_ij * scale * C[idx_ij][m]
// Neither operand exists in memory.  Per step of 8 input rows a workgroup
//   - evaluates span + weights for its 128 samples x 8 inputs (span exactly, in
//     fp64; weights in fp32) and scatters them as bf16 into a zeroed LDS tile,
//   - reads idx/gain/bias of its 8 x 128 edges (coalesced, read once per batch
//     tile), gathers the codewords, dequantises, scales by gain and writes the
//     bf16 coefficient tile to LDS (bias is kept out of the bf16 product: the
//     bases sum to one, so it is summed in fp32 and added at the end),
//   - contracts the two tiles with v_mfma_f32_32x32x16_bf16 (fp32 accumulate).
// Workgroups tile (batch, outputs) as 128 x 128 and split i into chunks; chunk
// partial sums go through the same fixed-order reduction as the gather path.

#include "kan_device.hpp"
#include "kan_internal.hpp"

namespace kan {
namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BM = 128, BN = 128;      // workgroup tile: samples x outputs
constexpr int IT = 8;                  // input rows per step
constexpr int KT = IT * kG;            // 80 = 5 MFMA k-steps of 16
constexpr int LDK = 88;                // LDS row stride in bf16 (176 B = 11 x 16 B)

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, v);
}

template <typename IdxT, typename GbT, typename CbT>
__global__ __launch_bounds__(kThreads) void kan_mfma_kernel(const GatherArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LDK];   // Phi tile   [b][k]
  __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LDK];   // Chat tile  [j][k]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int head = blockIdx.z, chunk = blockIdx.y;
  const int jt = blockIdx.x % a.n_jt, bt = blockIdx.x / a.n_jt;
  const int b0 = bt * BM, j0 = jt * BN;
  const int n_in = a.n_in, n_out = a.n_out;
  const int i_begin = chunk * a.rows_per_chunk;
  const int i_end = min(n_in, i_begin + a.rows_per_chunk);

  const LayerPtrs hp = a.h[head];
  const float* xh = a.x + (long long)head * a.x_head_stride;
  const IdxT* idx = (const IdxT*)hp.idx;
  const GbT* gain = (const GbT*)hp.gain;
  const GbT* bias = (const GbT*)hp.bias;
  const CbT* cb = (const CbT*)hp.cb;
  const float scale = sizeof(CbT) == 1 ? hp.scale : 1.0f;

  // basis generation: this thread owns sample pb and inputs pi..pi+3 of every step
  const int pb = tid >> 1, pi = (tid & 1) * 4;
  const bool b_ok = (b0 + pb) < a.B;
  // coefficient generation: input row ci of the step, outputs cj + 32*p, p = 0..3
  const int ci = tid >> 5, cj = tid & 31;

  const int wm = wave >> 1, wn = wave & 1;     // 2 x 2 waves, 64 x 64 each
  f32x16 acc[2][2];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.f;
  float bsum[4] = {0.f, 0.f, 0.f, 0.f};

  for (int s0 = i_begin; s0 < i_end; s0 += IT) {
    __syncthreads();   // previous step's MFMA reads are done
    // ---- Phi tile --------------------------------------------------------------------
    {
      uint32_t* rowp = (uint32_t*)(sA + pb * LDK + pi * kG);     // 80 B, 16-byte aligned
      const uint4 z = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int q = 0; q < 5; ++q) ((uint4*)rowp)[q] = z;
      if (b_ok) {
        const float* xp = xh + (long long)(b0 + pb) * n_in + s0 + pi;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (s0 + pi + q < i_end) {
            const float xc = fminf(fmaxf(xp[q], -1.0f), 1.0f);
            // exact span: t = (7x + 7) / 2 is exact in fp64; span = min(floor(t), 6)
            const double t = fma((double)xc, 3.5, 3.5);
            const int l = min((int)t, kSpans - 1);
            const float u = (float)(t - (double)l);
            const float u2 = u * u, u3 = u2 * u, om = 1.0f - u;
            const float w0 = om * om * om * (1.0f / 6.0f);
            const float w3 = u3 * (1.0f / 6.0f);
            const float w1 = fmaf(0.5f, u3, fmaf(-1.0f, u2, 2.0f / 3.0f));
            const float w2 = fmaf(-0.5f, u3, fmaf(0.5f, u2, fmaf(0.5f, u, 1.0f / 6.0f)));
            const uint32_t w01 = pack_bf16(w0, w1), w23 = pack_bf16(w2, w3);
            const bool odd = l & 1;
            const uint32_t t0 = odd ? (w01 << 16) : w01;
            const uint32_t t1 = odd ? ((w01 >> 16) | (w23 << 16)) : w23;
            const uint32_t t2 = odd ? (w23 >> 16) : 0u;
            uint32_t* d = rowp + q * 5 + (l >> 1);    // words (l>>1) .. (l>>1)+2 of this input's 5
            d[0] = t0;
            d[1] = t1;
            if (odd) d[2] = t2;                       // l odd => l <= 5, word index <= 4
          }
        }
      }
    }
    // ---- coefficient tile ---------------------------------------------------------------
    {
      const int i = s0 + ci;
      const bool i_ok = i < i_end;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int jl = cj + 32 * p;
        const int j = j0 + jl;
        uint32_t w[5] = {0u, 0u, 0u, 0u, 0u};
        if (i_ok && j < n_out) {
          const long long e = (long long)i * n_out + j;
          uint32_t id[1];
          float g[1], bv[1];
          load_idx<IdxT, 1>(idx + e, id);
          load_gb<GbT, 1>(gain + e, g);
          load_gb<GbT, 1>(bias + e, bv);
          float c[kG];
          fetch_row<CbT>(cb, id[0], g[0] * scale, c);
#pragma unroll
          for (int m = 0; m < 5; ++m) w[m] = pack_bf16(c[2 * m], c[2 * m + 1]);
          bsum[p] += bv[0];
        }
        uint32_t* d = (uint32_t*)(sB + jl * LDK + ci * kG);
#pragma unroll
        for (int m = 0; m < 5; ++m) d[m] = w[m];
      }
    }
    __syncthreads();
    // ---- contraction ------------------------------------------------------------------------
#pragma unroll
    for (int ks = 0; ks < KT / 16; ++ks) {
      const int ko = ks * 16 + (lane >> 5) * 8;
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int m = 0; m < 2; ++m)
        fa[m] = __builtin_bit_cast(bf16x8, *(const uint4*)(sA + (wm * 64 + m * 32 + (lane & 31)) * LDK + ko));
#pragma unroll
      for (int n = 0; n < 2; ++n)
        fb[n] = __builtin_bit_cast(bf16x8, *(const uint4*)(sB + (wn * 64 + n * 32 + (lane & 31)) * LDK + ko));
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[m], fb[n], acc[m][n], 0, 0, 0);
    }
  }

  // ---- bias: sum the 8 per-row partial sums of every output column ---------------------------
  __syncthreads();
  float* sBias = (float*)sA;                 // [IT][BN]
#pragma unroll
  for (int p = 0; p < 4; ++p) sBias[ci * BN + cj + 32 * p] = bsum[p];
  __syncthreads();

  // ---- epilogue: D layout of the 32x32 MFMA: lane holds column (lane & 31), rows
  //      8*(r/4) + 4*(lane/32) + r%4 for r = 0..15 -------------------------------------------
  float* dst = a.dst + (long long)head * a.dst_head_stride + (long long)chunk * a.dst_chunk_stride;
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    const int jl = wn * 64 + n * 32 + (lane & 31);
    const int j = j0 + jl;
    float bs = 0.f;
#pragma unroll
    for (int r = 0; r < IT; ++r) bs += sBias[r * BN + jl];
    if (j < n_out) {
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int b = b0 + wm * 64 + m * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (b < a.B) {
            float v = acc[m][n][r] + bs;
            if (a.apply_tanh) v = tanhf(v);
            dst[(long long)b * n_out + j] = v;
          }
        }
    }
  }
}

template <typename IdxT>
hipError_t launch_types(const GatherCfg& c, const GatherArgs& a, dim3 grid, hipStream_t s) {
  if (c.code == kCbI8) {
    if (c.gb_f16)
      hipLaunchKernelGGL((kan_mfma_kernel<IdxT, __half, int8_t>), grid, dim3(kThreads), 0, s, a);
    else
      hipLaunchKernelGGL((kan_mfma_kernel<IdxT, float, int8_t>), grid, dim3(kThreads), 0, s, a);
  } else {
    if (c.gb_f16)
      hipLaunchKernelGGL((kan_mfma_kernel<IdxT, __half, float>), grid, dim3(kThreads), 0, s, a);
    else
      hipLaunchKernelGGL((kan_mfma_kernel<IdxT, float, float>), grid, dim3(kThreads), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_mfma(const GatherCfg& c, const GatherArgs& a, dim3 grid, hipStream_t s) {
  if (c.code == kDense) return hipErrorInvalidValue;
  return c.idx_u32 ? launch_types<uint32_t>(c, a, grid, s) : launch_types<uint16_t>(c, a, grid, s);
}

}  // namespace kan
