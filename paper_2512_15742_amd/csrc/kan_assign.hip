// Compression-side assignment step (paper section 4.2, steps 1 and 3 of the post-training
// procedure): every edge's grid of G = 10 coefficients is normalised - its mean becomes the
// bias, the norm of the centred grid the gain - and assigned to the nearest of the K
// codebook shapes.  (Learning the shapes, step 2, is not part of this library.)
//
// Nearest centroid = largest score s(e, k) = n_e . C_k - |C_k|^2 / 2, a dense
// [K x 10] x [10 x E] contraction: it runs on the matrix cores.  To keep the decision at
// fp32 quality with fp16 operands, both operands are split into a high and a low fp16 part
// and the contraction runs over 32 slots (two v_mfma_f32_32x32x16_f16 per 32 x 32 tile):
//     centroid side  [ hi(C) (10) | lo(C) (10) | hi(C) (10) | hi(-|C|^2/2) | lo(-|C|^2/2) ]
//     edge side      [ hi(n) (10) | hi(n) (10) | lo(n) (10) |      1       |      1       ]
// (the dropped lo x lo term is ~1e-7 of the score).  Centroids are the MFMA rows and edges
// the columns, so a lane owns one edge and 16 of the 32 centroids of a tile: the running
// maximum over centroids never crosses lanes until the very end.
//
// The arg-max costs vector instructions per score, which is what would bound the kernel, so the
// common case is kept to half an instruction per score: the maximum of a lane's 16 scores of a
// tile is 8 three-input maxima, and only when it beats the lane's running best - the t-th tile
// does so with probability ~1/t - is the row looked up.  Exactly equal scores (duplicate shapes)
// resolve to the lower index within a half-wave's rows; which of two half-waves' equal scores
// wins is decided by index at the end.

#include "kan_device.hpp"
#include "kan_internal.hpp"
#include "kan_mfma_common.hpp"

namespace kan {
namespace {

constexpr int kAssignThreads = 256;
constexpr int kEdgeTilesPerWave = 4;                                   // 4 x 32 edges per wave
constexpr int kEdgesPerWg = (kAssignThreads / kWave) * kEdgeTilesPerWave * 32;   // 512
constexpr int kSlots = 32;                                             // contraction length

__device__ __forceinline__ void split_h(float v, _Float16& hi, _Float16& lo) {
  hi = (_Float16)v;
  lo = (_Float16)(v - (float)hi);
}

// Centroid-side operands in MFMA A-fragment order: record [(tile * 2 + kstep) * 64 + lane]
// holds slots kstep*16 + (lane/32)*8 .. +8 of centroid tile*32 + (lane & 31).  Rows past K get
// a hugely negative norm term so that they never win.
__global__ __launch_bounds__(256) void kan_assign_prep_kernel(const float* __restrict__ cb, int K, int n_tiles,
                                                              uint4* __restrict__ out) {
  const long long rec = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (rec >= (long long)n_tiles * 2 * 64) return;
  const int lane = (int)(rec & 63), ks = (int)((rec >> 6) & 1);
  const int c = (int)(rec >> 7) * 32 + (lane & 31);
  const int s0 = ks * 16 + (lane >> 5) * 8;
  _Float16 v[8];
  float nrm = 0.f;
  float row[kG];
#pragma unroll
  for (int m = 0; m < kG; ++m) {
    row[m] = c < K ? cb[(long long)c * kG + m] : 0.f;
    nrm = fmaf(row[m], row[m], nrm);
  }
  const float half_norm = c < K ? -0.5f * nrm : -30000.0f;
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int s = s0 + t;
    _Float16 hi, lo;
    if (s < 30) {
      split_h(row[s % kG], hi, lo);
      v[t] = (s >= 10 && s < 20) ? lo : hi;
    } else {
      split_h(half_norm, hi, lo);
      v[t] = s == 30 ? hi : lo;
    }
  }
  h16x8 pk = {v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7]};
  out[rec] = __builtin_bit_cast(uint4, pk);
}

struct AssignArgs {
  const float* coef;        // [E][10]
  const uint4* cent;        // prepared centroid operands
  long long E;
  int n_tiles;              // ceil(K / 32)
  void* idx;
  float* gain;
  float* bias;
};

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <typename IdxT>
__global__ __launch_bounds__(kAssignThreads, 4) void kan_assign_kernel(const AssignArgs a) {
  // edge-side operands of the workgroup's 512 edges: [edge][32 slots] fp16
  __shared__ __attribute__((aligned(16))) _Float16 sB[kEdgesPerWg * kSlots];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long e_wg = (long long)blockIdx.x * kEdgesPerWg;

  // ---- step 1: bias = mean, gain = norm of the centred grid, n = centred / gain ------------
  for (int q = tid; q < kEdgesPerWg; q += kAssignThreads) {
    const long long e = e_wg + q;
    const long long ec = e < a.E ? e : a.E - 1;
    float c[kG];
#pragma unroll
    for (int m = 0; m < kG / 2; ++m) {
      const float2 v = ((const float2*)(a.coef + ec * kG))[m];
      c[2 * m] = v.x;
      c[2 * m + 1] = v.y;
    }
    float mean = 0.f;
#pragma unroll
    for (int m = 0; m < kG; ++m) mean += c[m];
    mean /= (float)kG;       // a true division: the mean of ten equal values is that value
    float ss = 0.f;
#pragma unroll
    for (int m = 0; m < kG; ++m) {
      c[m] -= mean;
      ss = fmaf(c[m], c[m], ss);
    }
    const float g = sqrtf(ss);
    const float inv = g > 0.f ? 1.0f / g : 0.f;
    if (e < a.E) {
      a.gain[e] = g;
      a.bias[e] = mean;
    }
    _Float16* p = sB + q * kSlots;
#pragma unroll
    for (int m = 0; m < kG; ++m) {
      _Float16 hi, lo;
      split_h(c[m] * inv, hi, lo);
      p[m] = hi;
      p[10 + m] = hi;
      p[20 + m] = lo;
    }
    p[30] = (_Float16)1.0f;
    p[31] = (_Float16)1.0f;
  }
  __syncthreads();

  // ---- this wave's edge fragments (MFMA B operand: column = lane & 31, slots (lane/32)*8..+8) --
  h16x8 fb[kEdgeTilesPerWave][2];
#pragma unroll
  for (int nb = 0; nb < kEdgeTilesPerWave; ++nb)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int q = (wave * kEdgeTilesPerWave + nb) * 32 + (lane & 31);
      fb[nb][ks] = *(const h16x8*)(sB + q * kSlots + ks * 16 + (lane >> 5) * 8);
    }

  float best[kEdgeTilesPerWave];
  int best_tile[kEdgeTilesPerWave], best_row[kEdgeTilesPerWave];
#pragma unroll
  for (int nb = 0; nb < kEdgeTilesPerWave; ++nb) {
    best[nb] = -3.0e38f;
    best_tile[nb] = 0;
    best_row[nb] = 0;
  }

  // ---- step 3: stream the centroid tiles (two tiles in flight) -----------------------------------
  const uint4* cp = a.cent + lane;
  auto load_tile = [&](int t, uint4 (&fa)[2]) {
    const int tc = t < a.n_tiles ? t : a.n_tiles - 1;        // past the end: a harmless re-read
    fa[0] = cp[(long long)(tc * 2) * 64];
    fa[1] = cp[(long long)(tc * 2 + 1) * 64];
  };
  f32x16 zero;
#pragma unroll
  for (int r = 0; r < 16; ++r) zero[r] = 0.f;
  auto score_tile = [&](int t, const uint4 (&fa)[2]) {
    const h16x8 a0 = __builtin_bit_cast(h16x8, fa[0]), a1 = __builtin_bit_cast(h16x8, fa[1]);
#pragma unroll
    for (int nb = 0; nb < kEdgeTilesPerWave; ++nb) {
      f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, fb[nb][0], zero, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, fb[nb][1], acc, 0, 0, 0);
      // maximum of the lane's 16 scores: 8 three-input maxima
      const float m0 = max3(acc[0], acc[1], acc[2]), m1 = max3(acc[3], acc[4], acc[5]);
      const float m2 = max3(acc[6], acc[7], acc[8]), m3 = max3(acc[9], acc[10], acc[11]);
      const float m4 = max3(acc[12], acc[13], acc[14]);
      const float m = max3(max3(m0, m1, m2), m3, max3(m4, acc[15], -3.0e38f));
      // A new best is rare (the t-th tile improves a lane's running maximum with probability
      // ~1/t), so the row is looked for only then.  Strictly greater: the earliest tile, and in
      // it the lowest register, keeps a tie.
      if (m > best[nb]) {
        int r_best = 15;
#pragma unroll
        for (int r = 14; r >= 0; --r) r_best = acc[r] == m ? r : r_best;
        best[nb] = m;
        best_tile[nb] = t;
        best_row[nb] = r_best;
      }
    }
  };
  uint4 fa0[2], fa1[2];
  load_tile(0, fa0);
  load_tile(1, fa1);
  for (int t = 0; t < a.n_tiles; t += 2) {
    score_tile(t, fa0);
    load_tile(t + 2, fa0);
    if (t + 1 < a.n_tiles) score_tile(t + 1, fa1);
    load_tile(t + 3, fa1);
  }

  // ---- the two half-waves hold different rows of the same edges: keep the better one ------------
#pragma unroll
  for (int nb = 0; nb < kEdgeTilesPerWave; ++nb) {
    const int r = best_row[nb];
    // D layout of the 32x32 MFMA: register r of a lane is row 8*(r/4) + 4*(lane/32) + r%4
    int id = best_tile[nb] * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    float sc = best[nb];
    const float sc_o = __shfl_xor(sc, 32, kWave);
    const int id_o = __shfl_xor(id, 32, kWave);
    if (sc_o > sc || (sc_o == sc && id_o < id)) id = id_o;
    const long long e = e_wg + (wave * kEdgeTilesPerWave + nb) * 32 + (lane & 31);
    if (lane < 32 && e < a.E) ((IdxT*)a.idx)[e] = (IdxT)id;
  }
}

// ---- reconstruction quality ---------------------------------------------------------------------
// Sums for R^2 between the dense grids and their reconstruction gain * C[idx] + bias:
// per workgroup {sum of squared residuals, sum of c, sum of c^2} in fp64, then one
// fixed-order pass over the workgroups.
template <typename IdxT>
__global__ __launch_bounds__(256) void kan_recon_partial_kernel(const float* __restrict__ coef,
                                                                const float* __restrict__ cb,
                                                                const IdxT* __restrict__ idx,
                                                                const float* __restrict__ gain,
                                                                const float* __restrict__ bias, long long E,
                                                                double* __restrict__ part) {
  __shared__ double red[3][256];
  double sr = 0.0, s1 = 0.0, s2 = 0.0;
  for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < E; e += (long long)gridDim.x * blockDim.x) {
    const float* c = coef + e * kG;
    const float* r = cb + (long long)idx[e] * kG;
    const double g = gain[e], b = bias[e];
#pragma unroll
    for (int m = 0; m < kG; ++m) {
      const double v = c[m], d = v - (g * (double)r[m] + b);
      sr += d * d;
      s1 += v;
      s2 += v * v;
    }
  }
  red[0][threadIdx.x] = sr;
  red[1][threadIdx.x] = s1;
  red[2][threadIdx.x] = s2;
  __syncthreads();
  if (threadIdx.x < 3) {
    double t = 0.0;
    for (int q = 0; q < 256; ++q) t += red[threadIdx.x][q];
    part[(long long)blockIdx.x * 3 + threadIdx.x] = t;
  }
}

// sums[0..2] = the three totals; sums[3] = R^2 = 1 - SS_res / SS_tot with SS_tot taken about the
// overall mean of the n_coef coefficients (section 4.2).
__global__ void kan_recon_final_kernel(const double* __restrict__ part, int n_blocks, double n_coef,
                                       double* __restrict__ sums) {
  __shared__ double tot[3];
  if (threadIdx.x < 3) {
    double t = 0.0;
    for (int q = 0; q < n_blocks; ++q) t += part[(long long)q * 3 + threadIdx.x];
    sums[threadIdx.x] = t;
    tot[threadIdx.x] = t;
  }
  __syncthreads();
  if (threadIdx.x == 0) sums[3] = 1.0 - tot[0] / (tot[2] - tot[1] * tot[1] / n_coef);
}

}  // namespace

size_t assign_centroid_bytes(int K) { return (size_t)((K + 31) / 32) * 2 * 64 * sizeof(uint4); }
int recon_blocks(long long E) {
  const long long b = (E + 255) / 256;
  return (int)(b < 1024 ? b : 1024);
}

hipError_t launch_assign(const float* coef, long long E, const float* cb, int K, int idx_u32, void* idx, float* gain,
                         float* bias, void* ws, hipStream_t s) {
  const int n_tiles = (K + 31) / 32;
  const long long recs = (long long)n_tiles * 2 * 64;
  hipLaunchKernelGGL(kan_assign_prep_kernel, dim3((unsigned)((recs + 255) / 256)), dim3(256), 0, s, cb, K, n_tiles,
                     (uint4*)ws);
  AssignArgs a;
  a.coef = coef;
  a.cent = (const uint4*)ws;
  a.E = E;
  a.n_tiles = n_tiles;
  a.idx = idx;
  a.gain = gain;
  a.bias = bias;
  dim3 grid((unsigned)((E + kEdgesPerWg - 1) / kEdgesPerWg));
  if (idx_u32) hipLaunchKernelGGL(kan_assign_kernel<uint32_t>, grid, dim3(kAssignThreads), 0, s, a);
  else hipLaunchKernelGGL(kan_assign_kernel<uint16_t>, grid, dim3(kAssignThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_recon_sums(const float* coef, long long E, const float* cb, int idx_u32, const void* idx,
                             const float* gain, const float* bias, double* part, double* sums, hipStream_t s) {
  const int nb = recon_blocks(E);
  if (idx_u32)
    hipLaunchKernelGGL(kan_recon_partial_kernel<uint32_t>, dim3(nb), dim3(256), 0, s, coef, cb, (const uint32_t*)idx,
                       gain, bias, E, part);
  else
    hipLaunchKernelGGL(kan_recon_partial_kernel<uint16_t>, dim3(nb), dim3(256), 0, s, coef, cb, (const uint16_t*)idx,
                       gain, bias, E, part);
  hipLaunchKernelGGL(kan_recon_final_kernel, dim3(1), dim3(64), 0, s, (const double*)part, nb, (double)E * kG, sums);
  return hipGetLastError();
}

}  // namespace kan
