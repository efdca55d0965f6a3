// Vector-ALU path of the KAN forward pass for gfx950 (fp32): VQ layers at batch 1 and the
// dense-coefficient baseline at any batch.
//
// Mapping.  Lanes own outputs j (JPL consecutive ones each), so the per-edge
// metadata idx/gain/bias[i][j..] of paper Eq. (1) is one contiguous, coalesced,
// read-once stream per i-row, and everything that depends on x_bi alone (the
// interval index and the four basis weights, App. A.1 / section 4.1) is the same
// for all lanes of a wave: it is computed once per (b, i) into LDS and broadcast.
// VQ layers, one sample (KAN_BT = 1): only the 4 coefficients under the nonzero
// bases are gathered (from L2), scaled by gain (and the Int8 scale) while they are
// unpacked; bias is summed once per edge because the bases sum to 1.
// Dense baseline (any batch tile): the 10 coefficients of an edge are read straight
// from coef[in][out][10]; for tiles of 4 or 16 samples the weights are stored as a
// 10-vector (zeros outside span..span+3) so that the edge evaluation is 10
// branch-free fmas with no register indexing by span.
// A workgroup is 4 waves: WJ of them side by side along j, 4/WJ interleaved
// along i, whose partial sums meet in LDS.  Workgroups split i into chunks; the
// chunk partial sums are written out and reduced in a fixed order by
// kan_reduce (deterministic: no atomics).
//
// This file is compiled once per batch tile (KAN_BT = 1, 4, 16).

#include "kan_device.hpp"
#include "kan_internal.hpp"

#ifndef KAN_BT
#error "compile with -DKAN_BT=<batch tile>"
#endif

namespace kan {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kSub = 32;   // i-rows whose basis data is staged in LDS at a time

// SL (window form only): the input is still in slices, the previous layer's partial sums.
template <typename IdxT, typename GbT, typename CbT, int CODE, int BT, int JPL, bool SL = false>
__global__ __launch_bounds__(kThreads) void kan_gather_kernel(const GatherArgs a, const int wj_count) {
  static_assert(!SL || (BT == 1 && CODE != kDense), "slices of the input: VQ layers, one sample per tile");
  // LDS: basis data for kSub rows x BT samples; later reused for the cross-wave sum.
  constexpr bool kWindow = (BT == 1 && CODE != kDense);
  constexpr int kWStride = kWindow ? 5 : 12;             // floats of basis data per (row, sample)
  constexpr int kBasisFloats = kSub * BT * kWStride;
  constexpr int kRedFloats = (kWaves - 1) * BT * kWave * JPL;
  constexpr int kLdsFloats = kBasisFloats > kRedFloats ? kBasisFloats : kRedFloats;
  __shared__ __attribute__((aligned(16))) float lds[kLdsFloats];
  float4* const sw = (float4*)lds;                       // window form: [kSub] weights
  int* const ss = (int*)(lds + kSub * BT * 4);           // window form: [kSub] spans

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid >> 6;
  const int wi_count = kWaves / wj_count;
  const int wj = wave % wj_count;
  const int wi = wave / wj_count;

  int head = blockIdx.z, chunk = blockIdx.y, tile = blockIdx.x;
  if constexpr (SL) {
    // Workgroups go to the eight XCDs in turn (linear id mod 8), each with an L2 of its own.  The output
    // tiles of a chunk read the same slices, and a chunk of 16 rows is half a 128-byte line per slice,
    // whose other half the next chunk reads: runs of consecutive (chunk, tile) items per XCD fetch every
    // line once.
    const unsigned T = gridDim.x, C = gridDim.y, W = T * C * gridDim.z;
    const unsigned L = blockIdx.x + T * (blockIdx.y + C * blockIdx.z);
    const unsigned xcd = L & 7u, m = L >> 3, q = W >> 3, r = W & 7u;
    const unsigned item = xcd * q + min(xcd, r) + m;          // XCD x owns q + (x < r) items
    head = (int)(item / (T * C));
    const unsigned rem = item % (T * C);
    chunk = (int)(rem / T);
    tile = (int)(rem % T);
  }
  const int jt = tile % a.n_jt;
  const int btile = tile / a.n_jt;

  const LayerPtrs hp = a.h[head];
  const int n_in = a.n_in, n_out = a.n_out;
  const int b0 = btile * BT;
  const int i_begin = chunk * a.rows_per_chunk;
  const int i_end = min(n_in, i_begin + a.rows_per_chunk);
  const int j0 = (jt * wj_count + wj) * (kWave * JPL) + lane * JPL;
  const bool j_ok = j0 < n_out;          // n_out % JPL == 0, so the whole group is in range

  const float* xh = a.x + (long long)head * a.x_head_stride;
  const IdxT* idx = (const IdxT*)hp.idx;
  const GbT* gain = (const GbT*)hp.gain;
  const GbT* bias = (const GbT*)hp.bias;
  const Q8Params qp = {hp.gain_log2_lo, hp.gain_log2_step, hp.bias_scale};
  const CbT* cb = (const CbT*)hp.cb;
  const float scale = (CODE == kCbI8) ? hp.scale : 1.0f;

  if constexpr (BT == 1 && CODE != kDense) {
    // Warm this XCD's L2 with the codebook before the random gathers start: the workgroups
    // that share an XCD (linear id mod 8) each stream one slice of it, coalesced.
    if (a.cb_bytes > 0) {
      const long long wg = blockIdx.x + (long long)gridDim.x * (blockIdx.y + (long long)gridDim.y * blockIdx.z);
      const long long per_xcd = ((long long)gridDim.x * gridDim.y * gridDim.z + 7) / 8;
      const long long slice = ((a.cb_bytes + per_xcd - 1) / per_xcd + 4095) / 4096 * 4096;
      const long long lo = (wg >> 3) * slice, hi = min(lo + slice, a.cb_bytes - 16);
      uint32_t v = 0;
      for (long long off = lo + tid * 16; off < hi; off += kThreads * 16) {
        uint4 q;
        __builtin_memcpy(&q, (const uint8_t*)cb + off, 16);
        v ^= q.x ^ q.y ^ q.z ^ q.w;
      }
      asm volatile("" ::"v"(v));      // keep the loads; the value is not used
    }
  }

  float acc[BT][JPL];
  float bsum[JPL];
#pragma unroll
  for (int p = 0; p < JPL; ++p) {
    bsum[p] = 0.f;
#pragma unroll
    for (int bb = 0; bb < BT; ++bb) acc[bb][p] = 0.f;
  }

  // SL: the kRuns threads that share a row take consecutive runs of slices, up to 16 loads in
  // flight each; their sums are added in run order when the row's basis data is built.
  constexpr int kRuns = kThreads / kSub;
  __shared__ float sxr[SL ? kRuns : 1][SL ? kSub : 1];

  for (int s0 = i_begin; s0 < i_end; s0 += kSub) {
    const int rows = min(kSub, i_end - s0);
    __syncthreads();
    if constexpr (SL) {
      const int r = tid % kSub, g = tid / kSub;
      const int per_run = (a.x_parts + kRuns - 1) / kRuns;
      const int p_begin = min(g * per_run, a.x_parts), p_end = min(a.x_parts, p_begin + per_run);
      const float* src = xh + (long long)b0 * n_in + s0 + min(r, rows - 1);
      float sum = 0.f;
      for (int p0 = p_begin; p0 < p_end; p0 += 16) {
        float t[16];
#pragma unroll
        for (int pp = 0; pp < 16; ++pp)               // (slices past the last one are re-reads of it, added as zero)
          t[pp] = src[(long long)min(p0 + pp, a.x_parts - 1) * a.x_part_stride];
#pragma unroll
        for (int pp = 0; pp < 16; ++pp) sum += (p0 + pp < p_end) ? t[pp] : 0.f;
      }
      sxr[g][r] = sum;
      __syncthreads();
    }
    // ---- span + weights for (row, sample) of this sub-chunk ----------------------
    for (int t = tid; t < kSub * BT; t += kThreads) {
      const int bb = t / kSub, r = t % kSub;
      BasisW bw = {0.f, 0.f, 0.f, 0.f, 0};
      if constexpr (SL) {
        float xv = sxr[0][r];
#pragma unroll
        for (int g = 1; g < kRuns; ++g) xv += sxr[g][r];
        if (r < rows) bw = basis_eval_rule(a.x_tanh ? tanhf(xv) : xv, a.rule);
      } else {
        if (r < rows && b0 + bb < a.B) bw = basis_eval_rule(xh[(long long)(b0 + bb) * n_in + s0 + r], a.rule);
      }
      if constexpr (kWindow) {
        sw[r] = make_float4(bw.w0, bw.w1, bw.w2, bw.w3);
        ss[r] = bw.span;
      } else {
        // 10-vector of weights, zeros outside span..span+3 (same thread: LDS keeps order)
        float* w10 = lds + (r * BT + bb) * kWStride;
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        ((float4*)w10)[0] = z;
        ((float4*)w10)[1] = z;
        ((float4*)w10)[2] = z;
        w10[bw.span] = bw.w0;
        w10[bw.span + 1] = bw.w1;
        w10[bw.span + 2] = bw.w2;
        w10[bw.span + 3] = bw.w3;
      }
    }
    __syncthreads();

    if constexpr (kWindow) {
      // one sample: only the 4 coefficients under the nonzero bases are fetched.  Rows are
      // taken four at a time so that all metadata loads, then all gathers, are in flight
      // together (rows past the end are clamped and contribute nothing).
      constexpr int R = 4;
      if (j_ok) {
        for (int r0 = wi; r0 < rows; r0 += wi_count * R) {
          uint32_t id[R][JPL];
          float g[R][JPL], bv[R][JPL];
#pragma unroll
          for (int q = 0; q < R; ++q) {
            const int r = min(r0 + q * wi_count, rows - 1);
            const long long e = (long long)(s0 + r) * n_out + j0;
            load_idx<IdxT, JPL>(idx + e, id[q]);
            load_gain<GbT, JPL>(gain + e, qp, g[q]);
            load_bias<GbT, JPL>(bias + e, qp, bv[q]);
          }
          typename WindowRaw<CbT>::type raw[R][JPL];
          int sp[R];
          float4 w[R];
#pragma unroll
          for (int q = 0; q < R; ++q) {
            const int r = min(r0 + q * wi_count, rows - 1);
            sp[q] = ss[r];
            w[q] = sw[r];
#pragma unroll
            for (int p = 0; p < JPL; ++p) raw[q][p] = load_window<CbT>(cb, id[q][p], sp[q]);
          }
#pragma unroll
          for (int q = 0; q < R; ++q) {
            const float live = (r0 + q * wi_count < rows) ? 1.0f : 0.0f;
#pragma unroll
            for (int p = 0; p < JPL; ++p) {
              float c[4];
              dequant_window<CbT>(raw[q][p], live * g[q][p] * scale, c);
              float v = acc[0][p];
              v = fmaf(w[q].x, c[0], v);
              v = fmaf(w[q].y, c[1], v);
              v = fmaf(w[q].z, c[2], v);
              v = fmaf(w[q].w, c[3], v);
              acc[0][p] = v;
              bsum[p] = fmaf(live, bv[q][p], bsum[p]);
            }
          }
        }
      }
    } else if (j_ok) {
      for (int r = wi; r < rows; r += wi_count) {
        const long long e = (long long)(s0 + r) * n_out + j0;
        {
          float c[JPL][kG];
          if constexpr (CODE == kDense) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            const f32x2* row = (const f32x2*)((const float*)cb + e * kG);
#pragma unroll
            for (int p = 0; p < JPL; ++p)
#pragma unroll
              for (int m = 0; m < kG / 2; ++m) {
                const f32x2 v = __builtin_nontemporal_load(row + p * (kG / 2) + m);
                c[p][2 * m] = v.x;
                c[p][2 * m + 1] = v.y;
              }
          } else {
            uint32_t id[JPL];
            float g[JPL], bv[JPL];
            load_idx<IdxT, JPL>(idx + e, id);
            load_gain<GbT, JPL>(gain + e, qp, g);
            load_bias<GbT, JPL>(bias + e, qp, bv);
#pragma unroll
            for (int p = 0; p < JPL; ++p) {
              fetch_row<CbT>(cb, id[p], g[p] * scale, c[p]);
              bsum[p] += bv[p];
            }
          }
#pragma unroll
          for (int bb = 0; bb < BT; ++bb) {
            const float4* w10 = (const float4*)(lds + (r * BT + bb) * kWStride);
            const float4 wa = w10[0], wb = w10[1], wc = w10[2];
#pragma unroll
            for (int p = 0; p < JPL; ++p) {
              float v = acc[bb][p];
              v = fmaf(wa.x, c[p][0], v);
              v = fmaf(wa.y, c[p][1], v);
              v = fmaf(wa.z, c[p][2], v);
              v = fmaf(wa.w, c[p][3], v);
              v = fmaf(wb.x, c[p][4], v);
              v = fmaf(wb.y, c[p][5], v);
              v = fmaf(wb.z, c[p][6], v);
              v = fmaf(wb.w, c[p][7], v);
              v = fmaf(wc.x, c[p][8], v);
              v = fmaf(wc.y, c[p][9], v);
              acc[bb][p] = v;
            }
          }
        }
      }
    }
  }

  // ---- sum over the waves interleaved along i ------------------------------------
  if (wi_count > 1) {
    __syncthreads();
    float* red = lds;    // [(wi-1)][wj][BT][JPL][lane]
    if (wi > 0) {
      float* dstp = red + (((wi - 1) * wj_count + wj) * BT * JPL) * kWave + lane;
#pragma unroll
      for (int bb = 0; bb < BT; ++bb)
#pragma unroll
        for (int p = 0; p < JPL; ++p) dstp[(bb * JPL + p) * kWave] = acc[bb][p];
    }
    __syncthreads();
    if (wi == 0) {
      for (int o = 1; o < wi_count; ++o) {
        const float* srcp = red + (((o - 1) * wj_count + wj) * BT * JPL) * kWave + lane;
#pragma unroll
        for (int bb = 0; bb < BT; ++bb)
#pragma unroll
          for (int p = 0; p < JPL; ++p) acc[bb][p] += srcp[(bb * JPL + p) * kWave];
      }
    }
    __syncthreads();   // bias sums travel in a second pass through the same buffer
    if (wi > 0) {
      float* dstp = red + (((wi - 1) * wj_count + wj) * JPL) * kWave + lane;
#pragma unroll
      for (int p = 0; p < JPL; ++p) dstp[p * kWave] = bsum[p];
    }
    __syncthreads();
    if (wi == 0) {
      for (int o = 1; o < wi_count; ++o) {
        const float* srcp = red + (((o - 1) * wj_count + wj) * JPL) * kWave + lane;
#pragma unroll
        for (int p = 0; p < JPL; ++p) bsum[p] += srcp[p * kWave];
      }
    }
  }

  // ---- write y, the hidden activation, or this chunk's partial sums -------------
  if (wi == 0 && j_ok) {
    float* dst = a.dst + (long long)head * a.dst_head_stride + (long long)chunk * a.dst_chunk_stride;
#pragma unroll
    for (int bb = 0; bb < BT; ++bb) {
      if (b0 + bb < a.B) {
        float* o = dst + (long long)(b0 + bb) * n_out + j0;
#pragma unroll
        for (int p = 0; p < JPL; ++p) {
          float v = acc[bb][p] + bsum[p];
          if (a.apply_tanh) v = tanhf(v);
          o[p] = v;
        }
      }
    }
  }
}

template <typename IdxT, typename GbT, typename CbT, int CODE, int JPL>
hipError_t launch_one(const GatherCfg& c, const GatherArgs& a, dim3 grid, hipStream_t s) {
  if constexpr (KAN_BT == 1 && CODE != kDense) {
    if (a.x_parts > 1) {
      hipLaunchKernelGGL((kan_gather_kernel<IdxT, GbT, CbT, CODE, KAN_BT, JPL, true>), grid, dim3(kThreads), 0, s,
                         a, c.wj);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((kan_gather_kernel<IdxT, GbT, CbT, CODE, KAN_BT, JPL>), grid, dim3(kThreads), 0, s,
                     a, c.wj);
  return hipGetLastError();
}

template <typename IdxT, typename GbT, typename CbT, int CODE>
hipError_t launch_jpl(const GatherCfg& c, const GatherArgs& a, dim3 grid, hipStream_t s) {
  switch (c.jpl) {
    case 1: return launch_one<IdxT, GbT, CbT, CODE, 1>(c, a, grid, s);
    case 2: return launch_one<IdxT, GbT, CbT, CODE, 2>(c, a, grid, s);
    case 4: return launch_one<IdxT, GbT, CbT, CODE, 4>(c, a, grid, s);
#if KAN_BT <= 4
    case 8: return launch_one<IdxT, GbT, CbT, CODE, 8>(c, a, grid, s);
#endif
    default: return hipErrorInvalidValue;
  }
}

// The vector-ALU kernel serves VQ layers at batch 1 only (larger batches go to the fused
// matrix-core kernel); the batch tiles 4 and 16 exist for the dense baseline.
#if KAN_BT == 1
template <typename IdxT>
hipError_t launch_types(const GatherCfg& c, const GatherArgs& a, dim3 grid, hipStream_t s) {
  if (c.code == kCbI8) {
    if (c.gb_kind == kGbQ8) return launch_jpl<IdxT, q8_t, int8_t, kCbI8>(c, a, grid, s);
    return c.gb_kind == kGbF16 ? launch_jpl<IdxT, __half, int8_t, kCbI8>(c, a, grid, s)
                               : launch_jpl<IdxT, float, int8_t, kCbI8>(c, a, grid, s);
  }
  if (c.gb_kind == kGbQ8) return hipErrorInvalidValue;      // byte-coded gain/bias go with Int8 codebooks
  if (c.code == kCbBfp8)
    return c.gb_kind == kGbF16 ? launch_jpl<IdxT, __half, bfp8_t, kCbBfp8>(c, a, grid, s)
                               : launch_jpl<IdxT, float, bfp8_t, kCbBfp8>(c, a, grid, s);
  if (c.code == kCbF16)
    return c.gb_kind == kGbF16 ? launch_jpl<IdxT, __half, __half, kCbF16>(c, a, grid, s)
                               : launch_jpl<IdxT, float, __half, kCbF16>(c, a, grid, s);
  return c.gb_kind == kGbF16 ? launch_jpl<IdxT, __half, float, kCbF32>(c, a, grid, s)
                             : launch_jpl<IdxT, float, float, kCbF32>(c, a, grid, s);
}
#endif

}  // namespace

#define KAN_CAT2(a, b) a##b
#define KAN_CAT(a, b) KAN_CAT2(a, b)

hipError_t KAN_CAT(launch_gather_bt, KAN_BT)(const GatherCfg& c, const GatherArgs& a, dim3 grid,
                                              hipStream_t s) {
  if (c.bt != KAN_BT) return hipErrorInvalidValue;
  // slices of the input: the window form only (VQ layers, one sample per tile)
  if (a.x_parts > 1 && (KAN_BT != 1 || c.code == kDense || a.x_parts > kGatherChainMaxParts)) return hipErrorInvalidValue;
  if (c.code == kDense) return launch_jpl<uint16_t, float, float, kDense>(c, a, grid, s);
#if KAN_BT == 1
  return c.idx_u32 ? launch_types<uint32_t>(c, a, grid, s) : launch_types<uint16_t>(c, a, grid, s);
#else
  return hipErrorInvalidValue;
#endif
}

}  // namespace kan
