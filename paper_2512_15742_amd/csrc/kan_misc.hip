// Small kernels around the main paths: fixed-order reduction of i-chunk partial
// sums (+ the inter-layer tanh), the stand-alone span/basis kernel, and the
// debug kernels that expose what the load routines fetch.

#include "kan_device.hpp"
#include "kan_internal.hpp"

namespace kan {
namespace {

// dst[n] = act(sum_c partial[c][n]).  A workgroup covers 256 / CG consecutive
// outputs; CG threads share one output, each summing every CG-th chunk with
// four independent loads in flight, and their CG sums are added in fixed order
// through LDS, so the result does not depend on scheduling.
template <int CG>
__global__ __launch_bounds__(256) void kan_reduce_kernel(const float* __restrict__ partial,
                                                         long long head_stride, long long chunk_stride,
                                                         int n_chunks, float* __restrict__ dst,
                                                         long long dst_head_stride, long long count,
                                                         int apply_tanh) {
  constexpr int NPB = 256 / CG;     // outputs per workgroup
  __shared__ float red[CG][NPB];
  const int head = blockIdx.y;
  const float* p = partial + (long long)head * head_stride;
  float* d = dst + (long long)head * dst_head_stride;
  const int nn = threadIdx.x % NPB, cg = threadIdx.x / NPB;
  for (long long n0 = (long long)blockIdx.x * NPB; n0 < count; n0 += (long long)gridDim.x * NPB) {
    const long long n = n0 + nn;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (n < count) {
      int c = cg;
      for (; c + 3 * CG < n_chunks; c += 4 * CG) {
        s0 += __builtin_nontemporal_load(p + (long long)c * chunk_stride + n);
        s1 += __builtin_nontemporal_load(p + (long long)(c + CG) * chunk_stride + n);
        s2 += __builtin_nontemporal_load(p + (long long)(c + 2 * CG) * chunk_stride + n);
        s3 += __builtin_nontemporal_load(p + (long long)(c + 3 * CG) * chunk_stride + n);
      }
      for (; c < n_chunks; c += CG) s0 += __builtin_nontemporal_load(p + (long long)c * chunk_stride + n);
    }
    float s = (s0 + s1) + (s2 + s3);
    if constexpr (CG > 1) {
      red[cg][nn] = s;
      __syncthreads();
      if (cg == 0) {
#pragma unroll
        for (int g = 1; g < CG; ++g) s += red[g][nn];
      }
      __syncthreads();
    }
    if (cg == 0 && n < count) d[n] = apply_tanh ? tanhf(s) : s;
  }
}

// Large tensors: one thread adds four consecutive outputs over all chunks with 16-byte loads,
// four chunks in flight (fixed order: chunks c, c+4, c+8, ... into accumulator c mod 4, then
// (s0 + s1) + (s2 + s3)).
__global__ __launch_bounds__(256) void kan_reduce_vec4_kernel(const float* __restrict__ partial,
                                                              long long head_stride, long long chunk_stride,
                                                              int n_chunks, float* __restrict__ dst,
                                                              long long dst_head_stride, long long count4,
                                                              int apply_tanh) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const int head = blockIdx.y;
  const f32x4* p = (const f32x4*)(partial + (long long)head * head_stride);
  f32x4* d = (f32x4*)(dst + (long long)head * dst_head_stride);
  const long long cs4 = chunk_stride / 4;
  for (long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x; n < count4;
       n += (long long)gridDim.x * blockDim.x) {
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0, s2 = s0, s3 = s0;
    int c = 0;
    for (; c + 3 < n_chunks; c += 4) {
      s0 += __builtin_nontemporal_load(p + (long long)c * cs4 + n);
      s1 += __builtin_nontemporal_load(p + (long long)(c + 1) * cs4 + n);
      s2 += __builtin_nontemporal_load(p + (long long)(c + 2) * cs4 + n);
      s3 += __builtin_nontemporal_load(p + (long long)(c + 3) * cs4 + n);
    }
    for (; c < n_chunks; ++c) s0 += __builtin_nontemporal_load(p + (long long)c * cs4 + n);
    f32x4 v = (s0 + s1) + (s2 + s3);
    if (apply_tanh) {
      v.x = tanhf(v.x);
      v.y = tanhf(v.y);
      v.z = tanhf(v.z);
      v.w = tanhf(v.w);
    }
    d[n] = v;
  }
}

__global__ __launch_bounds__(256) void kan_basis_kernel(const float* __restrict__ x, long long n,
                                                        uint8_t* __restrict__ span, float* __restrict__ w) {
  for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < n;
       t += (long long)gridDim.x * blockDim.x) {
    const BasisW b = basis_eval(x[t]);
    span[t] = (uint8_t)b.span;
    ((float4*)w)[t] = make_float4(b.w0, b.w1, b.w2, b.w3);
  }
}

// Index k (0..8) and the two weights (1 - u, u) of the two-tap rule, for parity checks.
__global__ __launch_bounds__(256) void kan_pli_basis_kernel(const float* __restrict__ x, long long n,
                                                            uint8_t* __restrict__ index, float* __restrict__ w) {
  for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < n;
       t += (long long)gridDim.x * blockDim.x) {
    const PliIndex p = pli_index(x[t]);
    index[t] = (uint8_t)p.k;
    ((float2*)w)[t] = make_float2((float)(1.0 - p.u), (float)p.u);
  }
}

// The four-entry window (first entry, four weights) of either rule as the forward kernels form
// it: FAST = false through basis_eval / basis_eval_pli (vector-ALU and bucket kernels), FAST =
// true through basis_fast (fused kernel, basis preparation of the streaming contraction).
template <bool FAST>
__global__ __launch_bounds__(256) void kan_basis_window_kernel(const float* __restrict__ x, long long n, int rule,
                                                               uint8_t* __restrict__ start, float* __restrict__ w) {
  for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < n;
       t += (long long)gridDim.x * blockDim.x) {
    const BasisW b = FAST ? basis_fast(x[t], rule) : basis_eval_rule(x[t], rule);
    start[t] = (uint8_t)b.span;
    ((float4*)w)[t] = make_float4(b.w0, b.w1, b.w2, b.w3);
  }
}

template <typename IdxT, typename CbT>
__global__ __launch_bounds__(256) void kan_debug_gather_kernel(const IdxT* __restrict__ idx,
                                                               const CbT* __restrict__ cb, float scale,
                                                               long long edges, uint32_t* __restrict__ ids,
                                                               float* __restrict__ rows) {
  for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < edges;
       e += (long long)gridDim.x * blockDim.x) {
    uint32_t id[1];
    load_idx<IdxT, 1>(idx + e, id);
    if (ids) ids[e] = id[0];
    if (rows) {
      float c[kG];
      fetch_row<CbT>(cb, id[0], scale, c);
#pragma unroll
      for (int m = 0; m < kG; ++m) rows[e * kG + m] = c[m];
    }
  }
}

template <typename IdxT>
__global__ __launch_bounds__(256) void kan_count_bad_kernel(const IdxT* __restrict__ idx, long long edges,
                                                            uint32_t K, uint32_t* __restrict__ count) {
  uint32_t bad = 0;
  for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < edges;
       e += (long long)gridDim.x * blockDim.x)
    bad += ((uint32_t)idx[e] >= K) ? 1u : 0u;
  if (bad) atomicAdd(count, bad);
}

__global__ void kan_zero_u32_kernel(uint32_t* p) { *p = 0u; }

// Smallest nonzero and largest magnitude of the fp16 coefficient operand of the matrix-core
// kernels, gain * q (Int8 codes) or gain * C (floating codebooks), over all edges and entries.
// Magnitudes are non-negative floats, whose order is that of their bit patterns.
__global__ void kan_range_init_kernel(uint32_t* r) {
  r[0] = 0x7f800000u;      // +inf: no nonzero product seen
  r[1] = 0u;
}
template <typename IdxT, typename GbT, typename CbT>
__global__ __launch_bounds__(256) void kan_coef_range_kernel(const IdxT* __restrict__ idx, const GbT* __restrict__ gain,
                                                             const CbT* __restrict__ cb, Q8Params qp, long long edges,
                                                             uint32_t* __restrict__ r) {
  float lo = __uint_as_float(0x7f800000u), hi = 0.f;
  for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < edges;
       e += (long long)gridDim.x * blockDim.x) {
    uint32_t id[1];
    float g[1];
    load_idx<IdxT, 1>(idx + e, id);
    load_gain<GbT, 1>(gain + e, qp, g);
    float c[kG];
    fetch_row<CbT>(cb, id[0], g[0], c);
#pragma unroll
    for (int m = 0; m < kG; ++m) {
      const float v = fabsf(c[m]);
      hi = fmaxf(hi, v);
      if (v > 0.f) lo = fminf(lo, v);
    }
  }
  atomicMin(r, __float_as_uint(lo));
  atomicMax(r + 1, __float_as_uint(hi));
}

inline int blocks_for(long long n, int cap = 65536) {
  long long b = (n + 255) / 256;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (int)b;
}

}  // namespace

hipError_t launch_reduce(const float* partial, long long head_stride, long long chunk_stride, int n_chunks,
                         float* dst, long long dst_head_stride, long long count, int n_heads,
                         int apply_tanh, hipStream_t s) {
  const long long total = count * n_heads;
  // large tensors whose rows are 16-byte aligned: vector loads, one thread per four outputs
  if (total >= (1 << 18) && count % 4 == 0 && head_stride % 4 == 0 && chunk_stride % 4 == 0 &&
      dst_head_stride % 4 == 0 && ((uintptr_t)partial % 16) == 0 && ((uintptr_t)dst % 16) == 0) {
    const long long count4 = count / 4;
    long long blocks = (count4 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(kan_reduce_vec4_kernel, dim3((unsigned)blocks, n_heads), dim3(256), 0, s, partial, head_stride,
                       chunk_stride, n_chunks, dst, dst_head_stride, count4, apply_tanh);
    return hipGetLastError();
  }
  // few outputs and many chunks: spread the chunks of one output over several threads
  const int cg = (n_chunks >= 32 && total <= (1 << 16)) ? 16 : ((n_chunks >= 8 && total <= (1 << 20)) ? 4 : 1);
  const int npb = 256 / cg;
  long long blocks = (count + npb - 1) / npb;
  if (blocks > 8192) blocks = 8192;
  dim3 grid((unsigned)blocks, n_heads);
  if (cg == 16)
    hipLaunchKernelGGL(kan_reduce_kernel<16>, grid, dim3(256), 0, s, partial, head_stride, chunk_stride,
                       n_chunks, dst, dst_head_stride, count, apply_tanh);
  else if (cg == 4)
    hipLaunchKernelGGL(kan_reduce_kernel<4>, grid, dim3(256), 0, s, partial, head_stride, chunk_stride,
                       n_chunks, dst, dst_head_stride, count, apply_tanh);
  else
    hipLaunchKernelGGL(kan_reduce_kernel<1>, grid, dim3(256), 0, s, partial, head_stride, chunk_stride,
                       n_chunks, dst, dst_head_stride, count, apply_tanh);
  return hipGetLastError();
}

hipError_t launch_basis(const float* x, long long n, uint8_t* span, float* w, hipStream_t s) {
  hipLaunchKernelGGL(kan_basis_kernel, dim3(blocks_for(n)), dim3(256), 0, s, x, n, span, w);
  return hipGetLastError();
}

hipError_t launch_pli_basis(const float* x, long long n, uint8_t* index, float* w, hipStream_t s) {
  hipLaunchKernelGGL(kan_pli_basis_kernel, dim3(blocks_for(n)), dim3(256), 0, s, x, n, index, w);
  return hipGetLastError();
}

hipError_t launch_basis_window(const float* x, long long n, int rule, int fast, uint8_t* start, float* w,
                               hipStream_t s) {
  if (fast) hipLaunchKernelGGL(kan_basis_window_kernel<true>, dim3(blocks_for(n)), dim3(256), 0, s, x, n, rule, start, w);
  else hipLaunchKernelGGL(kan_basis_window_kernel<false>, dim3(blocks_for(n)), dim3(256), 0, s, x, n, rule, start, w);
  return hipGetLastError();
}

template <typename IdxT>
void debug_gather_types(const LayerPtrs& h, int code, long long edges, uint32_t* ids, float* rows, dim3 grid,
                        hipStream_t s) {
  const dim3 block(256);
  if (code == kCbI8)
    hipLaunchKernelGGL((kan_debug_gather_kernel<IdxT, int8_t>), grid, block, 0, s, (const IdxT*)h.idx,
                       (const int8_t*)h.cb, h.scale, edges, ids, rows);
  else if (code == kCbBfp8)
    hipLaunchKernelGGL((kan_debug_gather_kernel<IdxT, bfp8_t>), grid, block, 0, s, (const IdxT*)h.idx,
                       (const bfp8_t*)h.cb, 1.0f, edges, ids, rows);
  else if (code == kCbF16)
    hipLaunchKernelGGL((kan_debug_gather_kernel<IdxT, __half>), grid, block, 0, s, (const IdxT*)h.idx,
                       (const __half*)h.cb, 1.0f, edges, ids, rows);
  else
    hipLaunchKernelGGL((kan_debug_gather_kernel<IdxT, float>), grid, block, 0, s, (const IdxT*)h.idx,
                       (const float*)h.cb, 1.0f, edges, ids, rows);
}

hipError_t launch_debug_gather(const LayerPtrs& h, int idx_u32, int code, long long edges, uint32_t* ids,
                               float* rows, hipStream_t s) {
  if (code != kCbI8 && code != kCbF16 && code != kCbF32 && code != kCbBfp8) return hipErrorInvalidValue;
  const dim3 grid(blocks_for(edges));
  if (idx_u32)
    debug_gather_types<uint32_t>(h, code, edges, ids, rows, grid, s);
  else
    debug_gather_types<uint16_t>(h, code, edges, ids, rows, grid, s);
  return hipGetLastError();
}

namespace {
template <typename IdxT, typename GbT, typename CbT>
void coef_range_launch(const LayerPtrs& h, long long edges, float* range, hipStream_t s) {
  hipLaunchKernelGGL((kan_coef_range_kernel<IdxT, GbT, CbT>), dim3(blocks_for(edges, 2048)), dim3(256), 0, s,
                     (const IdxT*)h.idx, (const GbT*)h.gain, (const CbT*)h.cb,
                     Q8Params{h.gain_log2_lo, h.gain_log2_step, h.bias_scale}, edges, (uint32_t*)range);
}
template <typename IdxT>
hipError_t coef_range_types(const LayerPtrs& h, int gb_kind, int code, long long edges, float* range, hipStream_t s) {
  if (code == kCbI8) {
    if (gb_kind == kGbQ8) coef_range_launch<IdxT, q8_t, int8_t>(h, edges, range, s);
    else if (gb_kind == kGbF16) coef_range_launch<IdxT, __half, int8_t>(h, edges, range, s);
    else coef_range_launch<IdxT, float, int8_t>(h, edges, range, s);
  } else if (gb_kind == kGbQ8) {
    return hipErrorInvalidValue;
  } else if (code == kCbBfp8) {
    if (gb_kind == kGbF16) coef_range_launch<IdxT, __half, bfp8_t>(h, edges, range, s);
    else coef_range_launch<IdxT, float, bfp8_t>(h, edges, range, s);
  } else if (code == kCbF16) {
    if (gb_kind == kGbF16) coef_range_launch<IdxT, __half, __half>(h, edges, range, s);
    else coef_range_launch<IdxT, float, __half>(h, edges, range, s);
  } else if (code == kCbF32) {
    if (gb_kind == kGbF16) coef_range_launch<IdxT, __half, float>(h, edges, range, s);
    else coef_range_launch<IdxT, float, float>(h, edges, range, s);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
}  // namespace

hipError_t launch_coef_range(const LayerPtrs& h, int idx_u32, int gb_kind, int code, long long edges, float* range,
                             hipStream_t s) {
  hipLaunchKernelGGL(kan_range_init_kernel, dim3(1), dim3(1), 0, s, (uint32_t*)range);
  return idx_u32 ? coef_range_types<uint32_t>(h, gb_kind, code, edges, range, s)
                 : coef_range_types<uint16_t>(h, gb_kind, code, edges, range, s);
}

hipError_t launch_count_bad(const void* idx, int idx_u32, long long edges, uint32_t K, uint32_t* count,
                            hipStream_t s) {
  hipLaunchKernelGGL(kan_zero_u32_kernel, dim3(1), dim3(1), 0, s, count);
  dim3 grid(blocks_for(edges, 2048)), block(256);
  if (idx_u32)
    hipLaunchKernelGGL((kan_count_bad_kernel<uint32_t>), grid, block, 0, s, (const uint32_t*)idx, edges, K, count);
  else
    hipLaunchKernelGGL((kan_count_bad_kernel<uint16_t>), grid, block, 0, s, (const uint16_t*)idx, edges, K, count);
  return hipGetLastError();
}

}  // namespace kan
