// Small-batch path over a prepared layer: the codebook lives in LDS.
//
// At batch 1 a layer is one pass over its per-edge metadata (paper section 4.2: the
// memory-bound regime) plus one codeword lookup per edge (Eq. (1)).  Lookups that go to L2
// are limited by the rate at which a CU can issue divergent addresses, far below what the
// metadata stream could sustain; lookups in LDS are not.  The 655 KB Int8 codebook does not
// fit the 160 KB LDS of a CU, but an eighth of it does, so the edges are regrouped once
// (kan_vq_prepare) by bucket = idx / 8192 (fp32 rows: idx / 2048) and every workgroup serves
// one bucket: it copies the 80 KB of codeword rows into LDS, builds the span/basis table of
// all inputs of its sample there as well, and then streams its share of the bucket's edges.
//
// Inside a bucket the edges are ordered by output j, then input i, so a segment (the run of
// edges of one output) is summed by one wave with a fixed-order tree, and the per-bucket
// sums are added by the fixed-order reduction kernel: no atomics, reproducible bits.
// The bias of an edge needs no lookup at all: the four bases sum to 1 on [-1,1], so
// sum_i bias_ij is a per-output constant computed at preparation time.
//
// This file also holds the three preparation kernels (count, scan, fill).

#include "kan_device.hpp"
#include "kan_internal.hpp"

namespace kan {
namespace {

constexpr int kWaves = kBucketThreads / kWave;   // 16
constexpr int kUnroll = 4;                       // edges per lane per chunk (256 per wave)

// Gains travel as raw bits (uint16_t for fp16, float for fp32).
template <typename GRaw>
struct ChunkRegs {
  uint32_t i[kUnroll], q[kUnroll];
  GRaw g[kUnroll];
};

struct ChunkDesc {
  int n;         // edges in the chunk (0..256)
  int j;         // output the chunk belongs to
  bool last;     // chunk ends its segment
  bool valid;
};

__device__ __forceinline__ float gain_to_float(float g) { return g; }
__device__ __forceinline__ float gain_to_float(__half g) { return __half2float(g); }
__device__ __forceinline__ float gain_to_float(uint16_t g) { return __half2float(__ushort_as_half(g)); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

template <typename GbT, bool I8>
__global__ __launch_bounds__(kBucketThreads) void kan_bucket_kernel(const BucketArgs a) {   // GbT: uint16_t | float
  __shared__ __attribute__((aligned(16))) uint32_t cb[kBucketBytes / 4 + 4];
  __shared__ float4 bas[kBucketMaxIn];

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int head = blockIdx.z, b = blockIdx.y;
  const int bucket = blockIdx.x % a.n_buckets, part = blockIdx.x / a.n_buckets;
  const BucketHead H = a.h[head];
  const char* prep = (const char*)H.prepared;
  const uint32_t* __restrict__ seg = (const uint32_t*)(prep + a.off_seg) + (size_t)bucket * a.n_out;
  const uint16_t* __restrict__ pi = (const uint16_t*)(prep + a.off_i);
  const uint16_t* __restrict__ pq = (const uint16_t*)(prep + a.off_q);
  const GbT* __restrict__ pg = (const GbT*)(prep + a.off_g);

  const int j0 = part * a.jw;
  const int j1 = min(j0 + a.jw, a.n_out);
  const int first_j = j0 + wave;
  const int n_seg = first_j < j1 ? (j1 - first_j + kWaves - 1) / kWaves : 0;   // segments of this wave

  // ---- generator over this wave's chunks (all state wave-uniform) ------------------
  int k = 0;
  bool have = n_seg > 0;
  uint32_t pos = 0, end = 0, nxt_pos = 0, nxt_end = 0;
  if (have) {
    pos = seg[first_j];
    end = seg[first_j + 1];
    if (n_seg > 1) {
      nxt_pos = seg[first_j + kWaves];
      nxt_end = seg[first_j + kWaves + 1];
    }
  }
  auto next = [&](ChunkRegs<GbT>& c, ChunkDesc& d) {
    d.valid = have;
    if (!have) return;
    d.j = first_j + k * kWaves;
    const uint32_t left = end - pos;
    d.n = (int)(left < (uint32_t)(kWave * kUnroll) ? left : (uint32_t)(kWave * kUnroll));
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int o = u * kWave + lane;
      const size_t e = (size_t)pos + o;
      const bool v = o < d.n;
      c.i[u] = v ? (uint32_t)__builtin_nontemporal_load(pi + e) : 0u;
      c.q[u] = v ? (uint32_t)__builtin_nontemporal_load(pq + e) : 0u;
      c.g[u] = v ? __builtin_nontemporal_load(pg + e) : GbT(0);
    }
    pos += (uint32_t)d.n;
    d.last = pos == end;
    if (d.last) {
      ++k;
      have = k < n_seg;
      pos = nxt_pos;
      end = nxt_end;
      if (k + 1 < n_seg) {
        nxt_pos = seg[first_j + (k + 1) * kWaves];
        nxt_end = seg[first_j + (k + 1) * kWaves + 1];
      }
    }
  };

  ChunkRegs<GbT> A, B;
  ChunkDesc dA, dB;
  next(A, dA);   // the first records travel while the tables are built

  // ---- codebook bucket -> LDS ---------------------------------------------------------
  {
    const long long start = (long long)bucket * kBucketBytes;
    const long long rest = a.cb_bytes - start;
    const int nbytes = (int)(rest < kBucketBytes ? rest : kBucketBytes);
    const char* src = (const char*)H.cb + start;
    const int n16 = nbytes >> 4;
    for (int t = tid; t < n16; t += kBucketThreads) ((uint4*)cb)[t] = ((const uint4*)src)[t];
    const int tail = nbytes & 15;
    if (tid < tail) ((uint8_t*)cb)[n16 * 16 + tid] = ((const uint8_t*)src)[n16 * 16 + tid];
  }
  // ---- span + weights of every input of sample b -> LDS (span in the sign bits of w0..w2) --
  {
    const float* xr = a.x + (long long)head * a.x_head_stride + (long long)b * a.n_in;
    for (int i = tid; i < a.n_in; i += kBucketThreads) {
      const BasisW w = basis_eval(xr[i]);
      float4 v;
      v.x = __uint_as_float(__float_as_uint(w.w0) | ((uint32_t)(w.span & 1) << 31));
      v.y = __uint_as_float(__float_as_uint(w.w1) | ((uint32_t)((w.span >> 1) & 1) << 31));
      v.z = __uint_as_float(__float_as_uint(w.w2) | ((uint32_t)((w.span >> 2) & 1) << 31));
      v.w = w.w3;
      bas[i] = v;
    }
  }
  __syncthreads();

  float* dst = a.dst + (long long)head * a.dst_head_stride + (long long)bucket * a.dst_chunk_stride +
               (long long)b * a.n_out;
  const float* bias_sum = (const float*)(prep + a.off_bias);
  const float scale = I8 ? H.scale : 1.0f;
  float acc = 0.f;

  auto consume = [&](const ChunkRegs<GbT>& c, const ChunkDesc& d) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const float4 w = bas[c.i[u]];
      const uint32_t span = (__float_as_uint(w.x) >> 31) | ((__float_as_uint(w.y) >> 31) << 1) |
                            ((__float_as_uint(w.z) >> 31) << 2);
      const uint32_t at = c.q[u] * 10u + span;
      float c0, c1, c2, c3;
      if constexpr (I8) {
        // bytes at .. at+3 of the bucket: two aligned dwords, funnel-shifted
        const uint32_t lo = cb[at >> 2], hi = cb[(at >> 2) + 1];
        const uint32_t win = __builtin_amdgcn_alignbyte(hi, lo, at & 3u);
        c0 = (float)(int)(int8_t)(win & 0xff);
        c1 = (float)(int)(int8_t)((win >> 8) & 0xff);
        c2 = (float)(int)(int8_t)((win >> 16) & 0xff);
        c3 = (float)(int)(int8_t)(win >> 24);
      } else {
        const float* cf = (const float*)cb;
        c0 = cf[at];
        c1 = cf[at + 1];
        c2 = cf[at + 2];
        c3 = cf[at + 3];
      }
      float s = w.w * c3;
      s = fmaf(fabsf(w.z), c2, s);
      s = fmaf(fabsf(w.y), c1, s);
      s = fmaf(fabsf(w.x), c0, s);
      // lanes past the end of the chunk looked up row 0 with gain 0; keep even a non-finite
      // row 0 out of the sum
      acc = (u * kWave + lane < d.n) ? fmaf(gain_to_float(c.g[u]), s, acc) : acc;
    }
    if (d.last) {
      const float t = wave_sum(acc);
      if (lane == 0) {
        float v = scale * t + (bucket == 0 ? bias_sum[d.j] : 0.0f);
        if (a.apply_tanh && a.n_buckets == 1) v = tanhf(v);
        dst[d.j] = v;
      }
      acc = 0.f;
    }
  };

  while (true) {
    next(B, dB);
    if (!dA.valid) break;
    consume(A, dA);
    next(A, dA);
    if (!dB.valid) break;
    consume(B, dB);
  }
}

// ---- preparation ------------------------------------------------------------------------
// Thread (j, bucket) counts the edges of its segment, walking i upwards.
template <typename IdxT>
__global__ __launch_bounds__(256) void kan_prepare_count_kernel(const IdxT* __restrict__ idx, int n_in, int n_out,
                                                                int rows_shift, uint32_t* __restrict__ seg) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t bucket = blockIdx.y;
  if (j >= n_out) return;
  uint32_t c = 0;
  for (int i = 0; i < n_in; ++i) c += ((uint32_t)idx[(size_t)i * n_out + j] >> rows_shift) == bucket;
  seg[(size_t)bucket * n_out + j] = c;
}

// In-place exclusive scan of n counts by one workgroup; seg[n] = total.
__global__ __launch_bounds__(1024) void kan_prepare_scan_kernel(uint32_t* __restrict__ seg, long long n) {
  __shared__ uint32_t part[1024];
  const int t = threadIdx.x;
  const long long per = (n + 1023) / 1024;
  const long long lo = t * per, hi = lo + per < n ? lo + per : n;
  uint32_t s = 0;
  for (long long p = lo; p < hi; ++p) s += seg[p];
  part[t] = s;
  __syncthreads();
  if (t == 0) {
    uint32_t run = 0;
    for (int q = 0; q < 1024; ++q) {
      const uint32_t v = part[q];
      part[q] = run;
      run += v;
    }
    seg[n] = run;
  }
  __syncthreads();
  uint32_t run = part[t];
  for (long long p = lo; p < hi; ++p) {
    const uint32_t v = seg[p];
    seg[p] = run;
    run += v;
  }
}

// Thread (j, bucket) writes the records of its segment in order of i; bucket 0 also sums
// the biases of output j (in fp64, rounded once).
template <typename IdxT, typename GbT>
__global__ __launch_bounds__(256) void kan_prepare_fill_kernel(const IdxT* __restrict__ idx,
                                                               const GbT* __restrict__ gain,
                                                               const GbT* __restrict__ bias, int n_in, int n_out,
                                                               int rows_shift, const uint32_t* __restrict__ seg,
                                                               uint16_t* __restrict__ pi, uint16_t* __restrict__ pq,
                                                               GbT* __restrict__ pg, float* __restrict__ bias_sum) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t bucket = blockIdx.y;
  if (j >= n_out) return;
  size_t pos = seg[(size_t)bucket * n_out + j];
  const uint32_t mask = (1u << rows_shift) - 1u;
  double bs = 0.0;
  for (int i = 0; i < n_in; ++i) {
    const size_t e = (size_t)i * n_out + j;
    const uint32_t id = (uint32_t)idx[e];
    if ((id >> rows_shift) == bucket) {
      pi[pos] = (uint16_t)i;
      pq[pos] = (uint16_t)(id & mask);
      pg[pos] = gain[e];
      ++pos;
    }
    if (bucket == 0) bs += (double)gain_to_float(bias[e]);
  }
  if (bucket == 0) bias_sum[j] = (float)bs;
}

template <typename IdxT, typename GbT>
hipError_t prepare_typed(const LayerPtrs& h, int n_in, int n_out, const BucketGeom& g, void* prepared,
                         hipStream_t s) {
  char* p = (char*)prepared;
  uint32_t* seg = (uint32_t*)(p + g.off_seg);
  dim3 grid((unsigned)((n_out + 255) / 256), (unsigned)g.n_buckets);
  hipLaunchKernelGGL((kan_prepare_count_kernel<IdxT>), grid, dim3(256), 0, s, (const IdxT*)h.idx, n_in, n_out,
                     g.rows_shift, seg);
  hipLaunchKernelGGL(kan_prepare_scan_kernel, dim3(1), dim3(1024), 0, s, seg, (long long)g.n_buckets * n_out);
  hipLaunchKernelGGL((kan_prepare_fill_kernel<IdxT, GbT>), grid, dim3(256), 0, s, (const IdxT*)h.idx,
                     (const GbT*)h.gain, (const GbT*)h.bias, n_in, n_out, g.rows_shift, (const uint32_t*)seg,
                     (uint16_t*)(p + g.off_i), (uint16_t*)(p + g.off_q), (GbT*)(p + g.off_g),
                     (float*)(p + g.off_bias));
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bucket_prepare(const LayerPtrs& h, int idx_u32, int gb_f16, int n_in, int n_out,
                                 const BucketGeom& g, void* prepared, hipStream_t s) {
  if (idx_u32) {
    if (gb_f16) return prepare_typed<uint32_t, __half>(h, n_in, n_out, g, prepared, s);
    return prepare_typed<uint32_t, float>(h, n_in, n_out, g, prepared, s);
  }
  if (gb_f16) return prepare_typed<uint16_t, __half>(h, n_in, n_out, g, prepared, s);
  return prepare_typed<uint16_t, float>(h, n_in, n_out, g, prepared, s);
}

hipError_t launch_bucket(bool cb_i8, bool gb_f16, const BucketArgs& a, int parts, int heads, hipStream_t s) {
  if (a.n_in > kBucketMaxIn || a.n_buckets < 1 || parts < 1 || a.jw < 1 || (long long)parts * a.jw < a.n_out)
    return hipErrorInvalidValue;
  dim3 grid((unsigned)(parts * a.n_buckets), (unsigned)a.B, (unsigned)heads);
  dim3 block(kBucketThreads);
  if (cb_i8) {
    if (gb_f16) hipLaunchKernelGGL((kan_bucket_kernel<uint16_t, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((kan_bucket_kernel<float, true>), grid, block, 0, s, a);
  } else {
    if (gb_f16) hipLaunchKernelGGL((kan_bucket_kernel<uint16_t, false>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((kan_bucket_kernel<float, false>), grid, block, 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace kan
