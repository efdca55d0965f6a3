// Small-batch path over a prepared layer: the codebook lives in LDS.
//
// At batch 1 a layer is one pass over its per-edge metadata (paper section 4.2: the
// memory-bound regime) plus one codeword lookup per edge (Eq. (1)).  Lookups that go to L2
// are limited by the rate at which a CU can issue divergent addresses, far below what the
// metadata stream could sustain; lookups in LDS are not.  The 655 KB Int8 codebook does not
// fit the 160 KB LDS of a CU, but an eighth of it does, so the edges are regrouped once
// (kan_vq_prepare) by bucket = idx / 8192 (fp16 and block-floating-point rows: idx / 4096, fp32 rows:
// idx / 2048; half of that for layers
// with more than 2048 inputs) and every workgroup serves one bucket: it copies the bucket's
// codeword rows into LDS, builds the span/basis table of all inputs of its sample there as
// well, and streams its block of the bucket's edges.
//
// Inside a bucket the edges are ordered by output j, then input i.  A workgroup owns the
// block of edges of a run of outputs, reads it flat (thread t holds 8 consecutive edges per
// pass: 16-byte loads whose addresses depend on nothing but the block's first edge), puts the
// per-edge products into LDS and then sums every segment (the edges of one output) with one
// wave in a fixed order; the per-bucket sums are added by the fixed-order reduction kernel
// or by the next bucket layer itself: no atomics on this path, reproducible bits.  (The one
// exception is the side path for non-finite products - a codeword holding Inf or NaN that an
// edge refers to - which counts and places such products with LDS atomics; finite data never
// takes it, and its results are non-finite whatever the order.)
// The bias of an edge needs no lookup at all: the four bases sum to 1 on [-1,1], so
// sum_i bias_ij is a per-output constant computed at preparation time.
//
// This file also holds the column kernel for small prepared layers (one workgroup per output and
// sample, windows gathered from L2, no partial sums) and the preparation kernels (count, scan,
// fill, bias sums, block tables).

#include <type_traits>

#include "kan_device.hpp"
#include "kan_internal.hpp"

namespace kan {
namespace {

constexpr int kWaves = kBucketThreads / kWave;     // 16
constexpr int kEpt = 8;                            // consecutive edges per thread and pass
constexpr int kPass = kBucketThreads * kEpt;       // 8192 edges per workgroup and pass
constexpr int kBadMax = 32;                        // non-finite products of a pass that are placed one by one

// Raw records of one pass: edges e0 .. e0 + 7 of the thread (16-byte loads; the eight gains
// are 32 bytes as fp32 - two loads -, 16 as fp16, 8 as byte codes).  GK is the GbKind.
template <int GK>
struct PassRegs {
  u32x4 i, q;
  typename std::conditional<GK == kGbQ8, u32x2, u32x4>::type g0;
  typename std::conditional<GK == kGbF32, u32x4, char>::type g1;
};

__device__ __forceinline__ float bias_to_float(float b, const Q8Params&) { return b; }
__device__ __forceinline__ float bias_to_float(__half b, const Q8Params&) { return __half2float(b); }
__device__ __forceinline__ float bias_to_float(q8_t b, const Q8Params& qp) { return q8_bias(b.v, qp); }

__device__ __forceinline__ uint32_t dword_of(const u32x4& v, int n) {
  return n == 0 ? v.x : (n == 1 ? v.y : (n == 2 ? v.z : v.w));
}
__device__ __forceinline__ uint32_t u16_of(const u32x4& v, int u) {   // u = 0..7
  const uint32_t w = dword_of(v, u >> 1);
  return (u & 1) ? (w >> 16) : (w & 0xffffu);
}
template <int GK>
__device__ __forceinline__ float gain_of(const PassRegs<GK>& c, int u, const Q8Params& qp) {
  if constexpr (GK == kGbF16) {
    return __half2float(__ushort_as_half((uint16_t)u16_of(c.g0, u)));
  } else if constexpr (GK == kGbQ8) {
    const uint32_t w = u < 4 ? c.g0.x : c.g0.y;
    return q8_gain((w >> (8 * (u & 3))) & 0xffu, qp);
  } else {
    return __uint_as_float(u < 4 ? dword_of(c.g0, u) : dword_of(c.g1, u - 4));
  }
}

// Sum over the 64 lanes of a wave, delivered in lane 63, with data-parallel-primitive moves
// (register crossbar: a few clocks each) instead of LDS permutes (a dependent chain of six
// LDS round trips per segment).  The order of the additions is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false);
  return v + __int_as_float(moved);
}

// Sum over a row of 16 lanes, delivered in every lane of the row.
__device__ __forceinline__ float row_sum(float v) {
  v = dpp_add<0xB1, 0xf>(v);
  v = dpp_add<0x4E, 0xf>(v);
  v = dpp_add<0x141, 0xf>(v);
  v = dpp_add<0x140, 0xf>(v);
  return v;
}

__device__ __forceinline__ float wave_sum_to_last_lane(float v) {
  v = dpp_add<0xB1, 0xf>(v);       // quad_perm [1,0,3,2]: neighbours
  v = dpp_add<0x4E, 0xf>(v);       // quad_perm [2,3,0,1]: every lane holds its quad's sum
  v = dpp_add<0x141, 0xf>(v);      // row_half_mirror: sums of 8
  v = dpp_add<0x140, 0xf>(v);      // row_mirror: every lane holds its row's sum (16 lanes)
  v = dpp_add<0x142, 0xa>(v);      // row_bcast 15 into rows 1 and 3: sums of 32 in rows 1, 3
  v = dpp_add<0x143, 0xc>(v);      // row_bcast 31 into rows 2 and 3: lane 63 holds the sum of 64
  return v;
}

// Every global load below is unconditional (addresses are clamped into valid memory instead
// of being predicated): with no branch around a load the compiler counts outstanding loads
// exactly, so each wait covers only the loads whose data is needed next, and table
// building, record traffic and arithmetic overlap.
//
// MAXIN: inputs the basis table holds (2048 or 4096); the bucket shrinks to make room.
template <int GK, int CODE, int MAXIN>
__global__ __launch_bounds__(kBucketThreads) void kan_bucket_kernel(const BucketArgs a) {
  constexpr int kCbBytes = bucket_bytes(MAXIN);
  // bytes from one bucket's rows to the next's in the codebook: the whole LDS share, except for the 12-byte
  // block-floating-point rows (a power of two of them per bucket: 4096 or 2048)
  constexpr int kCbStride = CODE == kCbBfp8 ? kCbBytes / 20 * 12 : kCbBytes;
  constexpr int kXPerThread = MAXIN / kBucketThreads;
  constexpr int kCbPerThread = (kCbBytes / 16 + kBucketThreads - 1) / kBucketThreads;   // 16-byte units per thread
  __shared__ __attribute__((aligned(16))) uint32_t cb[kCbBytes / 4 + 8];   // + 16 bytes read-ahead, + 16 spare
  __shared__ float4 bas[MAXIN];             // {w0, w1, w2, span as integer bits}; w3 = 1 - w0 - w1 - w2
  __shared__ __attribute__((aligned(16))) float prod[kPass];   // per-edge products of the current pass
  __shared__ float res[kBucketMaxJw];       // sums of this workgroup's segments
  __shared__ uint32_t segl[kBucketMaxJw + 1];   // first edge of every segment of the block (+ end)
  __shared__ int seg_first[2];                  // first segment that reaches into the pass (by pass parity)
  __shared__ float wave_total[kWaves];          // prefix mode: the sum of each wave's 512 products of the pass
  __shared__ int bad_n[2];                      // prefix mode: non-finite products of the pass (by pass parity) ...
  __shared__ uint32_t bad_pos[kBadMax];         // ... their edges ...
  __shared__ float bad_val[kBadMax];            // ... and values: they are added to their own segment only

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int head = blockIdx.z, b = blockIdx.y;
  const BucketHead H = a.h[head];
  const char* prep = (const char*)H.prepared;
  // the block of this workgroup: outputs [j0, j1) of one bucket, edges [blk_lo, blk_hi)
  const uint32_t* __restrict__ ent = (const uint32_t*)(prep + a.off_blk) + (size_t)blockIdx.x * kBucketEntryWords;
  const int bucket = (int)ent[0];
  const int j0 = (int)ent[1], j1 = (int)ent[2];
  const uint32_t blk_lo = ent[3], blk_hi = ent[4];
  const int njw = j1 - j0;
  const uint32_t* __restrict__ seg = (const uint32_t*)(prep + a.off_seg) + (size_t)bucket * a.n_out;
  const uint16_t* __restrict__ pi = (const uint16_t*)(prep + a.off_i);
  const uint16_t* __restrict__ pq = (const uint16_t*)(prep + a.off_q);
  const char* __restrict__ pg = prep + a.off_g;
  constexpr int kGainBytes = gb_bytes(GK);
  const Q8Params qp = {H.gain_log2_lo, H.gain_log2_step, 0.f};


  // Loads are issued in the order their data is needed (they return in order): the inputs
  // of the sample, the codebook bucket, the segment table; then, after the basis table has
  // been built from the inputs, two passes of records.

  // ---- (1) inputs: x itself, or the previous layer's per-bucket sums still to be added
  //          (fixed order) and squashed ----------------------------------------------------
  float xv[kXPerThread];
  {
    const float* xr = a.x + (long long)head * a.x_head_stride + (long long)b * a.n_in;
    int xi[kXPerThread];
#pragma unroll
    for (int r = 0; r < kXPerThread; ++r) {
      xi[r] = min(tid + r * kBucketThreads, a.n_in - 1);
      xv[r] = xr[xi[r]];
    }
    // further slices eight at a time, all their loads in flight together; the additions keep
    // the order p = 1, 2, ... (slices past the last one are re-reads of it, added as zero)
    for (int p0 = 1; p0 < a.x_parts; p0 += 8) {
      float t[8][kXPerThread];
#pragma unroll
      for (int pp = 0; pp < 8; ++pp) {
        const float* xp = xr + (long long)min(p0 + pp, a.x_parts - 1) * a.x_part_stride;
#pragma unroll
        for (int r = 0; r < kXPerThread; ++r) t[pp][r] = xp[xi[r]];
      }
#pragma unroll
      for (int pp = 0; pp < 8; ++pp)
#pragma unroll
        for (int r = 0; r < kXPerThread; ++r) xv[r] += (p0 + pp < a.x_parts) ? t[pp][r] : 0.f;
    }
  }

  // ---- (2) codebook bucket, 16 bytes per thread and round.  The workgroups of a bucket
  //          start at different offsets so that they do not all ask the same L2 channel
  //          for the same line at the same moment ------------------------------------------
  const long long cb_start = (long long)bucket * kCbStride;
  const long long cb_rest = a.cb_bytes - cb_start;
  const int cb_nbytes = (int)(cb_rest < kCbStride ? cb_rest : kCbStride);
  const char* cb_src = (const char*)H.cb + cb_start;
  const int n16 = cb_nbytes >> 4;
  const int cb_tail = cb_nbytes & 15;
  const int rot = (int)((long long)blockIdx.x * n16 / gridDim.x);
  // a bucket shorter than 16 bytes, or without tail bytes: the (unused) load goes to the
  // prepared buffer, which always has that many bytes
  const u32x4* cb_src16 = n16 > 0 ? (const u32x4*)cb_src : (const u32x4*)prep;
  const uint8_t* cb_tailp = cb_tail > 0 ? (const uint8_t*)cb_src + n16 * 16 + min(tid, cb_tail - 1)
                                        : (const uint8_t*)prep;
  // (plain arrays with compile-time indices only; every element is assigned unconditionally,
  // so they live in registers)
  int cbu[kCbPerThread];
  u32x4 cbv[kCbPerThread];
#pragma unroll
  for (int r = 0; r < kCbPerThread; ++r) {
    const int t = tid + r * kBucketThreads;
    int u = t + rot;
    if (u >= n16) u -= n16;
    cbu[r] = t < n16 ? u : kCbBytes / 16;          // no unit: the spare slot behind the bucket
    cbv[r] = cb_src16[t < n16 ? u : 0];
  }
  const uint8_t cb_tailv = *cb_tailp;

  // ---- (3) segment table of the block ---------------------------------------------------------
  const uint32_t sv0 = seg[j0 + min(tid, njw)];
  const uint32_t sv1 = seg[j0 + min(tid + kBucketThreads, njw)];

  __builtin_amdgcn_sched_barrier(0);   // keep the loads above in this order, ahead of their uses

  // ---- span + weights of every input -> LDS ---------------------------------------------------
  {
#pragma unroll
    for (int r = 0; r < kXPerThread; ++r) {
      if (r * kBucketThreads < a.n_in) {        // uniform: rounds past the last input are skipped
        const int i = tid + r * kBucketThreads;
        const float xin = a.x_tanh ? tanhf(xv[r]) : xv[r];
        const BasisW w = basis_eval_rule(xin, a.rule);
        // (threads past the last input of the round write entries nobody reads)
        bas[i] = make_float4(w.w0, w.w1, w.w2, __uint_as_float((uint32_t)w.span));
      }
    }
  }
  // ---- (4) records (their addresses need the block's bounds, two dependent scalar loads that
  //          have had the basis evaluation above to arrive).  Pass p covers edges
  //          [base + p * 8192, + 8192), base = blk_lo rounded down to a multiple of 8, so that
  //          every thread's group of 8 is 16-byte aligned.
  //          Groups past the block re-read its last group; the arrays are padded, so a group
  //          that straddles the end of the last block stays inside the buffer. -----------------
  const uint32_t base = blk_lo & ~7u;
  const uint32_t last_group = blk_hi > 0u ? (blk_hi - 1u) & ~7u : 0u;
  const int n_pass = blk_hi > blk_lo ? (int)((blk_hi - base + kPass - 1) / kPass) : 0;
  auto load_pass = [&](PassRegs<GK>& c, int p) {
    const uint32_t e0 = min(base + (uint32_t)p * kPass + (uint32_t)tid * kEpt, last_group);
    c.i = __builtin_nontemporal_load((const u32x4*)(pi + e0));
    c.q = __builtin_nontemporal_load((const u32x4*)(pq + e0));
    if constexpr (GK == kGbQ8) c.g0 = __builtin_nontemporal_load((const u32x2*)(pg + (size_t)e0 * kGainBytes));
    else c.g0 = __builtin_nontemporal_load((const u32x4*)(pg + (size_t)e0 * kGainBytes));
    if constexpr (GK == kGbF32) c.g1 = __builtin_nontemporal_load((const u32x4*)(pg + (size_t)e0 * kGainBytes) + 1);
  };
  PassRegs<GK> A, B;
  load_pass(A, 0);
  load_pass(B, 1);

  __builtin_amdgcn_sched_barrier(0);

  // ---- codebook rows, segment table -> LDS (unconditional stores: a store inside a branch
  //      would pull its load into the branch, behind all the others) ------------------------------
  {
#pragma unroll
    for (int r = 0; r < kCbPerThread; ++r) ((u32x4*)cb)[cbu[r]] = cbv[r];
    ((uint8_t*)cb)[tid < cb_tail ? n16 * 16 + tid : kCbBytes + 16 + (tid & 15)] = cb_tailv;
  }
  segl[min(tid, njw)] = sv0;
  segl[min(tid + kBucketThreads, njw)] = sv1;
  for (int t = tid; t < njw; t += kBucketThreads) res[t] = 0.f;
  if (tid < 2) bad_n[tid] = 0;
  __syncthreads();

  // Segment sums, two ways.  Long segments (more than 512 edges on the block's average): a whole
  // wave adds one segment's products.  Shorter ones: the products of a pass are turned into
  // running sums over each wave's 512 edges (eight per thread, then a scan across the lanes),
  // and a segment's sum is the difference of the running sums at its two ends, plus whole
  // waves in between: one thread per segment, three dependent LDS reads instead of a chain
  // per group of lanes.  Both ways add in a fixed order.
  const uint32_t avg_len_x = blk_hi - blk_lo;                               // compared with len * njw: uniform
  const bool use_prefix = avg_len_x <= 512u * (uint32_t)njw;
  // products of the thread's 8 edges of pass p -> prod
  auto products = [&](const PassRegs<GK>& c, int p) {
    // edge e belongs to the block iff blk_lo <= e < blk_hi, i.e. (e - blk_lo) < (blk_hi - blk_lo) unsigned
    const uint32_t rel0 = base + (uint32_t)p * kPass + (uint32_t)tid * kEpt - blk_lo, len = blk_hi - blk_lo;
    float pr[kEpt];
#pragma unroll
    for (int u = 0; u < kEpt; ++u) pr[u] = 0.f;
    // Groups wholly outside the block (past its end in the last pass) skip the lookups.  The
    // group holds an edge of the block iff rel0 + u < len for some u in 0..7; rel0 is "negative"
    // (wrapped, -7..-1) only for the group that straddles the block's start, and adding 7 to
    // both sides covers that case as well.
    if (rel0 + (uint32_t)(kEpt - 1) < len + (uint32_t)(kEpt - 1)) {
#pragma unroll
    for (int u = 0; u < kEpt; ++u) {
      const float4 w = bas[u16_of(c.i, u)];
      const uint32_t at = u16_of(c.q, u) * (CODE == kCbBfp8 ? 12u : 10u) + __float_as_uint(w.w);
      float c0, c1, c2, c3;
      if constexpr (CODE == kCbI8 || CODE == kCbBfp8) {
        // bytes at .. at+3 of the bucket: two aligned dwords, funnel-shifted; q + 128 as
        // unsigned bytes (the differences below do not see the offset)
        const uint32_t lo = cb[at >> 2], hi = cb[(at >> 2) + 1];
        const uint32_t win = __builtin_amdgcn_alignbyte(hi, lo, at & 3u) ^ 0x80808080u;
        c0 = (float)(win & 0xffu);
        c1 = (float)((win >> 8) & 0xffu);
        c2 = (float)((win >> 16) & 0xffu);
        c3 = (float)(win >> 24);
      } else if constexpr (CODE == kCbF16) {
        // halves at .. at+3 of the bucket (8 bytes from byte 2 * at): three aligned dwords,
        // funnel-shifted by 0 or 2 bytes
        const uint32_t d = at >> 1, sh = (at & 1u) * 2u;
        const uint32_t w0 = __builtin_amdgcn_alignbyte(cb[d + 1], cb[d], sh);
        const uint32_t w1 = __builtin_amdgcn_alignbyte(cb[d + 2], cb[d + 1], sh);
        c0 = half_bits_to_float(w0 & 0xffffu);
        c1 = half_bits_to_float(w0 >> 16);
        c2 = half_bits_to_float(w1 & 0xffffu);
        c3 = half_bits_to_float(w1 >> 16);
      } else {
        const float* cf = (const float*)cb;
        c0 = cf[at];
        c1 = cf[at + 1];
        c2 = cf[at + 2];
        c3 = cf[at + 3];
      }
      // sum_k w_k c_k with w3 = 1 - w0 - w1 - w2 (the bases sum to 1)
      float s = (CODE == kCbI8 || CODE == kCbBfp8) ? c3 - 128.0f : c3;
      s = fmaf(w.z, c2 - c3, s);
      s = fmaf(w.y, c1 - c3, s);
      s = fmaf(w.x, c0 - c3, s);
      if constexpr (CODE == kCbBfp8) s *= bfp8_row_scale(cb[u16_of(c.q, u) * 3u + 2u]);     // the row's own power of two
      // Edges outside the block (groups that straddle its ends, re-read groups) contribute
      // an exact zero rather than gain * s, so that a non-finite codeword which no edge of
      // the block refers to cannot reach a sum.
      pr[u] = (rel0 + (uint32_t)u < len) ? gain_of<GK>(c, u, qp) * s : 0.f;
    }
    }
    if (use_prefix) {
      float run[kEpt];                    // running sums of the thread's eight products
      run[0] = pr[0];
#pragma unroll
      for (int u = 1; u < kEpt; ++u) run[u] = run[u - 1] + pr[u];
      // A running sum would carry a non-finite product (a codeword with an Inf or NaN that an
      // edge does refer to) into the segments behind it: such products are set aside.  The
      // thread's total is finite iff all its eight products are.
      if (!__builtin_isfinite(run[kEpt - 1])) {
        float keep = 0.f;
#pragma unroll
        for (int u = 0; u < kEpt; ++u) {
          if (__builtin_isfinite(pr[u])) {
            keep += pr[u];
          } else {
            const int k = atomicAdd(&bad_n[p & 1], 1);
            if (k < kBadMax) {
              bad_pos[k] = base + (uint32_t)p * kPass + (uint32_t)tid * kEpt + (uint32_t)u;
              bad_val[k] = pr[u];
            }
          }
          run[u] = keep;
        }
      }
#pragma unroll
      for (int u = 0; u < kEpt; ++u) pr[u] = run[u];
      float v = pr[kEpt - 1];            // inclusive scan of the threads' totals over the wave
      v = dpp_add<0x111, 0xf>(v);        // row_shr 1, 2, 4, 8: within rows of 16 lanes
      v = dpp_add<0x112, 0xf>(v);
      v = dpp_add<0x114, 0xf>(v);
      v = dpp_add<0x118, 0xf>(v);
      v = dpp_add<0x142, 0xa>(v);        // row_bcast 15: rows 1 and 3 add the total of the row before
      v = dpp_add<0x143, 0xc>(v);        // row_bcast 31: rows 2 and 3 add the total of the first half
      const float before = __shfl_up(v, 1, 64);
      const float ex = lane == 0 ? 0.f : before;
#pragma unroll
      for (int u = 0; u < kEpt; ++u) pr[u] += ex;
      if (lane == kWave - 1) wave_total[wave] = v;
    }
    ((float4*)prod)[tid * 2] = make_float4(pr[0], pr[1], pr[2], pr[3]);
    ((float4*)prod)[tid * 2 + 1] = make_float4(pr[4], pr[5], pr[6], pr[7]);
    // The first segment that ends after the start of the pass: thread t answers for segment t
    // (exactly one does), so that the sums below visit only the segments of the pass and a
    // block of 1024 short segments does not walk all of them in every pass.
    const uint32_t pa = base + (uint32_t)p * kPass;
    if (tid < njw && segl[tid + 1] > pa && (tid == 0 || segl[tid] <= pa)) seg_first[p & 1] = tid;
  };

  auto segment_sums = [&](int p) {
    const uint32_t pa = base + (uint32_t)p * kPass;        // prod[n] is edge pa + n
    if (use_prefix) {
      for (int jj = seg_first[p & 1] + tid; jj < njw; jj += kBucketThreads) {
        const uint32_t s0 = segl[jj], s1 = segl[jj + 1];
        if (s0 >= pa + (uint32_t)kPass) break;             // in order: the rest lies behind the pass
        const uint32_t lo = max(s0, pa) - pa, hi = min(s1, pa + (uint32_t)kPass) - pa;
        if (lo < hi) {
          const int wl = (int)(lo >> 9), wh = (int)((hi - 1) >> 9);       // 512 products per wave
          float sum = prod[hi - 1];
          for (int w = wh - 1; w >= wl; --w) sum += wave_total[w];        // whole waves, and the first wave's total
          if (lo & 511u) sum -= prod[lo - 1];
          res[jj] += sum;
        }
      }
      const int nb = bad_n[p & 1];                          // (uniform; almost always 0)
      if (nb > 0) {
        __syncthreads();                                    // the sums above are in res
        if (nb > kBadMax) {                                 // too many to place: the whole block is not a number
          for (int t = tid; t < njw; t += kBucketThreads) res[t] = __builtin_nanf("");
        } else if (tid < nb) {
          const uint32_t e = bad_pos[tid];                  // its segment: segl[jj] <= e < segl[jj + 1]
          int lo_j = 0, hi_j = njw;
          while (hi_j - lo_j > 1) {
            const int mid = (lo_j + hi_j) >> 1;
            if (segl[mid] <= e) lo_j = mid; else hi_j = mid;
          }
          atomicAdd(&res[lo_j], bad_val[tid]);
        }
        __syncthreads();
        if (tid == 0) bad_n[p & 1] = 0;                     // next written two passes on, behind two barriers
      }
      return;
    }
    // a whole wave per segment; wave w takes segments w, w + 16, ... of the pass
    constexpr int group_shift = 6;
    const int glanes = 1 << group_shift, per_wave = kWave >> group_shift;
    const int grp = lane >> group_shift, gl = lane & (glanes - 1);
    for (int jj = seg_first[p & 1] + wave * per_wave + grp; jj < njw; jj += kWaves * per_wave) {
      const uint32_t s0 = segl[jj], s1 = segl[jj + 1];
      if (s0 >= pa + (uint32_t)kPass) break;               // in order: the rest lies behind the pass (the groups of a wave leave one by one)
      const uint32_t lo = max(s0, pa), hi = min(s1, pa + (uint32_t)kPass);
      float acc = 0.f;
      for (uint32_t e = lo + (uint32_t)gl; e < hi; e += (uint32_t)glanes) acc += prod[e - pa];
      acc = row_sum(acc);                                   // every lane: the sum of its row of 16
      if (group_shift >= 5) acc = dpp_add<0x142, 0xa>(acc); // rows 1 and 3: the sum of their half wave
      if (group_shift == 6) acc = dpp_add<0x143, 0xc>(acc); // row 3: the sum of the wave
      if (gl == glanes - 1 && lo < hi) res[jj] += acc;
    }
  };

  // two passes are always in flight: a slot is refilled as soon as it has been consumed
  // (after the last pass the refills are harmless re-reads)
  for (int p = 0; p < n_pass; p += 2) {
    products(A, p);
    load_pass(A, p + 2);
    __syncthreads();
    segment_sums(p);
    __syncthreads();
    if (p + 1 >= n_pass) break;
    products(B, p + 1);
    load_pass(B, p + 3);
    __syncthreads();
    segment_sums(p + 1);
    __syncthreads();
  }

  // ---- segment sums -> memory (coalesced): scale, bias sum (first bucket only), activation ----
  float* dst = a.dst + (long long)head * a.dst_head_stride + (long long)bucket * a.dst_chunk_stride +
               (long long)b * a.n_out;
  const float* bias_sum = (const float*)(prep + a.off_bias);
  const float scale = CODE == kCbI8 ? H.scale : 1.0f;
  for (int t = tid; t < njw; t += kBucketThreads) {
    float v = scale * res[t] + (bucket == 0 ? bias_sum[j0 + t] : 0.0f);
    if (a.apply_tanh && a.n_buckets == 1) v = tanhf(v);
    dst[j0 + t] = v;
  }
}

// ---- column kernel: small prepared layers ------------------------------------------------
// A layer of a few hundred thousand edges gives a bucket workgroup a thousand edges or fewer:
// what it does then is wait - for 80 KB of codeword rows to reach its LDS, for its block
// bounds, for a reduction launch behind it.  Such a layer is served by one workgroup per
// (output j, sample) instead.  The prepared buffer of a small layer also holds ids and gains
// transposed ([output][input]), so thread t owns inputs t, t + 256, ... of the sample: it loads
// x, id and gain of its edges at once (coalesced, nothing depends on anything), evaluates the
// basis of its own inputs, fetches each edge's four-coefficient window straight from the
// codebook in L2 (Eq. (1); a thousand gathers per CU are a microsecond) and adds the products
// in a fixed order: per thread by ascending input, then across the lanes, then the waves.
// It writes the finished output - bias sum, activation - so no reduction pass follows.
// PER: edges per thread and round, 8 (2048 inputs per round) or 4 for layers of at most 1024 inputs, whose
// upper four slots would only re-read the last input (the address units see every load, used or not).

template <int GK, typename CbT, int PER>
__global__ __launch_bounds__(kColumnThreads) void kan_column_kernel(const BucketArgs a) {
  __shared__ float wave_sum[kColumnThreads / kWave];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int j = blockIdx.x, b = blockIdx.y, head = blockIdx.z;
  const BucketHead H = a.h[head];
  const char* prep = (const char*)H.prepared;
  constexpr int kGainBytes = gb_bytes(GK);
  const uint32_t* __restrict__ ti = (const uint32_t*)(prep + a.off_ti) + (size_t)j * a.n_in;
  const char* __restrict__ tg = prep + a.off_tg + (size_t)j * a.n_in * kGainBytes;
  const Q8Params qp = {H.gain_log2_lo, H.gain_log2_step, 0.f};
  const CbT* __restrict__ cbk = (const CbT*)H.cb;
  const float* xr = a.x + (long long)head * a.x_head_stride + (long long)b * a.n_in;
  const float bias_sum = ((const float*)(prep + a.off_bias))[j];

  float acc = 0.f;
  for (int i0 = 0; i0 < a.n_in; i0 += kColumnThreads * PER) {       // one round for up to 256 * PER inputs
    // ---- everything the round needs from memory except the windows: unconditional loads,
    //      clamped addresses (inputs past the end re-read the last one and count as zero) ----
    int xi[PER];
    float xv[PER], gain[PER];
    uint32_t row[PER];
#pragma unroll
    for (int r = 0; r < PER; ++r) {
      xi[r] = min(i0 + tid + r * kColumnThreads, a.n_in - 1);
      xv[r] = xr[xi[r]];
      row[r] = ti[xi[r]];
      if constexpr (GK == kGbF16) gain[r] = __half2float(((const __half*)tg)[xi[r]]);
      else if constexpr (GK == kGbQ8) gain[r] = q8_gain(((const uint8_t*)tg)[xi[r]], qp);
      else gain[r] = ((const float*)tg)[xi[r]];
    }
    // the input is x itself, or the previous layer's per-bucket sums still to be added (in order) and squashed
    for (int p0 = 1; p0 < a.x_parts; p0 += 8) {
      float t[8][PER];
#pragma unroll
      for (int pp = 0; pp < 8; ++pp) {
        const float* xp = xr + (long long)min(p0 + pp, a.x_parts - 1) * a.x_part_stride;
#pragma unroll
        for (int r = 0; r < PER; ++r) t[pp][r] = xp[xi[r]];
      }
#pragma unroll
      for (int pp = 0; pp < 8; ++pp)
#pragma unroll
        for (int r = 0; r < PER; ++r) xv[r] += (p0 + pp < a.x_parts) ? t[pp][r] : 0.f;
    }
    // ---- basis of the thread's own inputs, then the windows of its edges ----------------------
    BasisW w[PER];
    typename WindowRaw<CbT>::type raw[PER];
#pragma unroll
    for (int r = 0; r < PER; ++r) {
      w[r] = basis_eval_rule(a.x_tanh ? tanhf(xv[r]) : xv[r], a.rule);
      raw[r] = load_window<CbT>(cbk, row[r], w[r].span);
    }
#pragma unroll
    for (int r = 0; r < PER; ++r) {
      float c[4];
      dequant_window<CbT>(raw[r], 1.0f, c);
      // sum_k w_k c_k with w3 = 1 - w0 - w1 - w2 (the bases sum to 1)
      float sv = c[3];
      sv = fmaf(w[r].w2, c[2] - c[3], sv);
      sv = fmaf(w[r].w1, c[1] - c[3], sv);
      sv = fmaf(w[r].w0, c[0] - c[3], sv);
      acc += (i0 + tid + r * kColumnThreads < a.n_in) ? gain[r] * sv : 0.f;
    }
  }
  acc = wave_sum_to_last_lane(acc);
  if (lane == kWave - 1) wave_sum[wave] = acc;
  __syncthreads();
  if (tid == 0) {
    const float scale = sizeof(CbT) == 1 ? H.scale : 1.0f;
    float v = scale * ((wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3])) + bias_sum;
    if (a.apply_tanh) v = tanhf(v);
    a.dst[(long long)head * a.dst_head_stride + (long long)b * a.n_out + j] = v;
  }
}

// ---- preparation ------------------------------------------------------------------------
// The regrouping is a counting sort of the edges by (bucket, output j), input i ascending
// inside a run, and at the same time a transposition: the layer stores consecutive outputs side
// by side, the prepared layout consecutive inputs.  It is done tile by tile (kPrepareRows inputs x
// kPrepareCols outputs per workgroup), so that both the reads (rows of the tile) and the writes
// (runs of one (bucket, output) within the tile's row block) move whole runs of bytes:
//   count   per tile: edges per (bucket, output) -> tcnt[row block][bucket][output] and, added
//           up over the row blocks with integer atomics, the segment lengths; bias sums per
//           (row block, output) in fp64
//   scan    exclusive prefix over the segment lengths (bucket-major) -> segment table
//   fill    per tile: the tile's idx and gain staged in LDS; a wave takes a column, and for
//           every 64 rows ranks its lanes within their bucket (ballots) behind the edges of the
//           earlier row blocks and rows
//   bias    per output: the row blocks' sums added in order, rounded once to fp32

template <typename IdxT, typename GbT>
__global__ __launch_bounds__(256) void kan_prepare_count_kernel(const IdxT* __restrict__ idx,
                                                                const GbT* __restrict__ bias, int n_in, int n_out,
                                                                int rows_shift, int n_buckets,
                                                                uint32_t* __restrict__ seg, uint16_t* __restrict__ tcnt,
                                                                double* __restrict__ tbias, Q8Params qp) {
  extern __shared__ uint32_t cnt[];                 // [n_buckets][kPrepareCols]
  __shared__ double bsum[4][kPrepareCols];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * kPrepareCols + lane;
  const int i0 = blockIdx.y * kPrepareRows + wave * (kPrepareRows / 4);
  for (int t = threadIdx.x; t < n_buckets * kPrepareCols; t += 256) cnt[t] = 0u;
  __syncthreads();
  double bs = 0.0;
  if (j < n_out) {
    const int i1 = min(i0 + kPrepareRows / 4, n_in);
    for (int i = i0; i < i1; ++i) {
      const size_t e = (size_t)i * n_out + j;
      const uint32_t b = min((uint32_t)idx[e] >> rows_shift, (uint32_t)(n_buckets - 1));
      atomicAdd(&cnt[b * kPrepareCols + lane], 1u);            // (waves share a column: integer, order-free)
      bs += (double)bias_to_float(bias[e], qp);
    }
  }
  bsum[wave][lane] = bs;
  __syncthreads();
  for (int t = threadIdx.x; t < n_buckets * kPrepareCols; t += 256) {
    const int b = t / kPrepareCols, jj = blockIdx.x * kPrepareCols + (t % kPrepareCols);
    if (jj < n_out) {
      const uint32_t c = cnt[t];
      tcnt[((size_t)blockIdx.y * n_buckets + b) * n_out + jj] = (uint16_t)c;
      if (c) atomicAdd(&seg[(size_t)b * n_out + jj], c);
    }
  }
  if (wave == 0 && j < n_out)
    tbias[(size_t)blockIdx.y * n_out + j] = ((bsum[0][lane] + bsum[1][lane]) + bsum[2][lane]) + bsum[3][lane];
}

__global__ __launch_bounds__(256) void kan_prepare_zero_kernel(uint32_t* __restrict__ p, long long n) {
  for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += (long long)gridDim.x * blockDim.x) p[t] = 0u;
}

__global__ __launch_bounds__(256) void kan_prepare_bias_kernel(const double* __restrict__ tbias, int n_row_blocks, int n_out,
                                                               float* __restrict__ bias_sum) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n_out) return;
  double s = 0.0;
  for (int r = 0; r < n_row_blocks; ++r) s += tbias[(size_t)r * n_out + j];
  bias_sum[j] = (float)s;
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

template <typename IdxT, typename GbT>
__global__ __launch_bounds__(256) void kan_prepare_fill_kernel(const IdxT* __restrict__ idx, const GbT* __restrict__ gain,
                                                               int n_in, int n_out, int rows_shift, int n_buckets,
                                                               const uint32_t* __restrict__ seg,
                                                               const uint16_t* __restrict__ tcnt,
                                                               uint16_t* __restrict__ pi, uint16_t* __restrict__ pq,
                                                               GbT* __restrict__ pg, uint32_t* __restrict__ ti,
                                                               GbT* __restrict__ tgo) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  // tile of ids and gains, [row][column], then the running position of every bucket, one table per wave
  IdxT* tid_ = (IdxT*)lds_raw;
  GbT* tg = (GbT*)(lds_raw + (size_t)kPrepareRows * kPrepareCols * sizeof(IdxT));
  uint32_t* base = (uint32_t*)(lds_raw + (size_t)kPrepareRows * kPrepareCols * (sizeof(IdxT) + sizeof(GbT)));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j0 = blockIdx.x * kPrepareCols, i0 = blockIdx.y * kPrepareRows;
  const int rows = min(kPrepareRows, n_in - i0), cols = min(kPrepareCols, n_out - j0);
  for (int r = wave; r < rows; r += 4) {                     // a wave reads a row of the tile
    if (lane < cols) {
      const size_t e = (size_t)(i0 + r) * n_out + j0 + lane;
      tid_[r * kPrepareCols + lane] = idx[e];
      tg[r * kPrepareCols + lane] = gain[e];
    }
  }
  __syncthreads();
  uint32_t* wbase = base + (size_t)wave * n_buckets;
  const uint32_t mask = (1u << rows_shift) - 1u;
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int c = wave; c < cols; c += 4) {                     // a wave takes a column
    const int j = j0 + c;
    // where this row block's edges of (bucket, j) start: the segment's start plus the earlier row blocks
    for (int b = lane; b < n_buckets; b += 64) {
      uint32_t at = seg[(size_t)b * n_out + j];
      for (int rb = 0; rb < (int)blockIdx.y; ++rb) at += tcnt[((size_t)rb * n_buckets + b) * n_out + j];
      wbase[b] = at;
    }
    __builtin_amdgcn_wave_barrier();
    for (int r0 = 0; r0 < rows; r0 += 64) {
      const int r = r0 + lane;
      const bool live = r < rows;
      const uint32_t id = live ? (uint32_t)tid_[r * kPrepareCols + c] : 0u;
      if (ti && live) {        // small layers: ids and gains once more, the inputs of an output side by side
        ti[(size_t)j * n_in + i0 + r] = id;
        tgo[(size_t)j * n_in + i0 + r] = tg[r * kPrepareCols + c];
      }
      const uint32_t b = min(id >> rows_shift, (uint32_t)(n_buckets - 1));
      unsigned long long todo = __ballot(live);
      uint32_t pos = 0;
      while (todo) {                                         // one round per bucket present among the 64 rows
        const int first = __ffsll((long long)todo) - 1;
        const uint32_t kb = __shfl(b, first);
        const unsigned long long same = __ballot(live && b == kb) & todo;
        const uint32_t start = wbase[kb];
        if (live && b == kb) pos = start + (uint32_t)__popcll(same & lt);
        __builtin_amdgcn_wave_barrier();
        if (lane == first) wbase[kb] = start + (uint32_t)__popcll(same);
        __builtin_amdgcn_wave_barrier();
        todo &= ~same;
      }
      if (live) {
        pi[pos] = (uint16_t)(i0 + r);
        pq[pos] = (uint16_t)(id & mask);
        pg[pos] = tg[r * kPrepareCols + c];
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// Blocks per bucket for a table of W blocks (prefix sums -> cnt[0 .. n_buckets]): every bucket
// gets min_blocks, the rest goes in proportion to the edges (cumulative rounding).
__global__ void kan_prepare_block_counts_kernel(const uint32_t* __restrict__ seg, int n_out, int n_buckets,
                                                int min_blocks, int W, uint32_t* __restrict__ cnt) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  const unsigned long long E = seg[(size_t)n_buckets * n_out];
  const unsigned long long spare = (unsigned long long)(W - (long long)n_buckets * min_blocks);
  unsigned long long given = 0;
  uint32_t run = 0;
  cnt[0] = 0;
  for (int b = 0; b < n_buckets; ++b) {
    const unsigned long long upto = seg[(size_t)(b + 1) * n_out];          // edges of buckets 0..b
    const unsigned long long target = E > 0 ? (spare * upto + E / 2) / E : 0;
    run += (uint32_t)min_blocks + (uint32_t)(target - given);
    given = target;
    cnt[b + 1] = run;
  }
}

// The entries of one bucket (thread = bucket): its outputs are cut into its blocks so that
// the blocks hold about equal numbers of edges, never more than kBucketMaxJw outputs each
// (the cuts are made one after the other so that the limit holds for every block).
//
// Where a block sits in the table decides its XCD (workgroups go to the 8 XCDs in turn): the
// bucket-sorted list of blocks is dealt out in 8 contiguous runs, run x taking the positions
// x, x + 8, ..., so that an XCD serves few buckets and its L2 holds only their rows (with 8
// equal buckets: one bucket per XCD, the codebook crosses the fabric once).
__device__ __forceinline__ int bucket_table_position(int s, int W) {
  const int base = W >> 3, rem = W & 7;
  int x = 0, start = 0;
  while (x < 7) {
    const int c = base + (x < rem ? 1 : 0);
    if (s < start + c) break;
    start += c;
    ++x;
  }
  return (s - start) * 8 + x;
}

__global__ __launch_bounds__(256) void kan_prepare_blocks_kernel(const uint32_t* __restrict__ seg, int n_out,
                                                                 int n_buckets, const uint32_t* __restrict__ cnt,
                                                                 uint32_t* __restrict__ table) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= n_buckets) return;
  const int W = (int)cnt[n_buckets];
  const int first = (int)cnt[b], nb = (int)(cnt[b + 1] - cnt[b]);
  const uint32_t* sb = seg + (size_t)b * n_out;     // sb[0 .. n_out] are valid (the prefix runs on)
  const unsigned long long e0 = sb[0], eb = sb[n_out] - sb[0];
  int j0 = 0;
  for (int q = 0; q < nb; ++q) {
    int j1 = n_out;
    if (q + 1 < nb) {
      const unsigned long long target = e0 + eb * (unsigned long long)(q + 1) / (unsigned long long)nb;
      int a = 0, c = n_out;                          // smallest j with sb[j] >= target
      while (a < c) {
        const int mid = (a + c) >> 1;
        if (sb[mid] >= target) c = mid; else a = mid + 1;
      }
      const int lo_c = max(j0, n_out - (nb - q - 1) * kBucketMaxJw);   // the blocks after this one can take the rest
      const int hi_c = min(j0 + kBucketMaxJw, n_out);
      j1 = min(max(a, lo_c), hi_c);
    }
    uint32_t* e = table + (size_t)bucket_table_position(first + q, W) * kBucketEntryWords;
    e[0] = (uint32_t)b;
    e[1] = (uint32_t)j0;
    e[2] = (uint32_t)j1;
    e[3] = sb[j0];
    e[4] = sb[j1];
    e[5] = e[6] = e[7] = 0u;
    j0 = j1;
  }
}

template <typename IdxT, typename GbT>
hipError_t prepare_typed(const LayerPtrs& h, int n_in, int n_out, const BucketGeom& g, void* prepared,
                         hipStream_t s) {
  char* p = (char*)prepared;
  uint32_t* seg = (uint32_t*)(p + g.off_seg);
  uint16_t* tcnt = (uint16_t*)(p + g.off_tcnt);
  double* tbias = (double*)(p + g.off_tbias);
  const long long n_seg = (long long)g.n_buckets * n_out;
  const Q8Params qp = {h.gain_log2_lo, h.gain_log2_step, h.bias_scale};
  dim3 grid((unsigned)((n_out + kPrepareCols - 1) / kPrepareCols), (unsigned)g.n_row_blocks);
  const size_t lds_count = (size_t)g.n_buckets * kPrepareCols * sizeof(uint32_t);
  const size_t lds_fill = (size_t)kPrepareRows * kPrepareCols * (sizeof(IdxT) + sizeof(GbT)) + (size_t)4 * g.n_buckets * sizeof(uint32_t);
  if (lds_count > 64 * 1024 || lds_fill > 150 * 1024) return hipErrorInvalidValue;     // (n_buckets <= 256 fits)
  // (dynamic LDS beyond 64 KB has to be asked for; the tile of 4-byte ids and 4-byte gains takes 128 KB)
  hipError_t err = hipFuncSetAttribute((const void*)kan_prepare_fill_kernel<IdxT, GbT>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_fill);
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(kan_prepare_zero_kernel, dim3((unsigned)((n_seg + 1 + 255) / 256 > 1024 ? 1024 : (n_seg + 1 + 255) / 256)),
                     dim3(256), 0, s, seg, n_seg + 1);
  hipLaunchKernelGGL((kan_prepare_count_kernel<IdxT, GbT>), grid, dim3(256), lds_count, s, (const IdxT*)h.idx,
                     (const GbT*)h.bias, n_in, n_out, g.rows_shift, g.n_buckets, seg, tcnt, tbias, qp);
  hipLaunchKernelGGL(kan_prepare_scan_kernel, dim3(1), dim3(1024), 0, s, seg, n_seg);
  hipLaunchKernelGGL((kan_prepare_fill_kernel<IdxT, GbT>), grid, dim3(256), lds_fill, s, (const IdxT*)h.idx,
                     (const GbT*)h.gain, n_in, n_out, g.rows_shift, g.n_buckets, (const uint32_t*)seg,
                     (const uint16_t*)tcnt, (uint16_t*)(p + g.off_i), (uint16_t*)(p + g.off_q), (GbT*)(p + g.off_g),
                     g.off_ti ? (uint32_t*)(p + g.off_ti) : nullptr, g.off_tg ? (GbT*)(p + g.off_tg) : nullptr);
  hipLaunchKernelGGL(kan_prepare_bias_kernel, dim3((unsigned)((n_out + 255) / 256)), dim3(256), 0, s, (const double*)tbias,
                     g.n_row_blocks, n_out, (float*)(p + g.off_bias));
  const int min_blocks = (n_out + kBucketMaxJw - 1) / kBucketMaxJw;
  for (int t = 0; t < kBucketTables; ++t) {
    uint32_t* cnt = (uint32_t*)(p + g.off_cnt) + (size_t)t * (g.n_buckets + 1);
    uint32_t* table = (uint32_t*)(p + g.off_blk) + (size_t)g.tab_first[t] * kBucketEntryWords;
    hipLaunchKernelGGL(kan_prepare_block_counts_kernel, dim3(1), dim3(64), 0, s, (const uint32_t*)seg, n_out,
                       g.n_buckets, min_blocks, g.tab_w[t], cnt);
    hipLaunchKernelGGL(kan_prepare_blocks_kernel, dim3((unsigned)((g.n_buckets + 255) / 256)), dim3(256), 0, s,
                       (const uint32_t*)seg, n_out, g.n_buckets, (const uint32_t*)cnt, table);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bucket_prepare(const LayerPtrs& h, int idx_u32, int gb_kind, int n_in, int n_out,
                                 const BucketGeom& g, void* prepared, hipStream_t s) {
  if (idx_u32) {
    if (gb_kind == kGbQ8) return prepare_typed<uint32_t, q8_t>(h, n_in, n_out, g, prepared, s);
    if (gb_kind == kGbF16) return prepare_typed<uint32_t, __half>(h, n_in, n_out, g, prepared, s);
    return prepare_typed<uint32_t, float>(h, n_in, n_out, g, prepared, s);
  }
  if (gb_kind == kGbQ8) return prepare_typed<uint16_t, q8_t>(h, n_in, n_out, g, prepared, s);
  if (gb_kind == kGbF16) return prepare_typed<uint16_t, __half>(h, n_in, n_out, g, prepared, s);
  return prepare_typed<uint16_t, float>(h, n_in, n_out, g, prepared, s);
}

hipError_t launch_bucket(int code, int gb_kind, const BucketArgs& a, int blocks, int heads, hipStream_t s) {
  if (a.n_in > kBucketMaxIn || a.n_buckets < 1 || blocks < a.n_buckets) return hipErrorInvalidValue;
  if (code != kCbI8 && code != kCbF16 && code != kCbF32 && code != kCbBfp8) return hipErrorInvalidValue;
  if (gb_kind == kGbQ8 && code != kCbI8) return hipErrorInvalidValue;      // byte-coded gains go with Int8 codebooks
  dim3 grid((unsigned)blocks, (unsigned)a.B, (unsigned)heads);
  dim3 block(kBucketThreads);
  const bool wide = a.n_in > 2048;
#define KAN_LAUNCH_BUCKET(GK, CODE)                                                                    \
  do {                                                                                                 \
    if (wide) hipLaunchKernelGGL((kan_bucket_kernel<GK, CODE, 4096>), grid, block, 0, s, a);           \
    else hipLaunchKernelGGL((kan_bucket_kernel<GK, CODE, 2048>), grid, block, 0, s, a);                \
  } while (0)
  if (code == kCbI8) {
    if (gb_kind == kGbQ8) KAN_LAUNCH_BUCKET(kGbQ8, kCbI8);
    else if (gb_kind == kGbF16) KAN_LAUNCH_BUCKET(kGbF16, kCbI8);
    else KAN_LAUNCH_BUCKET(kGbF32, kCbI8);
  } else if (code == kCbF16) {
    if (gb_kind == kGbF16) KAN_LAUNCH_BUCKET(kGbF16, kCbF16);
    else KAN_LAUNCH_BUCKET(kGbF32, kCbF16);
  } else if (code == kCbBfp8) {
    if (gb_kind == kGbF16) KAN_LAUNCH_BUCKET(kGbF16, kCbBfp8);
    else KAN_LAUNCH_BUCKET(kGbF32, kCbBfp8);
  } else {
    if (gb_kind == kGbF16) KAN_LAUNCH_BUCKET(kGbF16, kCbF32);
    else KAN_LAUNCH_BUCKET(kGbF32, kCbF32);
  }
#undef KAN_LAUNCH_BUCKET
  return hipGetLastError();
}

hipError_t launch_column(int code, int gb_kind, const BucketArgs& a, int heads, hipStream_t s) {
  if ((long long)a.n_in * a.n_out > kColumnMaxEdges || a.off_ti <= 0 || a.off_tg <= 0) return hipErrorInvalidValue;
  if (code != kCbI8 && code != kCbF16 && code != kCbF32 && code != kCbBfp8) return hipErrorInvalidValue;
  if (gb_kind == kGbQ8 && code != kCbI8) return hipErrorInvalidValue;
  dim3 grid((unsigned)a.n_out, (unsigned)a.B, (unsigned)heads);
  dim3 block(kColumnThreads);
#define KAN_LAUNCH_COLUMN(GK, CB)                                                                                  \
  do {                                                                                                             \
    if (a.n_in <= 4 * kColumnThreads) hipLaunchKernelGGL((kan_column_kernel<GK, CB, 4>), grid, block, 0, s, a);    \
    else hipLaunchKernelGGL((kan_column_kernel<GK, CB, 8>), grid, block, 0, s, a);                                 \
  } while (0)
  if (code == kCbI8) {
    if (gb_kind == kGbQ8) KAN_LAUNCH_COLUMN(kGbQ8, int8_t);
    else if (gb_kind == kGbF16) KAN_LAUNCH_COLUMN(kGbF16, int8_t);
    else KAN_LAUNCH_COLUMN(kGbF32, int8_t);
  } else if (code == kCbF16) {
    if (gb_kind == kGbF16) KAN_LAUNCH_COLUMN(kGbF16, __half);
    else KAN_LAUNCH_COLUMN(kGbF32, __half);
  } else if (code == kCbBfp8) {
    if (gb_kind == kGbF16) KAN_LAUNCH_COLUMN(kGbF16, bfp8_t);
    else KAN_LAUNCH_COLUMN(kGbF32, bfp8_t);
  } else {
    if (gb_kind == kGbF16) KAN_LAUNCH_COLUMN(kGbF16, float);
    else KAN_LAUNCH_COLUMN(kGbF32, float);
  }
#undef KAN_LAUNCH_COLUMN
  return hipGetLastError();
}

}  // namespace kan
