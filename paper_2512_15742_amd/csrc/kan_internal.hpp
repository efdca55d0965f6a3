// Host-side structures shared by the dispatcher (kan_api.hip) and the kernel
// translation units.  Nothing here is part of the public C-ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kan {

constexpr int kMaxGroup = 64;   // heads per grouped launch (descriptor table lives in kernarg)

// Pointers of one layer of one head (device pointers).  For the dense baseline
// `cb` points at coef[in][out][10] and the other three are unused.
struct LayerPtrs {
  const void* idx;
  const void* gain;
  const void* bias;
  const void* cb;
  float scale;
  float gain_log2_lo, gain_log2_step, bias_scale;   // byte-coded gain/bias only
};

enum CodeKind : int { kCbF32 = 0, kCbI8 = 1, kDense = 2, kCbF16 = 3, kCbBfp8 = 4 };
constexpr int cb_row_bytes(int code) { return code == kCbI8 ? 10 : (code == kCbF16 ? 20 : (code == kCbBfp8 ? 12 : 40)); }
enum GbKind : int { kGbF32 = 0, kGbF16 = 1, kGbQ8 = 2 };     // fp32, fp16, one byte each (log gain, linear bias)
constexpr int gb_bytes(int kind) { return kind == kGbF32 ? 4 : (kind == kGbF16 ? 2 : 1); }

// ---- gather path (fp32 vector arithmetic) --------------------------------------
struct GatherCfg {
  int bt;          // batch tile: 1, 4 or 16 samples per workgroup
  int jpl;         // consecutive outputs per lane: 1, 2, 4 or 8
  int wj;          // waves of the 4-wave workgroup laid along j (1, 2 or 4); 4/wj along i
  int idx_u32;     // 0: uint16 indices, 1: uint32
  int gb_kind;     // GbKind of gain/bias
  int code;        // CodeKind
};

struct GatherArgs {
  const float* x;              // [heads or 1][B][n_in]
  long long x_head_stride;     // elements between heads; 0 when all heads share x
  float* dst;                  // y, hidden activation, or partial sums
  long long dst_head_stride;   // elements
  long long dst_chunk_stride;  // elements between i-chunks (partials); unused when n_chunks == 1
  int n_in, n_out, B;
  int rows_per_chunk;          // i-rows per workgroup (multiple of 4/wj)
  int n_jt;                    // j-tiles; blockIdx.x = bt_index * n_jt + jt
  int apply_tanh;              // only honoured when the kernel writes final values
  long long cb_bytes;          // codebook bytes per head (0: no L2 warm-up of the codebook)
  int rule;                    // edge function: 0 cubic B-spline, 1 two-tap linear interpolation
  // Chained input (VQ layers at batch tile 1 only): x is the previous layer's partial sums,
  // [head][x_parts][B][n_in]; a workgroup adds the slices of its own rows in a fixed order and
  // squashes them (x_tanh) while it builds its basis data.
  int x_parts;                 // 0 or 1: plain x
  long long x_part_stride;
  int x_tanh;
  LayerPtrs h[kMaxGroup];
};
constexpr int kGatherChainMaxParts = 256;

hipError_t launch_gather_bt1(const GatherCfg&, const GatherArgs&, dim3 grid, hipStream_t);
hipError_t launch_gather_bt4(const GatherCfg&, const GatherArgs&, dim3 grid, hipStream_t);
hipError_t launch_gather_bt16(const GatherCfg&, const GatherArgs&, dim3 grid, hipStream_t);

// ---- matrix-core path (fp16 operands, fp32 accumulate) ----------------------------
constexpr int kMfmaPrepRows = 32;   // input rows per partial bias sum (and per prep workgroup)

struct PrepCoefArgs {
  uint4* cf;                   // coefficient fragments, [head][step][5][2][2][n_out] records of 16 bytes
  uint4* cf_lo;                // split form: the low parts (c - fp16(c)) * 2048 in the same layout; null otherwise
  long long cf_head_stride;    // in records
  float* bias_partial;         // [head][ceil(n_in / 32)][n_out]
  long long bp_head_stride;    // in floats
  int n_in, n_out;
  LayerPtrs h[kMaxGroup];
};

// One launch for all a single head's call can prepare before its first contraction: the
// coefficient records of up to kStartJobs matrix-core layers of the same storage types, and
// the basis words of the first layer's input.
constexpr int kStartJobs = 4;
struct PrepStartArgs {
  int n_jobs;
  int first_block[kStartJobs + 1];   // filled by the launcher: job k takes blocks first_block[k] .. first_block[k+1]-1,
                                     // the basis job those from first_block[n_jobs] on
  struct Job {
    uint4* cf;
    uint4* cf_lo;                    // split form only
    float* bp;
    int n_in, n_out;
    int nx;                          // filled by the launcher: blocks along the outputs
    LayerPtrs h;
  } job[kStartJobs];
  const float* x;                    // [B][n_in] of the first layer
  uint2* W;
  uint2* W_lo;                       // split form only
  int n_in, B, rule;
  int basis_nx;                      // filled by the launcher
};

struct MfmaArgs {
  const uint4* cf;
  long long cf_head_stride;
  const uint2* W;              // packed basis weights + span, [head or 1][n_in][B]
  long long w_head_stride;     // 0 when all heads share the input
  const float* bias_partial;
  long long bp_head_stride;
  int bias_on;                 // 0: this launch adds no bias sums (the dense baseline has none)
  // Split form (passes == 3): the low parts of both operands; the kernel runs its steps three
  // times, (W, cf_lo), (W_lo, cf), then scales the sums by lo_scale and goes on with (W, cf).
  int passes;                  // 1 or 3
  const uint4* cf_lo;
  const uint2* W_lo;
  float lo_scale;              // 1 / 2048: the factor the low parts carry
  float* dst;
  long long dst_head_stride, dst_chunk_stride;
  int n_in, n_out, B;
  int rows_per_chunk;          // multiple of kMfmaPrepRows
  int n_jt;
  int apply_tanh;
  float scale[kMaxGroup];      // Int8 scale per head (1 for fp32 codebooks)
};

// Workgroups of that launch (its grid is one-dimensional: at most 2^24 - 1 workgroups of 256 threads).
inline long long prep_start_blocks(const PrepStartArgs& a) {
  long long blocks = (long long)((a.n_in + 31) / 32) * ((a.B + 31) / 32);
  for (int k = 0; k < a.n_jobs; ++k)
    blocks += (long long)((a.job[k].n_out + 63) / 64) * ((a.job[k].n_in + kMfmaPrepRows - 1) / kMfmaPrepRows);
  return blocks;
}
constexpr long long kPrepStartMaxBlocks = (1ll << 24) - 1;
hipError_t launch_prep_start(const GatherCfg&, PrepStartArgs&, bool split, hipStream_t);
hipError_t launch_prep_coef(const GatherCfg&, const PrepCoefArgs&, int heads, hipStream_t);
// Dense fp32 coefficients coef[n_in][n_out][10] into the split form (high and low fp16 records).
hipError_t launch_prep_dense(const float* coef, uint4* cf, uint4* cf_lo, int n_in, int n_out, hipStream_t);
// The input of the layer is x, or act(sum of x_parts slices of x) when the previous layer left
// its partial sums (slices x_part_stride elements apart).
// W_lo (split form, else null): the low parts (w - hi) * 2048 of the weights, hi = w cut to fp16 towards zero.
hipError_t launch_prep_basis(const float* x, long long x_head_stride, int x_parts, long long x_part_stride,
                             int x_tanh, uint2* W, uint2* W_lo, long long w_head_stride, int n_in, int B, int heads,
                             int rule, hipStream_t);
hipError_t launch_mfma(const MfmaArgs&, int tile_m, int tile_n, dim3 grid, hipStream_t);   // samples (64 | 128) x outputs (128; 256 with 128 samples) per tile

// ---- fused gather + matrix-core kernel (batch tiles of 32 or 64 samples) --------------
constexpr int kFusedTileN = 128;      // outputs per workgroup

struct FusedArgs {
  const float* x;              // [head or 1][B][n_in]
  long long x_head_stride;     // 0 when all heads share the input
  float* dst;
  long long dst_head_stride, dst_chunk_stride;
  int n_in, n_out, B;
  int rows_per_chunk;          // multiple of 8
  int n_jt;                    // output tiles; blockIdx.x = batch_tile * n_jt + jt
  int apply_tanh;
  int rule;                    // edge function: 0 cubic B-spline, 1 two-tap linear interpolation
  // Chained input (launch_fused_chained only): x is the previous layer's partial sums,
  // [head][x_parts][B][n_in]; a workgroup adds the slices of its own inputs in a fixed order
  // and squashes them (x_tanh) before its first step.
  int x_parts;                 // 0 or 1: plain x
  long long x_part_stride;
  int x_tanh;
  LayerPtrs h[kMaxGroup];
};

hipError_t launch_fused(const GatherCfg&, const FusedArgs&, bool f32, dim3 grid, hipStream_t);
// The same kernels for tiles of 32 samples whose input is still in slices (x_parts > 1).  The
// chunk's inputs are kept in LDS: 32 * rows_per_chunk floats of dynamic shared memory, at most
// kFusedChainFloats; n_in and rows_per_chunk are multiples of four (16-byte loads).
constexpr int kFusedChainFloats = 2048;
constexpr int kFusedChainMaxParts = 64;
hipError_t launch_fused_chained(const GatherCfg&, const FusedArgs&, bool f32, dim3 grid, hipStream_t);

// ---- bucketed small-batch path (prepared layers) ----------------------------------
// A prepared layer holds its edges regrouped by codebook bucket (a run of consecutive
// codewords whose rows fit in LDS) and, inside a bucket, by output j then input i; a
// segment is the run of edges of one (bucket, j).  Per edge it keeps the input index, the
// codeword id relative to the bucket and the gain; the biases of an output are summed once
// (the bases sum to 1, so they do not depend on x).
constexpr int kBucketMaxIn = 4096;      // the basis table of all inputs lives in LDS beside the bucket
constexpr int kBucketThreads = 1024;
constexpr int kBucketMaxJw = 1024;      // outputs per workgroup (their sums are staged in LDS)
// Codebook bytes per bucket: 8192 Int8, 4096 fp16 or 2048 fp32 rows for layers of up to 2048
// inputs, half of that for wider layers (whose basis table takes twice the LDS); 4096 (2048)
// block-floating-point rows of 12 bytes use 48 (24) KB of it.
constexpr int bucket_bytes(int n_in) { return n_in > 2048 ? 40960 : 81920; }
// The preparation regroups a layer tile by tile: kPrepareRows inputs x kPrepareCols outputs per workgroup.
constexpr int kPrepareRows = 256;
constexpr int kPrepareCols = 64;

// Workgroups of a launch are laid out by block tables made at preparation time: a block is a
// run of outputs of one bucket, and the outputs of a bucket are cut so that the blocks of a
// table hold about the same number of edges whatever the histogram of the codewords is (a
// bucket gets blocks in proportion to its edges, at least ceil(n_out / kBucketMaxJw), so an
// empty bucket still writes its zeros).  Table t < 4 serves (samples x heads) = t + 1 with
// about 256 / (t + 1) blocks, table 4 every larger product with the fewest blocks allowed.
constexpr int kBucketWorkgroups = 256;  // one workgroup of 1024 threads per CU
constexpr int kBucketTables = 5;
constexpr int kBucketEntryWords = 8;    // {bucket, first output, end output, first edge, end edge, 0, 0, 0}

// Small prepared layers: one workgroup per (output, sample) reads the output's inputs side by side from a
// transposed copy of ids and gains in the prepared buffer, gathers the windows from L2 and writes the
// finished output (no bucket copies, no partial sums, no reduction launch).
constexpr long long kColumnMaxEdges = 1ll << 20;
constexpr int kColumnThreads = 256;

struct BucketGeom {
  int rows_shift;      // log2(codewords per bucket)
  int n_buckets;
  size_t off_seg;      // uint32 [n_buckets * n_out + 1] first edge of every segment
  size_t off_bias;     // float  [n_out]                 sum over i of bias_ij
  size_t off_i;        // uint16 [E]                     input index
  size_t off_q;        // uint16 [E]                     codeword id - first id of the bucket
  size_t off_g;        // gain   [E]                     in the layer's gain dtype
  size_t off_blk;      // uint32 [sum of tab_w][8]       block tables, one after the other
  size_t off_cnt;      // uint32 [kBucketTables][n_buckets + 1]  blocks per bucket (prefix sums), scratch of the preparation
  size_t off_tcnt;     // uint16 [row blocks][n_buckets][n_out]  edges per (row block, bucket, output), scratch of the preparation
  size_t off_tbias;    // double [row blocks][n_out]             bias sums per row block, scratch of the preparation
  size_t off_ti;       // uint32 [n_out][n_in]   small layers only (at most kColumnMaxEdges edges, else 0): codeword ids ...
  size_t off_tg;       // gain   [n_out][n_in]   ... and gains with the inputs of an output side by side (column kernel)
  int n_row_blocks;    // row blocks of kPrepareRows inputs
  int tab_w[kBucketTables];        // blocks of every table
  int tab_first[kBucketTables];    // first entry of every table
  size_t total;
};

inline int bucket_table_for(long long samples_times_heads) {
  return samples_times_heads <= 4 ? (int)(samples_times_heads < 1 ? 1 : samples_times_heads) - 1 : kBucketTables - 1;
}

inline BucketGeom bucket_geometry(int n_in, int n_out, int K, int code, int gb_kind) {
  // 32 bytes of slack after every array: threads load aligned groups of eight records
  auto up = [](size_t v) { return (v + 32 + 255) / 256 * 256; };
  BucketGeom g;
  // (block-floating-point rows: 4096 rows of 12 bytes, 48 KB of the 80 KB a bucket may take)
  g.rows_shift = (code == kCbI8 ? 13 : ((code == kCbF16 || code == kCbBfp8) ? 12 : 11)) - (n_in > 2048 ? 1 : 0);
  g.n_buckets = (K + (1 << g.rows_shift) - 1) >> g.rows_shift;
  const size_t E = (size_t)n_in * n_out;
  g.off_seg = 0;
  g.off_bias = up(((size_t)g.n_buckets * n_out + 1) * 4);
  g.off_i = g.off_bias + up((size_t)n_out * 4);
  g.off_q = g.off_i + up(E * 2);
  g.off_g = g.off_q + up(E * 2);
  g.off_blk = g.off_g + up(E * gb_bytes(gb_kind));
  const long long w_min = (long long)g.n_buckets * ((n_out + kBucketMaxJw - 1) / kBucketMaxJw);
  long long entries = 0;
  for (int t = 0; t < kBucketTables; ++t) {
    long long w = t + 1 < kBucketTables ? kBucketWorkgroups / (t + 1) : w_min;
    if (w < w_min) w = w_min;
    g.tab_w[t] = (int)w;
    g.tab_first[t] = (int)entries;
    entries += w;
  }
  g.off_cnt = g.off_blk + up((size_t)entries * kBucketEntryWords * 4);
  g.n_row_blocks = (n_in + kPrepareRows - 1) / kPrepareRows;
  g.off_tcnt = g.off_cnt + up((size_t)kBucketTables * ((size_t)g.n_buckets + 1) * 4);
  g.off_tbias = g.off_tcnt + up((size_t)g.n_row_blocks * g.n_buckets * n_out * 2);
  g.total = g.off_tbias + up((size_t)g.n_row_blocks * n_out * 8);
  g.off_ti = g.off_tg = 0;
  if ((long long)E <= kColumnMaxEdges) {
    g.off_ti = g.total;
    g.off_tg = g.off_ti + up(E * 4);
    g.total = g.off_tg + up(E * gb_bytes(gb_kind));
  }
  return g;
}

struct BucketHead {
  const void* prepared;
  const void* cb;
  float scale;
  float gain_log2_lo, gain_log2_step;     // byte-coded gains only
  int pad;
};

struct BucketArgs {
  const float* x;              // [head or 1][x_parts][B][n_in]
  long long x_head_stride;     // 0 when all heads share the input
  long long x_part_stride;     // the input of the layer is act(sum over x_parts slices of x): the
  int x_parts, x_tanh;         //   previous layer's per-bucket sums are consumed without a reduction pass
  float* dst;                  // final values (one bucket) or per-bucket partial sums
  long long dst_head_stride, dst_chunk_stride;
  int n_in, n_out, B;
  int n_buckets;               // blockIdx.x = entry of the block table at off_blk
  int rows_shift;
  long long cb_bytes;          // whole codebook, bytes
  int apply_tanh;              // honoured only when n_buckets == 1
  int rule;                    // edge function: 0 cubic B-spline, 1 two-tap linear interpolation
  long long off_seg, off_bias, off_i, off_q, off_g;
  long long off_ti, off_tg;    // column kernel: transposed ids and gains
  long long off_blk;           // byte offset of the block table this launch uses
  BucketHead h[kMaxGroup];
};

hipError_t launch_bucket(int code, int gb_kind, const BucketArgs&, int blocks, int heads, hipStream_t);
hipError_t launch_column(int code, int gb_kind, const BucketArgs&, int heads, hipStream_t);
// One-time regrouping of a layer into the layout above (three kernels: count, scan, fill).
hipError_t launch_bucket_prepare(const LayerPtrs&, int idx_u32, int gb_kind, int n_in, int n_out,
                                 const BucketGeom&, void* prepared, hipStream_t);

// ---- compression-side assignment (nearest codebook shape per edge) ---------------------------
size_t assign_centroid_bytes(int K);       // prepared centroid operands (workspace)
int recon_blocks(long long E);             // workgroups of the reconstruction-sums pass
hipError_t launch_assign(const float* coef, long long E, const float* cb, int K, int idx_u32, void* idx,
                         float* gain, float* bias, void* ws, hipStream_t);
hipError_t launch_recon_sums(const float* coef, long long E, const float* cb, int idx_u32, const void* idx,
                             const float* gain, const float* bias, double* part, double* sums, hipStream_t);

// ---- reduction of i-chunk partial sums ------------------------------------------
// dst[n] = act( sum_c partial[c * chunk_stride + n] ), n < count, for every head.
hipError_t launch_reduce(const float* partial, long long head_stride, long long chunk_stride,
                         int n_chunks, float* dst, long long dst_head_stride, long long count,
                         int n_heads, int apply_tanh, hipStream_t);

// ---- debug / parity kernels -------------------------------------------------------
hipError_t launch_basis(const float* x, long long n, uint8_t* span, float* w, hipStream_t);
hipError_t launch_pli_basis(const float* x, long long n, uint8_t* index, float* w, hipStream_t);
hipError_t launch_basis_window(const float* x, long long n, int rule, int fast, uint8_t* start, float* w, hipStream_t);
hipError_t launch_debug_gather(const LayerPtrs&, int idx_u32, int code, long long edges,
                               uint32_t* ids, float* rows, hipStream_t);
hipError_t launch_count_bad(const void* idx, int idx_u32, long long edges, uint32_t K,
                            uint32_t* count, hipStream_t);
// range[0], range[1] = smallest nonzero and largest |gain * codeword entry| over the layer
hipError_t launch_coef_range(const LayerPtrs&, int idx_u32, int gb_kind, int code, long long edges, float* range,
                             hipStream_t);

}  // namespace kan
