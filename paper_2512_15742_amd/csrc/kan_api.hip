// C-ABI of the library (include/kan.h): host-side validation, launch planning
// and dispatch.  All arithmetic of the method runs in the kernels; this file
// only decides which kernels run, with what grid, and where their scratch data
// lives inside the caller's workspace.

#include "../../include/kan.h"

#include <hip/hip_runtime.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "kan_internal.hpp"

// Scratch memory of kan_vq_head_forward_static: one array per GPU, held from the moment the
// library's code is loaded on that GPU until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress; the address the kernels get is looked up per device.
static __device__ __align__(256) unsigned char scratch[KAN_STATIC_SCRATCH_BYTES];

namespace kan {
namespace {

// Device address of `scratch` on the current device (looked up on the first call per device).
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

kan_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return KAN_ERR_LAUNCH;
  if (dev < 0 || dev >= kMaxDevices) return KAN_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KAN_ERR_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return KAN_OK;
}

// ---- per-kernel event timing ---------------------------------------------------
struct Prof {
  bool on = false;
  int cap = 0, n = 0;
  std::vector<hipEvent_t> ev;
  std::vector<const char*> names;
  std::vector<int> layer;     // 1-based layer of a head call the launch belongs to, 0: none
  int cur_layer = 0;
} g_prof;

template <typename F>
kan_status run(const char* name, hipStream_t s, F&& f) {
  hipError_t err;
  if (g_prof.on && g_prof.n < g_prof.cap) {
    const int n = g_prof.n++;
    g_prof.names[n] = name;
    g_prof.layer[n] = g_prof.cur_layer;
    (void)hipEventRecord(g_prof.ev[2 * n], s);
    err = f();
    (void)hipEventRecord(g_prof.ev[2 * n + 1], s);
  } else {
    err = f();
  }
  return err == hipSuccess ? KAN_OK : KAN_ERR_LAUNCH;
}

// ---- validation ------------------------------------------------------------------
constexpr int64_t kMaxDim = 1 << 20;
constexpr int64_t kMaxBatch = 1 << 24;

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int gb_kind_of(const kan_vq_layer& L) {
  return L.gb_dtype == KAN_F32 ? kGbF32 : (L.gb_dtype == KAN_F16 ? kGbF16 : kGbQ8);
}

int code_of(const kan_vq_layer& L) {
  return L.cb_dtype == KAN_I8 ? kCbI8 : (L.cb_dtype == KAN_F16 ? kCbF16 : (L.cb_dtype == KAN_BFP8 ? kCbBfp8 : kCbF32));
}

kan_status validate_layer(const kan_vq_layer* L) {
  if (!L) return KAN_ERR_NULL;
  if (L->G != 10 || L->degree != 3) return KAN_ERR_UNSUPPORTED;
  if (L->rule != KAN_RULE_BSPLINE3 && L->rule != KAN_RULE_PLI2) return KAN_ERR_UNSUPPORTED;
  if (L->in < 1 || L->out < 1 || L->in > kMaxDim || L->out > kMaxDim || L->K < 1) return KAN_ERR_SHAPE;
  if (L->idx_dtype != KAN_U16 && L->idx_dtype != KAN_U32) return KAN_ERR_DTYPE;
  if (L->gb_dtype != KAN_F32 && L->gb_dtype != KAN_F16 && L->gb_dtype != KAN_Q8) return KAN_ERR_DTYPE;
  if (L->cb_dtype != KAN_F32 && L->cb_dtype != KAN_F16 && L->cb_dtype != KAN_I8 && L->cb_dtype != KAN_BFP8) return KAN_ERR_DTYPE;
  if (L->idx_dtype == KAN_U16 && L->K > 65536) return KAN_ERR_SHAPE;
  // byte-coded gain/bias belong to the fully quantised format: one-byte codebook entries too
  if (L->gb_dtype == KAN_Q8 && L->cb_dtype != KAN_I8) return KAN_ERR_UNSUPPORTED;
  if (L->flags & ~KAN_LAYER_NO_COLUMN) return KAN_ERR_UNSUPPORTED;
  if (!L->idx || !L->gain || !L->bias || !L->codebook) return KAN_ERR_NULL;
  const size_t idx_sz = L->idx_dtype == KAN_U16 ? 2 : 4;
  const size_t gb_sz = L->gb_dtype == KAN_F32 ? 4 : (L->gb_dtype == KAN_F16 ? 2 : 1);
  if (!aligned(L->idx, idx_sz) || !aligned(L->gain, gb_sz) || !aligned(L->bias, gb_sz)) return KAN_ERR_SHAPE;
  if (!aligned(L->codebook, L->cb_dtype == KAN_F32 ? 8 : (L->cb_dtype == KAN_I8 ? 2 : 4))) return KAN_ERR_SHAPE;
  return KAN_OK;
}

// ---- planning -----------------------------------------------------------------------
// Everything below is a pure function of shapes, dtypes, batch, head count and
// pointer alignment, so the workspace query and the forward call always agree.

enum PlanKind { kPlanGather = 0, kPlanMfma = 1, kPlanFused16 = 2, kPlanFused32 = 3, kPlanBucket = 4, kPlanColumn = 5 };

struct LayerPlan {
  GatherCfg cfg;
  int n_jt, n_bt, n_chunks, rows_per_chunk;
  int tile_n = 0;              // matrix-core path: outputs per workgroup tile (128: four waves, 256: eight)
  int kind;          // PlanKind
  bool mfma;         // kind == kPlanMfma (coefficient + basis preparation, streaming contraction)
  int products = 1;  // 3: both operands in high and low fp16 parts, hi*hi + hi*lo + lo*hi (three passes inside the kernel)
  const char* name;
};

constexpr int kTargetWorkgroups = 512;    // two workgroups of 4 waves per CU
constexpr int kEnoughWorkgroups = 384;

// Geometry for one choice of outputs-per-lane.  The four waves of a workgroup are
// interleaved along i whenever the layer has rows for them (their sums meet in LDS), so a
// workgroup spans 64*jpl outputs and parallelism comes from output tiles first; i is split
// into chunks only as far as the partial sums stay small next to the parameter stream
// (n_chunks * B * out * 4 bytes <= a quarter of in * out * bytes_per_edge).
void gather_geometry(LayerPlan& p, int n_in, int n_out, int64_t B, int n_heads, int jpl, int bytes_per_edge) {
  p.cfg.jpl = jpl;
  const int lanes_j = (n_out + jpl - 1) / jpl;
  p.cfg.wj = n_in >= 16 ? 1 : (lanes_j > 128 ? 4 : (lanes_j > 64 ? 2 : 1));
  const int wi = 4 / p.cfg.wj;
  p.n_jt = (lanes_j + 64 * p.cfg.wj - 1) / (64 * p.cfg.wj);
  p.n_bt = (int)((B + p.cfg.bt - 1) / p.cfg.bt);
  const long long base = (long long)n_heads * p.n_jt * p.n_bt;
  long long chunks = (kTargetWorkgroups + base - 1) / (base > 0 ? base : 1);
  const int rows_per_wave = p.cfg.bt == 1 ? 4 : 2;
  const long long max_by_rows = n_in / (wi * rows_per_wave);
  const long long max_by_bytes = (long long)n_in * bytes_per_edge / (16 * (B > 0 ? B : 1));
  if (chunks > max_by_rows) chunks = max_by_rows;
  if (chunks > max_by_bytes) chunks = max_by_bytes;
  if (chunks < 1) chunks = 1;
  int rows = (int)((n_in + chunks - 1) / chunks);
  rows = (rows + wi - 1) / wi * wi;
  p.rows_per_chunk = rows;
  p.n_chunks = (n_in + rows - 1) / rows;
}

LayerPlan plan_gather(int n_in, int n_out, int64_t B, int n_heads, int idx_u32, int gb_kind, int code,
                      bool vec_ok) {
  LayerPlan p;
  p.mfma = false;
  p.kind = kPlanGather;
  p.cfg.idx_u32 = idx_u32;
  p.cfg.gb_kind = gb_kind;
  p.cfg.code = code;
  p.cfg.bt = B <= 1 ? 1 : (B <= 4 ? 4 : 16);
  p.name = p.cfg.bt == 1 ? "kan_gather_bt1" : (p.cfg.bt == 4 ? "kan_gather_bt4" : "kan_gather_bt16");
  const int bytes_per_edge = code == kDense ? 40 : (idx_u32 ? 4 : 2) + 2 * gb_bytes(gb_kind);
  const int jpl_max = p.cfg.bt == 16 ? 4 : 8;
  // Widest per-lane vector that divides the row and still gives the chip enough workgroups;
  // narrower vectors mean more output tiles (load width does not matter to the stream).
  int best = 1;
  long long best_wgs = -1;
  for (int c = vec_ok ? jpl_max : 1; c >= 1; c >>= 1) {
    if (n_out % c != 0 || (c > 1 && n_out / c < 64)) continue;
    gather_geometry(p, n_in, n_out, B, n_heads, c, bytes_per_edge);
    const long long wgs = (long long)n_heads * p.n_jt * p.n_bt * p.n_chunks;
    if (wgs >= kEnoughWorkgroups) { best = c; break; }
    if (wgs > best_wgs) { best = c; best_wgs = wgs; }
  }
  gather_geometry(p, n_in, n_out, B, n_heads, best, bytes_per_edge);
  return p;
}

// Matrix-core path: tiles of 64 or 128 samples x 128 outputs (128 x 256 for eight waves), i split so that
// every CU has two workgroups of four waves (or one of eight).
constexpr int kMfmaTileN = 128;
constexpr int kMfmaRowsStep = kMfmaPrepRows;   // chunk boundaries coincide with partial bias sums
constexpr int kMfmaTargetWorkgroups = 512;
constexpr int kMfmaMinRows = 64;
constexpr int kMfmaMaxSteps = 256;            // steps of 16 inputs per workgroup of the streaming contraction
constexpr int64_t kHalfFusedMaxBatch = 64;   // fp16 path: fused kernel up to here, streaming contraction above
constexpr int64_t kFusedTwoTilesMaxBatch = 128;            // ... and up to here (both paths) for layers of at least
constexpr long long kFusedTwoTilesMinEdges = 1ll << 22;    // this many edges whose codeword rows are one gather each
constexpr long long kFusedMinEdgesForResidency = 1 << 17;   // ... for layers of at least this many edges per head
constexpr long long kFusedSmallLayerEdges = 1 << 19;   // fused kernel: layers up to here may write partial sums as large as their stream
constexpr int kFusedMinWgsPerHead = 20;      // fused kernel, several heads: workgroups per head (L2 residency of the codebooks)
// Precise path: from this batch on the split-operand matrix-core form.  Its time hardly depends on
// the batch below 128 (config 3: 96 us, config 2: 44 us) while the fused fp32 kernel's doubles with
// its second tile of 64 samples (config 3: 97 us at 64, 113 at 80; config 2: 33 and 57).
constexpr int64_t kSplitMinBatch = 65;
// The dense baseline's switch from its fp32 FMA kernel (config 2's twin: 35 us at batch 16, 54 at 24;
// the split form 35-37 us anywhere below batch 64).
constexpr int64_t kDenseSplitMinBatch = 17;
constexpr int64_t kAutoMfmaBatch = 32;    // KAN_PATH_AUTO switches to the matrix cores from here (measured crossover 16-32)

LayerPlan plan_mfma(int n_in, int n_out, int64_t B, int n_heads, int idx_u32, int gb_kind, int code, bool split3 = false) {
  LayerPlan p;
  p.mfma = true;
  p.kind = kPlanMfma;
  p.name = "kan_mfma";
  p.cfg.jpl = 1;
  p.cfg.wj = 1;
  p.cfg.idx_u32 = idx_u32;
  p.cfg.gb_kind = gb_kind;
  p.cfg.code = code;
  const long long max_chunks = n_in / kMfmaMinRows;
  // Tiles of 128 outputs by 128 samples (half the coefficient bytes per MFMA through the
  // vector cache), unless their grid would need more than eight chunks of inputs to give
  // every CU two workgroups (64-sample tiles then halve the chunks and with them the
  // partial sums written and read back), or would be padded with many more empty rows.
  p.n_jt = (n_out + kMfmaTileN - 1) / kMfmaTileN;
  const long long big = (long long)n_heads * p.n_jt * ((B + 127) / 128);
  const long long rows128 = (B + 127) / 128 * 128, rows64 = (B + 63) / 64 * 64;     // sample rows the tiles cover
  p.cfg.bt = (big * 8 >= kMfmaTargetWorkgroups && rows128 * 10 <= rows64 * 11) ? 128 : 64;
  p.n_bt = (int)((B + p.cfg.bt - 1) / p.cfg.bt);
  // 128-sample tiles come 256 outputs wide, for one workgroup of eight waves per CU instead of two of four:
  // the eight waves read one Phi tile, so it is built (and its basis words are loaded) once per CU and step, not
  // twice (config 3 at batch 1024: layer 1 43.3 -> 38.2 us, at 4096 139 -> 121.6; config 5 2.22 -> 2.01 ms; the
  // split form at batch 1024 103 -> 89.6 us), unless the wider tiles would pad the outputs by more than an eighth.
  p.tile_n = kMfmaTileN;
  if (p.cfg.bt == 128 && (long long)((n_out + 255) / 256 * 256) * 8 <= (long long)p.n_jt * kMfmaTileN * 9) {
    p.tile_n = 2 * kMfmaTileN;
    p.n_jt = (n_out + p.tile_n - 1) / p.tile_n;
  }
  const long long base = (long long)n_heads * p.n_jt * p.n_bt * (p.tile_n / kMfmaTileN);   // in workgroups of four waves
  long long chunks = kMfmaTargetWorkgroups / (base > 0 ? base : 1);
  // A workgroup that lives for hundreds of steps drifts away from the others of its XCD, which work on
  // the same rows and columns of the operands, by more steps than that XCD's L2 holds: operands are then
  // fetched again and again (config 5 with patches of 8 x 8 tiles and 256 steps: 15 GB for 0.6 GB of
  // operands, L2 hit rate 46 %, 2.56 ms; capped at 128 steps 2.27 ms + 65 us for the reduction).  With the
  // patches of 32 sample tiles x 2 output tiles the kernel uses now (64 workgroups share two slices of the
  // coefficient records, the larger operand) the uncapped form is the faster one: 2.50 against 2.62 ms per
  // step, no partial sums, no reduction.  The cap remains for layers of more than 4096 inputs.
  const long long by_steps = ((n_in + 15) / 16 + kMfmaMaxSteps - 1) / kMfmaMaxSteps;
  if (chunks < by_steps) chunks = by_steps;
  if (chunks > max_chunks) chunks = max_chunks;
  if (chunks < 1) chunks = 1;
  int rows = (int)((n_in + chunks - 1) / chunks);
  rows = (rows + kMfmaRowsStep - 1) / kMfmaRowsStep * kMfmaRowsStep;
  p.rows_per_chunk = rows;
  p.n_chunks = (n_in + rows - 1) / rows;
  if (split3) {
    p.products = 3;
    p.name = "kan_mfma_split";
  }
  return p;
}

// Fused gather + matrix-core kernel: batch tiles of 32 (B <= 32) or 64 samples, output tiles
// of 128.  With one batch tile every edge is gathered once and the work is bound by the
// gather rate of the CUs' address units, so every CU should be busy: i is split while the
// partial sums stay below the size of the parameter stream.
LayerPlan plan_fused(int n_in, int n_out, int64_t B, int n_heads, int idx_u32, int gb_kind, int code, bool f32) {
  LayerPlan p;
  p.mfma = false;
  p.kind = f32 ? kPlanFused32 : kPlanFused16;
  p.name = f32 ? "kan_fused_f32" : "kan_fused_f16";
  p.cfg.bt = B <= 32 ? 32 : 64;
  p.cfg.jpl = 1;
  p.cfg.wj = 4;
  p.cfg.idx_u32 = idx_u32;
  p.cfg.gb_kind = gb_kind;
  p.cfg.code = code;
  p.n_jt = (n_out + kFusedTileN - 1) / kFusedTileN;
  p.n_bt = (int)((B + p.cfg.bt - 1) / p.cfg.bt);
  const int bytes_per_edge = (idx_u32 ? 4 : 2) + 2 * gb_bytes(gb_kind);
  const long long base = (long long)n_heads * p.n_jt * p.n_bt;
  // (64-sample tiles: with a workgroup per CU and twice the steps each, the metadata of the next
  // steps is in flight behind the gathers of the current one: config 3 at batch 64 57.8 -> 51.1 us
  // on the fp16 path, 96.7 -> 82.9 us on the precise path; 32-sample tiles are better off with two)
  // Two per CU again where the chunks stay long even so: at least 8 steps each for the precise form
  // (4096 x 4096 with K = 262,144 at batch 64: 338 -> 249 us; 4096 x 1024: 67.6 -> 56.5; 2048 x 2048:
  // 65.6 -> 56.2; 8192 x 512: 67.6 -> 60.4), at least 16 for the fp16 form (4096 x 4096: 124 -> 119 us;
  // with 8 steps each it loses: 4096 x 1024 37.8 -> 42 us, 2048 x 2048 36.8 -> 40).
  long long target = p.cfg.bt == 64 ? kTargetWorkgroups / 2 : kTargetWorkgroups;
  if (p.cfg.bt == 64 && (long long)(n_in / 8) * base >= (f32 ? 16 : 32) * target) target *= 2;
  long long chunks = (target + base - 1) / (base > 0 ? base : 1);
  // Several heads in one launch: the kernel gives every XCD a contiguous run of heads, and an XCD
  // (64 resident workgroups) should work on at most two or three heads at a time so that their
  // codebooks stay in its L2: at least kFusedMinWgsPerHead workgroups per head.
  // (layers whose whole codebook traffic is small gain nothing from it: their workgroups would
  // only get shorter)
  if (n_heads > 1 && (long long)n_in * n_out >= kFusedMinEdgesForResidency) {
    const long long per_head = (long long)p.n_jt * p.n_bt;
    const long long want = (kFusedMinWgsPerHead + per_head - 1) / per_head;
    if (chunks < want) chunks = want;
  }
  const long long max_by_rows = n_in / 16;                                   // at least two steps each
  // Partial sums up to a quarter of the parameter stream - up to the whole of it for small layers, whose
  // launch is a latency chain and not a stream: capped at a quarter, config 3's second layer (262,144 edges) ran
  // on 48 workgroups at batch 64 and took 17-28 us; with the cap at the stream's size it runs on 128 and takes
  // 12.5-14.7 us (the head at batch 32 / 48 / 64: 39.9 / 57.5 / 60.0 against 46.7 / 62.8 / 71.5 us precise, 30.3 /
  // 41.0 / 43.8 against 36.9 / 43.5 / 47.6 us fp16; at batch 32 its chunks also become short enough to take the
  // first layer's partial sums as they are).  Layers of a million edges and more gain nothing from it.
  const long long max_by_bytes =
      (long long)n_in * bytes_per_edge / ((long long)n_in * n_out <= kFusedSmallLayerEdges ? B : 4 * B);
  if (chunks > max_by_rows) chunks = max_by_rows;
  if (chunks > max_by_bytes) chunks = max_by_bytes;
  if (chunks < 1) chunks = 1;
  int rows = (int)((n_in + chunks - 1) / chunks);
  rows = (rows + 7) / 8 * 8;
  p.rows_per_chunk = rows;
  p.n_chunks = (n_in + rows - 1) / rows;
  return p;
}

// Bucket path (prepared layers): one workgroup per (bucket, slice of the outputs, sample).
// A workgroup occupies a whole CU (LDS), so the slices are cut to give every CU one: the
// cuts come from the block table that the preparation made for this many (samples x heads).
constexpr int64_t kBucketMaxBatch = 4;
// A pass over the records per sample costs in proportion to the edges, the fused kernel's single pass for up to
// 16 samples does not: on the largest layers the fourth sample tips it (4096 x 4096, K = 262,144, batch 2 / 3 / 4:
// 61 / 89 / 117 us against 105-109 us fused; 4096 x 1024 and 2048 x 2048: 21 / 28 / 30-31 against 33-35 us).
constexpr long long kBucketThreeSamplesMinEdges = 1ll << 23;
constexpr int64_t bucket_max_batch(long long edges) { return edges >= kBucketThreeSamplesMinEdges ? 3 : kBucketMaxBatch; }

LayerPlan plan_bucket(const kan_vq_layer& L, int64_t B, int n_heads) {
  LayerPlan p;
  p.mfma = false;
  p.kind = kPlanBucket;
  p.name = "kan_bucket";
  p.cfg.bt = 1;
  p.cfg.jpl = 1;
  p.cfg.wj = 1;
  p.cfg.idx_u32 = L.idx_dtype == KAN_U32;
  p.cfg.gb_kind = gb_kind_of(L);
  p.cfg.code = code_of(L);
  const BucketGeom g = bucket_geometry(L.in, L.out, L.K, code_of(L), gb_kind_of(L));
  p.n_jt = g.tab_w[bucket_table_for((long long)B * n_heads)];       // blocks of the table a full group of heads uses
  p.n_bt = (int)B;
  p.n_chunks = g.n_buckets;          // the per-bucket sums are the partial sums
  p.rows_per_chunk = L.in;
  return p;
}

// Small prepared layers: one workgroup per (output, sample) reads the output's ids and gains from the
// transposed copy in the prepared buffer, gathers from L2 and writes finished outputs (no bucket
// copies, no partial sums, no reduction launch).  It is ahead of the bucket kernel while the layer's
// edges x samples stay within about 2^20 (measured, a layer alone, cold, column against bucket kernel:
// 1024 x 256 at batch 1 / 2 / 4: 11.0 / 9.6 / 9.6 against 14.7 / 13.3 / 13.2 us; 1024 x 512: 10.9 / 9.7 /
// 13.1 against 14.9 / 13.5 / 13.1; 1024 x 1024: 10.8 / 13.3 / 22.2 against 14.5 / 12.9 / 15.0; 2048 x 1024:
// 14.0 / 21.6 / 38.3 against 14.4 / 15.6 / 20.0); config 3's head with it on the second layer: 21.8 -> 15.8 us
// at batch 1, 24.2 -> 20.9 at batch 2.
constexpr long long kColumnMaxWork = 1ll << 20;     // edges x samples

bool layer_column_ok(const kan_vq_layer& L) {
  if (L.flags & KAN_LAYER_NO_COLUMN) return false;
  return (long long)L.in * L.out <= kColumnMaxEdges;
}

LayerPlan plan_column(const kan_vq_layer& L, int64_t B) {
  LayerPlan p;
  p.mfma = false;
  p.kind = kPlanColumn;
  p.name = "kan_column";
  p.cfg.bt = 1;
  p.cfg.jpl = 1;
  p.cfg.wj = 1;
  p.cfg.idx_u32 = L.idx_dtype == KAN_U32;
  p.cfg.gb_kind = gb_kind_of(L);
  p.cfg.code = code_of(L);
  p.n_jt = L.out;
  p.n_bt = (int)B;
  p.n_chunks = 1;
  p.rows_per_chunk = L.in;
  return p;
}

bool layer_prepared_ok(const kan_vq_layer& L) {
  return L.prepared != nullptr && aligned(L.prepared, 256) && aligned(L.codebook, 16) && L.in <= kBucketMaxIn &&
         (long long)L.in * L.out <= (1ll << 31);
}

// Which kernels serve a layer:
//   precise path, prepared layers, B <= kBucketMaxBatch (3 for layers of 2^23 edges or more): the bucket kernel
//     (codebook in LDS);
//   precise path (KAN_PATH_GATHER, and AUTO below batch 32): B = 1 the window-gather kernel,
//     B >= 2 the fused kernel with fp32 matrix-core operands (the fp32 FMA kernel remains the
//     dense baseline's), from kSplitMinBatch the preparation + streaming contraction of the
//     fp16 path on operands split into high and low fp16 parts, the contraction making
//     three passes (hi*lo, lo*hi, hi*hi: fp32-grade sums at matrix-core speed);
//   fp16 path (KAN_PATH_MFMA, and AUTO from batch 32): up to kHalfFusedMaxBatch the fused
//     kernel with fp16 operands, above that coefficient/basis preparation + the streaming
//     contraction;
//   layers of kFusedTwoTilesMinEdges edges or more (not fp32 codebooks) keep the fused kernel up to
//     kFusedTwoTilesMaxBatch on either path.
LayerPlan plan_vq(const kan_vq_layer& L, int64_t B, int n_heads, bool vec_ok, bool prepared_ok, int32_t path,
                  bool column_ok) {
  const int code = code_of(L);
  const int u32 = L.idx_dtype == KAN_U32, gbk = gb_kind_of(L);
  const bool half_path = path == KAN_PATH_MFMA || (path == KAN_PATH_AUTO && B >= kAutoMfmaBatch);
  // Large layers stay on the fused kernel for a second batch tile: gathering every row twice costs less
  // than preparing the records of 4 M edges or more and contracting them (4096 x 4096, K = 262,144, batch
  // 96-128: 288-290 -> 210-213 us on the fp16 path, 587 -> 474-478 us precise; 4096 x 1024: 60.8 -> 57.2 and
  // 103 -> 90-95 us; a 2048 x 1024 layer gains at batch 96 and loses at 128, config 3's head 57.5 -> 61.0 us,
  // fp32 rows - three loads per gather - lose: config 2 at batch 128 32.4 -> 35.7 us; at batch 192 all lose).
  const bool two_tiles = (long long)L.in * L.out >= kFusedTwoTilesMinEdges && code != kCbF32;
  const int64_t fused_max = two_tiles ? kFusedTwoTilesMaxBatch : kHalfFusedMaxBatch;
  if (half_path) {
    // one batch tile: every edge is needed once, so nothing is staged in memory (the streaming
    // path would write 20 bytes per edge and read them back for no reuse)
    if (B <= fused_max) return plan_fused(L.in, L.out, B, n_heads, u32, gbk, code, false);
    return plan_mfma(L.in, L.out, B, n_heads, u32, gbk, code);
  }
  if (prepared_ok && B <= bucket_max_batch((long long)L.in * L.out))
    return column_ok && (long long)L.in * L.out * B <= kColumnMaxWork ? plan_column(L, B) : plan_bucket(L, B, n_heads);
  // large batches: the fp16 machinery with both operands split into high and low parts
  if (B >= kSplitMinBatch && B > fused_max) return plan_mfma(L.in, L.out, B, n_heads, u32, gbk, code, true);
  if (B >= 2) return plan_fused(L.in, L.out, B, n_heads, u32, gbk, code, true);
  return plan_gather(L.in, L.out, B, n_heads, u32, gbk, code, vec_ok);
}

bool layer_vec_ok(const kan_vq_layer& L) {
  return aligned(L.idx, 16) && aligned(L.gain, 16) && aligned(L.bias, 16);
}

size_t partial_bytes(const LayerPlan& p, int n_out, int64_t B, int heads_in_group) {
  if (p.n_chunks <= 1) return 0;
  return round_up((size_t)heads_in_group * p.n_chunks * (size_t)B * n_out * sizeof(float), 256);
}

// Scratch regions inside the caller's workspace (each a multiple of 256 bytes;
// sized for the largest layer and for one group of heads).
struct WsLayout {
  size_t hidden = 0;    // one of two ping-pong hidden-activation buffers, [n_heads][B][out]
  size_t partial = 0;   // i-chunk partial sums
  size_t partial2 = 0;  // second buffer of per-bucket sums when consecutive bucket layers are chained
  size_t cf = 0;        // matrix-core path: fp16 coefficient fragments, a region per layer (layers after the
  size_t bp = 0;        //   first are prepared beside the first one's work) / partial bias sums, likewise
  std::vector<size_t> cf_off, bp_off;   // start of each layer's region within cf / bp
  size_t u = 0;         // matrix-core path: packed basis weights + span
  int n_layers = 1;
  size_t total() const { return (n_layers > 1 ? 2 * hidden : 0) + partial + partial2 + cf + bp + u; }
};

size_t mfma_cf_records(int n_in, int n_out) { return (size_t)((n_in + 15) / 16) * 20 * (size_t)n_out; }
size_t mfma_bp_floats(int n_in, int n_out) { return (size_t)((n_in + kMfmaPrepRows - 1) / kMfmaPrepRows) * n_out; }

hipError_t launch_gather(const LayerPlan& p, const GatherArgs& a, int heads, hipStream_t s) {
  dim3 grid((unsigned)(p.n_jt * p.n_bt), (unsigned)p.n_chunks, (unsigned)heads);
  switch (p.cfg.bt) {
    case 1: return launch_gather_bt1(p.cfg, a, grid, s);
    case 4: return launch_gather_bt4(p.cfg, a, grid, s);
    default: return launch_gather_bt16(p.cfg, a, grid, s);
  }
}

// Pointers of the scratch regions for the current call.
struct WsPtrs {
  float* hid[2];
  float* partial;
  float* partial2;
  uint4* cf;
  float* bp;
  uint2* u;
};

// One layer of a group of heads.  `a` carries x, shapes and the per-head pointers;
// `final_dst` receives act(y).  Gather path: main kernel, then (if i was split) the
// fixed-order reduction.  Matrix-core path: coefficient and basis preparation first.
// How a layer receives its input and hands on its output when it is chained to its
// neighbours: the partial sums of layer l (per bucket, or per chunk of inputs) are added and
// squashed by layer l+1 itself: by the bucket kernel while it loads x, or by the basis
// preparation of the matrix-core path.
// (config 3 at batch 65-128, whose first layer is cut into 32 chunks: 55.3-56.4 us with the 32 slices handed
// on against 56.7-57.4 us with a reduction launch)
constexpr int kMaxChainedSlices = 32;   // more slices than this go through the reduction pass (more loads in flight per output)

struct Chain {
  int in_parts = 1;              // slices of the input to add (1: plain x)
  long long in_part_stride = 0;
  int in_tanh = 0;
  bool out = false;              // leave the per-bucket sums for the next layer (no reduction pass)
  float* partial = nullptr;      // where this layer's partial sums go (default: w.partial)
  // matrix-core path: stages the head's first launch has already covered
  bool coef_done = false;
  bool basis_done = false;
};

// Matrix-core path, stage 1: coefficient records (and bias sums) of one layer of a group of heads.
// Depends on the layer's parameters only, not on x.
kan_status run_prep_coef(const LayerPlan& p, const GatherArgs& a, int heads, const WsPtrs& w, PrepCoefArgs* out,
                         bool launch, hipStream_t s) {
  PrepCoefArgs& pc = *out;
  memset(&pc, 0, sizeof(pc));
  pc.cf = w.cf;
  pc.cf_head_stride = (long long)mfma_cf_records(a.n_in, a.n_out);
  pc.cf_lo = p.products == 3 ? w.cf + (long long)heads * pc.cf_head_stride : nullptr;
  pc.bias_partial = w.bp;
  pc.bp_head_stride = (long long)mfma_bp_floats(a.n_in, a.n_out);
  pc.n_in = a.n_in;
  pc.n_out = a.n_out;
  memcpy(pc.h, a.h, sizeof(pc.h));
  if (!launch) return KAN_OK;
  if (p.cfg.code == kDense)
    return run("kan_prep_dense", s, [&] { return launch_prep_dense((const float*)a.h[0].cb, pc.cf, pc.cf_lo, a.n_in, a.n_out, s); });
  return run("kan_prep_coef", s, [&] { return launch_prep_coef(p.cfg, pc, heads, s); });
}

// Stage 2: packed basis weights and spans of the layer's input (x, or the previous layer's
// partial sums added and squashed).
struct BasisBufs {
  uint2* u_lo;
  long long u_stride;
};
kan_status run_prep_basis(const LayerPlan& p, const GatherArgs& a, int heads, bool x_shared, const WsPtrs& w,
                          const Chain& chain, BasisBufs* out, bool launch, hipStream_t s) {
  const long long u_elems = (long long)((a.n_in + 15) / 16 * 16) * a.B;
  out->u_stride = x_shared ? 0 : u_elems;
  out->u_lo = p.products == 3 ? w.u + (x_shared ? 1 : heads) * u_elems : nullptr;
  if (!launch) return KAN_OK;
  return run("kan_prep_basis", s, [&] {
    return launch_prep_basis(a.x, a.x_head_stride, chain.in_parts, chain.in_part_stride, chain.in_tanh, w.u, out->u_lo,
                             out->u_stride, a.n_in, a.B, x_shared ? 1 : heads, a.rule, s);
  });
}

kan_status run_layer_group(const LayerPlan& p, GatherArgs& a, const void* const* prepared, int heads,
                           bool x_shared, float* final_dst, long long final_head_stride, const WsPtrs& w,
                           int apply_tanh, hipStream_t s, const Chain& chain = Chain()) {
  const long long count = (long long)a.B * a.n_out;
  const bool split = p.n_chunks > 1;
  float* const partial = chain.partial ? chain.partial : w.partial;
  float* dst = split ? partial : final_dst;
  const long long dst_head_stride = split ? count * p.n_chunks : final_head_stride;
  const long long dst_chunk_stride = split ? count : 0;
  const int tanh_in_kernel = split ? 0 : apply_tanh;
  kan_status st;
  if (p.mfma) {
    PrepCoefArgs pc;
    const bool split3 = p.products == 3;
    st = run_prep_coef(p, a, heads, w, &pc, !chain.coef_done, s);
    if (st != KAN_OK) return st;
    BasisBufs bb;
    st = run_prep_basis(p, a, heads, x_shared, w, chain, &bb, !chain.basis_done, s);
    if (st != KAN_OK) return st;
    uint2* const u_lo = bb.u_lo;
    const long long u_stride = bb.u_stride;
    MfmaArgs m;
    memset(&m, 0, sizeof(m));
    m.cf = w.cf;
    m.cf_head_stride = pc.cf_head_stride;
    m.W = w.u;
    m.w_head_stride = u_stride;
    // (the dense form has no bias sums: the kernel still reads the rows it would add, so it is
    // given valid memory - the coefficient records, which are larger - and told not to add them)
    m.bias_partial = p.cfg.code == kDense ? (const float*)w.cf : w.bp;
    m.bp_head_stride = pc.bp_head_stride;
    m.dst = dst;
    m.dst_head_stride = dst_head_stride;
    m.dst_chunk_stride = dst_chunk_stride;
    m.n_in = a.n_in;
    m.n_out = a.n_out;
    m.B = a.B;
    m.rows_per_chunk = p.rows_per_chunk;
    m.n_jt = p.n_jt;
    m.apply_tanh = tanh_in_kernel;
    m.bias_on = p.cfg.code == kDense ? 0 : 1;            // the dense form has no bias
    for (int h = 0; h < heads; ++h) m.scale[h] = p.cfg.code == kCbI8 ? a.h[h].scale : 1.0f;
    if (split3) {                                        // hi*lo and lo*hi first, scaled by 1/2048, then hi*hi on top
      m.passes = 3;
      m.cf_lo = pc.cf_lo;
      m.W_lo = u_lo;
      m.lo_scale = 1.0f / 2048.0f;
    } else {
      m.passes = 1;
    }
    dim3 grid((unsigned)(p.n_jt * p.n_bt), (unsigned)p.n_chunks, (unsigned)heads);
    st = run(p.name, s, [&] { return launch_mfma(m, p.cfg.bt, p.tile_n ? p.tile_n : kMfmaTileN, grid, s); });
  } else if (p.kind == kPlanBucket || p.kind == kPlanColumn) {
    const BucketGeom g = bucket_geometry(a.n_in, a.n_out, (int)(a.cb_bytes / cb_row_bytes(p.cfg.code)), p.cfg.code,
                                         p.cfg.gb_kind);
    BucketArgs k;
    memset(&k, 0, sizeof(k));
    k.x = a.x;
    k.x_head_stride = a.x_head_stride;
    k.x_parts = chain.in_parts;
    k.x_part_stride = chain.in_part_stride;
    k.x_tanh = chain.in_tanh;
    k.dst = dst;
    k.dst_head_stride = dst_head_stride;
    k.dst_chunk_stride = dst_chunk_stride;
    k.n_in = a.n_in;
    k.n_out = a.n_out;
    k.B = a.B;
    k.n_buckets = g.n_buckets;
    const int table = bucket_table_for((long long)a.B * heads);     // by the heads of this very launch
    k.off_blk = (long long)(g.off_blk + (size_t)g.tab_first[table] * kBucketEntryWords * 4);
    k.rows_shift = g.rows_shift;
    k.cb_bytes = a.cb_bytes;
    k.apply_tanh = tanh_in_kernel;
    k.rule = a.rule;
    k.off_seg = (long long)g.off_seg;
    k.off_bias = (long long)g.off_bias;
    k.off_i = (long long)g.off_i;
    k.off_q = (long long)g.off_q;
    k.off_g = (long long)g.off_g;
    k.off_ti = (long long)g.off_ti;
    k.off_tg = (long long)g.off_tg;
    for (int h = 0; h < heads; ++h) {
      k.h[h].prepared = prepared[h];
      k.h[h].cb = a.h[h].cb;
      k.h[h].scale = a.h[h].scale;
      k.h[h].gain_log2_lo = a.h[h].gain_log2_lo;
      k.h[h].gain_log2_step = a.h[h].gain_log2_step;
    }
    if (p.kind == kPlanColumn) st = run(p.name, s, [&] { return launch_column(p.cfg.code, p.cfg.gb_kind, k, heads, s); });
    else st = run(p.name, s, [&] { return launch_bucket(p.cfg.code, p.cfg.gb_kind, k, g.tab_w[table], heads, s); });
  } else if (p.kind == kPlanFused16 || p.kind == kPlanFused32) {
    const bool f32 = p.kind == kPlanFused32;
    FusedArgs f;
    memset(&f, 0, sizeof(f));
    f.x = a.x;
    f.x_head_stride = a.x_head_stride;
    f.dst = dst;
    f.dst_head_stride = dst_head_stride;
    f.dst_chunk_stride = dst_chunk_stride;
    f.n_in = a.n_in;
    f.n_out = a.n_out;
    f.B = a.B;
    f.rows_per_chunk = p.rows_per_chunk;
    f.n_jt = p.n_jt;
    f.apply_tanh = tanh_in_kernel;
    f.rule = a.rule;
    f.x_parts = chain.in_parts;
    f.x_part_stride = chain.in_part_stride;
    f.x_tanh = chain.in_tanh;
    memcpy(f.h, a.h, sizeof(f.h));
    dim3 grid((unsigned)(p.n_jt * p.n_bt), (unsigned)p.n_chunks, (unsigned)heads);
    if (chain.in_parts > 1) st = run(p.name, s, [&] { return launch_fused_chained(p.cfg, f, f32, grid, s); });
    else st = run(p.name, s, [&] { return launch_fused(p.cfg, f, f32, grid, s); });
  } else {
    a.dst = dst;
    a.dst_head_stride = dst_head_stride;
    a.dst_chunk_stride = dst_chunk_stride;
    a.apply_tanh = tanh_in_kernel;
    a.x_parts = chain.in_parts;
    a.x_part_stride = chain.in_part_stride;
    a.x_tanh = chain.in_tanh;
    st = run(p.name, s, [&] { return launch_gather(p, a, heads, s); });
  }
  if (st != KAN_OK || !split || chain.out) return st;
  return run("kan_reduce", s, [&] {
    return launch_reduce(partial, dst_head_stride, count, p.n_chunks, final_dst, final_head_stride, count,
                         heads, apply_tanh, s);
  });
}

kan_status check_path(int32_t path) {
  if (path == KAN_PATH_AUTO || path == KAN_PATH_GATHER || path == KAN_PATH_MFMA) return KAN_OK;
  return KAN_ERR_UNSUPPORTED;
}

// Layer l leaves its partial sums to layer l+1 (one group of heads only: the buffers are
// sized for one group).  Consumers: the bucket kernel (after a bucket layer), the basis
// preparation of the matrix-core path (after any layer that splits its inputs), the fused
// kernel on tiles of 32 samples (after any such layer: see fused_takes_slices) and the
// vector-ALU kernel at batch 1.
bool fused_takes_slices(const LayerPlan& from, const LayerPlan& to, int n_in, int64_t B);

bool chained(const std::vector<LayerPlan>& plans, int l, int n_heads, const kan_vq_layer* layers, int64_t B) {
  if (l < 0 || l + 1 >= (int)plans.size() || n_heads > kMaxGroup || plans[l].n_chunks <= 1) return false;
  if (plans[l + 1].kind == kPlanBucket || plans[l + 1].kind == kPlanColumn) return plans[l].kind == kPlanBucket;
  if (plans[l + 1].kind == kPlanFused16 || plans[l + 1].kind == kPlanFused32)
    return fused_takes_slices(plans[l], plans[l + 1], layers[l + 1].in, B);
  // the vector-ALU kernel at batch 1: the threads that share a row of the basis table split the
  // slices; few output tiles (each adds the slices again)
  if (plans[l + 1].kind == kPlanGather)
    return plans[l + 1].cfg.bt == 1 && plans[l + 1].cfg.code != kDense && plans[l].n_chunks <= kGatherChainMaxParts &&
           plans[l + 1].n_jt <= 4;
  return plans[l + 1].kind == kPlanMfma && plans[l].n_chunks <= kMaxChainedSlices;
}

// The fused kernel adds the slices of its own chunk of inputs before its first step when that
// is cheaper than a reduction launch in between: tiles of 32 samples, the chunk's inputs of the
// tile within the kernel's LDS array, 16-byte loads (inputs in fours), at most 32 such loads
// per thread (two rounds in flight; with three, batch 32 of config 3, nothing was gained), and
// few output tiles (every one of them adds the slices again).
bool fused_takes_slices(const LayerPlan& from, const LayerPlan& to, int n_in, int64_t B) {
  if (to.cfg.bt != 32 || from.n_chunks > kFusedChainMaxParts || to.n_jt > 8) return false;
  if (n_in % 4 != 0 || to.rows_per_chunk % 4 != 0 || 32ll * to.rows_per_chunk > kFusedChainFloats) return false;
  const long long rows = B < 32 ? B : 32;
  return (long long)from.n_chunks * rows * (to.rows_per_chunk / 4) <= 32 * 256;
}

// Validates a [n_heads][n_layers] descriptor table; fills per-layer plans and scratch sizes.
kan_status plan_head(const kan_vq_layer* layers, int32_t n_layers, int32_t n_heads, int64_t B, int32_t path,
                     std::vector<LayerPlan>* plans, WsLayout* ws) {
  if (!layers) return KAN_ERR_NULL;
  if (n_layers < 1 || n_heads < 1 || n_layers > 64 || n_heads > (1 << 16)) return KAN_ERR_SHAPE;
  if (B < 0 || B > kMaxBatch) return KAN_ERR_SHAPE;
  kan_status st = check_path(path);
  if (st != KAN_OK) return st;
  for (int h = 0; h < n_heads; ++h)
    for (int l = 0; l < n_layers; ++l) {
      const kan_vq_layer& L = layers[(size_t)h * n_layers + l];
      st = validate_layer(&L);
      if (st != KAN_OK) return st;
      const kan_vq_layer& R = layers[l];
      if (L.in != R.in || L.out != R.out || L.K != R.K || L.idx_dtype != R.idx_dtype ||
          L.gb_dtype != R.gb_dtype || L.cb_dtype != R.cb_dtype || L.rule != R.rule)
        return KAN_ERR_UNSUPPORTED;
      if (l > 0 && L.in != layers[(size_t)h * n_layers + l - 1].out) return KAN_ERR_SHAPE;
    }
  const int group = n_heads < kMaxGroup ? n_heads : kMaxGroup;
  *ws = WsLayout();
  ws->n_layers = n_layers;
  plans->clear();
  for (int l = 0; l < n_layers; ++l) {
    const kan_vq_layer& R = layers[l];
    bool vec_ok = true, prepared_ok = true, column_ok = true;
    for (int h = 0; h < n_heads; ++h) {
      vec_ok = vec_ok && layer_vec_ok(layers[(size_t)h * n_layers + l]);
      prepared_ok = prepared_ok && layer_prepared_ok(layers[(size_t)h * n_layers + l]);
      column_ok = column_ok && layer_column_ok(layers[(size_t)h * n_layers + l]);
    }
    LayerPlan p = plan_vq(R, B, group, vec_ok, prepared_ok, path, column_ok);
    plans->push_back(p);
    auto grow = [](size_t& dst, size_t v) { if (v > dst) dst = v; };
    grow(ws->partial, partial_bytes(p, R.out, B, group));
    ws->cf_off.push_back(ws->cf);
    ws->bp_off.push_back(ws->bp);
    if (p.mfma) {
      ws->cf += round_up((size_t)(p.products == 3 ? 2 : 1) * group * mfma_cf_records(R.in, R.out) * sizeof(uint4), 256);
      ws->bp += round_up((size_t)group * mfma_bp_floats(R.in, R.out) * sizeof(float), 256);
    }
    if (p.mfma)
      grow(ws->u, round_up((size_t)(p.products == 3 ? 2 : 1) * (size_t)(l == 0 ? 1 : group) * (size_t)((R.in + 15) / 16 * 16) * (size_t)B * sizeof(uint2), 256));
    if (l + 1 < n_layers) grow(ws->hidden, round_up((size_t)n_heads * (size_t)B * R.out * sizeof(float), 256));
  }
  // chained layers hand their partial sums straight on: two buffers, used in turn
  for (int l = 0; l + 1 < n_layers; ++l)
    if (chained(*plans, l, n_heads, layers, B)) ws->partial2 = ws->partial;
  return KAN_OK;
}

}  // namespace
}  // namespace kan

using namespace kan;

extern "C" {

const char* kan_status_string(int32_t status) {
  switch (status) {
    case KAN_OK: return "ok";
    case KAN_ERR_NULL: return "required pointer is NULL";
    case KAN_ERR_SHAPE: return "invalid or inconsistent size or alignment";
    case KAN_ERR_DTYPE: return "dtype not allowed for this operand";
    case KAN_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KAN_ERR_UNSUPPORTED: return "unsupported configuration";
    case KAN_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

kan_status kan_bspline_basis(const float* x, int64_t n, uint8_t* span, float* w, void* stream) {
  if (n < 0) return KAN_ERR_SHAPE;
  if (n == 0) return KAN_OK;
  if (!x || !span || !w) return KAN_ERR_NULL;
  if (!aligned(w, 16) || !aligned(x, 4)) return KAN_ERR_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  return run("kan_basis", s, [&] { return launch_basis(x, n, span, w, s); });
}

kan_status kan_pli_basis(const float* x, int64_t n, uint8_t* index, float* w, void* stream) {
  if (n < 0) return KAN_ERR_SHAPE;
  if (n == 0) return KAN_OK;
  if (!x || !index || !w) return KAN_ERR_NULL;
  if (!aligned(w, 8) || !aligned(x, 4)) return KAN_ERR_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  return run("kan_pli_basis", s, [&] { return launch_pli_basis(x, n, index, w, s); });
}

kan_status kan_basis_window(const float* x, int64_t n, int32_t rule, int32_t variant, uint8_t* start, float* w,
                            void* stream) {
  if (n < 0) return KAN_ERR_SHAPE;
  if (rule != KAN_RULE_BSPLINE3 && rule != KAN_RULE_PLI2) return KAN_ERR_UNSUPPORTED;
  if (variant != 0 && variant != 1) return KAN_ERR_UNSUPPORTED;
  if (n == 0) return KAN_OK;
  if (!x || !start || !w) return KAN_ERR_NULL;
  if (!aligned(w, 16) || !aligned(x, 4)) return KAN_ERR_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  return run("kan_basis_window", s, [&] { return launch_basis_window(x, n, rule, variant, start, w, s); });
}

size_t kan_vq_workspace_bytes(const kan_vq_layer* layers, int32_t n_layers, int32_t n_heads, int64_t B,
                              int32_t path) {
  std::vector<LayerPlan> plans;
  WsLayout wl;
  if (plan_head(layers, n_layers, n_heads, B, path, &plans, &wl) != KAN_OK) return (size_t)-1;
  if (B == 0) return 0;
  return wl.total();
}

namespace {
// The forward of a group of heads.  static_ws: take the scratch regions from the library's own
// per-device array instead of a caller's workspace (ws, ws_bytes are then ignored).
kan_status head_forward(const kan_vq_layer* layers, int32_t n_layers, int32_t n_heads, const float* x, int64_t B,
                        float* y, void* ws, size_t ws_bytes, bool static_ws, int32_t path, void* stream) {
  std::vector<LayerPlan> plans;
  WsLayout wl;
  kan_status st = plan_head(layers, n_layers, n_heads, B, path, &plans, &wl);
  if (st != KAN_OK) return st;
  if (B == 0) return KAN_OK;
  if (!x || !y) return KAN_ERR_NULL;
  if (!aligned(x, 4) || !aligned(y, 4)) return KAN_ERR_SHAPE;
  const size_t need = wl.total();
  if (static_ws) {
    if (need > (size_t)KAN_STATIC_SCRATCH_BYTES) return KAN_ERR_WORKSPACE;     // beyond the fixed array: use kan_vq_head_forward
    ws = nullptr;
    ws_bytes = KAN_STATIC_SCRATCH_BYTES;
    if (need > 0) {
      st = static_scratch(&ws);
      if (st != KAN_OK) return st;
    }
  }
  if (need > 0 && (!ws || !aligned(ws, 256) || ws_bytes < need)) return KAN_ERR_WORKSPACE;

  hipStream_t s = (hipStream_t)stream;
  char* wsp = (char*)ws;
  WsPtrs w;
  const size_t hid2 = n_layers > 1 ? 2 * wl.hidden : 0;
  w.hid[0] = (float*)wsp;
  w.hid[1] = (float*)(wsp + wl.hidden);
  w.partial = (float*)(wsp + hid2);
  w.partial2 = (float*)(wsp + hid2 + wl.partial);
  const size_t after_partial = hid2 + wl.partial + wl.partial2;
  uint4* const cf_base = (uint4*)(wsp + after_partial);
  float* const bp_base = (float*)(wsp + after_partial + wl.cf);
  w.cf = cf_base;
  w.bp = bp_base;
  w.u = (uint2*)(wsp + after_partial + wl.cf + wl.bp);

  auto layer_args = [&](int l, int h0, int heads, const float* src, long long src_head_stride, GatherArgs* out,
                        const void** prepared) {
    const kan_vq_layer& R = layers[l];
    GatherArgs& a = *out;
    memset(&a, 0, sizeof(a));
    a.x = src + (long long)h0 * src_head_stride;
    a.x_head_stride = src_head_stride;
    a.n_in = R.in;
    a.n_out = R.out;
    a.B = (int)B;
    a.rows_per_chunk = plans[l].rows_per_chunk;
    a.n_jt = plans[l].n_jt;
    a.cb_bytes = (long long)R.K * cb_row_bytes(code_of(R));
    a.rule = R.rule;
    for (int h = 0; h < heads; ++h) {
      const kan_vq_layer& L = layers[(size_t)(h0 + h) * n_layers + l];
      a.h[h].idx = L.idx;
      a.h[h].gain = L.gain;
      a.h[h].bias = L.bias;
      a.h[h].cb = L.codebook;
      a.h[h].scale = L.scale;
      a.h[h].gain_log2_lo = L.gain_log2_lo;
      a.h[h].gain_log2_step = L.gain_log2_step;
      a.h[h].bias_scale = L.bias_scale;
      if (prepared) prepared[h] = L.prepared;
    }
  };

  // A single head on the matrix cores: one launch prepares the coefficient records of its
  // matrix-core layers (those stored like the first one, up to kStartJobs) and the first layer's
  // basis words; the layers below then skip these stages.
  std::vector<char> coef_done(n_layers, 0);
  bool basis0_done = false;
  if (n_heads == 1 && plans[0].mfma) {
    PrepStartArgs ps;
    memset(&ps, 0, sizeof(ps));
    const LayerPlan& p0 = plans[0];
    for (int l = 0; l < n_layers && ps.n_jobs < kStartJobs; ++l) {
      const LayerPlan& p = plans[l];
      if (!p.mfma || p.products != p0.products || p.cfg.code != p0.cfg.code || p.cfg.gb_kind != p0.cfg.gb_kind ||
          p.cfg.idx_u32 != p0.cfg.idx_u32)
        continue;
      GatherArgs a;
      layer_args(l, 0, 1, x, 0, &a, nullptr);
      WsPtrs wl_ptrs = w;
      wl_ptrs.cf = cf_base + wl.cf_off[l] / sizeof(uint4);
      wl_ptrs.bp = bp_base + wl.bp_off[l] / sizeof(float);
      PrepCoefArgs pc;
      (void)run_prep_coef(p, a, 1, wl_ptrs, &pc, false, s);
      PrepStartArgs::Job& job = ps.job[ps.n_jobs++];
      job.cf = pc.cf;
      job.cf_lo = pc.cf_lo;
      job.bp = pc.bias_partial;
      job.n_in = pc.n_in;
      job.n_out = pc.n_out;
      job.h = pc.h[0];
      coef_done[l] = 1;
    }
    GatherArgs a0;
    layer_args(0, 0, 1, x, 0, &a0, nullptr);
    BasisBufs bb;
    (void)run_prep_basis(p0, a0, 1, true, w, Chain(), &bb, false, s);
    ps.x = x;
    ps.W = w.u;
    ps.W_lo = bb.u_lo;
    ps.n_in = a0.n_in;
    ps.B = a0.B;
    ps.rule = a0.rule;
    if (prep_start_blocks(ps) <= kPrepStartMaxBlocks) {
      st = run("kan_prep_start", s, [&] { return launch_prep_start(p0.cfg, ps, p0.products == 3, s); });
      if (st != KAN_OK) return st;
      basis0_done = true;
    } else {                                   // too many workgroups for one grid: the layers launch their own
      coef_done.assign(n_layers, 0);
    }
  }

  struct LayerScope {      // launches of the loop below are timed per layer
    ~LayerScope() { if (g_prof.on) g_prof.cur_layer = 0; }
  } layer_scope;
  for (int l = 0; l < n_layers; ++l) {
    if (g_prof.on) g_prof.cur_layer = l + 1;       // (timing hooks: one thread, nothing else in flight)
    const kan_vq_layer& R = layers[l];
    const bool last = (l + 1 == n_layers);
    w.cf = cf_base + wl.cf_off[l] / sizeof(uint4);
    w.bp = bp_base + wl.bp_off[l] / sizeof(float);
    const float* src = (l == 0) ? x : w.hid[(l - 1) & 1];
    long long src_head_stride = (l == 0) ? 0 : (long long)B * R.in;
    Chain chain;
    chain.partial = (l & 1) ? w.partial2 : w.partial;
    if (!wl.partial2) chain.partial = w.partial;
    chain.out = chained(plans, l, n_heads, layers, B);
    if (chained(plans, l - 1, n_heads, layers, B)) {
      src = ((l - 1) & 1) ? w.partial2 : w.partial;
      chain.in_parts = plans[l - 1].n_chunks;
      chain.in_part_stride = (long long)B * R.in;
      chain.in_tanh = 1;
      src_head_stride = chain.in_part_stride * chain.in_parts;
    }
    float* dst = last ? y : w.hid[l & 1];
    const long long dst_head_stride = (long long)B * R.out;
    for (int h0 = 0; h0 < n_heads; h0 += kMaxGroup) {
      const int heads = (n_heads - h0) < kMaxGroup ? (n_heads - h0) : kMaxGroup;
      GatherArgs a;
      const void* prepared[kMaxGroup];
      layer_args(l, h0, heads, src, src_head_stride, &a, prepared);
      chain.coef_done = coef_done[l] != 0;
      chain.basis_done = l == 0 && basis0_done;
      st = run_layer_group(plans[l], a, prepared, heads, l == 0, dst + (long long)h0 * dst_head_stride, dst_head_stride, w,
                           last ? 0 : 1, s, chain);
      if (st != KAN_OK) return st;
    }
  }
  return KAN_OK;
}
}  // namespace

kan_status kan_vq_head_forward(const kan_vq_layer* layers, int32_t n_layers, int32_t n_heads, const float* x,
                               int64_t B, float* y, void* ws, size_t ws_bytes, int32_t path, void* stream) {
  return head_forward(layers, n_layers, n_heads, x, B, y, ws, ws_bytes, false, path, stream);
}

kan_status kan_vq_head_forward_static(const kan_vq_layer* layers, int32_t n_layers, int32_t n_heads, const float* x,
                                      int64_t B, float* y, int32_t path, void* stream) {
  return head_forward(layers, n_layers, n_heads, x, B, y, nullptr, 0, true, path, stream);
}

kan_status kan_vq_layer_forward(const kan_vq_layer* L, const float* x, int64_t B, float* y, void* ws,
                                size_t ws_bytes, int32_t path, void* stream) {
  return kan_vq_head_forward(L, 1, 1, x, B, y, ws, ws_bytes, path, stream);
}

// The dense baseline: the fp32 FMA kernel, and from kDenseSplitMinBatch the split-operand matrix-core
// form the precise VQ path uses (a converter of the coefficients in place of gather + dequantise).
static LayerPlan plan_dense(int32_t in, int32_t out, int64_t B) {
  if (B >= kDenseSplitMinBatch) {
    LayerPlan p = plan_mfma(in, out, B, 1, 0, 0, kDense, true);
    p.name = "kan_dense_split";
    return p;
  }
  LayerPlan p = plan_gather(in, out, B, 1, 0, 0, kDense, true);
  p.name = "kan_dense";
  return p;
}

static void dense_ws(const LayerPlan& p, int32_t in, int32_t out, int64_t B, size_t* partial, size_t* cf, size_t* u) {
  *partial = partial_bytes(p, out, B, 1);
  *cf = p.mfma ? round_up(2 * mfma_cf_records(in, out) * sizeof(uint4), 256) : 0;
  *u = p.mfma ? round_up(2 * (size_t)((in + 15) / 16 * 16) * (size_t)B * sizeof(uint2), 256) : 0;
}

size_t kan_dense_workspace_bytes(int32_t in, int32_t out, int64_t B) {
  if (in < 1 || out < 1 || in > kMaxDim || out > kMaxDim || B < 0 || B > kMaxBatch) return (size_t)-1;
  if (B == 0) return 0;
  size_t partial, cf, u;
  dense_ws(plan_dense(in, out, B), in, out, B, &partial, &cf, &u);
  return partial + cf + u;
}

kan_status kan_dense_layer_forward(const float* coef, int32_t in, int32_t out, int32_t G, const float* x,
                                   int64_t B, float* y, void* ws, size_t ws_bytes, void* stream) {
  if (G != 10) return KAN_ERR_UNSUPPORTED;
  if (in < 1 || out < 1 || in > kMaxDim || out > kMaxDim || B < 0 || B > kMaxBatch) return KAN_ERR_SHAPE;
  if (B == 0) return KAN_OK;
  if (!coef || !x || !y) return KAN_ERR_NULL;
  if (!aligned(coef, 8) || !aligned(x, 4) || !aligned(y, 4)) return KAN_ERR_SHAPE;
  const LayerPlan p = plan_dense(in, out, B);
  size_t partial, cf, u;
  dense_ws(p, in, out, B, &partial, &cf, &u);
  const size_t need = partial + cf + u;
  if (need > 0 && (!ws || !aligned(ws, 256) || ws_bytes < need)) return KAN_ERR_WORKSPACE;
  GatherArgs a;
  memset(&a, 0, sizeof(a));
  a.x = x;
  a.n_in = in;
  a.n_out = out;
  a.B = (int)B;
  a.rows_per_chunk = p.rows_per_chunk;
  a.n_jt = p.n_jt;
  a.h[0].cb = coef;
  a.h[0].scale = 1.0f;
  WsPtrs w;
  memset(&w, 0, sizeof(w));
  w.partial = (float*)ws;
  w.cf = (uint4*)((char*)ws + partial);
  w.u = (uint2*)((char*)ws + partial + cf);
  return run_layer_group(p, a, nullptr, 1, true, y, (long long)B * out, w, 0, (hipStream_t)stream);
}

size_t kan_vq_prepared_bytes(const kan_vq_layer* L) {
  if (validate_layer(L) != KAN_OK) return (size_t)-1;
  if (L->in > kBucketMaxIn || (long long)L->in * L->out > (1ll << 31)) return 0;
  return bucket_geometry(L->in, L->out, L->K, code_of(*L), gb_kind_of(*L)).total;
}

kan_status kan_vq_prepare(const kan_vq_layer* L, void* prepared, size_t prepared_bytes, void* stream) {
  kan_status st = validate_layer(L);
  if (st != KAN_OK) return st;
  if (L->in > kBucketMaxIn) return KAN_ERR_UNSUPPORTED;
  if ((long long)L->in * L->out > (1ll << 31)) return KAN_ERR_UNSUPPORTED;   // 32-bit segment offsets
  const BucketGeom g = bucket_geometry(L->in, L->out, L->K, code_of(*L), gb_kind_of(*L));
  if (!prepared || !aligned(prepared, 256) || prepared_bytes < g.total) return KAN_ERR_WORKSPACE;
  LayerPtrs h = {L->idx, L->gain, L->bias, L->codebook, L->scale, L->gain_log2_lo, L->gain_log2_step, L->bias_scale};
  hipStream_t s = (hipStream_t)stream;
  return run("kan_vq_prepare", s, [&] {
    return launch_bucket_prepare(h, L->idx_dtype == KAN_U32, gb_kind_of(*L), L->in, L->out, g, prepared, s);
  });
}

size_t kan_vq_assign_workspace_bytes(int32_t K) {
  if (K < 1) return (size_t)-1;
  return round_up(assign_centroid_bytes(K), 256);
}

namespace {
kan_status check_assign_shapes(int32_t in, int32_t out, int32_t K, int32_t idx_dtype) {
  if (in < 1 || out < 1 || in > kMaxDim || out > kMaxDim || K < 1) return KAN_ERR_SHAPE;
  if ((long long)in * out > (1ll << 31)) return KAN_ERR_SHAPE;
  if (idx_dtype != KAN_U16 && idx_dtype != KAN_U32) return KAN_ERR_DTYPE;
  if (idx_dtype == KAN_U16 && K > 65536) return KAN_ERR_SHAPE;
  return KAN_OK;
}
}  // namespace

kan_status kan_vq_assign(const float* coef, int32_t in, int32_t out, const float* codebook, int32_t K,
                         int32_t idx_dtype, void* idx, float* gain, float* bias, void* ws, size_t ws_bytes,
                         void* stream) {
  kan_status st = check_assign_shapes(in, out, K, idx_dtype);
  if (st != KAN_OK) return st;
  if (!coef || !codebook || !idx || !gain || !bias) return KAN_ERR_NULL;
  if (!aligned(coef, 8) || !aligned(codebook, 4) || !aligned(gain, 4) || !aligned(bias, 4) ||
      !aligned(idx, idx_dtype == KAN_U16 ? 2 : 4))
    return KAN_ERR_SHAPE;
  if (!ws || !aligned(ws, 256) || ws_bytes < kan_vq_assign_workspace_bytes(K)) return KAN_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  return run("kan_vq_assign", s, [&] {
    return launch_assign(coef, (long long)in * out, codebook, K, idx_dtype == KAN_U32, idx, gain, bias, ws, s);
  });
}

size_t kan_vq_reconstruction_workspace_bytes(int32_t in, int32_t out) {
  if (in < 1 || out < 1 || in > kMaxDim || out > kMaxDim) return (size_t)-1;
  return round_up((size_t)recon_blocks((long long)in * out) * 3 * sizeof(double), 256);
}

kan_status kan_vq_reconstruction_sums(const float* coef, int32_t in, int32_t out, const float* codebook, int32_t K,
                                      int32_t idx_dtype, const void* idx, const float* gain, const float* bias,
                                      double* sums, void* ws, size_t ws_bytes, void* stream) {
  kan_status st = check_assign_shapes(in, out, K, idx_dtype);
  if (st != KAN_OK) return st;
  if (!coef || !codebook || !idx || !gain || !bias || !sums) return KAN_ERR_NULL;
  if (!aligned(coef, 4) || !aligned(codebook, 4) || !aligned(gain, 4) || !aligned(bias, 4) || !aligned(sums, 8) ||
      !aligned(idx, idx_dtype == KAN_U16 ? 2 : 4))
    return KAN_ERR_SHAPE;
  if (!ws || !aligned(ws, 256) || ws_bytes < kan_vq_reconstruction_workspace_bytes(in, out)) return KAN_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  return run("kan_vq_reconstruction_sums", s, [&] {
    return launch_recon_sums(coef, (long long)in * out, codebook, idx_dtype == KAN_U32, idx, gain, bias, (double*)ws,
                             sums, s);
  });
}

kan_status kan_vq_debug_gather(const kan_vq_layer* L, uint32_t* ids, float* rows, void* stream) {
  kan_status st = validate_layer(L);
  if (st != KAN_OK) return st;
  if (!ids && !rows) return KAN_ERR_NULL;
  LayerPtrs h = {L->idx, L->gain, L->bias, L->codebook, L->scale, 0.f, 0.f, 0.f};
  hipStream_t s = (hipStream_t)stream;
  return run("kan_debug_gather", s, [&] {
    return launch_debug_gather(h, L->idx_dtype == KAN_U32, code_of(*L),
                               (long long)L->in * L->out, ids, rows, s);
  });
}

kan_status kan_vq_count_bad_indices(const kan_vq_layer* L, uint32_t* count, void* stream) {
  kan_status st = validate_layer(L);
  if (st != KAN_OK) return st;
  if (!count) return KAN_ERR_NULL;
  hipStream_t s = (hipStream_t)stream;
  return run("kan_count_bad", s, [&] {
    return launch_count_bad(L->idx, L->idx_dtype == KAN_U32, (long long)L->in * L->out, (uint32_t)L->K,
                            count, s);
  });
}

kan_status kan_vq_coef_range(const kan_vq_layer* L, float* range, void* stream) {
  kan_status st = validate_layer(L);
  if (st != KAN_OK) return st;
  if (!range) return KAN_ERR_NULL;
  if (!aligned(range, 4)) return KAN_ERR_SHAPE;
  LayerPtrs h = {L->idx, L->gain, L->bias, L->codebook, L->scale, L->gain_log2_lo, L->gain_log2_step, L->bias_scale};
  hipStream_t s = (hipStream_t)stream;
  return run("kan_coef_range", s, [&] {
    return launch_coef_range(h, L->idx_dtype == KAN_U32, gb_kind_of(*L), code_of(*L), (long long)L->in * L->out, range, s);
  });
}

const char* kan_vq_planned_kernel(const kan_vq_layer* L, int64_t B, int32_t n_heads, int32_t path) {
  if (validate_layer(L) != KAN_OK || check_path(path) != KAN_OK || B < 1 || n_heads < 1) return "invalid";
  return plan_vq(*L, B, n_heads < kMaxGroup ? n_heads : kMaxGroup, layer_vec_ok(*L), layer_prepared_ok(*L), path, layer_column_ok(*L))
      .name;
}

const char* kan_dense_planned_kernel(int32_t in, int32_t out, int64_t B) {
  if (in < 1 || out < 1 || in > kMaxDim || out > kMaxDim || B < 1 || B > kMaxBatch) return "invalid";
  return plan_dense(in, out, B).name;
}

kan_status kan_prof_begin(int32_t max_launches) {
  if (max_launches < 1 || max_launches > (1 << 20)) return KAN_ERR_SHAPE;
  if (g_prof.on) return KAN_ERR_UNSUPPORTED;
  g_prof.ev.assign(2 * (size_t)max_launches, nullptr);
  g_prof.names.assign(max_launches, nullptr);
  g_prof.layer.assign(max_launches, 0);
  for (auto& e : g_prof.ev)
    if (hipEventCreate(&e) != hipSuccess) return KAN_ERR_LAUNCH;
  g_prof.cap = max_launches;
  g_prof.n = 0;
  g_prof.on = true;
  return KAN_OK;
}

kan_status kan_prof_end(kan_prof_record* out, int32_t cap, int32_t* n_out) {
  if (!g_prof.on) return KAN_ERR_UNSUPPORTED;
  g_prof.on = false;
  int n_rec = 0;
  kan_status st = KAN_OK;
  for (int n = 0; n < g_prof.n; ++n) {
    float ms = 0.f;
    if (hipEventSynchronize(g_prof.ev[2 * n + 1]) != hipSuccess ||
        hipEventElapsedTime(&ms, g_prof.ev[2 * n], g_prof.ev[2 * n + 1]) != hipSuccess) {
      st = KAN_ERR_LAUNCH;
      break;
    }
    char key[sizeof(out[0].name)];
    if (g_prof.layer[n] > 0) snprintf(key, sizeof(key), "%s@L%d", g_prof.names[n], g_prof.layer[n]);
    else snprintf(key, sizeof(key), "%s", g_prof.names[n]);
    int r = 0;
    for (; r < n_rec; ++r)
      if (strcmp(out[r].name, key) == 0) break;
    if (r == n_rec) {
      if (!out || n_rec >= cap) continue;
      memset(&out[r], 0, sizeof(out[r]));
      memcpy(out[r].name, key, sizeof(key));
      ++n_rec;
    }
    out[r].launches += 1;
    out[r].total_ms += ms;
  }
  for (auto& e : g_prof.ev)
    if (e) (void)hipEventDestroy(e);
  g_prof.ev.clear();
  g_prof.names.clear();
  g_prof.layer.clear();
  g_prof.cur_layer = 0;
  if (n_out) *n_out = n_rec;
  return st;
}

}  // extern "C"
