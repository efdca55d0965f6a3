// Fused matrix-core kernel of the VQ-KAN forward pass (small and medium batch).
//
// Same contraction as kan_mfma.hip, Y = Phi * Chat (+ bias), but the coefficient operand
// is not written to memory first; every batch tile of 32 or 64 samples gathers the
// codewords it needs itself (with one tile every edge is gathered exactly once; with
// several, the repeated gathers cost less than the fp32 matrix-core time they feed, and
// for fp16 operands the dispatcher switches to the streaming kernel instead).  The lane that feeds output column j of the MFMA B operand reads
// idx/gain/bias of its own edges (coalesced along j), gathers their codewords,
// dequantises them and keeps the fragments in registers; metadata is prefetched three
// steps ahead and codewords one step ahead through small register rings.  The work is
// bound by the rate of random codeword gathers (one per edge), not by arithmetic.
//
// Operand precisions (fp16 forms: v_mfma_f32_32x32x16_f16 with k-step s < 4, lane half h:
// coefficients 0..7 of input 4h+s; k-step 4: coefficients 8, 9 of inputs 4h..4h+3):
//   F32 = false  fp16 operands; the Int8 scale is applied at the end.
//   F32 = true   the precise path (sums match the float64 definition to ~1e-6), in two forms:
//     32-sample tiles: fp32 operands, v_mfma_f32_32x32x2f32: MFMA t = 10*s + m multiplies, in
//                lane half h, coefficient m of input 4h+s.  With one row block the 40 MFMAs of a
//                step take about as long as its gathers.
//     16-sample tiles (batch <= 16): fp32 operands, v_mfma_f32_16x16x4f32 on two blocks of 16
//                columns per wave: half the matrix-pipe time, no empty rows (T16 below).
//     64-sample tiles: both operands split into high and low fp16 parts (v = hi + lo / 2048,
//                22 significant bits), three fp16 products per k-step (hi*lo and lo*hi into one
//                set of accumulators, hi*hi into another); every fp16 x fp16 product is exact in
//                the fp32 accumulators: a fifth of the matrix-pipe time of fp32 operands.
// Workgroup: 256 threads = 4 waves, each 32 output columns; tile of 32*MBLK samples.
// The basis tile Phi is built in LDS (double buffered) straight from x: with at most 64
// samples the strided reads of x are few, and no preparation kernel is launched.

#include <type_traits>

#include "kan_device.hpp"
#include "kan_internal.hpp"
#include "kan_mfma_common.hpp"

namespace kan {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int IT = 8;                  // input rows per step
constexpr int BN = kFusedTileN;        // outputs per workgroup: 4 waves x 32
constexpr int LDH = 88;                // fp16 tile: row stride in halves (176 B)
constexpr int LDF = 84;                // fp32 tile: row stride in floats (336 B); row = [h][s][m]

// STAGE: the per-edge metadata of two steps (16 input rows x the wave's 32
// columns) comes in with one 16-byte load per lane and array and is dealt to the lanes that own
// the columns through a wave-private strip of LDS, instead of one 2-byte load per lane, row and
// array: 3 vector-memory instructions per two steps instead of 24 (the address unit of the CU,
// which every such instruction occupies for its 64 lanes, is what bounds this kernel).  Needs
// n_out % 16 == 0 and 16-byte aligned arrays.
// T16 (fp32 operands, batch <= 16): the tile is 16 samples high and the step runs on
// v_mfma_f32_16x16x4_f32, half the matrix-pipe time of the 32-row instruction, whose upper rows would
// be empty (the 40 fp32 MFMAs of a step are 8 of the 26 us that layer 1 of configuration 3 takes at
// batch 16).  The wave's 32 columns are two blocks of 16; a lane serves column (lane % 16) of both
// blocks and the inputs 2 kg, 2 kg + 1 of every step (kg = lane / 16 is its k index in the
// instruction): slot s of a lane's four edges is input 2 kg + s % 2 in block s / 2, instead of input
// 4 lh + s in one column.  (The other forms are compiled from the same text as before: every place
// that differs is a branch on T16.)
// CH (32-sample tiles): the input arrives as the previous layer's partial sums, one slice per
// chunk of that layer's inputs.  Before its first step the workgroup adds the slices of its own
// chunk of inputs (16-byte loads, up to 16 in flight per thread; threads that share an item take
// consecutive runs of slices and their sums are added in run order through LDS), squashes them and
// keeps them in dynamic shared memory, [valid sample rows][inputs of the chunk]; the steps read
// their inputs from there.  The reduction launch between the two layers and the round trip of the
// hidden activation through memory go.  The kernels without CH are compiled from the same text as
// before: every place that differs is a branch on CH.
template <typename IdxT, typename GbT, typename CbT, bool F32, int MBLK, bool STAGE, bool T16 = false, bool CH = false>
__global__ __launch_bounds__(kThreads, 2) void kan_fused_kernel(const FusedArgs a) {
  static_assert(!T16 || (F32 && MBLK == 1), "16-sample tiles: fp32 operands only");
  static_assert(!CH || MBLK == 1, "chained input: 32-sample tiles only");
  constexpr int BM = 32 * MBLK;
  constexpr int NPAIR = MBLK;          // (sample, input) pairs per thread and step
  // The precise path comes in two forms: fp32 operands for 32-sample tiles (one row block: the 40 fp32
  // MFMAs of a step take about as long as its gathers, and nothing has to be split), split fp16 operands
  // for 64-sample tiles (two row blocks: a fifth of the matrix-pipe time).
  constexpr bool kFp32Ops = F32 && MBLK == 1;
  constexpr bool kSplit = F32 && MBLK == 2;
  constexpr int kHalfTile = BM * LDH * 2;                       // one fp16 tile
  constexpr int kTileBytes = kFp32Ops ? BM * LDF * 4 : (kSplit ? 2 * kHalfTile : kHalfTile);   // split form: high parts, then low parts
  __shared__ __attribute__((aligned(16))) unsigned char sTile[2][kTileBytes];
  __shared__ __attribute__((aligned(16))) uint32_t sSel[kSpans][8];
  // (filled by the pipelines below once their first loads are on their way: nothing reads it before the first tile)
  [[maybe_unused]] auto fill_selectors = [&]() {
    if constexpr (!kFp32Ops) {
      fill_weight_selectors(sSel, threadIdx.x);
      __syncthreads();
    }
  };

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  // Which (head, chunk of inputs, tile) this workgroup takes.  Workgroups go to the eight XCDs in
  // turn (linear index mod 8) and every XCD has its own 4 MB L2.  With several heads in a launch
  // the plain order would put workgroups of every resident head on every XCD, and the codebooks
  // of all of them (655 KB each as Int8) would compete for each L2.  Instead the list of work
  // items, sorted by head, is cut into eight contiguous runs, one per XCD, taken in order: an XCD
  // then works on two or three heads at a time and a codebook enters one L2 only.
  // (CH: the same renumbering for a single head: the output tiles of a chunk read the same slices of
  // the input, and neighbouring chunks the two halves of the same 128-byte lines when a chunk is 16
  // inputs long, so runs of consecutive (chunk, tile) items on one XCD fetch every line once: config
  // 3's second layer at batch 16 fetched 22.8 MiB with the plain order, 4 MiB of slices four times over.)
  int head = blockIdx.z, chunk = blockIdx.y, tile = blockIdx.x;
  if (gridDim.z > 1 || CH) {
    const unsigned T = gridDim.x, C = gridDim.y, W = T * C * gridDim.z;
    const unsigned L = blockIdx.x + T * (blockIdx.y + C * blockIdx.z);
    const unsigned xcd = L & 7u, m = L >> 3, q = W >> 3, r = W & 7u;
    const unsigned item = xcd * q + min(xcd, r) + m;          // XCD x owns q + (x < r) items
    head = (int)(item / (T * C));
    const unsigned rem = item % (T * C);
    chunk = (int)(rem / T);
    tile = (int)(rem % T);
  }
  const int jt = tile % a.n_jt, b0 = (tile / a.n_jt) * (32 * MBLK);
  const int n_in = a.n_in, n_out = a.n_out, B = a.B;
  const int i_begin = chunk * a.rows_per_chunk;
  const int i_end = min(n_in, i_begin + a.rows_per_chunk);
  const int n_steps = (i_end - i_begin + IT - 1) / IT;

  const LayerPtrs hp = a.h[head];
  const IdxT* idx = (const IdxT*)hp.idx;
  const GbT* gain = (const GbT*)hp.gain;
  const GbT* bias = (const GbT*)hp.bias;
  const Q8Params qp = {hp.gain_log2_lo, hp.gain_log2_step, hp.bias_scale};
  const CbT* cb = (const CbT*)hp.cb;
  const float scale = sizeof(CbT) == 1 ? hp.scale : 1.0f;
  const float gmul = F32 ? scale : 1.0f;        // the precise form's coefficients carry the scale themselves
  const float* xh = a.x + (long long)head * a.x_head_stride;

  // Phi generation: input pin of every step for the sample rows psm, psm + 32, ...  Eight neighbouring lanes
  // read eight consecutive inputs of one sample, so a load of x touches 8 cache lines, not 64 (lanes along
  // the samples made every such load as dear to the address unit as a codeword gather).
  static_assert(IT == 8, "eight inputs per step: one per lane of a group of eight");
  const int pin = tid & 7, psm = tid >> 3;
  const float* xrow[NPAIR];
#pragma unroll
  for (int q = 0; q < NPAIR; ++q) xrow[q] = xh + (long long)min(b0 + psm + 32 * q, B - 1) * n_in;
  extern __shared__ __attribute__((aligned(16))) float sX[];      // CH: the chunk's inputs (dynamic; none otherwise)
  // CH: valid sample rows of the tile; inputs of the chunk, a multiple of four (the host checks n_in and the chunk length)
  [[maybe_unused]] const int x_rows = min(BM, B - b0), x_len = i_end - i_begin;
  // Two halves, called by the pipelines below: chain_issue once their first metadata loads are on their
  // way (it requests the first 16 slices of the thread's first item and waits for nothing), chain_finish
  // once the first gathers are out (it adds those slices, fetches what is left, and fills sX).
  struct ChainItem {
    int row, c4, p_begin, p_end;
    bool live;
    const float* src;
  };
  [[maybe_unused]] auto chain_item = [&](int q0) {
    const int len4 = x_len >> 2;
    const int n_items = x_rows * len4;                  // 16-byte items of the tile
    const int parts = a.x_parts;
    const int runs = n_items >= kThreads ? 1 : kThreads / n_items;    // threads per item
    const int per_run = (parts + runs - 1) / runs;
    const int q = runs > 1 ? tid % n_items : q0 + tid;
    const int g = runs > 1 ? tid / n_items : 0;
    ChainItem it;
    it.live = q < n_items && g < runs;
    const int qq = it.live ? q : 0;
    it.row = qq / len4;
    it.c4 = qq - it.row * len4;
    it.src = xh + (long long)(b0 + it.row) * n_in + i_begin + 4 * it.c4;
    it.p_begin = min(g * per_run, parts);
    it.p_end = min(parts, it.p_begin + per_run);
    return it;
  };
  [[maybe_unused]] auto chain_load = [&](const ChainItem& it, int p0, f32x4 (&t)[16]) {
#pragma unroll
    for (int pp = 0; pp < 16; ++pp)                     // (slices past the last one are re-reads of it, added as zero)
      t[pp] = *(const f32x4*)(it.src + (long long)min(p0 + pp, a.x_parts - 1) * a.x_part_stride);
  };
  [[maybe_unused]] auto chain_issue = [&](f32x4 (&t)[16]) {
    const ChainItem it = chain_item(0);
    chain_load(it, it.p_begin, t);
  };
  [[maybe_unused]] auto chain_finish = [&](const f32x4 (&first)[16]) {
    static_assert(!CH || kTileBytes >= kThreads * 16, "the runs' sums pass through the first tile");
    const int n_items = x_rows * (x_len >> 2);
    const int runs = n_items >= kThreads ? 1 : kThreads / n_items;
    f32x4* const scr = (f32x4*)sTile[0];
    for (int q0 = 0; q0 < n_items; q0 += kThreads) {
      const ChainItem it = chain_item(q0);
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
      auto add = [&](const f32x4 (&t)[16], int p0) {
#pragma unroll
        for (int pp = 0; pp < 16; ++pp) {
          const bool in = p0 + pp < it.p_end;
          sum.x += in ? t[pp].x : 0.f;
          sum.y += in ? t[pp].y : 0.f;
          sum.z += in ? t[pp].z : 0.f;
          sum.w += in ? t[pp].w : 0.f;
        }
      };
      int p0 = it.p_begin;
      if (q0 == 0) {                                    // (uniform) the slices chain_issue asked for
        add(first, p0);
        p0 += 16;
      }
      for (; p0 < it.p_end; p0 += 16) {
        f32x4 t[16];
        chain_load(it, p0, t);
        add(t, p0);
      }
      bool owner = it.live;
      if (runs > 1) {                                   // (uniform; the loop then has this one round)
        scr[tid] = sum;
        __syncthreads();
        owner = tid < n_items;
        if (owner)
          for (int gg = 1; gg < runs; ++gg) sum += scr[gg * n_items + tid];
      }
      if (owner) {
        if (a.x_tanh) {
          sum.x = tanhf(sum.x);
          sum.y = tanhf(sum.y);
          sum.z = tanhf(sum.z);
          sum.w = tanhf(sum.w);
        }
        *(f32x4*)(sX + it.row * x_len + 4 * it.c4) = sum;
      }
    }
    __syncthreads();
  };
  // coefficient operand: column jc, input rows 4*lh .. 4*lh+3 of every step
  const int j = jt * BN + wave * 32 + ln;
  const bool j_ok = j < n_out;
  const int jc = min(j, n_out - 1);
  // T16: slot -> input of the step, column within the wave's 32, and that column's validity and clamped index
  const int kg = lane >> 4, c16 = lane & 15;
  auto t16_col = [&](int s) { return jt * BN + wave * 32 + 16 * (s >> 1) + c16; };
  f32x4 acc4[T16 ? 2 : 1];             // T16: one accumulator per block of 16 columns
  float bsum2[T16 ? 2 : 1];
  if constexpr (T16) {
    acc4[0] = acc4[1] = f32x4{0.f, 0.f, 0.f, 0.f};
    bsum2[0] = bsum2[1] = 0.f;
  }

  f32x16 acc[MBLK], acc_x[MBLK];       // (acc_x: the cross products of the split form)
#pragma unroll
  for (int m = 0; m < MBLK; ++m)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      acc[m][r] = 0.f;
      acc_x[m][r] = 0.f;
    }
  float bsum = 0.f;

  struct Meta {
    uint32_t id[4];
    float g[4], b[4];
  };
  struct Frag {                         // B operand of one step
    uint4 h[kFp32Ops ? 1 : 5];          // 5 k-steps of 8 halves (split form: the high parts)
    uint4 l[kSplit ? 5 : 1];            // split form: the low parts
    float f[kFp32Ops ? 4 : 1][kG];      // fp32 operands: [s][m]
  };
  // fp32 coefficients of the four rows of a step -> high and low fragments
  auto split_step = [&](const float (&c)[4][kG], Frag& out) {
    uint32_t th[4], tl[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      uint32_t hi[5], lo[5];
      split_consecutive(c[s], hi, lo);
      out.h[kSplit ? s : 0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
      out.l[kSplit ? s : 0] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
      th[s] = hi[4];
      tl[s] = lo[4];
    }
    out.h[kSplit ? 4 : 0] = make_uint4(th[0], th[1], th[2], th[3]);
    out.l[kSplit ? 4 : 0] = make_uint4(tl[0], tl[1], tl[2], tl[3]);
  };

  auto load_meta = [&](int k, Meta& m) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      int i;
      bool ok;
      long long e;
      if constexpr (T16) {
        i = i_begin + k * IT + 2 * kg + (s & 1);
        ok = t16_col(s) < n_out && i < i_end;
        e = (long long)min(i, i_end - 1) * n_out + min(t16_col(s), n_out - 1);
      } else {
        i = i_begin + k * IT + 4 * lh + s;
        ok = j_ok && i < i_end;
        e = (long long)min(i, i_end - 1) * n_out + jc;
      }
      uint32_t id[1];
      float g[1], bv[1];
      load_idx<IdxT, 1>(idx + e, id);
      load_gain<GbT, 1>(gain + e, qp, g);
      load_bias<GbT, 1>(bias + e, qp, bv);
      m.id[s] = id[0];
      m.g[s] = ok ? g[0] * gmul : 0.f;      // out-of-range edges contribute nothing
      m.b[s] = ok ? bv[0] : 0.f;
    }
  };
  auto gather_rows = [&](const Meta& m, RawRow<CbT> (&rows)[4]) {
#pragma unroll
    for (int s = 0; s < 4; ++s) load_row<CbT>(cb, m.id[s], rows[s]);
  };
  auto dequant_step = [&](RawRow<CbT> (&rows)[4], const Meta& m, Frag& out) {
#pragma unroll
    for (int s = 0; s < 4; ++s) align_row<CbT>(rows[s], row_odd<CbT>(cb, m.id[s]));
    if constexpr (kFp32Ops) {
#pragma unroll
      for (int s = 0; s < 4; ++s) dequant_row_f32<CbT>(rows[s], m.g[s], out.f[s]);
    } else if constexpr (kSplit) {
      float c[4][kG];
#pragma unroll
      for (int s = 0; s < 4; ++s) dequant_row_f32<CbT>(rows[s], m.g[s], c[s]);
      split_step(c, out);
    } else {
      uint32_t tail[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        uint32_t w[5];
        dequant_row<CbT>(rows[s], m.g[s], w);
        out.h[s] = make_uint4(w[0], w[1], w[2], w[3]);
        tail[s] = w[4];
      }
      out.h[4] = make_uint4(tail[0], tail[1], tail[2], tail[3]);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if constexpr (T16) bsum2[s >> 1] += m.b[s];
      else bsum += m.b[s];
    }
  };

  // -- the same three pieces for the deep pipeline below (indices apart from gains and biases,
  //    every load unconditional)
  struct Ids { uint32_t id[4]; };
  struct GainBias { float g[4], b[4]; };
  // Every load of the pipeline is unconditional, so that the compiler counts the loads in
  // flight exactly and a wait covers only what is needed next.  Steps past the end of the
  // chunk read the chunk's last row again (coalesced) and gather codeword 0 with every lane (one
  // cache line per wave instead of 64), which costs next to nothing; their edges have gain 0.
  auto load_meta_deep = [&](int k, Ids& ids, GainBias& gb) {
    const bool live = k < n_steps;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int i = i_begin + k * IT + 4 * lh + s;
      const bool ok = j_ok && i < i_end;
      const long long e = (long long)min(i, i_end - 1) * n_out + jc;
      uint32_t id[1];
      float g[1], bv[1];
      load_idx<IdxT, 1>(idx + e, id);
      load_gain<GbT, 1>(gain + e, qp, g);
      load_bias<GbT, 1>(bias + e, qp, bv);
      ids.id[s] = live ? id[0] : 0u;
      gb.g[s] = ok ? g[0] * gmul : 0.f;      // out-of-range edges contribute nothing
      gb.b[s] = ok ? bv[0] : 0.f;
    }
  };
  // (the alignment bits of a step's four rows travel in one word beside the rows)
  auto gather_ids = [&](const Ids& m, RawRow<CbT> (&rows)[4], uint32_t& odd) {
    odd = 0u;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      load_row<CbT>(cb, m.id[s], rows[s]);
      odd |= row_odd<CbT>(cb, m.id[s]) << s;
    }
  };
  auto dequant_deep = [&](RawRow<CbT> (&rows)[4], const uint32_t odd, const GainBias& m, Frag& out) {
#pragma unroll
    for (int s = 0; s < 4; ++s) align_row<CbT>(rows[s], (odd >> s) & 1u);
    if constexpr (kFp32Ops) {
#pragma unroll
      for (int s = 0; s < 4; ++s) dequant_row_f32<CbT>(rows[s], m.g[s], out.f[s]);
    } else if constexpr (kSplit) {
      float c[4][kG];
#pragma unroll
      for (int s = 0; s < 4; ++s) dequant_row_f32<CbT>(rows[s], m.g[s], c[s]);
      split_step(c, out);
    } else {
      uint32_t tail[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        uint32_t w[5];
        dequant_row<CbT>(rows[s], m.g[s], w);
        out.h[s] = make_uint4(w[0], w[1], w[2], w[3]);
        tail[s] = w[4];
      }
      out.h[4] = make_uint4(tail[0], tail[1], tail[2], tail[3]);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) bsum += m.b[s];
  };

  // ---- staged metadata (STAGE): a pair of steps per load -------------------------------------
  constexpr int EI = (int)sizeof(IdxT), EG = (int)sizeof(GbT);
  constexpr int NLI = (EI + 1) / 2, NLG = (EG + 1) / 2;          // 16-byte loads per lane and pair: 32 E units over 64 lanes
  constexpr int kStripBytes = STAGE ? 512 * (EI + 2 * EG) : 16;   // idx, gain, bias tiles of 16 rows x 32 columns
  __shared__ __attribute__((aligned(16))) unsigned char sMeta[4][kStripBytes];
  struct MetaRaw {
    u32x4 i[NLI], g[NLG], b[NLG];
  };
  // unit t of an array with E-byte elements: row t / (2 E) of the pair, 16 / E columns from (t % (2 E)) * 16 / E
  auto stage_issue = [&](int pair, MetaRaw& m) {
    const int col0 = jt * BN + wave * 32;
    auto one = [&](const void* base, auto E_, u32x4* dst, int u) {
      constexpr int E = decltype(E_)::value;
      const int t = (lane + 64 * u) & (32 * E - 1);              // (one-byte arrays: the upper half of the wave repeats the lower)
      const int r = t / (2 * E), part = t % (2 * E);
      const int i = min(i_begin + pair * 16 + r, i_end - 1);      // rows past the chunk re-read its last row
      const int col = min(col0 + part * (16 / E), n_out - 16 / E);
      dst[u] = __builtin_nontemporal_load((const u32x4*)((const char*)base + ((size_t)i * n_out + col) * E));
    };
#pragma unroll
    for (int u = 0; u < NLI; ++u) one(idx, std::integral_constant<int, EI>{}, m.i, u);
#pragma unroll
    for (int u = 0; u < NLG; ++u) one(gain, std::integral_constant<int, EG>{}, m.g, u);
#pragma unroll
    for (int u = 0; u < NLG; ++u) one(bias, std::integral_constant<int, EG>{}, m.b, u);
  };
  // raw tiles -> the wave's strip; then every lane picks the values of its own column and rows
  auto stage_commit = [&](const MetaRaw& m) {
    unsigned char* strip = sMeta[wave];
    __builtin_amdgcn_wave_barrier();                             // earlier reads of the strip stay before these writes
#pragma unroll
    for (int u = 0; u < NLI; ++u) *(u32x4*)(strip + (((lane + 64 * u) & (32 * EI - 1)) * 16)) = m.i[u];
#pragma unroll
    for (int u = 0; u < NLG; ++u) *(u32x4*)(strip + 512 * EI + (((lane + 64 * u) & (32 * EG - 1)) * 16)) = m.g[u];
#pragma unroll
    for (int u = 0; u < NLG; ++u) *(u32x4*)(strip + 512 * (EI + EG) + (((lane + 64 * u) & (32 * EG - 1)) * 16)) = m.b[u];
    __builtin_amdgcn_wave_barrier();
  };
  // the values of step `k` (half `sp` = k & 1 of the pair in the strip), with the masks of load_meta_deep
  auto stage_read_into = [&](int k, int sp, uint32_t (&out_id)[4], float (&out_g)[4], float (&out_b)[4]) {
    const unsigned char* strip = sMeta[wave];
    const bool live = k < n_steps;
    // columns past n_out were read from the last 16 / E columns of the row: this lane's slot then holds another
    // column's value, which the masks below discard (gain and bias 0; the codeword it gathers is a valid row)
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      auto decode = [&](IdxT idv, GbT gv, GbT bv, bool ok, bool col_ok) {
        float g, b;
        if constexpr (EG == 1) {
          g = q8_gain(gv.v, qp);
          b = q8_bias(bv.v, qp);
        } else if constexpr (EG == 2) {
          g = __half2float(gv);
          b = __half2float(bv);
        } else {
          g = gv;
          b = bv;
        }
        out_id[s] = (live && col_ok) ? (uint32_t)idv : 0u;
        out_g[s] = ok ? g * gmul : 0.f;
        out_b[s] = ok ? b : 0.f;
      };
      if constexpr (T16) {
        const int r = sp * 8 + 2 * kg + (s & 1), cw = 16 * (s >> 1) + c16;
        const int i = i_begin + k * IT + 2 * kg + (s & 1);
        const bool col_ok = t16_col(s) < n_out;
        decode(*(const IdxT*)(strip + (r * 32 + cw) * EI), *(const GbT*)(strip + 512 * EI + (r * 32 + cw) * EG),
               *(const GbT*)(strip + 512 * (EI + EG) + (r * 32 + cw) * EG), col_ok && i < i_end, col_ok);
      } else {
        const int r = sp * 8 + 4 * lh + s;
        const int i = i_begin + k * IT + 4 * lh + s;
        const bool ok = j_ok && i < i_end;
        const IdxT idv = *(const IdxT*)(strip + (r * 32 + ln) * EI);
        const GbT gv = *(const GbT*)(strip + 512 * EI + (r * 32 + ln) * EG);
        const GbT bv = *(const GbT*)(strip + 512 * (EI + EG) + (r * 32 + ln) * EG);
        float g, b;
        if constexpr (EG == 1) {
          g = q8_gain(gv.v, qp);
          b = q8_bias(bv.v, qp);
        } else if constexpr (EG == 2) {
          g = __half2float(gv);
          b = __half2float(bv);
        } else {
          g = gv;
          b = bv;
        }
        out_id[s] = (live && j_ok) ? (uint32_t)idv : 0u;
        out_g[s] = ok ? g * gmul : 0.f;
        out_b[s] = ok ? b : 0.f;
      }
    }
  };
  auto stage_read = [&](int k, int sp, Ids& ids, GainBias& gb) { stage_read_into(k, sp, ids.id, gb.g, gb.b); };

  auto load_u = [&](int k, float (&uv)[NPAIR]) {
    if constexpr (CH) {
      uv[0] = sX[min(psm, x_rows - 1) * x_len + min(k * IT + pin, x_len - 1)];
      return;
    }
    const int i = min(i_begin + k * IT + pin, n_in - 1);
#pragma unroll
    for (int q = 0; q < NPAIR; ++q) uv[q] = xrow[q][i];
  };
  auto gen_phi = [&](const float (&uv)[NPAIR], unsigned char* tile) {
#pragma unroll
    for (int q = 0; q < NPAIR; ++q) {
      const int pb = psm + 32 * q, h = pin >> 2, s = pin & 3;
      const BasisW bw = basis_fast(uv[q], a.rule);
      const int l = bw.span;
      const float w0 = bw.w0, w1 = bw.w1, w2 = bw.w2, w3 = bw.w3;
      if constexpr (kFp32Ops) {
        float* p = (float*)tile + pb * LDF + h * 40 + s * kG;      // 8-byte aligned
        const float2 z = make_float2(0.f, 0.f);
#pragma unroll
        for (int m = 0; m < kG / 2; ++m) ((float2*)p)[m] = z;
        p[l] = w0;                  // same thread: LDS keeps the order of its stores
        p[l + 1] = w1;
        p[l + 2] = w2;
        p[l + 3] = w3;
        continue;
      }
      uint32_t w01, w23, l01 = 0u, l23 = 0u;
      if constexpr (kSplit) {
        split_weights(w0, w1, w01, l01);
        split_weights(w2, w3, w23, l23);
      } else {
        w01 = pack_h2(w0, w1);
        w23 = pack_h2(w2, w3);
      }
      const uint4 sl = *(const uint4*)&sSel[l][0];
      const uint32_t sh = sSel[l][4];
      auto place = [&](uint32_t a01, uint32_t a23, unsigned char* t) {
        uint4 lo;
        lo.x = __builtin_amdgcn_perm(a23, a01, sl.x);
        lo.y = __builtin_amdgcn_perm(a23, a01, sl.y);
        lo.z = __builtin_amdgcn_perm(a23, a01, sl.z);
        lo.w = __builtin_amdgcn_perm(a23, a01, sl.w);
        const uint32_t hi = __builtin_amdgcn_perm(a23, a01, sh);
        uint16_t* rowp = (uint16_t*)t + pb * LDH;
        *(uint4*)(rowp + 16 * s + 8 * h) = lo;
        *(uint32_t*)(rowp + 64 + 8 * h + 2 * s) = hi;
      };
      place(w01, w23, tile);
      if constexpr (kSplit) place(l01, l23, tile + kHalfTile);
    }
  };

  // Precise form: cross products (high x low, low x high; they carry a factor 2048) into acc_x,
  // the main product into acc; every fp16 x fp16 product is exact in the fp32 accumulators.
  auto mfma_step = [&](const unsigned char* tile, const Frag& bf) {
    if constexpr (T16) {            // MFMA t = 10 e + m multiplies, in lane group kg, coefficient m of input 2 kg + e
      const float* p = (const float*)tile + c16 * LDF + kg * 20;
      float av[20];
#pragma unroll
      for (int q = 0; q < 5; ++q) {
        const float4 v = *(const float4*)(p + 4 * q);
        av[4 * q] = v.x;
        av[4 * q + 1] = v.y;
        av[4 * q + 2] = v.z;
        av[4 * q + 3] = v.w;
      }
#pragma unroll
      for (int t = 0; t < 20; ++t)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
          acc4[T16 ? cb : 0] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[t], bf.f[kFp32Ops ? 2 * cb + t / kG : 0][t % kG],
                                                                   acc4[T16 ? cb : 0], 0, 0, 0);
      return;
    }
    if constexpr (kFp32Ops) {       // MFMA t = 10 s + m multiplies, in lane half h, coefficient m of input 4h + s
      const float* p = (const float*)tile + ln * LDF + lh * 40;
#pragma unroll
      for (int q = 0; q < 10; ++q) {
        const float4 av = *(const float4*)(p + 4 * q);       // slots 4q .. 4q+3 of [s][m]
        const float avs[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int t = 4 * q + e;
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(avs[e], bf.f[kFp32Ops ? t / kG : 0][t % kG], acc[0], 0, 0, 0);
        }
      }
      return;
    }
#pragma unroll
    for (int ks = 0; ks < 5; ++ks) {
      const h16x8 fb = __builtin_bit_cast(h16x8, bf.h[kFp32Ops ? 0 : ks]);
#pragma unroll
      for (int m = 0; m < MBLK; ++m) {
        const uint16_t* ap = (const uint16_t*)tile + (m * 32 + ln) * LDH + ks * 16 + lh * 8;
        const h16x8 fa = __builtin_bit_cast(h16x8, *(const uint4*)ap);
        if constexpr (kSplit) {
          const h16x8 fbl = __builtin_bit_cast(h16x8, bf.l[kSplit ? ks : 0]);
          const h16x8 fal = __builtin_bit_cast(h16x8, *(const uint4*)(ap + kHalfTile / 2));
          acc_x[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa, fbl, acc_x[m], 0, 0, 0);
          acc_x[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fal, fb, acc_x[m], 0, 0, 0);
        }
        acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa, fb, acc[m], 0, 0, 0);
      }
    }
  };

  // Two pipelines.  The deep one pays off where a step holds enough MFMA work and chunks are
  // long (fp16 operands, 64-sample tiles: 66.7 -> 57.7 us for configuration 3 at batch 64);
  // with short chunks its extra prologue loads cost more than they hide (batch 2..16: +2..10 %),
  // and the precise form's three products per k-step already cover the gathers.
  constexpr bool kDeep = !F32 && MBLK == 2;
  if constexpr (kDeep) {
    // ---- pipeline (rings indexed by compile-time slots, loop unrolled by 8) ------------------
    // With few samples a step is a handful of MFMAs, far shorter than a gather's trip to L2, so
    // the rings are deep.  Top of step k: fragments and Phi tile of step k are ready; codeword
    // rows of steps k+1 .. k+RD-1 are held or in flight; so are indices up to step k+RD+1,
    // gains/biases up to step k+RD+1 and inputs up to step k+3.  Step k dequantises step k+1,
    // builds tile k+1, multiplies step k and issues the gathers of step k+RD plus the metadata
    // of step k+RD+2.  RD = 4 for one- and two-byte codebook entries, 2 for fp32 rows (registers).
    constexpr int RD = sizeof(CbT) == 4 ? 2 : 4;
    Ids ids[4];
    GainBias gbr[8];
    RawRow<CbT> rows[RD][4];
    uint32_t odd[RD];
    float uv[4][NPAIR];
    Frag frag[2];
    MetaRaw mraw;                                     // STAGE: the pair of steps on its way from memory
    if constexpr (STAGE) {
      static_assert(RD == 4, "the staged pipeline is laid out for four steps of codewords in flight");
      MetaRaw m0, m1, m2;
      stage_issue(0, m0);
      stage_issue(1, m1);
      stage_issue(2, m2);
  #pragma unroll
      for (int q = 0; q < 4; ++q) load_u(q, uv[q]);
      stage_commit(m0);
      stage_read(0, 0, ids[0], gbr[0]);
      stage_read(1, 1, ids[1], gbr[1]);
      stage_commit(m1);
      stage_read(2, 0, ids[2], gbr[2]);
      stage_read(3, 1, ids[3], gbr[3]);
  #pragma unroll
      for (int q = 0; q < RD; ++q) gather_ids(ids[q & 3], rows[q], odd[q]);
      stage_commit(m2);
      stage_read(4, 0, ids[0], gbr[4]);               // (the gathers above have read slots 0, 1)
      stage_read(5, 1, ids[1], gbr[5]);
      stage_issue(3, mraw);
    } else {
  #pragma unroll
      for (int q = 0; q < RD; ++q) load_meta_deep(q, ids[q & 3], gbr[q & 7]);
  #pragma unroll
      for (int q = 0; q < 4; ++q) load_u(q, uv[q]);
  #pragma unroll
      for (int q = 0; q < RD; ++q) gather_ids(ids[q & 3], rows[q], odd[q]);
  #pragma unroll
      for (int q = RD; q < RD + 2; ++q) load_meta_deep(q, ids[q & 3], gbr[q & 7]);     // (the gathers above have read slots 0, 1)
    }
    fill_selectors();
    dequant_deep(rows[0], odd[0], gbr[0], frag[0]);
    gen_phi(uv[0], sTile[0]);

    auto step = [&](auto T, int k) {
      constexpr int t = decltype(T)::value;          // k mod 8
      __syncthreads();     // tile k is complete; every wave is done reading tile k-1
      dequant_deep(rows[(t + 1) % RD], odd[(t + 1) % RD], gbr[(t + 1) & 7], frag[(t + 1) & 1]);   // step k+1 fragments
      gather_ids(ids[(t + RD) & 3], rows[t % RD], odd[t % RD]);                    // step k+RD codewords
      if constexpr (STAGE) {
        // even steps: the pair k+6, k+7 (requested two steps ago) goes through the strip into the rings,
        // and the pair k+8, k+9 is requested
        if constexpr ((t & 1) == 0) {
          stage_commit(mraw);
          stage_read(k + 6, 0, ids[(t + 6) & 3], gbr[(t + 6) & 7]);
          stage_read(k + 7, 1, ids[(t + 7) & 3], gbr[(t + 7) & 7]);
          stage_issue((k >> 1) + 4, mraw);
        }
      } else {
        load_meta_deep(k + RD + 2, ids[(t + RD + 2) & 3], gbr[(t + RD + 2) & 7]);          // step k+RD+2 metadata
      }
      mfma_step(sTile[t & 1], frag[t & 1]);
      gen_phi(uv[(t + 1) & 3], sTile[(t + 1) & 1]);                                 // step k+1 basis tile
      load_u(k + 4, uv[t & 3]);
    };
    // Branch-free groups of eight steps, then a nested tail: a step that follows a branch
    // taken or not would make the compiler wait for every load in flight.
    int k = 0;
    for (; k + 8 <= n_steps; k += 8) {
      step(std::integral_constant<int, 0>{}, k);
      step(std::integral_constant<int, 1>{}, k + 1);
      step(std::integral_constant<int, 2>{}, k + 2);
      step(std::integral_constant<int, 3>{}, k + 3);
      step(std::integral_constant<int, 4>{}, k + 4);
      step(std::integral_constant<int, 5>{}, k + 5);
      step(std::integral_constant<int, 6>{}, k + 6);
      step(std::integral_constant<int, 7>{}, k + 7);
    }
    if (k < n_steps) {
      step(std::integral_constant<int, 0>{}, k);
      if (k + 1 < n_steps) {
        step(std::integral_constant<int, 1>{}, k + 1);
        if (k + 2 < n_steps) {
          step(std::integral_constant<int, 2>{}, k + 2);
          if (k + 3 < n_steps) {
            step(std::integral_constant<int, 3>{}, k + 3);
            if (k + 4 < n_steps) {
              step(std::integral_constant<int, 4>{}, k + 4);
              if (k + 5 < n_steps) {
                step(std::integral_constant<int, 5>{}, k + 5);
                if (k + 6 < n_steps) step(std::integral_constant<int, 6>{}, k + 6);
              }
            }
          }
        }
      }
    }

  } else {
    // ---- pipeline (rings indexed by compile-time slots, loop unrolled by 4) ------------------
    // Top of step k: fragments and Phi tile of step k are ready; codeword rows and basis words
    // of step k+1 are in flight; metadata of steps k+1 .. k+3 is held or in flight.
    Meta meta[4];
    RawRow<CbT> rows[2][4];
    float uv[2][NPAIR];
    Frag frag[2];
    // Nothing is fetched for steps past the end: the address units that serve the random
    // codeword gathers are the bottleneck of this kernel, so wasted gathers are not free.
    MetaRaw mraw;                                     // STAGE: the pair of steps on its way from memory
    [[maybe_unused]] f32x4 xfirst[CH ? 16 : 1];       // CH: the first slices of the thread's item
    if constexpr (STAGE) {
      // 32-sample tiles: both pairs of steps are requested before the first is waited for - chunks are often
      // four steps long, and the second request would otherwise leave only when the first has crossed the
      // memory system (config 3 at batch 16, layer 1 of the precise path: 21.6 -> 20.1 us).  The 64-sample
      // forms, which have no registers to spare, keep the second request behind the first (batch 64: 71.5 us
      // against 73.2-73.5 with both up front).
      if constexpr (MBLK == 1) {
        MetaRaw mfirst;
        stage_issue(0, mfirst);
        if (2 < n_steps) stage_issue(1, mraw);
        if constexpr (CH) chain_issue(xfirst);
        stage_commit(mfirst);
        stage_read_into(0, 0, meta[0].id, meta[0].g, meta[0].b);
        stage_read_into(1, 1, meta[1].id, meta[1].g, meta[1].b);
      } else {
        stage_issue(0, mraw);
        stage_commit(mraw);
        stage_read_into(0, 0, meta[0].id, meta[0].g, meta[0].b);
        stage_read_into(1, 1, meta[1].id, meta[1].g, meta[1].b);
        if (2 < n_steps) stage_issue(1, mraw);
      }
      if constexpr (!CH) load_u(0, uv[0]);
      gather_rows(meta[0], rows[0]);
      if (1 < n_steps) gather_rows(meta[1], rows[1]);
    } else {
      load_meta(0, meta[0]);
      if (1 < n_steps) load_meta(1, meta[1]);
      if constexpr (CH) chain_issue(xfirst);
      if constexpr (!CH) load_u(0, uv[0]);
      gather_rows(meta[0], rows[0]);
      if (2 < n_steps) load_meta(2, meta[2]);
      if (1 < n_steps) gather_rows(meta[1], rows[1]);
      if (3 < n_steps) load_meta(3, meta[3]);
    }
    if constexpr (CH) {                               // the chunk's inputs, behind the first gathers
      chain_finish(xfirst);
      load_u(0, uv[0]);
    }
    load_u(1, uv[1]);
    fill_selectors();
    dequant_step(rows[0], meta[0], frag[0]);
    gen_phi(uv[0], sTile[0]);

    auto step = [&](auto T, int k) {
      constexpr int t = decltype(T)::value;          // k mod 4
      __syncthreads();     // tile k is complete; every wave is done reading tile k-1
      if (k + 1 < n_steps) dequant_step(rows[(t + 1) & 1], meta[(t + 1) & 3], frag[(t + 1) & 1]);   // step k+1 fragments
      if constexpr (STAGE && (t & 1) == 0) {
        // the pair of steps k+2, k+3 arrived behind the codewords that the fragments above waited for
        if (k + 2 < n_steps) {
          stage_commit(mraw);
          stage_read_into(k + 2, 0, meta[(t + 2) & 3].id, meta[(t + 2) & 3].g, meta[(t + 2) & 3].b);
          stage_read_into(k + 3, 1, meta[(t + 3) & 3].id, meta[(t + 3) & 3].g, meta[(t + 3) & 3].b);
          if (k + 4 < n_steps) stage_issue((k >> 1) + 2, mraw);                                     // steps k+4, k+5
        }
      }
      if (k + 2 < n_steps) gather_rows(meta[(t + 2) & 3], rows[t & 1]);                             // step k+2 codewords
      if constexpr (!STAGE) {
        if (k + 4 < n_steps) load_meta(k + 4, meta[t & 3]);                                         // step k+4 metadata
      }
      mfma_step(sTile[t & 1], frag[t & 1]);
      if (k + 1 < n_steps) gen_phi(uv[(t + 1) & 1], sTile[(t + 1) & 1]);                            // step k+1 basis tile
      if (k + 2 < n_steps) load_u(k + 2, uv[t & 1]);
    };
    for (int k = 0; k < n_steps; k += 4) {
      step(std::integral_constant<int, 0>{}, k);
      if (k + 1 < n_steps) step(std::integral_constant<int, 1>{}, k + 1);
      if (k + 2 < n_steps) step(std::integral_constant<int, 2>{}, k + 2);
      if (k + 3 < n_steps) step(std::integral_constant<int, 3>{}, k + 3);
    }

  }

  // ---- epilogue.  D layout of the 32x32 MFMA: lane holds column (lane & 31), rows
  //      8*(r/4) + 4*(lane/32) + r%4 for r = 0..15 -------------------------------------------
  const float bs = bsum + __shfl_xor(bsum, 32);      // both lane halves: all 8 input rows
  const float oscale = F32 ? 1.0f : scale;
  float* dst = a.dst + (long long)head * a.dst_head_stride + (long long)chunk * a.dst_chunk_stride;
  if constexpr (T16) {
    // D layout of the 16x16 MFMA: lane holds column (lane % 16) of its block, rows 4 * (lane / 16) + r
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      float bs16 = bsum2[T16 ? cb : 0];                // the four lane groups: all 8 input rows
      bs16 += __shfl_xor(bs16, 16);
      bs16 += __shfl_xor(bs16, 32);
      const int col = t16_col(2 * cb);
      if (col < n_out) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int b = b0 + 4 * kg + r;
          if (b < B) {
            float v = acc4[T16 ? cb : 0][r] + bs16;    // (the scale went in with the gains)
            if (a.apply_tanh) v = tanhf(v);
            dst[(long long)b * n_out + col] = v;
          }
        }
      }
    }
    return;
  }
  if (j_ok) {
#pragma unroll
    for (int m = 0; m < MBLK; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int b = b0 + m * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
        if (b < B) {
          float v;
          if constexpr (kSplit) v = fmaf(1.0f / 2048.0f, acc_x[m][r], acc[m][r]) + bs;   // (the scale went in with the gains)
          else v = fmaf(oscale, acc[m][r], bs);
          if (a.apply_tanh) v = tanhf(v);
          dst[(long long)b * n_out + jc] = v;
        }
      }
  }
}

#ifndef KAN_FUSED_CH
#define KAN_FUSED_CH 0          // 1: this translation unit holds the kernels with chained input (launch_fused_chained)
#endif

#if KAN_FUSED_CH
template <typename IdxT, typename GbT, typename CbT>
hipError_t launch_variant(const FusedArgs& a, bool f32, int mblk, bool stage_ok, dim3 grid, hipStream_t s) {
  if (mblk != 1) return hipErrorInvalidValue;
  const bool stage = stage_ok && sizeof(GbT) <= 2;
  const unsigned lds = 32u * (unsigned)a.rows_per_chunk * 4u;       // the chunk's inputs of the tile's 32 sample rows
  if (f32 && a.B <= 16) {                    // 16-sample tiles
    if (stage) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 1, true, true, true>), grid, dim3(kThreads), lds, s, a);
    else hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 1, false, true, true>), grid, dim3(kThreads), lds, s, a);
  } else if (f32) {
    if (stage) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 1, true, false, true>), grid, dim3(kThreads), lds, s, a);
    else hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 1, false, false, true>), grid, dim3(kThreads), lds, s, a);
  } else {
    if (stage) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, false, 1, true, false, true>), grid, dim3(kThreads), lds, s, a);
    else hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, false, 1, false, false, true>), grid, dim3(kThreads), lds, s, a);
  }
  return hipGetLastError();
}
#else
template <typename IdxT, typename GbT, typename CbT>
hipError_t launch_variant(const FusedArgs& a, bool f32, int mblk, bool stage_ok, dim3 grid, hipStream_t s) {
  // In the shallow pipeline the staged loads pay off for one- and two-byte gains and biases; with fp32 ones
  // (two 16-byte loads per array and pair, 20 more registers) config 2 at batch 16 went from 21.0 to 27.1 us.
  const bool stage = stage_ok && sizeof(GbT) <= 2;
  if (f32 && mblk == 1 && a.B <= 16) {       // 16-sample tiles
    if (stage) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 1, true, true>), grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 1, false, true>), grid, dim3(kThreads), 0, s, a);
  } else if (f32) {
    if (mblk == 1 && stage) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 1, true>), grid, dim3(kThreads), 0, s, a);
    else if (mblk == 1) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 1, false>), grid, dim3(kThreads), 0, s, a);
    else if (stage) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 2, true>), grid, dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, true, 2, false>), grid, dim3(kThreads), 0, s, a);
  } else {
    if (mblk == 1 && stage) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, false, 1, true>), grid, dim3(kThreads), 0, s, a);
    else if (mblk == 1) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, false, 1, false>), grid, dim3(kThreads), 0, s, a);
    else if constexpr (sizeof(CbT) != 4) {            // (fp32 rows keep two steps of codewords in flight: not staged)
      if (stage_ok) hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, false, 2, true>), grid, dim3(kThreads), 0, s, a);
      else hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, false, 2, false>), grid, dim3(kThreads), 0, s, a);
    } else {
      hipLaunchKernelGGL((kan_fused_kernel<IdxT, GbT, CbT, false, 2, false>), grid, dim3(kThreads), 0, s, a);
    }
  }
  return hipGetLastError();
}
#endif

template <typename IdxT>
hipError_t launch_types(const GatherCfg& c, const FusedArgs& a, bool f32, int mblk, bool stage, dim3 grid, hipStream_t s) {
  if (c.code == kCbI8) {
    if (c.gb_kind == kGbQ8) return launch_variant<IdxT, q8_t, int8_t>(a, f32, mblk, stage, grid, s);
    return c.gb_kind == kGbF16 ? launch_variant<IdxT, __half, int8_t>(a, f32, mblk, stage, grid, s)
                               : launch_variant<IdxT, float, int8_t>(a, f32, mblk, stage, grid, s);
  }
  if (c.gb_kind == kGbQ8) return hipErrorInvalidValue;      // byte-coded gain/bias go with Int8 codebooks
  if (c.code == kCbBfp8)
    return c.gb_kind == kGbF16 ? launch_variant<IdxT, __half, bfp8_t>(a, f32, mblk, stage, grid, s)
                               : launch_variant<IdxT, float, bfp8_t>(a, f32, mblk, stage, grid, s);
  if (c.code == kCbF16)
    return c.gb_kind == kGbF16 ? launch_variant<IdxT, __half, __half>(a, f32, mblk, stage, grid, s)
                               : launch_variant<IdxT, float, __half>(a, f32, mblk, stage, grid, s);
  return c.gb_kind == kGbF16 ? launch_variant<IdxT, __half, float>(a, f32, mblk, stage, grid, s)
                             : launch_variant<IdxT, float, float>(a, f32, mblk, stage, grid, s);
}

}  // namespace

#if KAN_FUSED_CH
hipError_t launch_fused_chained(const GatherCfg& c, const FusedArgs& a, bool f32, dim3 grid, hipStream_t s) {
  if (c.code == kDense || a.B < 1 || c.bt != 32) return hipErrorInvalidValue;
  // what the kernel's 16-byte loads of the slices and its tile of inputs in LDS assume
  if (a.x_parts < 2 || a.x_parts > kFusedChainMaxParts || a.n_in % 4 != 0 || a.rows_per_chunk % 4 != 0 ||
      a.rows_per_chunk < 4 || 32ll * a.rows_per_chunk > kFusedChainFloats || a.x_part_stride % 4 != 0 ||
      a.x_head_stride % 4 != 0 || (uintptr_t)a.x % 16 != 0)
    return hipErrorInvalidValue;
#else
hipError_t launch_fused(const GatherCfg& c, const FusedArgs& a, bool f32, dim3 grid, hipStream_t s) {
  if (c.code == kDense || a.B < 1 || (c.bt != 32 && c.bt != 64)) return hipErrorInvalidValue;
  if (a.x_parts > 1) return hipErrorInvalidValue;       // slices of the input: launch_fused_chained
#endif
  const int mblk = c.bt / 32;
  // the staged metadata loads need rows of the per-edge arrays that are whole 16-byte units
  bool stage = a.n_out % 16 == 0;
  for (unsigned h = 0; h < grid.z && stage; ++h)
    stage = ((uintptr_t)a.h[h].idx % 16 == 0) && ((uintptr_t)a.h[h].gain % 16 == 0) && ((uintptr_t)a.h[h].bias % 16 == 0);
  return c.idx_u32 ? launch_types<uint32_t>(c, a, f32, mblk, stage, grid, s)
                   : launch_types<uint16_t>(c, a, f32, mblk, stage, grid, s);
}

}  // namespace kan
