/*
 * kan.h - C-ABI of the MI355X (gfx950) forward pass of vector-quantised
 * Kolmogorov-Arnold layers (SHARe-KAN compression, LUTHAM-style runtime).
 *
 * What a layer computes (paper section 3 and Eq. (1), section 4.2):
 *     c_ij   = gain_ij * C[idx_ij] + bias_ij          reconstructed coefficients
 *     phi_ij = sum_m B_{m,3}(x_i) * c_ij[m]            cubic B-spline, G = 10
 *     y_j    = sum_i phi_ij(x_i)
 * with one K x G codebook C per layer (fp32, fp16, block floating point with 8-bit
 * mantissas, or Int8 with value = scale * q: the codebook precisions of Table 1; Int8 is the one-byte-per-coefficient
 * codebook of sections 4.3 / 5.4), splines on the
 * range [-1, 1] (App. A.1): 7 uniform intervals, 14 knots t_m = -1 + (m-3)*2/7.
 * Inputs are clamped to [-1, 1].  x = +1 belongs to the last interval.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  Descriptor
 *     structs (kan_vq_layer) live in HOST memory and are read during the call
 *     only.  The library never allocates, frees or keeps device memory: scratch
 *     space comes in through the caller's workspace (ws, ws_bytes), whose
 *     required size the *_workspace_bytes functions return (fixed buffers, no
 *     runtime malloc: paper section 4.3).  ws must be 256-byte aligned.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream).  No call synchronises the device or reads results back.
 *   - The forward calls keep no state between calls, on the host or on the device: calls
 *     from different host threads or on different streams are independent as long as each
 *     has its own workspace and output, and may overlap on the GPU (the timing hooks
 *     kan_prof_begin / kan_prof_end, and kan_vq_head_forward_static with its one scratch
 *     array per GPU, are the exceptions: see there).
 *   - Arguments are validated on the host first: every status but KAN_OK and
 *     KAN_ERR_LAUNCH means that nothing has been enqueued.  KAN_ERR_LAUNCH (the HIP
 *     runtime rejected a kernel launch) can come after earlier kernels of the same
 *     call are already on the stream; outputs and workspace are then undefined.
 *   - Layouts: x[B][in] and y[B][out] row-major fp32; per-edge arrays
 *     idx/gain/bias[in][out] with edge e = i*out + j (j fastest); codebook
 *     [K][10] row-major, unpadded; dense coefficients coef[in][out][10].
 *   - Every array is aligned to its element size; fp32 codebooks to 8 bytes, fp16 and
 *     block-floating-point codebooks to 4 bytes; else KAN_ERR_SHAPE.
 *   - idx values must be < K; they are not checked by the forward calls (use
 *     kan_vq_count_bad_indices).  y must not alias x or the workspace.
 *   - Value range on the matrix cores (KAN_PATH_MFMA at any batch; KAN_PATH_GATHER from
 *     batch 33, the dense baseline from batch 17): the coefficient operand is carried as
 *     fp16 numbers gain * q (Int8 codebooks, q the byte code) or gain * C (floating
 *     codebooks, dense coefficients), so these products must stay below 65504 in magnitude
 *     (gains up to about 515 with Int8 codes) or the result is infinite; products below
 *     6.1e-5 in magnitude keep fewer bits (the split form of the precise path: the 11 bits
 *     of its low part).  The stated bounds hold for layers whose |gain * q| or |gain * C| lie
 *     in [6.1e-5, 65504] or are 0; kan_vq_coef_range reports the range of a layer.  The
 *     vector-ALU, bucket and column kernels and the fused kernel on fp32 operands
 *     (KAN_PATH_GATHER up to batch 32) have no such limit.
 */
#ifndef KAN_MI355X_H
#define KAN_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum kan_status {
  KAN_OK = 0,
  KAN_ERR_NULL = 1,        /* a required pointer is NULL                          */
  KAN_ERR_SHAPE = 2,       /* a size is <= 0, too large, or inconsistent          */
  KAN_ERR_DTYPE = 3,       /* dtype code not allowed for that operand             */
  KAN_ERR_WORKSPACE = 4,   /* ws NULL, misaligned or smaller than required        */
  KAN_ERR_UNSUPPORTED = 5, /* G != 10, degree != 3, unknown path, ...             */
  KAN_ERR_LAUNCH = 6       /* the HIP runtime rejected a launch                   */
} kan_status;

typedef enum kan_dtype {
  KAN_F32 = 0, KAN_F16 = 1, KAN_I8 = 2, KAN_U16 = 3, KAN_U32 = 4,
  KAN_Q8 = 5,  /* gain and bias as one byte each: logarithmic gain code, linear bias code */
  KAN_BFP8 = 6 /* codebook rows in block floating point, 8-bit mantissas: see kan_vq_layer  */
} kan_dtype;

/* Which arithmetic carries the edge evaluation.
 *   KAN_PATH_GATHER  the precise path: fp32 operands, fp32 accumulation; matches the
 *                    float64 definition to ~1e-6 (bound 1e-5).  Batch 1: one 4-byte
 *                    codeword-window gather per edge on the vector ALUs; from batch 2:
 *                    fused gather + matrix-core kernel (fp32 operands up to batch 32; from
 *                    33 coefficients and basis weights split into high and low fp16 parts,
 *                    three products, fp32-grade sums); from batch 65 (129 for layers of
 *                    2^22 edges or more whose codebook is not fp32): the kernels of the fp16
 *                    path on such split operands.  Prepared layers (see kan_vq_prepare),
 *                    batch <= 4 (<= 3 for layers of 2^23 edges or more): codebook buckets
 *                    in LDS.
 *   KAN_PATH_MFMA    fp16 operands on the matrix cores, fp32 accumulation; ~3e-4
 *                    relative per layer (bound 2e-2).  Batch <= 64 (128 for those large
 *                    layers): fused gather + MFMA kernel; above: coefficients dequantised
 *                    once per call into the workspace in matrix-core operand order, then a
 *                    streaming contraction.
 *   KAN_PATH_AUTO    the precise path below batch 32, the fp16 path from there on.   */
typedef enum kan_path { KAN_PATH_AUTO = 0, KAN_PATH_GATHER = 1, KAN_PATH_MFMA = 2 } kan_path;

/* How a codeword's G = 10 numbers define the edge function C[k](x) of Eq. (1).
 *   KAN_RULE_BSPLINE3  coefficients of a cubic B-spline on 7 uniform intervals of [-1,1]
 *                      (App. A.1: the spline family of the models that are compressed).
 *   KAN_RULE_PLI2      the rule of the paper's runtime operator (sections 4.1, 4.3): samples at
 *                      the uniform nodes n_k = -1 + 2k/9; index floor((x+1)/dx) with
 *                      dx = 2/9, then linear interpolation between entries k and k+1.
 *                      x = +1 belongs to the last interval (k = 8, u = 1).
 * In both rules the weights of the entries sum to 1 on [-1,1], so gain * C[k](x) + bias
 * equals the rule applied to the reconstructed vector gain * C[k] + bias.               */
typedef enum kan_rule { KAN_RULE_BSPLINE3 = 0, KAN_RULE_PLI2 = 1 } kan_rule;

/* One VQ-KAN layer (Eq. (1)): host struct, device pointers. */
typedef struct kan_vq_layer {
  int32_t in, out;       /* N_in, N_out, both >= 1                                  */
  int32_t G, degree;     /* must be 10 and 3 (App. A.1), else KAN_ERR_UNSUPPORTED   */
  int32_t K;             /* codebook entries, >= 1; <= 65536 when idx is KAN_U16    */
  int32_t idx_dtype;     /* KAN_U16 | KAN_U32                                       */
  int32_t gb_dtype;      /* KAN_F32 | KAN_F16 | KAN_Q8 (gain and bias share it)     */
  int32_t cb_dtype;      /* KAN_F32 | KAN_F16 | KAN_I8 | KAN_BFP8                   */
  const void* idx;       /* [in][out]                                               */
  const void* gain;      /* [in][out]                                               */
  const void* bias;      /* [in][out]                                               */
  const void* codebook;  /* [K][10]; KAN_BFP8: [K] rows of 12 bytes (below)         */
  float scale;           /* Int8: value = scale * q.  Ignored for KAN_F32 and KAN_F16
                            codebooks (Table 1 lists FP32, FP16 and Int8 codebooks)  */
  int32_t rule;          /* KAN_RULE_BSPLINE3 (0) | KAN_RULE_PLI2                   */
  const void* prepared;  /* NULL, or the buffer kan_vq_prepare filled for this very
                            layer (small-batch path, see below)                     */
  /* KAN_Q8 only (section 4.2: gains on a logarithmic and biases on a linear Int8 grid, 16 bits
   * per edge beside the index; the paper prints no formula, this is the reading used here):
   *   gain[e] is an unsigned byte: 0 means 0, code c in 1..255 means
   *           exp2(gain_log2_lo + gain_log2_step * c);
   *   bias[e] is a signed byte:    bias_scale * c, c in -127..127.
   * Needs cb_dtype == KAN_I8 (the fully quantised 4-bytes-per-edge format), else
   * KAN_ERR_UNSUPPORTED.  Ignored for the other gain/bias dtypes.                            */
  float gain_log2_lo, gain_log2_step, bias_scale;
  int32_t flags;         /* 0, or KAN_LAYER_NO_COLUMN (below, with kan_vq_prepare)    */
  /* KAN_BFP8 codebooks (Table 1 lists a block-floating-point row between FP16 and Int8; the
   * paper defines no format, this is the one used here): a codeword row is one block of 12
   * bytes, 4-byte aligned: ten signed mantissa bytes q[0..9] in -127..127, one signed exponent
   * byte e in -126..127 shared by the row, one zero byte; entry m means q[m] * 2^e.  `scale` is
   * ignored.  Served by every kernel family, the prepared layout of kan_vq_prepare included
   * (buckets of 4096 such rows, 48 KB).                                                      */
} kan_vq_layer;

/* Spans and basis weights of step "index lookup" (section 4.1) for the cubic
 * family of App. A.1: for every x[n] (clamped to [-1,1]) the interval index
 * span[n] in 0..6 and the four nonzero Cox-de Boor weights w[n][0..3], which
 * multiply coefficients span..span+3.  Parity/debug entry point: it runs the device
 * routine of the vector-ALU and bucket kernels (exact comparisons of 7x with the
 * knots' numerators in fp64, weights in fp64 rounded once); the fused kernel and the
 * basis preparation of the streaming contraction use a second routine, which
 * kan_basis_window exposes.  x, span, w: device.  n >= 0 (n == 0 is a no-op).     */
kan_status kan_bspline_basis(const float* x, int64_t n, uint8_t* span, float* w, void* stream);

/* The same for KAN_RULE_PLI2: index[n] = k in 0..8 (the interval [n_k, n_k+1) that holds the
 * clamped x[n]; x = +1 gives 8) and w[n][0..1] = (1 - u, u), the weights of entries k, k+1.   */
kan_status kan_pli_basis(const float* x, int64_t n, uint8_t* index, float* w, void* stream);

/* The window of four consecutive codeword entries and their four weights, as the forward kernels
 * form it for either rule (sections 4.1 / 4.3 and App. A.1): start[n] = first entry (cubic rule:
 * the interval index 0..6; two-tap rule: min(k, 6), the taps 1 - u, u sitting at offset k - start,
 * the other two weights 0) and w[n][0..3].  variant 0: the routine of the vector-ALU and bucket
 * kernels (what kan_bspline_basis / kan_pli_basis run); variant 1: the routine of the fused kernel
 * and of the basis preparation (index by one fp64 fma and truncation, which is exact, weights in
 * fp32).  Both must give the same start for every fp32 x; parity/debug entry point.
 * x, start, w: device; w 16-byte aligned.                                                        */
kan_status kan_basis_window(const float* x, int64_t n, int32_t rule, int32_t variant, uint8_t* start, float* w,
                            void* stream);

/* Bytes of workspace kan_vq_layer_forward / kan_vq_head_forward need for these
 * descriptors (host array [n_heads][n_layers]), batch B and path.  Returns 0
 * when none is needed and (size_t)-1 when the arguments are invalid.            */
size_t kan_vq_workspace_bytes(const kan_vq_layer* layers, int32_t n_layers, int32_t n_heads,
                              int64_t B, int32_t path);

/* y[B][out] = forward of one VQ layer (section 3 sum over Eq. (1) edges).
 * B == 0 is a no-op returning KAN_OK.                                            */
kan_status kan_vq_layer_forward(const kan_vq_layer* L, const float* x, int64_t B, float* y,
                                void* ws, size_t ws_bytes, int32_t path, void* stream);

/* Dense-coefficient KAN layer (the uncompressed 40-bytes-per-edge form of
 * section 4.2): y[b][j] = sum_i sum_m B_m(x_bi) * coef[i][j][m].  G must be 10.
 * coef, x, y and ws are device pointers (ws 256-byte aligned, at least
 * kan_dense_workspace_bytes(in, out, B) bytes, (size_t)-1 for invalid sizes; contents need
 * not survive between calls).  Result within 1e-5 relative at every batch size: up to batch 16 an
 * fp32 FMA kernel, from 17 on the matrix cores on coefficients and basis weights split
 * into high and low fp16 parts (hi*hi + hi*lo + lo*hi), as the precise VQ path does.  */
size_t kan_dense_workspace_bytes(int32_t in, int32_t out, int64_t B);
kan_status kan_dense_layer_forward(const float* coef, int32_t in, int32_t out, int32_t G,
                                   const float* x, int64_t B, float* y,
                                   void* ws, size_t ws_bytes, void* stream);

/* One-time regrouping of a layer for the memory-bound small-batch regime (section 4.2:
 * batch-1 inference moves the per-edge metadata once; section 4.3: the codebook must be
 * served from on-chip memory).  The edges are regrouped by codebook bucket (8192 Int8,
 * 4096 fp16 or 2048 fp32 consecutive codewords, 80 KB: what one CU's LDS holds beside the
 * basis table, or 4096 block-floating-point rows, 48 KB; half of that for layers with more
 * than 2048 inputs),
 * then by output, then by input; per edge the buffer keeps (input index u16, codeword id
 * within the bucket u16, gain), and per output the sum of its biases (the bases sum to 1 on
 * [-1,1], so the bias term does not depend on x), and tables that cut the work into blocks
 * of about equal edge counts whatever the histogram of the codewords.  With L->prepared set, the precise path
 * serves batches up to 4 from this layout: every workgroup copies one bucket into LDS and
 * streams that bucket's edges, so no lookup leaves the CU.  Values are unchanged (same
 * products, different summation order: within the 1e-5 bound).
 * A small prepared layer (edges x samples at most 2^20) would leave such a workgroup with little
 * more than the wait for its bucket; it is served by one workgroup per output and sample instead,
 * which reads the output's ids and gains from a transposed copy that the buffer of a small layer
 * also holds, fetches the codeword windows from the L2-resident codebook and writes the finished
 * output (no partial sums).  KAN_LAYER_NO_COLUMN in L->flags keeps such a layer on the bucket kernel; the flags
 * of all heads of a layer must agree.
 *   kan_vq_prepared_bytes  size of the buffer; 0 if the layer is not eligible (in > 4096),
 *                          (size_t)-1 if the descriptor is invalid.
 *                          L->prepared is ignored.
 *   kan_vq_prepare         fills `prepared` (device, 256-byte aligned, >= that size) on
 *                          `stream`.  Requires in <= 4096 (else KAN_ERR_UNSUPPORTED).
 *                          The buffer depends on idx, gain, bias and the codebook's dtype
 *                          (not on the codebook values or scale) and must be rebuilt when
 *                          they change.  The caller owns it
 *                          and stores its address in L->prepared for later forward calls;
 *                          the codebook must then be 16-byte aligned, else the forward call
 *                          ignores the prepared buffer.                                  */
#define KAN_LAYER_NO_COLUMN 1
size_t kan_vq_prepared_bytes(const kan_vq_layer* L);
kan_status kan_vq_prepare(const kan_vq_layer* L, void* prepared, size_t prepared_bytes, void* stream);

/* n_heads independent heads of n_layers VQ layers each, applied to the same
 * x[B][in0] (multi-expert deployment, section 5.6); tanh between layers, none
 * after the last.  layers: host array [n_heads][n_layers]; layer l of every
 * head must have the same in/out/K/dtypes/rule (else KAN_ERR_UNSUPPORTED) and
 * out of layer l == in of layer l+1.  y: [n_heads][B][out_last].
 * n_heads <= 64 per call group is handled internally (any n_heads >= 1).        */
kan_status kan_vq_head_forward(const kan_vq_layer* layers, int32_t n_layers, int32_t n_heads,
                               const float* x, int64_t B, float* y,
                               void* ws, size_t ws_bytes, int32_t path, void* stream);

/* kan_vq_head_forward for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, kernels and results as kan_vq_head_forward, but the scratch regions (partial
 * sums, hidden activations, matrix-core operand records) live in a fixed array of
 * KAN_STATIC_SCRATCH_BYTES inside the library, one per GPU, which that GPU holds from the moment
 * the library's code is loaded there until the process ends.  The call allocates and frees
 * nothing (no hipMalloc / hipFree, no HIP objects); the first call on a device looks up the
 * array's address there.  Calls whose kan_vq_workspace_bytes exceeds KAN_STATIC_SCRATCH_BYTES are
 * rejected with KAN_ERR_WORKSPACE and enqueue nothing (small and medium batches fit: the
 * two-layer 2048 -> 1024 -> 256 head up to batch 64 on either path).  Nothing in the array has to
 * start at zero - every region is written before it is read within the call -, and it keeps the
 * last call's contents.  All calls on one GPU share the one array: calls that overlap in time on
 * the same GPU (different streams, or host threads) race on it; order them on one stream.      */
#define KAN_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
kan_status kan_vq_head_forward_static(const kan_vq_layer* layers, int32_t n_layers, int32_t n_heads,
                                      const float* x, int64_t B, float* y, int32_t path, void* stream);

/* Debug / parity: what the kernels' own load routines fetch for every edge.
 * ids[e] = zero-extended codeword id of edge e; rows[e][0..9] = dequantised
 * codeword (scale*q or the fp32 row) before gain/bias.  Either output may be
 * NULL.  ids, rows: device.                                                      */
kan_status kan_vq_debug_gather(const kan_vq_layer* L, uint32_t* ids, float* rows, void* stream);

/* Debug: *count (device uint32, overwritten) = number of edges with idx >= K.   */
kan_status kan_vq_count_bad_indices(const kan_vq_layer* L, uint32_t* count, void* stream);

/* Debug: the range of the fp16 coefficient operand of the matrix-core kernels for this layer
 * (the reconstructed coefficients of section 4.2 without bias and Int8 scale, which stay fp32):
 * range[0] = smallest nonzero and range[1] = largest magnitude of gain * q (Int8 codebooks, q the
 * byte code) or gain * C (floating codebooks) over all edges and their ten entries; +inf and 0
 * when every product is 0.  The matrix-core paths keep their bounds for ranges inside
 * [6.1e-5, 65504] (see the conventions above).  range: device, 2 floats, overwritten.            */
kan_status kan_vq_coef_range(const kan_vq_layer* L, float* range, void* stream);

/* Compression side (section 4.2, steps 1 and 3 of the post-training procedure; learning the
 * codebook itself, step 2, is not part of this library).  For every edge e = i*out + j of a dense
 * layer coef[in][out][10]:
 *   bias[e] = mean of the 10 coefficients, gain[e] = Euclidean norm of the centred grid
 *             (so that the normalised grid is zero-mean and unit-norm like the codebook shapes;
 *             the paper normalises to unit variance: same shapes, gains differ by sqrt(10));
 *   idx[e]  = index of the codebook row nearest (squared Euclidean distance) to the normalised
 *             grid; for an all-constant grid (gain 0) the row of smallest norm.
 * The distance contraction runs on the matrix cores with split fp16 operands (fp32-grade
 * scores, ~1e-6 relative): rows that near to a tie may resolve to either index.
 * codebook: fp32 [K][10]; idx: KAN_U16 (K <= 65536) or KAN_U32 array [in][out]; gain, bias:
 * fp32 [in][out].  ws: kan_vq_assign_workspace_bytes(K) bytes, 256-byte aligned.  All device. */
size_t kan_vq_assign_workspace_bytes(int32_t K);
kan_status kan_vq_assign(const float* coef, int32_t in, int32_t out, const float* codebook, int32_t K,
                         int32_t idx_dtype, void* idx, float* gain, float* bias,
                         void* ws, size_t ws_bytes, void* stream);

/* Reconstruction quality of an assignment ("R^2 between the original grids and the
 * reconstructed gain * C[idx] + bias", section 4.2): sums[0] = sum of squared residuals,
 * sums[1] = sum of all coefficients, sums[2] = sum of their squares (accumulated in fp64 in a
 * fixed order), and sums[3] = R^2 = 1 - sums[0] / (sums[2] - sums[1]^2 / (10 * in * out)),
 * the total sum of squares taken about the overall mean.  sums: device, 4 doubles.
 * ws: kan_vq_reconstruction_workspace_bytes(in, out) bytes, 256-byte aligned.               */
size_t kan_vq_reconstruction_workspace_bytes(int32_t in, int32_t out);
kan_status kan_vq_reconstruction_sums(const float* coef, int32_t in, int32_t out, const float* codebook,
                                      int32_t K, int32_t idx_dtype, const void* idx, const float* gain,
                                      const float* bias, double* sums, void* ws, size_t ws_bytes,
                                      void* stream);

/* Per-kernel timing with HIP events on the launch stream, for benchmarks.
 * kan_prof_begin creates up to max_launches event pairs (this is the one place
 * the library creates HIP objects) and brackets every kernel it launches from
 * then on.  kan_prof_end synchronises those events, aggregates by kernel name
 * (launches that belong to layer l = 1, 2, ... of a head call as "name@Ll")
 * into out[0..cap) (host), stores the number of distinct kernels in *n_out,
 * destroys the events and stops recording.  Not thread-safe.                     */
typedef struct kan_prof_record {
  char name[56];
  int32_t launches;
  float total_ms;
} kan_prof_record;
kan_status kan_prof_begin(int32_t max_launches);
kan_status kan_prof_end(kan_prof_record* out, int32_t cap, int32_t* n_out);

const char* kan_status_string(int32_t status);
/* Name of the kernel family the dispatcher would pick (for reports). */
const char* kan_vq_planned_kernel(const kan_vq_layer* L, int64_t B, int32_t n_heads, int32_t path);
const char* kan_dense_planned_kernel(int32_t in, int32_t out, int64_t B);

#ifdef __cplusplus
}
#endif
#endif /* KAN_MI355X_H */
