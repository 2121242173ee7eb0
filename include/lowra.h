/*
 * lowra.h -- C ABI of the MI355X (gfx950) LowRA hot path.
 *
 * LowRA (arXiv 2502.08141) quantizes the frozen base weight W [N,K] (N output channels, K input
 * features, fp32 row-major) at a precision chosen PER OUTPUT CHANNEL from {1,2,4} bits
 * (Sec. 4.1 "Per-Output-Channel Quantization", Sec. 6.2), with 64-element groups along K that
 * are each normalised by their absmax (Sec. 4.1 "Groupwise Normalization"), per-channel sorted
 * thresholds ("bin edges") for encoding and per-channel mappings (representative values) for
 * decoding (Sec. 4.1 "Per-Output-Channel Thresholds and Mappings").  App. A describes the two
 * primitives (quantize, dequantize); every LoRA step then evaluates the frozen linear on the
 * decoded weights (Sec. 3, Sec. 2.1).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) pointers, "host" pointers are host memory.
 *   - bf16 tensors are passed as uint16_t bit patterns.
 *   - The caller owns every buffer.  The library allocates device memory only inside
 *     lowra_layout_create (a few small index arrays; freed in lowra_layout_destroy) and
 *     lowra_fwd_batch_create (the batch's descriptors; freed in lowra_fwd_batch_destroy).
 *   - Every compute call enqueues on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and returns without synchronising.
 *   - Errors are returned as lowra_status; nothing throws or aborts.  Arguments are validated
 *     on the host only; device data is never scanned.  Preconditions on device data
 *     (finite W, ascending thresholds) are the caller's.
 *   - Base pointers must be 16-byte aligned (LOWRA_MISALIGNED otherwise).
 *
 * Tables.  `thresholds` and `mappings` are [C][16] fp32, one row per codebook.  A codebook of
 * b bits uses the first 2^b - 1 thresholds (ascending; the rest are ignored) and the first 2^b
 * mappings.  codebook_id[n] selects the row used by channel n, so C == N gives the paper's
 * one-table-per-channel model and a small C gives shared tables.  Thresholds are read only by
 * lowra_quantize, mappings only by the decoding calls.
 *
 * Packed layout (App. A writes each channel's codes at an offset that follows from the
 * precisions; the byte order below is this library's).  Channel n owns bytes [row_offset[n], row_offset[n] + K*bits[n]/8) where
 * row_offset is the exclusive prefix sum in channel order; inside a row, code k occupies bits
 * [k*b, (k+1)*b) of the row's bit stream, stream bit i being bit (i mod 8) of byte (i div 8).
 */
#ifndef LOWRA_H
#define LOWRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int lowra_status;
enum {
    LOWRA_OK = 0,
    LOWRA_INVALID_ARG = 1,         /* null pointer, non-positive size, inconsistent tables */
    LOWRA_UNSUPPORTED = 2,         /* group != 64, bits outside {1,2,4}, K % 64 != 0, ... */
    LOWRA_MISALIGNED = 3,          /* a base pointer is not 16-byte aligned */
    LOWRA_WORKSPACE_TOO_SMALL = 4, /* workspace_bytes < lowra_workspace_bytes(...) */
    LOWRA_HIP_ERROR = 5,           /* a HIP runtime call or kernel launch failed */
    LOWRA_OUT_OF_MEMORY = 6        /* a host allocation inside the library failed */
};

enum { LOWRA_OP_LINEAR_FWD = 0, LOWRA_OP_LINEAR_BWD_INPUT = 1, LOWRA_OP_ADAPTER_GRADS = 2, LOWRA_OP_LOFTQ_INIT = 3 };
enum { LOWRA_OUT_BF16 = 0, LOWRA_OUT_FP32 = 1 };
enum { LOWRA_PATH_AUTO = 0, LOWRA_PATH_GEMV = 1, LOWRA_PATH_GEMM = 2, LOWRA_PATH_GEMV_GENERAL = 3 };

/* Static description of a status code. */
const char* lowra_status_string(lowra_status st);

/* Opaque description of one quantized matrix: the part of the paper's "quantization state"
 * (Sec. 3) that is not a tensor -- shape, per-channel precisions ("Precs", App. A), table
 * indices, row offsets. */
typedef struct lowra_layout lowra_layout;

/* Host-only helper: row_offset_host[N+1] = exclusive prefix sum of K*bits[n]/8 (bytes).
 * Touches no device.  Errors: INVALID_ARG (null, N < 0, K <= 0), UNSUPPORTED (group != 64,
 * K % 64 != 0, a width outside {1,2,4}, more than 4 GiB of codes). */
lowra_status lowra_plan_rows(int N, int K, int group, const uint8_t* bits_host,
                             int64_t* row_offset_host);

/* Build a layout from HOST arrays and upload its index arrays to the current device.
 *   bits_host[N]          precision of each output channel, in {1,2,4}
 *   codebook_id_host[N]   table row of each channel, in [0,C)
 *   codebook_bits_host[C] precision each table row was built for; must equal bits of every
 *                         channel that selects it (INVALID_ARG otherwise)
 * All host validation happens before the first HIP call.  On success *out owns a few small
 * device arrays until lowra_layout_destroy.  HIP_ERROR if no device is usable. */
lowra_status lowra_layout_create(int N, int K, int group, const uint8_t* bits_host,
                                 const int32_t* codebook_id_host, int C,
                                 const uint8_t* codebook_bits_host, lowra_layout** out);
void lowra_layout_destroy(lowra_layout* layout);

/* Type of the stored group scales (Sec. 4.1 "Groupwise Normalization" does not fix it).  LOWRA_SCALE_FP32
 * (default): absmax is fp32 [N,K/64].  LOWRA_SCALE_BF16: the group's maximum is rounded to bf16 (nearest
 * even; a maximum that would round to infinity keeps the largest finite bf16) BEFORE it normalises the
 * group, and that value is stored and multiplies the decoded level: absmax is then uint16 bf16 bit
 * patterns [N,K/64] (2 instead of 4 bytes per group: 0.28 instead of 0.31 B per weight at 2.0 bits),
 * passed through the same `absmax` parameters (declared float*), 16-byte aligned as before.  Host
 * only; set it before the layout's first use and keep it for the life of the quantized state.
 * With bf16 scales lowra_quantize, lowra_dequantize, lowra_linear_fwd(_static) and
 * lowra_linear_bwd_input work as documented (the streaming small-token kernels read the bf16 scales
 * as they are; the other kernels run on a copy widened into the call's workspace, which
 * lowra_workspace_bytes accounts for); the batch entry points take them when every matrix of the
 * batch has bf16 scales and runs the streaming kernel (else LOWRA_UNSUPPORTED); lowra_loftq_init
 * returns LOWRA_UNSUPPORTED.  INVALID_ARG: null layout, unknown dtype. */
enum { LOWRA_SCALE_FP32 = 0, LOWRA_SCALE_BF16 = 1 };
lowra_status lowra_layout_set_scale_dtype(lowra_layout* layout, int scale_dtype);

/* Size in bytes of the packed code buffer: sum_n K*bits[n]/8 (the paper's bit accounting,
 * Sec. 6.2).  0 for a null layout. */
size_t lowra_packed_bytes(const lowra_layout* layout);

/* Device scratch a linear call needs (op = LOWRA_OP_*), for M tokens and LoRA rank r.
 * It holds the rank-r intermediate and padded copies of the adapter operands; for the forward with
 * M <= 16 also the small-token kernel's descriptors and per-chunk partial outputs, so it can be
 * non-zero at r == 0. */
size_t lowra_workspace_bytes(const lowra_layout* layout, int op, int M, int r);

/* Quantize (App. A.1).  For every 64-element group: absmax a = max|w| is stored; every weight is
 * normalised as u = w * (1/a) (one IEEE fp32 reciprocal per group, u = 0 when a == 0) and coded
 * as the number of its channel's thresholds strictly below u; codes are bit-packed at the
 * channel's width into the layout above.  4-bit channels find that number by bisection, which is the same
 * number for ascending thresholds (equal neighbours allowed); with thresholds out of order -- a violated
 * precondition -- the code is some value below 16 and nothing else goes wrong.  The same holds for the 4-bit
 * binning of lowra_channel_mse and lowra_learn_tables.
 *   W [N,K] fp32 dev (in) | thresholds [C][16] fp32 dev (in)
 *   packed lowra_packed_bytes(layout) dev (out) | absmax [N,K/64] fp32 dev (out; bf16 bit patterns when the
 *   layout's scale type is LOWRA_SCALE_BF16, here and in every call below) */
lowra_status lowra_quantize(const lowra_layout* layout, const float* W, const float* thresholds,
                            uint8_t* packed, float* absmax, void* stream);

/* The same quantization (App. A.1) of `count` matrices -- a decoder layer's, say -- with as few launches as
 * possible (eight matrices each): results are bit for bit those of `count` calls of lowra_quantize, without the
 * idle gap between two launches on a stream (2-3 us, a tenth of the time of a 4096 x 4096 matrix).
 *   layouts, W, thresholds, packed, absmax: HOST arrays of `count` entries; entry i holds the arguments that
 *   lowra_quantize takes for matrix i (device pointers, same shapes, alignment and scale type rules; the
 *   layouts may differ in every respect).  The arrays are read before the call returns.  Output ranges of
 *   different matrices must not overlap.
 * Nothing is launched unless every entry is valid: INVALID_ARG for count < 0, a null array, a null layout or
 * thresholds entry, or a null W / packed / absmax entry of a matrix with channels; MISALIGNED as in
 * lowra_quantize.  Matrices without channels are skipped; count == 0 is a no-op.  Allocates nothing. */
lowra_status lowra_quantize_batch(int count, const lowra_layout* const* layouts, const float* const* W,
                                  const float* const* thresholds, uint8_t* const* packed, float* const* absmax,
                                  void* stream);

/* Dequantize (App. A.2): What[n,k] = mappings[codebook_id[n]][code] * absmax[n,k/64], one fp32
 * multiply, written as fp32 (LOWRA_OUT_FP32) or rounded to nearest-even bf16 (LOWRA_OUT_BF16).
 *   out [N,K] dev, row-major. */
lowra_status lowra_dequantize(const lowra_layout* layout, const uint8_t* packed,
                              const float* absmax, const float* mappings, int out_dtype,
                              void* out, void* stream);

/* Frozen-base LoRA linear, forward (Sec. 2.1, Sec. 3): y = x What^T + s (x A^T) B^T with What
 * decoded on the fly (never written to HBM), bf16 operands, fp32 accumulation, bf16 result.
 *   x [M,K] bf16 dev | A [r,K] bf16 dev | B [N,r] bf16 dev | y [M,N] bf16 dev (out)
 *   r == 0 drops the LoRA term (A, B may be null).  N % 8 == 0 is required (UNSUPPORTED).
 *   workspace: dev, >= lowra_workspace_bytes(layout, LOWRA_OP_LINEAR_FWD, M, r), 16-byte aligned;
 *   contents are scratch.  M <= 16 takes the bandwidth-bound small-token path. */
lowra_status lowra_linear_fwd(const lowra_layout* layout, const uint8_t* packed,
                              const float* absmax, const float* mappings, const uint16_t* x,
                              int M, const uint16_t* A, const uint16_t* B, int r, float s,
                              uint16_t* y, void* workspace, size_t workspace_bytes,
                              void* stream);

/* lowra_linear_fwd for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * results as lowra_linear_fwd (both paths, bit for bit) without `workspace`: the rank-r intermediate and
 * the padded adapter copy live in a static device array of LOWRA_STATIC_SCRATCH_BYTES that every GPU the
 * library runs on holds until the process ends.  The call allocates and frees nothing (no hipMalloc /
 * hipFree, no allocating library routine); the array's device address is looked up once per device, in
 * lowra_layout_create or at the first call on that device.
 *   WORKSPACE_TOO_SMALL: lowra_workspace_bytes(layout, LOWRA_OP_LINEAR_FWD, M, r) exceeds
 *   LOWRA_STATIC_SCRATCH_BYTES (e.g. more than 32768 tokens at rank 64) -- use lowra_linear_fwd.
 *   INVALID_ARG also when the current device is not the layout's.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race on it; calls on one stream are ordered and safe.  The array keeps the last call's
 * contents; the call needs nothing in it to start at zero. */
#define LOWRA_STATIC_SCRATCH_BYTES (4u << 20)
lowra_status lowra_linear_fwd_static(const lowra_layout* layout, const uint8_t* packed,
                                     const float* absmax, const float* mappings, const uint16_t* x,
                                     int M, const uint16_t* A, const uint16_t* B, int r, float s,
                                     uint16_t* y, void* stream);

/* Input gradient of the same layer: dX = dY What + s (dY B) A.  The base is frozen, so there is
 * no weight gradient (Sec. 3).
 *   dY [M,N] bf16 dev | dX [M,K] bf16 dev (out); other arguments as in lowra_linear_fwd. */
lowra_status lowra_linear_bwd_input(const lowra_layout* layout, const uint8_t* packed,
                                    const float* absmax, const float* mappings,
                                    const uint16_t* dY, int M, const uint16_t* A,
                                    const uint16_t* B, int r, float s, uint16_t* dX,
                                    void* workspace, size_t workspace_bytes, void* stream);

/* Mapping/threshold learner (Sec. 5 "Weighted Lloyd's for LoRA Quantization", App. G): for every
 * output channel, `iterations` rounds of weighted Lloyd-Max on its normalised weights
 * u = w * (1/absmax) (the quantizer's normalisation), each element weighted by its block's absmax,
 * started from the channel's initial tables (row codebook_id[n] of the two init arrays, App. F).
 * A round bins u by the current thresholds (the quantizer's rule), replaces every level by the
 * weighted mean of its bin (an empty bin keeps its level) and every threshold by the midpoint of
 * its two levels.  It stops early after the first round whose weighted mean squared error is not
 * below the previous one; the tables computed last are returned (Sec. 5).
 *   W [N,K] fp32 dev | init_thresholds, init_mappings [C][16] fp32 dev
 *   thresholds_out, mappings_out [N][16] fp32 dev (out): per-channel tables, unused entries +inf / 0
 *   mse_out [N][iterations+1] fp32 dev (out): error of the initial tables, then after each round
 *   (entries past an early stop repeat the last value).
 * The results feed lowra_quantize / lowra_dequantize through a layout with one table per channel
 * (C == N, codebook_id[n] == n).  UNSUPPORTED: K > 16384, iterations > 64.  A channel of zeros
 * keeps its initial tables. */
lowra_status lowra_learn_tables(const lowra_layout* layout, const float* W,
                                const float* init_thresholds, const float* init_mappings,
                                int iterations, float* thresholds_out, float* mappings_out,
                                float* mse_out, void* stream);

/* Threshold averaging (Sec. 5, last paragraph), in place on per-channel thresholds [N][16] fp32
 * dev: entry j of every b-bit channel becomes the mean of entry j over the matrix's b-bit
 * channels. */
lowra_status lowra_average_thresholds(const lowra_layout* layout, float* thresholds, void* stream);

/* Adapter gradients of the same layer (Sec. 2.1; only the low-rank tensors are trained, Sec. 3):
 *   dB[n,j] = s sum_m dY[m,n] (x A^T)[m,j]        dA[j,k] = s sum_m (dY B)[m,j] x[m,k]
 * bf16 operands, fp32 accumulation, fp32 results; the rank-r intermediates are rounded to bf16 as in
 * the two linear calls.  The quantized base does not enter (the layout supplies N and K).
 *   x [M,K], dY [M,N], A [r,K], B [N,r] bf16 dev | dA [r,K], dB [N,r] fp32 dev (out)
 *   workspace: dev, >= lowra_workspace_bytes(layout, LOWRA_OP_ADAPTER_GRADS, M, r), 16-byte aligned.
 * UNSUPPORTED: r > 64, N % 8 != 0.  M == 0 writes zeros. */
lowra_status lowra_adapter_grads(const lowra_layout* layout, const uint16_t* x, const uint16_t* dY,
                                 int M, const uint16_t* A, const uint16_t* B, int r, float s,
                                 float* dA, float* dB, void* workspace, size_t workspace_bytes,
                                 void* stream);

/* The same gradients from the rank-r intermediates the two linear calls of the step have already formed (Sec. 2.1: the
 * forward needs s x A^T, the input gradient s dY B), so that this call reads x and dY once and A, B not at all.
 * `lowra_linear_side_product` returns where a finished lowra_linear_fwd (op LOWRA_OP_LINEAR_FWD: s x A^T) or
 * lowra_linear_bwd_input (LOWRA_OP_LINEAR_BWD_INPUT: s dY B) call with the same M and r left its intermediate inside the
 * workspace that was passed to it: bf16 [M][64] dev, row-major, valid until that workspace is written again; NULL when
 * the call keeps none in that form (r == 0, r > 64, or M <= 16 unless LOWRA_PATH_GEMM is set: the small-token kernels).
 * A host-side computation: nothing is launched.
 *   x [M,K], dY [M,N] bf16 dev | st = s x A^T, su = s dY B: bf16 [M][64] dev (in), from the calls above on the SAME x, A, s
 *   and dY, B, s | dA [r,K], dB [N,r] fp32 dev (out), bit-identical to lowra_adapter_grads on the same inputs
 *   workspace: dev, >= lowra_workspace_bytes(layout, LOWRA_OP_ADAPTER_GRADS, M, r), 16-byte aligned, not the
 *   workspaces that hold st and su.
 * UNSUPPORTED: r > 64, N % 8 != 0.  M == 0 writes zeros. */
const uint16_t* lowra_linear_side_product(const lowra_layout* layout, int op, int M, int r, const void* workspace);
lowra_status lowra_adapter_grads_from_side(const lowra_layout* layout, const uint16_t* x, const uint16_t* dY, int M, int r,
                                           const uint16_t* st, const uint16_t* su, float* dA, float* dB,
                                           void* workspace, size_t workspace_bytes, void* stream);

/* Alternating low-rank initialisation of the adapter (Sec. 4.1, "Using LoftQ as low-rank initializer";
 * App. D; the paper runs five steps): from B A = 0, each step quantizes W - B A with the layout's widths
 * and the given tables (step 1 therefore quantizes W itself), decodes it, and fits B A of rank r to what
 * the quantized weights miss, W - What.  The paper takes that fit from an SVD; this library approximates
 * it by `power_iterations` rounds of block power iteration per step (products with E and E^T, rows of A
 * re-orthonormalised every round), started from `omega` in step 1 and from the previous A afterwards.
 * A has orthonormal rows and B = E A^T, so B A is the projection of E onto A's row space; any other split
 * of the same product is an equally valid reading of the paper.
 *   W [N,K] fp32 dev | thresholds, mappings [C,16] fp32 dev | omega [r,K] bf16 dev: the caller's random
 *   start (e.g. N(0,1)) | packed, absmax (out): the last step's quantized state, layout as lowra_quantize
 *   A [r,K], B [N,r] bf16 dev (out) | workspace: dev, >= lowra_workspace_bytes(layout,
 *   LOWRA_OP_LOFTQ_INIT, 0, r) (about 6 N K bytes), 16-byte aligned.
 * r == 0: plain quantization, A / B / omega / workspace unused.  UNSUPPORTED: r > 64, more than 64 steps
 * or rounds.  INVALID_ARG: steps < 1 or power_iterations < 1. */
lowra_status lowra_loftq_init(const lowra_layout* layout, const float* W, const float* thresholds,
                              const float* mappings, int r, int steps, int power_iterations,
                              const uint16_t* omega, uint8_t* packed, float* absmax, uint16_t* A,
                              uint16_t* B, void* workspace, size_t workspace_bytes, void* stream);

/* Per-channel error table (Sec. 6.1: each channel's MSE under 1-, 2- and 4-bit quantization):
 *   mse_out[n][p] = (1/K) sum_k (W[n,k] - mappings3[p][code] * absmax)^2,  p = 0, 1, 2 for 1, 2, 4 bits,
 * with absmax, normalisation and binning as in lowra_quantize and the fp32 decode of
 * lowra_dequantize, fused in one pass over W (nothing is packed).
 *   W [N,K] fp32 dev | thresholds3, mappings3 [3][16] fp32 dev (rows: 1, 2, 4 bits) | mse_out [N][3] fp32 dev (out)
 * UNSUPPORTED: K % 64 != 0. */
lowra_status lowra_channel_mse(int N, int K, const float* W, const float* thresholds3,
                               const float* mappings3, float* mse_out, void* stream);

/* Host only.  Greedy budgeted precision assignment, a stand-in for the two-level ILP of Sec. 6:
 * minimise sum_n params[n] * mse[n][p_n] subject to sum_n params[n] * bits[n] <= budget * sum_n
 * params[n].  Every channel starts at 1 bit; the upgrade (1 -> 2, then 2 -> 4 bits) with the
 * largest error reduction per added bit that fits the remaining budget and lowers the error is
 * applied until none is left; ties go to the lower channel.
 *   channel_params_host [N] (weights per channel; several matrices may be concatenated)
 *   mse_host [N][3] (lowra_channel_mse's layout) | bits_out_host [N] in {1,2,4} (out)
 * INVALID_ARG: budget below 1 bit per parameter, a non-positive channel size, null pointers. */
lowra_status lowra_assign_precisions(int N, const int64_t* channel_params_host, const float* mse_host,
                                     double budget_bits_per_param, uint8_t* bits_out_host);

/* Test hook: force the small-token path or the MFMA GEMM path of the two linear calls
 * regardless of M (LOWRA_PATH_*).  For M <= 16 LOWRA_PATH_AUTO and LOWRA_PATH_GEMV_GENERAL run the general
 * small-token kernel; LOWRA_PATH_GEMV runs the streaming kernel of the batched entry point on the single
 * matrix where its shape is supported (slower per call: its set-up is sized for many matrices), and makes
 * lowra_fwd_batch_create... use it as usual; LOWRA_PATH_GEMV_GENERAL keeps a batch on the general kernel.
 * Process-wide (one atomic); not for production use.  INVALID_ARG on an unknown value. */
lowra_status lowra_set_linear_path(int path);

/* Test and measurement hook: the output tiling of the forward fused GEMM (lowra_linear_fwd on the MFMA path).
 * The kernel covers the first cols_a 256-channel columns with token tiles of rows_a rows and the remaining
 * columns with tiles of rows_b rows (rows_* in {256, 192, 128}, rows_b <= rows_a; cols_a is clamped to the
 * matrix).  By default a planner picks the plan with the shortest estimated run time for the shape and
 * the device's compute-unit count; lowra_set_fwd_tiling(0, 0, 0) returns to that.  The results do not depend on
 * the plan (every output is the same sum in the same order).  Process-wide (one atomic); not for production use.
 * INVALID_ARG on any other value. */
lowra_status lowra_set_fwd_tiling(int rows_a, int rows_b, int cols_a);

/* Host only (touches no device): the plan the forward GEMM's planner picks for N output channels and M tokens on a
 * device with `compute_units` compute units, in the terms of lowra_set_fwd_tiling: the first *cols_a 256-channel
 * columns in token tiles of *rows_a rows, the others in tiles of *rows_b rows (*rows_a == *rows_b and *cols_a = all
 * columns for a single height).  A compute unit runs one tile at a time; the planner minimises the finish time of
 * the last tile with tile costs 1 : 0.80 : 0.62 for 256 : 192 : 128 rows.  INVALID_ARG: a non-positive size or a
 * null pointer. */
lowra_status lowra_plan_fwd_tiling(int N, int M, int compute_units, int* rows_a, int* rows_b, int* cols_a);

/* Several small-token forwards as one run (the operation of lowra_linear_fwd, Sec. 2.1 / Sec. 3, for
 * M <= 16 tokens on n independent matrices: e.g. the projections of one decoder layer that read the
 * same activations, or a pass over a whole weight set).  A single matrix at 1-2 bits is only a few MB,
 * less than the chip must have in flight to cover one memory round trip, so one launch per matrix cannot
 * stream at the memory's rate; here every pointer of every matrix is fixed when the batch is created
 * (descriptors in device memory), and a run is one launch for the rank-r partial sums plus one launch
 * per group of matrices that take the same kernel instantiation.  Per matrix the arithmetic is that of
 * lowra_linear_fwd on the small-token path (the contraction may be split over another number of
 * wavefronts: same sums, fp32 order may differ).
 *   items: host array of n entries (read during create only); every pointer in an item is a device
 *   pointer with the layout / dtype of the same argument of lowra_linear_fwd; the tensors must stay
 *   valid and in place for the life of the batch; items may share x, A, B but not y.
 *   mappings, M (1..16), r, s: shared by all items.  workspace: dev, >= lowra_fwd_batch_workspace_bytes,
 *   16-byte aligned, owned by the caller, used by every run (runs of one batch must not overlap).
 * create: INVALID_ARG (null / n <= 0 / M < 1), UNSUPPORTED (M > 16, r > 128, N % 8 != 0, K too long for
 * the small-token path: > 16384), MISALIGNED, WORKSPACE_TOO_SMALL, HIP_ERROR.  create allocates device
 * memory for the descriptors and copies them synchronously; run only launches; destroy frees. */
typedef struct lowra_fwd_item {
    const lowra_layout* layout;
    const uint8_t* packed;
    const float* absmax;
    const uint16_t* x;   /* [M,K] bf16 */
    const uint16_t* A;   /* [r,K] bf16, null when r == 0 */
    const uint16_t* B;   /* [N,r] bf16, null when r == 0 */
    uint16_t* y;         /* [M,N] bf16 (out) */
} lowra_fwd_item;
typedef struct lowra_fwd_batch lowra_fwd_batch;
size_t lowra_fwd_batch_workspace_bytes(int n, const lowra_fwd_item* items, int r);
lowra_status lowra_fwd_batch_create(int n, const lowra_fwd_item* items, const float* mappings, int M,
                                    int r, float s, void* workspace, size_t workspace_bytes,
                                    lowra_fwd_batch** out);
lowra_status lowra_fwd_batch_run(const lowra_fwd_batch* batch, void* stream);
void lowra_fwd_batch_destroy(lowra_fwd_batch* batch);

/* Several small-token input gradients as one run (the operation of lowra_linear_bwd_input, Sec. 2.1 /
 * Sec. 4.1, for M <= 16 tokens on n independent matrices).  Same contract as the forward batch above:
 * every pointer is fixed at create, a run is three launches (dY gathered into the kernel's channel
 * order and the partial sums of dY B; the streaming kernel; the sum of its partial results plus the
 * rank-r term, rounded to bf16).  Per matrix the result is that of lowra_linear_bwd_input up to the
 * order of the fp32 sums; the group scale multiplies dY (rounded to bf16) instead of the decoded level.
 *   items: as above with dY [M,N] in and dX [M,K] out; items may share A but not dX.
 *   Every matrix must take the streaming kernel: at most 4 (width, table) classes and 3 tables, K a
 *   multiple of 256 in [1024, 16384], r <= 32, and all layouts must agree on codebook_bits.
 * create: INVALID_ARG, UNSUPPORTED (a shape outside the above, M > 16), MISALIGNED, WORKSPACE_TOO_SMALL,
 * OUT_OF_MEMORY, HIP_ERROR.  create allocates device memory for the descriptors and copies them
 * synchronously; run only launches (runs of one batch must not overlap); destroy frees. */
typedef struct lowra_bwd_item {
    const lowra_layout* layout;
    const uint8_t* packed;
    const float* absmax;
    const uint16_t* dY;  /* [M,N] bf16 */
    const uint16_t* A;   /* [r,K] bf16, null when r == 0 */
    const uint16_t* B;   /* [N,r] bf16, null when r == 0 */
    uint16_t* dX;        /* [M,K] bf16 (out) */
} lowra_bwd_item;
typedef struct lowra_bwd_batch lowra_bwd_batch;
size_t lowra_bwd_batch_workspace_bytes(int n, const lowra_bwd_item* items, int M, int r);
lowra_status lowra_bwd_batch_create(int n, const lowra_bwd_item* items, const float* mappings, int M,
                                    int r, float s, void* workspace, size_t workspace_bytes,
                                    lowra_bwd_batch** out);
lowra_status lowra_bwd_batch_run(const lowra_bwd_batch* batch, void* stream);
void lowra_bwd_batch_destroy(lowra_bwd_batch* batch);

/* Measurement hook: while set, every quantize, dequantize and linear call records `start_event`
 * right before and `stop_event` right after the launch of its dominant kernel (the quantize or
 * dequantize kernel, the fused dequant GEMM, or the small-token kernel), on the call's stream, so
 * a benchmark can time that kernel alone.  Both are
 * hipEvent_t passed as void*; pass two nulls to clear.  Process-wide.  INVALID_ARG if exactly one
 * is null. */
lowra_status lowra_set_kernel_timer(void* start_event, void* stop_event);

/* Measurement kernels (not part of the hot path): the ceilings a benchmark prints beside the library's own
 * rates, measured on the same device in the same run.  All enqueue on `stream` and return.
 *   lowra_measure_copy: dst[0..bytes) = src[0..bytes), 16 bytes per lane, a contiguous 16 KB piece per workgroup (dev pointers, 16-byte
 *     aligned, bytes % 16 == 0): bytes read + bytes written per second is the copy ceiling.
 *   lowra_measure_read: streams src[0..bytes) once (result discarded; out4: 4 bytes of device scratch).
 *   lowra_measure_mfma: `workgroups` x 4 wavefronts each issue `iterations` x 4 independent
 *     v_mfma_f32_32x32x16_bf16 on registers; *flops_out (host, may be null) receives the flop count.
 *   lowra_measure_mfma_random: the same loop on operands that change with every instruction and hold pseudo-random
 *     bf16 values of order one (iterations % 4 == 0): the matrix pipe's sustained rate depends on what the data
 *     toggles, so this is the ceiling of a GEMM on real data, the constant-operand figure that of the pipe alone. */
lowra_status lowra_measure_copy(void* dst, const void* src, size_t bytes, void* stream);
lowra_status lowra_measure_read(const void* src, size_t bytes, void* out4, void* stream);
lowra_status lowra_measure_mfma(int workgroups, int iterations, void* out4, double* flops_out, void* stream);
lowra_status lowra_measure_mfma_random(int workgroups, int iterations, void* out4, double* flops_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LOWRA_H */
