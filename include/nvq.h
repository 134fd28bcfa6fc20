/*
 * nvq.h -- C ABI of libnvq: decode-time linear layers over int4
 * group-quantised weights on AMD MI355X (gfx950), each layer run as W4A16
 * or W4A8 under a per-layer precision map.
 *
 * The operations are the ones the paper's section "Per-Layer Precision
 * Dispatch and the W4A8 Path" and its appendix "CUDA Kernel Implementation
 * Details" describe; citations below name the passage that defines each one.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless marked "host".  The caller
 *     owns every buffer; the library allocates nothing.
 *   - Work is enqueued on the HIP stream passed as `stream` (a hipStream_t
 *     cast to void*, NULL = the default stream).  No call synchronises.
 *   - Return value: NVQ_OK or an error code; on error nothing was enqueued.
 *     Arguments are validated on the host before any launch.  Inputs are
 *     assumed finite; NaN/Inf are not checked.
 *   - Shapes: a linear layer has K inputs and N outputs, weights are [N][K]
 *     with K contiguous, K % 32 == 0, G = K / 32 groups per row, M tokens.
 *   - Device pointers must be 16-byte aligned (4-byte for fp32/int32 vectors
 *     and outputs, 2-byte for fp16 scales).
 *
 * Packed weight layout (shared by every entry point)
 *   qweight[n][g*16 + j], j < 16 : low nibble  = element k = 32 g + j,
 *                                  high nibble = element k = 32 g + 16 + j,
 *   stored nibble = signed code + 8 (code in [-8, 7]; the paper's block
 *   format centres the unsigned nibble at 8).  scales[n][g] holds IEEE
 *   binary16 bits.  18 bytes per 32 weights = 4.5 bits per weight, as in the
 *   paper, but nibbles and scales are two planes so that one 128-bit load
 *   fetches exactly one group.
 */
#ifndef NVQ_H
#define NVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    NVQ_OK = 0,
    NVQ_ERR_INVALID_ARG = 1, /* NULL pointer, unknown enum value */
    NVQ_ERR_SHAPE = 2,       /* N, K, M out of range, K % 32 != 0 */
    NVQ_ERR_ALIGN = 3,       /* pointer not aligned as stated above */
    NVQ_ERR_UNSUPPORTED = 4, /* valid request this build cannot run */
    NVQ_ERR_HIP = 5,         /* a HIP runtime call failed */
    NVQ_ERR_WORKSPACE = 6    /* workspace missing or too small */
};

enum { NVQ_F32 = 0, NVQ_BF16 = 1 };  /* y_dtype */
enum { NVQ_W4A8 = 0, NVQ_W4A16 = 1 }; /* precision */

/* Upper bounds accepted by the entry points. */
#define NVQ_MAX_M 32
#define NVQ_MAX_K 65536

/* Human-readable name of a status code (host pointer to a static string). */
const char *nvq_status_string(int status);

/* Text of the last HIP error seen by this thread's most recent failing call
 * (host pointer to a static buffer; empty string if none). */
const char *nvq_last_hip_error(void);

/*
 * nvq_pack_int4 -- quantise and pack weights (load time, not per token).
 * Paper: weight format paragraph of the W4A8 section (32-weight blocks, one
 * fp16 scale, nibbles centred at 8).  Scale rule (this build's reading, the
 * paper gives none): s = fp16_rne(absmax / 7); code = clamp(rne(w / s), -8, 7)
 * with IEEE binary32 division; a zero scale gives all-zero codes.
 *   W        [N][K] fp32, device, read only
 *   group    must be 32
 *   qweight  [N][K/2] u8, device, written
 *   scales   [N][K/32] fp16 bits, device, written
 * A block whose absmax/7 overflows fp16 gets an infinite scale and zero codes.
 */
int nvq_pack_int4(const float *W, int64_t N, int64_t K, int group,
                  uint8_t *qweight, uint16_t *scales, void *stream);

/*
 * nvq_quant_act_i8 -- dynamic int8 quantisation of activations.
 * Paper: appendix "F16 -> Q8 Activation Quantization": s = amax / 127,
 * q = round(x / s) clamped to [-127, 127]; the result is reused by every
 * matmul that reads the same input.  round = half-to-even, "/" = IEEE
 * binary32 division; activations are bfloat16.
 *   x_bf16    [M][K] bf16 bits, read only
 *   act_group 0  = one scale per token (xscale is [M]);
 *             32 = one scale per 32 elements, the paper's granularity
 *                  (xscale is [M][K/32])
 *   xq        [M][K] int8, written
 *   xscale    fp32, written
 *   xgsum     [M][K/32] int32, written: sum of the codes of each block of 32,
 *             the "sum_x" term of the paper's deferred bias correction.
 *             Required (the W4A8 GEMV consumes it).
 */
int nvq_quant_act_i8(const uint16_t *x_bf16, int M, int K, int act_group,
                     int8_t *xq, float *xscale, int32_t *xgsum, void *stream);

/*
 * nvq_gemv_w4a16 -- y[m][n] = sum_g s_w[n][g] * sum_{j<32} code[n][32g+j] * x[m][32g+j]
 * with bf16 activations, weights dequantised in registers, fp32 accumulate.
 * Paper: the W4A16 branch of the precision dispatch (kernel table, row
 * "matvec_w4a16": in-register dequantisation, cross-lane reduction, no
 * integer dot product).
 *   y        [M][N], fp32 or bf16 according to y_dtype, written
 */
int nvq_gemv_w4a16(const uint8_t *qweight, const uint16_t *scales, int N, int K,
                   const uint16_t *x_bf16, int M, void *y, int y_dtype, void *stream);

/*
 * nvq_gemv_w4a8 -- acc[m][n][g] = sum_{j<32} code[n][32g+j] * xq[m][32g+j]  (int32),
 * y[m][n] = xscale[m] * sum_g s_w[n][g] * acc[m][n][g]                (act_group 0)
 *         = sum_g s_w[n][g] * xscale[m][g] * acc[m][n][g]             (act_group 32)
 * Paper: W4A8 kernel description and appendix "W4A8 dp4a Matrix-Vector
 * Product": packed int8 dot products on the unsigned nibbles, int32
 * accumulate, then result = s_w * s_x * (sumi - 8 * sum_x).
 *   xq, xscale, xgsum  as written by nvq_quant_act_i8 with the same act_group
 *   acc_debug  NULL, or [M][N][K/32] int32 that receives every block
 *              accumulator (for bit-exact checks; slower)
 */
int nvq_gemv_w4a8(const uint8_t *qweight, const uint16_t *scales, int N, int K,
                  const int8_t *xq, const float *xscale, const int32_t *xgsum,
                  int act_group, int M, void *y, int y_dtype, int32_t *acc_debug,
                  void *stream);

/*
 * nvq_rms_norm_bf16 / nvq_silu_mul_bf16 -- the two elementwise neighbours of
 * the decode linears (paper: kernel table, the RMS-norm and SiLU-multiply
 * kernels; the paper names them without restating the formulas, the usual ones
 * are taken).  All tensors device, bf16 bits, 16-byte aligned, [M][K] except
 * gamma [K]; K % 32 == 0, M <= NVQ_MAX_M; every result is rounded to bf16 once.
 *   rms_norm: h = x (+ res if res != NULL, the sum rounded to bf16 and stored
 *             to h_out if h_out != NULL);
 *             out[m][k] = bf16(h[m][k] * gamma[k] / sqrt(mean_k(h[m]^2) + eps))
 *   silu_mul: out = bf16(g / (1 + exp(-g)) * u)
 * Sums of squares, the scale and exp are evaluated in binary32; against a
 * binary64 evaluation about one output in 10^4 differs by one bf16 unit.
 * Enqueue on `stream`.  Errors as for the other entry points.
 */
int nvq_rms_norm_bf16(const uint16_t *x, const uint16_t *res, const uint16_t *gamma, float eps,
                      int M, int K, uint16_t *out, uint16_t *h_out, void *stream);
int nvq_silu_mul_bf16(const uint16_t *g, const uint16_t *u, int M, int K, uint16_t *out,
                      void *stream);

/*
 * One linear layer of a decode step.  `precision` is the routing decision of
 * the paper's rule route(i) = W4A16 if normalised score >= tau else W4A8; all
 * linears of one transformer block carry their block's decision.
 * `in_op` names what stands between x_bf16 and the layer (the neighbouring
 * kernels of the paper's kernel table, applied while the input is prepared, so
 * that they cost no launch and no extra pass over memory):
 *   NVQ_IN_PLAIN     the layer reads x_bf16
 *   NVQ_IN_RMSNORM   the layer reads nvq_rms_norm_bf16(x_bf16, x2_bf16, gamma_bf16, eps)
 *                    (x2_bf16 may be NULL; with x2_bf16 the sum x + x2 goes to
 *                    h_out_bf16 if that is not NULL: the updated residual stream)
 *   NVQ_IN_SILU_MUL  the layer reads nvq_silu_mul_bf16(x_bf16, x2_bf16)
 */
enum { NVQ_IN_PLAIN = 0, NVQ_IN_RMSNORM = 1, NVQ_IN_SILU_MUL = 2 };
typedef struct nvq_linear {
    const uint8_t *qweight;  /* [N][K/2] */
    const uint16_t *scales;  /* [N][K/32] */
    int32_t N, K;
    const uint16_t *x_bf16;  /* [M][K] input of this layer */
    void *y;                 /* [M][N] output */
    int32_t y_dtype;         /* NVQ_F32 | NVQ_BF16 */
    int32_t precision;       /* NVQ_W4A8 | NVQ_W4A16 */
    int32_t in_op;           /* NVQ_IN_* */
    float eps;               /* NVQ_IN_RMSNORM */
    const uint16_t *x2_bf16;     /* [M][K] second operand, or NULL */
    const uint16_t *gamma_bf16;  /* [K] (NVQ_IN_RMSNORM) */
    uint16_t *h_out_bf16;        /* [M][K] or NULL (NVQ_IN_RMSNORM with x2_bf16) */
} nvq_linear;

/*
 * nvq_decode_linears -- walk a list of linears in order under its precision
 * map (the hot loop of one decode step, linear layers only).
 * Paper: routing rule of the precision-dispatch section; activation codes
 * are reused across projections that read the same input; the whole step is
 * issued without per-kernel host round trips (the paper's graph-capture
 * paragraph gives the reason).
 *   layers   host array of n entries (read during the call only)
 *   Entries complete in order: entry i may read what an earlier entry wrote.
 *   Consecutive entries with the same x_bf16, K and precision form a phase
 *   (at most four entries): they share one activation quantisation and run
 *   concurrently.  Results are those of running the phases one after the
 *   other: a phase whose input overlaps an earlier phase's output, or whose
 *   output overlaps an earlier phase's input or output, starts only after
 *   that phase has completed; phases that share no buffer may overlap.
 *   Inside a phase nothing is ordered: no output of a phase (y of each of its
 *   layers, h_out_bf16) may overlap what the phase reads (x_bf16, x2_bf16,
 *   gamma_bf16) or another of its outputs; such a list is refused with
 *   NVQ_ERR_INVALID_ARG.
 *   workspace  device buffer of at least nvq_decode_workspace_bytes(...)
 *              bytes, 256-byte aligned; its contents are scratch.
 * At M = 1 the whole list runs as ONE persistent kernel that keeps streaming
 * the weights of coming phases while a phase is being set up (needs every
 * K <= 14336).  In that kernel an input operand (x_bf16, or x2_bf16 of an input
 * transform) that is exactly the bf16 output y of one earlier layer (same
 * address, N of that layer = K of this one), or exactly the h_out_bf16 of an
 * earlier phase, and has not been written since, is handed over "by mail": the
 * producing waves post each value a second time, tagged, in the workspace, and
 * the consumers poll those words instead of waiting for flags and reading the
 * caller's buffer (which still receives every output).  This is the fast way
 * for the links of a real decode step (output projection -> next norm, gate
 * and up -> SiLU-multiply, down projection -> next block); all other
 * dependencies wait through per-workgroup flags.  The persistent kernel may
 * take two neighbouring phases in the other order: where a phase reads what its
 * predecessor writes and the phase after it shares no buffer with either, that
 * one goes first, so that the waves have work while the results travel (a
 * decode step whose attention runs elsewhere has one such phase per block, the
 * output projection).  Phases that share no buffer give the same results in
 * any order; NVQ_PLAN_ORDERED keeps the list's order.  At 2 <= M <= 32 with per-token activation scales and every
 * K a multiple of 128, phases that do not depend on each other share two or
 * three launches on the matrix cores.  Otherwise one or two launches per phase
 * are enqueued.  All give the same results (up to the fp32 summation order).
 * nvq_decode_linears copies its tables to the device on every call (blocking
 * copies: the phase table, a few KiB, and at M = 1 one byte per streaming wave
 * and phase, ~0.4 MB for 129 phases); a plan does that once.  At M = 1 the
 * workspace also reserves that table for the largest grid (13312 bytes per
 * phase).
 * nvq_decode_workspace_bytes returns 0 for invalid arguments.
 * The persistent kernels wait for each other with bounded spins; a wait that
 * gives up (the grid was not co-resident, say because another stream held
 * compute units) sets a status word in the workspace and leaves the outputs
 * invalid.  nvq_decode_linears itself does not look at it (it does not
 * synchronise): nvq_decode_status synchronises `stream` and reports the word of
 * the last walk that used `workspace` (the uint32 at byte
 * NVQ_WORKSPACE_STATUS_OFFSET; plan creation clears it).
 */
#define NVQ_WORKSPACE_STATUS_OFFSET 4096
size_t nvq_decode_workspace_bytes(const nvq_linear *layers, int n, int M, int act_group);
int nvq_decode_linears(const nvq_linear *layers, int n, int M, int act_group,
                       void *workspace, size_t workspace_bytes, void *stream);
int nvq_decode_status(const void *workspace, void *stream, int *timed_out);

/*
 * nvq_decode_linears_static -- the same walk for callers that cannot allocate
 * device memory or pass a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It only enqueues kernels
 * (one or two launches per phase plus one per input transform; no copies, no
 * hipMalloc / hipFree, no allocating library call), so it is slower than the
 * persistent kernel of nvq_decode_linears but can be captured.  The
 * activation codes, scales and code sums of the phase being run (and its
 * transformed input) live in a device array inside the library, one copy of
 * NVQ_STATIC_SCRATCH_BYTES per GPU held until the process ends; a list that
 * needs more (M * maxK * 3 bytes with input transforms, M * maxK without, plus
 * M * maxK / 4) is refused with NVQ_ERR_WORKSPACE.  Results equal those of
 * nvq_decode_linears up to the fp32 summation order.  Every call on a GPU
 * uses that GPU's one array: calls that overlap on one GPU (two streams, two
 * threads) race; issue them on one stream.  Nothing has to be cleared between
 * calls (a phase writes what it reads there before reading it).
 */
#define NVQ_STATIC_SCRATCH_BYTES (2u << 20)
int nvq_decode_linears_static(const nvq_linear *layers, int n, int M, int act_group,
                              void *stream);

/*
 * Plans: the same walk, prepared once and run many times (the role graph
 * capture plays in the paper's decode loop).  A plan is a small host object
 * (the only thing the library allocates, with new/delete); it keeps a copy of
 * the layer list and owns nothing on the device.  The workspace must stay
 * untouched by others between nvq_plan_create and nvq_plan_destroy, and runs
 * of one plan must not overlap (issue them on one stream).
 *   nvq_plan_create  validates, uploads the phase table on `stream`.  flags:
 *                    NVQ_PLAN_ORDERED makes every phase wait for the one
 *                    before it even when they share no buffer (the timing of
 *                    a fully dependent chain on independent inputs)
 *   nvq_plan_run     enqueues one walk on `stream`
 *   nvq_plan_info    streaming = 1 if the persistent kernel is used, 2 or 3 if
 *                    the walk is issued as grouped small-batch launches (two
 *                    per batch of independent phases; 3: the product runs as
 *                    a persistent grid fed through LDS rings, which needs
 *                    every K a multiple of 512 and 16-byte aligned scale
 *                    rows), 0 for launches per phase;
 *                    waits = number of phases that wait for an earlier phase,
 *                    through flags or for mail (grouped launches: number of
 *                    batch boundaries)
 *   nvq_plan_status  synchronises `stream` and reports whether a wait inside
 *                    a persistent kernel gave up (its spins are bounded so
 *                    that a grid that cannot be co-resident ends with an
 *                    error instead of a hang); outputs are invalid then.
 *                    *timed_out = 0, or a code: low byte = which wait (1 flags
 *                    of an earlier phase, 2 a prepared input, 3 room for an
 *                    input in local memory, 4 its announcement, 5 mail; the
 *                    small-batch kernel: 1), the bits above it = the phase
 *                    (mail: 2 * phase + 0 for x, + 1 for x2)
 *   nvq_plan_trace   diagnostic: give a device buffer of phases * 8 uint64
 *                    (or NULL to stop); later runs of the persistent kernel
 *                    store workgroup 0's timestamps per phase in it (100 MHz
 *                    wall clock), taken by its first wave (phases in which
 *                    that wave has no rows and no barrier keep what was there).
 *                    A buffer of workgroups * phases * 8 words (workgroups =
 *                    compute units of the device) makes every workgroup
 *                    record, workgroup after workgroup.  Per phase:
 *                    [0] phase entered, [1] flags seen (phases that wait),
 *                    [2] input staged, [3] the workgroup's share of the
 *                    operands has arrived (phases that wait; phases that
 *                    publish through flags: all waves done), [4] published (or:
 *                    the first of two mail operands has arrived),
 *                    [5] this wave's share of the operands has arrived,
 *                    [6] rows done by the last of the workgroup's waves (clear
 *                    the buffer before the walk: it is a running maximum),
 *                    [7] own rows done
 */
typedef struct nvq_plan nvq_plan;
enum { NVQ_PLAN_DEFAULT = 0, NVQ_PLAN_ORDERED = 1 };
int nvq_plan_create(const nvq_linear *layers, int n, int M, int act_group, int flags,
                    void *workspace, size_t workspace_bytes, void *stream, nvq_plan **plan);
int nvq_plan_run(nvq_plan *plan, void *stream);
int nvq_plan_info(const nvq_plan *plan, int *streaming, int *phases, int *waits);
int nvq_plan_status(nvq_plan *plan, void *stream, int *timed_out);
int nvq_plan_trace(nvq_plan *plan, uint64_t *buf, size_t bytes);
/*
 * nvq_plan_describe -- the host-side planning of a walk, without touching a
 * device (for inspection and tests; the pointers in `layers` are only compared
 * and checked for alignment, never followed).  `workgroups` = compute units the
 * persistent kernel would use.  out (host, out_words int32): [0] phases,
 * [1] the number of streaming waves the rows are dealt to if the list
 * qualifies for the persistent kernel, else 0; then 16 words per
 * phase, in the order the kernel takes them (see nvq_decode_linears): first
 * entry, entries, the latest earlier phase it must wait for (-1:
 * none; in the persistent kernel: through the flags, operands that arrive by
 * mail do not count), and for the persistent kernel: published (someone waits
 * for it through the flags),
 * rows, rows per wave, waves with one more row, the wave that gets the first
 * of those, offset of the activation image in the LDS image area, the latest
 * phase whose image it overwrites there (-1: none), image bytes, 1 if the
 * image is prepared in the prologue, the unit the rows are dealt in (that many
 * neighbouring rows go to the same wave, and the two counts before count units:
 * more than 1 where an independent phase has too few rows to give every wave a
 * few KiB), and 2 if neighbouring rows are streamed in pairs (K = 3072 with an
 * even number of rows in every layer of the phase), else 0, and 1 if the order
 * the waves are dealt rows in runs over the workgroups first (phases that wait
 * or are waited for), 0 if over the waves of a workgroup first, and which
 * operands the phase takes from a mailbox instead of the caller's buffer (bit 0:
 * x, bit 1: x2; see nvq_decode_linears), bit 2: it posts an output or its
 * residual sum as mail.
 * NVQ_ERR_WORKSPACE if out is too small.
 */
int nvq_plan_describe(const nvq_linear *layers, int n, int M, int act_group, int flags,
                      int workgroups, int32_t *out, int out_words);
/*
 * nvq_plan_describe_skips -- likewise the skip table of the persistent batch-1
 * kernel: out (host) receives workgroups * 12 rows (workgroup * 12 + streaming
 * wave; the kernel counts its workgroups XCD by XCD for this: of a grid of a
 * multiple of 8, workgroup b is number (b mod 8) * grid / 8 + b / 8) of *stride
 * bytes; byte p of a row = the number of phases from p on (at
 * most 255) that the wave passes without a look: it has no rows in them, they
 * wait for nobody and nobody waits for them.  One row per workgroup follows:
 * byte p = 1 if all its waves pass phase p (its loader wave then leaves that
 * phase's activations where they are), else 0.  *stride = 0 and nothing written if
 * the list does not qualify for that kernel; NVQ_ERR_WORKSPACE if out is too
 * small (out_bytes < workgroups * 13 * stride, stride = phases + 4 rounded up to 4).
 */
int nvq_plan_describe_skips(const nvq_linear *layers, int n, int M, int act_group, int flags,
                            int workgroups, uint8_t *out, size_t out_bytes, int *stride);
/*
 * nvq_plan_describe_batches -- likewise for the grouped small-batch launches
 * (M > 1): out[0] = batches of mutually independent phases (0 if the list does
 * not qualify for the matrix-core kernels), out[1] = 1 if the persistent kernel
 * serves them; then 24 words per batch: first and last phase, units (pairs of
 * 16-row tiles), input jobs, workgroups and parts of the persistent kernel,
 * 9 words unit index at which each part begins (the last one = units; unused:
 * -1), 9 words phase of the unit at each cut.  The grid assumes the current
 * device's compute units (256 without a device).
 */
int nvq_plan_describe_batches(const nvq_linear *layers, int n, int M, int act_group, int flags,
                              int32_t *out, int out_words);
void nvq_plan_destroy(nvq_plan *plan);

/*
 * nvq_dequant_bf16 -- dense bf16 weights for the prefill / large-batch path
 * (paper: kernel table, the dequantisation kernel that materialises 16-bit
 * weights for a library GEMM).  out[n][k] = bf16(code[n][k] * scale[n][k/32]),
 * rounded to nearest even once (the product is exact in binary32).
 *   qweight  device, [N][K/2], layout of nvq_pack_int4, 16-byte aligned
 *   scales   device, [N][K/32] fp16 bits
 *   out_bf16 device, [N][K] bf16 bits, 16-byte aligned, owned by the caller
 * Enqueues on `stream`; K % 32 == 0.  Errors: NVQ_ERR_INVALID_ARG (null
 * pointer), NVQ_ERR_SHAPE, NVQ_ERR_ALIGN, NVQ_ERR_HIP.
 */
int nvq_dequant_bf16(const uint8_t *qweight, const uint16_t *scales, int64_t N, int64_t K,
                     uint16_t *out_bf16, void *stream);

/*
 * nvq_gemm_w4a16 -- the prefill / large-batch product (paper: kernel table,
 * dequantise to 16-bit weights, then a dense GEMM; limitations: large batches
 * are bound by compute).  y[m][n] = sum_k x[m][k] * wd[n][k] with wd the bf16
 * weights nvq_dequant_bf16 would store, bf16 x bf16 products accumulated in
 * fp32 on the matrix cores (the summation order is the kernel's); the dense
 * weights are never written to memory.  For any M >= 1; meant for M of a few
 * hundred and more (below that the batch-1 and small-batch paths read the
 * weights once and are faster).  Note that the weights are rounded to bf16
 * here, as in the paper's prefill path, and are not in nvq_gemv_w4a16.
 * Two kernels: tiles of 256 tokens x 256 rows when K % 256 == 0, the scales
 * are 16-byte aligned and the output has at least 32 of them, tiles of 256 x
 * 128 otherwise (the environment
 * variable NVQ_GEMM_TILE = wide | narrow overrides the choice where both can
 * run; both add the same products in the same order).  On an MI355X the 8B
 * block's projections at 4096 tokens (q+k+v, o, gate+up, down as one launch
 * each) run at 1.1-1.2 PFLOP/s, 47 % of the bf16 matrix peak; the paper's own
 * route, weights dequantised with nvq_dequant_bf16 and a library bf16 GEMM on
 * them, reaches 1.3-1.45 PFLOP/s on the same machine (1.3-1.4 with the
 * dequantisation repeated in every step) and is the faster one wherever the
 * dense copy (2 bytes per weight instead of 0.5625) fits; this kernel is for
 * where it does not.
 *   qweight  device, [N][K/2], layout of nvq_pack_int4, 16-byte aligned
 *   scales   device, [N][K/32] fp16 bits
 *   x_bf16   device, [M][K] bf16 bits, 16-byte aligned
 *   y        device, [M][N] f32 or bf16 (y_dtype), owned by the caller
 * Enqueues on `stream`; K % 32 == 0.  Errors: NVQ_ERR_INVALID_ARG (null
 * pointer, y_dtype), NVQ_ERR_SHAPE, NVQ_ERR_ALIGN, NVQ_ERR_HIP.
 */
int nvq_gemm_w4a16(const uint8_t *qweight, const uint16_t *scales, int64_t N, int64_t K,
                   const uint16_t *x_bf16, int64_t M, void *y, int y_dtype, void *stream);

/*
 * Calibration statistics of the paper's Algorithm 1 (Monte Carlo activation
 * profiling), run once per model over a few prompts, not per decoded token.
 *
 * nvq_token_norms -- the magnitude Algorithm 1 takes per layer and token:
 * out[m] = sqrt(sum_n a[m][n]^2 + sum_n b[m][n]^2), the Euclidean norm of the
 * rows of a and b side by side (query and value projection outputs for the
 * attention proxy; the feed-forward output alone, b = NULL, Nb = 0, for the
 * other).  a [M][Na], b [M][Nb]: device, f32 or bf16 (dtype, the y_dtype
 * constants), e.g. the y buffers of a decode list; out: device, M floats.
 * Sums in fp32.  Enqueues on `stream`.
 *
 * nvq_mcap_scores -- host code: the score line.  a_attn, a_ffn (host, [L][T]):
 * the magnitudes of the L layers for the tokens of k prompts one after the
 * other, prompt_len[j] tokens each (T their sum); scores[i] = mean over the
 * prompts of the mean over a prompt's tokens of (a_attn + a_ffn).  Its output
 * feeds nvq_precision_from_scores.
 * Errors: NVQ_ERR_INVALID_ARG (null pointer, dtype), NVQ_ERR_SHAPE (sizes or a
 * prompt length <= 0), NVQ_ERR_ALIGN, NVQ_ERR_HIP.
 */
int nvq_token_norms(const void *a, int Na, const void *b, int Nb, int M, int dtype, float *out,
                    void *stream);
int nvq_mcap_scores(const float *a_attn, const float *a_ffn, const int *prompt_len, int k, int L,
                    double *scores);

/*
 * nvq_precision_from_scores -- host helper: the normalise-and-assign tail of
 * the paper's Algorithm 1.  scores (host, L doubles) are min-max normalised;
 * if max - min < eps every normalised score is 0; out[i] = NVQ_W4A16 if the
 * normalised score >= tau else NVQ_W4A8.  Pure host code, no GPU work.
 */
int nvq_precision_from_scores(const double *scores, int L, double tau, double eps,
                              int32_t *out);

/*
 * Measurement helpers (not part of the method): a streaming read that sums a
 * buffer into `out` (8 bytes) and a plain copy, used to find the HBM ceiling
 * of the machine and to calibrate profiler byte counters.  bytes % 16 == 0.
 */
int nvq_stream_read(const void *src, size_t bytes, void *out, void *stream);
int nvq_stream_copy(void *dst, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NVQ_H */
