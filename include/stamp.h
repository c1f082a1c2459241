/*
 * stamp.h - C ABI of the MI355X (gfx950) STaMP quantized linear layer.
 *
 * STaMP (Sequence Transform and Mixed Precision, arXiv 2510.26771) wraps a linear layer as
 *
 *     Y = L^-1( Q(L X) W ) + 1 bias^T            (section "Method", commutation identity;
 *                                                  Algorithm "STaMP Linear")
 *
 * where L is an orthogonal transform along the sequence (token) dimension (here the Haar DWT of
 * section "Efficient Energy Concentration", 1-D over a token stream or 2-D over an image-token
 * grid), Q quantizes every transformed token with its own scale (Background, Eq. 1) at 8 bits
 * for the first k tokens and 4 bits for the rest (section "Optimal bit allocation"), and W is
 * quantized per output channel.
 *
 * General conventions
 *   - Every pointer whose name ends in _dev is DEVICE memory owned by the caller; _host is host
 *     memory.  The library never frees or keeps caller pointers beyond the call, except that
 *     stamp_plan_create reads W and bias asynchronously on the given stream (keep them alive
 *     until that stream has drained).
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  All compute
 *     calls are asynchronous on that stream and never synchronize it.
 *   - No call allocates device memory except stamp_plan_create (the plan owns its quantized
 *     weights until stamp_plan_destroy).  Scratch memory comes in through `workspace_dev`.
 *   - Every argument error is detected on the host BEFORE anything is launched and reported
 *     through the return code; nothing is launched in that case.  The compute calls only read the
 *     plan, so one plan may be used from several streams or host threads at once with distinct
 *     workspaces.  The two switches stamp_plan_set_unfused / stamp_plan_set_gemm_engine are the
 *     exception: they modify the plan, are meant for tests and measurements, and must not run while
 *     another thread uses the plan.
 *   - Non-finite inputs give unspecified numbers but never a fault.
 *
 * Tensor layouts
 *   X        [batch, seq_len, d_in]  row-major, d_in contiguous, dtype x_dtype.
 *   W        [d_in, d_out] row-major (w_is_out_by_in = 0) or [d_out, d_in] (= 1), dtype w_dtype.
 *   Y        [batch, seq_len, d_out] row-major, dtype y_dtype, original token order.
 *   Transformed tokens ("coefficients") are numbered in STaMP order: lowest frequencies first.
 *     1-D, J levels over s tokens: slots 0 .. s/2^J - 1 are the level-J approximations (sums of 2^J
 *     consecutive tokens / 2^(J/2)); slot p >= s/2^J with m = floor(log2 p) is the Haar wavelet of
 *     level log2(s) - m at position p - 2^m (+ on its first half, - on its second half).  With
 *     J = log2(s): slot 0 = sum/sqrt(s).
 *     2-D, J levels over a grid_h x grid_w grid, token t = r*grid_w + c: the level-J low-low block
 *     row-major, then for level J..1 the bands [difference along width, difference along height,
 *     diagonal], each row-major.
 *   The quantized activation is stored in the plan's PHYSICAL row order (a permutation of STaMP
 *   order chosen so that one GEMM tile holds whole Haar sub-trees); stamp_plan_row_of_coeff
 *   returns it.  With n_top = stamp_plan_hi_rows(plan) (k_hi, or the number of level-J approximations if
 *   that is larger), R = seq_len / n_top and physical row r of sequence b:
 *     scales  [batch, seq_len] float: scale of the coefficient at physical row r.  Plans with
 *             act_quant = STAMP_ACT_ASYMMETRIC use a buffer of [2][batch, seq_len] floats: the
 *             scales, then the integer offsets z (as floats) in the same order.
 *     q_hi    [batch, n_top, d_in] int8: STaMP slot p < n_top is row p of q_hi (its physical row is
 *             p*R): the k_hi 8-bit tokens and, when the transform leaves more approximations than
 *             k_hi, the remaining approximations, whose 4-bit codes are held as int8 values.
 *     q_lo    the 4-bit tokens at their physical row, two channels per byte (two's complement
 *             nibbles, low nibble = even channel), tiled for the GEMM: with m = b*seq_len + r the
 *             row over all sequences, Kp = d_in rounded up to 128 and Mp = batch*seq_len rounded
 *             up to 256, the byte of channels (c, c+1), c even, is at
 *               (((m / 256) * (Kp / 128) + c / 128) * 256 + m % 256) * 64 + (c % 128) / 2,
 *             i.e. [Mp/256][Kp/128][256 rows][64 bytes]; the buffer holds Mp * Kp / 2 bytes.
 *             Rows r with r % R == 0 (the rows whose coefficient lives in q_hi), rows >= batch *
 *             seq_len and channels >= d_in need not be filled: stamp_linear_forward_q ignores their
 *             content.  (stamp_quantize_act may write rows r % R == 0: it puts the packed form of the
 *             4-bit approximations there as well, for stamp_linear_forward's own use.)
 */
#ifndef STAMP_H_
#define STAMP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct stamp_plan stamp_plan_t; /* opaque, library-owned */

typedef enum {
  STAMP_OK = 0,
  STAMP_ERR_NULL = 1,        /* a required pointer is NULL */
  STAMP_ERR_SHAPE = 2,       /* sizes inconsistent: seq_len not 2^J, grid_h*grid_w != seq_len, k_hi > seq_len, ... */
  STAMP_ERR_UNSUPPORTED = 3, /* a valid STaMP setting this GPU library does not implement */
  STAMP_ERR_WORKSPACE = 4,   /* workspace_bytes < stamp_plan_workspace_bytes(plan) or workspace NULL/misaligned */
  STAMP_ERR_ALLOC = 5,       /* device allocation failed in stamp_plan_create */
  STAMP_ERR_DEVICE = 6       /* a HIP runtime call failed (no GPU, launch error) */
} stamp_status_t;

typedef enum { STAMP_F32 = 0, STAMP_BF16 = 1 } stamp_dtype_t;
/* Sequence transform L.  STAMP_L_IDENTITY: none (levels = 0), for the layers the paper leaves
 * un-transformed (Experiments set-up: inputs without sequence structure) and as the baseline the
 * transform's cost is measured against: tokens are quantized as they are, the first k_hi of every
 * sequence at bits_hi, STaMP order = physical row order = token order, nothing is inverted. */
typedef enum {
  STAMP_L_IDENTITY = 0,
  STAMP_L_HAAR1D = 1,
  STAMP_L_HAAR2D = 2,
  STAMP_L_WHT = 3, /* orthonormal Walsh-Hadamard transform along the tokens, rows in sequency order (levels = 0) */
  STAMP_L_DCT = 4  /* orthonormal DCT-II along the tokens (levels = 0), evaluated in fp64 and rounded to fp32 */
} stamp_xform_t;
/* Activation quantizer (Background, Eq. 1), per transformed token i with b bits:
 *   STAMP_ACT_SYMMETRIC   a = max_j |t_ij|, scale = a / (2^(b-1) - 1), code = rne(t * (1 / scale)) in
 *                         [-(2^(b-1) - 1), 2^(b-1) - 1]; de-quantized value code * scale.
 *   STAMP_ACT_ASYMMETRIC  Eq. 1 in full with the min-max range of the Background section (what the
 *                         Experiments set-up uses): lo = min_j t_ij, hi = max_j t_ij, range = hi - lo
 *                         (the token's own range, whether or not it contains 0; a token with hi = lo
 *                         takes range = |hi|), scale = range / (2^b - 1), integer offset
 *                         z = rne(-lo / scale) (any integer: negative for an all-positive token),
 *                         code = clamp(rne(t / scale) + z, 0, 2^b - 1); de-quantized value
 *                         (code - z) * scale.  The library STORES code - 2^(b-1) (two's complement
 *                         int8 / nibble) and returns z next to the scales.  Results are exact as
 *                         described while |z| < 2^22, i.e. |lo| / range < 2^22 / (2^b - 1).
 * Either way scale and its reciprocal are two fp32 divisions and rne is round-half-to-even. */
typedef enum { STAMP_ACT_SYMMETRIC = 0, STAMP_ACT_ASYMMETRIC = 1 } stamp_act_quant_t;

/* Everything the paper's statement of the layer leaves to the user: the shape of X (Background),
 * the transform L and its depth (section "Efficient Energy Concentration"), the number k of
 * high-precision tokens and the two bit widths (section "Optimal bit allocation"), and the
 * weight bit width. */
typedef struct {
  int32_t batch, seq_len, d_in, d_out;
  int32_t xform;            /* stamp_xform_t */
  int32_t levels;           /* Haar levels J, 1 <= J <= log2(seq_len) (2-D: log2 of the grid side) */
  int32_t grid_h, grid_w;   /* HAAR2D only; powers of two, grid_h*grid_w == seq_len (fast path: square) */
  int32_t k_hi;             /* tokens kept at bits_hi, 0 .. seq_len (fast path: a power of two, 2-D a power of four) */
  int32_t bits_hi, bits_lo, bits_w; /* 8, 4, 4 */
  int32_t x_dtype, y_dtype, w_dtype; /* stamp_dtype_t values; bf16 weights are widened exactly at plan time */
  int32_t w_is_out_by_in;   /* 0: W[d_in, d_out];  1: W[d_out, d_in] (the algorithm's X W^T) */
  int32_t act_quant;        /* stamp_act_quant_t: which form of Eq. 1 quantizes the activation */
  int32_t skip_first;       /* HAAR1D only: 1 = the first token of every sequence is left out of L (it is STaMP slot 0 as
                               it is; the transform runs over the other seq_len - 1 tokens), the paper's language-model
                               setting (appendix "Experimental details", LLMs) */
  int32_t bias_mode;        /* 0: Y = L^-1(..) + 1 bias^T (the algorithm's last step); 1: the transformed bias
                               (L 1) bias^T is added before the inverse (third form of the commutation identity) */
  int32_t group_size;       /* 0: one scale per token / per output channel; 64: per-block scales, one per 64 consecutive
                               input channels, for activations (per token) and weights (per output channel): the
                               W4A4 setting of the paper's image-model table */
} stamp_plan_desc_t;

/* Two implementations serve a plan.
 * FAST path (the benchmark configurations): HAAR1D on a power-of-two seq_len without skip_first, HAAR2D on a square
 * grid, IDENTITY, all with group_size 0 and bias_mode 0, and with a block structure the kernels have (listed below).
 * GENERAL path: everything else that is valid: HAAR1D of any seq_len (an odd number of approximations at a level: the
 * last one is carried to the next level unchanged; every level is the orthonormal butterfly (x0 +- x1) * fl(1/sqrt 2))
 * with 0 <= levels <= the depth that leaves one approximation, skip_first, HAAR2D on a rectangular grid (sides powers of
 * two), WHT (seq_len a power of two), DCT, bias_mode 1, group_size 64, and the HAAR1D / HAAR2D settings outside the
 * fast path's block structure (any 0 <= k_hi <= seq_len, any depth, any block size).  The transform runs as a few passes
 * (several levels each) over fp32 copies of the activation in the workspace, the quantizer and the GEMM treat the
 * transformed tokens as rows in STaMP order (physical row = STaMP slot), the inverse again runs in passes after the GEMM.
 * Limits of the general path (STAMP_ERR_UNSUPPORTED beyond them): bits 8/4/4; d_in a multiple of 32, at most 32768;
 * d_out at most 2^21 (both paths);
 * group_size 0 or 64, and 64 needs d_in a multiple of 64 and the symmetric quantizer; seq_len <= 65535, batch <= 65535,
 * batch * k_hi <= 65535 (grid dimensions); DCT: seq_len <= 16384 (a dense seq_len x seq_len matrix).  With group_size =
 * 64 the buffers of stamp_quantize_act / stamp_linear_forward_q are: q_hi [batch, seq_len, d_in] int8 codes of ALL
 * tokens in STaMP order (stamp_plan_hi_rows returns seq_len), q_lo unused (may be NULL), scales [batch, seq_len,
 * d_in / 64].
 *
 * Served by the fast path (any other valid setting goes to the general path, within its limits):
 *   xform IDENTITY with levels 0, any seq_len and 0 <= k_hi <= seq_len; or
 *   xform HAAR1D or HAAR2D (square grid) of any depth J, with n_top = max(k_hi, approximations left by J
 *   levels) <= 256 and seq_len/n_top in {8,16,32,64,128} (1-D) or {16,64} (2-D: 4x4 or 8x8 token blocks);
 *   k_hi a power of two (four in 2-D) when k_hi >= the number of approximations, any 0 <= k_hi below it
 *   (e.g. the 3-level transform of 2048 tokens with 64 8-bit tokens: 256 approximations, 192 of them at
 *   4 bits); in that second case n_top may exceed 256 (3 levels on 8192 tokens: 1024 approximations);
 *   bits 8/4/4;
 *   d_in a multiple of 32 and at most 32768 (above 8192, or 4096 for fp32 input or 2-D grids, the transform
 *   + quantization kernel splits the channels over workgroups and reads X twice: row ranges, then codes);
 *   act_quant symmetric or asymmetric; batch <= 65535 and batch * n_top <= 65535 (grid dimensions of the
 *   transform kernels). */

/* Validates desc, quantizes W per output channel (absmax/7, round to nearest even; section
 * "Large Language Models", Set-up: round-to-nearest weights, one scale per output channel) into
 * the layout the GEMM kernel reads, copies bias (fp32 [d_out], may be NULL).
 * W_dev, bias_dev: device, read on hip_stream.  *out receives the plan. */
stamp_status_t stamp_plan_create(const stamp_plan_desc_t* desc, const void* W_dev,
                                 const float* bias_dev_or_null, void* hip_stream,
                                 stamp_plan_t** out);

/* Frees the plan's device memory.  The caller must have drained every stream using it. */
stamp_status_t stamp_plan_destroy(stamp_plan_t* plan);

/* Bytes of workspace any entry point below may need (256-byte aligned pointer expected). */
size_t stamp_plan_workspace_bytes(const stamp_plan_t* plan);

/* Rows per sequence of the q_hi buffer: max(k_hi, number of approximation coefficients the J-level
 * transform leaves); k_hi for plans without transform; 0 for a NULL plan. */
int32_t stamp_plan_hi_rows(const stamp_plan_t* plan);

/* host_out[p] = physical row (0 <= row < seq_len) of STaMP slot p; a permutation. */
stamp_status_t stamp_plan_row_of_coeff(const stamp_plan_t* plan, int32_t* host_out);

/* Steps 1-2 of Algorithm "STaMP Linear": T = L X along the tokens, then per-token quantization of
 * Eq. 1 in the form the plan's act_quant selects (see stamp_act_quant_t), at 8 bits for the first
 * k_hi STaMP slots and 4 bits for the rest.  Outputs in the layouts above.
 * One quantized activation may feed several linears (the paper's q/k/v fan-out). */
stamp_status_t stamp_quantize_act(const stamp_plan_t* plan, const void* X_dev, int8_t* q_hi_dev,
                                  uint8_t* q_lo_dev, float* scales_dev, void* workspace_dev,
                                  size_t workspace_bytes, void* hip_stream);

/* The whole layer, Algorithm "STaMP Linear": quantize_act, the integer GEMM on the matrix cores (the
 * exact integer sums under either engine, see stamp_plan_set_gemm_engine; the default is the FP6 pipeline
 * for the 4-bit rows and the int8 pipeline for the 8-bit rows), dequantization, inverse transform, bias,
 * store Y.  The 8-bit rows' integer sums are converted to fp32 exactly while 128 * 7 * d_in < 2^24
 * (d_in <= 18720); on wider layers a sum beyond 2^24 (only reachable by adversarial inputs) is rounded
 * to fp32 (relative 2^-24) before it is scaled. */
stamp_status_t stamp_linear_forward(const stamp_plan_t* plan, const void* X_dev, void* Y_dev,
                                    void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* stamp_linear_forward for callers that cannot allocate or pass device scratch memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation and same kernels; the
 * scratch memory is a static device array of STAMP_STATIC_SCRATCH_BYTES inside the library (one per GPU, held
 * until the process ends) instead of a caller workspace.  The call allocates nothing.  A plan whose
 * stamp_plan_workspace_bytes exceeds STAMP_STATIC_SCRATCH_BYTES is refused with STAMP_ERR_WORKSPACE before
 * anything is launched.  Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU
 * (different streams or threads) race; issue them on one stream, or order them with events.  Nothing in the
 * array has to be cleared between calls (each call writes what it later reads). */
#define STAMP_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
stamp_status_t stamp_linear_forward_static(const stamp_plan_t* plan, const void* X_dev, void* Y_dev,
                                           void* hip_stream);

/* Steps 3-5 from an already quantized activation (buffers as written by stamp_quantize_act). */
stamp_status_t stamp_linear_forward_q(const stamp_plan_t* plan, const int8_t* q_hi_dev,
                                      const uint8_t* q_lo_dev, const float* scales_dev, void* Y_dev,
                                      void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* Step 4 alone: Y = L^-1 Yt for Yt_dev [batch, seq_len, n_cols] fp32 in STaMP order; adds the
 * plan's bias (after the inverse, whatever bias_mode says) when n_cols == d_out and a bias was given;
 * Y_dev [batch, seq_len, n_cols] y_dtype.  Workspace: batch * stamp_plan_hi_rows(plan) * n_cols * 4 bytes on the
 * fast path; on the general path two buffers of batch * seq_len * n_cols * 4 bytes, each rounded up to 256.
 * Yt_dev is only read.  STAMP_ERR_UNSUPPORTED for a fast-path plan without transform. */
stamp_status_t stamp_inverse(const stamp_plan_t* plan, const float* Yt_dev, int32_t n_cols,
                             void* Y_dev, void* workspace_dev, size_t workspace_bytes,
                             void* hip_stream);

/* ---- parity / debug exports (not on the timed path) ---- */

/* Step 3 alone: acc_dev[b*seq_len + p, n] = sum_c code[b, p, c] * qW[c, n], int32, rows in STaMP
 * order; `code` is the STORED code (asymmetric plans: the unsigned code minus 2^(b-1)).  With the FP6
 * engine selected the converted operand lives in a temporary that this call allocates and frees. */
stamp_status_t stamp_debug_gemm_acc(const stamp_plan_t* plan, const int8_t* q_hi_dev,
                                    const uint8_t* q_lo_dev, int32_t* acc_dev, void* hip_stream);

/* The plan's weight codes [d_in, d_out] int8 (values -7..7) and scales [d_out] (group_size = 64: [d_in / 64][d_out]),
 * copied to host.  Synchronizes the device. */
stamp_status_t stamp_debug_weight_codes(const stamp_plan_t* plan, int8_t* qW_host, float* sw_host);

/* Launches ONE stage of stamp_linear_forward on its own, so that a benchmark can time it between
 * two events (buffers exactly as stamp_linear_forward lays them out; q_hi/q_lo/scales as written by
 * stamp_quantize_act, workspace as used by the preceding stages).  stage:
 *   0 bottom-levels transform + 4-bit quantization kernel   1 top levels + 8-bit rows
 *   2 GEMM of the 8-bit rows                                3 top levels of the inverse
 *   4 GEMM of the 4-bit rows (with the fused inverse unless the plan is set unfused)
 *   5 in-block inverse kernel (unfused plans only)
 *   6 conversion of the packed 4-bit rows to the FP6 engine's operand layout (FP6 engine only; with
 *     that engine stage 4 is the GEMM alone and reads what stage 6 wrote to the workspace)
 * Plans whose transform has no levels above the blocks: stage 0 also quantizes the block sums, stage 2 writes
 * the block sums of the inverse itself, stages 1 and 3 launch nothing.
 * Plans without transform: 0 the quantization kernel, 2 GEMM of the 8-bit rows, 3 their output pass,
 * 6 and 4 as above; 1 and 5 return STAMP_ERR_UNSUPPORTED. */
stamp_status_t stamp_debug_run_stage(const stamp_plan_t* plan, int32_t stage, const void* X_dev,
                                     int8_t* q_hi_dev, uint8_t* q_lo_dev, float* scales_dev,
                                     void* Y_dev, void* workspace_dev, size_t workspace_bytes,
                                     void* hip_stream);

/* Selects the implementation of steps 3-5: 0 = GEMM with the dequantization and the in-block
 * inverse transform fused into its epilogue (default where the shape allows it), 1 = GEMM writing
 * dequantized fp32 rows to the workspace followed by a separate inverse kernel.
 * For tests and measurements: it modifies the plan (not thread-safe, no call on the plan may be in
 * progress on another host thread) and changes stamp_plan_workspace_bytes, which must be queried again. */
stamp_status_t stamp_plan_set_unfused(stamp_plan_t* plan, int32_t unfused);

/* Matrix pipeline that multiplies the 4-bit rows (step "Y <- X W" of Algorithm "STaMP Linear" for the
 * rows quantized to bits_lo = 4 against the 4-bit weights).  Both compute the same integer sums
 * acc[m, n] = sum_c code[m, c] * qW[c, n] exactly, so every result of the library is bit-identical
 * under either setting (one exception, to fp32 rounding: in plans without top levels that keep fewer 8-bit
 * tokens than approximations, stamp_linear_forward under STAMP_GEMM_FP6 multiplies the 4-bit approximations
 * in one piece, where the other setting may add them up from dequantized partial sums over parts of the depth):
 *   STAMP_GEMM_FP6   (default) the codes as 6-bit floating point numbers code / 8 (E2M3, exact),
 *                    FP6 x FP6 -> fp32 MFMA, twice the int8 rate per clock; the fp32 accumulator holds
 *                    acc / 64 exactly (|acc| <= 49 d_in < 2^24).  Costs one conversion pass over the
 *                    packed rows inside stamp_linear_forward(_q);
 *   STAMP_GEMM_INT8  the codes as int8, int8 x int8 -> int32 MFMA.
 * The 8-bit rows always run on the int8 pipeline.  May be changed between calls (it modifies the plan:
 * not thread-safe, no call on the plan may be in progress on another host thread); the workspace size
 * does not depend on it.  Returns STAMP_ERR_UNSUPPORTED for any other value. */
typedef enum { STAMP_GEMM_INT8 = 0, STAMP_GEMM_FP6 = 1 } stamp_gemm_engine_t;
stamp_status_t stamp_plan_set_gemm_engine(stamp_plan_t* plan, int32_t engine);

/* Measurement aid (not part of the layer): the rate, in 1e12 operations per second, that the matrix
 * pipeline of `engine` sustains on the current device over pseudo-random 4-bit codes held in registers,
 * with no memory traffic: the ceiling that the GEMM of that engine can approach on such values (it
 * lies below the data-sheet peak, because the clock under a matrix load depends on the operand data).
 * Runs on the default stream, allocates 4 bytes, blocks for a few tens of milliseconds. */
stamp_status_t stamp_debug_mfma_rate(int32_t engine, double* tera_ops_per_s_host);

const char* stamp_status_string(stamp_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* STAMP_H_ */
