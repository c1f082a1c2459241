// Internal declarations shared by the HIP sources of the STaMP library (gfx950 only).
#ifndef STAMP_INTERNAL_H_
#define STAMP_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "stamp.h"

#define STAMP_HD __host__ __device__ __forceinline__

// ---------------------------------------------------------------------------------------------
// Geometry of a plan.  The J-level transform is split at level r = log2(seq_len / k_hi) (1-D) or
// log4 (2-D): the "bottom" r levels act inside aligned blocks of R tokens and produce the R-1
// 4-bit rows of each block; the "top" J-r levels act on the k_hi block sums and produce the k_hi
// 8-bit rows.
// ---------------------------------------------------------------------------------------------
struct StampGeom {
  int32_t B, s, d, N;
  int32_t is2d;      // 0: 1-D stream, 1: 2-D grid
  int32_t J;         // total levels of the transform (plan argument)
  int32_t L;         // top levels J - r: levels applied to the k block sums (0 = the block sums themselves)
  int32_t r;         // bottom levels (inside a block)
  int32_t R;         // tokens per block: 2^r (1-D) or 4^r (2-D)
  int32_t k;         // number of blocks per sequence = rows of the top part (held as int8 codes, q_hi)
  int32_t khi;       // how many of them are 8-bit rows (k_hi); the others carry 4-bit codes (J < log2(seq_len / k_hi))
  int32_t G;         // 2-D: blocks per grid side (k = G*G); 1-D: unused (0)
  int32_t g;         // 2-D: tokens per block side (2^r); 1-D: unused (0)
  int32_t gridW;     // 2-D: tokens per grid row
  int32_t x_bf16;    // input dtype is bf16
  int32_t y_bf16;    // output dtype is bf16
  int32_t asym;      // asymmetric activation codes: stored code - 2^(b-1), offsets z next to the scales
  int32_t ident;     // no sequence transform: tokens 0..k-1 are the 8-bit rows, physical row = token (J = r = 0, R = 1)
                     // (also set for plans of the general path, whose quantizer and GEMM see transformed tokens as rows)
};

// General path: the transform runs level by level over fp32 buffers in the workspace (stamp_general.hip).
enum StampGenKind { kGenNone = 0, kGenCopy, kGenHaarRagged, kGenHaarClassic, kGenHaar2d, kGenWht, kGenDct };
struct StampGen {
  int32_t kind;        // StampGenKind
  int32_t levels;
  int32_t skip;        // first token left out (ragged Haar)
  int32_t group;       // 0 or 64
  int32_t bias_mode;   // 1: transformed bias
  int32_t gridH, gridW;
};

// Position inside a block ("e", 0 = the block sum, e >= 1 the in-block detail rows in STaMP
// order) of the coefficient that the in-place butterfly network leaves at natural position q.
// 1-D: in-place butterflies at stride 2^l leave the level-l difference of pair i at position
// i*2^l + 2^(l-1).
STAMP_HD int stamp_e_of_natural_1d(int q, int n /* block length, power of two */) {
  if (q == 0) return 0;
  int t = __builtin_ctz((unsigned)q);  // level - 1
  return (n >> (t + 1)) + (q >> (t + 1));
}

// 2-D: natural position (y, x) in a g x g block; the in-place network leaves at
// (2^l i + dy 2^(l-1), 2^l j + dx 2^(l-1)) the band (dy, dx) of level l: (0,1) = difference along
// the width, (1,0) = along the height, (1,1) = diagonal.
STAMP_HD int stamp_e_of_natural_2d(int y, int x, int g) {
  if (y == 0 && x == 0) return 0;
  int t = __builtin_ctz((unsigned)(y | x));  // level - 1
  int by = (y >> t) & 1, bx = (x >> t) & 1;
  int band = by ? (bx ? 2 : 1) : 0;          // W, H, D
  int gl = g >> (t + 1);                     // side of each band of that level
  return gl * gl * (1 + band) + (y >> (t + 1)) * gl + (x >> (t + 1));
}

// Top part, L levels over n block sums (1-D) / G x G block sums (2-D): STaMP slot (< n, < G*G) of the
// coefficient that L in-place butterfly levels leave at natural position q / (y, x), and its level counted
// within the top part (L for the remaining approximations, which come first in STaMP order).
STAMP_HD int stamp_top_slot_1d(int q, int n, int L, int* lvl_top) {
  const int t = (q == 0) ? 32 : __builtin_ctz((unsigned)q);
  if (t >= L) { *lvl_top = L; return q >> L; }
  *lvl_top = t + 1;
  return (n >> (t + 1)) + (q >> (t + 1));
}
STAMP_HD int stamp_top_slot_2d(int y, int x, int G, int L, int* lvl_top) {
  const int t = ((y | x) == 0) ? 32 : __builtin_ctz((unsigned)(y | x));
  if (t >= L) { *lvl_top = L; return (y >> L) * (G >> L) + (x >> L); }
  *lvl_top = t + 1;
  return stamp_e_of_natural_2d(y, x, G);
}
// Level (counted over the whole transform) of the 8-bit STaMP slot p.
STAMP_HD int stamp_level_of_top_slot(int p, int k, int G, int is2d, int r, int L) {
  if (!is2d) {
    if (p < (k >> L)) return r + L;
    return r + (31 - __builtin_clz((unsigned)k)) - (31 - __builtin_clz((unsigned)p));
  }
  if (p < (G >> L) * (G >> L)) return r + L;
  return r + (31 - __builtin_clz((unsigned)G)) - ((31 - __builtin_clz((unsigned)p)) >> 1);
}

// STaMP slot p (whole sequence) of in-block position e >= 1 of block j.
// 1-D: e = 2^m + i  ->  p = (k + j) * 2^m + i.
STAMP_HD int stamp_slot_of_block_e_1d(int j, int e, int k) {
  int m = 31 - __builtin_clz((unsigned)e);
  return ((k + j) << m) + (e - (1 << m));
}

// 2-D: block (bi, bj) of a G x G block grid, e = gl^2 (1 + band) + yy gl + xx  ->
// p = (G gl)^2 (1 + band) + (bi gl + yy)(G gl) + bj gl + xx.
STAMP_HD int stamp_slot_of_block_e_2d(int bi, int bj, int e, int G) {
  int m = (31 - __builtin_clz((unsigned)e)) >> 1;  // gl = 2^m, since gl^2 <= e < 4 gl^2
  int gl = 1 << m;
  int band = (e >> (2 * m)) - 1;
  int rem = e - ((1 + band) << (2 * m));
  int yy = rem >> m, xx = rem & (gl - 1);
  int Gl = G * gl;
  return Gl * Gl * (1 + band) + (bi * gl + yy) * Gl + bj * gl + xx;
}

// Level (1 = finest) of in-block position e >= 1 in a block of R tokens.
STAMP_HD int stamp_level_of_e_1d(int e, int r) { return r - (31 - __builtin_clz((unsigned)e)); }
STAMP_HD int stamp_level_of_e_2d(int e, int r) { return r - ((31 - __builtin_clz((unsigned)e)) >> 1); }

// Byte offset of (output column n, permuted channel position c) in the stored weight:
// [Npad/128][Kpad/128][128 columns][128 positions].
STAMP_HD size_t stamp_w_offset(int n, int c, int Kpad) {
  return (((size_t)(n >> 7) * (size_t)(Kpad >> 7) + (size_t)(c >> 7)) * 128 + (size_t)(n & 127)) * 128 + (size_t)(c & 127);
}

// Byte offset of (physical row m over all sequences, channel c) in the tiled 4-bit activation:
// [Mpad/256][Kpad/128][256 rows][64 bytes], two channels per byte.
STAMP_HD size_t stamp_qlo_offset(size_t m, int c, int Kpad) {
  return (((m >> 8) * (size_t)(Kpad >> 7) + (size_t)(c >> 7)) * 256 + (m & 255)) * 64 + (size_t)((c & 127) >> 1);
}

// ---------------------------------------------------------------------------------------------
// The plan.
// ---------------------------------------------------------------------------------------------
struct stamp_plan {
  stamp_plan_desc_t desc;
  StampGeom geom;
  int32_t Kpad, Npad;       // GEMM-padded depth and width of the stored weight
  int32_t Mpad;             // batch * seq_len rounded up to the GEMM's 256-row tile
  int8_t* qW_dev;           // tiled int8 weight codes * 16 (see stamp_w_offset), K order permuted per 16 channels
  float* sw_dev;            // [Npad] weight scales (0 beyond d_out)
  float* bias_dev;          // [Npad] bias or nullptr
  float* colsum_dev;        // [Npad] sum over input channels of the weight codes (exact integers as fp32)
  int32_t* row_of_coeff;    // host, [s]
  uint8_t* qW6_dev;         // the same weight codes as E2M3 numbers in the operand layout of the FP6 GEMM
  int32_t engine;           // matrix pipeline of the 4-bit rows' GEMM: STAMP_GEMM_INT8 or STAMP_GEMM_FP6
  int32_t hi_ksplit;        // parts the depth of the 8-bit rows' GEMM is split into (partial rows in the workspace)
  int32_t hi_ksplit_own;    // the same when only the first khi top rows go through that GEMM (stamp_own_top)
  int32_t unfused;          // 1: separate inverse kernel
  int32_t fused_ok;         // shape allows the fused epilogue
  StampGen gen;             // general path (kind != kGenNone)
  int32_t* perm_dev;        // general path, WHT: [s] STaMP slot of every row of the Hadamard-ordered result
  float* ell_dev;           // general path, transformed bias: [s] l = L 1
  double* dct_dev;          // general path, DCT: [s][s] orthonormal DCT-II matrix
  int8_t* qWg_dev;          // per-block scales: weight codes [Npad128][d_in] int8
  float* swg_dev;           // per-block scales: [d_in / 64][Npad128]
  size_t ws_T[3], ws_Yt[3], ws_codes8, ws_scalesg;  // general path workspace (byte offsets)
  // workspace layout (byte offsets, 256-aligned)
  size_t ws_abot, ws_rowmax, ws_gpart, ws_qhi, ws_qlo, ws_scales, ws_ythi, ws_P, ws_a6, ws_ytlo, ws_total;
};

// Dynamic-LDS limit of a kernel, raised once per device and kernel (the attribute belongs to the device's
// copy of the function): `done` is the kernel's own table, one size per device.
constexpr int kStampMaxDevices = 64;
inline std::mutex& stamp_lds_mutex() {
  static std::mutex m;  // one lock for all tables: taken once per launch, never contended for long
  return m;
}
inline hipError_t stamp_allow_lds(const void* kernel, size_t bytes, size_t (&done)[kStampMaxDevices]) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kStampMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(stamp_lds_mutex());  // plans may be used from several host threads
  if (bytes <= done[dev]) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) done[dev] = bytes;
  return e;
}

// ---- launchers implemented in the kernel files (all asynchronous on `st`) ----
hipError_t stamp_launch_weight_quant(const stamp_plan* p, const float* W, hipStream_t st, uint32_t* colmax_tmp);
// part: 1 = bottom kernel only, 2 = top + 8-bit rows only, 3 = both
// scales: [B*s] scales, followed by [B*s] offsets z for asymmetric plans
// gpart: [2][nsplit][B*s] partial row maxima when the channels are split over workgroups (nsplit > 1), else unused
int stamp_actquant_nsplit(const stamp_plan* p);
// plans without top levels and without channel splits: the bottom kernel also quantizes the block sums (no k_top, no k_quant_hi)
bool stamp_top_in_bottom(const stamp_plan* p);
hipError_t stamp_launch_actquant(const stamp_plan* p, const void* X, int8_t* q_hi, uint8_t* q_lo,
                                 float* scales, float* abot, uint32_t* rowmax, uint32_t* gpart, hipStream_t st, int part = 3);
// mode: 0 = int32 accumulators in STaMP row order (debug), 1 = dequantized fp32 rows (hi -> Yt_hi
// [hi_ksplit][B*k, N] partial rows, lo -> Yt_lo [B*s, N] physical rows), 2 = lo rows with fused in-block inverse -> Y,
// 3 = lo rows of an identity plan: dequantized + bias -> Y.
bool stamp_hi_wide_tiles(int M, int Npad);
int stamp_hi_ksplit(const stamp_plan* p, int rows_per_seq);
// ld_out > 0 (mode 1): row stride of `out` in floats instead of d_out
// first_khi_only (mode 1): only the first khi rows of every sequence are multiplied, depth split into
// hi_ksplit_own parts, rows of `out` numbered b * khi + p
hipError_t stamp_launch_gemm_hi(const stamp_plan* p, const int8_t* q_hi, const float* scales, int mode,
                                void* out, hipStream_t st, int ld_out = 0, bool first_khi_only = false);
// P[row][0..ncols) = sum over the parts of src[part][row][0..ncols), rows < nrows
hipError_t stamp_launch_sum_parts(const float* src, int nparts, int nrows, int ncols, float* P, int ldP, hipStream_t st);
bool stamp_hi_rows_are_block_sums(const stamp_plan* p);
// mode 2 of stamp_launch_gemm_hi is available: dequantization + top levels of the inverse in the GEMM's tiles, out = P
bool stamp_hi_top_fused(const stamp_plan* p);
hipError_t stamp_launch_gemm_lo(const stamp_plan* p, const uint8_t* q_lo, const float* scales, int mode,
                                void* out, const float* P, hipStream_t st);
// FP6 engine of the 4-bit rows: operand sizes, plan-time weight codes (colmax: bit patterns of the column
// maxima, as left by stamp_launch_weight_quant), conversion of the packed 4-bit rows, and the GEMM (modes as above).
size_t stamp_a6_bytes(const stamp_plan* p);
size_t stamp_b6_bytes(const stamp_plan* p);
hipError_t stamp_launch_weight_quant6(const stamp_plan* p, const float* W, const uint32_t* colmax, hipStream_t st);
hipError_t stamp_launch_repack6(const stamp_plan* p, const uint8_t* q_lo, uint8_t* a6, hipStream_t st);
// own_top (mode 2, plans without top levels): the blocks from khi on take their sum from their own coefficient 0,
// a 4-bit row of a6 like any other (the quantizer writes it there as well), and P holds khi rows per sequence
hipError_t stamp_launch_gemm_lo6(const stamp_plan* p, const uint8_t* a6, const float* scales, int mode, void* out,
                                 const float* P, hipStream_t st, int own_top = 0);
// identity plans: 8-bit rows' dequantized partial rows [nparts][B*k][N] (+ bias) -> Y rows of tokens 0..k-1
hipError_t stamp_launch_hi_rows_out(const stamp_plan* p, const float* Yt_hi, void* Y, hipStream_t st, int nparts);
// P: block sums [B*k][ldP]; nparts partial sources (each B*k*ncols floats apart) are added while reading
hipError_t stamp_launch_inverse_top(const stamp_plan* p, const float* Yt_hi, int hi_row_stride_is_stamp,
                                    int ncols, float* P, int ldP, hipStream_t st, int nparts = 1);
hipError_t stamp_launch_inverse_bottom(const stamp_plan* p, const float* Yt_lo, int src_is_stamp_order,
                                       const float* P, int ldP, int ncols, const float* bias, void* Y, hipStream_t st);

// ---- general path (stamp_general.hip) ----
hipError_t stamp_gen_plan_tables(stamp_plan* p, const float* W, hipStream_t st);  // device tables and grouped weights
void stamp_gen_plan_free(stamp_plan* p);
// X -> transformed tokens T [B, s, d] fp32 in STaMP order; returns the buffer that holds T (one of the three)
hipError_t stamp_gen_forward(const stamp_plan* p, const void* X, float* const (&buf)[3], float** T_out, hipStream_t st);
// Yt [B, s, ncols] fp32 in STaMP order (buf[0], only read) -> Y; buf[1], buf[2]: the levels' work buffers
hipError_t stamp_gen_inverse(const stamp_plan* p, float* const (&buf)[3], int ncols, const float* bias, void* Y, hipStream_t st);
hipError_t stamp_launch_quant_rows_f32(const stamp_plan* p, const float* T, int8_t* q_hi, uint8_t* q_lo, float* scales, hipStream_t st);
hipError_t stamp_launch_quant_rows_grouped(const stamp_plan* p, const float* T, int8_t* codes, float* scales, hipStream_t st);
hipError_t stamp_launch_gemm_grouped(const stamp_plan* p, const int8_t* codes, const float* scales, float* Yt, hipStream_t st);
hipError_t stamp_launch_bf16_to_f32(const void* src, float* dst, size_t n, hipStream_t st);
hipError_t stamp_launch_merge_hi(const stamp_plan* p, const float* ythi, int nparts, float* Yt, hipStream_t st);
hipError_t stamp_launch_add_ell_bias(const stamp_plan* p, float* Yt, hipStream_t st);

#endif  // STAMP_INTERNAL_H_
