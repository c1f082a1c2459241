// General path of the STaMP linear layer on gfx950: the sequence transforms that do not have the block structure
// the fast path relies on, and per-block (group) scales.
//
//   Haar DWT of any sequence length, optionally with the first token left out of L (section "Efficient Energy
//   Concentration", footnote on padding; appendix "Experimental details", LLMs): a level pairs the current
//   approximations (0,1), (2,3), ...; an odd one out is carried to the next level unchanged.  Every level is the
//   orthonormal butterfly a = (x0 + x1) * C, d = (x0 - x1) * C, C = fl(1 / sqrt 2), each operation rounded.
//   Power-of-two Haar transforms (1-D and 2-D) in the fast path's arithmetic (plain sums, one multiplication by the
//   level's norm at the end), for plans that need the general path for another reason (per-block scales, transformed
//   bias).
//   WHT in sequency order and the orthonormal DCT-II along the tokens (same section).
//   Per-block scales: one scale per 64 consecutive channels, for activations and weights (Experiments, LVM set-up).
//
// The forward transform runs as one kernel per level over fp32 buffers [B, s, d] in the workspace (thread = one
// butterfly of one channel, consecutive threads = consecutive channels), leaves T in STaMP order; the quantizer and
// the GEMM then treat the transformed tokens as rows (physical row = STaMP slot); the inverse runs level by level
// over [B, s, d_out].  The floating-point order of the FORWARD transform is the oracle's (it decides the codes);
// the inverse and the de-quantization only have to meet the output tolerance.  Compiled with -ffp-contract=off.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <vector>

#include "stamp_internal.h"

namespace {

constexpr float kC = 0.70710678118654752440f;  // fl(1 / sqrt 2) = 0x3F3504F3

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// grid: x = ceil(row_elems / blockDim.x), y = rows of this launch, z = batch; one thread per element of a row
#define GEN_INDEX                                      \
  const int c = blockIdx.x * blockDim.x + threadIdx.x; \
  const int i = blockIdx.y;                            \
  const size_t bo = (size_t)blockIdx.z * seq * ld;     \
  if (c >= ld) return

// X (bf16 or fp32) -> fp32
__global__ __launch_bounds__(256) void k_gen_cast(const void* __restrict__ X, float* __restrict__ dst, int seq, int ld, int bf16) {
  GEN_INDEX;
  const size_t idx = bo + (size_t)i * ld + c;
  dst[idx] = bf16 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(X)[idx] << 16) : reinterpret_cast<const float*>(X)[idx];
}

// One element of the input of a transform pass: X itself (bf16 or fp32) or an fp32 work buffer.
__device__ __forceinline__ float gen_load(const void* in, int kind, size_t idx) {
  return kind == 2 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(in)[idx] << 16) : reinterpret_cast<const float*>(in)[idx];
}
__device__ __forceinline__ void gen_store_y(void* Y, int y_bf16, size_t idx, float v) {
  if (y_bf16) reinterpret_cast<uint16_t*>(Y)[idx] = f32_to_bf16_rne(v);
  else reinterpret_cast<float*>(Y)[idx] = v;
}

// per-pass factors of the power-of-two ("classic") arithmetic: det[i] multiplies the details of the pass's i-th
// level, apx the approximations when the pass is the last one
struct GenNorm {
  float det[5];
  float apx;
};

// NLEV levels of the 1-D Haar transform in one pass.  The current approximations (n_lo of them, rows o + i of `in`)
// fall into blocks of 2^NLEV; a thread owns one block of one channel, loads it, runs the levels in registers and
// writes every detail to its STaMP slot in T (the details of a level with n approximations left sit in slots
// o + n .. ) and the block's one approximation to row o + block of apx_out (of T, times nm.apx, when `last`).
// Pairs are (2 i, 2 i + 1); an approximation without partner is carried up unchanged, so a short last block is a
// sub-tree of its own.  scaled: every butterfly is (x0 +- x1) * C (the form for any length); else plain sums and one
// multiplication per finished coefficient (the power-of-two form).  in_kind: 0 fp32 buffer, 1 X fp32, 2 X bf16; with
// X as input and o = 1, block 0 also copies token 0 to slot 0.  Grid: x = ceil(ld / 256), y = blocks, z = batch.
template <int NLEV>
__global__ __launch_bounds__(256) void k_gen_haar1d_fwd(const void* __restrict__ in, int in_kind, float* __restrict__ apx_out,
                                                        float* __restrict__ T, int seq, int ld, int o, int n_lo, int scaled,
                                                        int last, GenNorm nm) {
  GEN_INDEX;
  constexpr int W = 1 << NLEV;
  float v[W];
#pragma unroll
  for (int j = 0; j < W; ++j) {
    const int gi = i * W + j;
    v[j] = gi < n_lo ? gen_load(in, in_kind, bo + (size_t)(o + gi) * ld + c) : 0.0f;
  }
  int n_prev = n_lo;
#pragma unroll
  for (int li = 0; li < NLEV; ++li) {
    const int n_cur = (n_prev + 1) >> 1;
#pragma unroll
    for (int j = 0; j < (W >> (li + 1)); ++j) {
      const int gi = i * (W >> (li + 1)) + j;
      if (gi < n_cur) {
        if (2 * gi + 1 < n_prev) {
          const float x0 = v[2 * j], x1 = v[2 * j + 1];
          float a = __fadd_rn(x0, x1), dd = __fsub_rn(x0, x1);
          if (scaled) {
            a = __fmul_rn(a, kC);
            dd = __fmul_rn(dd, kC);
          } else {
            dd = __fmul_rn(dd, nm.det[li]);
          }
          T[bo + (size_t)(o + n_cur + gi) * ld + c] = dd;
          v[j] = a;
        } else {
          v[j] = v[2 * j];
        }
      }
    }
    n_prev = n_cur;
  }
  if (last) T[bo + (size_t)(o + i) * ld + c] = scaled ? v[0] : __fmul_rn(v[0], nm.apx);
  else apx_out[bo + (size_t)(o + i) * ld + c] = v[0];
  if (in_kind != 0 && o != 0 && i == 0) T[bo + c] = gen_load(in, in_kind, bo + c);
}

// The inverse of such a pass: the block's approximation (row o + block of apx_in) and the details (slots of S) ->
// the 2^NLEV (or fewer) finer approximations, rows o + i of apx_out, or, when `last`, the tokens themselves: rows
// o + i of Y (+ bias, output type); then block 0 also writes the token that was left out (slot 0 of S).
template <int NLEV>
__global__ __launch_bounds__(256) void k_gen_haar1d_inv(const float* __restrict__ apx_in, const float* __restrict__ S,
                                                        float* __restrict__ apx_out, void* __restrict__ Y,
                                                        const float* __restrict__ bias, int y_bf16, int seq, int ld, int o,
                                                        int n_lo, int last) {
  GEN_INDEX;
  constexpr int W = 1 << NLEV;
  int n[NLEV + 1];
  n[0] = n_lo;
#pragma unroll
  for (int li = 0; li < NLEV; ++li) n[li + 1] = (n[li] + 1) >> 1;
  float v[W];
  v[0] = apx_in[bo + (size_t)(o + i) * ld + c];
#pragma unroll
  for (int li = NLEV - 1; li >= 0; --li) {
#pragma unroll
    for (int j = (W >> (li + 1)) - 1; j >= 0; --j) {
      const int gi = i * (W >> (li + 1)) + j;
      if (gi < n[li + 1]) {
        const float a = v[j];
        if (2 * gi + 1 < n[li]) {
          const float dd = S[bo + (size_t)(o + n[li + 1] + gi) * ld + c];
          v[2 * j] = (a + dd) * kC;
          v[2 * j + 1] = (a - dd) * kC;
        } else {
          v[2 * j] = a;
        }
      }
    }
  }
  const float bv = (last && bias != nullptr) ? bias[c] : 0.0f;
#pragma unroll
  for (int j = 0; j < W; ++j) {
    const int gi = i * W + j;
    if (gi < n_lo) {
      const size_t idx = bo + (size_t)(o + gi) * ld + c;
      if (last) gen_store_y(Y, y_bf16, idx, v[j] + bv);
      else apx_out[idx] = v[j];
    }
  }
  if (last && o != 0 && i == 0) gen_store_y(Y, y_bf16, bo + c, S[bo + c] + bv);
}

// NLEV levels of the 2-D Haar pyramid in one pass (power-of-two grids).  The current low-low region is
// h_lo x w_lo (cells_lo = h_lo * w_lo tokens) at the top-left of `in` (grid pitch gridW, token = r * gridW + col); a thread owns one patch of
// 2^NLEV x 2^NLEV of one channel.  Per level: plain sums for the low-low value, the three details times 2^-level
// to their STaMP slots (bands W, H, D of the level, each row-major, base[li] = slot of the level's band W).  The
// patch's low-low value goes to grid position (pi, pj) of ll_out, or, when `last`, times apx_norm to slot
// pi * (w_lo >> NLEV) + pj of T.  blockIdx.y = pi * (w_lo >> NLEV) + pj.
struct GenBands {
  int base[3];
  float norm[3];
};
template <int NLEV>
__global__ __launch_bounds__(256) void k_gen_haar2d_fwd(const void* __restrict__ in, int in_kind, float* __restrict__ ll_out,
                                                        float* __restrict__ T, int seq, int ld, int gridW, int w_lo,
                                                        int cells_lo, GenBands bd, int last, float apx_norm) {
  GEN_INDEX;
  constexpr int P = 1 << NLEV;
  const int wp = w_lo >> NLEV, pi = i / wp, pj = i - pi * wp;
  float v[P][P];
#pragma unroll
  for (int a = 0; a < P; ++a)
#pragma unroll
    for (int b = 0; b < P; ++b) v[a][b] = gen_load(in, in_kind, bo + ((size_t)(pi * P + a) * gridW + (pj * P + b)) * ld + c);
#pragma unroll
  for (int li = 0; li < NLEV; ++li) {
    const int wl = w_lo >> (li + 1), cells = cells_lo >> (2 * (li + 1));
#pragma unroll
    for (int ca = 0; ca < (P >> (li + 1)); ++ca)
#pragma unroll
      for (int cb = 0; cb < (P >> (li + 1)); ++cb) {
        const float p = v[2 * ca][2 * cb], q = v[2 * ca][2 * cb + 1], u = v[2 * ca + 1][2 * cb], w = v[2 * ca + 1][2 * cb + 1];
        const float t0 = __fadd_rn(p, q), t1 = __fsub_rn(p, q), t2 = __fadd_rn(u, w), t3 = __fsub_rn(u, w);
        const int gi = (pi * (P >> (li + 1)) + ca) * wl + (pj * (P >> (li + 1)) + cb);
        float* const tb = T + bo + (size_t)(bd.base[li] + gi) * ld + c;
        tb[0] = __fmul_rn(__fadd_rn(t1, t3), bd.norm[li]);
        tb[(size_t)cells * ld] = __fmul_rn(__fsub_rn(t0, t2), bd.norm[li]);
        tb[(size_t)2 * cells * ld] = __fmul_rn(__fsub_rn(t1, t3), bd.norm[li]);
        v[ca][cb] = __fadd_rn(t0, t2);
      }
  }
  if (last) T[bo + (size_t)i * ld + c] = __fmul_rn(v[0][0], apx_norm);
  else ll_out[bo + ((size_t)pi * gridW + pj) * ld + c] = v[0][0];
}

// The inverse of such a pass: the patch's low-low value (grid position (pi, pj) of ll_in, or slot i of S when
// `first`) and the bands -> the 2^NLEV x 2^NLEV finer low-low values at the top-left of ll_out, or, when `last`,
// the tokens of Y (+ bias, output type).  Orthonormal butterflies: every output of a level times 1/2.
template <int NLEV>
__global__ __launch_bounds__(256) void k_gen_haar2d_inv(const float* __restrict__ ll_in, int first, const float* __restrict__ S,
                                                        float* __restrict__ ll_out, void* __restrict__ Y,
                                                        const float* __restrict__ bias, int y_bf16, int seq, int ld, int gridW,
                                                        int w_lo, int cells_lo, GenBands bd, int last) {
  GEN_INDEX;
  constexpr int P = 1 << NLEV;
  const int wp = w_lo >> NLEV, pi = i / wp, pj = i - pi * wp;
  float v[P][P];
  v[0][0] = first ? S[bo + (size_t)i * ld + c] : ll_in[bo + ((size_t)pi * gridW + pj) * ld + c];
#pragma unroll
  for (int li = NLEV - 1; li >= 0; --li) {
    const int wl = w_lo >> (li + 1), cells = cells_lo >> (2 * (li + 1));
#pragma unroll
    for (int ca = (P >> (li + 1)) - 1; ca >= 0; --ca)
#pragma unroll
      for (int cb = (P >> (li + 1)) - 1; cb >= 0; --cb) {
        const int gi = (pi * (P >> (li + 1)) + ca) * wl + (pj * (P >> (li + 1)) + cb);
        const float* const sb = S + bo + (size_t)(bd.base[li] + gi) * ld + c;
        const float cLL = v[ca][cb], cW = sb[0], cH = sb[(size_t)cells * ld], cD = sb[(size_t)2 * cells * ld];
        const float t0 = cLL + cH, t2 = cLL - cH, t1 = cW + cD, t3 = cW - cD;
        v[2 * ca][2 * cb] = (t0 + t1) * 0.5f;
        v[2 * ca][2 * cb + 1] = (t0 - t1) * 0.5f;
        v[2 * ca + 1][2 * cb] = (t2 + t3) * 0.5f;
        v[2 * ca + 1][2 * cb + 1] = (t2 - t3) * 0.5f;
      }
  }
  const float bv = (last && bias != nullptr) ? bias[c] : 0.0f;
#pragma unroll
  for (int a = 0; a < P; ++a)
#pragma unroll
    for (int b = 0; b < P; ++b) {
      const size_t idx = bo + ((size_t)(pi * P + a) * gridW + (pj * P + b)) * ld + c;
      if (last) gen_store_y(Y, y_bf16, idx, v[a][b] + bv);
      else ll_out[idx] = v[a][b];
    }
}

// NLEV stages of the Hadamard-ordered fast WHT in one pass: the stages with strides h_lo, 2 h_lo, ... combine the
// 2^NLEV rows base + j * h_lo, base = (i / h_lo) * (h_lo << NLEV) + i % h_lo (blockIdx.y = i).  in_kind as above.
// out_kind 0: fp32 rows in place; 1: the last pass of the forward transform, row r times norm to the STaMP slot
// inv_perm[r] of T (sequency order); 2: the last pass of the inverse, the same to rows of Y (+ bias, output type).
template <int NLEV>
__global__ __launch_bounds__(256) void k_gen_wht(const void* __restrict__ in, int in_kind, float* __restrict__ out,
                                                 void* __restrict__ Y, int out_kind, const int* __restrict__ inv_perm, float norm,
                                                 const float* __restrict__ bias, int y_bf16, int seq, int ld, int h_lo) {
  GEN_INDEX;
  constexpr int W = 1 << NLEV;
  const int hp = i / h_lo, t = i - hp * h_lo;
  const int base = hp * (h_lo << NLEV) + t;
  float v[W];
#pragma unroll
  for (int j = 0; j < W; ++j) v[j] = gen_load(in, in_kind, bo + (size_t)(base + j * h_lo) * ld + c);
#pragma unroll
  for (int st = 0; st < NLEV; ++st) {
#pragma unroll
    for (int j = 0; j < W; ++j) {
      if ((j & (1 << st)) == 0) {
        const float u = v[j], w = v[j + (1 << st)];
        v[j] = __fadd_rn(u, w);
        v[j + (1 << st)] = __fsub_rn(u, w);
      }
    }
  }
  const float bv = (out_kind == 2 && bias != nullptr) ? bias[c] : 0.0f;
#pragma unroll
  for (int j = 0; j < W; ++j) {
    const int r = base + j * h_lo;
    if (out_kind == 0) {
      out[bo + (size_t)r * ld + c] = v[j];
    } else {
      const float x = __fmul_rn(v[j], norm);
      const size_t idx = bo + (size_t)inv_perm[r] * ld + c;
      if (out_kind == 1) out[idx] = x;
      else gen_store_y(Y, y_bf16, idx, x + bv);
    }
  }
}

// dst[k, c] = fl32( sum_n Mx[k, n] * src[n, c] ) in fp64 (Mx = C, or C^T when transposed), per batch, on the fp64
// matrix pipeline: 64 x 64 outputs per workgroup of 4 waves (2 x 2), a wave 32 x 32 = 2 x 2 blocks of
// v_mfma_f64_16x16x4_f64, 16 values of n per pass through LDS.  A lane feeds A[row lane % 16][n lane / 16] and
// B[n lane / 16][column lane % 16] and holds D[row 4 i + lane / 16][column lane % 16], i = 0..3 (checked on the chip).
typedef double v4d __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void k_gen_dct(const double* __restrict__ Cm, int transposed, const float* __restrict__ src,
                                                 float* __restrict__ dst, int seq, int ld) {
  __shared__ double sM[16][65];
  __shared__ double sX[16][65];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wk = wave >> 1, wc = wave & 1, l16 = lane & 15, lk = lane >> 4;
  const int k0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const size_t bo = (size_t)blockIdx.z * seq * ld;
  v4d acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) acc[a][b] = (v4d){0.0, 0.0, 0.0, 0.0};
  for (int n0 = 0; n0 < seq; n0 += 16) {
    for (int e = threadIdx.x; e < 16 * 64; e += 256) {
      // the matrix: consecutive threads along its contiguous direction (n as stored, k when transposed)
      const int nn_m = transposed ? (e >> 6) : (e & 15), kk_m = transposed ? (e & 63) : (e >> 4);
      const int k = k0 + kk_m, n = n0 + nn_m;
      double mv = 0.0;
      if (k < seq && n < seq) mv = transposed ? Cm[(size_t)n * seq + k] : Cm[(size_t)k * seq + n];
      sM[nn_m][kk_m] = mv;
      const int nn = e >> 6, cc = c0 + (e & 63);
      sX[nn][e & 63] = (n0 + nn < seq && cc < ld) ? (double)src[bo + (size_t)(n0 + nn) * ld + cc] : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      double fa[2], fb[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        fa[a] = sM[kk * 4 + lk][wk * 32 + a * 16 + l16];
        fb[a] = sX[kk * 4 + lk][wc * 32 + a * 16 + l16];
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    __syncthreads();
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int k = k0 + wk * 32 + a * 16 + 4 * i + lk, cc = c0 + wc * 32 + b * 16 + l16;
        if (k < seq && cc < ld) dst[bo + (size_t)k * ld + cc] = (float)acc[a][b][i];
      }
}

__global__ void k_gen_dct_matrix(double* __restrict__ Cm, int s) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x, k = blockIdx.y;
  if (n >= s) return;
  const double pi = 3.14159265358979323846;
  Cm[(size_t)k * s + n] = (k == 0) ? sqrt(1.0 / s) : cos(pi * (2.0 * n + 1.0) * (double)k / (2.0 * s)) * sqrt(2.0 / s);
}

// bf16 -> fp32, flat (plan time: weights given in bf16)
__global__ __launch_bounds__(256) void k_gen_cast_flat(const uint16_t* __restrict__ src, float* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = __uint_as_float((uint32_t)src[i] << 16);
}

// fp32 [B, s, ncols] (+ bias) -> Y in the plan's output type
__global__ __launch_bounds__(256) void k_gen_store_y(const float* __restrict__ src, const float* __restrict__ bias,
                                                     void* __restrict__ Y, int seq, int ld, int y_bf16) {
  GEN_INDEX;
  const size_t idx = bo + (size_t)i * ld + c;
  float v = src[idx];
  if (bias != nullptr) v += bias[c];
  if (y_bf16) reinterpret_cast<uint16_t*>(Y)[idx] = f32_to_bf16_rne(v);
  else reinterpret_cast<float*>(Y)[idx] = v;
}

// Yt[b, p, n] += ell[p] * bias[n]
__global__ __launch_bounds__(256) void k_gen_add_ell_bias(float* __restrict__ Yt, const float* __restrict__ ell,
                                                          const float* __restrict__ bias, int seq, int ld) {
  GEN_INDEX;
  const float l = ell[i];
  if (l != 0.0f) Yt[bo + (size_t)i * ld + c] += l * bias[c];
}

// 8-bit rows of the general path: sum of the partial dequantized rows [nparts][B * k][N] -> rows 0 .. k-1 of Yt
__global__ __launch_bounds__(256) void k_gen_merge_hi(const float* __restrict__ ythi, int nparts, size_t part_stride,
                                                      float* __restrict__ Yt, int seq, int ld, int k) {
  GEN_INDEX;
  const size_t idx = ((size_t)blockIdx.z * k + i) * ld + c;
  float v = ythi[idx];
  for (int part = 1; part < nparts; ++part) v += ythi[idx + part * part_stride];
  Yt[bo + (size_t)i * ld + c] = v;
}

// ---------------------------------------------------------------------------------------------
// Per-block scales
// ---------------------------------------------------------------------------------------------
// One workgroup per transformed token; a thread owns 8 consecutive channels, 8 consecutive lanes one group of 64:
// a = max |t| over the group, scale = a / qmax, inv = qmax / a, code = rne(t * inv) (the per-token quantizer's
// arithmetic, per group).  codes int8 [B * s][d], scales [B * s][d / 64].
__global__ __launch_bounds__(256) void k_gen_quant_grouped(const float* __restrict__ T, int8_t* __restrict__ codes,
                                                           float* __restrict__ scales, int s, int d, int khi) {
  const int pr = blockIdx.x, b = blockIdx.y;
  const size_t m = (size_t)b * s + pr;
  const float qmax = pr < khi ? 127.0f : 7.0f;
  const int G = d >> 6;
  for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
    const float4 v0 = *reinterpret_cast<const float4*>(T + m * d + c), v1 = *reinterpret_cast<const float4*>(T + m * d + c + 4);
    const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    float a = 0.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t) a = fmaxf(a, fabsf(v[t]));
    int x = (int)__float_as_uint(a), y;  // non-negative floats order like their bit patterns
    y = __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false); x = max(x, y);   // quad_perm [1,0,3,2]
    y = __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false); x = max(x, y);   // quad_perm [2,3,0,1]
    y = __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false); x = max(x, y);  // row_half_mirror: the other quad of the 8
    a = __uint_as_float((uint32_t)x);
    float scale = 0.0f, inv = 0.0f;
    if (a > 0.0f) {
      scale = __fdiv_rn(a, qmax);
      inv = __fdiv_rn(qmax, a);
    }
    if ((threadIdx.x & 7) == 0) scales[m * G + (c >> 6)] = scale;
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float q = fminf(fmaxf(rintf(__fmul_rn(v[t], inv)), -qmax), qmax);
      w[t >> 2] |= ((uint32_t)((int)q) & 0xFFu) << (8 * (t & 3));
    }
    *reinterpret_cast<uint2*>(codes + m * d + c) = make_uint2(w[0], w[1]);
  }
}

// Weights with per-block scales (plan time): one thread per (output column, group).  qWg [Npad][d] int8 (row = output
// column, channels contiguous), swg [G][Npad].
__global__ __launch_bounds__(256) void k_gen_wquant_grouped(const float* __restrict__ W, int8_t* __restrict__ qWg,
                                                            float* __restrict__ swg, int d, int N, int Npad, size_t sc, size_t sn) {
  const int n = blockIdx.x * 256 + threadIdx.x, g = blockIdx.y;
  if (n >= Npad) return;
  float a = 0.0f;
  if (n < N)
    for (int i = 0; i < 64; ++i) a = fmaxf(a, fabsf(W[(size_t)(g * 64 + i) * sc + (size_t)n * sn]));
  float scale = 0.0f, inv = 0.0f;
  if (a > 0.0f) {
    scale = __fdiv_rn(a, 7.0f);
    inv = __fdiv_rn(7.0f, a);
  }
  swg[(size_t)g * Npad + n] = scale;
  for (int i = 0; i < 64; ++i) {
    int q = 0;
    if (n < N) q = (int)fminf(fmaxf(rintf(__fmul_rn(W[(size_t)(g * 64 + i) * sc + (size_t)n * sn], inv)), -7.0f), 7.0f);
    qWg[(size_t)n * d + g * 64 + i] = (int8_t)q;
  }
}

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));

// Y'[m, n] = sum_g (float(acc_g[m, n]) * sa[m, g]) * swg[g, n], acc_g = the integer sum over the 64 channels of group
// g on v_mfma_i32_32x32x32_i8 (two per group and 32 x 32 block), groups added in increasing order (conversion,
// multiplication by the row's scale, fused multiply-add with the column's: three vector instructions per output and
// group, which is what bounds this kernel: the two MFMAs of a group and block take a quarter of that time).  Workgroup: 4 waves (2 x 2), tile 128 x 128, wave 64 x 64 = 2 x 2 blocks.
// Lane group kg of an MFMA takes the channels [32 ks + 16 kg, +16) of the group in sub-step ks (both operands alike).
constexpr int kGPitch = 80;  // bytes per staged row: 64 codes + 16 (conflict-free 16-byte fragment reads)
__global__ __launch_bounds__(256) void k_gen_gemm_grouped(const int8_t* __restrict__ A, const float* __restrict__ sa,
                                                          const int8_t* __restrict__ Wq, const float* __restrict__ swg,
                                                          float* __restrict__ Yt, int M, int N, int Npad, int d) {
  __shared__ __attribute__((aligned(16))) uint8_t sA[128 * kGPitch];
  __shared__ __attribute__((aligned(16))) uint8_t sB[128 * kGPitch];
  __shared__ __attribute__((aligned(16))) float sSa[128];
  __shared__ __attribute__((aligned(16))) float sSw[128];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, kg = lane >> 5;
  const int m0 = blockIdx.y * 128, n0 = blockIdx.x * 128;
  const int G = d >> 6;
  float acc[2][2][16];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
  // staging: thread -> (row tid / 2, 32-byte half tid % 2) of each operand tile
  const int srow = tid >> 1, shalf = tid & 1;
  const int8_t* gA = A + (size_t)min(m0 + srow, M - 1) * d + shalf * 32;
  const int8_t* gB = Wq + (size_t)(n0 + srow) * d + shalf * 32;  // Npad rows exist
  // the next group's operands and scales travel from global memory to registers while the current group is
  // multiplied and rescaled
  const float* gS = tid < 128 ? sa + (size_t)min(m0 + tid, M - 1) * G : swg + n0 + (tid - 128);
  const size_t sstep = tid < 128 ? 1 : (size_t)Npad;
  uint4 a0 = *reinterpret_cast<const uint4*>(gA), a1 = *reinterpret_cast<const uint4*>(gA + 16);
  uint4 b0 = *reinterpret_cast<const uint4*>(gB), b1 = *reinterpret_cast<const uint4*>(gB + 16);
  float fs = gS[0];
  for (int g = 0; g < G; ++g) {
    __syncthreads();  // the previous group's fragments have been read
    *reinterpret_cast<uint4*>(sA + srow * kGPitch + shalf * 32) = a0;
    *reinterpret_cast<uint4*>(sA + srow * kGPitch + shalf * 32 + 16) = a1;
    *reinterpret_cast<uint4*>(sB + srow * kGPitch + shalf * 32) = b0;
    *reinterpret_cast<uint4*>(sB + srow * kGPitch + shalf * 32 + 16) = b1;
    if (tid < 128) sSa[tid] = fs;
    else sSw[tid - 128] = fs;
    __syncthreads();
    if (g + 1 < G) {
      a0 = *reinterpret_cast<const uint4*>(gA + (g + 1) * 64);
      a1 = *reinterpret_cast<const uint4*>(gA + (g + 1) * 64 + 16);
      b0 = *reinterpret_cast<const uint4*>(gB + (g + 1) * 64);
      b1 = *reinterpret_cast<const uint4*>(gB + (g + 1) * 64 + 16);
      fs = gS[(size_t)(g + 1) * sstep];
    }
    v16i iacc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) iacc[a][b][v] = 0;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      v4i fa[2], fb[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const uint4 w = *reinterpret_cast<const uint4*>(sA + (wm * 64 + a * 32 + l32) * kGPitch + ks * 32 + kg * 16);
        fa[a] = (v4i){(int)w.x, (int)w.y, (int)w.z, (int)w.w};
        const uint4 u = *reinterpret_cast<const uint4*>(sB + (wn * 64 + a * 32 + l32) * kGPitch + ks * 32 + kg * 16);
        fb[a] = (v4i){(int)u.x, (int)u.y, (int)u.z, (int)u.w};
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) iacc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[a], fb[b], iacc[a][b], 0, 0, 0);
    }
    // element v of lane (l32, kg) of block (a, b): row 32 a + 8 (v / 4) + 4 kg + v % 4, column 32 b + l32
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f4 s4 = *reinterpret_cast<const f4*>(sSa + wm * 64 + a * 32 + 8 * q + 4 * kg);
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const float swn = sSw[wn * 64 + b * 32 + l32];
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[a][b][4 * q + j] = __fmaf_rn(__fmul_rn((float)iacc[a][b][4 * q + j], s4[j]), swn, acc[a][b][4 * q + j]);
        }
      }
    }
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int n = n0 + wn * 64 + b * 32 + l32;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 64 + a * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
        if (m < M && n < N) Yt[(size_t)m * N + n] = acc[a][b][v];
      }
    }
}

// workgroups of 256 threads along a row; of one wave when that would leave the chip short of workgroups
inline int rows_block(int ld, int rows, int B) { return (long)((ld + 255) / 256) * rows * B >= 2048 ? 256 : 64; }
inline dim3 rows_grid(int ld, int rows, int B) {
  const int bs = rows_block(ld, rows, B);
  return dim3((ld + bs - 1) / bs, rows, B);
}

// sizes of the approximations after every level of the ragged transform over n tokens
std::vector<int> ragged_sizes(int n, int levels) {
  std::vector<int> sz{n};
  for (int l = 0; l < levels; ++l) sz.push_back((sz.back() + 1) / 2);
  return sz;
}

float haar_norm_host(int level) { return std::ldexp((level & 1) ? kC : 1.0f, -(level >> 1)); }

}  // namespace

// ---------------------------------------------------------------------------------------------
// Plan-time tables
// ---------------------------------------------------------------------------------------------
void stamp_gen_plan_free(stamp_plan* p) {
  if (p->perm_dev) (void)hipFree(p->perm_dev);
  if (p->ell_dev) (void)hipFree(p->ell_dev);
  if (p->dct_dev) (void)hipFree(p->dct_dev);
  if (p->qWg_dev) (void)hipFree(p->qWg_dev);
  if (p->swg_dev) (void)hipFree(p->swg_dev);
  p->ell_dev = p->swg_dev = nullptr;
  p->perm_dev = nullptr;
  p->dct_dev = nullptr;
  p->qWg_dev = nullptr;
}

namespace {
// l = L 1 in fp32, following the forward transform's operation order (host)
std::vector<float> ell_of(const stamp_plan* p) {
  const StampGen& gn = p->gen;
  const int s = p->geom.s;
  std::vector<float> t(s, 1.0f), ell(s, 0.0f);
  switch (gn.kind) {
    case kGenCopy: ell.assign(s, 1.0f); break;
    case kGenHaarRagged: {
      const int o = gn.skip ? 1 : 0;
      int n = s - o;
      if (o) ell[0] = 1.0f;
      std::vector<float> w(t.begin() + o, t.end());
      for (int l = 0; l < gn.levels; ++l) {
        const int m = n / 2, nn = (n + 1) / 2;
        std::vector<float> a(nn);
        for (int i = 0; i < m; ++i) {
          a[i] = (w[2 * i] + w[2 * i + 1]) * kC;
          ell[o + nn + i] = (w[2 * i] - w[2 * i + 1]) * kC;
        }
        if (n & 1) a[m] = w[n - 1];
        w = a;
        n = nn;
      }
      for (int i = 0; i < n; ++i) ell[o + i] = w[i];
      break;
    }
    case kGenHaarClassic: {  // details of a constant vanish; approximations: 2^J * 2^(-J/2)
      const int na = s >> gn.levels;
      for (int i = 0; i < na; ++i) ell[i] = std::ldexp(1.0f, gn.levels) * haar_norm_host(gn.levels);
      break;
    }
    case kGenHaar2d: {
      const int na = (gn.gridH >> gn.levels) * (gn.gridW >> gn.levels);
      for (int i = 0; i < na; ++i) ell[i] = std::ldexp(1.0f, 2 * gn.levels) * std::ldexp(1.0f, -gn.levels);
      break;
    }
    case kGenWht: {
      int J = 0;
      while ((1 << J) < s) ++J;
      ell[0] = (float)s * haar_norm_host(J);
      break;
    }
    case kGenDct: {
      const double pi = 3.14159265358979323846;
      for (int k = 0; k < s; ++k) {
        double acc = 0.0;
        for (int n = 0; n < s; ++n) acc += (k == 0) ? std::sqrt(1.0 / s) : std::cos(pi * (2.0 * n + 1.0) * k / (2.0 * s)) * std::sqrt(2.0 / s);
        ell[k] = (float)acc;
      }
      break;
    }
    default: break;
  }
  return ell;
}

template <typename Tp>
hipError_t upload(Tp** dst, const std::vector<Tp>& v, hipStream_t st) {
  hipError_t e = hipMalloc(reinterpret_cast<void**>(dst), v.size() * sizeof(Tp));
  if (e != hipSuccess) return e;
  // the host vector does not outlive this call: a blocking copy
  e = hipMemcpy(*dst, v.data(), v.size() * sizeof(Tp), hipMemcpyHostToDevice);
  (void)st;
  return e;
}
}  // namespace

hipError_t stamp_gen_plan_tables(stamp_plan* p, const float* W, hipStream_t st) {
  const StampGen& gn = p->gen;
  const StampGeom& g = p->geom;
  const int s = g.s;
  hipError_t e = hipSuccess;
  if (gn.kind == kGenWht) {
    // STaMP slot q (sequency q) takes row rev(gray(q)) of the Hadamard-ordered result: stored inverted, the slot of
    // every row, for the scatter of the transform's last pass
    int J = 0;
    while ((1 << J) < s) ++J;
    std::vector<int32_t> inv(s);
    for (int q = 0; q < s; ++q) {
      const int gr = q ^ (q >> 1);
      int rev = 0;
      for (int b = 0; b < J; ++b) rev |= ((gr >> b) & 1) << (J - 1 - b);
      inv[rev] = q;
    }
    if ((e = upload(&p->perm_dev, inv, st)) != hipSuccess) return e;
  }
  if (gn.kind == kGenDct) {
    if ((e = hipMalloc(reinterpret_cast<void**>(&p->dct_dev), sizeof(double) * (size_t)s * s)) != hipSuccess) return e;
    hipLaunchKernelGGL(k_gen_dct_matrix, dim3((s + 255) / 256, s), dim3(256), 0, st, p->dct_dev, s);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (gn.bias_mode == 1 && p->bias_dev != nullptr) {
    if ((e = upload(&p->ell_dev, ell_of(p), st)) != hipSuccess) return e;
  }
  if (gn.group == 64) {
    const int Npad = ((g.N + 127) / 128) * 128, G = g.d / 64;
    if ((e = hipMalloc(reinterpret_cast<void**>(&p->qWg_dev), (size_t)Npad * g.d)) != hipSuccess) return e;
    if ((e = hipMalloc(reinterpret_cast<void**>(&p->swg_dev), sizeof(float) * (size_t)G * Npad)) != hipSuccess) return e;
    const size_t sc = p->desc.w_is_out_by_in ? 1 : (size_t)g.N, sn = p->desc.w_is_out_by_in ? (size_t)g.d : 1;
    hipLaunchKernelGGL(k_gen_wquant_grouped, dim3(Npad / 256 + 1, G), dim3(256), 0, st, W, p->qWg_dev, p->swg_dev, g.d, g.N, Npad, sc, sn);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// Forward and inverse transforms
// ---------------------------------------------------------------------------------------------
namespace {
constexpr int kPass1d = 5;  // levels per pass of the 1-D kernels (32 values per thread)
constexpr int kPass2d = 2;  // of the 2-D kernels (4 x 4 values per thread)

template <int NLEV>
void launch_haar1d_fwd(dim3 grid, hipStream_t st, const void* in, int in_kind, float* apx_out, float* T, int s, int ld, int o, int n_lo,
                       int scaled, int last, const GenNorm& nm) {
  hipLaunchKernelGGL(k_gen_haar1d_fwd<NLEV>, grid, dim3(rows_block(ld, grid.y, grid.z)), 0, st, in, in_kind, apx_out, T, s, ld, o, n_lo, scaled, last, nm);
}
template <int NLEV>
void launch_haar1d_inv(dim3 grid, hipStream_t st, const float* apx_in, const float* S, float* apx_out, void* Y, const float* bias,
                       int y_bf16, int s, int ld, int o, int n_lo, int last) {
  hipLaunchKernelGGL(k_gen_haar1d_inv<NLEV>, grid, dim3(rows_block(ld, grid.y, grid.z)), 0, st, apx_in, S, apx_out, Y, bias, y_bf16, s, ld, o, n_lo, last);
}
template <int NLEV>
void launch_haar2d_fwd(dim3 grid, hipStream_t st, const void* in, int in_kind, float* ll_out, float* T, int s, int ld, int gridW, int w_lo,
                       int cells_lo, const GenBands& bd, int last, float apx_norm) {
  hipLaunchKernelGGL(k_gen_haar2d_fwd<NLEV>, grid, dim3(rows_block(ld, grid.y, grid.z)), 0, st, in, in_kind, ll_out, T, s, ld, gridW, w_lo, cells_lo, bd, last, apx_norm);
}
template <int NLEV>
void launch_haar2d_inv(dim3 grid, hipStream_t st, const float* ll_in, int first, const float* S, float* ll_out, void* Y, const float* bias,
                       int y_bf16, int s, int ld, int gridW, int w_lo, int cells_lo, const GenBands& bd, int last) {
  hipLaunchKernelGGL(k_gen_haar2d_inv<NLEV>, grid, dim3(rows_block(ld, grid.y, grid.z)), 0, st, ll_in, first, S, ll_out, Y, bias, y_bf16, s, ld, gridW, w_lo, cells_lo, bd, last);
}
template <int NLEV>
void launch_wht(dim3 grid, hipStream_t st, const void* in, int in_kind, float* out, void* Y, int out_kind, const int* inv_perm, float norm,
                const float* bias, int y_bf16, int s, int ld, int h_lo) {
  hipLaunchKernelGGL(k_gen_wht<NLEV>, grid, dim3(rows_block(ld, grid.y, grid.z)), 0, st, in, in_kind, out, Y, out_kind, inv_perm, norm, bias, y_bf16, s, ld, h_lo);
}

// slot of band W of 2-D level l: the final low-low block and the bands of the coarser levels come first
int band_base_2d(const StampGen& gn, int l) {
  int base = (gn.gridH >> gn.levels) * (gn.gridW >> gn.levels);
  for (int l2 = gn.levels; l2 > l; --l2) base += 3 * (gn.gridH >> l2) * (gn.gridW >> l2);
  return base;
}
}  // namespace

// X -> T (fp32, STaMP order) in buf[2] (buf[0] when there is nothing to transform); buf[0], buf[1] take the
// approximations between passes.
hipError_t stamp_gen_forward(const stamp_plan* p, const void* X, float* const (&buf)[3], float** T_out, hipStream_t st) {
  const StampGen& gn = p->gen;
  const StampGeom& g = p->geom;
  const int s = g.s, d = g.d, B = g.B;
  const int xk = g.x_bf16 ? 2 : 1;
  float* const T = buf[2];
  float* tmp[2] = {buf[0], buf[1]};
  const bool haar1d = gn.kind == kGenHaarRagged || gn.kind == kGenHaarClassic;
  if (gn.kind == kGenCopy || ((haar1d || gn.kind == kGenHaar2d) && gn.levels == 0)) {
    hipLaunchKernelGGL(k_gen_cast, rows_grid(d, s, B), dim3(rows_block(d, s, B)), 0, st, X, buf[0], s, d, g.x_bf16);
    *T_out = buf[0];
    return hipGetLastError();
  }
  *T_out = T;
  if (haar1d) {
    const int o = gn.skip ? 1 : 0, scaled = gn.kind == kGenHaarRagged;
    const std::vector<int> sz = ragged_sizes(s - o, gn.levels);
    const void* in = X;
    int in_kind = xk, flip = 0;
    for (int l = 0; l < gn.levels;) {
      const int nlev = std::min(kPass1d, gn.levels - l), last = l + nlev == gn.levels;
      GenNorm nm = {};
      for (int i = 0; i < nlev; ++i) nm.det[i] = haar_norm_host(l + 1 + i);
      nm.apx = haar_norm_host(gn.levels);
      const dim3 grid = rows_grid(d, sz[l + nlev], B);
      float* out = tmp[flip];
      switch (nlev) {
        case 1: launch_haar1d_fwd<1>(grid, st, in, in_kind, out, T, s, d, o, sz[l], scaled, last, nm); break;
        case 2: launch_haar1d_fwd<2>(grid, st, in, in_kind, out, T, s, d, o, sz[l], scaled, last, nm); break;
        case 3: launch_haar1d_fwd<3>(grid, st, in, in_kind, out, T, s, d, o, sz[l], scaled, last, nm); break;
        case 4: launch_haar1d_fwd<4>(grid, st, in, in_kind, out, T, s, d, o, sz[l], scaled, last, nm); break;
        default: launch_haar1d_fwd<5>(grid, st, in, in_kind, out, T, s, d, o, sz[l], scaled, last, nm); break;
      }
      in = out;
      in_kind = 0;
      flip ^= 1;
      l += nlev;
    }
    return hipGetLastError();
  }
  if (gn.kind == kGenHaar2d) {
    const void* in = X;
    int in_kind = xk, flip = 0;
    for (int l = 0; l < gn.levels;) {
      const int nlev = std::min(kPass2d, gn.levels - l), last = l + nlev == gn.levels;
      GenBands bd = {};
      for (int i = 0; i < nlev; ++i) {
        bd.base[i] = band_base_2d(gn, l + 1 + i);
        bd.norm[i] = std::ldexp(1.0f, -(l + 1 + i));
      }
      const int w_lo = gn.gridW >> l, h_lo = gn.gridH >> l, wp = w_lo >> nlev, hp = h_lo >> nlev;
      const dim3 grid = rows_grid(d, hp * wp, B);
      float* out = tmp[flip];
      const float an = std::ldexp(1.0f, -gn.levels);
      switch (nlev) {
        case 1: launch_haar2d_fwd<1>(grid, st, in, in_kind, out, T, s, d, gn.gridW, w_lo, h_lo * w_lo, bd, last, an); break;
        case 2: launch_haar2d_fwd<2>(grid, st, in, in_kind, out, T, s, d, gn.gridW, w_lo, h_lo * w_lo, bd, last, an); break;
        default: launch_haar2d_fwd<3>(grid, st, in, in_kind, out, T, s, d, gn.gridW, w_lo, h_lo * w_lo, bd, last, an); break;
      }
      in = out;
      in_kind = 0;
      flip ^= 1;
      l += nlev;
    }
    return hipGetLastError();
  }
  if (gn.kind == kGenWht) {
    int J = 0;
    while ((1 << J) < s) ++J;
    if (J == 0) {  // one token: the transform is the identity
      hipLaunchKernelGGL(k_gen_cast, rows_grid(d, s, B), dim3(rows_block(d, s, B)), 0, st, X, buf[0], s, d, g.x_bf16);
      *T_out = buf[0];
      return hipGetLastError();
    }
    const void* in = X;
    int in_kind = xk, flip = 0;
    for (int l = 0; l < J;) {
      const int nlev = std::min(kPass1d, J - l), last = l + nlev == J;
      const dim3 grid = rows_grid(d, s >> nlev, B);
      float* out = last ? T : tmp[flip];
      const int ok = last ? 1 : 0;
      const float nrm = haar_norm_host(J);
      switch (nlev) {
        case 1: launch_wht<1>(grid, st, in, in_kind, out, nullptr, ok, p->perm_dev, nrm, nullptr, 0, s, d, 1 << l); break;
        case 2: launch_wht<2>(grid, st, in, in_kind, out, nullptr, ok, p->perm_dev, nrm, nullptr, 0, s, d, 1 << l); break;
        case 3: launch_wht<3>(grid, st, in, in_kind, out, nullptr, ok, p->perm_dev, nrm, nullptr, 0, s, d, 1 << l); break;
        case 4: launch_wht<4>(grid, st, in, in_kind, out, nullptr, ok, p->perm_dev, nrm, nullptr, 0, s, d, 1 << l); break;
        default: launch_wht<5>(grid, st, in, in_kind, out, nullptr, ok, p->perm_dev, nrm, nullptr, 0, s, d, 1 << l); break;
      }
      in = out;
      in_kind = 0;
      flip ^= 1;
      l += nlev;
    }
    return hipGetLastError();
  }
  if (gn.kind == kGenDct) {
    hipLaunchKernelGGL(k_gen_cast, rows_grid(d, s, B), dim3(rows_block(d, s, B)), 0, st, X, buf[0], s, d, g.x_bf16);
    hipLaunchKernelGGL(k_gen_dct, dim3((d + 63) / 64, (s + 63) / 64, B), dim3(256), 0, st, p->dct_dev, 0, buf[0], T, s, d);
    return hipGetLastError();
  }
  return hipErrorInvalidValue;
}

// buf[0] = S, the transformed output in STaMP order (only read: the details of every level come from it); buf[1],
// buf[2] take the approximations between passes.  The last pass adds the bias and writes Y in the plan's output type.
hipError_t stamp_gen_inverse(const stamp_plan* p, float* const (&buf)[3], int ncols, const float* bias, void* Y, hipStream_t st) {
  const StampGen& gn = p->gen;
  const StampGeom& g = p->geom;
  const int s = g.s, B = g.B, ld = ncols;
  const float* S = buf[0];
  float* tmp[2] = {buf[1], buf[2]};
  const bool haar1d = gn.kind == kGenHaarRagged || gn.kind == kGenHaarClassic;
  if (gn.kind == kGenCopy || ((haar1d || gn.kind == kGenHaar2d) && gn.levels == 0)) {
    hipLaunchKernelGGL(k_gen_store_y, rows_grid(ld, s, B), dim3(rows_block(ld, s, B)), 0, st, S, bias, Y, s, ld, g.y_bf16);
    return hipGetLastError();
  }
  if (haar1d) {
    const int o = gn.skip ? 1 : 0;
    const std::vector<int> sz = ragged_sizes(s - o, gn.levels);
    // passes of up to kPass1d levels counted from the bottom, run from the top
    std::vector<int> cut{0};
    while (cut.back() < gn.levels) cut.push_back(std::min(gn.levels, cut.back() + kPass1d));
    const float* in = S;
    int flip = 0;
    for (int pi = (int)cut.size() - 1; pi >= 1; --pi) {
      const int l_lo = cut[pi - 1], nlev = cut[pi] - l_lo, last = l_lo == 0;
      const dim3 grid = rows_grid(ld, sz[l_lo + nlev], B);
      float* out = tmp[flip];
      switch (nlev) {
        case 1: launch_haar1d_inv<1>(grid, st, in, S, out, Y, bias, g.y_bf16, s, ld, o, sz[l_lo], last); break;
        case 2: launch_haar1d_inv<2>(grid, st, in, S, out, Y, bias, g.y_bf16, s, ld, o, sz[l_lo], last); break;
        case 3: launch_haar1d_inv<3>(grid, st, in, S, out, Y, bias, g.y_bf16, s, ld, o, sz[l_lo], last); break;
        case 4: launch_haar1d_inv<4>(grid, st, in, S, out, Y, bias, g.y_bf16, s, ld, o, sz[l_lo], last); break;
        default: launch_haar1d_inv<5>(grid, st, in, S, out, Y, bias, g.y_bf16, s, ld, o, sz[l_lo], last); break;
      }
      in = out;
      flip ^= 1;
    }
    return hipGetLastError();
  }
  if (gn.kind == kGenHaar2d) {
    std::vector<int> cut{0};
    while (cut.back() < gn.levels) cut.push_back(std::min(gn.levels, cut.back() + kPass2d));
    const float* in = S;
    int flip = 0, first = 1;
    for (int pi = (int)cut.size() - 1; pi >= 1; --pi) {
      const int l_lo = cut[pi - 1], nlev = cut[pi] - l_lo, last = l_lo == 0;
      GenBands bd = {};
      for (int i = 0; i < nlev; ++i) bd.base[i] = band_base_2d(gn, l_lo + 1 + i);
      const int w_lo = gn.gridW >> l_lo, h_lo = gn.gridH >> l_lo, wp = w_lo >> nlev, hp = h_lo >> nlev;
      const dim3 grid = rows_grid(ld, hp * wp, B);
      float* out = tmp[flip];
      switch (nlev) {
        case 1: launch_haar2d_inv<1>(grid, st, in, first, S, out, Y, bias, g.y_bf16, s, ld, gn.gridW, w_lo, h_lo * w_lo, bd, last); break;
        case 2: launch_haar2d_inv<2>(grid, st, in, first, S, out, Y, bias, g.y_bf16, s, ld, gn.gridW, w_lo, h_lo * w_lo, bd, last); break;
        default: launch_haar2d_inv<3>(grid, st, in, first, S, out, Y, bias, g.y_bf16, s, ld, gn.gridW, w_lo, h_lo * w_lo, bd, last); break;
      }
      in = out;
      first = 0;
      flip ^= 1;
    }
    return hipGetLastError();
  }
  if (gn.kind == kGenWht) {
    // the sequency-ordered orthonormal WHT is its own inverse
    int J = 0;
    while ((1 << J) < s) ++J;
    if (J == 0) {
      hipLaunchKernelGGL(k_gen_store_y, rows_grid(ld, s, B), dim3(rows_block(ld, s, B)), 0, st, S, bias, Y, s, ld, g.y_bf16);
      return hipGetLastError();
    }
    const float* in = S;
    int flip = 0;
    for (int l = 0; l < J;) {
      const int nlev = std::min(kPass1d, J - l), last = l + nlev == J;
      const dim3 grid = rows_grid(ld, s >> nlev, B);
      float* out = tmp[flip];
      const int ok = last ? 2 : 0;
      const float nrm = haar_norm_host(J);
      switch (nlev) {
        case 1: launch_wht<1>(grid, st, in, 0, out, Y, ok, p->perm_dev, nrm, bias, g.y_bf16, s, ld, 1 << l); break;
        case 2: launch_wht<2>(grid, st, in, 0, out, Y, ok, p->perm_dev, nrm, bias, g.y_bf16, s, ld, 1 << l); break;
        case 3: launch_wht<3>(grid, st, in, 0, out, Y, ok, p->perm_dev, nrm, bias, g.y_bf16, s, ld, 1 << l); break;
        case 4: launch_wht<4>(grid, st, in, 0, out, Y, ok, p->perm_dev, nrm, bias, g.y_bf16, s, ld, 1 << l); break;
        default: launch_wht<5>(grid, st, in, 0, out, Y, ok, p->perm_dev, nrm, bias, g.y_bf16, s, ld, 1 << l); break;
      }
      in = out;
      flip ^= 1;
      l += nlev;
    }
    return hipGetLastError();
  }
  if (gn.kind == kGenDct) {
    hipLaunchKernelGGL(k_gen_dct, dim3((ld + 63) / 64, (s + 63) / 64, B), dim3(256), 0, st, p->dct_dev, 1, S, tmp[0], s, ld);
    hipLaunchKernelGGL(k_gen_store_y, rows_grid(ld, s, B), dim3(rows_block(ld, s, B)), 0, st, tmp[0], bias, Y, s, ld, g.y_bf16);
    return hipGetLastError();
  }
  return hipErrorInvalidValue;
}

hipError_t stamp_launch_bf16_to_f32(const void* src, float* dst, size_t n, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_cast_flat, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, static_cast<const uint16_t*>(src), dst, n);
  return hipGetLastError();
}

hipError_t stamp_launch_quant_rows_grouped(const stamp_plan* p, const float* T, int8_t* codes, float* scales, hipStream_t st) {
  const StampGeom& g = p->geom;
  hipLaunchKernelGGL(k_gen_quant_grouped, dim3(g.s, g.B), dim3(256), 0, st, T, codes, scales, g.s, g.d, g.khi);
  return hipGetLastError();
}

hipError_t stamp_launch_gemm_grouped(const stamp_plan* p, const int8_t* codes, const float* scales, float* Yt, hipStream_t st) {
  const StampGeom& g = p->geom;
  const int M = g.B * g.s, Npad = ((g.N + 127) / 128) * 128;
  hipLaunchKernelGGL(k_gen_gemm_grouped, dim3(Npad / 128, (M + 127) / 128), dim3(256), 0, st, codes, scales, p->qWg_dev, p->swg_dev, Yt,
                     M, g.N, Npad, g.d);
  return hipGetLastError();
}

hipError_t stamp_launch_merge_hi(const stamp_plan* p, const float* ythi, int nparts, float* Yt, hipStream_t st) {
  const StampGeom& g = p->geom;
  if (g.k == 0) return hipSuccess;
  hipLaunchKernelGGL(k_gen_merge_hi, rows_grid(g.N, g.k, g.B), dim3(rows_block(g.N, g.k, g.B)), 0, st, ythi, nparts, (size_t)g.B * g.k * (size_t)g.N, Yt, g.s,
                     g.N, g.k);
  return hipGetLastError();
}

hipError_t stamp_launch_add_ell_bias(const stamp_plan* p, float* Yt, hipStream_t st) {
  const StampGeom& g = p->geom;
  hipLaunchKernelGGL(k_gen_add_ell_bias, rows_grid(g.N, g.s, g.B), dim3(rows_block(g.N, g.s, g.B)), 0, st, Yt, p->ell_dev, p->bias_dev, g.s, g.N);
  return hipGetLastError();
}
