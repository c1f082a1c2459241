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

// grid: x = ceil(row_elems / 256), y = rows of this launch, z = batch; one thread per element of a row
#define GEN_INDEX                                      \
  const int c = blockIdx.x * 256 + threadIdx.x;        \
  const int i = blockIdx.y;                            \
  const size_t bo = (size_t)blockIdx.z * seq * ld;     \
  if (c >= ld) return

// X (bf16 or fp32) -> fp32
__global__ __launch_bounds__(256) void k_gen_cast(const void* __restrict__ X, float* __restrict__ dst, int seq, int ld, int bf16) {
  GEN_INDEX;
  const size_t idx = bo + (size_t)i * ld + c;
  dst[idx] = bf16 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(X)[idx] << 16) : reinterpret_cast<const float*>(X)[idx];
}

// dst rows [dst0, dst0 + rows) = src rows [src0, ...) * norm (norm_tab[dst row] if given), optionally through a row
// permutation: dst row r takes src row perm[r]
// (src may be dst: every thread reads and writes one element of its own)
__global__ __launch_bounds__(256) void k_gen_copy_rows(const float* src, float* dst, int seq, int ld,
                                                       int src0, int dst0, const float* __restrict__ norm_tab,
                                                       const int* __restrict__ perm) {
  GEN_INDEX;
  const int dr = dst0 + i;
  const int sr = perm != nullptr ? perm[dr] : src0 + i;
  float v = src[bo + (size_t)sr * ld + c];
  if (norm_tab != nullptr) v = __fmul_rn(v, norm_tab[dr]);
  dst[bo + (size_t)dr * ld + c] = v;
}

// One level of the 1-D Haar transform over the n approximations that start at row o of `src`: pair i < n / 2 ->
// approximation to row o + i of `dst`, detail to row o + ceil(n / 2) + i of `T`; an odd last approximation is
// carried to row o + n / 2 of `dst`.  scaled: multiply by C (ragged form); else plain sums (classic form).
__global__ __launch_bounds__(256) void k_gen_haar1d_fwd(const float* __restrict__ src, float* __restrict__ dst,
                                                        float* __restrict__ T, int seq, int ld, int o, int n, int scaled) {
  GEN_INDEX;
  const int m = n >> 1, nn = (n + 1) >> 1;
  if (i < m) {
    const float x0 = src[bo + (size_t)(o + 2 * i) * ld + c], x1 = src[bo + (size_t)(o + 2 * i + 1) * ld + c];
    float a = __fadd_rn(x0, x1), dd = __fsub_rn(x0, x1);
    if (scaled) {
      a = __fmul_rn(a, kC);
      dd = __fmul_rn(dd, kC);
    }
    dst[bo + (size_t)(o + i) * ld + c] = a;
    T[bo + (size_t)(o + nn + i) * ld + c] = dd;
  } else {  // i == m, n odd
    dst[bo + (size_t)(o + m) * ld + c] = src[bo + (size_t)(o + n - 1) * ld + c];
  }
}

// Inverse of one level: approximations rows [o, o + nn) of `src`, details rows [o + nn, o + nn + m) of `S` ->
// rows [o, o + n) of `dst`; both outputs times C (the orthonormal butterfly is its own inverse).
__global__ __launch_bounds__(256) void k_gen_haar1d_inv(const float* __restrict__ src, const float* __restrict__ S,
                                                        float* __restrict__ dst, int seq, int ld, int o, int n) {
  GEN_INDEX;
  const int m = n >> 1, nn = (n + 1) >> 1;
  if (i < m) {
    const float a = src[bo + (size_t)(o + i) * ld + c], dd = S[bo + (size_t)(o + nn + i) * ld + c];
    dst[bo + (size_t)(o + 2 * i) * ld + c] = (a + dd) * kC;
    dst[bo + (size_t)(o + 2 * i + 1) * ld + c] = (a - dd) * kC;
  } else {
    dst[bo + (size_t)(o + n - 1) * ld + c] = src[bo + (size_t)(o + m) * ld + c];
  }
}

// One level of the 2-D Haar pyramid on the h x w low-low region (grid pitch gridW, token = r * gridW + c) of `src`:
// cell (ci, cj) -> low-low to grid position (ci, cj) of `dst` (plain sums), the three details times 2^-level to
// their STaMP slots in `T` (band_base = slot of the level's first band; bands W, H, D, each (h/2) x (w/2)).
// blockIdx.y = cell index ci * (w / 2) + cj.
__global__ __launch_bounds__(256) void k_gen_haar2d_fwd(const float* __restrict__ src, float* __restrict__ dst,
                                                        float* __restrict__ T, int seq, int ld, int gridW, int w,
                                                        int band_base, float norm) {
  GEN_INDEX;
  const int w2 = w >> 1, ci = i / w2, cj = i - ci * w2;
  const size_t r0 = bo + ((size_t)(2 * ci) * gridW + 2 * cj) * ld + c, r1 = r0 + (size_t)gridW * ld;
  const float p = src[r0], q = src[r0 + ld], u = src[r1], v = src[r1 + ld];
  const float t0 = __fadd_rn(p, q), t1 = __fsub_rn(p, q), t2 = __fadd_rn(u, v), t3 = __fsub_rn(u, v);
  dst[bo + ((size_t)ci * gridW + cj) * ld + c] = __fadd_rn(t0, t2);
  const int cells = (int)gridDim.y;  // (h / 2) * (w / 2)
  T[bo + (size_t)(band_base + i) * ld + c] = __fmul_rn(__fadd_rn(t1, t3), norm);
  T[bo + (size_t)(band_base + cells + i) * ld + c] = __fmul_rn(__fsub_rn(t0, t2), norm);
  T[bo + (size_t)(band_base + 2 * cells + i) * ld + c] = __fmul_rn(__fsub_rn(t1, t3), norm);
}

// final low-low block (hl x wl at grid pitch gridW of `src`) -> STaMP slots 0 .. hl * wl - 1 of T, times norm
__global__ __launch_bounds__(256) void k_gen_ll_to_slots(const float* __restrict__ src, float* __restrict__ T, int seq, int ld,
                                                         int gridW, int wl, float norm) {
  GEN_INDEX;
  const int r = i / wl, cc = i - r * wl;
  T[bo + (size_t)i * ld + c] = __fmul_rn(src[bo + ((size_t)r * gridW + cc) * ld + c], norm);
}
__global__ __launch_bounds__(256) void k_gen_slots_to_ll(const float* __restrict__ S, float* __restrict__ dst, int seq, int ld,
                                                         int gridW, int wl) {
  GEN_INDEX;
  const int r = i / wl, cc = i - r * wl;
  dst[bo + ((size_t)r * gridW + cc) * ld + c] = S[bo + (size_t)i * ld + c];
}

// Inverse of one 2-D level: low-low (h/2 x w/2 region of `src`, grid layout) and the level's bands (STaMP slots of
// `S`) -> h x w region of `dst`; every output times 1/2 (the orthonormal 2-D butterfly).
__global__ __launch_bounds__(256) void k_gen_haar2d_inv(const float* __restrict__ src, const float* __restrict__ S,
                                                        float* __restrict__ dst, int seq, int ld, int gridW, int w, int band_base) {
  GEN_INDEX;
  const int w2 = w >> 1, ci = i / w2, cj = i - ci * w2, cells = (int)gridDim.y;
  const float cLL = src[bo + ((size_t)ci * gridW + cj) * ld + c];
  const float cW = S[bo + (size_t)(band_base + i) * ld + c], cH = S[bo + (size_t)(band_base + cells + i) * ld + c],
              cD = S[bo + (size_t)(band_base + 2 * cells + i) * ld + c];
  const float t0 = cLL + cH, t2 = cLL - cH, t1 = cW + cD, t3 = cW - cD;
  const size_t r0 = bo + ((size_t)(2 * ci) * gridW + 2 * cj) * ld + c, r1 = r0 + (size_t)gridW * ld;
  dst[r0] = (t0 + t1) * 0.5f;
  dst[r0 + ld] = (t0 - t1) * 0.5f;
  dst[r1] = (t2 + t3) * 0.5f;
  dst[r1 + ld] = (t2 - t3) * 0.5f;
}

// One level of the Hadamard-ordered fast WHT: rows j and j + h of every group of 2 h rows -> sum, difference.
// blockIdx.y = pair index.
__global__ __launch_bounds__(256) void k_gen_wht_level(const float* __restrict__ src, float* __restrict__ dst, int seq, int ld, int h) {
  GEN_INDEX;
  const int blk = i / h, t = i - blk * h;
  const size_t r0 = bo + (size_t)(blk * 2 * h + t) * ld + c, r1 = r0 + (size_t)h * ld;
  const float u = src[r0], v = src[r1];
  dst[r0] = __fadd_rn(u, v);
  dst[r1] = __fsub_rn(u, v);
}

// dst[k, c] = fl32( sum_n Mx[k, n] * src[n, c] ) in fp64 (Mx = C, or C^T when transposed), per batch.
// 64 x 64 outputs per workgroup of 256 threads (4 x 4 per thread), 16 values of n per pass through LDS.
__global__ __launch_bounds__(256) void k_gen_dct(const double* __restrict__ Cm, int transposed, const float* __restrict__ src,
                                                 float* __restrict__ dst, int seq, int ld) {
  __shared__ double sM[16][65];
  __shared__ double sX[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int k0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const size_t bo = (size_t)blockIdx.z * seq * ld;
  double acc[4][4] = {};
  for (int n0 = 0; n0 < seq; n0 += 16) {
    for (int e = threadIdx.x; e < 16 * 64; e += 256) {
      const int nn = e >> 6, kk = e & 63;  // consecutive threads: consecutive k
      const int k = k0 + kk, n = n0 + nn;
      double mv = 0.0;
      if (k < seq && n < seq) mv = transposed ? Cm[(size_t)n * seq + k] : Cm[(size_t)k * seq + n];
      sM[nn][kk] = mv;
      const int cc = c0 + kk;
      sX[nn][kk] = (n < seq && cc < ld) ? (double)src[bo + (size_t)n * ld + cc] : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int nn = 0; nn < 16; ++nn) {
      double mk[4], xc[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        mk[a] = sM[nn][ty * 4 + a];
        xc[a] = sX[nn][tx * 4 + a];
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] += mk[a] * xc[b];
    }
    __syncthreads();
  }
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int k = k0 + ty * 4 + a, cc = c0 + tx * 4 + b;
      if (k < seq && cc < ld) dst[bo + (size_t)k * ld + cc] = (float)acc[a][b];
    }
}

__global__ void k_gen_dct_matrix(double* __restrict__ Cm, int s) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x, k = blockIdx.y;
  if (n >= s) return;
  const double pi = 3.14159265358979323846;
  Cm[(size_t)k * s + n] = (k == 0) ? sqrt(1.0 / s) : cos(pi * (2.0 * n + 1.0) * (double)k / (2.0 * s)) * sqrt(2.0 / s);
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
// g on v_mfma_i32_32x32x32_i8 (two per group and 32 x 32 block), groups added in increasing order, every floating-
// point operation rounded on its own.  Workgroup: 4 waves (2 x 2), tile 128 x 128, wave 64 x 64 = 2 x 2 blocks.
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
  for (int g = 0; g < G; ++g) {
    const uint4 a0 = *reinterpret_cast<const uint4*>(gA + g * 64), a1 = *reinterpret_cast<const uint4*>(gA + g * 64 + 16);
    const uint4 b0 = *reinterpret_cast<const uint4*>(gB + g * 64), b1 = *reinterpret_cast<const uint4*>(gB + g * 64 + 16);
    float fsa = 0.0f, fsw = 0.0f;
    if (tid < 128) fsa = sa[(size_t)min(m0 + tid, M - 1) * G + g];
    else fsw = swg[(size_t)g * Npad + n0 + (tid - 128)];
    __syncthreads();  // the previous group's fragments have been read
    *reinterpret_cast<uint4*>(sA + srow * kGPitch + shalf * 32) = a0;
    *reinterpret_cast<uint4*>(sA + srow * kGPitch + shalf * 32 + 16) = a1;
    *reinterpret_cast<uint4*>(sB + srow * kGPitch + shalf * 32) = b0;
    *reinterpret_cast<uint4*>(sB + srow * kGPitch + shalf * 32 + 16) = b1;
    if (tid < 128) sSa[tid] = fsa;
    else sSw[tid - 128] = fsw;
    __syncthreads();
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
            acc[a][b][4 * q + j] = __fadd_rn(acc[a][b][4 * q + j], __fmul_rn(__fmul_rn((float)iacc[a][b][4 * q + j], s4[j]), swn));
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

inline dim3 rows_grid(int ld, int rows, int B) { return dim3((ld + 255) / 256, rows, B); }

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
  if (p->norm_dev) (void)hipFree(p->norm_dev);
  if (p->perm_dev) (void)hipFree(p->perm_dev);
  if (p->ell_dev) (void)hipFree(p->ell_dev);
  if (p->dct_dev) (void)hipFree(p->dct_dev);
  if (p->qWg_dev) (void)hipFree(p->qWg_dev);
  if (p->swg_dev) (void)hipFree(p->swg_dev);
  p->norm_dev = p->ell_dev = p->swg_dev = nullptr;
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
  if (gn.kind == kGenHaarClassic) {
    std::vector<float> nrm(s);
    const int na = s >> gn.levels;
    for (int i = 0; i < na; ++i) nrm[i] = haar_norm_host(gn.levels);
    for (int l = gn.levels; l >= 1; --l)
      for (int i = s >> l; i < (s >> (l - 1)); ++i) nrm[i] = haar_norm_host(l);
    if ((e = upload(&p->norm_dev, nrm, st)) != hipSuccess) return e;
  }
  if (gn.kind == kGenWht) {
    int J = 0;
    while ((1 << J) < s) ++J;
    std::vector<int32_t> perm(s);
    for (int q = 0; q < s; ++q) {
      const int gr = q ^ (q >> 1);
      int rev = 0;
      for (int b = 0; b < J; ++b) rev |= ((gr >> b) & 1) << (J - 1 - b);
      perm[q] = rev;
    }
    if ((e = upload(&p->perm_dev, perm, st)) != hipSuccess) return e;
    std::vector<float> nrm(s, haar_norm_host(J));
    if ((e = upload(&p->norm_dev, nrm, st)) != hipSuccess) return e;
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
hipError_t stamp_gen_forward(const stamp_plan* p, const void* X, float* const (&buf)[3], float** T_out, hipStream_t st) {
  const StampGen& gn = p->gen;
  const StampGeom& g = p->geom;
  const int s = g.s, d = g.d, B = g.B;
  float *P = buf[0], *Q = buf[1], *T = buf[2];
  hipLaunchKernelGGL(k_gen_cast, rows_grid(d, s, B), dim3(256), 0, st, X, P, s, d, g.x_bf16);
  switch (gn.kind) {
    case kGenCopy:
      *T_out = P;
      break;
    case kGenHaarRagged:
    case kGenHaarClassic: {
      const int o = gn.skip ? 1 : 0, scaled = gn.kind == kGenHaarRagged;
      int n = s - o;
      for (int l = 0; l < gn.levels; ++l) {
        hipLaunchKernelGGL(k_gen_haar1d_fwd, rows_grid(d, (n + 1) / 2, B), dim3(256), 0, st, P, Q, T, s, d, o, n, scaled);
        std::swap(P, Q);
        n = (n + 1) / 2;
      }
      // what is left: the approximations -> slots [o, o + n); token 0, when it is left out, -> slot 0
      hipLaunchKernelGGL(k_gen_copy_rows, rows_grid(d, n, B), dim3(256), 0, st, P, T, s, d, o, o,
                         static_cast<const float*>(nullptr), static_cast<const int*>(nullptr));
      if (o)
        hipLaunchKernelGGL(k_gen_copy_rows, rows_grid(d, 1, B), dim3(256), 0, st, buf[0], T, s, d, 0, 0,
                           static_cast<const float*>(nullptr), static_cast<const int*>(nullptr));
      if (!scaled && gn.levels > 0)  // classic form: one multiplication by the level's norm at the end
        hipLaunchKernelGGL(k_gen_copy_rows, rows_grid(d, s, B), dim3(256), 0, st, T, T, s, d, 0, 0, p->norm_dev,
                           static_cast<const int*>(nullptr));
      *T_out = T;
      break;
    }
    case kGenHaar2d: {
      int h = gn.gridH, w = gn.gridW;
      // slot of the first band of level l: the low-low block and the bands of the coarser levels come first
      for (int l = 1; l <= gn.levels; ++l) {
        int base = (gn.gridH >> gn.levels) * (gn.gridW >> gn.levels);
        for (int l2 = gn.levels; l2 > l; --l2) base += 3 * (gn.gridH >> l2) * (gn.gridW >> l2);
        hipLaunchKernelGGL(k_gen_haar2d_fwd, rows_grid(d, (h / 2) * (w / 2), B), dim3(256), 0, st, P, Q, T, s, d, gn.gridW, w, base,
                           std::ldexp(1.0f, -l));
        std::swap(P, Q);
        h /= 2;
        w /= 2;
      }
      hipLaunchKernelGGL(k_gen_ll_to_slots, rows_grid(d, h * w, B), dim3(256), 0, st, P, T, s, d, gn.gridW, w, std::ldexp(1.0f, -gn.levels));
      *T_out = T;
      break;
    }
    case kGenWht: {
      for (int h = 1; h < s; h *= 2) {
        hipLaunchKernelGGL(k_gen_wht_level, rows_grid(d, s / 2, B), dim3(256), 0, st, P, Q, s, d, h);
        std::swap(P, Q);
      }
      hipLaunchKernelGGL(k_gen_copy_rows, rows_grid(d, s, B), dim3(256), 0, st, P, T, s, d, 0, 0, p->norm_dev, p->perm_dev);
      *T_out = T;
      break;
    }
    case kGenDct:
      hipLaunchKernelGGL(k_gen_dct, dim3((d + 63) / 64, (s + 63) / 64, B), dim3(256), 0, st, p->dct_dev, 0, P, T, s, d);
      *T_out = T;
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// buf[0] = S, the transformed output in STaMP order (only read: the details of every level come from it); buf[1],
// buf[2] take the approximations of successive levels in turn.
hipError_t stamp_gen_inverse(const stamp_plan* p, float* const (&buf)[3], int ncols, const float* bias, void* Y, hipStream_t st) {
  const StampGen& gn = p->gen;
  const StampGeom& g = p->geom;
  const int s = g.s, B = g.B, ld = ncols;
  float* S = buf[0];
  const float* src = S;
  float* dst = buf[1];
  auto flip = [&]() {
    src = dst;
    dst = (dst == buf[1]) ? buf[2] : buf[1];
  };
  switch (gn.kind) {
    case kGenCopy:
      break;
    case kGenHaarRagged:
    case kGenHaarClassic: {
      const int o = gn.skip ? 1 : 0;
      const std::vector<int> sz = ragged_sizes(s - o, gn.levels);
      for (int l = gn.levels; l >= 1; --l) {
        hipLaunchKernelGGL(k_gen_haar1d_inv, rows_grid(ld, (sz[l - 1] + 1) / 2, B), dim3(256), 0, st, src, S, dst, s, ld, o, sz[l - 1]);
        flip();
      }
      if (gn.levels > 0 && o)  // the token that was left out of L sits in slot 0
        hipLaunchKernelGGL(k_gen_copy_rows, rows_grid(ld, 1, B), dim3(256), 0, st, S, const_cast<float*>(src), s, ld, 0, 0,
                           static_cast<const float*>(nullptr), static_cast<const int*>(nullptr));
      break;
    }
    case kGenHaar2d: {
      // approximations in grid layout (pitch gridW) in the top-left corner of the work buffers
      int h = gn.gridH >> gn.levels, w = gn.gridW >> gn.levels;
      const int ll = h * w;
      hipLaunchKernelGGL(k_gen_slots_to_ll, rows_grid(ld, ll, B), dim3(256), 0, st, S, dst, s, ld, gn.gridW, w);
      flip();
      for (int l = gn.levels; l >= 1; --l) {
        int base = ll;
        for (int l2 = gn.levels; l2 > l; --l2) base += 3 * (gn.gridH >> l2) * (gn.gridW >> l2);
        h *= 2;
        w *= 2;
        hipLaunchKernelGGL(k_gen_haar2d_inv, rows_grid(ld, (h / 2) * (w / 2), B), dim3(256), 0, st, src, S, dst, s, ld, gn.gridW, w, base);
        flip();
      }
      break;
    }
    case kGenWht: {
      // the sequency-ordered orthonormal WHT is its own inverse
      for (int h = 1; h < s; h *= 2) {
        hipLaunchKernelGGL(k_gen_wht_level, rows_grid(ld, s / 2, B), dim3(256), 0, st, src, dst, s, ld, h);
        flip();
      }
      hipLaunchKernelGGL(k_gen_copy_rows, rows_grid(ld, s, B), dim3(256), 0, st, src, dst, s, ld, 0, 0, p->norm_dev, p->perm_dev);
      flip();
      break;
    }
    case kGenDct:
      hipLaunchKernelGGL(k_gen_dct, dim3((ld + 63) / 64, (s + 63) / 64, B), dim3(256), 0, st, p->dct_dev, 1, src, dst, s, ld);
      flip();
      break;
    default:
      return hipErrorInvalidValue;
  }
  hipLaunchKernelGGL(k_gen_store_y, rows_grid(ld, s, B), dim3(256), 0, st, src, bias, Y, s, ld, g.y_bf16);
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
  hipLaunchKernelGGL(k_gen_merge_hi, rows_grid(g.N, g.k, g.B), dim3(256), 0, st, ythi, nparts, (size_t)g.B * g.k * (size_t)g.N, Yt, g.s,
                     g.N, g.k);
  return hipGetLastError();
}

hipError_t stamp_launch_add_ell_bias(const stamp_plan* p, float* Yt, hipStream_t st) {
  const StampGeom& g = p->geom;
  hipLaunchKernelGGL(k_gen_add_ell_bias, rows_grid(g.N, g.s, g.B), dim3(256), 0, st, Yt, p->ell_dev, p->bias_dev, g.s, g.N);
  return hipGetLastError();
}
