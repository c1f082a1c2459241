// Inverse sequence transform Y = L^-1 Y' = L^T Y' (step "Y <- L^-1 Y" of Algorithm "STaMP Linear";
// L is orthogonal, Theorem 1) as two kernels mirroring the forward split:
//   k_inverse_top     the J-r top levels: the k_hi coarse coefficients of every (sequence, column)
//                     -> the k_hi block sums P (the level-r sums of the inverse).
//   k_inverse_bottom  the r levels inside each block of R tokens, from P and the R-1 in-block
//                     coefficients, then bias and the store in original token order.
// Both work on a slice of 32 output columns held in LDS, butterflies in place (stride 2^l).
// Every coefficient is multiplied by the norm 2^(-l/2) of its level first (either by the producer,
// folded into the dequantization scale, or here when apply_norm is set); the butterflies are then
// plain sums and differences.  The output tolerance does not depend on this order.
#include "stamp_internal.h"

namespace {

typedef float f4v __attribute__((ext_vector_type(4)));
constexpr int kCols = 32;
constexpr int kStride = kCols + 1;
constexpr float kInvSqrt2 = 0.70710678118654752440f;

__device__ __forceinline__ float haar_norm_dev(int level, int is2d) {
  return is2d ? ldexpf(1.0f, -level) : ldexpf((level & 1) ? kInvSqrt2 : 1.0f, -(level >> 1));
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// in-place inverse butterflies, `levels` levels (strides 2^levels .. 2), over n (1-D) or side x side (2-D)
// entries of s_buf[.][kStride]
__device__ __forceinline__ void inverse_inplace(float* s_buf, int n, int side, int is2d, int levels, int ch, int grp,
                                                int ngrp) {
  if (!is2d) {
    for (int st = 1 << levels; st >= 2; st >>= 1) {
      const int npair = n / st;
      for (int i = grp; i < npair; i += ngrp) {
        float* pa = &s_buf[(i * st) * kStride + ch];
        float* pd = &s_buf[(i * st + (st >> 1)) * kStride + ch];
        const float a = *pa, dd = *pd;
        *pa = a + dd;
        *pd = a - dd;
      }
      __syncthreads();
    }
  } else {
    for (int st = 1 << levels; st >= 2; st >>= 1) {
      const int nc = side / st, h = st >> 1;
      for (int i = grp; i < nc * nc; i += ngrp) {
        const int cy = i / nc, cx = i - cy * nc;
        float* p00 = &s_buf[((cy * st) * side + cx * st) * kStride + ch];
        float* p01 = p00 + h * kStride;
        float* p10 = p00 + h * side * kStride;
        float* p11 = p10 + h * kStride;
        const float cLL = *p00, cW = *p01, cH = *p10, cD = *p11;
        const float t0 = cLL + cH, t2 = cLL - cH, t1 = cW + cD, t3 = cW - cD;
        *p00 = t0 + t1;
        *p01 = t0 - t1;
        *p10 = t2 + t3;
        *p11 = t2 - t3;
      }
      __syncthreads();
    }
  }
}

// src: hi rows; row of (b, p) = b * src_seq_rows + p; nparts partial copies, part_stride floats apart, are
// added in order.  P[(b*k + j) * ldP + n].
__global__ __launch_bounds__(256) void k_inverse_top(const float* __restrict__ src, int src_seq_rows, int apply_norm,
                                                     float* __restrict__ P, int ldP, int ncols, StampGeom g, int nparts,
                                                     size_t part_stride) {
  extern __shared__ float s_buf[];  // [k][kStride]
  const int b = blockIdx.y, n_base = blockIdx.x * kCols, tid = threadIdx.x;
  const int ch = tid & (kCols - 1), grp = tid / kCols, ngrp = 256 / kCols;
  const int n = n_base + ch;
  const bool nact = n < ncols;
  const int k = g.k;
  // plans without top levels may have more than 256 top rows: nothing is transformed, every workgroup (blockIdx.z)
  // moves its own 256 of them
  const int q0 = (int)blockIdx.z * 256, kq = min(k - q0, 256);
  for (int ql = grp; ql < kq; ql += ngrp) {
    const int q = q0 + ql;
    int e, lvl_top;
    if (!g.is2d) {
      e = stamp_top_slot_1d(q, k, g.L, &lvl_top);
    } else {
      const int y = q / g.G, x = q - y * g.G;
      e = stamp_top_slot_2d(y, x, g.G, g.L, &lvl_top);
    }
    float v = 0.0f;
    if (nact) {
      const size_t idx = ((size_t)b * src_seq_rows + e) * ncols + n;
      v = src[idx];
      for (int part = 1; part < nparts; ++part) v += src[idx + part * part_stride];
    }
    if (apply_norm) v *= haar_norm_dev(g.r + lvl_top, g.is2d);
    s_buf[ql * kStride + ch] = v;
  }
  __syncthreads();
  inverse_inplace(s_buf, kq, g.G, g.is2d, g.L, ch, grp, ngrp);  // L > 0: kq = k
  for (int ql = grp; ql < kq; ql += ngrp)
    if (nact) P[((size_t)b * k + q0 + ql) * ldP + n] = s_buf[ql * kStride + ch];
}

// src rows of block (b, j): physical (b*s + j*R + e) or STaMP slot order; Y [B, s, ncols].
__global__ __launch_bounds__(256) void k_inverse_bottom(const float* __restrict__ src, int src_is_stamp, int apply_norm,
                                                        const float* __restrict__ P, int ldP,
                                                        const float* __restrict__ bias, void* __restrict__ Y, int ncols,
                                                        StampGeom g) {
  extern __shared__ float s_buf[];  // [R][kStride]
  const int j = blockIdx.y, b = blockIdx.z, n_base = blockIdx.x * kCols, tid = threadIdx.x;
  const int ch = tid & (kCols - 1), grp = tid / kCols, ngrp = 256 / kCols;
  const int n = n_base + ch;
  const bool nact = n < ncols;
  const int R = g.R;
  const int bi = g.is2d ? j / g.G : 0, bj = g.is2d ? j - bi * g.G : 0;
  for (int q = grp; q < R; q += ngrp) {
    float v = 0.0f;
    if (q == 0) {
      if (nact) v = P[((size_t)b * g.k + j) * ldP + n];
    } else {
      int e, level;
      if (!g.is2d) {
        e = stamp_e_of_natural_1d(q, R);
        level = __builtin_ctz((unsigned)q) + 1;
      } else {
        const int y = q / g.g, x = q - y * g.g;
        e = stamp_e_of_natural_2d(y, x, g.g);
        level = __builtin_ctz((unsigned)(y | x)) + 1;
      }
      size_t row;
      if (src_is_stamp) {
        const int p = g.is2d ? stamp_slot_of_block_e_2d(bi, bj, e, g.G) : stamp_slot_of_block_e_1d(j, e, g.k);
        row = (size_t)b * g.s + p;
      } else {
        row = (size_t)b * g.s + (size_t)j * R + e;
      }
      if (nact) v = src[row * ncols + n];
      if (apply_norm) v *= haar_norm_dev(level, g.is2d);
    }
    s_buf[q * kStride + ch] = v;
  }
  __syncthreads();
  inverse_inplace(s_buf, R, g.g, g.is2d, g.r, ch, grp, ngrp);
  const float bias_n = (bias != nullptr && nact) ? bias[n] : 0.0f;
  for (int q = grp; q < R; q += ngrp) {
    size_t tok;
    if (!g.is2d) {
      tok = (size_t)b * g.s + (size_t)j * R + q;
    } else {
      const int y = q / g.g, x = q - y * g.g;
      tok = (size_t)b * g.s + (size_t)(bi * g.g + y) * g.gridW + (size_t)(bj * g.g + x);
    }
    if (nact) {
      const float yv = s_buf[q * kStride + ch] + bias_n;
      if (g.y_bf16) reinterpret_cast<uint16_t*>(Y)[tok * ncols + n] = f32_to_bf16_rne(yv);
      else reinterpret_cast<float*>(Y)[tok * ncols + n] = yv;
    }
  }
}

}  // namespace

namespace {
// identity plans: sum of the partial dequantized 8-bit rows + bias -> rows of tokens 0..k-1 of Y
__global__ __launch_bounds__(256) void k_hi_rows_out(const float* __restrict__ src, int nparts, size_t part_stride,
                                                     const float* __restrict__ bias, void* __restrict__ Y, int k, int s, int N,
                                                     int y_bf16) {
  const int row = blockIdx.y;  // b * k + p
  const int b = row / k, p = row - b * k;
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  const size_t idx = (size_t)row * N + n;
  float v = src[idx];
  for (int part = 1; part < nparts; ++part) v += src[idx + part * part_stride];
  if (bias != nullptr) v += bias[n];
  const size_t o = ((size_t)b * s + p) * N + n;
  if (y_bf16) reinterpret_cast<uint16_t*>(Y)[o] = f32_to_bf16_rne(v);
  else reinterpret_cast<float*>(Y)[o] = v;
}
}  // namespace

hipError_t stamp_launch_hi_rows_out(const stamp_plan* p, const float* Yt_hi, void* Y, hipStream_t st, int nparts) {
  const StampGeom& g = p->geom;
  if (g.k == 0) return hipSuccess;
  hipLaunchKernelGGL(k_hi_rows_out, dim3((g.N + 255) / 256, g.B * g.k), dim3(256), 0, st, Yt_hi, nparts,
                     (size_t)g.B * g.k * (size_t)g.N, p->bias_dev, Y, g.k, g.s, g.N, g.y_bf16);
  return hipGetLastError();
}

namespace {
// plans without top levels, split depth: P[row][n] = sum of the parts' rows (no transform, no reordering)
__global__ __launch_bounds__(256) void k_sum_parts(const float* __restrict__ src, int nparts, size_t part_stride,
                                                   float* __restrict__ P, int ldP, int ncols) {
  const int row = blockIdx.y;
  const int n = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (n >= ncols) return;
  const size_t idx = (size_t)row * ncols + n;
  if (n + 3 < ncols && (ncols & 3) == 0) {
    f4v v = *reinterpret_cast<const f4v*>(src + idx);
    for (int part = 1; part < nparts; ++part) v += *reinterpret_cast<const f4v*>(src + idx + part * part_stride);
    *reinterpret_cast<f4v*>(P + (size_t)row * ldP + n) = v;
  } else {
    for (int c = n; c < ncols && c < n + 4; ++c) {
      float v = src[(size_t)row * ncols + c];
      for (int part = 1; part < nparts; ++part) v += src[(size_t)row * ncols + c + part * part_stride];
      P[(size_t)row * ldP + c] = v;
    }
  }
}
}  // namespace

hipError_t stamp_launch_sum_parts(const float* src, int nparts, int nrows, int ncols, float* P, int ldP, hipStream_t st) {
  hipLaunchKernelGGL(k_sum_parts, dim3((ncols + 1023) / 1024, nrows), dim3(256), 0, st, src, nparts,
                     (size_t)nrows * (size_t)ncols, P, ldP, ncols);
  return hipGetLastError();
}

hipError_t stamp_launch_inverse_top(const stamp_plan* p, const float* src, int src_is_stamp, int ncols, float* P,
                                    int ldP, hipStream_t st, int nparts) {
  const StampGeom& g = p->geom;
  if (g.L == 0 && !src_is_stamp) {
    // nothing to invert and the rows are in place already: only the parts of a split depth are added
    return stamp_launch_sum_parts(src, nparts, g.B * g.k, ncols, P, ldP, st);
  }
  if (g.k > 256 && g.L != 0) return hipErrorInvalidValue;  // plan creation admits that many top rows only without top levels
  const int kl = g.k < 256 ? g.k : 256;
  const size_t lds = (size_t)kl * kStride * sizeof(float);
  hipLaunchKernelGGL(k_inverse_top, dim3((ncols + kCols - 1) / kCols, g.B, (g.k + 255) / 256), dim3(256), lds, st, src,
                     src_is_stamp ? g.s : g.k, src_is_stamp, P, ldP, ncols, g, nparts, (size_t)g.B * g.k * (size_t)ncols);
  return hipGetLastError();
}

hipError_t stamp_launch_inverse_bottom(const stamp_plan* p, const float* src, int src_is_stamp, const float* P,
                                       int ldP, int ncols, const float* bias, void* Y, hipStream_t st) {
  const StampGeom& g = p->geom;
  const size_t lds = (size_t)g.R * kStride * sizeof(float);
  hipLaunchKernelGGL(k_inverse_bottom, dim3((ncols + kCols - 1) / kCols, g.k, g.B), dim3(256), lds, st, src,
                     src_is_stamp, src_is_stamp, P, ldP, bias, Y, ncols, g);
  return hipGetLastError();
}
