// Plan-time weight quantization (not on the timed path): per output channel n,
// sw_n = max_c |W_cn| / 7 and code = rne(W_cn * (7 / max)) (round-to-nearest weights with one
// scale per output channel, paper sections "Experiments" set-up and "Large Language Models").
//
// Stored layout for the GEMM: int8 code * 16 (the GEMM keeps 4-bit values in the high nibble of an
// int8), tiled as [Npad/128 column tiles][Kpad/128 K steps][128 columns][128 channels], so that what
// one workgroup reads in one K step is one contiguous 16 KB run (spread over all memory channels)
// instead of 128 rows a power-of-two stride apart.  Inside every group of 16 input channels the order
// is [0,2,4,6, 1,3,5,7, 8,10,12,14, 9,11,13,15]: the order in which the GEMM's nibble unpack of 8
// packed activation bytes delivers its 16 channels.
#include "stamp_internal.h"

namespace {

__global__ void k_w_zero(uint32_t* colmax, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) colmax[i] = 0u;
}

// W element (c, n) at c * sc + n * sn
__global__ void k_w_colmax(const float* __restrict__ W, uint32_t* __restrict__ colmax, int d, int N, size_t sc,
                           size_t sn, int rows_per_block) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  const int c_begin = blockIdx.y * rows_per_block;
  const int c_end = min(d, c_begin + rows_per_block);
  float m = 0.0f;
  for (int c = c_begin; c < c_end; ++c) m = fmaxf(m, fabsf(W[(size_t)c * sc + (size_t)n * sn]));
  atomicMax(&colmax[n], __float_as_uint(m));
}

__global__ void k_w_quant(const float* __restrict__ W, const uint32_t* __restrict__ colmax, int8_t* __restrict__ qW,
                          float* __restrict__ sw, int d, int N, int Kpad, int Npad, size_t sc, size_t sn) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  const int g16 = blockIdx.y;
  if (n >= Npad) return;
  float a = 0.0f;
  if (n < N) a = __uint_as_float(colmax[n]);
  float scale = 0.0f, inv = 0.0f;
  if (a > 0.0f) {
    scale = __fdiv_rn(a, 7.0f);
    inv = __fdiv_rn(7.0f, a);
  }
  if (g16 == 0) sw[n] = scale;
  uint32_t out[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int pos = 0; pos < 16; ++pos) {
    // pos -> channel: half = pos / 8; within the half, first the four even channels, then the odd ones
    const int half = pos >> 3, i = pos & 7;
    const int c = g16 * 16 + half * 8 + ((i < 4) ? (2 * i) : (2 * (i - 4) + 1));
    int q = 0;
    if (n < N && c < d) {
      float r = rintf(__fmul_rn(W[(size_t)c * sc + (size_t)n * sn], inv));
      r = fminf(fmaxf(r, -7.0f), 7.0f);
      q = (int)r * 16;
    }
    out[pos >> 2] |= ((uint32_t)q & 0xFFu) << (8 * (pos & 3));
  }
  *reinterpret_cast<uint4*>(qW + stamp_w_offset(n, g16 * 16, Kpad)) = make_uint4(out[0], out[1], out[2], out[3]);
}

// Sum over the input channels of the weight codes of every output column, an exact integer held in fp32
// (|sum| <= 7 d_in): what the integer offset z of an asymmetric activation code multiplies, since
// sum_c (code_mc - z_m) qW_cn = sum_c code_mc qW_cn - z_m sum_c qW_cn (de-quantization function of the
// Background section).  Codes are recomputed from W exactly as k_w_quant does.
__global__ void k_w_colsum(const float* __restrict__ W, const uint32_t* __restrict__ colmax, float* __restrict__ colsum,
                           int d, int N, int Npad, size_t sc, size_t sn) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= Npad) return;
  int sum = 0;
  if (n < N) {
    const float a = __uint_as_float(colmax[n]);
    const float inv = a > 0.0f ? __fdiv_rn(7.0f, a) : 0.0f;
    for (int c = 0; c < d; ++c) {
      float r = rintf(__fmul_rn(W[(size_t)c * sc + (size_t)n * sn], inv));
      r = fminf(fmaxf(r, -7.0f), 7.0f);
      sum += (int)r;
    }
  }
  colsum[n] = (float)sum;
}

}  // namespace

hipError_t stamp_launch_weight_quant(const stamp_plan* p, const float* W, hipStream_t st, uint32_t* colmax_tmp) {
  const int d = p->geom.d, N = p->geom.N;
  const size_t sc = p->desc.w_is_out_by_in ? 1 : (size_t)N;
  const size_t sn = p->desc.w_is_out_by_in ? (size_t)d : 1;
  hipLaunchKernelGGL(k_w_zero, dim3((N + 255) / 256), dim3(256), 0, st, colmax_tmp, N);
  const int rows_per_block = 256;
  hipLaunchKernelGGL(k_w_colmax, dim3((N + 255) / 256, (d + rows_per_block - 1) / rows_per_block), dim3(256), 0, st, W,
                     colmax_tmp, d, N, sc, sn, rows_per_block);
  hipLaunchKernelGGL(k_w_quant, dim3((p->Npad + 255) / 256, p->Kpad / 16), dim3(256), 0, st, W, colmax_tmp, p->qW_dev,
                     p->sw_dev, d, N, p->Kpad, p->Npad, sc, sn);
  hipLaunchKernelGGL(k_w_colsum, dim3((p->Npad + 255) / 256), dim3(256), 0, st, W, colmax_tmp, p->colsum_dev, d, N, p->Npad,
                     sc, sn);
  return hipGetLastError();
}
