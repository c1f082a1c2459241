// Integer GEMM of the STaMP linear layer on gfx950 (step "Y <- X W" of Algorithm "STaMP Linear"):
//   acc[m, n] = sum_c code[m, c] * qW[c, n]     int8 x int8 -> int32 on v_mfma_i32_32x32x32_i8,
// followed in the same kernel by the dequantization Y' = float(acc) * scale_m * sw_n
// (Background, de-quantization function) and, in the fused mode, by the in-block levels of the
// inverse sequence transform (commutation identity of section "Method"), bias and the store of Y.
//
// Operands: 4-bit activation rows arrive packed two per byte; a packed dword w is split into
// (w << 4) & 0xF0F0F0F0 and w & 0xF0F0F0F0, i.e. the eight codes times 16 as int8.  The stored
// weights are code * 16 as well, pre-permuted to the channel order this split produces.  The
// factors 16 are exact powers of two and are folded into the row scale.
//
// Tile: 256 x 256 outputs per workgroup of 4 waves (2 x 2), 128 x 128 per wave = 4 x 4 MFMA blocks
// of 32 x 32; K step 128 codes; both operands staged in LDS K-major (row / column contiguous),
// double buffered, one barrier per K step.
#include "stamp_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 128;
constexpr int kStrideA4 = 80;    // bytes per LDS row of packed 4-bit A (64 data + 16 pad)
constexpr int kStrideB = 144;    // bytes per LDS row of int8 operand (128 data + 16 pad)
constexpr int kEpiStride = 33;   // floats per row of the per-wave epilogue staging tile

constexpr float kInvSqrt2 = 0.70710678118654752440f;

__device__ __forceinline__ float haar_norm_dev(int level, int is2d) {
  return is2d ? ldexpf(1.0f, -level) : ldexpf((level & 1) ? kInvSqrt2 : 1.0f, -(level >> 1));
}

struct GemmArgs {
  const uint8_t* A;      // A_INT4: q_lo [M][d/2]; else q_hi [M][d]
  const int8_t* Bq;      // [Npad][Kpad]
  const float* scales;   // [B*s] physical order
  const float* sw;       // [Npad]
  const float* bias;     // [Npad] or nullptr
  const float* P;        // [B*k][N] block sums of the inverse (fused mode)
  void* out;
  int M;                 // rows of A
  int N, Npad, Kpad;
  int a_row_bytes;       // valid bytes per A row
  StampGeom g;
};

// ---- in-register inverse of one block: x[e], e = in-block STaMP position -> natural token order ----
template <int R>
__device__ __forceinline__ void inverse_block_1d(float (&x)[R]) {
  // stage m: sums a[0 .. 2^m) sit in x[0 .. 2^m), differences in x[2^m .. 2^(m+1))
  float t[R];
#pragma unroll
  for (int n = 1; n < R; n <<= 1) {
#pragma unroll
    for (int i = 0; i < n; ++i) {
      t[2 * i] = x[i] + x[n + i];
      t[2 * i + 1] = x[i] - x[n + i];
    }
#pragma unroll
    for (int i = 0; i < 2 * n; ++i) x[i] = t[i];
  }
}

// 2-D: x[e] -> natural (y * g + x) order of a g x g block
template <int GS>
__device__ __forceinline__ void inverse_block_2d(float (&x)[GS * GS]) {
  float t[GS * GS];
#pragma unroll
  for (int n = 1; n < GS; n <<= 1) {  // current side of the sum grid
    // sums in x[0 .. n*n) row-major; bands W,H,D of side n at x[n*n*(1+band) + ...]
#pragma unroll
    for (int i = 0; i < n; ++i) {
#pragma unroll
      for (int j = 0; j < n; ++j) {
        const float cLL = x[i * n + j], cW = x[n * n + i * n + j], cH = x[2 * n * n + i * n + j],
                    cD = x[3 * n * n + i * n + j];
        const float t0 = cLL + cH, t2 = cLL - cH, t1 = cW + cD, t3 = cW - cD;
        t[(2 * i) * (2 * n) + 2 * j] = t0 + t1;
        t[(2 * i) * (2 * n) + 2 * j + 1] = t0 - t1;
        t[(2 * i + 1) * (2 * n) + 2 * j] = t2 + t3;
        t[(2 * i + 1) * (2 * n) + 2 * j + 1] = t2 - t3;
      }
    }
#pragma unroll
    for (int i = 0; i < 4 * n * n; ++i) x[i] = t[i];
  }
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// EPI: 0 = int32 accumulators to STaMP-ordered rows; 1 = dequantized fp32 rows (lo: physical rows of
// [B*s][N]; hi: [B*k][N]); 2 = fused in-block inverse + bias -> Y (A_INT4 only); RB = log2 of the
// block length for EPI 2 (1-D: tokens, 2-D: side).
template <bool A_INT4, int EPI, int RB, bool IS2D>
__global__ __launch_bounds__(256) void k_gemm(const GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  constexpr int strideA = A_INT4 ? kStrideA4 : kStrideB;
  constexpr int bytesA = BM * strideA, bytesB = BN * kStrideB;
  constexpr int stage = bytesA + bytesB;
  constexpr int a_chunks = A_INT4 ? 4 : 8;  // 16-byte chunks per A row per K step

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int ntn = a.Npad / BN;
  const int tn = blockIdx.x % ntn, tm = blockIdx.x / ntn;
  const int m0 = tm * BM, n0 = tn * BN;

  // global source of this thread: A row m0 + tid, B column n0 + tid
  const int arow = min(m0 + tid, a.M - 1);
  const uint8_t* gA = a.A + (size_t)arow * a.a_row_bytes;
  const int8_t* gB = a.Bq + (size_t)(n0 + tid) * a.Kpad;
  const int KT = a.Kpad / BK;

  uint4 ra[a_chunks], rb[8];
  auto gload = [&](int kt) {
#pragma unroll
    for (int c = 0; c < a_chunks; ++c) {
      const int off = kt * (A_INT4 ? 64 : 128) + c * 16;
      ra[c] = (off < a.a_row_bytes) ? *reinterpret_cast<const uint4*>(gA + off) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) rb[c] = *reinterpret_cast<const uint4*>(gB + kt * BK + c * 16);
  };
  auto sstore = [&](int buf) {
    uint8_t* sA = smem + buf * stage + tid * strideA;
    uint8_t* sB = smem + buf * stage + bytesA + tid * kStrideB;
#pragma unroll
    for (int c = 0; c < a_chunks; ++c) *reinterpret_cast<uint4*>(sA + c * 16) = ra[c];
#pragma unroll
    for (int c = 0; c < 8; ++c) *reinterpret_cast<uint4*>(sB + c * 16) = rb[c];
  };

  v16i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  gload(0);
  sstore(0);
  __syncthreads();

  const int l32 = lane & 31, kg = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) gload(kt + 1);
    const uint8_t* sA = smem + buf * stage + (wm * 128 + l32) * strideA;
    const uint8_t* sB = smem + buf * stage + bytesA + (wn * 128 + l32) * kStrideB;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      v4i fa[4], fb[4];
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
        if constexpr (A_INT4) {
          const uint2 w = *reinterpret_cast<const uint2*>(sA + mi * 32 * strideA + ks * 16 + kg * 8);
          fa[mi][0] = (int)((w.x << 4) & 0xF0F0F0F0u);
          fa[mi][1] = (int)(w.x & 0xF0F0F0F0u);
          fa[mi][2] = (int)((w.y << 4) & 0xF0F0F0F0u);
          fa[mi][3] = (int)(w.y & 0xF0F0F0F0u);
        } else {
          const uint4 w = *reinterpret_cast<const uint4*>(sA + mi * 32 * strideA + ks * 32 + kg * 16);
          // natural channel order -> the order of the stored weights: evens then odds per 8 channels
          fa[mi][0] = (int)__builtin_amdgcn_perm(w.y, w.x, 0x06040200u);
          fa[mi][1] = (int)__builtin_amdgcn_perm(w.y, w.x, 0x07050301u);
          fa[mi][2] = (int)__builtin_amdgcn_perm(w.w, w.z, 0x06040200u);
          fa[mi][3] = (int)__builtin_amdgcn_perm(w.w, w.z, 0x07050301u);
        }
      }
#pragma unroll
      for (int ni = 0; ni < 4; ++ni) {
        const uint4 w = *reinterpret_cast<const uint4*>(sB + ni * 32 * kStrideB + ks * 32 + kg * 16);
        fb[ni][0] = (int)w.x; fb[ni][1] = (int)w.y; fb[ni][2] = (int)w.z; fb[ni][3] = (int)w.w;
      }
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
    }
    if (kt + 1 < KT) sstore(buf ^ 1);
    __syncthreads();
  }

  // ------------------------------------------------------------------------------------------
  // Epilogue.  Accumulator element v of lane l in block (mi, ni): row 32 mi + 8 (v / 4) + 4 (l / 32)
  // + v % 4, column 32 ni + l % 32 of the wave tile.
  // ------------------------------------------------------------------------------------------
  const StampGeom& g = a.g;
  float* s_rowfac = reinterpret_cast<float*>(smem);            // [256]
  int* s_rowdst = reinterpret_cast<int*>(smem + 1024);         // [256] destination row or -1
  {
    const int m = m0 + tid;
    float fac = 0.0f;
    int dst = -1;
    if (m < a.M) {
      if constexpr (A_INT4) {
        const int b = m / g.s, pr = m - b * g.s;
        const int j = pr / g.R, e = pr - j * g.R;
        if (e != 0) {
          const int level = g.is2d ? stamp_level_of_e_2d(e, g.r) : stamp_level_of_e_1d(e, g.r);
          if constexpr (EPI != 0) fac = a.scales[m] * haar_norm_dev(level, g.is2d) * (1.0f / 256.0f);
          if (EPI == 0) {
            const int p = g.is2d ? stamp_slot_of_block_e_2d(j / g.G, j % g.G, e, g.G) : stamp_slot_of_block_e_1d(j, e, g.k);
            dst = b * g.s + p;
          } else {
            dst = m;
          }
        }
      } else {
        const int b = m / g.k, p = m - b * g.k;
        int level = g.J;
        if (p > 0) {
          const int lg = 31 - __builtin_clz((unsigned)p);
          level = g.J - (g.is2d ? (lg >> 1) : lg);
        }
        if constexpr (EPI != 0)
          fac = a.scales[(size_t)b * g.s + (size_t)p * g.R] * haar_norm_dev(level, g.is2d) * (1.0f / 16.0f);
        dst = (EPI == 0) ? (b * g.s + p) : m;
      }
    }
    s_rowfac[tid] = fac;
    s_rowdst[tid] = dst;
  }
  __syncthreads();

  if constexpr (EPI == 0 || EPI == 1) {
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int n = n0 + wn * 128 + ni * 32 + l32;
      const float swn = a.sw[n];
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int rl = wm * 128 + mi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
          const int dst = s_rowdst[rl];
          if (dst >= 0 && n < a.N) {
            if constexpr (EPI == 0) {
              reinterpret_cast<int32_t*>(a.out)[(size_t)dst * a.N + n] = acc[mi][ni][v] >> (A_INT4 ? 8 : 4);
            } else {
              reinterpret_cast<float*>(a.out)[(size_t)dst * a.N + n] = ((float)acc[mi][ni][v] * s_rowfac[rl]) * swn;
            }
          }
        }
      }
    }
  } else {
    // fused: per 32-column strip, dequantize into this wave's LDS tile [128][33], then each lane takes
    // one column of one block, inverts it in registers and stores R tokens.
    constexpr int R = IS2D ? (1 << (2 * RB)) : (1 << RB);
    constexpr int nblk = 128 / R;  // blocks per wave tile
    float* s_tile = reinterpret_cast<float*>(smem + 2048) + wave * (128 * kEpiStride);
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int n = n0 + wn * 128 + ni * 32 + l32;
      const float swn = a.sw[n];
      const float bias_n = (a.bias != nullptr) ? a.bias[n] : 0.0f;
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int rw = mi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
          s_tile[rw * kEpiStride + l32] = ((float)acc[mi][ni][v] * s_rowfac[wm * 128 + rw]) * swn;
        }
      }
      __syncthreads();
      for (int blk = kg; blk < nblk; blk += 2) {
        const int mrow = m0 + wm * 128 + blk * R;  // physical row of e = 0 of this block
        if (mrow < a.M && n < a.N) {
          const int b = mrow / g.s, pr = mrow - b * g.s;
          const int j = pr / g.R;
          float x[R];
#pragma unroll
          for (int e = 1; e < R; ++e) x[e] = s_tile[(blk * R + e) * kEpiStride + l32];
          x[0] = a.P[((size_t)b * g.k + j) * a.N + n];
          size_t tok0;
          int tstride_row;
          if constexpr (IS2D) {
            inverse_block_2d<(1 << RB)>(x);
            const int bi = j / g.G, bj = j - bi * g.G;
            tok0 = (size_t)b * g.s + (size_t)(bi << RB) * g.gridW + (size_t)(bj << RB);
            tstride_row = g.gridW;
          } else {
            inverse_block_1d<R>(x);
            tok0 = (size_t)b * g.s + (size_t)j * R;
            tstride_row = 0;
          }
#pragma unroll
          for (int t = 0; t < R; ++t) {
            size_t tok;
            if constexpr (IS2D) tok = tok0 + (size_t)(t >> RB) * tstride_row + (t & ((1 << RB) - 1));
            else tok = tok0 + t;
            const float y = x[t] + bias_n;
            if (g.y_bf16) reinterpret_cast<uint16_t*>(a.out)[tok * a.N + n] = f32_to_bf16_rne(y);
            else reinterpret_cast<float*>(a.out)[tok * a.N + n] = y;
          }
        }
      }
      __syncthreads();
    }
  }
}

template <bool A_INT4, int EPI, int RB, bool IS2D>
hipError_t launch(const GemmArgs& a, hipStream_t st) {
  constexpr int strideA = A_INT4 ? kStrideA4 : kStrideB;
  constexpr size_t main_lds = 2 * (size_t)(BM * strideA + BN * kStrideB);
  constexpr size_t epi_lds = 2048 + 4 * 128 * kEpiStride * sizeof(float);
  constexpr size_t lds = main_lds > epi_lds ? main_lds : epi_lds;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<A_INT4, EPI, RB, IS2D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int mt = (a.M + BM - 1) / BM, nt = a.Npad / BN;
  hipLaunchKernelGGL((k_gemm<A_INT4, EPI, RB, IS2D>), dim3(mt * nt), dim3(256), lds, st, a);
  return hipGetLastError();
}

GemmArgs make_args(const stamp_plan* p, const float* scales, void* out) {
  GemmArgs a;
  a.Bq = p->qW_dev;
  a.scales = scales;
  a.sw = p->sw_dev;
  a.bias = p->bias_dev;
  a.P = nullptr;
  a.out = out;
  a.N = p->geom.N;
  a.Npad = p->Npad;
  a.Kpad = p->Kpad;
  a.g = p->geom;
  a.A = nullptr;
  a.M = 0;
  a.a_row_bytes = 0;
  return a;
}

}  // namespace

hipError_t stamp_launch_gemm_hi(const stamp_plan* p, const int8_t* q_hi, const float* scales, int mode, void* out,
                                hipStream_t st) {
  GemmArgs a = make_args(p, scales, out);
  a.A = reinterpret_cast<const uint8_t*>(q_hi);
  a.M = p->geom.B * p->geom.k;
  a.a_row_bytes = p->geom.d;
  if (mode == 0) return launch<false, 0, 0, false>(a, st);
  if (mode == 1) return launch<false, 1, 0, false>(a, st);
  return hipErrorInvalidValue;
}

hipError_t stamp_launch_gemm_lo(const stamp_plan* p, const uint8_t* q_lo, const float* scales, int mode, void* out,
                                const float* P, hipStream_t st) {
  GemmArgs a = make_args(p, scales, out);
  a.A = q_lo;
  a.M = p->geom.B * p->geom.s;
  a.a_row_bytes = p->geom.d / 2;
  a.P = P;
  if (mode == 0) return launch<true, 0, 0, false>(a, st);
  if (mode == 1) return launch<true, 1, 0, false>(a, st);
  if (mode != 2) return hipErrorInvalidValue;
  const StampGeom& g = p->geom;
  if (!g.is2d) {
    switch (g.r) {
      case 3: return launch<true, 2, 3, false>(a, st);
      case 4: return launch<true, 2, 4, false>(a, st);
      case 5: return launch<true, 2, 5, false>(a, st);
      case 6: return launch<true, 2, 6, false>(a, st);
      default: return hipErrorInvalidValue;
    }
  }
  switch (g.r) {
    case 2: return launch<true, 2, 2, true>(a, st);
    case 3: return launch<true, 2, 3, true>(a, st);
    default: return hipErrorInvalidValue;
  }
}
