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
// of 32 x 32 (256 accumulator registers per lane); K step of 128 codes.  Both operands are staged in
// LDS K-major (one row / column = one contiguous run of 64 or 128 bytes) in 16-byte chunks whose slot
// is XOR-swizzled with the row number, so that the 16 lanes of a fragment read hit 16 distinct
// 16-byte bank groups; two stages, one barrier per K step.  Lane group kg (lane / 32) of an MFMA
// takes channels [64 kg + 16 ks, +16) of the step in sub-step ks: any assignment is valid as long
// as both operands use it, and this one makes every fragment read a whole 16-byte chunk.
// Workgroups are renumbered so that the 32 workgroups resident on one XCD cover 8 x 4 neighbouring
// tiles and share operand panels in that XCD's L2.
#include <cstdlib>
#include <type_traits>

#include "stamp_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));  // first-class 16-byte value (keeps staging arrays in registers)
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BK = 128;  // BN = 64 * NI (NI = 32-column MFMA blocks per wave along N)
constexpr int kEpiStride = 36;  // floats per row of the per-wave epilogue staging tile (16-byte aligned rows)
constexpr int kNumXcd = 8;
constexpr int kGroupM = 8;

constexpr float kInvSqrt2 = 0.70710678118654752440f;

__device__ __forceinline__ float haar_norm_dev(int level, int is2d) {
  return is2d ? ldexpf(1.0f, -level) : ldexpf((level & 1) ? kInvSqrt2 : 1.0f, -(level >> 1));
}

struct GemmArgs {
  const uint8_t* A;      // A_INT4: q_lo tiled [Mpad/256][KT][256][64]; else q_hi [M][d]
  const int8_t* Bq;      // tiled [Npad/128][Kpad/128][128][128]
  const float* scales;   // [B*s] physical order
  const float* sw;       // [Npad]
  const float* bias;     // [Npad] or nullptr
  const float* P;        // [B*k][Npad] block sums of the inverse (fused mode)
  void* out;
  int M;                 // rows of A
  int N, Npad, Kpad;
  int a_row_bytes;       // valid bytes per A row
  size_t a_last16;       // byte offset of the last 16-byte chunk of A (loads are clamped to it)
  StampGeom g;
};


typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

// Where one lane stores the tokens of one unit (a block or an aligned part of one): 4 adjacent output
// columns per token, written as one 8-byte (bf16) or 16-byte (fp32) store when d_out allows it.
template <bool YBF16, bool VEC>
struct OutQuad {
  void* Y;
  size_t base;        // element index of token 0 of the block, first of the 4 columns
  size_t tok_stride;  // d_out
  size_t row_stride;  // 2-D: grid_w * d_out
  f4 bias;
  int nvalid;         // how many of the 4 columns exist (d_out tail)
  __device__ __forceinline__ void put(size_t idx, f4 v) const {
    v += bias;
    if constexpr (YBF16) {
      // round-to-nearest-even pairs in hardware (v_cvt_pk_bf16_f32)
      const uint32_t lo = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){v[0], v[1]}, bf2));
      const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){v[2], v[3]}, bf2));
      uint16_t* y = reinterpret_cast<uint16_t*>(Y) + idx;
      if constexpr (VEC) {
        *reinterpret_cast<uint2*>(y) = make_uint2(lo, hi);
      } else {
        if (nvalid > 0) y[0] = (uint16_t)lo;
        if (nvalid > 1) y[1] = (uint16_t)(lo >> 16);
        if (nvalid > 2) y[2] = (uint16_t)hi;
        if (nvalid > 3) y[3] = (uint16_t)(hi >> 16);
      }
    } else {
      float* y = reinterpret_cast<float*>(Y) + idx;
      if constexpr (VEC) {
        *reinterpret_cast<f4*>(y) = v;
      } else {
        if (nvalid > 0) y[0] = v[0];
        if (nvalid > 1) y[1] = v[1];
        if (nvalid > 2) y[2] = v[2];
        if (nvalid > 3) y[3] = v[3];
      }
    }
  }
};

// Depth-first inverse of one unit for 4 columns.  The unit is the subtree rooted at node (M0, h) of a
// block's Haar tree; node (M, I) of that subtree holds the sum `a` of its tokens; tile[e * kEpiStride]
// is the block's coefficient at in-block STaMP position e = 2^M + (h << (M - M0)) + I.  Only O(r)
// values are live at any time and every coefficient is read once.
template <int RLOG, int M0, int M, int I, typename Out>
__device__ __forceinline__ void dfs1d(const float* tile, int h, f4 a, const Out& o) {
  if constexpr (M == RLOG) {
    o.put(o.base + (size_t)((h << (RLOG - M0)) + I) * o.tok_stride, a);
  } else {
    const f4 d = *reinterpret_cast<const f4*>(tile + ((1 << M) + (h << (M - M0)) + I) * kEpiStride);
    dfs1d<RLOG, M0, M + 1, 2 * I, Out>(tile, h, a + d, o);
    dfs1d<RLOG, M0, M + 1, 2 * I + 1, Out>(tile, h, a - d, o);
  }
}

// 2-D: the unit is the quadtree node (M0, hy, hx) of a g x g block; bands W, H, D of level-node side
// gl = 2^M sit at e = gl^2 (1 + band) + iy * gl + ix.
template <int RLOG, int M0, int M, int IY, int IX, typename Out>
__device__ __forceinline__ void dfs2d(const float* tile, int hy, int hx, f4 a, const Out& o) {
  if constexpr (M == RLOG) {
    o.put(o.base + (size_t)((hy << (RLOG - M0)) + IY) * o.row_stride + (size_t)((hx << (RLOG - M0)) + IX) * o.tok_stride, a);
  } else {
    constexpr int gl = 1 << M;
    const int e0 = ((hy << (M - M0)) + IY) * gl + ((hx << (M - M0)) + IX);
    const f4 cW = *reinterpret_cast<const f4*>(tile + (gl * gl + e0) * kEpiStride);
    const f4 cH = *reinterpret_cast<const f4*>(tile + (2 * gl * gl + e0) * kEpiStride);
    const f4 cD = *reinterpret_cast<const f4*>(tile + (3 * gl * gl + e0) * kEpiStride);
    const f4 t0 = a + cH, t2 = a - cH, t1 = cW + cD, t3 = cW - cD;
    dfs2d<RLOG, M0, M + 1, 2 * IY, 2 * IX, Out>(tile, hy, hx, t0 + t1, o);
    dfs2d<RLOG, M0, M + 1, 2 * IY, 2 * IX + 1, Out>(tile, hy, hx, t0 - t1, o);
    dfs2d<RLOG, M0, M + 1, 2 * IY + 1, 2 * IX, Out>(tile, hy, hx, t2 + t3, o);
    dfs2d<RLOG, M0, M + 1, 2 * IY + 1, 2 * IX + 1, Out>(tile, hy, hx, t2 - t3, o);
  }
}

// Shape of the fused epilogue for block size RB: R tokens per block, units of at most 16 tokens (the
// subtree at depth M0 of a block's tree), U units per block, npass passes of 8 units per wave tile.
template <int RB, bool IS2D>
struct EpiShape {
  static constexpr int R = IS2D ? (1 << (2 * RB)) : (1 << RB);
  static constexpr int nblk = 128 / R;
  static constexpr int M0 = IS2D ? (RB == 3 ? 1 : 0) : (RB > 4 ? RB - 4 : 0);
  static constexpr int U = IS2D ? (1 << (2 * M0)) : (1 << M0);
  static constexpr int npass = (nblk * U) / 8;
};

// EPI: 0 = int32 accumulators to STaMP-ordered rows; 1 = dequantized fp32 rows (lo: physical rows of
// [B*s][N]; hi: [B*k][N]); 2 = fused in-block inverse + bias -> Y (A_INT4 only); RB = log2 of the
// block length for EPI 2 (1-D: tokens, 2-D: side).
template <bool A_INT4, int EPI, int RB, bool IS2D, int NI, bool YBF16>
__global__ __launch_bounds__(256, (NI == 2 ? 2 : 1)) void k_gemm(const GemmArgs a) {
  constexpr int BN = 64 * NI;
  constexpr int nB = BN / 32;                   // B chunks per thread per step (BN columns * 8 chunks / 256 threads)
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  constexpr int rowA = A_INT4 ? 64 : 128;       // bytes per A row per K step
  constexpr int chA = rowA / 16;                // 16-byte chunks per A row (4 or 8)
  constexpr int bytesA = BM * rowA, bytesB = BN * 128;
  constexpr int stage = bytesA + bytesB;
  constexpr int nA = chA;                       // A chunks per thread per step (256 rows * chA / 256 threads)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;  // wave tile: rows [128 wm, +128), columns [32 NI wn, +32 NI)
  const int l32 = lane & 31, kg = lane >> 5;

  // ---- workgroup -> tile, XCD aware: consecutive ids on one XCD walk 8 M-tiles, then the next N-tile ----
  const int mt = (a.M + BM - 1) / BM, nt = a.Npad / BN;
  int tm, tn;
  {
    const int total = mt * nt;
    const int bid = blockIdx.x;
    const int xcd = bid % kNumXcd, local = bid / kNumXcd;
    const int tall = total / kNumXcd, rem = total % kNumXcd;
    const int sid = xcd * tall + min(xcd, rem) + local;
    const int per_group = kGroupM * nt;
    const int grp = sid / per_group, in_grp = sid - grp * per_group;
    const int gm = min(kGroupM, mt - grp * kGroupM);
    tm = grp * kGroupM + in_grp % gm;
    tn = in_grp / gm;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const int KT = a.Kpad / BK;

  // ---- global -> LDS assignment: chunk q = i * 256 + tid of the tile, consecutive lanes = consecutive
  //      chunks.  Row / column of chunk i is (row0 + i * rows_per_pass); its swizzled slot does not
  //      depend on i, so one base address per operand and a uniform stride per pass suffice. ----
  constexpr int rowsPerPassA = 256 / chA;  // 64 (4-bit) or 32 (8-bit) rows per pass of 256 threads
  const int rowA0 = tid / chA, slotA = tid % chA;
  const int cA = A_INT4 ? (slotA ^ ((rowA0 >> 2) & 3)) : (slotA ^ ((rowA0 >> 1) & 7));
  const int koffA = cA * 16;
  // Addresses are a wave-uniform base (tile and K step) plus a per-thread 32-bit offset that never
  // changes, so the per-step address arithmetic is scalar.
  // 4-bit rows come tiled [M/256][KT][256 rows][64 bytes] (one contiguous 16 KB run per tile and step;
  // rows beyond M and channels beyond d_in hold whatever is there: masked in the epilogue, or multiplied
  // by the zero padding of the stored weights).  8-bit rows are plain row-major [M][d_in]: rows beyond M
  // re-read row M-1, chunks past the end of a row are clamped into the buffer (zero weights there).
  uint32_t offA[nA];
  const uint8_t* baseGA = a.A;
  const size_t kStepA = A_INT4 ? (size_t)(256 * 64) : (size_t)128;
#pragma unroll
  for (int i = 0; i < nA; ++i) {
    if constexpr (A_INT4) {
      offA[i] = (uint32_t)((rowA0 + i * rowsPerPassA) * 64 + koffA);
    } else {
      offA[i] = (uint32_t)(min(m0 + rowA0 + i * rowsPerPassA, a.M - 1) - m0) * (uint32_t)a.a_row_bytes + koffA;
    }
  }
  if constexpr (A_INT4) baseGA += (size_t)tm * KT * (256 * 64);
  else baseGA += (size_t)m0 * a.a_row_bytes;
  // byte offset (from baseGA) of the last 16-byte chunk that may be read
  const size_t lastA = a.a_last16 - (size_t)(baseGA - a.A);
  const int colB0 = tid >> 3, slotB = tid & 7;
  const int cB = slotB ^ ((colB0 >> 1) & 7);
  // stored weight: [Npad/128][KT][128 columns][128 bytes]; pass i of this thread is column colB0 + 32 i
  // (column tiles of 128: a 256-wide tile spans two of them, KT * 16 KB apart)
  const int8_t* baseGB = a.Bq + stamp_w_offset(n0, 0, a.Kpad);
  uint32_t offB[nB];
#pragma unroll
  for (int i = 0; i < nB; ++i) {
    const int col = colB0 + 32 * i;
    offB[i] = (uint32_t)(col >> 7) * (uint32_t)(KT * 128 * 128) + (uint32_t)((col & 127) * 128 + cB * 16);
  }
  constexpr int kStepB = 128 * 128;  // bytes between consecutive K steps of one column tile

  // ---- LDS -> fragment addresses (bytes inside a stage).  The swizzle term of a row depends only on
  //      lane bits, and sub-step ks enters through an XOR of bits 4-5, so per operand one base per lane
  //      is enough: address(block i, ks) = (base ^ (ks << 4)) + i * block_stride. ----
  int baseA, baseB;
  {
    const int r = wm * 128 + l32;
    baseA = A_INT4 ? (r * 64 + (((2 * kg) ^ ((r >> 2) & 3)) << 4)) : (r * 128 + (((4 * kg) ^ ((r >> 1) & 7)) << 4));
    const int n = wn * (32 * NI) + l32;
    baseB = bytesA + n * 128 + (((4 * kg) ^ ((n >> 1) & 7)) << 4);
  }
  constexpr int blkA = 32 * rowA, blkB = 32 * 128;  // LDS bytes between consecutive 32-row blocks

  v16i acc[4][NI];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  // Operand staging: asynchronous global -> LDS loads (16 bytes per lane, a wave instruction fills 1 KB
  // of contiguous LDS; the XOR swizzle is applied on the global-address side).  No registers are held
  // while a K step is in flight and nothing has to be copied into LDS by the waves.
#define STAMP_REQUEST(KSTEP, STG)                                                                          \
  do {                                                                                                     \
    uint8_t* so_ = smem + (STG) * stage + wave * 1024;                                                     \
    const size_t ka_ = (size_t)(KSTEP) * kStepA, kb_ = (size_t)(KSTEP) * kStepB;                           \
    _Pragma("unroll") for (int i = 0; i < nA; ++i) {                                                       \
      const uint8_t* src_ = A_INT4 ? (baseGA + ka_ + offA[i]) : (baseGA + min(ka_ + offA[i], lastA));      \
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src_,                \
                                       (void __attribute__((address_space(3)))*)(so_ + i * 4096), 16, 0, 0); \
    }                                                                                                      \
    _Pragma("unroll") for (int i = 0; i < nB; ++i)                                                         \
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(baseGB + kb_ + offB[i]), \
                                         (void __attribute__((address_space(3)))*)(so_ + bytesA + i * 4096), 16, 0, 0); \
  } while (0)

  // Fused epilogue: its global operands (weight scales, bias, block sums P of this lane's units) are
  // requested here, ahead of the main loop, so that their latency is not on the epilogue's path.
  using ES = EpiShape<(EPI == 2 ? RB : 3), IS2D>;
  [[maybe_unused]] float e_sw[NI];
  [[maybe_unused]] f4 e_bias[NI];
  [[maybe_unused]] f4 e_top[NI][ES::npass];
  if constexpr (EPI == 2) {
    const int c4 = (lane & 7) * 4, ug = lane >> 3;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int nw = n0 + wn * (32 * NI) + ni * 32;
      e_sw[ni] = a.sw[nw + l32];
      e_bias[ni] = (a.bias != nullptr) ? *reinterpret_cast<const f4*>(a.bias + nw + c4) : (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int pass = 0; pass < ES::npass; ++pass) {
        const int blk = (pass * 8 + ug) / ES::U;
        const int mrow = min(m0 + wm * 128 + blk * ES::R, a.M - 1);
        e_top[ni][pass] = *reinterpret_cast<const f4*>(a.P + (size_t)(mrow / a.g.R) * a.Npad + nw + c4);
      }
    }
  }

  constexpr int NSTAGE = (NI == 4 && A_INT4) ? 3 : 2;  // LDS stages: loads run NSTAGE-1 K steps ahead of the MFMAs
  constexpr int kLoadsPerStep = nA + nB;
#pragma unroll
  for (int p = 0; p < NSTAGE - 1; ++p)
    if (p < KT) STAMP_REQUEST(p, p);

  // Step kt: wait for this wave's loads of step kt (the NSTAGE-2 younger steps stay in flight), then the
  // workgroup barrier (every wave's loads of step kt have landed, and every wave has left step kt-1,
  // whose stage is now free); request step kt+NSTAGE-1 into that free stage; run the MFMAs of step kt.
  for (int kt = 0; kt < KT; ++kt) {
    const uint8_t* st = smem + (kt % NSTAGE) * stage;
    asm volatile("" ::: "memory");
    if (NSTAGE == 3 && kt + 1 < KT) __builtin_amdgcn_s_waitcnt(0x0F70 | (kLoadsPerStep & 15) | ((kLoadsPerStep >> 4) << 14));  // vmcnt(one step's loads)
    else __builtin_amdgcn_s_waitcnt(0x0F70);                                               // vmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kt + NSTAGE - 1 < KT) STAMP_REQUEST(kt + NSTAGE - 1, (kt + NSTAGE - 1) % NSTAGE);
    __builtin_amdgcn_sched_barrier(0);

    v4i fb[2][NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const u4 w = *reinterpret_cast<const u4*>(st + baseB + ni * blkB);
      fb[0][ni][0] = (int)w.x; fb[0][ni][1] = (int)w.y; fb[0][ni][2] = (int)w.z; fb[0][ni][3] = (int)w.w;
    }
    if constexpr (A_INT4) {
      u4 pa[4][2];
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
        pa[mi][0] = *reinterpret_cast<const u4*>(st + baseA + mi * blkA);
        pa[mi][1] = *reinterpret_cast<const u4*>(st + (baseA ^ 16) + mi * blkA);
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        if (ks < 3) {
#pragma unroll
          for (int ni = 0; ni < NI; ++ni) {
            const u4 w = *reinterpret_cast<const u4*>(st + (baseB ^ ((ks + 1) << 4)) + ni * blkB);
            fb[(ks + 1) & 1][ni][0] = (int)w.x; fb[(ks + 1) & 1][ni][1] = (int)w.y;
            fb[(ks + 1) & 1][ni][2] = (int)w.z; fb[(ks + 1) & 1][ni][3] = (int)w.w;
          }
        }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
          const u4 p = pa[mi][ks >> 1];
          const uint32_t w0 = (ks & 1) ? p.z : p.x, w1 = (ks & 1) ? p.w : p.y;
          v4i fa;
          fa[0] = (int)((w0 << 4) & 0xF0F0F0F0u);
          fa[1] = (int)(w0 & 0xF0F0F0F0u);
          fa[2] = (int)((w1 << 4) & 0xF0F0F0F0u);
          fa[3] = (int)(w1 & 0xF0F0F0F0u);
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb[ks & 1][ni], acc[mi][ni], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        u4 wa[4];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) wa[mi] = *reinterpret_cast<const u4*>(st + (baseA ^ (ks << 4)) + mi * blkA);
        if (ks < 3) {
#pragma unroll
          for (int ni = 0; ni < NI; ++ni) {
            const u4 w = *reinterpret_cast<const u4*>(st + (baseB ^ ((ks + 1) << 4)) + ni * blkB);
            fb[(ks + 1) & 1][ni][0] = (int)w.x; fb[(ks + 1) & 1][ni][1] = (int)w.y;
            fb[(ks + 1) & 1][ni][2] = (int)w.z; fb[(ks + 1) & 1][ni][3] = (int)w.w;
          }
        }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
          const u4 w = wa[mi];
          // natural channel order -> the order of the stored weights: evens then odds per 8 channels
          v4i fa;
          fa[0] = (int)__builtin_amdgcn_perm(w.y, w.x, 0x06040200u);
          fa[1] = (int)__builtin_amdgcn_perm(w.y, w.x, 0x07050301u);
          fa[2] = (int)__builtin_amdgcn_perm(w.w, w.z, 0x06040200u);
          fa[3] = (int)__builtin_amdgcn_perm(w.w, w.z, 0x07050301u);
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb[ks & 1][ni], acc[mi][ni], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }

  }
  __syncthreads();
#undef STAMP_REQUEST

  // ------------------------------------------------------------------------------------------
  // Epilogue.  Accumulator element v of lane l in block (mi, ni): row 32 mi + 8 (v / 4) + 4 (l / 32)
  // + v % 4, column 32 ni + l % 32 of the wave tile.
  // ------------------------------------------------------------------------------------------
  const StampGeom& g = a.g;
  float* s_rowfac = reinterpret_cast<float*>(smem);     // [256]
  int* s_rowdst = reinterpret_cast<int*>(smem + 1024);  // [256] destination row or -1
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
    for (int ni = 0; ni < NI; ++ni) {
      const int n = n0 + wn * (32 * NI) + ni * 32 + l32;
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
    // fused: per 32-column strip, dequantize into this wave's LDS tile [128][kEpiStride]; then the wave's
    // 8 groups of 8 lanes each take one unit (a block, or an aligned 16-token part of one) and 4 columns
    // per lane, and run the depth-first inverse, storing the unit's tokens.
    constexpr int R = ES::R, M0 = ES::M0, U = ES::U, npass = ES::npass;
    float* s_tile = reinterpret_cast<float*>(smem + 2048) + wave * (128 * kEpiStride);
    // row factors of this lane's 64 accumulator rows, read before any staging write
    f4 rf[4][4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        rf[mi][q] = *reinterpret_cast<const f4*>(s_rowfac + wm * 128 + mi * 32 + 8 * q + 4 * kg);
    const int c4 = (lane & 7) * 4, ug = lane >> 3;
    auto run_strips = [&](auto vec_tag) __attribute__((always_inline)) {
    constexpr bool VEC = decltype(vec_tag)::value;
    OutQuad<YBF16, VEC> o;
    o.Y = a.out;
    o.tok_stride = (size_t)a.N;
    o.row_stride = (size_t)g.gridW * a.N;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int nw = n0 + wn * (32 * NI) + ni * 32;  // first column of the strip
      const float swn = e_sw[ni];
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int rw = mi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
          s_tile[rw * kEpiStride + l32] = ((float)acc[mi][ni][v] * rf[mi][v >> 2][v & 3]) * swn;
        }
      }
      // the staging tile is private to this wave: its own LDS writes only have to complete (the LDS
      // executes one wave's operations in order), no workgroup barrier is needed
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
      asm volatile("" ::: "memory");
      const int n = nw + c4;
      o.nvalid = a.N - n;
      o.bias = e_bias[ni];
#pragma unroll
      for (int pass = 0; pass < npass; ++pass) {
        const int unit = pass * 8 + ug;
        const int blk = unit / U, h = unit % U;
        const int mrow = m0 + wm * 128 + blk * R;  // physical row of e = 0 of this block
        if (mrow < a.M && n < a.N) {
          const int b = mrow / g.s, pr = mrow - b * g.s;
          const int j = pr / g.R;
          f4 top = e_top[ni][pass];
          const float* tile = s_tile + blk * R * kEpiStride + c4;
          if constexpr (IS2D) {
            const int bi = j / g.G, bj = j - bi * g.G;
            o.base = ((size_t)b * g.s + (size_t)(bi << RB) * g.gridW + (size_t)(bj << RB)) * a.N + n;
            const int hy = h >> 1, hx = h & 1;
            if constexpr (M0 == 1) {
              const f4 cW = *reinterpret_cast<const f4*>(tile + 1 * kEpiStride);
              const f4 cH = *reinterpret_cast<const f4*>(tile + 2 * kEpiStride);
              const f4 cD = *reinterpret_cast<const f4*>(tile + 3 * kEpiStride);
              const f4 t0 = top + cH, t2 = top - cH, t1 = cW + cD, t3 = cW - cD;
              top = hy ? (hx ? (t2 - t3) : (t2 + t3)) : (hx ? (t0 - t1) : (t0 + t1));
            }
            dfs2d<RB, M0, M0, 0, 0, OutQuad<YBF16, VEC>>(tile, hy, hx, top, o);
          } else {
            o.base = ((size_t)b * g.s + (size_t)j * R) * a.N + n;
#pragma unroll
            for (int m = 0; m < M0; ++m) {
              const f4 d = *reinterpret_cast<const f4*>(tile + ((1 << m) + (h >> (M0 - m))) * kEpiStride);
              top = ((h >> (M0 - m - 1)) & 1) ? (top - d) : (top + d);
            }
            dfs1d<RB, M0, M0, 0, OutQuad<YBF16, VEC>>(tile, h, top, o);
          }
        }
      }
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0xC07F);  // this wave's reads of the tile are done before the next strip overwrites it
      asm volatile("" ::: "memory");
    }
    };
    if ((a.N & 3) == 0) run_strips(std::true_type{});
    else run_strips(std::false_type{});
  }
}

template <bool A_INT4, int EPI, int RB, bool IS2D, int NI, bool YBF16>
hipError_t launch_ni(const GemmArgs& a, hipStream_t st) {
  constexpr int BN = 64 * NI;
  constexpr size_t main_lds = ((NI == 4 && A_INT4) ? 3 : 2) * (size_t)(BM * (A_INT4 ? 64 : 128) + BN * 128);
  constexpr size_t epi_lds = 2048 + 4 * 128 * kEpiStride * sizeof(float);
  constexpr size_t lds = main_lds > epi_lds ? main_lds : epi_lds;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<A_INT4, EPI, RB, IS2D, NI, YBF16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int mt = (a.M + BM - 1) / BM, nt = a.Npad / BN;
  hipLaunchKernelGGL((k_gemm<A_INT4, EPI, RB, IS2D, NI, YBF16>), dim3(mt * nt), dim3(256), lds, st, a);
  return hipGetLastError();
}

// Tile width: 128 (two workgroups per CU, default) or 256 (one per CU); STAMP_GEMM_TILE_N overrides (tuning aid).
int gemm_ni() {
  static int ni = 0;
  if (ni == 0) {
    const char* e = getenv("STAMP_GEMM_TILE_N");
    ni = (e != nullptr && atoi(e) == 256) ? 4 : 2;
  }
  return ni;
}

template <bool A_INT4, int EPI, int RB, bool IS2D>
hipError_t launch(const GemmArgs& a, hipStream_t st) {
  // the output type only matters to the fused epilogue
  if constexpr (EPI == 2) {
    if (a.g.y_bf16) {
      if (gemm_ni() == 4) return launch_ni<A_INT4, EPI, RB, IS2D, 4, true>(a, st);
      return launch_ni<A_INT4, EPI, RB, IS2D, 2, true>(a, st);
    }
  }
  if (gemm_ni() == 4) return launch_ni<A_INT4, EPI, RB, IS2D, 4, false>(a, st);
  return launch_ni<A_INT4, EPI, RB, IS2D, 2, false>(a, st);
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
  a.a_last16 = 0;
  return a;
}

}  // namespace

hipError_t stamp_launch_gemm_hi(const stamp_plan* p, const int8_t* q_hi, const float* scales, int mode, void* out,
                                hipStream_t st) {
  GemmArgs a = make_args(p, scales, out);
  a.A = reinterpret_cast<const uint8_t*>(q_hi);
  a.M = p->geom.B * p->geom.k;
  a.a_row_bytes = p->geom.d;
  a.a_last16 = (size_t)a.M * a.a_row_bytes - 16;
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
  a.a_last16 = (size_t)p->Mpad * (p->Kpad / 2) - 16;
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
