// Device code shared by the GEMM kernels of the STaMP linear layer (gfx950): the workgroup -> tile
// map, the per-row dequantization factors, and the epilogue (dequantization Y' = acc * scale_m * sw_n
// of the Background section, then, in the fused mode, the in-block levels of the inverse sequence
// transform by the commutation identity of section "Method", bias and the store of Y).
//
// A workgroup computes 256 rows x 128 or 256 columns with 4 or 8 waves (2 x 2 or 2 x 4); a wave owns
// 128 x 64 outputs = 4 x 2 MFMA blocks of 32 x 32, 16 accumulator registers per block and lane:
// element v of lane l of block (mi, ni) is row 32 mi + 8 (v / 4) + 4 (l / 32) + v % 4, column
// 32 ni + l % 32 of the wave tile.
#ifndef STAMP_GEMM_COMMON_H_
#define STAMP_GEMM_COMMON_H_

#include <type_traits>

#include "stamp_internal.h"

namespace stamp_gemm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));  // first-class 16-byte value (keeps staging arrays in registers)
typedef uint32_t u2 __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef float f8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

constexpr int BM = 256, BK = 128;
constexpr int NI = 2;           // 32-column MFMA blocks per wave along N
constexpr int kEpiStride = 68;  // floats per row of the per-wave epilogue staging tile (64 columns + 4, rows 16-byte aligned)
constexpr int kWaveTileBytes = 64 * kEpiStride * 4;  // one wave's staging tile of the fused epilogue: 64 rows x 64 columns
constexpr int kRowInfoBytes = 3 * 1024;  // per-row factors, destinations and offsets of one 256-row tile
constexpr int kNumXcd = 8;
constexpr int kGroupM = 8;

constexpr float kInvSqrt2 = 0.70710678118654752440f;

__device__ __forceinline__ float haar_norm_dev(int level, int is2d) {
  return is2d ? ldexpf(1.0f, -level) : ldexpf((level & 1) ? kInvSqrt2 : 1.0f, -(level >> 1));
}

struct GemmArgs {
  const uint8_t* A;      // activation codes in the layout of the kernel's operand format
  const uint8_t* Bq;     // weight codes in the layout of the kernel's operand format
  const float* scales;   // [B*s] physical order; asymmetric plans: followed by the [B*s] offsets z
  const float* colsum;   // [Npad] sums of the weight codes per output column (asymmetric plans)
  const float* sw;       // [Npad]
  const float* bias;     // [Npad] or nullptr
  const float* P;        // [B*k][Npad] block sums of the inverse (fused mode)
  void* out;
  int M;                 // rows of A
  int N, Npad, Kpad;
  int a_row_bytes;       // 8-bit rows: valid bytes per A row
  size_t a_last16;       // 8-bit rows: byte offset of the last 16-byte chunk of A (loads are clamped to it)
  int ld_out;            // dequantized mode (EPI 1): floats between consecutive rows of `out`
  int ksplit;            // 8-bit rows, dequantized mode: the depth is split over this many workgroups per tile,
  size_t split_stride;   // each writing its partial rows to out + split * split_stride (floats)
  int a_seq_rows;        // 8-bit rows: rows every sequence has in A, and how many of them (the first ones) this
  int a_seq_used;        // GEMM multiplies: row m of the GEMM is row m + (m / a_seq_used) (a_seq_rows - a_seq_used) of A
  int own_top;           // 4-bit rows, fused mode: coefficient 0 of the blocks from g.khi on is a 4-bit row of A (see
                         // compute_row_info); P then holds g.khi rows per sequence
  StampGeom g;
};

// How a kernel's accumulators map to the integer sum acc = sum_c code[m, c] * qW[c, n]:
//   int8 MFMA, 4-bit rows: both operands are held as code * 16         -> register = 256 acc
//   int8 MFMA, 8-bit rows: the weights are held as code * 16           -> register = 16 acc
//   FP6 MFMA, 4-bit rows:  both operands are held as code / 8 (E2M3)   -> register = acc / 64 (exact in fp32)
// kZeroShift = 2^(b-1): asymmetric codes are stored as code - kZeroShift, so the offset that goes with
// the stored code is z - kZeroShift.
struct AccI8Lo {
  typedef v16i V;
  static constexpr bool kLoRows = true;
  static constexpr float kZeroShift = 8.0f;
  static constexpr float kToAcc = 1.0f / 256.0f;
  static __device__ __forceinline__ int to_i32(int x) { return x >> 8; }
};
struct AccI8Hi {
  typedef v16i V;
  static constexpr bool kLoRows = false;
  static constexpr float kZeroShift = 128.0f;
  static constexpr float kToAcc = 1.0f / 16.0f;
  static __device__ __forceinline__ int to_i32(int x) { return x >> 4; }
};
struct AccF6Lo {
  typedef v16f V;
  static constexpr bool kLoRows = true;
  static constexpr float kZeroShift = 8.0f;
  static constexpr float kToAcc = 64.0f;
  static __device__ __forceinline__ int to_i32(float x) { return (int)(x * 64.0f); }
};

// workgroup -> tile, XCD aware: consecutive ids on one XCD walk 8 M-tiles, then the next N-tile, so
// that the 32 workgroups resident on one XCD cover 8 x 4 neighbouring tiles and share operand panels
// in that XCD's L2.
__device__ __forceinline__ void tile_of_block(int M, int Npad, int bn, int& tm, int& tn) {
  const int mt = (M + BM - 1) / BM, nt = Npad / bn;
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

// Split depth (few tiles, most CUs idle otherwise): `ksplit` consecutive workgroups share a tile; no
// regard to the XCDs.
__device__ __forceinline__ void tile_of_block_split(int M, int ksplit, int& tm, int& tn, int& split) {
  const int mt = (M + BM - 1) / BM;
  const int tile = blockIdx.x / ksplit;
  split = blockIdx.x - tile * ksplit;
  tm = tile % mt;
  tn = tile / mt;
}

// Where one lane stores the tokens of one unit (an aligned part of a block): 8 adjacent output columns
// per token, written as one 16-byte store (bf16) or two (fp32) when d_out allows it.  The 8 lanes of a
// unit's group thus cover the wave tile's 64 columns: whole 128-byte lines of a bf16 Y.
template <bool YBF16, bool VEC>
struct OutOct {
  void* Y;
  size_t base;        // element index of token 0 of the block, first of the 8 columns
  size_t tok_stride;  // d_out
  size_t row_stride;  // 2-D: grid_w * d_out
  f8 scale;           // weight scales of the 8 columns
  f8 offset;          // block sum of the unit's block + bias, per column
  int nvalid;         // how many of the 8 columns exist (d_out tail)
  // v = the token's sum of +-detail coefficients, still without the weight scale: one fma per output
  __device__ __forceinline__ void put(size_t idx, f8 v) const {
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = __builtin_fmaf(v[t], scale[t], offset[t]);
    if constexpr (YBF16) {
      // round-to-nearest-even pairs in hardware (v_cvt_pk_bf16_f32)
      u4 w;
      w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){v[0], v[1]}, bf2));
      w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){v[2], v[3]}, bf2));
      w.z = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){v[4], v[5]}, bf2));
      w.w = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){v[6], v[7]}, bf2));
      uint16_t* y = reinterpret_cast<uint16_t*>(Y) + idx;
      if constexpr (VEC) {
        __builtin_nontemporal_store(w, reinterpret_cast<u4*>(y));  // Y is not read again here: keep it out of the way of the operands in L2
      } else {
#pragma unroll
        for (int t = 0; t < 8; ++t)
          if (t < nvalid) y[t] = (uint16_t)(w[t >> 1] >> (16 * (t & 1)));
      }
    } else {
      float* y = reinterpret_cast<float*>(Y) + idx;
      if constexpr (VEC) {
        __builtin_nontemporal_store((f4){v[0], v[1], v[2], v[3]}, reinterpret_cast<f4*>(y));
        __builtin_nontemporal_store((f4){v[4], v[5], v[6], v[7]}, reinterpret_cast<f4*>(y + 4));
      } else {
#pragma unroll
        for (int t = 0; t < 8; ++t)
          if (t < nvalid) y[t] = v[t];
      }
    }
  }
};

// One coefficient row of the staging tile for this lane's 8 columns.  The tile keeps the wave tile's
// column c = 8 j + t at position 4 j + t (t < 4) or 32 + 4 j + (t - 4): the 8 lanes of a group then
// read two contiguous runs of 128 bytes, and `tile` already points at position 4 j.
__device__ __forceinline__ f8 tile_row(const float* tile, int e) {
  const f4 lo = *reinterpret_cast<const f4*>(tile + e * kEpiStride);
  const f4 hi = *reinterpret_cast<const f4*>(tile + e * kEpiStride + 32);
  return (f8){lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
}

// Depth-first inverse of one unit for 8 columns.  The unit is the subtree rooted at node (M0, h) of a
// block's Haar tree; node (M, I) of that subtree holds in `a` the signed sum of the detail coefficients on
// the path from the block's root (the block sum and the weight scale are applied by Out::put: the inverse
// is linear along the tokens, so the per-column scale can wait until the end); row e of the tile is
// the block's coefficient at in-block STaMP position e = 2^M + (h << (M - M0)) + I.  Only O(r) values
// are live at any time and every coefficient is read once.
template <int RLOG, int M0, int M, int I, typename Out>
__device__ __forceinline__ void dfs1d(const float* tile, int h, f8 a, const Out& o) {
  if constexpr (M == RLOG) {
    o.put(o.base + (size_t)((h << (RLOG - M0)) + I) * o.tok_stride, a);
  } else {
    const f8 d = tile_row(tile, (1 << M) + (h << (M - M0)) + I);
    dfs1d<RLOG, M0, M + 1, 2 * I, Out>(tile, h, a + d, o);
    dfs1d<RLOG, M0, M + 1, 2 * I + 1, Out>(tile, h, a - d, o);
  }
}

// 2-D: the unit is the quadtree node (M0, hy, hx) of a g x g block; bands W, H, D of level-node side
// gl = 2^M sit at e = gl^2 (1 + band) + iy * gl + ix.
template <int RLOG, int M0, int M, int IY, int IX, typename Out>
__device__ __forceinline__ void dfs2d(const float* tile, int hy, int hx, f8 a, const Out& o) {
  if constexpr (M == RLOG) {
    o.put(o.base + (size_t)((hy << (RLOG - M0)) + IY) * o.row_stride + (size_t)((hx << (RLOG - M0)) + IX) * o.tok_stride, a);
  } else {
    constexpr int gl = 1 << M;
    const int e0 = ((hy << (M - M0)) + IY) * gl + ((hx << (M - M0)) + IX);
    const f8 cW = tile_row(tile, gl * gl + e0);
    const f8 cH = tile_row(tile, 2 * gl * gl + e0);
    const f8 cD = tile_row(tile, 3 * gl * gl + e0);
    const f8 t0 = a + cH, t2 = a - cH, t1 = cW + cD, t3 = cW - cD;
    dfs2d<RLOG, M0, M + 1, 2 * IY, 2 * IX, Out>(tile, hy, hx, t0 + t1, o);
    dfs2d<RLOG, M0, M + 1, 2 * IY, 2 * IX + 1, Out>(tile, hy, hx, t0 - t1, o);
    dfs2d<RLOG, M0, M + 1, 2 * IY + 1, 2 * IX, Out>(tile, hy, hx, t2 + t3, o);
    dfs2d<RLOG, M0, M + 1, 2 * IY + 1, 2 * IX + 1, Out>(tile, hy, hx, t2 - t3, o);
  }
}

// Shape of the fused epilogue for block size RB.  The wave tile's 128 rows are handled as two halves of
// 64 rows (64 / R whole blocks of R tokens).  A unit is the subtree at depth M0 of a block's tree: 8
// tokens in 1-D, 2 x 2 tokens in 2-D; U units per block; npass passes of 8 units (one per group of 8
// lanes) cover a half.
template <int RB, bool IS2D>
struct EpiShape {
  static constexpr int R = IS2D ? (1 << (2 * RB)) : (1 << RB);
  static constexpr int nblk = 64 / R;
  static constexpr int M0 = IS2D ? (RB - 1) : (RB - 3);
  static constexpr int U = IS2D ? (1 << (2 * M0)) : (1 << M0);
  static constexpr int npass = (nblk * U) / 8;
  static_assert(R <= 64 && M0 >= 0 && nblk * U >= 8, "block size outside the fused epilogue's range");
};

// Global operands of the fused epilogue (weight scales, bias, block sums P of this lane's units),
// requested ahead of the main loop so that their latency is not on the epilogue's path.
template <int EPI, int RB, bool IS2D>
struct EpiOperands {
  using ES = EpiShape<(EPI == 2 ? RB : 3), IS2D>;
  float cs[NI];  // column sums of the weight codes (asymmetric plans)
  f8 sw8;        // weight scales of this lane's 8 output columns
  f8 bias;
  f8 top[2][ES::npass];
  __device__ __forceinline__ void request(const GemmArgs& a, int m0, int n0, int lane, int wm, int wn) {
    if constexpr (EPI == 2 || EPI == 3) {
      const int c8 = (lane & 7) * 8, ug = lane >> 3, l32 = lane & 31;
      const int nw = n0 + wn * 64;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        cs[ni] = a.g.asym ? a.colsum[nw + ni * 32 + l32] : 0.0f;
      }
      const f4 s0 = *reinterpret_cast<const f4*>(a.sw + nw + c8), s1 = *reinterpret_cast<const f4*>(a.sw + nw + c8 + 4);
      sw8 = (f8){s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
      const f4 zero = (f4){0.0f, 0.0f, 0.0f, 0.0f};
      const f4 b0 = (a.bias != nullptr) ? *reinterpret_cast<const f4*>(a.bias + nw + c8) : zero;
      const f4 b1 = (a.bias != nullptr) ? *reinterpret_cast<const f4*>(a.bias + nw + c8 + 4) : zero;
      bias = (f8){b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
      if constexpr (EPI == 2) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
        for (int pass = 0; pass < ES::npass; ++pass) {
          const int blk = (pass * 8 + ug) / ES::U;
          const int mrow = min(m0 + wm * 128 + hf * 64 + blk * ES::R, a.M - 1);
          const float* src = a.P + (size_t)(mrow / a.g.R) * a.Npad + nw + c8;
          const f4 p0 = *reinterpret_cast<const f4*>(src), p1 = *reinterpret_cast<const f4*>(src + 4);
          top[hf][pass] = (f8){p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
        }
      }
      }
    }
  }
};

// Per-row dequantization factor (activation scale * Haar norm of the row's level * the operand
// format's constant), destination row, and (asymmetric plans) the offset of the stored code in
// accumulator units, of tile row `tid`, written to LDS at row_info (kRowInfoBytes) before the main
// loop; the main loop's barriers publish them.
template <typename Acc, int EPI>
__device__ __forceinline__ void compute_row_info(const GemmArgs& a, int m0, int tid, float& fac, int& dst, float& rz) {
  const StampGeom& g = a.g;
  const int m = m0 + tid;
  fac = 0.0f;
  rz = 0.0f;
  dst = -1;
  const size_t zeros_off = (size_t)g.B * g.s;
  if (m < a.M && g.ident) {
    // no sequence transform: row = token, level 0 (norm 1); tokens 0..k-1 of a sequence are the 8-bit rows
    size_t row;
    bool mine;
    if constexpr (Acc::kLoRows) {
      row = (size_t)m;
      mine = (m % g.s) >= g.k;
    } else {
      const int b = m / g.k;
      row = (size_t)b * g.s + (size_t)(m - b * g.k);
      mine = true;
    }
    if (mine) {
      if constexpr (EPI != 0) {
        fac = a.scales[row] * Acc::kToAcc;
        if (g.asym) rz = (a.scales[zeros_off + row] - Acc::kZeroShift) * (1.0f / Acc::kToAcc);
      }
      dst = (Acc::kLoRows || EPI == 0) ? (int)row : m;
    }
  } else if (m < a.M) {
    if constexpr (Acc::kLoRows) {
      const int b = m / g.s, pr = m - b * g.s;
      const int j = pr / g.R, e = pr - j * g.R;
      // own_top (plans without top levels, 1-D): the block sums beyond the first khi are 4-bit rows like any other and
      // sit at coefficient 0 of their block, level = that of the whole block; dst 1 marks them for the epilogue
      const bool own = e == 0 && a.own_top != 0 && j >= g.khi;
      if (e != 0 || own) {
        const int level = own ? g.r : (g.is2d ? stamp_level_of_e_2d(e, g.r) : stamp_level_of_e_1d(e, g.r));
        if constexpr (EPI != 0) {
          fac = a.scales[m] * haar_norm_dev(level, g.is2d) * Acc::kToAcc;
          if (g.asym) rz = (a.scales[zeros_off + m] - Acc::kZeroShift) * (1.0f / Acc::kToAcc);
        }
        if (EPI == 0) {
          const int p = g.is2d ? stamp_slot_of_block_e_2d(j / g.G, j % g.G, e, g.G) : stamp_slot_of_block_e_1d(j, e, g.k);
          dst = b * g.s + p;
        } else {
          dst = own ? 1 : m;
        }
      }
    } else {
      const int b = m / g.k, p = m - b * g.k;
      const int level = stamp_level_of_top_slot(p, g.k, g.G, g.is2d, g.r, g.L);
      if constexpr (EPI != 0) {
        const size_t row = (size_t)b * g.s + (size_t)p * g.R;
        fac = a.scales[row] * haar_norm_dev(level, g.is2d) * Acc::kToAcc;
        // top rows beyond the first khi carry 4-bit codes: their stored form is code - 8
        if (g.asym) rz = (a.scales[zeros_off + row] - (p < g.khi ? Acc::kZeroShift : 8.0f)) * (1.0f / Acc::kToAcc);
      }
      dst = (EPI == 0) ? (b * g.s + p) : m;
    }
  }
}

__device__ __forceinline__ void write_row_info(uint8_t* row_info, int tid, float fac, int dst, float rz) {
  reinterpret_cast<float*>(row_info)[tid] = fac;        // [256]
  reinterpret_cast<int*>(row_info + 1024)[tid] = dst;   // [256] destination row or -1
  reinterpret_cast<float*>(row_info + 2048)[tid] = rz;  // [256] (z - 2^(b-1)) / kToAcc
}

template <typename Acc, int EPI>
__device__ __forceinline__ void store_row_info(const GemmArgs& a, int m0, int tid, uint8_t* row_info) {
  float fac, rz;
  int dst;
  compute_row_info<Acc, EPI>(a, m0, tid, fac, dst, rz);
  write_row_info(row_info, tid, fac, dst, rz);
}

// Epilogue of one workgroup tile; to be called after a workgroup barrier that follows the last read
// of the operand stages (the fused mode reuses smem[0, waves * kWaveTileBytes) as staging).  Wave
// `wave` of the workgroup owns rows [128 wm, +128) and columns [64 wn, +64) of the tile.
// EPI: 0 = integer sums to STaMP-ordered rows [B*s][N] int32; 1 = dequantized fp32 rows (4-bit rows:
// physical rows of [B*s][N]; 8-bit rows: [B*k][N]); 2 = fused in-block inverse + bias -> Y (4-bit
// rows only); RB = log2 of the block length for EPI 2 (1-D: tokens, 2-D: side); 3 = plans without a
// sequence transform: dequantized rows + bias -> Y through the same staging (4-bit rows only).
// PAIRCOLS: the weights are stored so that MFMA column l32 of block ni is column 2 l32 + ni of the wave's 64
// (the FP6 engine's layout) instead of 32 ni + l32.
template <typename Acc, int EPI, int RB, bool IS2D, bool YBF16, bool PAIRCOLS = false>
__device__ __forceinline__ void epilogue(const GemmArgs& a, typename Acc::V (&acc)[4][NI], uint8_t* smem,
                                         const uint8_t* row_info, const EpiOperands<EPI, RB, IS2D>& eo, int m0,
                                         int n0, int lane, int wave, int wm, int wn) {
  const StampGeom& g = a.g;
  const int l32 = lane & 31, kg = lane >> 5;
  const float* s_rowfac = reinterpret_cast<const float*>(row_info);
  const int* s_rowdst = reinterpret_cast<const int*>(row_info + 1024);
  const float* s_rowz = reinterpret_cast<const float*>(row_info + 2048);

  if constexpr (EPI == 1 && PAIRCOLS && NI == 2) {
    // a lane holds two neighbouring columns (2 l32, 2 l32 + 1) of every row: one 8-byte store per row when the
    // output rows keep them 8-byte aligned (even row pitch), else two 4-byte stores
    const int n = n0 + wn * 64 + 2 * l32;
    const bool in0 = n < a.N, in1 = n + 1 < a.N;
    const float sw0 = in0 ? a.sw[n] : 0.0f, sw1 = in1 ? a.sw[n + 1] : 0.0f;
    const float cs0 = (g.asym && in0) ? a.colsum[n] : 0.0f, cs1 = (g.asym && in1) ? a.colsum[n + 1] : 0.0f;
    const bool vec = in1 && (a.ld_out & 1) == 0;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int rl = wm * 128 + mi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
        const int dst = s_rowdst[rl];
        if (dst >= 0 && in0) {
          const float rz = s_rowz[rl], rf = s_rowfac[rl];
          // asymmetric: the integer sum over (stored code - offset), exact in one fma (rz = 0 otherwise)
          const float y0 = (__builtin_fmaf(-rz, cs0, (float)acc[mi][0][v]) * rf) * sw0;
          const float y1 = (__builtin_fmaf(-rz, cs1, (float)acc[mi][1][v]) * rf) * sw1;
          float* o = reinterpret_cast<float*>(a.out) + (size_t)dst * a.ld_out + n;
          if (vec) {
            *reinterpret_cast<f2*>(o) = f2{y0, y1};
          } else {
            o[0] = y0;
            if (in1) o[1] = y1;
          }
        }
      }
    }
  } else if constexpr (EPI == 0 || EPI == 1) {
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int n = n0 + wn * (32 * NI) + (PAIRCOLS ? 2 * l32 + ni : ni * 32 + l32);
      const float swn = a.sw[n];
      const float csn = (EPI == 1 && g.asym) ? a.colsum[n] : 0.0f;
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int rl = wm * 128 + mi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
          const int dst = s_rowdst[rl];
          if (dst >= 0 && n < a.N) {
            if constexpr (EPI == 0) {
              reinterpret_cast<int32_t*>(a.out)[(size_t)dst * a.N + n] = Acc::to_i32(acc[mi][ni][v]);
            } else {
              // asymmetric: the integer sum over (stored code - offset), exact in one fma
              const float af = g.asym ? __builtin_fmaf(-s_rowz[rl], csn, (float)acc[mi][ni][v]) : (float)acc[mi][ni][v];
              reinterpret_cast<float*>(a.out)[(size_t)dst * a.ld_out + n] = (af * s_rowfac[rl]) * swn;
            }
          }
        }
      }
    }
  } else {
    // fused: per half of 64 rows, scale by the row factors into this wave's LDS tile [64][kEpiStride]; then the wave's
    // 8 groups of 8 lanes each take one unit and 8 columns per lane, and run the depth-first inverse,
    // storing the unit's tokens.
    using ES = EpiShape<(EPI == 2 ? RB : 3), IS2D>;
    [[maybe_unused]] constexpr int R = ES::R, M0 = ES::M0, U = ES::U, npass = ES::npass;
    float* s_tile = reinterpret_cast<float*>(smem) + wave * (64 * kEpiStride);
    const int c8 = (lane & 7) * 8, ug = lane >> 3;
    // staging position of this lane's accumulator column 32 ni + l32 = 8 j + t (see tile_row)
    const int pos0 = ((l32 & 4) ? 32 : 0) + 4 * (l32 >> 3) + (l32 & 3);
    const int nw = n0 + wn * 64;  // first column of the wave tile
    const int n = nw + c8;        // first of this lane's 8 output columns
    auto run_halves = [&](auto vec_tag) __attribute__((always_inline)) {
      constexpr bool VEC = decltype(vec_tag)::value;
      OutOct<YBF16, VEC> o;
      o.Y = a.out;
      o.tok_stride = (size_t)a.N;
      o.row_stride = (size_t)g.gridW * a.N;
      o.nvalid = a.N - n;
      o.scale = eo.sw8;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        if (!g.asym) {
          // row factors of this lane's 32 accumulator rows of the half
          f4 rf[2][4];
#pragma unroll
          for (int mh = 0; mh < 2; ++mh)
#pragma unroll
            for (int q = 0; q < 4; ++q)
              rf[mh][q] = *reinterpret_cast<const f4*>(s_rowfac + wm * 128 + (2 * hf + mh) * 32 + 8 * q + 4 * kg);
#pragma unroll
          for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
            for (int mh = 0; mh < 2; ++mh) {
              const int mi = 2 * hf + mh;
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int rw = mh * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                s_tile[rw * kEpiStride + pos0 + 16 * ni] = (float)acc[mi][ni][v] * rf[mh][v >> 2][v & 3];
              }
            }
          }
        } else {
          // asymmetric codes: the integer sum over (stored code - offset) = acc - rowz * colsum, exact in
          // one fma; four rows at a time, their factors and offsets read one group ahead of the staging
          // writes (LDS operations execute in order, and a read placed after a write would wait for it)
          const int rbase = wm * 128 + 2 * hf * 32 + 4 * kg;
          f4 rf_n = *reinterpret_cast<const f4*>(s_rowfac + rbase);
          f4 rz_n = *reinterpret_cast<const f4*>(s_rowz + rbase);
#pragma unroll
          for (int gq = 0; gq < 8; ++gq) {
            const int mh = gq >> 2, q = gq & 3, mi = 2 * hf + mh;
            const f4 rf4 = rf_n, rz4 = rz_n;
            if (gq + 1 < 8) {
              const int r1 = rbase + ((gq + 1) >> 2) * 32 + 8 * ((gq + 1) & 3);
              rf_n = *reinterpret_cast<const f4*>(s_rowfac + r1);
              rz_n = *reinterpret_cast<const f4*>(s_rowz + r1);
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
              for (int vv = 0; vv < 4; ++vv) {
                const int rw = mh * 32 + 8 * q + 4 * kg + vv;
                const float af = __builtin_fmaf(-rz4[vv], eo.cs[ni], (float)acc[mi][ni][4 * q + vv]);
                s_tile[rw * kEpiStride + pos0 + 16 * ni] = af * rf4[vv];
              }
            }
          }
        }
        // the staging tile is private to this wave: its own LDS writes only have to complete (the LDS
        // executes one wave's operations in order), no workgroup barrier is needed
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
        asm volatile("" ::: "memory");
        if constexpr (EPI == 3) {
          // identity plans: the staged rows are the output rows; 8 lanes write one row's 64 columns
          o.offset = eo.bias;
#pragma unroll
          for (int pass = 0; pass < 8; ++pass) {
            const int rw = pass * 8 + ug;
            const int dst = s_rowdst[wm * 128 + hf * 64 + rw];
            if (dst >= 0 && n < a.N) o.put((size_t)dst * a.N + n, tile_row(s_tile + 4 * (lane & 7), rw));
          }
        } else {
#pragma unroll
        for (int pass = 0; pass < npass; ++pass) {
          const int unit = pass * 8 + ug;
          const int blk = unit / U, h = unit % U;
          const int mrow = m0 + wm * 128 + hf * 64 + blk * R;  // physical row of e = 0 of this block
          if (mrow < a.M && n < a.N) {
            const int b = mrow / g.s, pr = mrow - b * g.s;
            const int j = pr / g.R;
            o.offset = eo.top[hf][pass] + eo.bias;
            f8 top = (f8){0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};  // signed detail sum on the path to the unit
            const float* tile = s_tile + blk * R * kEpiStride + 4 * (lane & 7);
            if constexpr (IS2D) {
              const int bi = j / g.G, bj = j - bi * g.G;
              o.base = ((size_t)b * g.s + (size_t)(bi << RB) * g.gridW + (size_t)(bj << RB)) * a.N + n;
              const int hy = h >> M0, hx = h & ((1 << M0) - 1);
              // walk from the block's root down to the unit's node: at level m the ancestor is node
              // (hy >> (M0 - m), hx >> (M0 - m)); keep the quadrant that holds the unit
#pragma unroll
              for (int m = 0; m < M0; ++m) {
                const int gl = 1 << m;
                const int e0 = (hy >> (M0 - m)) * gl + (hx >> (M0 - m));
                const f8 cW = tile_row(tile, gl * gl + e0);
                const f8 cH = tile_row(tile, 2 * gl * gl + e0);
                const f8 cD = tile_row(tile, 3 * gl * gl + e0);
                const f8 t0 = top + cH, t2 = top - cH, t1 = cW + cD, t3 = cW - cD;
                const int qy = (hy >> (M0 - m - 1)) & 1, qx = (hx >> (M0 - m - 1)) & 1;
                top = qy ? (qx ? (t2 - t3) : (t2 + t3)) : (qx ? (t0 - t1) : (t0 + t1));
              }
              dfs2d<RB, M0, M0, 0, 0, OutOct<YBF16, VEC>>(tile, hy, hx, top, o);
            } else {
              o.base = ((size_t)b * g.s + (size_t)j * R) * a.N + n;
#pragma unroll
              for (int m = 0; m < M0; ++m) {
                const f8 d = tile_row(tile, (1 << m) + (h >> (M0 - m)));
                top = ((h >> (M0 - m - 1)) & 1) ? (top - d) : (top + d);
              }
              dfs1d<RB, M0, M0, 0, OutOct<YBF16, VEC>>(tile, h, top, o);
            }
          }
        }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);  // this wave's reads of the tile are done before the next half overwrites it
        asm volatile("" ::: "memory");
      }
    };
    if ((a.N & 7) == 0) run_halves(std::true_type{});
    else run_halves(std::false_type{});
  }
}

}  // namespace stamp_gemm

// arguments common to every GEMM launch of a plan (host)
stamp_gemm::GemmArgs stamp_gemm_args(const stamp_plan* p, const float* scales, void* out);

#endif  // STAMP_GEMM_COMMON_H_
