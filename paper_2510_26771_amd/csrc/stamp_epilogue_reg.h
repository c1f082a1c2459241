// Register-resident epilogue of the FP6 GEMM over the 4-bit rows: dequantization Y' = acc * scale_m * sw_n
// (Background, de-quantization), the in-block levels of the inverse sequence transform (step "Y <- L^-1 Y" of
// Algorithm "STaMP Linear", valid per output column by the commutation identity of section "Method"), bias and
// the store of Y, all without leaving the registers.
//
// A wave owns 128 rows x 64 columns as 4 x 2 MFMA blocks of 32 x 32; lane (kg = lane / 32, l32 = lane % 32)
// holds of block (mi, ni) the column l32 and the rows 32 mi + 8 q + 4 kg + j (register v = 4 q + j).  One
// v_permlane32_swap per register pair exchanges the rows 8 q + 4 + j of lane group 0 with the rows 8 q + j of
// lane group 1, after which each lane group holds WHOLE blocks of R = 8 .. 64 rows (Haar sub-trees) of its
// column: lane group kg owns the blocks 2 t + kg of the wave tile, t < 64 / R.  The inverse butterflies are then
// plain register arithmetic.  The weights are stored so that MFMA column l32 of block ni is output column
// 2 l32 + ni of the wave's 64: a lane's two results are neighbours, one 4-byte (bf16) or 8-byte (fp32) store per
// token, and the 32 lanes of a group write one contiguous 128- or 256-byte run.
#ifndef STAMP_EPILOGUE_REG_H_
#define STAMP_EPILOGUE_REG_H_

#include "stamp_gemm_common.h"

namespace stamp_gemm {

// Register (mi, v) that holds, after the swaps, coefficient e (in-block position) of the lane's t-th block.
template <int RL>
struct RegMap {
  static constexpr int R = 1 << RL;
  static constexpr int nb = 64 / R;  // blocks per lane
  static_assert(RL >= 3 && RL <= 6, "blocks of 8 .. 64 rows");
  static constexpr int mi(int t, int e) {
    return RL == 6 ? ((e >> 5) + 2 * ((e >> 2) & 1)) : RL == 5 ? (2 * t + ((e >> 2) & 1)) : RL == 4 ? t : (t >> 1);
  }
  static constexpr int v(int t, int e) {
    return RL >= 5   ? (4 * ((e >> 3) & 3) + (e & 3))
           : RL == 4 ? (4 * (((e >> 3) & 1) + 2 * ((e >> 2) & 1)) + (e & 3))
                     : (4 * (2 * (t & 1) + ((e >> 2) & 1)) + (e & 3));
  }
};

// Four independent swaps in one statement: the wait states are needed once before the first and once after the last
// (nothing else can come between them).
__device__ __forceinline__ void swap32x4(float& x0, float& y0, float& x1, float& y1, float& x2, float& y2, float& x3, float& y3) {
  asm volatile(
      "s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_permlane32_swap_b32 %2, %3\n\tv_permlane32_swap_b32 %4, %5\n\t"
      "v_permlane32_swap_b32 %6, %7\n\ts_nop 1"
      : "+v"(x0), "+v"(y0), "+v"(x1), "+v"(y1), "+v"(x2), "+v"(y2), "+v"(x3), "+v"(y3));
}

__device__ __forceinline__ void swap32(float& x, float& y) {
  // lanes 32..63 of x <-> lanes 0..31 of y.  Written as an asm statement: the builtin form is treated as
  // rematerialisable, i.e. executed once per result with both inputs kept alive, which doubles the live
  // registers of the epilogue.  The wait states around it cover the instruction's read-after-VALU-write and
  // VALU-read-after-it hazards, which the assembler does not see inside an asm statement.
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(x), "+v"(y));
}

// Two neighbouring output columns of one token.
template <bool YBF16, bool VEC>
__device__ __forceinline__ void put_pair(void* Y, size_t idx, float v0, float v1, int nvalid) {
  if constexpr (YBF16) {
    const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){v0, v1}, bf2));  // v_cvt_pk_bf16_f32, RNE
    uint16_t* y = reinterpret_cast<uint16_t*>(Y) + idx;
    if constexpr (VEC) {
      __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(y));  // Y is not read again here
    } else {
      if (nvalid > 0) y[0] = (uint16_t)w;
      if (nvalid > 1) y[1] = (uint16_t)(w >> 16);
    }
  } else {
    float* y = reinterpret_cast<float*>(Y) + idx;
    if constexpr (VEC) {
      __builtin_nontemporal_store((f2){v0, v1}, reinterpret_cast<f2*>(y));
    } else {
      if (nvalid > 0) y[0] = v0;
      if (nvalid > 1) y[1] = v1;
    }
  }
}

// The same pair at a 32-bit byte offset from a wave-uniform base (the tile's first output row): the address is the
// scalar base plus one 32-bit vector offset, no 64-bit vector arithmetic per store.
template <bool YBF16>
__device__ __forceinline__ void put_pair_at(char* base, uint32_t byte_off, float v0, float v1) {
  if constexpr (YBF16) {
    const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector((f2){v0, v1}, bf2));  // v_cvt_pk_bf16_f32, RNE
    __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(base + byte_off));  // Y is not read again here
  } else {
    __builtin_nontemporal_store((f2){v0, v1}, reinterpret_cast<f2*>(base + byte_off));
  }
}

// Operands of the epilogue that come from global memory: requested during the last K step of a tile.
template <int EPI, int RL>
struct RegEpiOperands {
  static constexpr int nb = (EPI == 2) ? 64 / (1 << RL) : 1;
  f2 sw, bias, cs;
  f2 P[nb];
  __device__ __forceinline__ void request(const GemmArgs& a, int m0, int nw, int wm, int lane) {
    const int l32 = lane & 31, kg = lane >> 5;
    const int n = nw + 2 * l32;  // Npad is a multiple of 256: always inside the padded arrays
    sw = *reinterpret_cast<const f2*>(a.sw + n);
    bias = (a.bias != nullptr) ? *reinterpret_cast<const f2*>(a.bias + n) : (f2){0.0f, 0.0f};
    cs = a.g.asym ? *reinterpret_cast<const f2*>(a.colsum + n) : (f2){0.0f, 0.0f};
    if constexpr (EPI == 2) {
      constexpr int R = 1 << RL;
#pragma unroll
      for (int t = 0; t < nb; ++t) {
        const int mrow = min(m0 + wm * 128 + (2 * t + kg) * R, a.M - 1);
        // P holds the first pk block sums of every sequence (all k of them unless the blocks beyond khi carry their
        // own, see blocks_reg); blocks beyond read a row that is there and is not used
        const int blk = mrow / R, pk = a.own_top ? a.g.khi : a.g.k;
        const int b = blk / a.g.k, j = blk - b * a.g.k;
        P[t] = *reinterpret_cast<const f2*>(a.P + (size_t)(b * pk + min(j, pk - 1)) * a.Npad + n);
      }
    }
  }
};

// Where a lane stores the tokens of one block, two neighbouring columns per token.
// B32 (1-D plans): Y is the tile's first output row and base / tok_stride are 32-bit BYTE offsets from it (256 rows
// of d_out elements: below 2^32 for d_out up to 2^21, which plan creation checks); otherwise element indices into Y.
template <bool YBF16, bool VEC, bool B32>
struct RegOut {
  typedef typename std::conditional<B32, uint32_t, size_t>::type IDX;
  void* Y;
  IDX base;           // token 0 of the block, first of the two columns
  IDX tok_stride;     // d_out
  IDX row_stride;     // 2-D: grid_w * d_out
  float sw0, sw1;     // weight scales of the two columns
  float off0, off1;   // block sum + bias
  int nvalid;
  // v = the token's signed sum of detail coefficients, still without the weight scale
  __device__ __forceinline__ void put(IDX idx, float v0, float v1) const {
    if constexpr (B32) put_pair_at<YBF16>(reinterpret_cast<char*>(Y), idx, __builtin_fmaf(v0, sw0, off0), __builtin_fmaf(v1, sw1, off1));
    else put_pair<YBF16, VEC>(Y, idx, __builtin_fmaf(v0, sw0, off0), __builtin_fmaf(v1, sw1, off1), nvalid);
  }
};

// Depth-first inverse of the lane's T-th block from the registers: node I of level M holds the signed sum of
// the detail coefficients on the path from the block's root; coefficient e = 2^M + I splits it into the
// nodes 2 I (sum) and 2 I + 1 (difference) of the next level.  Only O(log R) values are live.
template <int RL, int T, int M, int I, typename Out>
__device__ __forceinline__ void dfs1d_reg(const float (&acc)[4][NI][16], float a0, float a1, const Out& o) {
  using RM = RegMap<RL>;
  if constexpr (M == RL) {
    o.put(o.base + (typename Out::IDX)I * o.tok_stride, a0, a1);
    if constexpr ((I & 7) == 7) __builtin_amdgcn_sched_barrier(0);  // bounds how far stores and their addresses run ahead
  } else {
    constexpr int e = (1 << M) + I;
    const float d0 = acc[RM::mi(T, e)][0][RM::v(T, e)], d1 = acc[RM::mi(T, e)][1][RM::v(T, e)];
    dfs1d_reg<RL, T, M + 1, 2 * I, Out>(acc, a0 + d0, a1 + d1, o);
    dfs1d_reg<RL, T, M + 1, 2 * I + 1, Out>(acc, a0 - d0, a1 - d1, o);
  }
}

// 2-D: quadtree node (IY, IX) of level M (side 2^M); bands W, H, D at e = 4^M (1 + band) + IY 2^M + IX.
template <int RB, int T, int M, int IY, int IX, typename Out>
__device__ __forceinline__ void dfs2d_reg(const float (&acc)[4][NI][16], float a0, float a1, const Out& o) {
  using RM = RegMap<2 * RB>;
  if constexpr (M == RB) {
    o.put(o.base + (typename Out::IDX)IY * o.row_stride + (typename Out::IDX)IX * o.tok_stride, a0, a1);
    if constexpr ((IY & 1) && (IX & 1)) __builtin_amdgcn_sched_barrier(0);
  } else {
    constexpr int gl = 1 << M, e0 = IY * gl + IX;
    constexpr int eW = gl * gl + e0, eH = 2 * gl * gl + e0, eD = 3 * gl * gl + e0;
    float t0[2], t1[2], t2[2], t3[2];
    const float av[2] = {a0, a1};
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const float cW = acc[RM::mi(T, eW)][ni][RM::v(T, eW)], cH = acc[RM::mi(T, eH)][ni][RM::v(T, eH)],
                  cD = acc[RM::mi(T, eD)][ni][RM::v(T, eD)];
      t0[ni] = av[ni] + cH;
      t2[ni] = av[ni] - cH;
      t1[ni] = cW + cD;
      t3[ni] = cW - cD;
    }
    dfs2d_reg<RB, T, M + 1, 2 * IY, 2 * IX, Out>(acc, t0[0] + t1[0], t0[1] + t1[1], o);
    dfs2d_reg<RB, T, M + 1, 2 * IY, 2 * IX + 1, Out>(acc, t0[0] - t1[0], t0[1] - t1[1], o);
    dfs2d_reg<RB, T, M + 1, 2 * IY + 1, 2 * IX, Out>(acc, t2[0] + t3[0], t2[1] + t3[1], o);
    dfs2d_reg<RB, T, M + 1, 2 * IY + 1, 2 * IX + 1, Out>(acc, t2[0] - t3[0], t2[1] - t3[1], o);
  }
}

// the lane's blocks T .. NB-1, one after the other; mrow0 = physical row of e = 0 of the lane's block 0, rowfac0 /
// rowz0 = that row's entry of the per-row tables.  Per block: c = (acc - rowz * colsum) * rowfac in place, the
// dequantized coefficient without the weight scale (symmetric plans have rowz = 0 and colsum operand 0: the fma
// then leaves the sum as it is), then the depth-first inverse.
template <int RB, bool IS2D, int T, int NB, bool YBF16, bool VEC, bool SYM, int NP>
__device__ __forceinline__ void blocks_reg(const GemmArgs& a, float (&acc)[4][NI][16], const f2 (&P)[NP], f2 bias, f2 cs,
                                           RegOut<YBF16, VEC, !IS2D>& o, const float* rowfac0, const float* rowz0, int mrow0,
                                           int n, int m0) {
  if constexpr (T < NB) {
    constexpr int RL = IS2D ? 2 * RB : RB;
    constexpr int R = 1 << RL;
    using RM = RegMap<RL>;
    const StampGeom& g = a.g;
    const int mrow = mrow0 + 2 * T * R;
    if (mrow < a.M && o.nvalid > 0) {
#pragma unroll
      for (int e4 = 0; e4 < R; e4 += 4) {
        const f4 rf = *reinterpret_cast<const f4*>(rowfac0 + 2 * T * R + e4);
        f4 rz = {0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (!SYM) rz = *reinterpret_cast<const f4*>(rowz0 + 2 * T * R + e4);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int e = e4 + u;
#pragma unroll
          for (int ni = 0; ni < NI; ++ni) {
            // SYM (a kernel for symmetric plans): no offset term, the fma would add a zero
            if constexpr (SYM) acc[RM::mi(T, e)][ni][RM::v(T, e)] *= rf[u];
            else acc[RM::mi(T, e)][ni][RM::v(T, e)] = __builtin_fmaf(-rz[u], cs[ni], acc[RM::mi(T, e)][ni][RM::v(T, e)]) * rf[u];
          }
        }
        // keeps the factor reads of later groups from being hoisted (they would all be live at once)
        if ((e4 & 12) == 12) __builtin_amdgcn_sched_barrier(0);
      }
      // The block sum comes from the 8-bit rows' GEMM (P), or - plans without top levels, blocks from khi on, marked
      // in the row table - it is the block's own coefficient 0, dequantized above like every other row.
      const bool own = reinterpret_cast<const int*>(rowfac0)[256 + 2 * T * R] == 1;
      o.off0 = (own ? acc[RM::mi(T, 0)][0][RM::v(T, 0)] * o.sw0 : P[T][0]) + bias[0];
      o.off1 = (own ? acc[RM::mi(T, 0)][1][RM::v(T, 0)] * o.sw1 : P[T][1]) + bias[1];
      if constexpr (!IS2D) {
        // token 0 of block j of sequence b is physical row b s + j R; bytes from the tile's first row
        o.base = ((uint32_t)(mrow - m0) * (uint32_t)a.N + (uint32_t)n) * (uint32_t)(YBF16 ? 2 : 4);
        dfs1d_reg<RL, T, 0, 0, RegOut<YBF16, VEC, true>>(acc, 0.0f, 0.0f, o);
      } else {
        const int b = mrow / g.s, pr = mrow - b * g.s;
        const int j = pr / g.R;
        const int bi = j / g.G, bj = j - bi * g.G;
        o.base = ((size_t)b * g.s + (size_t)(bi << RB) * g.gridW + (size_t)(bj << RB)) * a.N + n;
        dfs2d_reg<RB, T, 0, 0, 0, RegOut<YBF16, VEC, false>>(acc, 0.0f, 0.0f, o);
      }
    }
    blocks_reg<RB, IS2D, T + 1, NB, YBF16, VEC, SYM, NP>(a, acc, P, bias, cs, o, rowfac0, rowz0, mrow0, n, m0);
  }
}

// EPI 2: fused in-block inverse (RB = log2 of the block length in 1-D, of the block side in 2-D);
// EPI 3: plans without a sequence transform (rows are tokens).
// accv: the wave's accumulators, 4 x NIW blocks; this call handles the column pair PAIR (blocks 2 PAIR, 2 PAIR + 1:
// the 64 columns from nw on).
template <int EPI, int RB, bool IS2D, bool YBF16, bool VEC, int NIW, int PAIR, bool SYM>
__device__ __forceinline__ void epilogue_reg_impl(const GemmArgs& a, const v16f (&accv)[4][NIW], const uint8_t* row_info,
                                                  const RegEpiOperands<EPI, (IS2D ? 2 * RB : RB)>& eo, int m0, int nw,
                                                  int wm, int lane) {
  const StampGeom& g = a.g;
  // single registers from here on (the accumulator tuples are dead after this copy)
  float acc[4][NI][16];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = accv[mi][2 * PAIR + ni][v];
  const int l32 = lane & 31, kg = lane >> 5;
  const float* s_rowfac = reinterpret_cast<const float*>(row_info);
  const int* s_rowdst = reinterpret_cast<const int*>(row_info + 1024);
  const float* s_rowz = reinterpret_cast<const float*>(row_info + 2048);
  const int n = nw + 2 * l32;
  const int nvalid = a.N - n;
  if constexpr (EPI == 3) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int r0 = wm * 128 + mi * 32 + 8 * q + 4 * kg;
        const f4 rf = *reinterpret_cast<const f4*>(s_rowfac + r0);
        const f4 rz = *reinterpret_cast<const f4*>(s_rowz + r0);
        const v4i rd = *reinterpret_cast<const v4i*>(s_rowdst + r0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float c0 = acc[mi][0][4 * q + j], c1 = acc[mi][1][4 * q + j];
          if (g.asym) {
            c0 = __builtin_fmaf(-rz[j], eo.cs[0], c0);
            c1 = __builtin_fmaf(-rz[j], eo.cs[1], c1);
          }
          if (rd[j] >= 0 && nvalid > 0)
            put_pair<YBF16, VEC>(a.out, (size_t)rd[j] * a.N + n, __builtin_fmaf(c0 * rf[j], eo.sw[0], eo.bias[0]),
                                 __builtin_fmaf(c1 * rf[j], eo.sw[1], eo.bias[1]), nvalid);
        }
      }
    }
  } else {
    constexpr int RL = IS2D ? 2 * RB : RB;
    using RM = RegMap<RL>;
    constexpr int R = RM::R, nb = RM::nb;
    // lane group kg takes the rows 8 q + 4 + j of its own blocks from the other group
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int t = 0; t < nb; ++t)
#pragma unroll
        for (int e = 0; e < R; ++e)
          if ((e & 7) == 0)  // rows e .. e + 3 against e + 4 .. e + 7
            swap32x4(acc[RM::mi(t, e)][ni][RM::v(t, e)], acc[RM::mi(t, e + 4)][ni][RM::v(t, e + 4)],
                     acc[RM::mi(t, e + 1)][ni][RM::v(t, e + 1)], acc[RM::mi(t, e + 5)][ni][RM::v(t, e + 5)],
                     acc[RM::mi(t, e + 2)][ni][RM::v(t, e + 2)], acc[RM::mi(t, e + 6)][ni][RM::v(t, e + 6)],
                     acc[RM::mi(t, e + 3)][ni][RM::v(t, e + 3)], acc[RM::mi(t, e + 7)][ni][RM::v(t, e + 7)]);
    // Every load requested before the epilogue (its operands, the next tile's row factors) has to be complete
    // here, stated in a form the compiler's wait-count bookkeeping sees: the uses below sit under branches, and a
    // load it believed pending at the end of the tile would make it wait for ALL loads inside the next main loop.
    asm volatile("" ::: "memory");       // no load may sink below the wait
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing but those loads is outstanding (no store was issued yet)
    RegOut<YBF16, VEC, !IS2D> o;
    o.sw0 = eo.sw[0];
    o.sw1 = eo.sw[1];
    o.nvalid = nvalid;
    if constexpr (!IS2D) {
      constexpr int esize = YBF16 ? 2 : 4;
      o.Y = reinterpret_cast<char*>(a.out) + (size_t)m0 * a.N * esize;
      o.tok_stride = (uint32_t)a.N * (uint32_t)esize;
      o.row_stride = 0;
    } else {
      o.Y = a.out;
      o.tok_stride = (size_t)a.N;
      o.row_stride = (size_t)g.gridW * a.N;
    }
    blocks_reg<RB, IS2D, 0, nb, YBF16, VEC, SYM>(a, acc, eo.P, eo.bias, eo.cs, o, s_rowfac + wm * 128 + kg * R, s_rowz + wm * 128 + kg * R,
                                            m0 + wm * 128 + kg * R, n, m0);
  }
}

template <int EPI, int RB, bool IS2D, bool YBF16, int NIW = NI, int PAIR = 0, bool SYM = false>
__device__ __forceinline__ void epilogue_reg(const GemmArgs& a, const v16f (&acc)[4][NIW], const uint8_t* row_info,
                                             const RegEpiOperands<EPI, (IS2D ? 2 * RB : RB)>& eo, int m0, int nw, int wm,
                                             int lane) {
  // pairs of columns are stored as one word when d_out is even (the pair then never straddles the end); the
  // fused inverse is only launched on even d_out (odd widths take the separate inverse kernel)
  if (EPI == 2 || (a.N & 1) == 0) epilogue_reg_impl<EPI, RB, IS2D, YBF16, true, NIW, PAIR, SYM>(a, acc, row_info, eo, m0, nw, wm, lane);
  else epilogue_reg_impl<EPI, RB, IS2D, YBF16, false, NIW, PAIR, SYM>(a, acc, row_info, eo, m0, nw, wm, lane);
}

}  // namespace stamp_gemm

#endif  // STAMP_EPILOGUE_REG_H_
