// Integer GEMM of the STaMP linear layer on gfx950 (step "Y <- X W" of Algorithm "STaMP Linear"):
//   acc[m, n] = sum_c code[m, c] * qW[c, n]     int8 x int8 -> int32 on v_mfma_i32_32x32x32_i8,
// followed in the same kernel by the shared epilogue (dequantization, in-block inverse transform, bias,
// store).  Serves the 8-bit rows and, as the integer engine, the 4-bit rows.
//
// Operands: 4-bit activation rows arrive packed two per byte; a packed dword w is split into
// (w << 4) & 0xF0F0F0F0 and w & 0xF0F0F0F0, i.e. the eight codes times 16 as int8.  The stored
// weights are code * 16 as well, pre-permuted to the channel order this split produces.  The
// factors 16 are exact powers of two and are folded into the row scale.
//
// Tile: 256 x 128 outputs per workgroup of 4 waves (2 x 2), two workgroups per CU; K step of 128
// codes.  Both operands are staged in LDS K-major (one row / column = one contiguous run of 64 or 128
// bytes) in 16-byte chunks whose slot is XOR-swizzled with the row number, so that fragment reads are
// free of bank conflicts; two stages, one barrier per K step.  Lane group kg (lane / 32) of an MFMA
// takes channels [64 kg + 16 ks, +16) of the step in sub-step ks: any assignment is valid as long as
// both operands use it, and this one makes every fragment read a whole 16-byte chunk.
#include <cstdlib>

#include "stamp_gemm_common.h"

namespace {

using namespace stamp_gemm;


// Epilogue of the 8-bit rows' GEMM that also runs the top levels of the inverse transform (the J - r levels over the
// k top coefficients of every sequence and output column): the tile's 256 rows are 256 / k whole sequences (k is a
// power of two, at most 256), so the block sums P of those sequences come out of the tile itself and the dequantized
// rows never go to memory.  Per pass of 32 WN columns (one 32-column MFMA block of every wave): the dequantized values,
// same arithmetic as the plain de-quantizing epilogue, go to LDS at [sequence][natural position][column] (the
// operand stages are free by now), the butterflies add and subtract the same pairs in the same order as
// k_inverse_top does (same bits: the coarse levels in place in LDS, the finest ones in registers), and row r of the
// result is block sum m0 + r.  Workgroup-wide: call from all threads.
template <typename Acc, int WN>
__device__ __forceinline__ void epilogue_top_inverse(const GemmArgs& a, typename Acc::V (&acc)[4][NI], uint8_t* smem,
                                                     uint8_t* row_info, int m0, int n0, int lane, int wm, int wn, int tid) {
  const StampGeom& g = a.g;
  constexpr int CW = 32 * WN, NT = 128 * WN;  // columns per pass; threads = 4 groups of CW
  float* s_buf = reinterpret_cast<float*>(smem);  // [256][CW]
  const float* s_rowfac = reinterpret_cast<const float*>(row_info);
  int* s_rowpos = reinterpret_cast<int*>(row_info + 1024);  // staging row of every tile row
  const float* s_rowz = reinterpret_cast<const float*>(row_info + 2048);
  const int l32 = lane & 31, kg = lane >> 5;
  const int k = g.k, nseq = 256 / k;
  // tile row seq * k + (slot e of natural position q) is staged at row seq * k + q
  for (int t = tid; t < 256; t += NT) {
    const int seq = t / k, q = t - seq * k;
    int e, lvl;
    if (!g.is2d) e = stamp_top_slot_1d(q, k, g.L, &lvl);
    else e = stamp_top_slot_2d(q / g.G, q % g.G, g.G, g.L, &lvl);
    s_rowpos[seq * k + e] = t;
  }
  __syncthreads();
  const int ch = tid % CW, grp = tid / CW;  // 4 groups
  float* P = reinterpret_cast<float*>(a.out);
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int n = n0 + wn * (32 * NI) + ni * 32 + l32;
    const float swn = a.sw[n];
    const float csn = g.asym ? a.colsum[n] : 0.0f;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int rl = wm * 128 + mi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
        float y = 0.0f;  // rows beyond the last sequence
        if (m0 + rl < a.M) {
          const float af = g.asym ? __builtin_fmaf(-s_rowz[rl], csn, (float)acc[mi][ni][v]) : (float)acc[mi][ni][v];
          y = (af * s_rowfac[rl]) * swn;
        }
        s_buf[s_rowpos[rl] * CW + wn * 32 + l32] = y;
      }
    }
    __syncthreads();
    // staged column ch = 32 w + l is output column n0 + 64 w + 32 ni + l (P is padded to whole tiles: no column check)
    const int nout = n0 + (ch >> 5) * (32 * NI) + ni * 32 + (ch & 31);
    // The coarse levels (pairs 16 or more rows apart; 2-D: cells of 8 x 8 and more) touch one row in 16 and run in
    // place in LDS; the fine levels of 16 neighbouring rows (2-D: of a 4 x 4 cell) run in registers, from where the
    // results go to P.  Every level adds and subtracts the same pairs as k_inverse_top does.
    const bool small_grid = g.is2d && g.G < 4;  // 2 x 2 blocks per sequence: all in LDS
    if (!g.is2d) {
      for (int st = 1 << g.L; st >= 32; st >>= 1) {
        const int npair = 256 / st;  // over all stacked sequences: st divides k
        for (int i = grp; i < npair; i += 4) {
          float* pa = &s_buf[(i * st) * CW + ch];
          float* pd = &s_buf[(i * st + (st >> 1)) * CW + ch];
          const float x = *pa, dd = *pd;
          *pa = x + dd;
          *pd = x - dd;
        }
        __syncthreads();
      }
      const int top = 1 << g.L;
      for (int u = grp; u < 16; u += 4) {
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = s_buf[(16 * u + i) * CW + ch];
#pragma unroll
        for (int st = 16; st >= 2; st >>= 1) {
          if (st <= top) {
#pragma unroll
            for (int i0 = 0; i0 < 16; i0 += st) {
              const float x = v[i0], dd = v[i0 + (st >> 1)];
              v[i0] = x + dd;
              v[i0 + (st >> 1)] = x - dd;
            }
          }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = 16 * u + i;
          if (m0 + r < a.M) P[(size_t)(m0 + r) * a.ld_out + nout] = v[i];
        }
      }
    } else {
      for (int st = 1 << g.L; st >= (small_grid ? 2 : 8); st >>= 1) {
        const int nc = g.G / st, h = st >> 1, cells = nc * nc;
        for (int i = grp; i < nseq * cells; i += 4) {
          const int seq = i / cells, c = i - seq * cells;
          const int cy = c / nc, cx = c - cy * nc;
          float* p00 = &s_buf[(seq * k + (cy * st) * g.G + cx * st) * CW + ch];
          float* p01 = p00 + h * CW;
          float* p10 = p00 + h * g.G * CW;
          float* p11 = p10 + h * CW;
          const float cLL = *p00, cW = *p01, cH = *p10, cD = *p11;
          const float t0 = cLL + cH, t2 = cLL - cH, t1 = cW + cD, t3 = cW - cD;
          *p00 = t0 + t1;
          *p01 = t0 - t1;
          *p10 = t2 + t3;
          *p11 = t2 - t3;
        }
        __syncthreads();
      }
      if (small_grid) {
        for (int r = grp; r < 256; r += 4)
          if (m0 + r < a.M) P[(size_t)(m0 + r) * a.ld_out + nout] = s_buf[r * CW + ch];
      } else {
        const int nc4 = g.G >> 2, cells = nc4 * nc4;  // 4 x 4 cells per sequence; nseq * cells = 16
        for (int u = grp; u < nseq * cells; u += 4) {
          const int seq = u / cells, c = u - seq * cells;
          const int cy = c / nc4, cx = c - cy * nc4;
          const int base = seq * k + (cy * 4) * g.G + cx * 4;
          float v[4][4];
#pragma unroll
          for (int dy = 0; dy < 4; ++dy)
#pragma unroll
            for (int dx = 0; dx < 4; ++dx) v[dy][dx] = s_buf[(base + dy * g.G + dx) * CW + ch];
#pragma unroll
          for (int st = 4; st >= 2; st >>= 1) {
            if (st <= (1 << g.L)) {
              const int h = st >> 1;
#pragma unroll
              for (int y0 = 0; y0 < 4; y0 += st)
#pragma unroll
                for (int x0 = 0; x0 < 4; x0 += st) {
                  const float cLL = v[y0][x0], cW = v[y0][x0 + h], cH = v[y0 + h][x0], cD = v[y0 + h][x0 + h];
                  const float t0 = cLL + cH, t2 = cLL - cH, t1 = cW + cD, t3 = cW - cD;
                  v[y0][x0] = t0 + t1;
                  v[y0][x0 + h] = t0 - t1;
                  v[y0 + h][x0] = t2 + t3;
                  v[y0 + h][x0 + h] = t2 - t3;
                }
            }
          }
#pragma unroll
          for (int dy = 0; dy < 4; ++dy)
#pragma unroll
            for (int dx = 0; dx < 4; ++dx) {
              const int r = base + dy * g.G + dx;
              if (m0 + r < a.M) P[(size_t)(m0 + r) * a.ld_out + nout] = v[dy][dx];
            }
        }
      }
    }
    __syncthreads();
  }
}

// 8-bit rows: row of A that row m of the GEMM multiplies (the first a_seq_used of every sequence's a_seq_rows)
__device__ __forceinline__ int a_row_of(const GemmArgs& a, int m) { return m + (m / a.a_seq_used) * (a.a_seq_rows - a.a_seq_used); }

// WN = waves along N: 2 -> 4 waves, tile 256 x 128, two workgroups per CU; 4 -> 8 waves, tile 256 x 256,
// one workgroup per CU (fewer, larger tiles: for the few 8-bit rows, whose whole GEMM is one round of tiles).
// EPI 4 (8-bit rows): de-quantization + the top levels of the inverse, block sums written directly (epilogue_top_inverse).
template <bool A_INT4, int EPI, int RB, bool IS2D, bool YBF16, int WN>
__global__ __launch_bounds__(128 * WN, (WN == 2 ? 2 : 1)) void k_gemm(const GemmArgs a_in) {
  GemmArgs a = a_in;
  using Acc = typename std::conditional<A_INT4, AccI8Lo, AccI8Hi>::type;
  constexpr int BN = 64 * WN, NT = 128 * WN;    // tile width, threads
  constexpr int kTileBytes = 2 * WN * kWaveTileBytes;  // the waves' epilogue staging tiles
  constexpr int nB = BN * 8 / NT;               // B chunks per thread per step (BN columns * 8 chunks / NT threads)
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  constexpr int rowA = A_INT4 ? 64 : 128;       // bytes per A row per K step
  constexpr int chA = rowA / 16;                // 16-byte chunks per A row (4 or 8)
  constexpr int bytesA = BM * rowA, bytesB = BN * 128;
  constexpr int stage = bytesA + bytesB;
  constexpr int nA = 256 * chA / NT;            // A chunks per thread per step (256 rows * chA / NT threads)
  constexpr int kMainBytes = 2 * stage;
  constexpr int kRowInfoOff = (EPI >= 2 && kTileBytes > kMainBytes) ? kTileBytes : kMainBytes;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
  const int wm = wave / WN, wn = wave % WN;  // wave tile: rows [128 wm, +128), columns [64 wn, +64)
  const int l32 = lane & 31, kg = lane >> 5;
  int tm, tn;
  const int KT = a.Kpad / BK;
  int kt0 = 0, kt1 = KT;  // K steps of this workgroup
  if constexpr (!A_INT4 && EPI == 1) {
    // split depth: partial dequantized rows per part (the consumer adds them); the zero-point term of
    // asymmetric codes goes with part 0 only
    int split = 0;
    if (a.ksplit > 1) tile_of_block_split(a.M, a.ksplit, tm, tn, split);
    else tile_of_block(a.M, a.Npad, BN, tm, tn);
    kt0 = (int)((long long)KT * split / a.ksplit);
    kt1 = (int)((long long)KT * (split + 1) / a.ksplit);
    a.out = reinterpret_cast<float*>(a.out) + (size_t)split * a.split_stride;
    if (split > 0) a.g.asym = 0;
  } else {
    tile_of_block(a.M, a.Npad, BN, tm, tn);
  }
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- global -> LDS assignment: chunk q = i * NT + tid of the tile, consecutive lanes = consecutive
  //      chunks.  Row / column of chunk i is (row0 + i * rows_per_pass); its swizzled slot does not
  //      depend on i, so one base address per operand and a uniform stride per pass suffice. ----
  constexpr int rowsPerPassA = NT / chA;   // rows per pass of NT threads
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
      offA[i] = (uint32_t)(a_row_of(a, min(m0 + rowA0 + i * rowsPerPassA, a.M - 1)) - a_row_of(a, m0)) * (uint32_t)a.a_row_bytes + koffA;
    }
  }
  if constexpr (A_INT4) baseGA += (size_t)tm * KT * (256 * 64);
  else baseGA += (size_t)a_row_of(a, m0) * a.a_row_bytes;
  // byte offset (from baseGA) of the last 16-byte chunk that may be read
  const size_t lastA = a.a_last16 - (size_t)(baseGA - a.A);
  const int colB0 = tid >> 3, slotB = tid & 7;
  const int cB = slotB ^ ((colB0 >> 1) & 7);
  // stored weight: [Npad/128][KT][128 columns][128 bytes]; pass i of this thread is column colB0 + 32 i
  // (column tiles of 128: a 256-wide tile spans two of them, KT * 16 KB apart)
  const uint8_t* baseGB = a.Bq + stamp_w_offset(n0, 0, a.Kpad);
  uint32_t offB[nB];
#pragma unroll
  for (int i = 0; i < nB; ++i) {
    const int col = colB0 + (NT / 8) * i;
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
  // Addresses: a buffer descriptor per operand (scalar base; the 8-bit rows' descriptor ends with the buffer, so a
  // chunk past the end of the last row reads zeros) + a scalar byte offset per K step + the thread's constant 32-bit
  // offset of the pass: no vector address arithmetic per load.
  const size_t restA = A_INT4 ? (size_t)0x7fffffff : (lastA + 16);
  // (the builtins exist in the device pass only; the host pass, which needs no more than the kernel's signature,
  // sees an empty request)
  __amdgpu_buffer_rsrc_t rdA, rdB;
#if defined(__HIP_DEVICE_COMPILE__)
  rdA = __builtin_amdgcn_make_buffer_rsrc((void*)baseGA, 0, (int)(restA < (size_t)0x7fffffff ? restA : (size_t)0x7fffffff), 0x00020000);
  rdB = __builtin_amdgcn_make_buffer_rsrc((void*)baseGB, 0, 0x7fffffff, 0x00020000);
#else
  (void)kStepA, (void)kStepB, (void)baseGB, (void)restA, (void)rdA, (void)rdB;
#endif
  auto request = [&](int kstep, int stg) __attribute__((always_inline)) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint8_t* so_ = smem + stg * stage + wave * 1024;
    const uint32_t ka_ = (uint32_t)kstep * (uint32_t)kStepA, kb_ = (uint32_t)kstep * (uint32_t)kStepB;
#pragma unroll
    for (int i = 0; i < nA; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rdA, (void __attribute__((address_space(3)))*)(so_ + i * (NT * 16)), 16, offA[i], ka_, 0, 0);
#pragma unroll
    for (int i = 0; i < nB; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rdB, (void __attribute__((address_space(3)))*)(so_ + bytesA + i * (NT * 16)), 16, offB[i],
                                               kb_, 0, 0);
#else
    (void)kstep;
    (void)stg;
#endif
  };
#define STAMP_REQUEST(KSTEP, STG) request((int)(KSTEP), (int)(STG))

  STAMP_REQUEST(kt0, 0);
  EpiOperands<EPI, RB, IS2D> eo;
  eo.request(a, m0, n0, lane, wm, wn);
  if (NT == 256 || tid < 256) store_row_info<Acc, EPI>(a, m0, tid, smem + kRowInfoOff);

  // Step kt: wait for this wave's loads of step kt, then the workgroup barrier (every wave's loads of
  // step kt have landed, and every wave has left step kt-1, whose stage is now free); request step
  // kt+1 into that free stage; run the MFMAs of step kt.
  for (int kt = kt0; kt < kt1; ++kt) {
    const uint8_t* st = smem + ((kt - kt0) & 1) * stage;
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kt + 1 < kt1) STAMP_REQUEST(kt + 1, (kt + 1 - kt0) & 1);
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
      // both operands' fragments of sub-step ks + 1 are read while sub-step ks is multiplied
      u4 wa[2][4];
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) wa[0][mi] = *reinterpret_cast<const u4*>(st + baseA + mi * blkA);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        if (ks < 3) {
#pragma unroll
          for (int mi = 0; mi < 4; ++mi)
            wa[(ks + 1) & 1][mi] = *reinterpret_cast<const u4*>(st + (baseA ^ ((ks + 1) << 4)) + mi * blkA);
#pragma unroll
          for (int ni = 0; ni < NI; ++ni) {
            const u4 w = *reinterpret_cast<const u4*>(st + (baseB ^ ((ks + 1) << 4)) + ni * blkB);
            fb[(ks + 1) & 1][ni][0] = (int)w.x; fb[(ks + 1) & 1][ni][1] = (int)w.y;
            fb[(ks + 1) & 1][ni][2] = (int)w.z; fb[(ks + 1) & 1][ni][3] = (int)w.w;
          }
        }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
          const u4 w = wa[ks & 1][mi];
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

  if constexpr (EPI == 4) epilogue_top_inverse<Acc, WN>(a, acc, smem, smem + kRowInfoOff, m0, n0, lane, wm, wn, tid);
  else epilogue<Acc, EPI, RB, IS2D, YBF16>(a, acc, smem, smem + kRowInfoOff, eo, m0, n0, lane, wave, wm, wn);
}

// ------------------------------------------------------------------------------------------------------------
// The 8-bit rows when the whole batch has at most 128 of them (e.g. 64 8-bit tokens of one sequence): the GEMM is a
// stream of the stored weights (1 byte per weight, tens of MB) against a few rows, bound by how many bytes are in
// flight, not by the matrix pipe.  Tile: MB (64 or 128) rows x 128 columns per workgroup of 4 waves (wave w: the 32
// columns 32 w.., all rows), K step 128, a ring of three stages of MB x 128 + 128 x 128 bytes filled by asynchronous
// loads two steps ahead, two workgroups per CU (one for 128 rows), the depth split over several workgroups per tile
// (partial rows, added
// by the consumer as for the large tiles).  Same operand layout in LDS, same fragment order and the same
// dequantization (EPI 1 of the shared epilogue) as k_gemm<false, 1, ...>: identical results.
template <int MB>
__global__ __launch_bounds__(256, 2) void k_gemm_hi_few(const GemmArgs a_in) {
  GemmArgs a = a_in;
  using Acc = AccI8Hi;
  constexpr int NT = 256, BNF = 128, MI = MB / 32, NS = 3;
  constexpr int bytesA = MB * 128, bytesB = BNF * 128, stage = bytesA + bytesB;
  constexpr int nA = MB * 8 / NT, nB = BNF * 8 / NT;  // 16-byte chunks per thread and step
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint8_t* const row_info = smem + NS * stage;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, kg = lane >> 5;
  const int KT = a.Kpad / BK;
  const int tn = (int)blockIdx.x / a.ksplit, split = (int)blockIdx.x - tn * a.ksplit;
  const int kt0 = (int)((long long)KT * split / a.ksplit), kt1 = (int)((long long)KT * (split + 1) / a.ksplit);
  a.out = reinterpret_cast<float*>(a.out) + (size_t)split * a.split_stride;
  if (split > 0) a.g.asym = 0;  // the zero-point term of asymmetric codes goes with part 0 only
  const int n0 = tn * BNF;

  // global -> LDS: chunk q = i * NT + tid of an operand's stage goes to byte 16 q = (row q / 8, slot q % 8); the slot
  // holds the row's chunk (slot ^ swizzle(row)), applied on the global side
  const int rowA0 = tid >> 3, slot = tid & 7;
  const uint32_t kofs = (uint32_t)((slot ^ ((rowA0 >> 1) & 7)) * 16);
  uint32_t offA[nA], offB[nB];
#pragma unroll
  for (int i = 0; i < nA; ++i) offA[i] = (uint32_t)a_row_of(a, min(rowA0 + i * (NT / 8), a.M - 1)) * (uint32_t)a.a_row_bytes + kofs;
#pragma unroll
  for (int i = 0; i < nB; ++i) offB[i] = (uint32_t)((rowA0 + i * (NT / 8)) * 128) + kofs;
  const uint8_t* baseGB = a.Bq + stamp_w_offset(n0, 0, a.Kpad);
  const size_t restA = a.a_last16 + 16;
  __amdgpu_buffer_rsrc_t rdA, rdB;
#if defined(__HIP_DEVICE_COMPILE__)
  rdA = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, (int)(restA < (size_t)0x7fffffff ? restA : (size_t)0x7fffffff), 0x00020000);
  rdB = __builtin_amdgcn_make_buffer_rsrc((void*)baseGB, 0, 0x7fffffff, 0x00020000);
#else
  (void)baseGB, (void)restA, (void)rdA, (void)rdB;
#endif
  auto request = [&](int kstep, int stg) __attribute__((always_inline)) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint8_t* so_ = smem + stg * stage + wave * 1024;
    const uint32_t ka_ = (uint32_t)kstep * 128u, kb_ = (uint32_t)kstep * (uint32_t)(128 * 128);
#pragma unroll
    for (int i = 0; i < nA; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rdA, (void __attribute__((address_space(3)))*)(so_ + i * (NT * 16)), 16, offA[i], ka_, 0, 0);
#pragma unroll
    for (int i = 0; i < nB; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rdB, (void __attribute__((address_space(3)))*)(so_ + bytesA + i * (NT * 16)), 16, offB[i],
                                               kb_, 0, 0);
#else
    (void)kstep, (void)stg;
#endif
  };

  // LDS -> fragments (hand-written reads: the compiler orders every LDS read it can see behind ALL asynchronous loads)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)smem;
  const uint32_t baseA = (uint32_t)(l32 * 128 + (((4 * kg) ^ ((l32 >> 1) & 7)) << 4));
  const int nl = wave * 32 + l32;
  const uint32_t baseB = (uint32_t)(bytesA + nl * 128 + (((4 * kg) ^ ((nl >> 1) & 7)) << 4));

  v16i acc[MI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0;

  const int nsteps = kt1 - kt0;
  request(kt0, 0);
  if (nsteps > 1) request(kt0 + 1, 1);
  if (tid < MB) store_row_info<Acc, 1>(a, 0, tid, row_info);
  for (int i = 0; i < nsteps; ++i) {
    asm volatile("" ::: "memory");
    if (i + 1 < nsteps) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(nA + nB) : "memory");  // the next step's loads may stay in flight
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (i + 2 < nsteps) request(kt0 + i + 2, (i + 2) % NS);  // into the stage of step i - 1, which every wave has left
    const uint32_t st = lds0 + (uint32_t)((i % NS) * stage);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u4 wb, wa[MI];
      asm volatile("ds_read_b128 %0, %1" : "=v"(wb) : "v"(st + (baseB ^ (uint32_t)(ks << 4))));
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(wa[mi]) : "v"(st + (baseA ^ (uint32_t)(ks << 4))), "n"(mi * 32 * 128));
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wb), "+v"(wa[0]), "+v"(wa[MI - 1]));
      if constexpr (MI == 4) asm volatile("" : "+v"(wa[1]), "+v"(wa[2]));
      v4i fb;
      fb[0] = (int)wb.x; fb[1] = (int)wb.y; fb[2] = (int)wb.z; fb[3] = (int)wb.w;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const u4 w = wa[mi];
        // natural channel order -> the order of the stored weights: evens then odds per 8 channels
        v4i fa;
        fa[0] = (int)__builtin_amdgcn_perm(w.y, w.x, 0x06040200u);
        fa[1] = (int)__builtin_amdgcn_perm(w.y, w.x, 0x07050301u);
        fa[2] = (int)__builtin_amdgcn_perm(w.w, w.z, 0x06040200u);
        fa[3] = (int)__builtin_amdgcn_perm(w.w, w.z, 0x07050301u);
        acc[mi] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb, acc[mi], 0, 0, 0);
      }
    }
  }
  __syncthreads();  // the row table (and, for a part without steps, nothing else) is complete

  const StampGeom& g = a.g;
  const float* s_rowfac = reinterpret_cast<const float*>(row_info);
  const int* s_rowdst = reinterpret_cast<const int*>(row_info + 1024);
  const float* s_rowz = reinterpret_cast<const float*>(row_info + 2048);
  const int n = n0 + nl;
  const float swn = a.sw[n];
  const float csn = g.asym ? a.colsum[n] : 0.0f;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rl = mi * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
      const int dst = s_rowdst[rl];
      if (dst >= 0 && n < a.N) {
        // asymmetric: the integer sum over (stored code - offset), exact in one fma
        const float af = g.asym ? __builtin_fmaf(-s_rowz[rl], csn, (float)acc[mi][v]) : (float)acc[mi][v];
        reinterpret_cast<float*>(a.out)[(size_t)dst * a.ld_out + n] = (af * s_rowfac[rl]) * swn;
      }
    }
  }
}

template <int MB>
hipError_t launch_hi_few(const GemmArgs& a, hipStream_t st) {
  constexpr size_t lds = 3 * (size_t)(MB * 128 + 128 * 128) + kRowInfoBytes;
  static size_t lds_done[kStampMaxDevices] = {};
  hipError_t e = stamp_allow_lds(reinterpret_cast<const void*>(&k_gemm_hi_few<MB>), lds, lds_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((k_gemm_hi_few<MB>), dim3((a.Npad / 128) * a.ksplit), dim3(256), lds, st, a);
  return hipGetLastError();
}

template <bool A_INT4, int EPI, int RB, bool IS2D, bool YBF16, int WN>
hipError_t launch_y(const GemmArgs& a, hipStream_t st) {
  constexpr int BN = 64 * WN;
  constexpr size_t main_lds = 2 * (size_t)(BM * (A_INT4 ? 64 : 128) + BN * 128);
  constexpr size_t epi_lds = (EPI >= 2) ? (size_t)(2 * WN * kWaveTileBytes) : 0;
  constexpr size_t lds = (main_lds > epi_lds ? main_lds : epi_lds) + kRowInfoBytes;  // + per-row factors, destinations, offsets
  static size_t lds_done[kStampMaxDevices] = {};
  hipError_t e = stamp_allow_lds(reinterpret_cast<const void*>(&k_gemm<A_INT4, EPI, RB, IS2D, YBF16, WN>), lds, lds_done);
  if (e != hipSuccess) return e;
  const int mt = (a.M + BM - 1) / BM, nt = a.Npad / BN;
  const int split = (!A_INT4 && EPI == 1) ? a.ksplit : 1;
  hipLaunchKernelGGL((k_gemm<A_INT4, EPI, RB, IS2D, YBF16, WN>), dim3(mt * nt * split), dim3(128 * WN), lds, st, a);
  return hipGetLastError();
}

template <bool A_INT4, int EPI, int RB, bool IS2D>
hipError_t launch(const GemmArgs& a, hipStream_t st) {
  // the output type only matters to the fused epilogue
  if constexpr (EPI == 2 || EPI == 3) {
    if (a.g.y_bf16) return launch_y<A_INT4, EPI, RB, IS2D, true, 2>(a, st);
  }
  if constexpr (!A_INT4) {
    if (stamp_hi_wide_tiles(a.M, a.Npad)) return launch_y<A_INT4, EPI, RB, IS2D, false, 4>(a, st);
  }
  return launch_y<A_INT4, EPI, RB, IS2D, false, 2>(a, st);
}

}  // namespace

namespace {
int device_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
  }
  return cus;
}
}  // namespace

// The 8-bit rows' GEMM keeps one 256 x 128 workgroup per CU (its stages hold unpacked int8 rows).  When
// that needs more than one round of tiles, 256 x 256 tiles (half as many, one round) finish sooner.
bool stamp_hi_wide_tiles(int M, int Npad) {
  const int tiles128 = ((M + stamp_gemm::BM - 1) / stamp_gemm::BM) * (Npad / 128);
  return tiles128 > device_cus();
}

// Plans without top levels: the dequantized top rows ARE the block sums P of the inverse (the top inverse has
// nothing to do), so the 8-bit rows' GEMM writes them where the 4-bit rows' epilogue reads them, unless its depth
// is split (then the partial rows go through the top inverse like any others: it adds the parts and moves nothing).
bool stamp_hi_rows_are_block_sums(const stamp_plan* p) { return !p->geom.ident && p->geom.L == 0 && p->hi_ksplit <= 1; }

// at most this many 8-bit rows over the whole batch: the kernel for few rows
constexpr int kHiFewRows = 128;

// Plans with top levels whose 8-bit rows' GEMM keeps its depth in one piece and runs the tiled kernel: a tile of 256
// rows holds whole sequences (k divides 256), so its epilogue can run the top levels of the inverse itself and write
// the block sums (no partial rows in memory, no k_inverse_top).
bool stamp_hi_top_fused(const stamp_plan* p) {
  const StampGeom& g = p->geom;
  return p->gen.kind == kGenNone && !g.ident && g.L > 0 && p->hi_ksplit <= 1 && g.B * g.k > kHiFewRows && g.k <= 256 &&
         (g.k & (g.k - 1)) == 0;
}

// The few 8-bit rows make few tiles: when they would leave most CUs idle, the depth of every tile is split
// over 2..4 workgroups (partial rows, added by the top inverse).

int stamp_hi_ksplit(const stamp_plan* p, int rows_per_seq) {
  const int M = p->geom.B * rows_per_seq;
  if (M == 0) return 1;
  if (M <= kHiFewRows) {
    // few rows: enough parts for one workgroup per CU, each with at least four K steps; a part's partial rows cost
    // 8 M d_out bytes of traffic (written here, read by the consumer), which more parts than that do not repay
    // (measured on the 2048-token language-model layer, 86 tiles: 2, 3, 4 parts -> step 0.113, 0.115, 0.116 ms)
    const int tiles = p->Npad / 128, KT = p->Kpad / stamp_gemm::BK;
    int s = (device_cus() + tiles - 1) / tiles;
    if (s > KT / 4) s = KT / 4;
    if (s > 4) s = 4;
    return s < 1 ? 1 : s;
  }
  const int mt = (M + stamp_gemm::BM - 1) / stamp_gemm::BM;
  const int tiles = mt * (p->Npad / (stamp_hi_wide_tiles(M, p->Npad) ? 256 : 128));
  const int KT = p->Kpad / stamp_gemm::BK;
  int s = device_cus() / tiles;
  if (s > 4) s = 4;
  while (s > 1 && KT / s < 2) --s;
  return s < 2 ? 1 : s;
}

stamp_gemm::GemmArgs stamp_gemm_args(const stamp_plan* p, const float* scales, void* out) {
  stamp_gemm::GemmArgs a;
  a.Bq = reinterpret_cast<const uint8_t*>(p->qW_dev);
  a.scales = scales;
  a.sw = p->sw_dev;
  a.colsum = p->colsum_dev;
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
  a.ld_out = p->geom.N;
  a.ksplit = 1;
  a.split_stride = 0;
  a.a_seq_rows = a.a_seq_used = 1;
  a.own_top = 0;
  return a;
}

hipError_t stamp_launch_gemm_hi(const stamp_plan* p, const int8_t* q_hi, const float* scales, int mode, void* out,
                                hipStream_t st, int ld_out, bool first_khi_only) {
  GemmArgs a = stamp_gemm_args(p, scales, out);
  a.A = reinterpret_cast<const uint8_t*>(q_hi);
  a.M = p->geom.B * p->geom.k;
  a.a_row_bytes = p->geom.d;
  a.a_last16 = (size_t)a.M * a.a_row_bytes - 16;
  if (mode == 0) return launch<false, 0, 0, false>(a, st);
  if (mode == 1) {
    if (ld_out > 0) a.ld_out = ld_out;
    a.ksplit = p->hi_ksplit;
    if (first_khi_only) {
      // the kernels see a plan of khi top rows per sequence; only the rows of A keep their places
      a.a_seq_rows = p->geom.k;
      a.a_seq_used = p->geom.khi;
      a.g.k = p->geom.khi;
      a.M = p->geom.B * p->geom.khi;
      a.ksplit = p->hi_ksplit_own;
    }
    a.split_stride = (size_t)a.M * a.N;
    if (a.M <= 64) return launch_hi_few<64>(a, st);
    if (a.M <= kHiFewRows) return launch_hi_few<128>(a, st);
    return launch<false, 1, 0, false>(a, st);
  }
  if (mode == 2) {
    // dequantization + top levels of the inverse in the tile: out = the block sums P, ld_out floats per row
    if (!stamp_hi_top_fused(p) || ld_out <= 0) return hipErrorInvalidValue;
    a.ld_out = ld_out;
    return launch<false, 4, 0, false>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t stamp_launch_gemm_lo(const stamp_plan* p, const uint8_t* q_lo, const float* scales, int mode, void* out,
                                const float* P, hipStream_t st) {
  GemmArgs a = stamp_gemm_args(p, scales, out);
  a.A = q_lo;
  a.M = p->geom.B * p->geom.s;
  a.a_row_bytes = p->geom.d / 2;
  a.a_last16 = (size_t)p->Mpad * (p->Kpad / 2) - 16;
  a.P = P;
  if (mode == 0) return launch<true, 0, 0, false>(a, st);
  if (mode == 1) return launch<true, 1, 0, false>(a, st);
  if (mode == 3) return launch<true, 3, 0, false>(a, st);
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
