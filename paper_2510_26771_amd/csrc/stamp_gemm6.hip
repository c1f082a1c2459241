// GEMM of the 4-bit rows of the STaMP linear layer on the FP6 matrix pipeline of gfx950 (step
// "Y <- X W" of Algorithm "STaMP Linear" for the rows quantized to 4 bits against 4-bit weights).
//
// A 4-bit code c in [-8, 7] is held as the E2M3 number c / 8: for |c| < 8 sign bit, exponent field 0,
// mantissa field |c| (a subnormal); |c| = 8 is 1.0 (exponent field 1, mantissa 0): either way the six
// bits are just sign and 4-bit magnitude.  v_mfma_f32_32x32x64_f8f6f4
// multiplies such operands exactly and accumulates in fp32; every product is a multiple of 1/64 and a
// whole sum stays below 2^24 / 64 in magnitude (|c c'| <= 56 and d_in <= 32768: 56 * 32768 < 2^24), so the fp32 accumulator
// holds acc / 64 EXACTLY, where acc is the integer sum the int8 pipeline computes: same result bit for
// bit, at twice the matrix rate per clock.  The factor 64 is folded into the row scale.
//
// Operand layout: the 32 codes that one lane feeds to one MFMA (channels 32 f .. 32 f + 31 of a K step of
// 128 channels, f = 0..3) are a little-endian stream of 6-bit fields = 24 bytes.  MFMA half k (0, 1) of a
// step consumes channels [64 k, 64 k + 64): lane group kg = lane / 32 takes f = 2 k + kg, so over a step a
// lane needs fragments kg and 2 + kg of its row: 48 bytes, kept as three 16-byte parts.  Per block of 32
// rows (columns) and K step: [3 parts][2 kg][32 rows][16 bytes] = 3 KB, so that the 64 lanes of a wave read
// 1 KB of consecutive addresses with one 16-byte LDS read (no bank conflicts, no swizzle; 16-byte reads
// move 1.75x the bytes per clock of 8-byte ones on this chip, and at 8 bytes the fragment reads of a step
// take as long as its MFMAs).  Per tile and K step, activations: 8 blocks = 24 KB, weights: 4 blocks = 12 KB
// per 128 columns.  The global image equals the LDS image, so a K step is staged by plain asynchronous
// 16-byte copies.
#include <type_traits>

#include "stamp_gemm_common.h"
#include "stamp_epilogue_reg.h"

namespace {

using namespace stamp_gemm;

typedef int v6i __attribute__((ext_vector_type(6)));
typedef uint32_t u6 __attribute__((ext_vector_type(6)));
// the FP6 operand of the MFMA builtin is declared as 8 registers, of which the instruction reads 6
__device__ __forceinline__ v8i widen(v6i x) { return __builtin_shufflevector(x, x, 0, 1, 2, 3, 4, 5, -1, -1); }

constexpr int kPart = 2 * 32 * 16;            // bytes of one part of a 32-row block: 1 KB
constexpr int kBlock6 = 3 * kPart;            // a 32-row block of one K step: 3 KB
constexpr int kStageB6 = 4 * kBlock6;         // 128 columns: 12 KB
constexpr int kStageA6 = 2 * kStageB6;        // 24 KB

// eight two's-complement nibbles -> eight sign-magnitude 6-bit fields (48 bits)
__device__ __forceinline__ uint64_t nib8_to_e2m3(uint32_t w) {
  const uint32_t s = w & 0x88888888u;  // sign bit of every nibble
  const uint32_t sg = s >> 3;          // 1 in every negative nibble
  // |c|: complement the negative nibbles and add 1 (no carry leaves a nibble: ~c + 1 <= 8).  |c| = 8
  // (the stored form of the asymmetric code 0) sets the low exponent bit: the E2M3 number 1.0 = 8 / 8.
  const uint32_t mag = (w ^ (sg * 15u)) + sg;
  uint64_t out = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t c = ((mag >> (4 * j)) & 15u) | (((s >> (4 * j + 3)) & 1u) << 5);
    out |= (uint64_t)c << (6 * j);
  }
  return out;
}

// 32 codes (one 16-byte chunk of packed nibbles, low nibble = even channel) -> 24 bytes
__device__ __forceinline__ void chunk_to_e2m3(u4 w, uint64_t (&part)[3]) {
  const uint64_t a = nib8_to_e2m3(w.x), b = nib8_to_e2m3(w.y), c = nib8_to_e2m3(w.z), d = nib8_to_e2m3(w.w);
  part[0] = a | (b << 48);
  part[1] = (b >> 16) | (c << 32);
  part[2] = (c >> 32) | (d << 16);
}

// q_lo (tiled [Mpad/256][KT][256 rows][64 bytes], channels in natural order) -> FP6 operand layout.
// One workgroup per (row tile, K step); thread = (row, kg): fragments kg and 2 + kg, three 16-byte stores.
__global__ __launch_bounds__(512) void k_repack6(const uint8_t* __restrict__ q_lo, uint8_t* __restrict__ a6) {
  const size_t blk = blockIdx.x;
  const int row = threadIdx.x & 255, kg = threadIdx.x >> 8;
  const uint8_t* src = q_lo + blk * (256 * 64) + row * 64 + kg * 16;
  uint8_t* dst = a6 + blk * kStageA6 + (row >> 5) * kBlock6 + kg * 512 + (row & 31) * 16;
  uint64_t lo[3], hi[3];
  chunk_to_e2m3(*reinterpret_cast<const u4*>(src), lo);
  chunk_to_e2m3(*reinterpret_cast<const u4*>(src + 32), hi);
  typedef uint64_t ul2 __attribute__((ext_vector_type(2)));
  *reinterpret_cast<ul2*>(dst) = ul2{lo[0], lo[1]};
  *reinterpret_cast<ul2*>(dst + kPart) = ul2{lo[2], hi[0]};
  *reinterpret_cast<ul2*>(dst + 2 * kPart) = ul2{hi[1], hi[2]};
}

// Plan-time weight codes in that layout: per output channel n, code = rne(W_cn * (7 / max)) as in
// the integer engine (round-to-nearest weights, one scale per output channel), stored as E2M3 c / 8.
// One thread per (column, 32-channel fragment).
__global__ __launch_bounds__(256) void k_w_quant6(const float* __restrict__ W, const uint32_t* __restrict__ colmax,
                                                  uint8_t* __restrict__ b6, int d, int N, int Kpad, int Npad, size_t sc,
                                                  size_t sn) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  const int frag = blockIdx.y;  // 32-channel fragment over the whole depth
  if (n >= Npad) return;
  float inv = 0.0f;
  if (n < N) {
    const float a = __uint_as_float(colmax[n]);
    if (a > 0.0f) inv = __fdiv_rn(7.0f, a);
  }
  uint64_t part[3] = {0, 0, 0};
  uint64_t acc = 0;
  int nbits = 0, o = 0;
  for (int i = 0; i < 32; ++i) {
    const int c = frag * 32 + i;
    uint32_t code = 0;
    if (n < N && c < d) {
      float r = rintf(__fmul_rn(W[(size_t)c * sc + (size_t)n * sn], inv));
      r = fminf(fmaxf(r, -7.0f), 7.0f);
      const int q = (int)r;
      code = (uint32_t)(q < 0 ? -q : q) | (q < 0 ? 32u : 0u);
    }
    acc |= (uint64_t)code << nbits;
    nbits += 6;
    if (nbits >= 64) {
      part[o++] = acc;
      nbits -= 64;
      acc = (nbits > 0) ? ((uint64_t)code >> (6 - nbits)) : 0;
    }
  }
  const int KT = Kpad >> 7;
  const int kt = frag >> 2, f = frag & 3;
  // fragment f is the (f >> 1)-th half of the 48-byte stream of lane group kg = f & 1
  // output column n = 64 w + 2 l + ni sits in the 32-column block 2 w + ni at row l: a lane of the GEMM then holds
  // two neighbouring output columns (stamp_epilogue_reg.h)
  const int blk = ((n & 127) >> 6) * 2 + (n & 1), rowb = (n & 63) >> 1;
  uint8_t* dst = b6 + ((size_t)(n >> 7) * KT + kt) * kStageB6 + (size_t)blk * kBlock6 + (f & 1) * 512 + rowb * 16;
  for (int p = 0; p < 3; ++p) {
    const int off = (f >> 1) * 24 + p * 8;
    *reinterpret_cast<uint64_t*>(dst + (off >> 4) * kPart + (off & 15)) = part[p];
  }
}

// Workgroup: 8 waves (2 x 4), tile 256 x 256, one workgroup per CU with two waves on every SIMD, all
// eight sharing one operand stage: 48 KB per K step for 256 x 256 x 128 products, a third less L2 -> LDS
// traffic per product than two independent 256 x 128 workgroups would need (the FP6 pipeline consumes a K
// step in half the time of the int8 one, which makes that traffic the bound).  Three stages: while step kt is
// multiplied, the stage of step kt+1 has landed or is landing and that of step kt+2 is in flight; the request for
// step kt+3 goes out late in step kt, into the stage that step kt has just given up.
//
// The kernel is persistent: one workgroup per CU walks its share of the tiles (the XCD-aware order of
// tile_of_sid, every workgroup of an XCD taking every wx-th tile of that XCD's range), and the operand
// pipeline runs on across tile boundaries: the first three K steps of the next tile are requested during the last
// three steps of the current one, so they, and the stores of the epilogue, are in flight while the epilogue
// computes.  The epilogue works in registers (stamp_epilogue_reg.h) and leaves the operand stages alone.
//
// Inside a step nothing waits for what it has just asked for: the LDS reads of an activation block fly under the
// MFMAs of the block before it, the one workgroup barrier sits before the last block (whose MFMAs cover the reads
// of the next step's first fragments), and the six loads of a stage request are issued one at a time among MFMAs (three in that last
// block, three in the first two blocks of the next step).
constexpr int BN6 = 256;
constexpr int kStage6 = kStageA6 + 2 * kStageB6;  // 48 KB
constexpr int kNumStage6 = 3;

// tile of position sid in the walk: 8 M-tiles, then the next N-tile, group of 8 M-tiles after group
__device__ __forceinline__ void tile_of_sid(int sid, int mt, int nt, int& tm, int& tn) {
  const int per_group = kGroupM * nt;
  const int grp = sid / per_group, in_grp = sid - grp * per_group;
  const int gm = min(kGroupM, mt - grp * kGroupM);
  tm = grp * kGroupM + in_grp % gm;
  tn = in_grp / gm;
}

// SYM: a fused-mode kernel for plans with symmetric activation codes (no offset term in the epilogue)
template <int EPI, int RB, bool IS2D, bool YBF16, bool SYM = false>
__global__ __launch_bounds__(512, 1) void k_gemm6(const GemmArgs a) {
  using Acc = AccF6Lo;
  constexpr int NIW = NI;  // 32-column MFMA blocks per wave along N
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  constexpr int NT = 512;  // threads
  constexpr int kMainBytes = kNumStage6 * kStage6;
  uint8_t* const row_info = smem + kMainBytes;  // two buffers of kRowInfoBytes, alternating from tile to tile
  constexpr int nA = kStageA6 / (NT * 16), nB = 2 * kStageB6 / (NT * 16);  // 16-byte chunks per thread and step
  constexpr int kLoadsPerStep = nA + nB;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
  // wave tile: rows [128 wm, +128), columns [32 NIW wn, +32 NIW)
  const int wm = wave >> 2, wn = wave & 3;
  const int KT = a.Kpad / BK;
  const int mt = (a.M + BM - 1) / BM, nt = a.Npad / BN6, total = mt * nt;

  // tiles of this workgroup: the XCD's contiguous range of the walk, every wx-th position from `local` on
  const int nwg = (int)gridDim.x, xcd = (int)blockIdx.x % kNumXcd, local = (int)blockIdx.x / kNumXcd;
  const int wx = (nwg - xcd + kNumXcd - 1) / kNumXcd;  // workgroups that run on this XCD
  const int tall = total / kNumXcd, rem = total % kNumXcd;
  const int first = xcd * tall + min(xcd, rem), count = tall + (xcd < rem ? 1 : 0);
  if (local >= count) return;

  // global image = LDS image: chunk q = i * NT + tid of an operand's stage goes to byte 16 q.  The
  // weight stage is two column tiles of 128 (KT * 12 KB apart in memory): chunks 0..767 and 768..1535;
  // the boundary falls between waves, so the source tile of a pass is wave-uniform.  Addresses are a
  // wave-uniform base (tile, K step, pass) plus this thread's constant 32-bit offset.
  const uint32_t off16 = (uint32_t)tid * 16u;
  // cursor of the requests: request rq_kt of the tile at position rq_pos of this workgroup's walk (all scalar).  The
  // loads address memory through two buffer descriptors (the tile's activation panel; its two weight panels, KT * 12 KB
  // apart) + a scalar byte offset + this thread's constant 32-bit offset: no vector address arithmetic per load.
  // K step of a tile's first request.  The workgroups of an XCD that share an operand panel (same row or column of
  // the XCD's 8 x 4 window of tiles) ask for a line at the same moment when they walk K in step: one misses L2, the
  // others wait on the same miss.  Started a few K steps apart (every tile walks all KT steps once, from its own
  // start, wrapping: an fp32 sum of these integers is exact in any order), most of them find the line in L2.
  int rq_k0;
  {
    int tm0_, tn0_;
    tile_of_sid(first + local, mt, nt, tm0_, tn0_);
    rq_k0 = (((tm0_ & 7) + 2 * (tn0_ & 3)) & 7) % KT;
  }
  int rq_pos = local, rq_kt = 0, rq_stg = 0, rq_kk = rq_k0;  // rq_kt counts the tile's requests, rq_kk is their K step
  __amdgpu_buffer_rsrc_t rdA, rdB;
  auto rq_tile = [&]() {
    int tm_, tn_;
    tile_of_sid(first + rq_pos, mt, nt, tm_, tn_);
    rdA = __builtin_amdgcn_make_buffer_rsrc((void*)(a.A + (size_t)tm_ * KT * kStageA6), 0, 0x7fffffff, 0x00020000);
    rdB = __builtin_amdgcn_make_buffer_rsrc((void*)(a.Bq + (size_t)(2 * tn_) * KT * kStageB6), 0, 0x7fffffff, 0x00020000);
  };
  rq_tile();
  // A request = the kLoadsPerStep loads of the next K step of the walk into the next stage of the ring.  rq_begin
  // fixes its addresses and advances the cursor, rq_issue<i> issues its i-th load: the
  // main loop spreads them among its MFMAs (eight waves issuing all their loads at once keep the address unit busy
  // for several hundred cycles, during which none of them can issue anything else).
  // Of a request's six loads three go out among the MFMAs of the step's last block, the others in the next step: two
  // in its first block (rq_tail2: still to be issued), the last before its second block (rq_tail3)
  bool rq_tail2 = false, rq_tail3 = false;
  uint8_t* rq_so = nullptr;
  uint32_t rq_oa = 0, rq_ob = 0;  // byte offsets of the request's K step in the activation / weight panels
  auto rq_begin = [&]() {
    if (__builtin_expect(rq_kt == KT, 0)) {  // the tile of the request before this one is complete: its descriptors are no longer needed
      rq_kt = 0;
      rq_pos += wx;
      if (rq_pos < count) {
        rq_tile();
      } else {
        // the walk is over: the remaining requests read nothing (a descriptor without records; the loads still count,
        // so every wait of the main loop is for the same number of them)
        rdA = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, 0, 0x00020000);
        rdB = rdA;
      }
    }
    rq_so = smem + rq_stg * kStage6 + wave * 1024;
    rq_oa = (uint32_t)rq_kk * (uint32_t)kStageA6;
    rq_ob = (uint32_t)rq_kk * (uint32_t)kStageB6;
    rq_kk = (rq_kk == KT - 1) ? 0 : rq_kk + 1;
    rq_stg = (rq_stg == kNumStage6 - 1) ? 0 : rq_stg + 1;
    ++rq_kt;
  };
  auto rq_issue = [&](auto i_tag) __attribute__((always_inline)) {
    constexpr int li = decltype(i_tag)::value;
    if constexpr (li < nA) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rdA, (void __attribute__((address_space(3)))*)(rq_so + li * (NT * 16)), 16, off16,
                                               rq_oa + (uint32_t)(li * (NT * 16)), 0, 0);
    } else {
      constexpr int i = li - nA;
      // chunk i * NT + tid of the 1536: column tile 1 (KT stages further on) from chunk 768 on (a whole number of waves)
      const bool half = (i * NT + wave * 64) >= 768;
      const uint32_t ob = rq_ob + (half ? (uint32_t)KT * (uint32_t)kStageB6 + (uint32_t)(i * NT * 16 - 768 * 16) : (uint32_t)(i * NT * 16));
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rdB, (void __attribute__((address_space(3)))*)(rq_so + kStageA6 + i * (NT * 16)), 16,
                                               off16, ob, 0, 0);
    }
  };
  static_assert(kLoadsPerStep == 6, "the main loop spreads six loads per wave and step");
  auto request_next = [&]() {
    rq_begin();
    rq_issue(std::integral_constant<int, 0>{});
    rq_issue(std::integral_constant<int, 1>{});
    rq_issue(std::integral_constant<int, 2>{});
    rq_issue(std::integral_constant<int, 3>{});
    rq_issue(std::integral_constant<int, 4>{});
    rq_issue(std::integral_constant<int, 5>{});
  };

  // LDS byte addresses of part 0 of this lane's 48 bytes in stage 0: 32-row block, then lane * 16
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)smem;
  const uint32_t adrA0 = (uint32_t)((wm * 4) * kBlock6 + lane * 16);
  const uint32_t adrB0 = (uint32_t)(kStageA6 + (wn >> 1) * kStageB6 + ((wn & 1) * 2) * kBlock6 + lane * 16);

  // ---- prologue: stages 0 and 1 requested, landed and published by a barrier; stage 2 requested ----
  request_next();
  request_next();
  {
    int tm0, tn0;
    tile_of_sid(first + local, mt, nt, tm0, tn0);
    if (tid < 256) store_row_info<Acc, EPI>(a, tm0 * BM, tid, row_info);
  }
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  request_next();
  int landed = 1;  // steps from here on whose loads are known to have landed (their barrier needs no wait)
  int stg = 0;     // stage of the step about to be multiplied
  int rbuf = 0;    // row-info buffer of the current tile

  // Fragment registers.  A lane's 48 bytes of one 32-row block and K step are the two 24-byte MFMA operands of the
  // step's halves, read as three 16-byte parts.  The parts of a fragment must land in 12 CONSECUTIVE registers (the
  // first operand is registers 0..5, the second 6..11), which the register allocator does not arrange for separate
  // asm outputs (it copies parts into fresh tuples and runs out of registers); the fragments therefore live in fixed
  // registers v184..v255: two activation sets (block mi + 1 is read while block mi is multiplied) and the weights'
  // NIW = 2 blocks double-buffered from step to step.
  static_assert(NIW == 2, "fixed fragment registers are laid out for two weight blocks per wave");
  struct Frag {
    u6 h0, h1;
  };
#define STAMP_RD3(f, H0, H1, P0, P1, P2, base, off)                                                                   \
  asm volatile("ds_read_b128 " P0 ", %2 offset:%3\n\tds_read_b128 " P1 ", %2 offset:%4\n\tds_read_b128 " P2 ", %2 offset:%5" \
               : "=&{" H0 "}"(f.h0), "=&{" H1 "}"(f.h1)                                                               \
               : "v"(base), "n"(off), "n"((off) + kPart), "n"((off) + 2 * kPart))
#define STAMP_RD_AS0(base, off) STAMP_RD3(As0, "v[184:189]", "v[190:195]", "v[184:187]", "v[188:191]", "v[192:195]", base, off)
#define STAMP_RD_AS1(base, off) STAMP_RD3(As1, "v[196:201]", "v[202:207]", "v[196:199]", "v[200:203]", "v[204:207]", base, off)
  // activation block 0 and the two weight blocks of a step in one statement, parts 0 and 1 of all three first (the
  // first MFMA half's operands), then the parts 2
#define STAMP_RD9(fa, fb0, fb1, AH0, AH1, B0H0, B0H1, B1H0, B1H1, A0, A1, A2, B00_, B01_, B02_, B10_, B11_, B12_, basea, baseb)         \
  asm volatile("ds_read_b128 " A0 ", %6 offset:0\n\tds_read_b128 " A1 ", %6 offset:%8\n\t"                                          \
               "ds_read_b128 " B00_ ", %7 offset:0\n\tds_read_b128 " B01_ ", %7 offset:%8\n\t"                                      \
               "ds_read_b128 " B10_ ", %7 offset:%10\n\tds_read_b128 " B11_ ", %7 offset:%11\n\t"                                   \
               "ds_read_b128 " A2 ", %6 offset:%9\n\tds_read_b128 " B02_ ", %7 offset:%9\n\tds_read_b128 " B12_ ", %7 offset:%12"   \
               : "=&{" AH0 "}"(fa.h0), "=&{" AH1 "}"(fa.h1), "=&{" B0H0 "}"(fb0.h0), "=&{" B0H1 "}"(fb0.h1), "=&{" B1H0 "}"(fb1.h0),  \
                 "=&{" B1H1 "}"(fb1.h1)                                                                                              \
               : "v"(basea), "v"(baseb), "n"(kPart), "n"(2 * kPart), "n"(kBlock6), "n"(kBlock6 + kPart), "n"(kBlock6 + 2 * kPart))
#define STAMP_RD9_PB0(basea, baseb)                                                                                                  \
  STAMP_RD9(As0, B00, B01, "v[184:189]", "v[190:195]", "v[208:213]", "v[214:219]", "v[220:225]", "v[226:231]", "v[184:187]", "v[188:191]", \
            "v[192:195]", "v[208:211]", "v[212:215]", "v[216:219]", "v[220:223]", "v[224:227]", "v[228:231]", basea, baseb)
#define STAMP_RD9_PB1(basea, baseb)                                                                                                  \
  STAMP_RD9(As0, B10, B11, "v[184:189]", "v[190:195]", "v[232:237]", "v[238:243]", "v[244:249]", "v[250:255]", "v[184:187]", "v[188:191]", \
            "v[192:195]", "v[232:235]", "v[236:239]", "v[240:243]", "v[244:247]", "v[248:251]", "v[252:255]", basea, baseb)
  // a wait names the fragments it covers (same registers in and out), which keeps their MFMAs behind it
#define STAMP_WAIT2(cnt, x, XR, y, YR) asm volatile("s_waitcnt lgkmcnt(" #cnt ")" : "={" XR "}"(x), "={" YR "}"(y) : "0"(x), "1"(y))
#define STAMP_WAITH(cnt, x, XR) asm volatile("s_waitcnt lgkmcnt(" #cnt ")" : "={" XR "}"(x) : "0"(x))
#define STAMP_WAIT1(cnt, f, H0, H1) asm volatile("s_waitcnt lgkmcnt(" #cnt ")" : "={" H0 "}"(f.h0), "={" H1 "}"(f.h1) : "0"(f.h0), "1"(f.h1))
#define STAMP_WAIT_AS0(cnt) STAMP_WAIT1(cnt, As0, "v[184:189]", "v[190:195]")
#define STAMP_WAIT_AS1(cnt) STAMP_WAIT1(cnt, As1, "v[196:201]", "v[202:207]")

  for (int pos = local; pos < count; pos += wx) {
    int tm, tn;
    tile_of_sid(first + pos, mt, nt, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN6;
    const int nw = n0 + wn * (32 * NIW);

    v16f acc[4][NIW];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < NIW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    Frag As0, As1, B00, B01, B10, B11;  // per tile: no fragment is carried across the epilogue
    // the four MFMAs of activation block mi: both halves against both weight blocks
    auto mfma4 = [&](const Frag& A, const Frag& W0, const Frag& W1, auto mi_tag) __attribute__((always_inline)) {
      constexpr int mi = decltype(mi_tag)::value;
      acc[mi][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)A.h0), widen((v6i)W0.h0), acc[mi][0], 2, 2, 0, 0, 0, 0);
      acc[mi][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)A.h0), widen((v6i)W1.h0), acc[mi][1], 2, 2, 0, 0, 0, 0);
      acc[mi][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)A.h1), widen((v6i)W0.h1), acc[mi][0], 2, 2, 0, 0, 0, 0);
      acc[mi][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)A.h1), widen((v6i)W1.h1), acc[mi][1], 2, 2, 0, 0, 0, 0);
    };

    // Step kt (pb = 0: weights in B00, B01, the next step's go to B10, B11; pb = 1: the other way round).  On entry
    // the reads of the step's weights and of activation block 0 have been issued (by the head of the tile or by the
    // step before).  Block 1 is requested, block 0 multiplied, block 2 requested, block 1 multiplied, ...: the LDS
    // reads of a block fly under the MFMAs of the block before.  After block 2 every read of this stage has
    // returned: the wave waits for its own loads of the NEXT step's stage (the step after that may still be in
    // flight), meets the others at the workgroup barrier (next stage visible, this stage free), requests the step
    // three ahead into this stage, issues the reads of the next step's block 0 and weights, and multiplies block 3
    // under them.  One barrier per step, none between a read and its use.
    auto step = [&](auto pb_tag) __attribute__((always_inline)) {
      constexpr int pb = decltype(pb_tag)::value;
      const uint32_t sa = lds0 + (uint32_t)(stg * kStage6);
      __builtin_amdgcn_sched_barrier(0);
      STAMP_RD_AS1(sa + adrA0, 1 * kBlock6);
      // block 0: of the 12 reads in flight the first 4 feed the first MFMA, 6 the second, 8 the third, 9 the fourth
      if constexpr (pb == 0) {
        STAMP_WAIT2(8, As0.h0, "v[184:189]", B00.h0, "v[208:213]");
        acc[0][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As0.h0), widen((v6i)B00.h0), acc[0][0], 2, 2, 0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (rq_tail2) rq_issue(std::integral_constant<int, 3>{});
        __builtin_amdgcn_sched_barrier(0);
        STAMP_WAITH(6, B01.h0, "v[220:225]");
        acc[0][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As0.h0), widen((v6i)B01.h0), acc[0][1], 2, 2, 0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (rq_tail2) rq_issue(std::integral_constant<int, 4>{});
        rq_tail3 = rq_tail2;
        rq_tail2 = false;
        __builtin_amdgcn_sched_barrier(0);
        STAMP_WAIT2(4, As0.h1, "v[190:195]", B00.h1, "v[214:219]");
        acc[0][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As0.h1), widen((v6i)B00.h1), acc[0][0], 2, 2, 0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        STAMP_WAITH(3, B01.h1, "v[226:231]");
        acc[0][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As0.h1), widen((v6i)B01.h1), acc[0][1], 2, 2, 0, 0, 0, 0);
      } else {
        STAMP_WAIT2(8, As0.h0, "v[184:189]", B10.h0, "v[232:237]");
        acc[0][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As0.h0), widen((v6i)B10.h0), acc[0][0], 2, 2, 0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (rq_tail2) rq_issue(std::integral_constant<int, 3>{});
        __builtin_amdgcn_sched_barrier(0);
        STAMP_WAITH(6, B11.h0, "v[244:249]");
        acc[0][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As0.h0), widen((v6i)B11.h0), acc[0][1], 2, 2, 0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (rq_tail2) rq_issue(std::integral_constant<int, 4>{});
        rq_tail3 = rq_tail2;
        rq_tail2 = false;
        __builtin_amdgcn_sched_barrier(0);
        STAMP_WAIT2(4, As0.h1, "v[190:195]", B10.h1, "v[238:243]");
        acc[0][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As0.h1), widen((v6i)B10.h1), acc[0][0], 2, 2, 0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        STAMP_WAITH(3, B11.h1, "v[250:255]");
        acc[0][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As0.h1), widen((v6i)B11.h1), acc[0][1], 2, 2, 0, 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      STAMP_RD_AS0(sa + adrA0, 2 * kBlock6);
      if (rq_tail3) rq_issue(std::integral_constant<int, 5>{});
      STAMP_WAIT_AS1(3);
      if constexpr (pb == 0) mfma4(As1, B00, B01, std::integral_constant<int, 1>{});
      else mfma4(As1, B10, B11, std::integral_constant<int, 1>{});
      __builtin_amdgcn_sched_barrier(0);
      STAMP_RD_AS1(sa + adrA0, 3 * kBlock6);
      rq_tail3 = false;
      STAMP_WAIT_AS0(3);
      if constexpr (pb == 0) mfma4(As0, B00, B01, std::integral_constant<int, 2>{});
      else mfma4(As0, B10, B11, std::integral_constant<int, 2>{});
      __builtin_amdgcn_sched_barrier(0);
      STAMP_WAIT_AS1(0);
      // ---- the next step's stage ----
      asm volatile("" ::: "memory");
      if (landed > 0) {
        --landed;
      } else {
        __builtin_amdgcn_s_waitcnt(0x0F70 | kLoadsPerStep);  // vmcnt(one step's loads): the request of the step before may be in flight
      }
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      rq_begin();
      __builtin_amdgcn_sched_barrier(0);
      stg = (stg == kNumStage6 - 1) ? 0 : stg + 1;
      {
        // (after the tile's last step these reads fetch the next tile's first fragments, which the epilogue's
        // registers cannot keep: they are dropped and read again by the next head)
        const uint32_t sn = lds0 + (uint32_t)(stg * kStage6);
        if constexpr (pb == 0) STAMP_RD9_PB1(sn + adrA0, sn + adrB0);
        else STAMP_RD9_PB0(sn + adrA0, sn + adrB0);
      }
      __builtin_amdgcn_sched_barrier(0);
      // block 3, the request's loads spread among its MFMAs
      const Frag& W0 = pb == 0 ? B00 : B10;
      const Frag& W1 = pb == 0 ? B01 : B11;
      rq_issue(std::integral_constant<int, 0>{});
      __builtin_amdgcn_sched_barrier(0);
      acc[3][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As1.h0), widen((v6i)W0.h0), acc[3][0], 2, 2, 0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      rq_issue(std::integral_constant<int, 1>{});
      __builtin_amdgcn_sched_barrier(0);
      acc[3][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As1.h0), widen((v6i)W1.h0), acc[3][1], 2, 2, 0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      rq_issue(std::integral_constant<int, 2>{});
      __builtin_amdgcn_sched_barrier(0);
      acc[3][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As1.h1), widen((v6i)W0.h1), acc[3][0], 2, 2, 0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_sched_barrier(0);
      acc[3][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen((v6i)As1.h1), widen((v6i)W1.h1), acc[3][1], 2, 2, 0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      rq_tail2 = true;  // loads 3, 4 and 5 follow among the MFMAs of the next step (or after the tile's last step)
    };
    // head of the tile: the barrier that published its first stage lies behind (prologue, or the last step of the
    // tile before)
    {
      const uint32_t sh = lds0 + (uint32_t)(stg * kStage6);
      STAMP_RD9_PB0(sh + adrA0, sh + adrB0);
    }
    for (int kt = 0; kt + 1 < KT; kt += 2) {
      step(std::integral_constant<int, 0>{});
      step(std::integral_constant<int, 1>{});
    }
    if (KT & 1) step(std::integral_constant<int, 0>{});
    if (rq_tail2) {
      rq_issue(std::integral_constant<int, 3>{});
      rq_issue(std::integral_constant<int, 4>{});
      rq_issue(std::integral_constant<int, 5>{});
      rq_tail2 = false;
    }
    // the last step's look-ahead reads must have returned before their registers are used for anything else
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

    // Everything requested so far (the next tile's first steps included) must have landed before the epilogue issues
    // its stores: the counter retires in order, so a later wait for a load would also wait for every store before
    // it.  The epilogue waits for that itself, after its lane swaps (the plain modes: before they start); after it
    // the next two steps therefore need no wait.
    landed = 2;
    // Per-lane values of the epilogue are derived from an opaque copy of the lane number, so that they are
    // computed here, once per tile, instead of being carried in registers across the main loop (which has none
    // to spare: a spilled value would be reloaded with a wait for all outstanding loads inside that loop).
    int lane_e = lane, tid_e = tid;
    asm volatile("" : "+v"(lane_e), "+v"(tid_e));
    // the epilogue's operands from global memory: their latency passes under the lane swaps
    RegEpiOperands<EPI, (IS2D ? 2 * RB : RB)> eo;
    if constexpr (EPI >= 2) eo.request(a, m0, nw, wm, lane_e);
    // row factors of the next tile: loaded now, written to the other buffer after the epilogue (a barrier of
    // the next tile's first step publishes them long before its epilogue reads them)
    float nfac = 0.0f, nrz = 0.0f;
    int ndst = -1;
    const bool has_next = pos + wx < count;
    if (has_next && tid_e < 256) {
      int tm1, tn1;
      tile_of_sid(first + pos + wx, mt, nt, tm1, tn1);
      compute_row_info<Acc, EPI>(a, tm1 * BM, tid_e, nfac, ndst, nrz);
    }
    const uint8_t* ri = row_info + rbuf * kRowInfoBytes;
    if constexpr (EPI != 2) {
      // The loads just requested complete here, on every path and in a form the compiler's wait-count bookkeeping
      // sees: a load it believed pending at the end of the tile would make it wait for ALL loads inside the next
      // main loop.  (The fused epilogue places this wait after its lane swaps.)
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    }
    if constexpr (EPI >= 2) {
      epilogue_reg<EPI, RB, IS2D, YBF16, NI, 0, SYM>(a, acc, ri, eo, m0, nw, wm, lane_e);
    } else {
      EpiOperands<EPI, RB, IS2D> none;
      epilogue<Acc, EPI, RB, IS2D, YBF16, true>(a, acc, smem, ri, none, m0, n0, lane_e, wave, wm, wn);
    }
    rbuf ^= 1;
    if (has_next && tid_e < 256) write_row_info(row_info + rbuf * kRowInfoBytes, tid_e, nfac, ndst, nrz);
  }
}

int gemm6_workgroups(int tiles) {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
  }
  return tiles < cus ? tiles : cus;
}

template <int EPI, int RB, bool IS2D, bool YBF16, bool SYM>
hipError_t launch_k(const GemmArgs& a, hipStream_t st) {
  constexpr size_t lds = (size_t)kNumStage6 * kStage6 + 2 * kRowInfoBytes;
  static size_t lds_done[kStampMaxDevices] = {};
  hipError_t e = stamp_allow_lds(reinterpret_cast<const void*>(&k_gemm6<EPI, RB, IS2D, YBF16, SYM>), lds, lds_done);
  if (e != hipSuccess) return e;
  const int mt = (a.M + BM - 1) / BM, nt = a.Npad / BN6;
  hipLaunchKernelGGL((k_gemm6<EPI, RB, IS2D, YBF16, SYM>), dim3(gemm6_workgroups(mt * nt)), dim3(512), lds, st, a);
  return hipGetLastError();
}

template <int EPI, int RB, bool IS2D, bool YBF16>
hipError_t launch_y(const GemmArgs& a, hipStream_t st) {
  if constexpr (EPI == 2) {
    if (!a.g.asym) return launch_k<EPI, RB, IS2D, YBF16, true>(a, st);
  }
  return launch_k<EPI, RB, IS2D, YBF16, false>(a, st);
}

template <int EPI, int RB, bool IS2D>
hipError_t launch(const GemmArgs& a, hipStream_t st) {
  if constexpr (EPI >= 2) {
    if (a.g.y_bf16) return launch_y<EPI, RB, IS2D, true>(a, st);
  }
  return launch_y<EPI, RB, IS2D, false>(a, st);
}

}  // namespace

size_t stamp_a6_bytes(const stamp_plan* p) { return (size_t)(p->Mpad / 256) * (p->Kpad / 128) * kStageA6; }
size_t stamp_b6_bytes(const stamp_plan* p) { return (size_t)(p->Npad / 128) * (p->Kpad / 128) * kStageB6; }

hipError_t stamp_launch_weight_quant6(const stamp_plan* p, const float* W, const uint32_t* colmax, hipStream_t st) {
  const int d = p->geom.d, N = p->geom.N;
  const size_t sc = p->desc.w_is_out_by_in ? 1 : (size_t)N;
  const size_t sn = p->desc.w_is_out_by_in ? (size_t)d : 1;
  hipLaunchKernelGGL(k_w_quant6, dim3((p->Npad + 255) / 256, p->Kpad / 32), dim3(256), 0, st, W, colmax, p->qW6_dev, d, N,
                     p->Kpad, p->Npad, sc, sn);
  return hipGetLastError();
}

hipError_t stamp_launch_repack6(const stamp_plan* p, const uint8_t* q_lo, uint8_t* a6, hipStream_t st) {
  hipLaunchKernelGGL(k_repack6, dim3((p->Mpad / 256) * (p->Kpad / 128)), dim3(512), 0, st, q_lo, a6);
  return hipGetLastError();
}

hipError_t stamp_launch_gemm_lo6(const stamp_plan* p, const uint8_t* a6, const float* scales, int mode, void* out,
                                 const float* P, hipStream_t st, int own_top) {
  GemmArgs a = stamp_gemm_args(p, scales, out);
  a.A = a6;
  a.Bq = p->qW6_dev;
  a.M = p->geom.B * p->geom.s;
  a.P = P;
  a.own_top = (mode == 2) ? own_top : 0;
  if (mode == 0) return launch<0, 0, false>(a, st);
  if (mode == 1) return launch<1, 0, false>(a, st);
  if (mode == 3) return launch<3, 0, false>(a, st);
  if (mode != 2) return hipErrorInvalidValue;
  const StampGeom& g = p->geom;
  if (!g.is2d) {
    switch (g.r) {
      case 3: return launch<2, 3, false>(a, st);
      case 4: return launch<2, 4, false>(a, st);
      case 5: return launch<2, 5, false>(a, st);
      case 6: return launch<2, 6, false>(a, st);
      default: return hipErrorInvalidValue;
    }
  }
  switch (g.r) {
    case 2: return launch<2, 2, true>(a, st);
    case 3: return launch<2, 3, true>(a, st);
    default: return hipErrorInvalidValue;
  }
}
