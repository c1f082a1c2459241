// Activation path of the STaMP linear layer on gfx950: T = L X along the tokens (Haar DWT, paper
// section "Efficient Energy Concentration"), per-token scale and rounding to 8- or 4-bit codes
// (Background Eq. 1, in its symmetric absmax form or in full with min-max range and integer offset;
// two-level allocation of section "Optimal bit allocation").  X is read from HBM once and the
// transformed activation never goes to HBM.
//
// Floating-point contract (decides the integer codes, so it is fixed): every coefficient is the
// difference (or sum) of two block sums built by plain pairwise fp32 adds, multiplied once by
// norm(l) = fl(2^(-l/2)); absmax a over the row; scale = a / qmax; inv = qmax / a (IEEE
// divisions); code = rne(fl(T * inv)).  Asymmetric form: hi = max T, nlo = max -T = -min T (the token's own
// range, whether or not it contains 0), range = hi + nlo (a token with max = min: range = |hi|), scale =
// range / qmax, inv = qmax / range with qmax = 2^b - 1, z = rne(fl(nlo * inv)) (any integer), code =
// clamp(rne(fl(T * inv)) + z, 0, qmax), stored as code - 2^(b-1).  This file is compiled with
// -ffp-contract=off.
//
// Kernels:
//   k_bottom1d / k_bottom2d  one workgroup per (sequence, block of R tokens), all d_in channels;
//                            each thread owns 8 channels for every token of the block, so the
//                            butterflies stay in registers; only the per-row absmax crosses lanes
//                            (DPP inside a wave, per-wave partial maxima in LDS across waves).  Emits the R-1
//                            4-bit rows of the block and the block sum (fp32, to scratch).
//   k_top                    the remaining levels over the k_hi block sums, in LDS, per channel
//                            slice; writes the normalised 8-bit-row coefficients to scratch and
//                            one partial absmax per (row, slice).
//   k_quant_hi               reduces the partial maxima of a row and rounds the row to int8.
#include <utility>

#include "stamp_internal.h"

namespace {

typedef uint32_t u4 __attribute__((ext_vector_type(4)));

constexpr float kInvSqrt2 = 0.70710678118654752440f;  // 0x3F3504F3
constexpr float kMagicLo = 12582920.0f;               // 1.5 * 2^23 + 8: fp32 add rounds to integer (RNE), low 4 bits = code + 8
constexpr uint32_t kMagicLoBits = 0x4B400000u;        // bit pattern of 1.5 * 2^23
constexpr uint32_t kPackBias = kMagicLoBits * 0x11111111u;  // sum over 8 nibble positions of the pattern's high bits (mod 2^32)

__device__ __forceinline__ float haar_norm(int level) {
  // 2^(-level/2): a power of two for even levels, fl(1/sqrt 2) times a power of two for odd ones
  return ldexpf((level & 1) ? kInvSqrt2 : 1.0f, -(level >> 1));
}

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// unsigned max over the 64 lanes (bit patterns of non-negative floats, or order keys of any floats);
// result is wave-uniform
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
  uint32_t y;
  y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false);  // quad_perm [1,0,3,2]
  x = max(x, y);
  y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, false);  // quad_perm [2,3,0,1]
  x = max(x, y);
  y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, false);  // row_half_mirror
  x = max(x, y);
  y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xF, 0xF, false);  // row_mirror
  x = max(x, y);
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0);
  const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32);
  const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
  return max(max(a, b), max(c, d));
}

// Order key of a float of either sign: a < b as floats  <=>  key(a) < key(b) as unsigned integers
// (negative: all bits flipped, otherwise the sign bit set).  0 is below the key of every number, so it is
// the neutral element of an unsigned max.  The asymmetric quantizer reduces max T and max -T in this form.
__device__ __forceinline__ uint32_t fkey(float f) {
  const uint32_t b = __float_as_uint(f);
  return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float fkey_inv(uint32_t k) {
  return __uint_as_float(k ^ ((uint32_t)((int32_t)~k >> 31) | 0x80000000u));
}

__device__ __forceinline__ uint32_t absbits(float f) { return __float_as_uint(f) & 0x7FFFFFFFu; }

__device__ __forceinline__ uint32_t row_absmax_bits(const float (&v)[8]) {
  float m = fmaxf(fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3]))),
                  fmaxf(fmaxf(fabsf(v[4]), fabsf(v[5])), fmaxf(fabsf(v[6]), fabsf(v[7]))));
  return __float_as_uint(m);
}

// 8 codes -> one dword of two's complement nibbles (channel c in nibble c).
// p[c] = T * inv, |p| <= 7 (+1 ulp).  fl(p + magic) has rne(p) + 8 in its low 4 bits.
__device__ __forceinline__ uint32_t pack8_int4(const float (&p)[8]) {
  uint32_t acc = __float_as_uint(__fadd_rn(p[7], kMagicLo));
#pragma unroll
  for (int c = 6; c >= 0; --c) acc = (acc << 4) + __float_as_uint(__fadd_rn(p[c], kMagicLo));
  return (acc - kPackBias) ^ 0x88888888u;
}

// Asymmetric form: p already clamped to [-z, 15 - z]; the nibble to store is that of q - 8 with
// q = rne(p) + z.  The addend must be EVEN, or a tie p = n + 1/2 would be broken by the parity of the sum
// instead of that of n: magic = 1.5 * 2^23 + 16 + (z - z % 2) puts rne(p) + z - z % 2 + 16 (15..31) into
// the low bits; the 16s and the constant pattern bits leave with the bias, z % 2 is added to all eight
// nibbles at once (no nibble exceeds 31 - 16 = 15), and the final XOR turns q into q - 8.
__device__ __forceinline__ uint32_t pack8_uint4(const float (&p)[8], float z) {
  const float zodd = z - 2.0f * floorf(0.5f * z);
  const float magic = __fadd_rn(12582928.0f, z - zodd);  // 1.5 * 2^23 + 16 + even part of z
  uint32_t acc = __float_as_uint(__fadd_rn(p[7], magic));
#pragma unroll
  for (int c = 6; c >= 0; --c) acc = (acc << 4) + __float_as_uint(__fadd_rn(p[c], magic));
  return ((acc - (kPackBias + 0x11111110u)) + (zodd != 0.0f ? 0x11111111u : 0u)) ^ 0x88888888u;
}

// max over the 8 values of v and of -v, as order keys
__device__ __forceinline__ void row_posneg_bits(const float (&v)[8], uint32_t& pos, uint32_t& neg) {
  float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
  float mn = fminf(fminf(fminf(v[0], v[1]), fminf(v[2], v[3])), fminf(fminf(v[4], v[5]), fminf(v[6], v[7])));
  pos = fkey(mx);
  neg = fkey(-mn);
}

// range, scale, reciprocal and offset of one token from hi = max T and nlo = max -T, qmax = 2^b - 1
__device__ __forceinline__ void asym_params(float hi, float nlo, float qmax, float& scale, float& inv, float& z) {
  float range = __fadd_rn(hi, nlo);
  if (range == 0.0f) range = fabsf(hi);  // max = min: the token is reproduced through range = |value|
  scale = 0.0f;
  inv = 0.0f;
  if (range > 0.0f) {
    scale = __fdiv_rn(range, qmax);
    inv = __fdiv_rn(qmax, range);
  }
  z = rintf(__fmul_rn(nlo, inv));
}

__device__ __forceinline__ void load8(const void* X, size_t elem_off, bool bf16, bool active, float (&v)[8]) {
  if (!active) {
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = 0.0f;
    return;
  }
  if (bf16) {
    const uint4 w = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(X) + elem_off);
    v[0] = bf16lo(w.x); v[1] = bf16hi(w.x); v[2] = bf16lo(w.y); v[3] = bf16hi(w.y);
    v[4] = bf16lo(w.z); v[5] = bf16hi(w.z); v[6] = bf16lo(w.w); v[7] = bf16hi(w.w);
  } else {
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(X) + elem_off);
    const float4 a = p[0], b = p[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
}

constexpr int trailing_ones(int x) { int n = 0; while (x & 1) { ++n; x >>= 1; } return n; }
constexpr int cmin(int a, int b) { return a < b ? a : b; }

// Shared tail of one streaming step: NR finished rows (unnormalised values rowv[r][0..7], level
// and in-block position given per row) are reduced over the workgroup, scaled, rounded, packed and
// stored.  `step` numbers the steps of this workgroup (rotating LDS buffers).
struct RowMeta { int level; int e; };
constexpr int kMaxRows = 18;  // most rows finished by one streaming step (2-D: 12 + 3 + 3)
constexpr int kPartWords = 2 * kMaxRows * 16;  // per-wave partial maxima of one step: [2 signs][row][wave]

// Channel split.  A workgroup covers at most 1024 (1-D) / 512 (2-D) threads x 8 channels; wider layers
// are split over blockIdx.z and run in two passes, because a row's range spans all channels:
//   PASS 1  transform, reduce each row over the workgroup's channels, write the partial maxima
//           gpart[sign][split][B*s] (no codes);
//   PASS 2  transform again, take each row's maximum over the splits from LDS (s_amax[sign][e], filled
//           from gpart before the first step), quantize and store.
//   PASS 0  is the single-pass kernel (one workgroup sees all channels).
struct SplitArgs {
  uint32_t* gpart;     // partial row maxima (bit patterns), PASS 1 writes / PASS 2 reads
  size_t part_rows;    // B * s
  int nsplit;
  int c_split;         // channels per split (a multiple of 8)
  int8_t* q_hi;        // non-null: the plan has no top levels (L = 0), so the block sum is itself a finished
  int khi;             // coefficient and the bottom kernel quantizes it (8 bits for blocks < khi, else 4)
};
constexpr int kMaxBlockRows = 128;

// ASYM: the asymmetric form of the quantizer; zeros_off = distance (in floats) from a row's scale to its offset z.
template <int NR, bool IS2D, bool ASYM, int PASS, typename MetaFn>
__device__ __forceinline__ void flush_rows(float (&rowv)[NR][8], MetaFn meta, int step, uint32_t (*s_max)[kPartWords],
                                           uint8_t* q_lo_blk /* row e=0 of the block, channel 0 (workgroup-uniform) */,
                                           uint32_t q_off /* this thread's byte offset inside a row */,
                                           float* scales_blk, size_t zeros_off, bool active, int tid,
                                           uint32_t* gpart_blk /* PASS 1: this split's partial maxima of the block's row e=0 */,
                                           size_t gpart_neg /* PASS 1: distance to the negative parts */,
                                           const uint32_t* s_amax /* PASS 2: [2][kMaxBlockRows] */, bool write_scales) {
  // Values derived from the thread index are recomputed in every step from an opaque copy: cheap, and it
  // keeps them from being carried (and spilled: a scratch reload waits for ALL outstanding memory
  // operations, the asynchronous loads of the next batches included) across the whole unrolled kernel.
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = tid >> 6;
  // [row][wave] partial maxima, double buffered; asymmetric: a second array for the negative parts
  uint32_t* part = &s_max[0][0] + (step & 1) * kPartWords;
  uint32_t* part_neg = part + kMaxRows * 16;
  if constexpr (PASS != 2) {
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    if constexpr (ASYM) {
      uint32_t pos, neg;
      row_posneg_bits(rowv[r], pos, neg);
      if (!active) pos = neg = 0u;  // lanes beyond the last channel hold zeros, which are not part of the token
      pos = wave_max_u32(pos);
      neg = wave_max_u32(neg);
      if (lane == 0) { part[r * 16 + wave] = pos; part_neg[r * 16 + wave] = neg; }
    } else {
      const uint32_t m = wave_max_u32(row_absmax_bits(rowv[r]));
      if (lane == 0) part[r * 16 + wave] = m;
    }
  }
  // Workgroup barrier that waits for this wave's LDS traffic only: __syncthreads() would also wait for
  // the global -> LDS loads of the next batch, which are meant to stay in flight across it.
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  }
  // lane r prepares row r: a = fl(absmaxU * norm); scale = a / 7; inv = 7 / a
  // (asymmetric: hi = fl(max t * norm), nlo = fl(max -t * norm), then asym_params with qmax = 15)
  float mul_lane = 0.0f;
  [[maybe_unused]] float z_lane = 0.0f;
  {
    const int r = lane < NR ? lane : 0;
    const RowMeta rm = meta(r);
    const int nw = (int)(blockDim.x >> 6);
    // The partial maxima are read by hand-written LDS reads: the compiler cannot tell this array from the
    // staging buffer that the asynchronous global -> LDS loads of the NEXT batches are writing, and would
    // make every ordinary LDS read here wait for all of them (vmcnt(0)), i.e. serialise memory and compute.
    auto reduce_waves = [&](const uint32_t* arr) {
      if constexpr (PASS == 2) {
        // the row's maximum over all channels, reduced before the first step
        const uint32_t adr1 = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) uint32_t*)(
            s_amax + (arr == part ? 0 : kMaxBlockRows) + rm.e);
        uint32_t bits;
        asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(bits) : "v"(adr1) : "memory");
        return bits;
      }
      const uint32_t adr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) uint32_t*)(arr + r * 16);
      u4 v0, v1, v2, v3;
      asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:16\n\tds_read_b128 %2, %4 offset:32\n\t"
                   "ds_read_b128 %3, %4 offset:48\n\ts_waitcnt lgkmcnt(0)"
                   : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
                   : "v"(adr)
                   : "memory");
      const u4 vv[4] = {v0, v1, v2, v3};
      uint32_t mbits = 0u;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (4 * q + 0 < nw) mbits = max(mbits, vv[q].x);
        if (4 * q + 1 < nw) mbits = max(mbits, vv[q].y);
        if (4 * q + 2 < nw) mbits = max(mbits, vv[q].z);
        if (4 * q + 3 < nw) mbits = max(mbits, vv[q].w);
      }
      return mbits;
    };
    if constexpr (PASS == 1) {
      const uint32_t mpos = reduce_waves(part);
      if (tid < NR) gpart_blk[rm.e] = mpos;
      if constexpr (ASYM) {
        const uint32_t mneg = reduce_waves(part_neg);
        if (tid < NR) gpart_blk[gpart_neg + rm.e] = mneg;
      }
      return;
    }
    const float nrm = IS2D ? ldexpf(1.0f, -rm.level) : haar_norm(rm.level);
    float scale = 0.0f, inv = 0.0f;
    if constexpr (ASYM) {
      const float hi = __fmul_rn(fkey_inv(reduce_waves(part)), nrm), nlo = __fmul_rn(fkey_inv(reduce_waves(part_neg)), nrm);
      asym_params(hi, nlo, 15.0f, scale, inv, z_lane);
      if (tid < NR && write_scales) scales_blk[zeros_off + rm.e] = z_lane;
    } else {
      const float a = __fmul_rn(__uint_as_float(reduce_waves(part)), nrm);
      if (a > 0.0f) {
        scale = __fdiv_rn(a, 7.0f);
        inv = __fdiv_rn(7.0f, a);
      }
    }
    // even 1-D levels and all 2-D levels have a power-of-two norm: fold it into the multiplier
    const bool fold = IS2D || ((rm.level & 1) == 0);
    mul_lane = fold ? __fmul_rn(inv, nrm) : inv;
    if (tid < NR && write_scales) scales_blk[rm.e] = scale;
  }
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const RowMeta rm = meta(r);  // r is a compile-time constant here
    const float mul = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mul_lane), r));
    float p[8];
    const bool fold = IS2D || ((rm.level & 1) == 0);
    if (fold) {
#pragma unroll
      for (int c = 0; c < 8; ++c) p[c] = __fmul_rn(rowv[r][c], mul);
    } else {
      const float nrm = haar_norm(rm.level);
#pragma unroll
      for (int c = 0; c < 8; ++c) p[c] = __fmul_rn(__fmul_rn(rowv[r][c], nrm), mul);
    }
    uint32_t w;
    if constexpr (ASYM) {
      const float z = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, z_lane), r));
      const float lo = -z, hi = 15.0f - z;  // clamp before rounding = clamp after it (integer bounds)
#pragma unroll
      for (int c = 0; c < 8; ++c) p[c] = __builtin_amdgcn_fmed3f(p[c], lo, hi);
      w = pack8_uint4(p, z);
    } else {
      w = pack8_int4(p);
    }
    if (active) *reinterpret_cast<uint32_t*>(q_lo_blk + rm.e * 64 + q_off) = w;  // tiled layout: 64 bytes per row and K step
  }
}

// Plans without top levels: the block sum, times the norm of the blocks' level, is STaMP slot j.  The whole
// workgroup reduces its range over the channels and quantizes it like any other top row: 8 bits for the first
// khi slots, 4-bit codes held as int8 beyond.  Called after the last streaming step (no loads in flight).
// The 4-bit ones also go, packed like every other 4-bit row, to the block's row 0 of q_lo (q_lo_row: this thread's
// word of it), which no other coefficient uses: the 4-bit rows' GEMM can then take the block sum from its own rows.
template <bool IS2D, bool ASYM>
__device__ __forceinline__ void finish_top_row(const float (&top)[8], int level, uint32_t* part /* >= 32 words, free */,
                                               int8_t* q_hi_row, uint8_t* q_lo_row, float* scale_out, size_t zeros_off,
                                               bool row8, bool active, int tid) {
  const int lane = tid & 63, wave = tid >> 6, nw = (int)(blockDim.x >> 6);
  const float nrm = IS2D ? ldexpf(1.0f, -level) : haar_norm(level);
  float t[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) t[c] = __fmul_rn(top[c], nrm);
  uint32_t pos, neg = 0u;
  if constexpr (ASYM) {
    row_posneg_bits(t, pos, neg);
    if (!active) pos = neg = 0u;
  } else {
    pos = row_absmax_bits(t);
  }
  pos = wave_max_u32(pos);
  neg = wave_max_u32(neg);
  if (lane == 0) { part[wave] = pos; part[16 + wave] = neg; }
  __syncthreads();
  uint32_t mp = 0u, mn = 0u;
  for (int i = 0; i < nw; ++i) { mp = max(mp, part[i]); mn = max(mn, part[16 + i]); }
  const float qmax = ASYM ? (row8 ? 255.0f : 15.0f) : (row8 ? 127.0f : 7.0f);
  float scale = 0.0f, inv = 0.0f, z = 0.0f;
  if constexpr (ASYM) {
    asym_params(fkey_inv(mp), fkey_inv(mn), qmax, scale, inv, z);
  } else {
    const float a = __uint_as_float(mp);
    if (a > 0.0f) {
      scale = __fdiv_rn(a, qmax);
      inv = __fdiv_rn(qmax, a);
    }
  }
  if (tid == 0) {
    scale_out[0] = scale;
    if constexpr (ASYM) scale_out[zeros_off] = z;
  }
  const float qlo = ASYM ? 0.0f : -qmax, qhi = qmax, shift = ASYM ? (row8 ? 128.0f : 8.0f) : 0.0f;
  uint32_t w[2] = {0u, 0u}, w4 = 0u;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float q = __fadd_rn(rintf(__fmul_rn(t[i], inv)), z);
    q = fminf(fmaxf(q, qlo), qhi) - shift;
    w[i >> 2] |= ((uint32_t)((int)q) & 0xFFu) << (8 * (i & 3));
    w4 |= ((uint32_t)((int)q) & 0xFu) << (4 * i);
  }
  if (active) {
    *reinterpret_cast<uint2*>(q_hi_row) = make_uint2(w[0], w[1]);
    if (!row8) *reinterpret_cast<uint32_t*>(q_lo_row) = w4;
  }
}

// ------------------------------------------------------------------------------------------
// 1-D bottom kernel
// ------------------------------------------------------------------------------------------
// level and in-block position of row r finished by streaming step IT (4 tokens) of a 1-D block of
// 2^RLOG tokens: rows 0,1 = level-1 differences, row 2 = level 2, row r >= 3 = level r (carry chain)
template <int RLOG, int IT>
__device__ __forceinline__ RowMeta meta1d(int r) {
  constexpr int R = 1 << RLOG;
  RowMeta m;
  if (r < 2) { m.level = 1; m.e = (R >> 1) + 2 * IT + r; }
  else if (r == 2) { m.level = 2; m.e = (R >> 2) + IT; }
  else { m.level = r; m.e = (R >> r) + (IT >> (r - 2)); }
  return m;
}

// The block's token rows are streamed through an LDS staging buffer by asynchronous global -> LDS
// loads (no registers are held while they are in flight): the buffer holds two batches of 4 token
// rows; batch IT+2 is requested as soon as batch IT has been read out of its half into registers,
// so two batches are always in flight or ready.  Every lane reads back exactly the 16-byte chunks it
// requested, so no barrier guards the buffer, only this wave's own vmcnt.
// Layout of one half: chunk (t, h) of thread tid at ((t * CPR + h) * nthreads + tid) * 16, CPR =
// 16-byte chunks per thread and row (1 for bf16, 2 for fp32).
template <bool BF16>
__device__ __forceinline__ void request_batch(const uint8_t* X_row /* row 0 of the batch, channel 0 (workgroup-uniform) */,
                                              uint32_t x_off /* byte offset of this thread's 8 channels in a row */,
                                              size_t row_bytes, uint8_t* half, int nthreads, int wave) {
  constexpr int CPR = BF16 ? 1 : 2;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int h = 0; h < CPR; ++h)
      __builtin_amdgcn_global_load_lds(
          (const void __attribute__((address_space(1)))*)(X_row + (size_t)t * row_bytes + 16 * h + x_off),
          (void __attribute__((address_space(3)))*)(half + ((t * CPR + h) * nthreads + wave * 64) * 16), 16, 0, 0);
}

template <int RLOG, int L, int IDX, int SLOT, int NP, int MAXR>
__device__ __forceinline__ void chain1d(float (&cur)[8], float (&pend)[NP][8], float (&rowv)[MAXR][8], float (&top)[8]) {
  if constexpr (L == RLOG) {
#pragma unroll
    for (int c = 0; c < 8; ++c) top[c] = cur[c];
  } else if constexpr ((IDX & 1) != 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float a = __fadd_rn(pend[L - 2][c], cur[c]);
      rowv[SLOT][c] = __fsub_rn(pend[L - 2][c], cur[c]);
      cur[c] = a;
    }
    chain1d<RLOG, L + 1, (IDX >> 1), SLOT + 1, NP, MAXR>(cur, pend, rowv, top);
  } else {
#pragma unroll
    for (int c = 0; c < 8; ++c) pend[L - 2][c] = cur[c];
  }
}

template <int RLOG, bool BF16, bool ASYM, int PASS, int IT, int NP>
__device__ __forceinline__ void step1d(const uint8_t* X_blk, uint32_t x_off, size_t row_bytes, uint8_t* stage, int nthreads,
                                       bool active, int tid, float (&pend)[NP][8], float (&top)[8],
                                       uint32_t (*s_max)[kPartWords], uint8_t* q_lo_blk, uint32_t q_off, float* scales_blk,
                                       size_t zeros_off, uint32_t* gpart_blk, size_t gpart_neg, const uint32_t* s_amax,
                                       bool write_scales) {
  constexpr int R = 1 << RLOG;
  constexpr int NIT = R / 4;
  constexpr int CH = cmin(trailing_ones(IT), RLOG - 2);
  constexpr int NR = 3 + CH;
  constexpr int CPR = BF16 ? 1 : 2;
  uint8_t* half = stage + (IT & 1) * (4 * CPR * nthreads * 16);
  // Wait until this wave's loads of batch IT have landed: everything requested after it (batch IT+1:
  // 4 * CPR loads) may stay in flight.  Stores issued since also count, so this can only over-wait.
  asm volatile("" ::: "memory");
  if constexpr (IT + 1 < NIT) __builtin_amdgcn_s_waitcnt(0x0F70 | (4 * CPR));  // vmcnt(4 * CPR)
  else __builtin_amdgcn_s_waitcnt(0x0F70);                                      // vmcnt(0)
  asm volatile("" ::: "memory");
  u4 raw[4][CPR];
  {
    int tid_l = tid;
    asm volatile("" : "+v"(tid_l));  // see flush_rows: recomputed, not carried
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int h = 0; h < CPR; ++h)
        raw[t][h] = *reinterpret_cast<const u4*>(half + ((t * CPR + h) * nthreads + tid_l) * 16);
  }
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the half has been read before it is requested again
  asm volatile("" ::: "memory");
  if constexpr (IT + 2 < NIT)
    request_batch<BF16>(X_blk + (size_t)(4 * (IT + 2)) * row_bytes, x_off, row_bytes, half, nthreads, tid >> 6);

  float rowv[NR][8];
  float a1[2][8];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    float x0[8], x1[8];
    const int t = 2 * u;
    if constexpr (BF16) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        x0[2 * w] = bf16lo(raw[t][0][w]);
        x0[2 * w + 1] = bf16hi(raw[t][0][w]);
        x1[2 * w] = bf16lo(raw[t + 1][0][w]);
        x1[2 * w + 1] = bf16hi(raw[t + 1][0][w]);
      }
    } else {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        x0[w] = __uint_as_float(raw[t][0][w]);
        x0[4 + w] = __uint_as_float(raw[t][CPR - 1][w]);
        x1[w] = __uint_as_float(raw[t + 1][0][w]);
        x1[4 + w] = __uint_as_float(raw[t + 1][CPR - 1][w]);
      }
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      a1[u][c] = __fadd_rn(x0[c], x1[c]);
      rowv[u][c] = __fsub_rn(x0[c], x1[c]);
    }
  }
  float cur[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    cur[c] = __fadd_rn(a1[0][c], a1[1][c]);
    rowv[2][c] = __fsub_rn(a1[0][c], a1[1][c]);
  }
  chain1d<RLOG, 2, IT, 3, NP, NR>(cur, pend, rowv, top);
  auto meta = [](int r) -> RowMeta { return meta1d<RLOG, IT>(r); };
  flush_rows<NR, false, ASYM, PASS>(rowv, meta, IT, s_max, q_lo_blk, q_off, scales_blk, zeros_off, active, tid, gpart_blk,
                                    gpart_neg, s_amax, write_scales);
}

template <int RLOG, bool BF16, bool ASYM, int PASS, int NP, int... ITS>
__device__ __forceinline__ void run1d(std::integer_sequence<int, ITS...>, const uint8_t* X_blk, uint32_t x_off,
                                      size_t row_bytes, uint8_t* stage, int nthreads, bool active, int tid,
                                      float (&pend)[NP][8], float (&top)[8], uint32_t (*s_max)[kPartWords],
                                      uint8_t* q_lo_blk, uint32_t q_off, float* scales_blk, size_t zeros_off,
                                      uint32_t* gpart_blk, size_t gpart_neg, const uint32_t* s_amax, bool write_scales) {
  (step1d<RLOG, BF16, ASYM, PASS, ITS, NP>(X_blk, x_off, row_bytes, stage, nthreads, active, tid, pend, top, s_max, q_lo_blk,
                                           q_off, scales_blk, zeros_off, gpart_blk, gpart_neg, s_amax, write_scales), ...);
}

// PASS 2: every row's maximum over the splits -> s_amax[sign][e] (before the first step; ordinary loads)
template <bool ASYM>
__device__ __forceinline__ void gather_row_maxima(const SplitArgs& sp, size_t row0, int R, int tid, uint32_t* s_amax) {
  if (tid < R) {
    uint32_t mpos = 0u, mneg = 0u;
    for (int q = 0; q < sp.nsplit; ++q) {
      mpos = max(mpos, sp.gpart[(size_t)q * sp.part_rows + row0 + tid]);
      if constexpr (ASYM) mneg = max(mneg, sp.gpart[((size_t)sp.nsplit + q) * sp.part_rows + row0 + tid]);
    }
    s_amax[tid] = mpos;
    s_amax[kMaxBlockRows + tid] = mneg;
  }
  __syncthreads();
}

template <int RLOG, bool BF16, bool ASYM, int PASS>
__global__ __launch_bounds__(1024) void k_bottom1d(const void* __restrict__ X, uint8_t* __restrict__ q_lo,
                                                   float* __restrict__ scales, float* __restrict__ abot, int s, int d,
                                                   int k, int Kpad, size_t zeros_off, SplitArgs sp) {
  constexpr int R = 1 << RLOG;
  constexpr int NP = RLOG > 2 ? RLOG - 2 : 1;
  constexpr int CPR = BF16 ? 1 : 2;
  extern __shared__ __attribute__((aligned(16))) uint8_t stage[];  // 2 halves x 4 rows x nthreads x (16 | 32) bytes
  __shared__ __attribute__((aligned(16))) uint32_t s_max[2][kPartWords];
  __shared__ uint32_t s_amax[PASS == 2 ? 2 * kMaxBlockRows : 1];
  const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int nthreads = blockDim.x;
  // channels of this workgroup: [c_lo, c_hi)
  const int c_lo = (PASS == 0) ? 0 : (int)blockIdx.z * sp.c_split;
  const int c_hi = (PASS == 0) ? d : min(d, c_lo + sp.c_split);
  const int c0 = c_lo + tid * 8;
  const bool active = c0 < c_hi;
  const size_t esz = BF16 ? 2 : 4;
  const size_t row0 = (size_t)b * s + (size_t)j * R;
  if constexpr (PASS == 2) gather_row_maxima<ASYM>(sp, row0, R, tid, s_amax);
  // threads beyond d_in / 8 (the workgroup is a whole number of waves) redo the last channel group:
  // duplicates cannot change a row maximum, and they store nothing
  // addresses = workgroup-uniform base + a 32-bit per-thread offset (keeps the per-thread state small)
  const uint8_t* X_blk = reinterpret_cast<const uint8_t*>(X) + row0 * d * esz;
  const uint32_t x_off = (uint32_t)(min(c0, c_hi - 8) * (int)esz);
  const uint32_t q_off = (uint32_t)(stamp_qlo_offset(0, min(c0, c_hi - 8), Kpad));
  const size_t row_bytes = (size_t)d * esz;
  request_batch<BF16>(X_blk, x_off, row_bytes, stage, nthreads, tid >> 6);
  if (R > 4) request_batch<BF16>(X_blk + 4 * row_bytes, x_off, row_bytes, stage + 4 * CPR * nthreads * 16, nthreads, tid >> 6);
  float pend[NP][8];
  float top[8];
  uint32_t* gpart_blk = (PASS == 1) ? sp.gpart + (size_t)blockIdx.z * sp.part_rows + row0 : nullptr;
  run1d<RLOG, BF16, ASYM, PASS, NP>(std::make_integer_sequence<int, R / 4>{}, X_blk, x_off, row_bytes, stage, nthreads, active,
                                    tid, pend, top, s_max, q_lo + stamp_qlo_offset(row0, 0, Kpad), q_off, scales + row0,
                                    zeros_off, gpart_blk, (size_t)sp.nsplit * sp.part_rows, s_amax,
                                    PASS == 0 || blockIdx.z == 0);
  if constexpr (PASS == 0) {
    if (sp.q_hi != nullptr) {
      // s_max[R/4 & 1] was last used two steps ago: every thread has passed a barrier since
      finish_top_row<false, ASYM>(top, RLOG, &s_max[(R / 4) & 1][0], sp.q_hi + ((size_t)b * k + j) * d + c0,
                                  q_lo + stamp_qlo_offset(row0, 0, Kpad) + q_off, scales + row0, zeros_off, j < sp.khi, active, tid);
      return;
    }
  }
  if (active && PASS != 1) {
    float4* o = reinterpret_cast<float4*>(abot + ((size_t)b * k + j) * d + c0);
    o[0] = make_float4(top[0], top[1], top[2], top[3]);
    o[1] = make_float4(top[4], top[5], top[6], top[7]);
  }
}

// ------------------------------------------------------------------------------------------
// 2-D bottom kernel: block of g x g tokens (g = 2^RLOG, RLOG in {2,3}), streamed in 4x4 sub-blocks
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void cell2d(const float (&p)[8], const float (&q)[8], const float (&u)[8], const float (&v)[8],
                                       float (&LL)[8], float (&W)[8], float (&H)[8], float (&D)[8]) {
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const float t0 = __fadd_rn(p[c], q[c]);
    const float t1 = __fsub_rn(p[c], q[c]);
    const float t2 = __fadd_rn(u[c], v[c]);
    const float t3 = __fsub_rn(u[c], v[c]);
    LL[c] = __fadd_rn(t0, t2);
    W[c] = __fadd_rn(t1, t3);
    H[c] = __fsub_rn(t0, t2);
    D[c] = __fsub_rn(t1, t3);
  }
}

template <int RLOG, bool BF16, bool ASYM, int PASS, int SB>
__device__ __forceinline__ void step2d(const void* X, size_t blk_elem_off, int gridW, int d, int c0, bool active, int tid,
                                       float (&pend)[4][8], float (&top)[8], uint32_t (*s_max)[kPartWords],
                                       uint8_t* q_lo_blk, uint32_t q_off, float* scales_blk, size_t zeros_off,
                                       uint32_t* gpart_blk, size_t gpart_neg, const uint32_t* s_amax, bool write_scales) {
  constexpr int g = 1 << RLOG;
  constexpr int sby = (g == 4) ? 0 : (SB >> 1), sbx = (g == 4) ? 0 : (SB & 1);
  constexpr bool LAST = (g == 8) && (SB == 3);
  constexpr int NR = LAST ? 18 : 15;
  float rowv[NR][8];
  float ll1[4][8];
  // all 16 tokens of the sub-block are requested before the first cell is computed (one memory latency per
  // sub-block instead of one per cell); the raw words give way to finished rows as the cells are consumed
  constexpr int WPT = BF16 ? 1 : 2;  // 16-byte words per token and thread
  uint4 raw[16][WPT];
#pragma unroll
  for (int tkn = 0; tkn < 16; ++tkn) {
    const int ci = tkn >> 2, q = tkn & 3;
    const int y = 4 * sby + 2 * (ci >> 1) + (q >> 1), x = 4 * sbx + 2 * (ci & 1) + (q & 1);
    const size_t eoff = blk_elem_off + ((size_t)y * gridW + x) * d;
#pragma unroll
    for (int h = 0; h < WPT; ++h) {
      if (active) {
        raw[tkn][h] = BF16 ? *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(X) + eoff)
                           : *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(X) + eoff + 4 * h);
      } else {
        raw[tkn][h] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
  }
#pragma unroll
  for (int ci = 0; ci < 4; ++ci) {
    float t[4][8];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint4 w0 = raw[4 * ci + q][0];
      if constexpr (BF16) {
        t[q][0] = bf16lo(w0.x); t[q][1] = bf16hi(w0.x); t[q][2] = bf16lo(w0.y); t[q][3] = bf16hi(w0.y);
        t[q][4] = bf16lo(w0.z); t[q][5] = bf16hi(w0.z); t[q][6] = bf16lo(w0.w); t[q][7] = bf16hi(w0.w);
      } else {
        const uint4 w1 = raw[4 * ci + q][WPT - 1];
        t[q][0] = __uint_as_float(w0.x); t[q][1] = __uint_as_float(w0.y); t[q][2] = __uint_as_float(w0.z);
        t[q][3] = __uint_as_float(w0.w); t[q][4] = __uint_as_float(w1.x); t[q][5] = __uint_as_float(w1.y);
        t[q][6] = __uint_as_float(w1.z); t[q][7] = __uint_as_float(w1.w);
      }
    }
    cell2d(t[0], t[1], t[2], t[3], ll1[ci], rowv[3 * ci + 0], rowv[3 * ci + 1], rowv[3 * ci + 2]);
  }
  float ll2[8];
  cell2d(ll1[0], ll1[1], ll1[2], ll1[3], ll2, rowv[12], rowv[13], rowv[14]);
  if constexpr (g == 4) {
#pragma unroll
    for (int c = 0; c < 8; ++c) top[c] = ll2[c];
  } else if constexpr (LAST) {
    cell2d(pend[0], pend[1], pend[2], ll2, top, rowv[15], rowv[16], rowv[17]);
  } else {
#pragma unroll
    for (int c = 0; c < 8; ++c) pend[SB][c] = ll2[c];
  }
  auto meta = [](int r) -> RowMeta {
    RowMeta m;
    if (r < 12) {
      const int ci = r / 3, bd = r - 3 * ci;
      constexpr int g1 = g >> 1;
      m.level = 1;
      m.e = g1 * g1 * (1 + bd) + (2 * sby + (ci >> 1)) * g1 + (2 * sbx + (ci & 1));
    } else if (r < 15) {
      constexpr int g2 = g >> 2;
      m.level = 2;
      m.e = g2 * g2 * (1 + (r - 12)) + sby * g2 + sbx;
    } else {
      m.level = 3;
      m.e = 1 + (r - 15);
    }
    return m;
  };
  flush_rows<NR, true, ASYM, PASS>(rowv, meta, SB, s_max, q_lo_blk, q_off, scales_blk, zeros_off, active, tid, gpart_blk,
                                   gpart_neg, s_amax, write_scales);
}

template <int RLOG, bool BF16, bool ASYM, int PASS, int... SBS>
__device__ __forceinline__ void run2d(std::integer_sequence<int, SBS...>, const void* X, size_t blk_elem_off, int gridW,
                                      int d, int c0, bool active, int tid, float (&pend)[4][8], float (&top)[8],
                                      uint32_t (*s_max)[kPartWords], uint8_t* q_lo_blk, uint32_t q_off, float* scales_blk,
                                      size_t zeros_off, uint32_t* gpart_blk, size_t gpart_neg, const uint32_t* s_amax,
                                      bool write_scales) {
  (step2d<RLOG, BF16, ASYM, PASS, SBS>(X, blk_elem_off, gridW, d, c0, active, tid, pend, top, s_max, q_lo_blk, q_off,
                                       scales_blk, zeros_off, gpart_blk, gpart_neg, s_amax, write_scales), ...);
}

template <int RLOG, bool BF16, bool ASYM, int PASS>
__global__ __launch_bounds__(512) void k_bottom2d(const void* __restrict__ X, uint8_t* __restrict__ q_lo,
                                                  float* __restrict__ scales, float* __restrict__ abot, int s, int d, int G,
                                                  int gridW, int Kpad, size_t zeros_off, SplitArgs sp) {
  constexpr int g = 1 << RLOG;
  constexpr int R = g * g;
  __shared__ __attribute__((aligned(16))) uint32_t s_max[2][kPartWords];
  __shared__ uint32_t s_amax[PASS == 2 ? 2 * kMaxBlockRows : 1];
  const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int bi = j / G, bj = j - bi * G;
  const int c_lo = (PASS == 0) ? 0 : (int)blockIdx.z * sp.c_split;
  const int c_hi = (PASS == 0) ? d : min(d, c_lo + sp.c_split);
  const int c0 = c_lo + tid * 8;
  const bool active = c0 < c_hi;
  const int k = G * G;
  const size_t tok0 = (size_t)b * s + (size_t)(bi * g) * gridW + (size_t)bj * g;  // first token of the block
  const size_t prow0 = (size_t)b * s + (size_t)j * R;                              // first physical row of the block
  if constexpr (PASS == 2) gather_row_maxima<ASYM>(sp, prow0, R, tid, s_amax);
  float pend[4][8];
  float top[8];
  uint32_t* gpart_blk = (PASS == 1) ? sp.gpart + (size_t)blockIdx.z * sp.part_rows + prow0 : nullptr;
  run2d<RLOG, BF16, ASYM, PASS>(std::make_integer_sequence<int, (g == 4 ? 1 : 4)>{}, X, tok0 * d + c0, gridW, d, c0, active,
                                tid, pend, top, s_max, q_lo + stamp_qlo_offset(prow0, 0, Kpad),
                                (uint32_t)stamp_qlo_offset(0, c0, Kpad), scales + prow0, zeros_off, gpart_blk,
                                (size_t)sp.nsplit * sp.part_rows, s_amax, PASS == 0 || blockIdx.z == 0);
  if constexpr (PASS == 0) {
    if (sp.q_hi != nullptr) {
      constexpr int nsteps = (g == 4) ? 1 : 4;
      finish_top_row<true, ASYM>(top, RLOG, &s_max[nsteps & 1][0], sp.q_hi + ((size_t)b * k + j) * d + c0,
                                 q_lo + stamp_qlo_offset(prow0, c0, Kpad), scales + prow0, zeros_off, j < sp.khi, active, tid);
      return;
    }
  }
  if (active && PASS != 1) {
    float4* o = reinterpret_cast<float4*>(abot + ((size_t)b * k + j) * d + c0);
    o[0] = make_float4(top[0], top[1], top[2], top[3]);
    o[1] = make_float4(top[4], top[5], top[6], top[7]);
  }
}

// ------------------------------------------------------------------------------------------
// Top levels over the k block sums.  Workgroup = (32-channel slice, sequence); the k x 32 slice
// sits in LDS and the butterflies run in place (stride 2^l).  Writes normalised coefficients in
// STaMP order over abot (in place: each workgroup owns its slice) and the row absmax.
// ------------------------------------------------------------------------------------------
constexpr int kTopCh = 32;

// asym: the partial maxima are order keys of max t; those of max -t follow npart words further on.
// L = number of top levels (0: the block sums are only normalised).
__global__ __launch_bounds__(256) void k_top(float* __restrict__ abot, uint32_t* __restrict__ rowmax_part, int k, int d,
                                             int is2d, int G, int r_bottom, int L, int asym, size_t npart) {
  extern __shared__ float s_buf[];  // [k][kTopCh + 1]
  const int b = blockIdx.y, c_base = blockIdx.x * kTopCh, tid = threadIdx.x;
  const int ch = tid & (kTopCh - 1), grp = tid / kTopCh, ngrp = 256 / kTopCh;
  const int stride = kTopCh + 1;
  const bool cact = (c_base + ch) < d;
  float* base = abot + (size_t)b * k * d;
  // Plans without top levels may have more than 256 block sums per sequence: nothing is transformed, so every
  // workgroup (blockIdx.z) takes its own 256 rows [q0, q0 + kq); with top levels kq = k.
  const int q0 = (int)blockIdx.z * 256, kq = min(k - q0, 256);
  base += (size_t)q0 * d;
  // four independent loads in flight per thread before the first LDS write (one load per loop trip would
  // pay one memory latency per row)
  for (int j0 = grp; j0 < kq; j0 += 4 * ngrp) {
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * ngrp;
      v[u] = (cact && j < kq) ? base[(size_t)j * d + c_base + ch] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * ngrp;
      if (j < kq) s_buf[j * stride + ch] = v[u];
    }
  }
  __syncthreads();
  if (!is2d) {
    for (int st = 2; st <= (1 << L); st <<= 1) {
      const int npair = k / st;
      for (int i = grp; i < npair; i += ngrp) {
        float* pa = &s_buf[(i * st) * stride + ch];
        float* pd = &s_buf[(i * st + (st >> 1)) * stride + ch];
        const float x0 = *pa, x1 = *pd;
        *pa = __fadd_rn(x0, x1);
        *pd = __fsub_rn(x0, x1);
      }
      __syncthreads();
    }
  } else {
    for (int st = 2; st <= (1 << L); st <<= 1) {
      const int nc = G / st;
      const int h = st >> 1;
      for (int i = grp; i < nc * nc; i += ngrp) {
        const int cy = i / nc, cx = i - cy * nc;
        float* p00 = &s_buf[((cy * st) * G + cx * st) * stride + ch];
        float* p01 = p00 + h * stride;
        float* p10 = p00 + h * G * stride;
        float* p11 = p10 + h * stride;
        const float p = *p00, q = *p01, u = *p10, v = *p11;
        const float t0 = __fadd_rn(p, q), t1 = __fsub_rn(p, q), t2 = __fadd_rn(u, v), t3 = __fsub_rn(u, v);
        *p00 = __fadd_rn(t0, t2);
        *p01 = __fadd_rn(t1, t3);
        *p10 = __fsub_rn(t0, t2);
        *p11 = __fsub_rn(t1, t3);
      }
      __syncthreads();
    }
  }
  // normalise, scatter to STaMP order, row absmax over this slice
  for (int q = grp; q < kq; q += ngrp) {
    int e, lvl_top;  // level counted within the top part (1 = first top level); slot 0 gets the deepest
    if (!is2d) {
      e = stamp_top_slot_1d(q, k, L, &lvl_top);
    } else {
      const int y = q / G, x = q - y * G;
      e = stamp_top_slot_2d(y, x, G, L, &lvl_top);
    }
    // (q0 > 0 only without top levels, where slot = position: e = q, counted from q0 like `base`)
    const int level = r_bottom + lvl_top;
    const float nrm = is2d ? ldexpf(1.0f, -level) : haar_norm(level);
    const float t = __fmul_rn(s_buf[q * stride + ch], nrm);
    if (cact) base[(size_t)e * d + c_base + ch] = t;
    // max over the 32 channels of this row: lanes of one row are 32 consecutive lanes
    auto max32 = [](uint32_t x) {
      uint32_t yv;
      yv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false); x = max(x, yv);
      yv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, false); x = max(x, yv);
      yv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, false); x = max(x, yv);
      yv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xF, 0xF, false); x = max(x, yv);
      yv = (uint32_t)__shfl_xor((int)x, 16, 64); x = max(x, yv);
      return x;
    };
    const size_t slot = ((size_t)b * k + q0 + e) * gridDim.x + blockIdx.x;
    if (!asym) {
      const uint32_t x = max32(absbits(t));
      if (ch == 0) rowmax_part[slot] = x;
    } else {
      // channels beyond d_in contribute the neutral key
      const uint32_t xp = max32(cact ? fkey(t) : 0u);
      const uint32_t xn = max32(cact ? fkey(-t) : 0u);
      if (ch == 0) { rowmax_part[slot] = xp; rowmax_part[npart + slot] = xn; }
    }
  }
}

// one workgroup per 8-bit row.  asym: min-max form, the stored code is code - 128 and the offset z goes
// zeros_off floats behind the row's scale.
__global__ __launch_bounds__(256) void k_quant_hi(const float* __restrict__ ttop, const uint32_t* __restrict__ rowmax_part,
                                                  int nslices, int8_t* __restrict__ q_hi, float* __restrict__ scales,
                                                  int k, int khi, int d, int s, int R, int asym, size_t npart,
                                                  size_t zeros_off, uint8_t* __restrict__ q_lo, int Kpad) {
  __shared__ uint32_t s_red[8];
  const int p = blockIdx.x, b = blockIdx.y;
  {
    uint32_t m = 0u, mneg = 0u;
    for (int i = threadIdx.x; i < nslices; i += 256) {
      const size_t slot = ((size_t)b * k + p) * nslices + i;
      m = max(m, rowmax_part[slot]);
      if (asym) mneg = max(mneg, rowmax_part[npart + slot]);
    }
    m = wave_max_u32(m);
    mneg = wave_max_u32(mneg);
    if ((threadIdx.x & 63) == 0) { s_red[threadIdx.x >> 6] = m; s_red[4 + (threadIdx.x >> 6)] = mneg; }
    __syncthreads();
  }
  const uint32_t mp = max(max(s_red[0], s_red[1]), max(s_red[2], s_red[3]));
  const uint32_t mn = max(max(s_red[4], s_red[5]), max(s_red[6], s_red[7]));
  // rows beyond the first khi are 4-bit rows (same data path, codes held as int8)
  const bool row8 = p < khi;
  const float qmax_s = row8 ? 127.0f : 7.0f, qmax_u = row8 ? 255.0f : 15.0f;
  float scale = 0.0f, inv = 0.0f, z = 0.0f;
  if (!asym) {
    const float a = __uint_as_float(mp);
    if (a > 0.0f) {
      scale = __fdiv_rn(a, qmax_s);
      inv = __fdiv_rn(qmax_s, a);
    }
  } else {
    asym_params(fkey_inv(mp), fkey_inv(mn), qmax_u, scale, inv, z);
  }
  if (threadIdx.x == 0) {
    scales[(size_t)b * s + (size_t)p * R] = scale;
    if (asym) scales[zeros_off + (size_t)b * s + (size_t)p * R] = z;
  }
  const float qlo = asym ? 0.0f : -qmax_s, qhi = asym ? qmax_u : qmax_s, shift = asym ? (row8 ? 128.0f : 8.0f) : 0.0f;
  const float* src = ttop + ((size_t)b * k + p) * d;
  int8_t* dst = q_hi + ((size_t)b * k + p) * d;
  for (int c = threadIdx.x * 4; c < d; c += 256 * 4) {
    const float4 t = *reinterpret_cast<const float4*>(src + c);
    const float v[4] = {t.x, t.y, t.z, t.w};
    uint32_t w = 0, w4 = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float q = __fadd_rn(rintf(__fmul_rn(v[i], inv)), z);
      q = fminf(fmaxf(q, qlo), qhi) - shift;
      w |= ((uint32_t)((int)q) & 0xFFu) << (8 * i);
      w4 |= ((uint32_t)((int)q) & 0xFu) << (4 * i);
    }
    *reinterpret_cast<uint32_t*>(dst + c) = w;
    // plans without top levels: a 4-bit row also goes, packed, to its block's row 0 of q_lo (see finish_top_row)
    if (q_lo != nullptr && !row8)
      *reinterpret_cast<uint16_t*>(q_lo + stamp_qlo_offset((size_t)b * s + (size_t)p * R, c, Kpad)) = (uint16_t)w4;
  }
}

// ------------------------------------------------------------------------------------------
// Plans without a sequence transform (the layers the paper leaves un-transformed, and the baseline the
// transform's cost is measured against): per-token quantization of X itself (Background, Eq. 1), tokens
// 0..k-1 of every sequence at 8 bits, the rest at 4 bits.  One workgroup per token: the row is read twice
// (range, then codes; the second read comes from cache).
// ------------------------------------------------------------------------------------------
template <bool BF16, bool ASYM>
__global__ __launch_bounds__(256) void k_quant_rows(const void* __restrict__ X, int8_t* __restrict__ q_hi,
                                                    uint8_t* __restrict__ q_lo, float* __restrict__ scales, int s, int d,
                                                    int k, int Kpad, size_t zeros_off) {
  __shared__ uint32_t s_red[8];
  const int pr = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const size_t m = (size_t)b * s + pr;
  const size_t xoff = m * (size_t)d;
  uint32_t mpos = 0u, mneg = 0u;
  for (int c = tid * 8; c < d; c += 256 * 8) {
    float v[8];
    load8(X, xoff + c, BF16, true, v);
    if constexpr (ASYM) {
      uint32_t pos, neg;
      row_posneg_bits(v, pos, neg);
      mpos = max(mpos, pos);
      mneg = max(mneg, neg);
    } else {
      mpos = max(mpos, row_absmax_bits(v));
    }
  }
  mpos = wave_max_u32(mpos);
  mneg = wave_max_u32(mneg);
  if ((tid & 63) == 0) { s_red[tid >> 6] = mpos; s_red[4 + (tid >> 6)] = mneg; }
  __syncthreads();
  const uint32_t mp = max(max(s_red[0], s_red[1]), max(s_red[2], s_red[3]));
  const uint32_t mn = max(max(s_red[4], s_red[5]), max(s_red[6], s_red[7]));
  const bool hi = pr < k;
  const float qmax = ASYM ? (hi ? 255.0f : 15.0f) : (hi ? 127.0f : 7.0f);
  float scale = 0.0f, inv = 0.0f, z = 0.0f;
  if constexpr (ASYM) {
    asym_params(fkey_inv(mp), fkey_inv(mn), qmax, scale, inv, z);
  } else {
    const float a = __uint_as_float(mp);
    if (a > 0.0f) {
      scale = __fdiv_rn(a, qmax);
      inv = __fdiv_rn(qmax, a);
    }
  }
  if (tid == 0) {
    scales[m] = scale;
    if constexpr (ASYM) scales[zeros_off + m] = z;
  }
  for (int c = tid * 8; c < d; c += 256 * 8) {
    float v[8];
    load8(X, xoff + c, BF16, true, v);
    if (hi) {
      const float qlo = ASYM ? 0.0f : -127.0f, qhi = ASYM ? 255.0f : 127.0f, shift = ASYM ? 128.0f : 0.0f;
      uint32_t w[2] = {0u, 0u};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float q = __fadd_rn(rintf(__fmul_rn(v[i], inv)), z);
        q = fminf(fmaxf(q, qlo), qhi) - shift;
        w[i >> 2] |= ((uint32_t)((int)q) & 0xFFu) << (8 * (i & 3));
      }
      *reinterpret_cast<uint2*>(q_hi + ((size_t)b * k + pr) * d + c) = make_uint2(w[0], w[1]);
    } else {
      float pq[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) pq[i] = __fmul_rn(v[i], inv);
      uint32_t w;
      if constexpr (ASYM) {
        const float lo = -z, hib = 15.0f - z;
#pragma unroll
        for (int i = 0; i < 8; ++i) pq[i] = __builtin_amdgcn_fmed3f(pq[i], lo, hib);
        w = pack8_uint4(pq, z);
      } else {
        w = pack8_int4(pq);
      }
      *reinterpret_cast<uint32_t*>(q_lo + stamp_qlo_offset(m, c, Kpad)) = w;
    }
  }
}

template <int RLOG, bool BF16, bool ASYM, int PASS>
hipError_t launch_bottom1d_pass(const stamp_plan* p, const void* X, uint8_t* q_lo, float* scales, float* abot, int nthreads,
                                const SplitArgs& sp, hipStream_t st) {
  const StampGeom& g = p->geom;
  const size_t lds = (size_t)8 * nthreads * (BF16 ? 16 : 32);  // staging buffer: 2 batches of 4 token rows
  if (lds > 160 * 1024 - 2048) return hipErrorInvalidValue;
  static size_t lds_done[kStampMaxDevices] = {};
  hipError_t e = stamp_allow_lds(reinterpret_cast<const void*>(&k_bottom1d<RLOG, BF16, ASYM, PASS>), lds, lds_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((k_bottom1d<RLOG, BF16, ASYM, PASS>), dim3(g.k, g.B, PASS == 0 ? 1 : sp.nsplit), dim3(nthreads), lds, st,
                     X, q_lo, scales, abot, g.s, g.d, g.k, p->Kpad, (size_t)g.B * g.s, sp);
  return hipGetLastError();
}

// one pass when a workgroup can hold all channels, else maxima pass + quantization pass over channel splits
template <int RLOG, bool BF16, bool ASYM>
hipError_t launch_bottom1d(const stamp_plan* p, const void* X, uint8_t* q_lo, float* scales, float* abot, int nthreads,
                           const SplitArgs& sp, hipStream_t st) {
  if (sp.nsplit == 1) return launch_bottom1d_pass<RLOG, BF16, ASYM, 0>(p, X, q_lo, scales, abot, nthreads, sp, st);
  hipError_t e = launch_bottom1d_pass<RLOG, BF16, ASYM, 1>(p, X, q_lo, scales, abot, nthreads, sp, st);
  if (e != hipSuccess) return e;
  return launch_bottom1d_pass<RLOG, BF16, ASYM, 2>(p, X, q_lo, scales, abot, nthreads, sp, st);
}

}  // namespace

// general path: per-token quantization of the transformed tokens T [B, s, d] fp32 (rows = STaMP slots)
hipError_t stamp_launch_quant_rows_f32(const stamp_plan* p, const float* T, int8_t* q_hi, uint8_t* q_lo, float* scales,
                                       hipStream_t st) {
  const StampGeom& g = p->geom;
  const dim3 grid_rows(g.s, g.B);
  const size_t zoff = (size_t)g.B * g.s;
  if (g.asym) hipLaunchKernelGGL((k_quant_rows<false, true>), grid_rows, dim3(256), 0, st, T, q_hi, q_lo, scales, g.s, g.d, g.k, p->Kpad, zoff);
  else hipLaunchKernelGGL((k_quant_rows<false, false>), grid_rows, dim3(256), 0, st, T, q_hi, q_lo, scales, g.s, g.d, g.k, p->Kpad, zoff);
  return hipGetLastError();
}

bool stamp_top_in_bottom(const stamp_plan* p) {
  return !p->geom.ident && p->geom.L == 0 && stamp_actquant_nsplit(p) == 1;
}

int stamp_actquant_nsplit(const stamp_plan* p) {
  const StampGeom& g = p->geom;
  if (g.ident) return 1;
  const int dmax = (g.is2d || !g.x_bf16) ? 4096 : 8192;  // channels one workgroup can hold
  return (g.d + dmax - 1) / dmax;
}

hipError_t stamp_launch_actquant(const stamp_plan* p, const void* X, int8_t* q_hi, uint8_t* q_lo, float* scales,
                                 float* abot, uint32_t* rowmax, uint32_t* gpart, hipStream_t st, int part) {
  const StampGeom& g = p->geom;
  if (g.ident) {
    if (!(part & 1)) return hipSuccess;
    const dim3 grid_rows(g.s, g.B);
    const size_t zoff = (size_t)g.B * g.s;
    if (g.asym) {
      if (g.x_bf16) hipLaunchKernelGGL((k_quant_rows<true, true>), grid_rows, dim3(256), 0, st, X, q_hi, q_lo, scales, g.s, g.d, g.k, p->Kpad, zoff);
      else hipLaunchKernelGGL((k_quant_rows<false, true>), grid_rows, dim3(256), 0, st, X, q_hi, q_lo, scales, g.s, g.d, g.k, p->Kpad, zoff);
    } else {
      if (g.x_bf16) hipLaunchKernelGGL((k_quant_rows<true, false>), grid_rows, dim3(256), 0, st, X, q_hi, q_lo, scales, g.s, g.d, g.k, p->Kpad, zoff);
      else hipLaunchKernelGGL((k_quant_rows<false, false>), grid_rows, dim3(256), 0, st, X, q_hi, q_lo, scales, g.s, g.d, g.k, p->Kpad, zoff);
    }
    return hipGetLastError();
  }
  SplitArgs sp;
  sp.gpart = gpart;
  sp.part_rows = (size_t)g.B * g.s;
  sp.nsplit = stamp_actquant_nsplit(p);
  sp.c_split = (sp.nsplit == 1) ? g.d : (((g.d + sp.nsplit - 1) / sp.nsplit + 511) / 512) * 512;
  if (sp.nsplit > 1 && gpart == nullptr) return hipErrorInvalidValue;
  // no top levels: the bottom kernel finishes the block sums itself (one launch instead of three)
  const bool top_in_bottom = stamp_top_in_bottom(p);
  sp.q_hi = top_in_bottom ? q_hi : nullptr;
  sp.khi = g.khi;
  const int nthreads = ((sp.c_split / 8 + 63) / 64) * 64;
  dim3 grid(g.k, g.B);
  const size_t zeros_off = (size_t)g.B * g.s;
#define LAUNCH1D(RL)                                                                                      \
  do {                                                                                                    \
    hipError_t le = g.asym ? (g.x_bf16 ? launch_bottom1d<RL, true, true>(p, X, q_lo, scales, abot, nthreads, sp, st)     \
                                       : launch_bottom1d<RL, false, true>(p, X, q_lo, scales, abot, nthreads, sp, st))   \
                           : (g.x_bf16 ? launch_bottom1d<RL, true, false>(p, X, q_lo, scales, abot, nthreads, sp, st)    \
                                       : launch_bottom1d<RL, false, false>(p, X, q_lo, scales, abot, nthreads, sp, st)); \
    if (le != hipSuccess) return le;                                                                      \
  } while (0)
#define LAUNCH2D__(RL, BF, AS, PASS)                                                                      \
  hipLaunchKernelGGL((k_bottom2d<RL, BF, AS, PASS>), dim3(g.k, g.B, PASS == 0 ? 1 : sp.nsplit), dim3(nthreads), 0, st, X, \
                     q_lo, scales, abot, g.s, g.d, g.G, g.gridW, p->Kpad, zeros_off, sp)
#define LAUNCH2D_(RL, BF, AS)                                                                             \
  do {                                                                                                    \
    if (sp.nsplit == 1) { LAUNCH2D__(RL, BF, AS, 0); }                                                    \
    else { LAUNCH2D__(RL, BF, AS, 1); LAUNCH2D__(RL, BF, AS, 2); }                                        \
  } while (0)
#define LAUNCH2D(RL)                                                                                      \
  do {                                                                                                    \
    if (g.asym) { if (g.x_bf16) LAUNCH2D_(RL, true, true); else LAUNCH2D_(RL, false, true); }             \
    else { if (g.x_bf16) LAUNCH2D_(RL, true, false); else LAUNCH2D_(RL, false, false); }                  \
  } while (0)
  if (!(part & 1)) {
    // bottom kernel skipped
  } else if (!g.is2d) {
    switch (g.r) {
      case 3: LAUNCH1D(3); break;
      case 4: LAUNCH1D(4); break;
      case 5: LAUNCH1D(5); break;
      case 6: LAUNCH1D(6); break;
      case 7: LAUNCH1D(7); break;
      default: return hipErrorInvalidValue;
    }
  } else {
    if (nthreads > 512) return hipErrorInvalidValue;
    switch (g.r) {
      case 2: LAUNCH2D(2); break;
      case 3: LAUNCH2D(3); break;
      default: return hipErrorInvalidValue;
    }
  }
#undef LAUNCH1D
#undef LAUNCH2D
#undef LAUNCH2D_
#undef LAUNCH2D__
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (!(part & 2) || top_in_bottom) return hipSuccess;
  if (g.k > 256 && g.L != 0) return hipErrorInvalidValue;  // plan creation admits that many top rows only without top levels
  const size_t lds = (size_t)(g.k < 256 ? g.k : 256) * (kTopCh + 1) * sizeof(float);
  const int nslices = (g.d + kTopCh - 1) / kTopCh;
  const size_t npart = (size_t)g.B * g.k * nslices;
  hipLaunchKernelGGL(k_top, dim3(nslices, g.B, (g.k + 255) / 256), dim3(256), lds, st, abot, rowmax, g.k, g.d, g.is2d, g.G, g.r, g.L, g.asym,
                     npart);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_quant_hi, dim3(g.k, g.B), dim3(256), 0, st, abot, rowmax, nslices, q_hi, scales, g.k, g.khi, g.d, g.s, g.R,
                     g.asym, npart, zeros_off, g.L == 0 ? q_lo : nullptr, p->Kpad);
  return hipGetLastError();
}
