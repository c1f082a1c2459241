// Host side of the C ABI declared in include/stamp.h: argument validation (always before any HIP
// call), plan construction, workspace layout and the launch sequences.
#include <cstdlib>
#include <cstring>
#include <new>

#include "stamp_internal.h"

// Scratch memory of stamp_linear_forward_static: one array per GPU, part of the loaded code object.  In host
// code this name only stands for the symbol; the device address comes from hipGetSymbolAddress (static_scratch()).
static __device__ __align__(256) unsigned char scratch[STAMP_STATIC_SCRATCH_BYTES];

namespace {

// device address of `scratch` on the current device, looked up once per device
stamp_status_t static_scratch(void** out) {
  static void* ptr[kStampMaxDevices] = {};
  static std::mutex mu;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStampMaxDevices) return STAMP_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return STAMP_ERR_DEVICE;
    }
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return STAMP_OK;
}

inline bool is_pow2(int64_t n) { return n >= 1 && (n & (n - 1)) == 0; }
inline int ilog2(int64_t n) { int l = 0; while ((int64_t(1) << (l + 1)) <= n) ++l; return l; }
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

int max_ragged_levels(int n) {
  int l = 0;
  while (n > 1) {
    n = (n + 1) / 2;
    ++l;
  }
  return l;
}

// Geometry of the fast path (blocks of tokens, top rows); STAMP_ERR_UNSUPPORTED when the setting has none.
stamp_status_t fast_geometry(const stamp_plan_desc_t* d, StampGeom* g, int* fused_ok, int side) {
  if (d->xform == STAMP_L_IDENTITY) {
    // tokens quantized as they are: any number of 8-bit tokens (none included), no blocks, no inverse
    if (d->batch > 65535 || (int64_t)d->batch * d->k_hi > 65535) return STAMP_ERR_UNSUPPORTED;  // grid dimensions
    g->ident = 1;
    g->R = 1;
    *fused_ok = 1;
    return STAMP_OK;
  }
  // More than 256 top rows: only where no kernel needs all top rows of a sequence in LDS at once, i.e. plans
  // without top levels (fewer 8-bit tokens than approximations).  E.g. 3 levels and 64 8-bit tokens on 4096 or 8192 tokens.
  // Blocks.  With at least as many 8-bit tokens as level-J approximations, the blocks hold seq_len / k_hi tokens
  // (the top part runs the remaining levels over the k_hi block sums).  With fewer, the blocks hold the 2^J
  // (4^J) tokens of one approximation, the top part is the approximations themselves, and those beyond the
  // first k_hi are 4-bit rows that stay with the 8-bit rows' data path (4-bit codes held as int8).
  if (d->xform == STAMP_L_HAAR1D) {
    g->is2d = 0;
    const int na = d->seq_len >> d->levels;
    if (d->k_hi >= na) {
      if (d->k_hi < 1 || !is_pow2(d->k_hi)) return STAMP_ERR_UNSUPPORTED;
      g->k = g->khi = d->k_hi;
    } else {
      g->k = na;
      g->khi = d->k_hi;
    }
    if (g->k > 256 && d->k_hi >= na) return STAMP_ERR_UNSUPPORTED;
    g->R = d->seq_len / g->k;
    g->r = ilog2(g->R);
    if (g->r < 3 || g->r > 7) return STAMP_ERR_UNSUPPORTED;
    *fused_ok = g->r <= 6;
  } else {
    const int sa = side >> d->levels;  // approximations per grid side
    if (d->k_hi >= sa * sa) {
      const int lk = ilog2(d->k_hi);
      if (d->k_hi < 1 || !is_pow2(d->k_hi) || lk % 2 != 0) return STAMP_ERR_UNSUPPORTED;  // k must be a power of four
      g->G = 1 << (lk / 2);
      g->k = g->khi = d->k_hi;
    } else {
      g->G = sa;
      g->k = sa * sa;
      g->khi = d->k_hi;
    }
    if (g->k > 256 && d->k_hi >= sa * sa) return STAMP_ERR_UNSUPPORTED;
    g->is2d = 1;
    g->R = d->seq_len / g->k;
    g->g = side / g->G;
    g->r = ilog2(g->g);
    g->gridW = d->grid_w;
    if (g->r < 2 || g->r > 3) return STAMP_ERR_UNSUPPORTED;
    *fused_ok = 1;
  }
  g->L = g->J - g->r;
  // batch and batch * (top rows) are grid dimensions y / z of the transform and inverse kernels
  if (d->batch > 65535 || (int64_t)d->batch * g->k > 65535) return STAMP_ERR_UNSUPPORTED;
  return STAMP_OK;
}

stamp_status_t validate(const stamp_plan_desc_t* d, StampGeom* g, int* fused_ok, StampGen* gen) {
  memset(gen, 0, sizeof(*gen));
  if (d->batch < 1 || d->seq_len < 1 || d->d_in < 1 || d->d_out < 1) return STAMP_ERR_SHAPE;
  if (d->xform < STAMP_L_IDENTITY || d->xform > STAMP_L_DCT) return STAMP_ERR_SHAPE;
  if (d->skip_first != 0 && d->skip_first != 1) return STAMP_ERR_SHAPE;
  if (d->skip_first && (d->xform != STAMP_L_HAAR1D || d->seq_len < 2)) return STAMP_ERR_SHAPE;  // defined for the 1-D Haar transform
  if (d->bias_mode != 0 && d->bias_mode != 1) return STAMP_ERR_SHAPE;
  if (d->group_size < 0) return STAMP_ERR_SHAPE;
  if (d->k_hi < 0 || d->k_hi > d->seq_len) return STAMP_ERR_SHAPE;
  if (d->bits_hi < 2 || d->bits_hi > 8 || d->bits_lo < 2 || d->bits_lo > 8 || d->bits_w < 2 || d->bits_w > 8)
    return STAMP_ERR_SHAPE;
  if (d->d_in % 2 != 0) return STAMP_ERR_SHAPE;
  for (int32_t t : {d->x_dtype, d->y_dtype, d->w_dtype})
    if (t != STAMP_F32 && t != STAMP_BF16) return STAMP_ERR_SHAPE;
  if (d->w_is_out_by_in != 0 && d->w_is_out_by_in != 1) return STAMP_ERR_SHAPE;
  if (d->act_quant != STAMP_ACT_SYMMETRIC && d->act_quant != STAMP_ACT_ASYMMETRIC) return STAMP_ERR_SHAPE;
  if ((int64_t)d->batch * d->seq_len > (int64_t)1 << 30) return STAMP_ERR_SHAPE;

  int J = 0, side = 0;
  const bool ragged = d->xform == STAMP_L_HAAR1D && (d->skip_first || !is_pow2(d->seq_len));
  if (ragged) {
    if (d->levels < 0 || d->levels > max_ragged_levels(d->seq_len - d->skip_first)) return STAMP_ERR_SHAPE;
  } else if (d->xform == STAMP_L_WHT) {
    if (!is_pow2(d->seq_len) || d->levels != 0) return STAMP_ERR_SHAPE;
  } else if (d->xform == STAMP_L_DCT) {
    if (d->levels != 0) return STAMP_ERR_SHAPE;
  } else if (d->xform == STAMP_L_HAAR1D) {
    J = ilog2(d->seq_len);
    if (d->levels < 1 || d->levels > J) return STAMP_ERR_SHAPE;
  } else if (d->xform == STAMP_L_HAAR2D) {
    if (d->grid_h < 1 || d->grid_w < 1 || (int64_t)d->grid_h * d->grid_w != d->seq_len) return STAMP_ERR_SHAPE;
    if (!is_pow2(d->grid_h) || !is_pow2(d->grid_w)) return STAMP_ERR_SHAPE;
    side = d->grid_h < d->grid_w ? d->grid_h : d->grid_w;
    J = ilog2(side);
    if (d->levels < 1 || d->levels > J) return STAMP_ERR_SHAPE;
  } else if (d->levels != 0) {
    return STAMP_ERR_SHAPE;  // no transform, no levels
  }

  // ---- valid STaMP settings from here on; what follows is what this library implements ----
  if (d->bits_hi != 8 || d->bits_lo != 4 || d->bits_w != 4) return STAMP_ERR_UNSUPPORTED;
  if (d->d_in % 32 != 0 || d->d_in > 32768) return STAMP_ERR_UNSUPPORTED;  // wider than one workgroup holds: channel splits, two passes
  if (d->d_out > (1 << 21)) return STAMP_ERR_UNSUPPORTED;  // the GEMM epilogues address a tile's 256 output rows with 32-bit byte offsets
  memset(g, 0, sizeof(*g));
  g->B = d->batch; g->s = d->seq_len; g->d = d->d_in; g->N = d->d_out;
  g->J = d->levels; g->k = g->khi = d->k_hi;
  g->x_bf16 = d->x_dtype == STAMP_BF16;
  g->y_bf16 = d->y_dtype == STAMP_BF16;
  g->asym = d->act_quant == STAMP_ACT_ASYMMETRIC;
  // ---- the fast path's geometry, where the setting has one ----
  const bool rect2d = d->xform == STAMP_L_HAAR2D && d->grid_h != d->grid_w;  // the fast path takes square grids only
  bool need_general = ragged || rect2d || d->xform == STAMP_L_WHT || d->xform == STAMP_L_DCT || d->bias_mode == 1 || d->group_size != 0;
  if (!need_general) {
    const stamp_status_t fs = fast_geometry(d, g, fused_ok, side);
    if (fs == STAMP_OK) return STAMP_OK;
    // a valid setting outside the fast path's block structure (block sizes, more than 256 top rows, an 8-bit token
    // count that is not a power of two, ...): the general path takes it
    need_general = true;
    memset(g, 0, sizeof(*g));
    g->B = d->batch; g->s = d->seq_len; g->d = d->d_in; g->N = d->d_out;
    g->k = g->khi = d->k_hi;
    g->x_bf16 = d->x_dtype == STAMP_BF16;
    g->y_bf16 = d->y_dtype == STAMP_BF16;
    g->asym = d->act_quant == STAMP_ACT_ASYMMETRIC;
  }
  // ---- general path: transforms without the fast path's block structure, transformed bias, per-block scales ----
  if (d->group_size != 0 && d->group_size != 64) return STAMP_ERR_UNSUPPORTED;
  if (d->group_size == 64 && (d->d_in % 64 != 0 || g->asym)) return STAMP_ERR_UNSUPPORTED;
  if (d->seq_len > 65535 || d->batch > 65535 || (int64_t)d->batch * d->k_hi > 65535) return STAMP_ERR_UNSUPPORTED;  // grid dimensions
  if (d->xform == STAMP_L_DCT && d->seq_len > 16384) return STAMP_ERR_UNSUPPORTED;  // dense s x s matrix in fp64
  gen->kind = ragged ? kGenHaarRagged
              : d->xform == STAMP_L_WHT ? kGenWht
              : d->xform == STAMP_L_DCT ? kGenDct
              : d->xform == STAMP_L_HAAR1D ? kGenHaarClassic
              : d->xform == STAMP_L_HAAR2D ? kGenHaar2d : kGenCopy;
  gen->levels = d->levels;
  gen->skip = d->skip_first;
  gen->group = d->group_size;
  gen->bias_mode = d->bias_mode;
  gen->gridH = d->grid_h;
  gen->gridW = d->grid_w;
  // the quantizer and the GEMM see the transformed tokens as rows: physical row = STaMP slot, no blocks
  g->J = 0;
  g->ident = 1;
  g->R = 1;
  if (d->group_size == 64) g->k = d->seq_len;  // every token's codes travel as int8 (khi of them are 8-bit rows)
  *fused_ok = 0;
  return STAMP_OK;
}

void layout_workspace(stamp_plan* p) {
  const StampGeom& g = p->geom;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
  if (p->gen.kind != kGenNone) {
    // general path: three fp32 copies of the activation and of the transformed output for the level kernels, and
    // the quantized activation (per-token scales: the buffers of the fast path; per-block scales: int8 codes)
    const bool grouped = p->gen.group != 0;
    p->ws_abot = p->ws_rowmax = p->ws_gpart = p->ws_P = p->ws_ytlo = 0;
    p->ws_qhi = take(grouped ? 0 : (size_t)g.B * g.k * g.d);
    p->ws_qlo = take(grouped ? 0 : (size_t)p->Mpad * (p->Kpad / 2));
    p->ws_scales = take(grouped ? 0 : (size_t)2 * g.B * g.s * sizeof(float));
    p->ws_ythi = take(grouped ? 0 : (size_t)p->hi_ksplit * g.B * g.k * g.N * sizeof(float));
    p->ws_a6 = take(grouped ? 0 : stamp_a6_bytes(p));
    for (size_t& o : p->ws_T) o = take((size_t)g.B * g.s * g.d * sizeof(float));
    for (size_t& o : p->ws_Yt) o = take((size_t)g.B * g.s * g.N * sizeof(float));
    p->ws_codes8 = take(grouped ? (size_t)g.B * g.s * g.d : 0);
    p->ws_scalesg = take(grouped ? (size_t)g.B * g.s * (g.d / 64) * sizeof(float) : 0);
    p->ws_total = off;
    return;
  }
  p->ws_abot = take((size_t)g.B * g.k * g.d * sizeof(float));
  p->ws_rowmax = take((size_t)2 * g.B * g.k * ((g.d + 31) / 32) * sizeof(uint32_t));  // partial row maxima (asymmetric: of both signs) per 32-channel slice
  {
    const int nsplit = stamp_actquant_nsplit(p);
    p->ws_gpart = take(nsplit > 1 ? (size_t)2 * nsplit * g.B * g.s * sizeof(uint32_t) : 0);  // row maxima per channel split
  }
  p->ws_qhi = take((size_t)g.B * g.k * g.d);
  p->ws_qlo = take((size_t)p->Mpad * (p->Kpad / 2));
  p->ws_scales = take((size_t)2 * g.B * g.s * sizeof(float));  // scales, then offsets (asymmetric plans)
  {
    // partial rows per part of a split depth, for either set of rows the 8-bit rows' GEMM may be run over
    const size_t all = (size_t)p->hi_ksplit * g.k, own = (size_t)p->hi_ksplit_own * g.khi;
    p->ws_ythi = take((all > own ? all : own) * g.B * g.N * sizeof(float));
  }
  p->ws_P = take((size_t)g.B * g.k * p->Npad * sizeof(float));
  p->ws_a6 = take(stamp_a6_bytes(p));
  p->ws_ytlo = off;
  if (p->unfused || !p->fused_ok) take((size_t)g.B * g.s * g.N * sizeof(float));
  p->ws_total = off;
}

inline bool ws_ok(const stamp_plan* p, const void* ws, size_t bytes, size_t need) {
  (void)p;
  return ws != nullptr && (reinterpret_cast<uintptr_t>(ws) & 255) == 0 && bytes >= need;
}

inline uint8_t* at(void* ws, size_t off) { return reinterpret_cast<uint8_t*>(ws) + off; }

// Plans without top levels that keep only some of the block sums at 8 bits (0 < khi < k), default route (FP6
// engine, fused inverse): the 4-bit block sums are rows of the 4-bit rows' GEMM (the quantizer has put their packed
// codes at coefficient 0 of their blocks), and the 8-bit rows' GEMM runs over the first khi rows of every sequence only.
inline bool own_top(const stamp_plan* p) {
  const StampGeom& g = p->geom;
  return p->gen.kind == kGenNone && !g.ident && g.L == 0 && g.khi > 0 && g.khi < g.k && p->engine == STAMP_GEMM_FP6 &&
         p->fused_ok && !p->unfused;
}

// block sums of the first khi blocks of every sequence -> P [B * khi][Npad]
inline hipError_t stamp_launch_block_sums_own(const stamp_plan* p, const int8_t* q_hi, const float* scales, float* ythi,
                                              float* P, hipStream_t st) {
  if (p->hi_ksplit_own <= 1) return stamp_launch_gemm_hi(p, q_hi, scales, 1, P, st, p->Npad, true);
  const hipError_t e = stamp_launch_gemm_hi(p, q_hi, scales, 1, ythi, st, 0, true);
  if (e != hipSuccess) return e;
  return stamp_launch_sum_parts(ythi, p->hi_ksplit_own, p->geom.B * p->geom.khi, p->geom.N, P, p->Npad, st);
}

// codes_are_ours: q_hi / q_lo were written by this library's quantizer (which also fills the rows of q_lo that
// own_top reads); buffers a caller packed need not hold them
stamp_status_t forward_q(const stamp_plan* p, const int8_t* q_hi, const uint8_t* q_lo, const float* scales, void* Y,
                         void* ws, hipStream_t st, bool codes_are_ours) {
  float* ythi = reinterpret_cast<float*>(at(ws, p->ws_ythi));
  float* P = reinterpret_cast<float*>(at(ws, p->ws_P));
  if (p->gen.kind != kGenNone) {
    // general path: dequantized rows in STaMP order -> (transformed bias) -> inverse level by level -> Y
    float* const yt[3] = {reinterpret_cast<float*>(at(ws, p->ws_Yt[0])), reinterpret_cast<float*>(at(ws, p->ws_Yt[1])),
                          reinterpret_cast<float*>(at(ws, p->ws_Yt[2]))};
    if (p->gen.group) {
      // q_hi carries every token's int8 codes, scales one per token and 64-channel group
      if (stamp_launch_gemm_grouped(p, q_hi, scales, yt[0], st) != hipSuccess) return STAMP_ERR_DEVICE;
    } else {
      if (p->geom.k > 0) {
        if (stamp_launch_gemm_hi(p, q_hi, scales, 1, ythi, st) != hipSuccess) return STAMP_ERR_DEVICE;
        if (stamp_launch_merge_hi(p, ythi, p->hi_ksplit, yt[0], st) != hipSuccess) return STAMP_ERR_DEVICE;
      }
      if (p->geom.k < p->geom.s) {
        if (p->engine == STAMP_GEMM_FP6) {
          uint8_t* a6g = at(ws, p->ws_a6);
          if (stamp_launch_repack6(p, q_lo, a6g, st) != hipSuccess) return STAMP_ERR_DEVICE;
          if (stamp_launch_gemm_lo6(p, a6g, scales, 1, yt[0], nullptr, st) != hipSuccess) return STAMP_ERR_DEVICE;
        } else {
          if (stamp_launch_gemm_lo(p, q_lo, scales, 1, yt[0], nullptr, st) != hipSuccess) return STAMP_ERR_DEVICE;
        }
      }
    }
    const bool tbias = p->gen.bias_mode == 1 && p->bias_dev != nullptr;
    if (tbias && stamp_launch_add_ell_bias(p, yt[0], st) != hipSuccess) return STAMP_ERR_DEVICE;
    return stamp_gen_inverse(p, yt, p->geom.N, tbias ? nullptr : p->bias_dev, Y, st) == hipSuccess ? STAMP_OK : STAMP_ERR_DEVICE;
  }
  if (p->geom.ident) {
    // no transform: the 8-bit rows' GEMM (partial rows) + their output pass, then the 4-bit rows straight to Y
    if (p->geom.k > 0) {
      if (stamp_launch_gemm_hi(p, q_hi, scales, 1, ythi, st) != hipSuccess) return STAMP_ERR_DEVICE;
      if (stamp_launch_hi_rows_out(p, ythi, Y, st, p->hi_ksplit) != hipSuccess) return STAMP_ERR_DEVICE;
    }
    if (p->geom.k == p->geom.s) return STAMP_OK;
    if (p->engine == STAMP_GEMM_FP6) {
      uint8_t* a6i = at(ws, p->ws_a6);
      if (stamp_launch_repack6(p, q_lo, a6i, st) != hipSuccess) return STAMP_ERR_DEVICE;
      return stamp_launch_gemm_lo6(p, a6i, scales, 3, Y, nullptr, st) == hipSuccess ? STAMP_OK : STAMP_ERR_DEVICE;
    }
    return stamp_launch_gemm_lo(p, q_lo, scales, 3, Y, nullptr, st) == hipSuccess ? STAMP_OK : STAMP_ERR_DEVICE;
  }
  const bool fused = p->fused_ok && !p->unfused;
  const bool own = codes_are_ours && own_top(p);
  if (own) {
    if (stamp_launch_block_sums_own(p, q_hi, scales, ythi, P, st) != hipSuccess) return STAMP_ERR_DEVICE;
  } else if (stamp_hi_rows_are_block_sums(p)) {
    if (stamp_launch_gemm_hi(p, q_hi, scales, 1, P, st, p->Npad) != hipSuccess) return STAMP_ERR_DEVICE;
  } else if (stamp_hi_top_fused(p)) {
    if (stamp_launch_gemm_hi(p, q_hi, scales, 2, P, st, p->Npad) != hipSuccess) return STAMP_ERR_DEVICE;
  } else {
    if (stamp_launch_gemm_hi(p, q_hi, scales, 1, ythi, st) != hipSuccess) return STAMP_ERR_DEVICE;
    if (stamp_launch_inverse_top(p, ythi, 0, p->geom.N, P, p->Npad, st, p->hi_ksplit) != hipSuccess) return STAMP_ERR_DEVICE;
  }
  float* ytlo = reinterpret_cast<float*>(at(ws, p->ws_ytlo));
  if (p->engine == STAMP_GEMM_FP6) {
    uint8_t* a6 = at(ws, p->ws_a6);
    if (stamp_launch_repack6(p, q_lo, a6, st) != hipSuccess) return STAMP_ERR_DEVICE;
    if (stamp_launch_gemm_lo6(p, a6, scales, fused ? 2 : 1, fused ? Y : ytlo, fused ? P : nullptr, st, own) != hipSuccess)
      return STAMP_ERR_DEVICE;
  } else {
    if (stamp_launch_gemm_lo(p, q_lo, scales, fused ? 2 : 1, fused ? Y : ytlo, fused ? P : nullptr, st) != hipSuccess)
      return STAMP_ERR_DEVICE;
  }
  if (!fused && stamp_launch_inverse_bottom(p, ytlo, 0, P, p->Npad, p->geom.N, p->bias_dev, Y, st) != hipSuccess)
    return STAMP_ERR_DEVICE;
  return STAMP_OK;
}

// general path, steps 1-2: forward transform level by level, then the row quantizer
stamp_status_t gen_quantize(const stamp_plan* p, const void* X, int8_t* q_hi, uint8_t* q_lo, float* scales, void* ws, hipStream_t st) {
  float* const tb[3] = {reinterpret_cast<float*>(at(ws, p->ws_T[0])), reinterpret_cast<float*>(at(ws, p->ws_T[1])),
                        reinterpret_cast<float*>(at(ws, p->ws_T[2]))};
  float* T = nullptr;
  if (stamp_gen_forward(p, X, tb, &T, st) != hipSuccess) return STAMP_ERR_DEVICE;
  const hipError_t e = p->gen.group ? stamp_launch_quant_rows_grouped(p, T, q_hi, scales, st)
                                    : stamp_launch_quant_rows_f32(p, T, q_hi, q_lo, scales, st);
  return e == hipSuccess ? STAMP_OK : STAMP_ERR_DEVICE;
}

}  // namespace

extern "C" {

const char* stamp_status_string(stamp_status_t s) {
  switch (s) {
    case STAMP_OK: return "ok";
    case STAMP_ERR_NULL: return "null pointer";
    case STAMP_ERR_SHAPE: return "inconsistent shape or parameter";
    case STAMP_ERR_UNSUPPORTED: return "setting not implemented by this library";
    case STAMP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case STAMP_ERR_ALLOC: return "device allocation failed";
    case STAMP_ERR_DEVICE: return "HIP runtime error";
  }
  return "unknown status";
}

stamp_status_t stamp_plan_create(const stamp_plan_desc_t* desc, const void* W_dev, const float* bias_dev,
                                 void* hip_stream, stamp_plan_t** out) {
  if (desc == nullptr || out == nullptr) return STAMP_ERR_NULL;
  *out = nullptr;
  StampGeom g;
  int fused_ok = 0;
  StampGen gen;
  stamp_status_t vs = validate(desc, &g, &fused_ok, &gen);
  if (vs != STAMP_OK) return vs;
  if (W_dev == nullptr) return STAMP_ERR_NULL;

  stamp_plan* p = new (std::nothrow) stamp_plan;
  if (p == nullptr) return STAMP_ERR_ALLOC;
  memset(p, 0, sizeof(*p));
  p->desc = *desc;
  p->geom = g;
  p->gen = gen;
  p->fused_ok = fused_ok && (g.ident || g.N % 2 == 0);  // the fused inverse stores pairs of columns: even d_out
  p->unfused = 0;
  p->engine = STAMP_GEMM_FP6;
  p->Kpad = ((g.d + 127) / 128) * 128;
  p->Npad = ((g.N + 255) / 256) * 256;
  p->Mpad = ((g.B * g.s + 255) / 256) * 256;
  p->hi_ksplit = gen.group ? 1 : stamp_hi_ksplit(p, g.k);
  p->hi_ksplit_own = gen.group ? 1 : stamp_hi_ksplit(p, g.khi);
  layout_workspace(p);

  // physical row of every STaMP slot
  p->row_of_coeff = static_cast<int32_t*>(malloc(sizeof(int32_t) * (size_t)g.s));
  if (p->row_of_coeff == nullptr) { delete p; return STAMP_ERR_ALLOC; }
  if (g.ident)
    for (int q = 0; q < g.s; ++q) p->row_of_coeff[q] = q;
  else
    for (int q = 0; q < g.k; ++q) p->row_of_coeff[q] = q * g.R;
  for (int j = 0; j < g.k && !g.ident; ++j)
    for (int e = 1; e < g.R; ++e) {
      const int slot = g.is2d ? stamp_slot_of_block_e_2d(j / g.G, j % g.G, e, g.G) : stamp_slot_of_block_e_1d(j, e, g.k);
      p->row_of_coeff[slot] = j * g.R + e;
    }

  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  uint32_t* colmax = nullptr;
  bool ok = hipMalloc(reinterpret_cast<void**>(&p->qW_dev), (size_t)p->Npad * p->Kpad) == hipSuccess &&
            hipMalloc(reinterpret_cast<void**>(&p->qW6_dev), stamp_b6_bytes(p)) == hipSuccess &&
            hipMalloc(reinterpret_cast<void**>(&p->sw_dev), sizeof(float) * p->Npad) == hipSuccess &&
            hipMalloc(reinterpret_cast<void**>(&p->colsum_dev), sizeof(float) * p->Npad) == hipSuccess &&
            hipMalloc(reinterpret_cast<void**>(&colmax), sizeof(uint32_t) * g.N) == hipSuccess;
  if (ok && bias_dev != nullptr) ok = hipMalloc(reinterpret_cast<void**>(&p->bias_dev), sizeof(float) * p->Npad) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    if (colmax) (void)hipFree(colmax);
    stamp_plan_destroy(p);
    return STAMP_ERR_ALLOC;
  }
  // weights given in bf16 are widened once (exactly) into a temporary that the plan-time kernels read
  const float* Wf = static_cast<const float*>(W_dev);
  float* wtmp = nullptr;
  if (desc->w_dtype == STAMP_BF16) {
    const size_t nw = (size_t)g.d * g.N;
    if (hipMalloc(reinterpret_cast<void**>(&wtmp), nw * sizeof(float)) != hipSuccess) {
      (void)hipGetLastError();
      (void)hipFree(colmax);
      stamp_plan_destroy(p);
      return STAMP_ERR_ALLOC;
    }
    Wf = wtmp;
  }
  bool dev_ok = true;
  if (wtmp != nullptr) dev_ok = stamp_launch_bf16_to_f32(W_dev, wtmp, (size_t)g.d * g.N, st) == hipSuccess;
  if (dev_ok && bias_dev != nullptr) {
    dev_ok = hipMemsetAsync(p->bias_dev, 0, sizeof(float) * p->Npad, st) == hipSuccess &&
             hipMemcpyAsync(p->bias_dev, bias_dev, sizeof(float) * g.N, hipMemcpyDeviceToDevice, st) == hipSuccess;
  }
  if (dev_ok) dev_ok = stamp_launch_weight_quant(p, Wf, st, colmax) == hipSuccess;
  if (dev_ok) dev_ok = stamp_launch_weight_quant6(p, Wf, colmax, st) == hipSuccess;
  if (dev_ok && gen.kind != kGenNone) dev_ok = stamp_gen_plan_tables(p, Wf, st) == hipSuccess;
  // the scratch buffers must outlive the kernels just enqueued: hipFree waits for the device
  (void)hipFree(colmax);
  if (wtmp != nullptr) (void)hipFree(wtmp);
  if (!dev_ok) {
    stamp_plan_destroy(p);
    return STAMP_ERR_DEVICE;
  }
  *out = p;
  return STAMP_OK;
}

stamp_status_t stamp_plan_destroy(stamp_plan_t* p) {
  if (p == nullptr) return STAMP_ERR_NULL;
  if (p->qW_dev) (void)hipFree(p->qW_dev);
  if (p->qW6_dev) (void)hipFree(p->qW6_dev);
  if (p->sw_dev) (void)hipFree(p->sw_dev);
  if (p->colsum_dev) (void)hipFree(p->colsum_dev);
  if (p->bias_dev) (void)hipFree(p->bias_dev);
  stamp_gen_plan_free(p);
  free(p->row_of_coeff);
  delete p;
  return STAMP_OK;
}

size_t stamp_plan_workspace_bytes(const stamp_plan_t* p) { return p ? p->ws_total : 0; }

int32_t stamp_plan_hi_rows(const stamp_plan_t* p) { return p ? p->geom.k : 0; }

stamp_status_t stamp_plan_set_unfused(stamp_plan_t* p, int32_t unfused) {
  if (p == nullptr) return STAMP_ERR_NULL;
  if (p->gen.kind != kGenNone) return STAMP_OK;  // the general path has one implementation
  p->unfused = unfused ? 1 : 0;
  layout_workspace(p);
  return STAMP_OK;
}

stamp_status_t stamp_plan_set_gemm_engine(stamp_plan_t* p, int32_t engine) {
  if (p == nullptr) return STAMP_ERR_NULL;
  if (engine != STAMP_GEMM_INT8 && engine != STAMP_GEMM_FP6) return STAMP_ERR_UNSUPPORTED;
  p->engine = engine;
  return STAMP_OK;
}

stamp_status_t stamp_plan_row_of_coeff(const stamp_plan_t* p, int32_t* host_out) {
  if (p == nullptr || host_out == nullptr) return STAMP_ERR_NULL;
  memcpy(host_out, p->row_of_coeff, sizeof(int32_t) * (size_t)p->geom.s);
  return STAMP_OK;
}

stamp_status_t stamp_quantize_act(const stamp_plan_t* p, const void* X, int8_t* q_hi, uint8_t* q_lo, float* scales,
                                  void* ws, size_t ws_bytes, void* hip_stream) {
  if (p == nullptr || X == nullptr || q_hi == nullptr || scales == nullptr) return STAMP_ERR_NULL;
  if (q_lo == nullptr && !p->gen.group) return STAMP_ERR_NULL;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  if (p->gen.kind != kGenNone) {
    if (!ws_ok(p, ws, ws_bytes, p->ws_total)) return STAMP_ERR_WORKSPACE;
    return gen_quantize(p, X, q_hi, q_lo, scales, ws, st);
  }
  if (!ws_ok(p, ws, ws_bytes, p->ws_qhi)) return STAMP_ERR_WORKSPACE;  // needs the block sums and row maxima only
  hipError_t e = stamp_launch_actquant(p, X, q_hi, q_lo, scales, reinterpret_cast<float*>(at(ws, p->ws_abot)),
                                       reinterpret_cast<uint32_t*>(at(ws, p->ws_rowmax)),
                                       reinterpret_cast<uint32_t*>(at(ws, p->ws_gpart)), st);
  return e == hipSuccess ? STAMP_OK : STAMP_ERR_DEVICE;
}

stamp_status_t stamp_linear_forward_q(const stamp_plan_t* p, const int8_t* q_hi, const uint8_t* q_lo,
                                      const float* scales, void* Y, void* ws, size_t ws_bytes, void* hip_stream) {
  if (p == nullptr || q_hi == nullptr || scales == nullptr || Y == nullptr) return STAMP_ERR_NULL;
  if (q_lo == nullptr && !p->gen.group) return STAMP_ERR_NULL;
  if (!ws_ok(p, ws, ws_bytes, p->ws_total)) return STAMP_ERR_WORKSPACE;
  return forward_q(p, q_hi, q_lo, scales, Y, ws, reinterpret_cast<hipStream_t>(hip_stream), false);
}

stamp_status_t stamp_linear_forward(const stamp_plan_t* p, const void* X, void* Y, void* ws, size_t ws_bytes,
                                    void* hip_stream) {
  if (p == nullptr || X == nullptr || Y == nullptr) return STAMP_ERR_NULL;
  if (!ws_ok(p, ws, ws_bytes, p->ws_total)) return STAMP_ERR_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  int8_t* q_hi = reinterpret_cast<int8_t*>(at(ws, p->ws_qhi));
  uint8_t* q_lo = at(ws, p->ws_qlo);
  float* scales = reinterpret_cast<float*>(at(ws, p->ws_scales));
  if (p->gen.kind != kGenNone) {
    if (p->gen.group) {
      q_hi = reinterpret_cast<int8_t*>(at(ws, p->ws_codes8));
      scales = reinterpret_cast<float*>(at(ws, p->ws_scalesg));
    }
    const stamp_status_t qs = gen_quantize(p, X, q_hi, q_lo, scales, ws, st);
    return qs != STAMP_OK ? qs : forward_q(p, q_hi, q_lo, scales, Y, ws, st, true);
  }
  hipError_t e = stamp_launch_actquant(p, X, q_hi, q_lo, scales, reinterpret_cast<float*>(at(ws, p->ws_abot)),
                                       reinterpret_cast<uint32_t*>(at(ws, p->ws_rowmax)),
                                       reinterpret_cast<uint32_t*>(at(ws, p->ws_gpart)), st);
  if (e != hipSuccess) return STAMP_ERR_DEVICE;
  return forward_q(p, q_hi, q_lo, scales, Y, ws, st, true);
}

stamp_status_t stamp_linear_forward_static(const stamp_plan_t* p, const void* X, void* Y, void* hip_stream) {
  if (p == nullptr || X == nullptr || Y == nullptr) return STAMP_ERR_NULL;
  if (p->ws_total > STAMP_STATIC_SCRATCH_BYTES) return STAMP_ERR_WORKSPACE;  // the plan needs more than the static array holds
  void* ws = nullptr;
  const stamp_status_t ss = static_scratch(&ws);
  if (ss != STAMP_OK) return ss;
  return stamp_linear_forward(p, X, Y, ws, STAMP_STATIC_SCRATCH_BYTES, hip_stream);
}

stamp_status_t stamp_inverse(const stamp_plan_t* p, const float* Yt, int32_t n_cols, void* Y, void* ws, size_t ws_bytes,
                             void* hip_stream) {
  if (p == nullptr || Yt == nullptr || Y == nullptr) return STAMP_ERR_NULL;
  if (n_cols < 1) return STAMP_ERR_SHAPE;
  if (p->gen.kind != kGenNone) {
    // two [batch, seq_len, n_cols] fp32 buffers for the levels; Yt itself is only read
    const size_t one = align256((size_t)p->geom.B * p->geom.s * (size_t)n_cols * sizeof(float));
    if (!ws_ok(p, ws, ws_bytes, 2 * one)) return STAMP_ERR_WORKSPACE;
    hipStream_t stg = reinterpret_cast<hipStream_t>(hip_stream);
    float* const yt[3] = {const_cast<float*>(Yt), reinterpret_cast<float*>(ws), reinterpret_cast<float*>(at(ws, one))};
    const float* gbias = (n_cols == p->geom.N) ? p->bias_dev : nullptr;
    return stamp_gen_inverse(p, yt, n_cols, gbias, Y, stg) == hipSuccess ? STAMP_OK : STAMP_ERR_DEVICE;
  }
  if (p->geom.ident) return STAMP_ERR_UNSUPPORTED;  // nothing to invert
  const size_t need = (size_t)p->geom.B * p->geom.k * (size_t)n_cols * sizeof(float);
  if (!ws_ok(p, ws, ws_bytes, need)) return STAMP_ERR_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  float* P = reinterpret_cast<float*>(ws);
  if (stamp_launch_inverse_top(p, Yt, 1, n_cols, P, n_cols, st) != hipSuccess) return STAMP_ERR_DEVICE;
  const float* bias = (n_cols == p->geom.N) ? p->bias_dev : nullptr;
  if (stamp_launch_inverse_bottom(p, Yt, 1, P, n_cols, n_cols, bias, Y, st) != hipSuccess) return STAMP_ERR_DEVICE;
  return STAMP_OK;
}

stamp_status_t stamp_debug_gemm_acc(const stamp_plan_t* p, const int8_t* q_hi, const uint8_t* q_lo, int32_t* acc,
                                    void* hip_stream) {
  if (p == nullptr || q_hi == nullptr || q_lo == nullptr || acc == nullptr) return STAMP_ERR_NULL;
  if (p->gen.group) return STAMP_ERR_UNSUPPORTED;  // per-block scales: there is no single integer sum per output
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  // accumulator mode never reads the activation scales
  if (p->geom.k > 0 && stamp_launch_gemm_hi(p, q_hi, nullptr, 0, acc, st) != hipSuccess) return STAMP_ERR_DEVICE;
  if (p->engine == STAMP_GEMM_FP6) {
    // parity aid, not a timed path: the converted operand lives in a temporary of its own
    uint8_t* a6 = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&a6), stamp_a6_bytes(p)) != hipSuccess) { (void)hipGetLastError(); return STAMP_ERR_ALLOC; }
    const bool ok = stamp_launch_repack6(p, q_lo, a6, st) == hipSuccess &&
                    stamp_launch_gemm_lo6(p, a6, nullptr, 0, acc, nullptr, st) == hipSuccess;
    (void)hipFree(a6);  // waits for the kernels above
    return ok ? STAMP_OK : STAMP_ERR_DEVICE;
  }
  if (stamp_launch_gemm_lo(p, q_lo, nullptr, 0, acc, nullptr, st) != hipSuccess) return STAMP_ERR_DEVICE;
  return STAMP_OK;
}

stamp_status_t stamp_debug_run_stage(const stamp_plan_t* p, int32_t stage, const void* X, int8_t* q_hi, uint8_t* q_lo,
                                     float* scales, void* Y, void* ws, size_t ws_bytes, void* hip_stream) {
  if (p == nullptr || X == nullptr || q_hi == nullptr || q_lo == nullptr || scales == nullptr || Y == nullptr)
    return STAMP_ERR_NULL;
  if (stage < 0 || stage > 6) return STAMP_ERR_SHAPE;
  if (p->gen.kind != kGenNone) return STAMP_ERR_UNSUPPORTED;  // the general path has no separately launchable stages
  if (stage == 6 && p->engine != STAMP_GEMM_FP6) return STAMP_ERR_UNSUPPORTED;
  if (stage == 5 && p->fused_ok && !p->unfused) return STAMP_ERR_UNSUPPORTED;
  if (!ws_ok(p, ws, ws_bytes, p->ws_total)) return STAMP_ERR_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  float* abot = reinterpret_cast<float*>(at(ws, p->ws_abot));
  uint32_t* rowmax = reinterpret_cast<uint32_t*>(at(ws, p->ws_rowmax));
  uint32_t* gpart = reinterpret_cast<uint32_t*>(at(ws, p->ws_gpart));
  float* ythi = reinterpret_cast<float*>(at(ws, p->ws_ythi));
  float* P = reinterpret_cast<float*>(at(ws, p->ws_P));
  float* ytlo = reinterpret_cast<float*>(at(ws, p->ws_ytlo));
  const bool fused = p->fused_ok && !p->unfused;
  hipError_t e = hipSuccess;
  if (p->geom.ident) {
    // stages of a plan without a transform: 0 quantization, 2 the 8-bit rows' GEMM, 3 their output pass,
    // 6 FP6 conversion, 4 the 4-bit rows' GEMM; 1 and 5 do not exist
    switch (stage) {
      case 0: e = stamp_launch_actquant(p, X, q_hi, q_lo, scales, abot, rowmax, gpart, st, 1); break;
      case 2: if (p->geom.k > 0) e = stamp_launch_gemm_hi(p, q_hi, scales, 1, ythi, st); break;
      case 3: e = stamp_launch_hi_rows_out(p, ythi, Y, st, p->hi_ksplit); break;
      case 4:
        if (p->engine == STAMP_GEMM_FP6) e = stamp_launch_gemm_lo6(p, at(ws, p->ws_a6), scales, 3, Y, nullptr, st);
        else e = stamp_launch_gemm_lo(p, q_lo, scales, 3, Y, nullptr, st);
        break;
      case 6: e = stamp_launch_repack6(p, q_lo, at(ws, p->ws_a6), st); break;
      default: return STAMP_ERR_UNSUPPORTED;
    }
    return e == hipSuccess ? STAMP_OK : STAMP_ERR_DEVICE;
  }
  switch (stage) {
    case 0: e = stamp_launch_actquant(p, X, q_hi, q_lo, scales, abot, rowmax, gpart, st, 1); break;
    case 1: e = stamp_launch_actquant(p, X, q_hi, q_lo, scales, abot, rowmax, gpart, st, 2); break;
    case 2:
      if (own_top(p)) e = stamp_launch_block_sums_own(p, q_hi, scales, ythi, P, st);
      else if (stamp_hi_top_fused(p)) e = stamp_launch_gemm_hi(p, q_hi, scales, 2, P, st, p->Npad);
      else
        e = stamp_hi_rows_are_block_sums(p) ? stamp_launch_gemm_hi(p, q_hi, scales, 1, P, st, p->Npad)
                                            : stamp_launch_gemm_hi(p, q_hi, scales, 1, ythi, st);
      break;
    case 3:  // nothing to launch when the plan has no top levels, or when the 8-bit rows' GEMM has run them
      if (!own_top(p) && !stamp_hi_rows_are_block_sums(p) && !stamp_hi_top_fused(p))
        e = stamp_launch_inverse_top(p, ythi, 0, p->geom.N, P, p->Npad, st, p->hi_ksplit);
      break;
    case 4:
      if (p->engine == STAMP_GEMM_FP6)
        e = stamp_launch_gemm_lo6(p, at(ws, p->ws_a6), scales, fused ? 2 : 1, fused ? Y : (void*)ytlo, fused ? P : nullptr, st,
                                  own_top(p));
      else
        e = stamp_launch_gemm_lo(p, q_lo, scales, fused ? 2 : 1, fused ? Y : (void*)ytlo, fused ? P : nullptr, st);
      break;
    case 6: e = stamp_launch_repack6(p, q_lo, at(ws, p->ws_a6), st); break;
    case 5: e = stamp_launch_inverse_bottom(p, ytlo, 0, P, p->Npad, p->geom.N, p->bias_dev, Y, st); break;
  }
  return e == hipSuccess ? STAMP_OK : STAMP_ERR_DEVICE;
}

stamp_status_t stamp_debug_weight_codes(const stamp_plan_t* p, int8_t* qW_host, float* sw_host) {
  if (p == nullptr || qW_host == nullptr || sw_host == nullptr) return STAMP_ERR_NULL;
  const int d = p->geom.d, N = p->geom.N;
  if (p->gen.group) {
    // per-block scales: codes [d_in, d_out], scales [d_in / 64][d_out]
    const int Npad = ((N + 127) / 128) * 128, G = d / 64;
    int8_t* tq = static_cast<int8_t*>(malloc((size_t)Npad * d));
    float* ts = static_cast<float*>(malloc(sizeof(float) * (size_t)G * Npad));
    bool ok = tq != nullptr && ts != nullptr && hipDeviceSynchronize() == hipSuccess &&
              hipMemcpy(tq, p->qWg_dev, (size_t)Npad * d, hipMemcpyDeviceToHost) == hipSuccess &&
              hipMemcpy(ts, p->swg_dev, sizeof(float) * (size_t)G * Npad, hipMemcpyDeviceToHost) == hipSuccess;
    if (ok) {
      for (int n = 0; n < N; ++n)
        for (int c = 0; c < d; ++c) qW_host[(size_t)c * N + n] = tq[(size_t)n * d + c];
      for (int gi = 0; gi < G; ++gi)
        for (int n = 0; n < N; ++n) sw_host[(size_t)gi * N + n] = ts[(size_t)gi * Npad + n];
    }
    free(tq);
    free(ts);
    return ok ? STAMP_OK : STAMP_ERR_DEVICE;
  }
  int8_t* tmp = static_cast<int8_t*>(malloc((size_t)p->Npad * p->Kpad));
  if (tmp == nullptr) return STAMP_ERR_ALLOC;
  if (hipDeviceSynchronize() != hipSuccess ||
      hipMemcpy(tmp, p->qW_dev, (size_t)p->Npad * p->Kpad, hipMemcpyDeviceToHost) != hipSuccess ||
      hipMemcpy(sw_host, p->sw_dev, sizeof(float) * N, hipMemcpyDeviceToHost) != hipSuccess) {
    free(tmp);
    return STAMP_ERR_DEVICE;
  }
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < d; ++c) {
      const int g16 = c >> 4, cc = c & 15, half = cc >> 3, c8 = cc & 7;
      const int pos = half * 8 + (c8 & 1) * 4 + (c8 >> 1);
      qW_host[(size_t)c * N + n] = (int8_t)(tmp[stamp_w_offset(n, g16 * 16 + pos, p->Kpad)] / 16);
    }
  free(tmp);
  return STAMP_OK;
}

}  // extern "C"
