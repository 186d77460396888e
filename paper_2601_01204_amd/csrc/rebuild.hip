// Building the next cache from the kept tokens and the new frame (paper Sec. 3.2 keep
// set, Sec. 3.3 Eq. 7-9): stable compaction along the keep list, per-channel key groups
// re-quantised where their ordered membership changed, value codes carried, the new
// frame's values quantised per token.
//
// Everything here decides integers that are compared bit-for-bit, so the arithmetic is
// fp32 with one rounding per operation: s = (max - min) / (2^b - 1) with an IEEE divide,
// z = rint(-min / s), code = clamp(int(rint(x / s)) + z, 0, 2^b - 1), rint to nearest
// even.  A constant group takes s = |min| (1 when min is 0).
#include "kvx_dev.h"

#include <algorithm>
#include <type_traits>

namespace kvx {

__device__ __forceinline__ float bf16_to_f32(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }

__device__ __forceinline__ void quant_params(float mn, float mx, int levels, float& s, int32_t& z) {
  s = (mx - mn) / (float)levels;
  if (mx == mn) s = (mn != 0.f) ? fabsf(mn) : 1.0f;
  z = (int32_t)rintf((-mn) / s);
}

// 16-bit metadata format (Eq. 8 with the scale rounded up to its storage format first).
__device__ __forceinline__ float half_bits_to_f32(uint32_t h16) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h16); }
__device__ __forceinline__ uint16_t f32_to_half_bits(float x) { return __builtin_bit_cast(uint16_t, (_Float16)x); }   // exact for the values stored here
// smallest fp32 >= x (x > 0) with at most 24 - drop significant bits
__device__ __forceinline__ float round_up_drop(float x, int drop) {
  uint32_t u = __float_as_uint(x);
  const uint32_t mask = (1u << drop) - 1u;
  if (u & mask) u = (u | mask) + 1u;
  return __uint_as_float(u);
}
__device__ __forceinline__ float clamp_scale16(float a, bool& clipped) {
  clipped = !(a >= kMeta16ScaleMin && a <= kMeta16ScaleMax);
  return fminf(fmaxf(a, kMeta16ScaleMin), kMeta16ScaleMax);
}
__device__ __forceinline__ int32_t zero_point16(float mn, float s, bool& clipped) {
  const float zf = rintf((-mn) / s);
  clipped = !(zf >= (float)kMeta16ZMin && zf <= (float)kMeta16ZMax);
  return (int32_t)fminf(fmaxf(zf, (float)kMeta16ZMin), (float)kMeta16ZMax);
}
// keys: a = s_raw * scale_log2 rounded up to 7 significant bits; s = a * inv_scale_log2
__device__ __forceinline__ void quant_params16_k(float mn, float mx, int levels, float c_log2, float inv_c, float& a, float& s, int32_t& z, bool& clipped) {
  float s_raw = (mx - mn) / (float)levels;
  if (mx == mn) s_raw = (mn != 0.f) ? fabsf(mn) : 1.0f;
  bool c0, c1;
  a = clamp_scale16(round_up_drop(s_raw * c_log2, 17), c0);
  s = a * inv_c;
  z = zero_point16(mn, s, c1);
  clipped = c0 || c1;
}
// values: s rounded up to a half (11 significant bits)
__device__ __forceinline__ void quant_params16_v(float mn, float mx, int levels, float& s, int32_t& z, bool& clipped) {
  float s_raw = (mx - mn) / (float)levels;
  if (mx == mn) s_raw = (mn != 0.f) ? fabsf(mn) : 1.0f;
  bool c0, c1;
  s = clamp_scale16(round_up_drop(s_raw, 13), c0);
  z = zero_point16(mn, s, c1);
  clipped = c0 || c1;
}

// fl(float(half) * f) in one instruction: the low / high half of w times the fp32 f (v_fma_mix_f32, addend +0).
__device__ __forceinline__ float mix_mul_lo(uint32_t w, float f) {
  float r;
  asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(f));
  return r;
}
__device__ __forceinline__ float mix_mul_hi(uint32_t w, float f) {
  float r;
  asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(f));
  return r;
}

__device__ __forceinline__ int quant_code(float x, float s, int32_t z, int levels) {
  const int q = (int)rintf(x / s) + z;
  return min(max(q, 0), levels);
}

// x / s for many x and one s.  The correctly rounded fp32 quotient is what the compiler's
// own expansion of `/` computes as a reciprocal refined by one Newton step followed by two
// fused residual corrections of the quotient; that expansion also rescales operands with
// extreme exponents.  With the refined reciprocal computed once per scale and s in a range
// where no rescaling happens, the five fused operations below are that expansion's core and
// give the same bits.  Scales outside the range take the plain division.
struct Divider {
  float s, r;
  bool safe;
};
__device__ __forceinline__ Divider make_divider(float s) {
  Divider d;
  d.s = s;
  const float r0 = __builtin_amdgcn_rcpf(s);
  const float e0 = __builtin_fmaf(-s, r0, 1.0f);
  d.r = __builtin_fmaf(e0, r0, r0);
  const float a = fabsf(s);
  d.safe = a > 0x1p-60f && a < 0x1p60f;
  return d;
}
__device__ __forceinline__ float div_by(float x, const Divider& d) {
  if (!d.safe || !(fabsf(x) < 0x1p60f)) return x / d.s;
  const float q0 = x * d.r;
  const float e1 = __builtin_fmaf(-d.s, q0, x);
  const float q1 = __builtin_fmaf(e1, d.r, q0);
  const float e2 = __builtin_fmaf(-d.s, q1, x);
  return __builtin_fmaf(e2, d.r, q1);
}
// The five fused operations alone, for a scale already known to be in the safe range.
__device__ __forceinline__ float div_fast(float x, float s, float r) {
  const float q0 = x * r;
  const float e1 = __builtin_fmaf(-s, q0, x);
  const float q1 = __builtin_fmaf(e1, r, q0);
  const float e2 = __builtin_fmaf(-s, q1, x);
  return __builtin_fmaf(e2, r, q1);
}
__device__ __forceinline__ int quant_code_div(float x, const Divider& d, int32_t z, int levels) {
  const int q = (int)rintf(div_by(x, d)) + z;
  return min(max(q, 0), levels);
}

// 16 consecutive channels of one row as fp32, from a quantised row (with that row's group
// metadata) or from an input row.
template <int B>
__device__ __forceinline__ void unpack16(const uint8_t* p, uint32_t (&w)[4]) {
  if constexpr (B == 2) {
    w[0] = *reinterpret_cast<const uint32_t*>(p);
  } else if constexpr (B == 4) {
    const uint2 t = *reinterpret_cast<const uint2*>(p);
    w[0] = t.x; w[1] = t.y;
  } else {
    const uint4 t = *reinterpret_cast<const uint4*>(p);
    w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
  }
}
template <int B>
__device__ __forceinline__ int code16(const uint32_t (&w)[4], int e) {
  if constexpr (B == 2) return (int)((w[0] >> (2 * e)) & 3u);
  if constexpr (B == 4) return (int)((w[e >> 3] >> (4 * (e & 7))) & 0xFu);
  return (int)((w[e >> 2] >> (8 * (e & 3))) & 0xFFu);
}
template <int B>
__device__ __forceinline__ void pack16(const int (&code)[16], uint8_t* p) {
  if constexpr (B == 2) {
    uint32_t w = 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) w |= (uint32_t)code[e] << (2 * e);
    *reinterpret_cast<uint32_t*>(p) = w;
  } else if constexpr (B == 4) {
    uint32_t w0 = 0, w1 = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      w0 |= (uint32_t)code[e] << (4 * e);
      w1 |= (uint32_t)code[8 + e] << (4 * e);
    }
    *reinterpret_cast<uint2*>(p) = make_uint2(w0, w1);
  } else {
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < 16; ++e) w[e >> 2] |= (uint32_t)code[e] << (8 * (e & 3));
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// 16 codes (floats holding integers 0 .. 2^B - 1) packed into a row piece: 16-bit halves are built in fp32 (exact:
// at most 16 bits) by fused multiply-adds, converted once and joined.
template <int B>
__device__ __forceinline__ void pack16f(const float (&c)[16], uint8_t* p) {
  constexpr int kPer = 16 / B;                  // codes per 16-bit half: 8, 4 or 2
  constexpr float kMul = (float)(1 << B);
  uint32_t half16[16 / kPer];
#pragma unroll
  for (int hh = 0; hh < 16 / kPer; ++hh) {
    float acc = c[hh * kPer + kPer - 1];
#pragma unroll
    for (int e = kPer - 2; e >= 0; --e) acc = __builtin_fmaf(acc, kMul, c[hh * kPer + e]);
    half16[hh] = (uint32_t)acc;
  }
  if constexpr (B == 2) {
    *reinterpret_cast<uint32_t*>(p) = half16[0] | (half16[1] << 16);
  } else if constexpr (B == 4) {
    *reinterpret_cast<uint2*>(p) = make_uint2(half16[0] | (half16[1] << 16), half16[2] | (half16[3] << 16));
  } else {
    *reinterpret_cast<uint4*>(p) = make_uint4(half16[0] | (half16[1] << 16), half16[2] | (half16[3] << 16),
                                              half16[4] | (half16[5] << 16), half16[6] | (half16[7] << 16));
  }
}

__device__ __forceinline__ void load_input16(const void* base, int64_t off, int in_f32, float (&x)[16]) {
  if (in_f32) {
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + off);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float4 t = p[i];
      x[4 * i] = t.x; x[4 * i + 1] = t.y; x[4 * i + 2] = t.z; x[4 * i + 3] = t.w;
    }
  } else {
    const uint4* p = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(base) + off);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint4 t = p[i];
      const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        x[8 * i + 2 * k] = __uint_as_float(w[k] << 16);
        x[8 * i + 2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
      }
    }
  }
}

// Keys.  One block = 64 consecutive positions of the next cache for one head (one key
// group of 64, or two of 32).  A group wholly below the first dropped position has the
// same ordered members as before and is copied verbatim; every other group is rebuilt
// from the fp32 values of its members: de-quantised codes for surviving tokens, input
// values for the new frame.
// Slot layout (SLOTS): the block's 64 positions are 64 consecutive slots of the one buffer; a row keeps its token
// unless the keep/drop decision freed it (newtok >= 0) or it lies in the never-used tail, and then takes the call's
// token newtok; a group that received no token is left as it is (the whole block returns early when neither of
// its groups did), every other group is rebuilt in place: each thread reads its own row piece before any write,
// and the group's old scale and zero-point are read before the second barrier and replaced after it.
template <int B, bool M16, bool SLOTS>
__global__ __launch_bounds__(256, 8) void rebuild_k_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.z];
  const int h = blockIdx.y;
  const int t_c = it.t_c;
  const int t_new = min(t_c + g.n_new, g.budget);
  const int p0 = blockIdx.x * kTileK;
  if (p0 >= t_new) return;
  const uint8_t* cur = cache_half(g, it.cache, it.cur);
  uint8_t* nxt = cache_half(g, it.cache, SLOTS ? it.cur : it.cur ^ 1);
  uint8_t* sc = cache_scratch(g, it.cache);
  const int32_t* keep = reinterpret_cast<const int32_t*>(sc + g.sl.keep);
  int32_t* sel = reinterpret_cast<int32_t*>(sc + g.sl.sel);
  constexpr int kRow = 8 * B;                          // bytes per key row
  const int levels = (1 << B) - 1;

  const int tid = threadIdx.x;
  const int r = tid >> 2, cb = tid & 3;                // row in block, 16-channel block
  const int p = p0 + r;
  const bool active = p < t_new;
  const int k_shift = g.k_group == 64 ? 6 : 5;       // groups of 64 or 32 tokens
  const int grp = p >> k_shift;
  __shared__ int touched[2];                           // slot layout: the block's groups that received a token
  int tok = -1;                                        // slot layout: the call's token this row receives
  int g0;                                              // compacting layout: first group whose membership changed
  bool carried;
  if constexpr (SLOTS) {
    g0 = 0;
    if (tid < 2) touched[tid] = 0;
    __syncthreads();
    if (active) tok = it.prune ? reinterpret_cast<const int32_t*>(sc + g.sl.newtok)[p] : (p >= t_c ? p - t_c : -1);
    if (tok >= 0 && cb == 0) touched[r >> k_shift] = 1;      // benign race: every writer stores 1
    __syncthreads();
    if (!touched[0] && !touched[1]) return;
    carried = !touched[r >> k_shift];
  } else {
    g0 = it.prune ? sel[1] : it.g0_host;
    carried = grp < g0;
  }

  __shared__ __attribute__((aligned(16))) float vals[kTileK][kHeadDim + 4];
  __shared__ float pmin[4][kHeadDim], pmax[4][kHeadDim];
  __shared__ __attribute__((aligned(16))) float gs[2][kHeadDim];
  __shared__ __attribute__((aligned(16))) float gr[2][kHeadDim];     // refined reciprocals of the scales
  __shared__ __attribute__((aligned(16))) int32_t gz[2][kHeadDim];
  __shared__ __attribute__((aligned(16))) float gzf[2][kHeadDim];    // the zero-points as floats
  __shared__ int unsafe_scales;                                      // some scale needs the plain division

  float x[16];
  uint32_t wsrc[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < 16; ++e) x[e] = 0.f;
  if (active) {
    const int src = SLOTS ? (tok >= 0 ? t_c + tok : p) : (it.prune ? keep[p] : p);
    if (src < t_c) {
      unpack16<B>(cur + g.lay.k_codes + ((int64_t)h * g.t_cap + src) * kRow + cb * 2 * B, wsrc);
      if (!carried && M16) {
        // 16 halfs each of logit-domain scales and 1024 + z, stored in the 0 4 1 5 2 6 3 7 order of every eight channels
        const int sg = src >> k_shift;
        const int64_t moff = ((int64_t)h * g.g_cap + sg) * kHeadDim + cb * 16;
        const uint4* ap = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(cur + g.lay.k_scale) + moff);
        const uint4* zp = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(cur + g.lay.k_zero) + moff);
        const uint4 a0 = ap[0], a1 = ap[1], z0 = zp[0], z1 = zp[1];
        const uint32_t aw[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        const uint32_t zw[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
        // word k of an octet holds channels k and k + 4, and so do the codes once masked: code - z is taken on both
        // at once as (1024 + code) - (1024 + z) in halves (integers below 2048: exact)
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int o = 0; o < 2; ++o) {
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            uint32_t cw;
            if constexpr (B == 4) {
              cw = (wsrc[o] >> (4 * k)) & 0x000F000Fu;
            } else {
              const uint32_t t = (wsrc[0] >> (16 * o + 2 * k)) & 0x0303u;      // codes k and k + 4 of the octet
              cw = (t | (t << 8)) & 0x00030003u;
            }
            const h2 d = __builtin_bit_cast(h2, cw | 0x64006400u) - __builtin_bit_cast(h2, zw[4 * o + k]);
            // s = fl(a * c), then fl(s * d): the mixed-precision multiply-add takes the half operand as it is and
            // rounds once, like a conversion (exact) followed by a multiply; the +0 addend changes nothing, no
            // product here is -0 (a, c, s > 0 and a zero difference is +0)
            const uint32_t aw2 = aw[4 * o + k], dw2 = __builtin_bit_cast(uint32_t, d);
            const float s0 = mix_mul_lo(aw2, g.inv_scale_log2), s1 = mix_mul_hi(aw2, g.inv_scale_log2);
            x[8 * o + k] = mix_mul_lo(dw2, s0);
            x[8 * o + k + 4] = mix_mul_hi(dw2, s1);
          }
        }
      } else if (!carried) {
        const int sg = src >> k_shift;
        const int64_t moff = ((int64_t)h * g.g_cap + sg) * kHeadDim + cb * 16;
        const float4* sp = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(cur + g.lay.k_scale) + moff);
        const int4* zp = reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(cur + g.lay.k_zero) + moff);
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
          const float4 sv = sp[v4];
          const int4 zv = zp[v4];
          x[4 * v4 + 0] = sv.x * (float)(code16<B>(wsrc, 4 * v4 + 0) - zv.x);
          x[4 * v4 + 1] = sv.y * (float)(code16<B>(wsrc, 4 * v4 + 1) - zv.y);
          x[4 * v4 + 2] = sv.z * (float)(code16<B>(wsrc, 4 * v4 + 2) - zv.z);
          x[4 * v4 + 3] = sv.w * (float)(code16<B>(wsrc, 4 * v4 + 3) - zv.w);
        }
      }
    } else {
      load_input16(it.k, (int64_t)(src - t_c) * g.tok_stride + (int64_t)h * g.head_stride + cb * 16, g.in_f32, x);
    }
  }
#pragma unroll
  for (int v4 = 0; v4 < 4; ++v4)
    *reinterpret_cast<float4*>(&vals[r][cb * 16 + 4 * v4]) = make_float4(x[4 * v4], x[4 * v4 + 1], x[4 * v4 + 2], x[4 * v4 + 3]);
  __syncthreads();

  if (tid == 0) unsafe_scales = 0;
  // per-channel min / max over each quarter of the rows
  {
    const int c = tid & 63, qtr = tid >> 6;
    float mn = INFINITY, mx = -INFINITY;
    if (p0 + kTileK <= t_new) {                       // all rows present: no per-row test
#pragma unroll
      for (int rr = 0; rr < 16; ++rr) {
        const float v = vals[qtr * 16 + rr][c];
        mn = fminf(mn, v);
        mx = fmaxf(mx, v);
      }
    } else {
      for (int rr = qtr * 16; rr < qtr * 16 + 16; ++rr) {
        if (p0 + rr < t_new) {
          const float v = vals[rr][c];
          mn = fminf(mn, v);
          mx = fmaxf(mx, v);
        }
      }
    }
    pmin[qtr][c] = mn;
    pmax[qtr][c] = mx;
  }
  __syncthreads();

  const int groups_in_block = kTileK >> k_shift;       // 1 or 2
  if (tid < groups_in_block * 64) {
    const int gi = tid >> 6, c = tid & 63;
    const int ggrp = (p0 >> k_shift) + gi;
    const int first_row = gi << k_shift;
    if (p0 + first_row < t_new) {
      const int64_t moff = ((int64_t)h * g.g_cap + ggrp) * kHeadDim + (M16 ? meta16_pos(c) : c);
      float s, a16 = 0.f;
      int32_t z;
      const bool group_carried = SLOTS ? !touched[gi] : ggrp < g0;
      if (SLOTS && group_carried) {
        s = 1.0f;                       // left as it is, in place: nothing to write, no row of it is quantised
        z = 0;
      } else if (group_carried) {
        if constexpr (M16) {
          a16 = half_bits_to_f32(reinterpret_cast<const uint16_t*>(cur + g.lay.k_scale)[moff]);
          s = a16 * g.inv_scale_log2;
          z = (int32_t)half_bits_to_f32(reinterpret_cast<const uint16_t*>(cur + g.lay.k_zero)[moff]) - 1024;
        } else {
          s = reinterpret_cast<const float*>(cur + g.lay.k_scale)[moff];
          z = reinterpret_cast<const int32_t*>(cur + g.lay.k_zero)[moff];
        }
      } else if constexpr (M16) {
        const int q_lo = first_row >> 4, q_hi = (first_row + g.k_group) >> 4;
        float mn = INFINITY, mx = -INFINITY;
        for (int qq = q_lo; qq < q_hi; ++qq) {
          mn = fminf(mn, pmin[qq][c]);
          mx = fmaxf(mx, pmax[qq][c]);
        }
        bool clipped;
        quant_params16_k(mn, mx, levels, g.scale_log2, g.inv_scale_log2, a16, s, z, clipped);
        if (h == 0 && c == 0) atomicAdd(&sel[2], 1);
        if (clipped) atomicAdd(&sel[5], 1);
      } else {
        const int q_lo = first_row >> 4, q_hi = (first_row + g.k_group) >> 4;
        float mn = INFINITY, mx = -INFINITY;
        for (int qq = q_lo; qq < q_hi; ++qq) {
          mn = fminf(mn, pmin[qq][c]);
          mx = fmaxf(mx, pmax[qq][c]);
        }
        quant_params(mn, mx, levels, s, z);
        if (h == 0 && c == 0) atomicAdd(&sel[2], 1);
        if (z > kZeroPointWarn || z < -kZeroPointWarn) atomicAdd(&sel[5], 1);
      }
      const Divider dv = make_divider(s);
      gs[gi][c] = s;
      gr[gi][c] = dv.r;
      gz[gi][c] = z;
      gzf[gi][c] = (float)z;
      if (!dv.safe || z >= (1 << 23) || z <= -(1 << 23)) unsafe_scales = 1;      // also: z not exact as a float
      if (SLOTS && group_carried) {
      } else if constexpr (M16) {
        reinterpret_cast<uint16_t*>(nxt + g.lay.k_scale)[moff] = f32_to_half_bits(a16);
        reinterpret_cast<uint16_t*>(nxt + g.lay.k_zero)[moff] = f32_to_half_bits((float)(1024 + z));
      } else {
        reinterpret_cast<float*>(nxt + g.lay.k_scale)[moff] = s;
        reinterpret_cast<int32_t*>(nxt + g.lay.k_zero)[moff] = z;
      }
    }
  }
  __syncthreads();

  if (active) {
    uint8_t* dst = nxt + g.lay.k_codes + ((int64_t)h * g.t_cap + p) * kRow + cb * 2 * B;
    if (SLOTS && carried) {
    } else if (carried) {
      if constexpr (B == 2) *reinterpret_cast<uint32_t*>(dst) = wsrc[0];
      else if constexpr (B == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(wsrc[0], wsrc[1]);
      else *reinterpret_cast<uint4*>(dst) = make_uint4(wsrc[0], wsrc[1], wsrc[2], wsrc[3]);
    } else {
      const int gi = r >> k_shift;
      if (unsafe_scales) {                      // block-uniform and rare
        int code[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) code[e] = quant_code(x[e], gs[gi][cb * 16 + e], gz[gi][cb * 16 + e], levels);
        pack16<B>(code, dst);
      } else {
        // rint(x / s) + z in floats: the quotient's five fused operations, then an exact integer sum (the rounded
        // quotient is an integer below 2^24 or the clamp decides; |z| < 2^23 here) clamped by one median.
        float cf[16];
        const float flev = (float)levels;
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
          const float4 sv = *reinterpret_cast<const float4*>(&gs[gi][cb * 16 + 4 * v4]);
          const float4 rv = *reinterpret_cast<const float4*>(&gr[gi][cb * 16 + 4 * v4]);
          const float4 zv = *reinterpret_cast<const float4*>(&gzf[gi][cb * 16 + 4 * v4]);
          const float sa[4] = {sv.x, sv.y, sv.z, sv.w}, ra[4] = {rv.x, rv.y, rv.z, rv.w}, za[4] = {zv.x, zv.y, zv.z, zv.w};
#pragma unroll
          for (int k = 0; k < 4; ++k)
            cf[4 * v4 + k] = __builtin_amdgcn_fmed3f(rintf(div_fast(x[4 * v4 + k], sa[k], ra[k])) + za[k], 0.f, flev);
        }
        pack16f<B>(cf, dst);
      }
    }
  }
}

// Values and token ids.  The next cache's positions [0, t_new - n) are surviving tokens,
// whose codes and (s, z) are carried; the last n positions are the new frame, quantised
// per token over groups of v_group channels.  Two kinds of blocks share the launch: copy
// blocks (a lane moves 16 bytes of one token's code row of one head, so 1, 2 or 4 lanes
// per row, and the row's metadata) and quantise blocks (64 new tokens per block, four
// lanes per token).

template <int B, bool M16>
__global__ __launch_bounds__(256) void rebuild_v_kernel(const KvxBatch b, int n_copy_blocks) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.z];
  const int h = blockIdx.y;
  const int t_c = it.t_c;
  const int t_new = min(t_c + g.n_new, g.budget);
  const int t_keep = t_new - g.n_new;      // survivors
  const int tid = threadIdx.x;
  const uint8_t* cur = cache_half(g, it.cache, it.cur);
  uint8_t* nxt = cache_half(g, it.cache, g.slots ? it.cur : it.cur ^ 1);
  const int32_t* keep = reinterpret_cast<const int32_t*>(cache_scratch(g, it.cache) + g.sl.keep);
  constexpr int kRow = 8 * B;
  const int ngv = kHeadDim / g.v_group;    // 1 or 2

  if ((int)blockIdx.x < n_copy_blocks) {
    constexpr int kLanes = kRow / 16;                      // lanes per row, 16 bytes of codes each
    const int p = blockIdx.x * (256 / kLanes) + tid / kLanes;
    const int part = tid % kLanes;
    if (p >= t_keep) return;
    const int src = it.prune ? keep[p] : p;
    const uint4 w = *reinterpret_cast<const uint4*>(cur + g.lay.v_codes + ((int64_t)h * g.t_cap + src) * kRow + part * 16);
    typedef typename std::conditional<M16, uint32_t, VMeta>::type MetaT;
    const MetaT* ms = reinterpret_cast<const MetaT*>(cur + g.lay.v_meta) + ((int64_t)h * g.t_cap + src) * ngv;
    MetaT* md = reinterpret_cast<MetaT*>(nxt + g.lay.v_meta) + ((int64_t)h * g.t_cap + p) * ngv;
    if (kLanes == 1) {
      md[0] = ms[0];
      if (ngv == 2) md[1] = ms[1];
    } else if (part < ngv) {
      md[part] = ms[part];
    }
    *reinterpret_cast<uint4*>(nxt + g.lay.v_codes + ((int64_t)h * g.t_cap + p) * kRow + part * 16) = w;
    if (h == 0 && part == 0) {
      const int32_t* ids = reinterpret_cast<const int32_t*>(cur + g.lay.ids);
      reinterpret_cast<int32_t*>(nxt + g.lay.ids)[p] = ids[src];
    }
    return;
  }

  const int levels = (1 << B) - 1;
  const int lanes_per_group = 4 / ngv;     // 4 or 2 lanes share one value group
  const int r = tid >> 2, cb = tid & 3;
  const int i_new = ((int)blockIdx.x - n_copy_blocks) * kTileK + r;     // token of the new frame
  const bool active = i_new < g.n_new;     // uniform over each group of 4 lanes
  // destination: behind the survivors, or (slot layout) the slot the selection assigned, the next unused one while filling
  int p = t_keep + i_new;
  if (g.slots && active) p = it.prune ? reinterpret_cast<const int32_t*>(cache_scratch(g, it.cache) + g.sl.assign)[i_new] : t_c + i_new;
  const int gv = cb / lanes_per_group;
  float x[16];
  float mn = INFINITY, mx = -INFINITY;
  if (active) {
    load_input16(it.v, (int64_t)i_new * g.tok_stride + (int64_t)h * g.head_stride + cb * 16, g.in_f32, x);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      mn = fminf(mn, x[e]);
      mx = fmaxf(mx, x[e]);
    }
  }
  // min / max over the lanes that share the group (executed by all lanes: no divergence around shuffles)
  mn = fminf(mn, __shfl_xor(mn, 1));
  mx = fmaxf(mx, __shfl_xor(mx, 1));
  if (lanes_per_group == 4) {
    mn = fminf(mn, __shfl_xor(mn, 2));
    mx = fmaxf(mx, __shfl_xor(mx, 2));
  }
  if (!active) return;
  float s;
  int32_t z;
  bool warn;
  if constexpr (M16) {
    quant_params16_v(mn, mx, levels, s, z, warn);
  } else {
    quant_params(mn, mx, levels, s, z);
    warn = z > kZeroPointWarn || z < -kZeroPointWarn;
  }
  int code[16];
  const Divider dv = make_divider(s);
#pragma unroll
  for (int e = 0; e < 16; ++e) code[e] = quant_code_div(x[e], dv, z, levels);
  pack16<B>(code, nxt + g.lay.v_codes + ((int64_t)h * g.t_cap + p) * kRow + cb * 2 * B);
  if ((cb % lanes_per_group) == 0) {
    if (warn) atomicAdd(reinterpret_cast<int32_t*>(cache_scratch(g, it.cache) + g.sl.sel) + 5, 1);
    if constexpr (M16) {
      reinterpret_cast<uint32_t*>(nxt + g.lay.v_meta)[((int64_t)h * g.t_cap + p) * ngv + gv] =
          (uint32_t)f32_to_half_bits(s) | ((uint32_t)f32_to_half_bits((float)(1024 + z)) << 16);
    } else {
      VMeta m;
      m.s = s;
      m.z = z;
      reinterpret_cast<VMeta*>(nxt + g.lay.v_meta)[((int64_t)h * g.t_cap + p) * ngv + gv] = m;
    }
  }
  if (h == 0 && cb == 0) reinterpret_cast<int32_t*>(nxt + g.lay.ids)[p] = it.frame * g.n + i_new;
}

// Uncompressed baseline: append the frame's K and V as bf16 rows [H][t_cap][64].
__global__ __launch_bounds__(256) void append_bf16_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.z];
  const int h = blockIdx.y;
  const int i = blockIdx.x * 32 + (threadIdx.x >> 3);
  const int c8 = (threadIdx.x & 7) * 8;
  if (i >= g.n_new) return;
  uint8_t* base = cache_half(g, it.cache, 0);
  const int64_t off = (int64_t)i * g.tok_stride + (int64_t)h * g.head_stride + c8;
  const int64_t dsto = ((int64_t)h * g.t_cap + it.t_c + i) * kHeadDim + c8;
  uint4 kk, vv;
  if (g.in_f32) {
    // fp32 input is rounded to bf16 (nearest even) for the baseline cache
    const float* kp = reinterpret_cast<const float*>(it.k) + off;
    const float* vp = reinterpret_cast<const float*>(it.v) + off;
    uint32_t kw[4], vw[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      typedef float f2 __attribute__((ext_vector_type(2)));
      typedef __bf16 b2 __attribute__((ext_vector_type(2)));
      f2 a = {kp[2 * e], kp[2 * e + 1]}, c = {vp[2 * e], vp[2 * e + 1]};
      kw[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, b2));
      vw[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(c, b2));
    }
    kk = make_uint4(kw[0], kw[1], kw[2], kw[3]);
    vv = make_uint4(vw[0], vw[1], vw[2], vw[3]);
  } else {
    kk = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(it.k) + off);
    vv = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(it.v) + off);
  }
  *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(base + g.lay.k_codes) + dsto) = kk;
  *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(base + g.lay.v_codes) + dsto) = vv;
  if (h == 0 && c8 == 0) reinterpret_cast<int32_t*>(base + g.lay.ids)[it.t_c + i] = it.frame * g.n + i;
}

void launch_rebuild_k(const KvxBatch& b, int max_tnew, hipStream_t st) {
  dim3 grid((max_tnew + kTileK - 1) / kTileK, b.g.H, b.n_items);
#define KVX_RK(B, M, S) hipLaunchKernelGGL((rebuild_k_kernel<B, M, S>), grid, dim3(256), 0, st, b)
  if (b.g.slots) {
    if (b.g.meta16) {
      if (b.g.k_bits == 2) KVX_RK(2, true, true); else KVX_RK(4, true, true);
    } else {
      switch (b.g.k_bits) {
        case 2: KVX_RK(2, false, true); break;
        case 4: KVX_RK(4, false, true); break;
        default: KVX_RK(8, false, true); break;
      }
    }
    return;
  }
  if (b.g.meta16) {
    if (b.g.k_bits == 2) KVX_RK(2, true, false); else KVX_RK(4, true, false);
    return;
  }
  switch (b.g.k_bits) {
    case 2: KVX_RK(2, false, false); break;
    case 4: KVX_RK(4, false, false); break;
    default: KVX_RK(8, false, false); break;
  }
#undef KVX_RK
}

void launch_rebuild_v(const KvxBatch& b, int max_tnew, hipStream_t st) {
  const int rows_per_block = 256 / (b.g.v_bits / 2);           // 16 bytes of codes per lane
  // the slot layout never moves a survivor: only the call's tokens are written
  const int n_copy_blocks = b.g.slots ? 0 : (std::max(max_tnew - b.g.n_new, 0) + rows_per_block - 1) / rows_per_block;
  dim3 grid(n_copy_blocks + (b.g.n_new + kTileK - 1) / kTileK, b.g.H, b.n_items);
  if (b.g.meta16) {
    switch (b.g.v_bits) {
      case 2: hipLaunchKernelGGL((rebuild_v_kernel<2, true>), grid, dim3(256), 0, st, b, n_copy_blocks); break;
      case 4: hipLaunchKernelGGL((rebuild_v_kernel<4, true>), grid, dim3(256), 0, st, b, n_copy_blocks); break;
      default: hipLaunchKernelGGL((rebuild_v_kernel<8, true>), grid, dim3(256), 0, st, b, n_copy_blocks); break;
    }
    return;
  }
  switch (b.g.v_bits) {
    case 2: hipLaunchKernelGGL((rebuild_v_kernel<2, false>), grid, dim3(256), 0, st, b, n_copy_blocks); break;
    case 4: hipLaunchKernelGGL((rebuild_v_kernel<4, false>), grid, dim3(256), 0, st, b, n_copy_blocks); break;
    default: hipLaunchKernelGGL((rebuild_v_kernel<8, false>), grid, dim3(256), 0, st, b, n_copy_blocks); break;
  }
}

void launch_append_bf16(const KvxBatch& b, hipStream_t st) {
  dim3 grid((b.g.n_new + 31) / 32, b.g.H, b.n_items);
  hipLaunchKernelGGL(append_bf16_kernel, grid, dim3(256), 0, st, b);
}

}  // namespace kvx
