// Attention of one frame's queries over [de-quantised cache ; the frame's own K/V]
// (paper Sec. 3.1 Eq. 1 with the de-quantisation of Sec. 3.3 Eq. 10 fused in).
//
// Work decomposition: a workgroup of 4 waves owns 256 query rows of one head and a
// contiguous range of 64-key tiles (split-KV); each wave owns 64 query rows.  Per tile
// the 256 threads de-quantise the K and V codes once into LDS (K row-major, V
// transposed), then every wave runs S^T = K Q^T and O^T += V^T P^T on the matrix cores
// with an online softmax in registers.  Computing the transposed products puts a query
// in a lane and its keys in that lane's registers, so row max / row sum need one
// cross-lane exchange and the probabilities feed the second MFMA straight from
// registers (the key order inside a 16-key step is a permutation shared by V^T's LDS
// layout).
//
// Precision.  A de-quantised key s * (code - z) is an fp32 value; rounding it to 8
// significand bits perturbs the logits of the dominant key channels by ~1e-2, far above
// the output tolerance.  K~ is therefore held as a bf16 pair hi + lo (hi = truncation,
// lo = truncated remainder, together 16 significand bits) and S^T takes two bf16 MFMAs
// (v_mfma_f32_32x32x16_bf16) against the exact bf16 queries; bf16 keys of the frame
// itself have lo = 0 and take one.  P (in [0, 1]) and V~ go through the f16 MFMA
// (v_mfma_f32_32x32x16_f16, 11 significand bits, same rate).  fp32 inputs are split the
// same way (queries too).
#include "kvx_dev.h"

namespace kvx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kLdsRow = 72;                       // bf16 elements per LDS row: 64 + 8 pad (144 B)
constexpr int kTileElems = kTileK * kLdsRow;      // one K or V^T tile
constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ int swap23(int x) { return (x & ~0xC) | ((x & 4) << 1) | ((x & 8) >> 1); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 x = {a, b};
  bf16x2 y = __builtin_convertvector(x, bf16x2);
  return __builtin_bit_cast(uint32_t, y);
}

// Two fp32 values -> packed f16, round to nearest even (v_cvt_pk_f16_f32).
__device__ __forceinline__ uint32_t pack_f16(float a, float b) {
  typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
  const f32x2 x = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, f16x2));
}
// Two fp32 values -> packed bf16 truncations (hi) and packed bf16 truncated remainders (lo).
__device__ __forceinline__ void split_bf16(float a, float b, uint32_t& hi, uint32_t& lo) {
  const uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
  hi = (ua >> 16) | (ub & 0xFFFF0000u);
  const float ra = a - __uint_as_float(ua & 0xFFFF0000u), rb = b - __uint_as_float(ub & 0xFFFF0000u);
  lo = (__float_as_uint(ra) >> 16) | (__float_as_uint(rb) & 0xFFFF0000u);
}
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <int B>
__device__ __forceinline__ int code_at(const uint32_t (&w)[2], int e) {
  if constexpr (B == 4) return (int)((w[0] >> (4 * e)) & 0xFu);
  if constexpr (B == 2) return (int)((w[0] >> (2 * e)) & 0x3u);
  return (int)((w[e >> 2] >> (8 * (e & 3))) & 0xFFu);
}

template <int B>
__device__ __forceinline__ void load_octet(const uint8_t* p, uint32_t (&w)[2]) {
  if constexpr (B == 4) {
    w[0] = *reinterpret_cast<const uint32_t*>(p);
    w[1] = 0;
  } else if constexpr (B == 2) {
    w[0] = *reinterpret_cast<const uint16_t*>(p);
    w[1] = 0;
  } else {
    uint2 t = *reinterpret_cast<const uint2*>(p);
    w[0] = t.x;
    w[1] = t.y;
  }
}

template <bool F32IN>
struct TileRaw {
  // cache tile: two keys x eight channels of codes, the channels' key metadata, the keys' value metadata
  uint32_t kc[2][2];
  float ks[8];
  int32_t kz[8];
  uint32_t vc[2][2];
  VMeta vm[2];
  // rows of the frame itself or of the uncompressed cache: two keys x eight channels
  uint4 ok[2], ov[2];                          // packed bf16
  float ok32[F32IN ? 2 : 1][8], ov32[F32IN ? 2 : 1][8];   // fp32 inputs
};

__device__ __forceinline__ void load8_f32(const void* base, int64_t off, float (&x)[8]) {
  const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + off);
  const float4 a = p[0], b = p[1];
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

template <int KB, int VB, bool F32IN>
__global__ __launch_bounds__(256, 2) void attn_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const int item_idx = blockIdx.z / g.n_splits;
  const int split = blockIdx.z % g.n_splits;
  const Item it = b.items[item_idx];
  const int h = blockIdx.y;
  const int q0 = blockIdx.x * kQTile;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hf = lane >> 5;

  __shared__ __attribute__((aligned(16))) uint16_t lds_khi[2][kTileElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_klo[2][kTileElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][kTileElems];

  const int n = g.n;
  const int t_c = it.t_c;
  const int ntc = (t_c + kTileK - 1) / kTileK;            // cache tiles
  const int nto = (n + kTileK - 1) / kTileK;              // own-frame tiles
  const int nt = ntc + nto;
  // contiguous, near-equal tile ranges per split
  const int tile_begin = (int)(((int64_t)nt * split) / g.n_splits);
  const int tile_end = (int)(((int64_t)nt * (split + 1)) / g.n_splits);

  const uint8_t* half = cache_half(g, it.cache, it.cur);
  const bool compressed = !g.uncompressed;

  // ---- this wave's query fragments (B operand of S^T = K Q^T) ---------------------
  bf16x8 qf[2][4];
  bf16x8 qlo[F32IN ? 2 : 1][4];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int qi = q0 + wave * 64 + nb * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int64_t off = (int64_t)qi * g.tok_stride + (int64_t)h * g.head_stride + ks * 16 + hf * 8;
      if constexpr (F32IN) {
        float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (qi < n) load8_f32(it.q, off, x);
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split_bf16(x[2 * e], x[2 * e + 1], hi[e], lo[e]);
        qf[nb][ks] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
        qlo[nb][ks] = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
      } else {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (qi < n) v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(it.q) + off);
        qf[nb][ks] = __builtin_bit_cast(bf16x8, v);
      }
    }
  }

  f32x16 o[2][2];
  float m_run[2], l_run[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    m_run[nb] = kNegBig;
    l_run[nb] = 0.f;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[cb][nb][r] = 0.f;
  }

  // staging role of this thread: keys (key_a, key_a + 1) of the tile, channels [8 co, 8 co + 8)
  const int kp = tid & 31;
  const int co = tid >> 5;
  const int key_a = swap23(2 * kp);
  constexpr int kKRow = 8 * KB;     // bytes per cached key row
  constexpr int kVRow = 8 * VB;
  const int ngv = kHeadDim / g.v_group;

  TileRaw<F32IN> raw;

  auto load_raw = [&](int tile) {
    if (tile < ntc && compressed) {
      const int ja = tile * kTileK + key_a;
      const uint8_t* kcp = half + g.lay.k_codes + ((int64_t)h * g.t_cap + ja) * kKRow + co * KB;
      load_octet<KB>(kcp, raw.kc[0]);
      load_octet<KB>(kcp + kKRow, raw.kc[1]);
      const int grp = ja / g.k_group;
      const int64_t moff = ((int64_t)h * g.g_cap + grp) * kHeadDim + co * 8;
      const float4* sp = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(half + g.lay.k_scale) + moff);
      const int4* zp = reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(half + g.lay.k_zero) + moff);
      float4 s0 = sp[0], s1 = sp[1];
      int4 z0 = zp[0], z1 = zp[1];
      raw.ks[0] = s0.x; raw.ks[1] = s0.y; raw.ks[2] = s0.z; raw.ks[3] = s0.w;
      raw.ks[4] = s1.x; raw.ks[5] = s1.y; raw.ks[6] = s1.z; raw.ks[7] = s1.w;
      raw.kz[0] = z0.x; raw.kz[1] = z0.y; raw.kz[2] = z0.z; raw.kz[3] = z0.w;
      raw.kz[4] = z1.x; raw.kz[5] = z1.y; raw.kz[6] = z1.z; raw.kz[7] = z1.w;
      const uint8_t* vcp = half + g.lay.v_codes + ((int64_t)h * g.t_cap + ja) * kVRow + co * VB;
      load_octet<VB>(vcp, raw.vc[0]);
      load_octet<VB>(vcp + kVRow, raw.vc[1]);
      const VMeta* vmp = reinterpret_cast<const VMeta*>(half + g.lay.v_meta) + ((int64_t)h * g.t_cap + ja) * ngv + (co * 8) / g.v_group;
      raw.vm[0] = vmp[0];
      raw.vm[1] = vmp[ngv];
    } else if (tile < ntc) {
      // uncompressed bf16 cache: rows of 64 bf16
      const int ja = tile * kTileK + key_a;
      const uint16_t* kb = reinterpret_cast<const uint16_t*>(half + g.lay.k_codes) + ((int64_t)h * g.t_cap + ja) * kHeadDim + co * 8;
      const uint16_t* vb = reinterpret_cast<const uint16_t*>(half + g.lay.v_codes) + ((int64_t)h * g.t_cap + ja) * kHeadDim + co * 8;
      raw.ok[0] = *reinterpret_cast<const uint4*>(kb);
      raw.ok[1] = *reinterpret_cast<const uint4*>(kb + kHeadDim);
      raw.ov[0] = *reinterpret_cast<const uint4*>(vb);
      raw.ov[1] = *reinterpret_cast<const uint4*>(vb + kHeadDim);
    } else {
      const int ia = (tile - ntc) * kTileK + key_a;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const bool ok = (ia + i) < n;
        const int64_t off = (int64_t)(ia + i) * g.tok_stride + (int64_t)h * g.head_stride + co * 8;
        if constexpr (F32IN) {
#pragma unroll
          for (int e = 0; e < 8; ++e) { raw.ok32[i][e] = 0.f; raw.ov32[i][e] = 0.f; }
          if (ok) { load8_f32(it.k, off, raw.ok32[i]); load8_f32(it.v, off, raw.ov32[i]); }
        } else {
          raw.ok[i] = make_uint4(0, 0, 0, 0);
          raw.ov[i] = make_uint4(0, 0, 0, 0);
          if (ok) {
            raw.ok[i] = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(it.k) + off);
            raw.ov[i] = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(it.v) + off);
          }
        }
      }
    }
  };

  // K: rows (key_a + i) get 8 channels of hi (and lo) as one 16-byte store each.
  // V: rows are channels; the two keys land side by side as one 4-byte store per channel.
  auto store_k_split = [&](int buf, int i, const float (&x)[8]) {
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split_bf16(x[2 * e], x[2 * e + 1], hi[e], lo[e]);
    *reinterpret_cast<uint4*>(lds_khi[buf] + (key_a + i) * kLdsRow + co * 8) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    *reinterpret_cast<uint4*>(lds_klo[buf] + (key_a + i) * kLdsRow + co * 8) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
  };
  auto store_v_pair = [&](int buf, const float (&a)[8], const float (&c)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) *reinterpret_cast<uint32_t*>(lds_v[buf] + (co * 8 + e) * kLdsRow + 2 * kp) = pack_f16(a[e], c[e]);
  };

  auto decode_store = [&](int tile, int buf) {
    if (tile < ntc && compressed) {
      const int ja = tile * kTileK + key_a;
      float va[8], vb[8];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const bool ok = (ja + i) < t_c;
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float kd = raw.ks[e] * (float)(code_at<KB>(raw.kc[i], e) - raw.kz[e]);
          x[e] = ok ? kd : 0.f;
          const float vd = raw.vm[i].s * (float)(code_at<VB>(raw.vc[i], e) - raw.vm[i].z);
          if (i == 0) va[e] = ok ? vd : 0.f; else vb[e] = ok ? vd : 0.f;
        }
        store_k_split(buf, i, x);
      }
      store_v_pair(buf, va, vb);
    } else {
      int base_row, limit;
      if (tile < ntc) { base_row = tile * kTileK; limit = t_c; } else { base_row = (tile - ntc) * kTileK; limit = n; }
      if (F32IN && tile >= ntc) {
        if constexpr (F32IN) {
          store_k_split(buf, 0, raw.ok32[0]);     // rows past the end were loaded as zeros
          store_k_split(buf, 1, raw.ok32[1]);
          store_v_pair(buf, raw.ov32[0], raw.ov32[1]);
        }
      } else {
        float va[8], vb[8];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          uint4 kk = raw.ok[i], vv = raw.ov[i];
          if (base_row + key_a + i >= limit) { kk = make_uint4(0, 0, 0, 0); vv = make_uint4(0, 0, 0, 0); }
          *reinterpret_cast<uint4*>(lds_khi[buf] + (key_a + i) * kLdsRow + co * 8) = kk;      // bf16 keys are exact: no lo part
          const uint32_t w4[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            if (i == 0) { va[2 * e2] = bf16lo_to_f32(w4[e2]); va[2 * e2 + 1] = bf16hi_to_f32(w4[e2]); }
            else { vb[2 * e2] = bf16lo_to_f32(w4[e2]); vb[2 * e2 + 1] = bf16hi_to_f32(w4[e2]); }
          }
        }
        store_v_pair(buf, va, vb);
      }
    }
  };

  auto compute = [&](int tile, int buf) {
    const uint16_t* lkh = lds_khi[buf];
    const uint16_t* lkl = lds_klo[buf];
    const uint16_t* lv = lds_v[buf];
    int valid;
    bool has_lo;
    if (tile < ntc) { valid = min(kTileK, t_c - tile * kTileK); has_lo = compressed; }
    else { valid = min(kTileK, n - (tile - ntc) * kTileK); has_lo = F32IN; }

    f32x16 s[2][2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[mb][nb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const int aoff = (mb * 32 + l32) * kLdsRow + ks * 16 + hf * 8;
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(lkh + aoff);
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nb][ks], s[mb][nb], 0, 0, 0);
        if constexpr (F32IN) {
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qlo[nb][ks], s[mb][nb], 0, 0, 0);
        }
      }
    }
    if (has_lo) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(lkl + (mb * 32 + l32) * kLdsRow + ks * 16 + hf * 8);
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nb][ks], s[mb][nb], 0, 0, 0);
        }
      }
    }
    if (valid < kTileK) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = mb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key >= valid) {
            s[mb][0][r] = kNegBig;
            s[mb][1][r] = kNegBig;
          }
        }
    }

    f16x8 pb[2][4];
    const float sc = g.scale_log2;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      float mx = s[0][nb][0];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mb][nb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[nb], mx * sc);
      const float alpha = __builtin_amdgcn_exp2f(m_run[nb] - m_new);
      m_run[nb] = m_new;
      float rs = 0.f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][nb][r], sc, -m_new));
          rs += p;
          s[mb][nb][r] = p;
        }
      }
      l_run[nb] = l_run[nb] * alpha + rs;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[cb][nb][r] *= alpha;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int mb = kk >> 1, r0 = (kk & 1) * 8;
        const uint4 w = make_uint4(pack_f16(s[mb][nb][r0 + 0], s[mb][nb][r0 + 1]), pack_f16(s[mb][nb][r0 + 2], s[mb][nb][r0 + 3]),
                                   pack_f16(s[mb][nb][r0 + 4], s[mb][nb][r0 + 5]), pack_f16(s[mb][nb][r0 + 6], s[mb][nb][r0 + 7]));
        pb[nb][kk] = __builtin_bit_cast(f16x8, w);
      }
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        const f16x8 a = *reinterpret_cast<const f16x8*>(lv + (cb * 32 + l32) * kLdsRow + kk * 16 + hf * 8);
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) o[cb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[nb][kk], o[cb][nb], 0, 0, 0);
      }
    }
  };

  // ---- tile loop: global loads for tile t+1 are in flight while tile t is computed --
  if (tile_begin < tile_end) {
    load_raw(tile_begin);
    decode_store(tile_begin, 0);
    __syncthreads();
    for (int t = tile_begin; t < tile_end; ++t) {
      const int buf = (t - tile_begin) & 1;
      const bool more = (t + 1) < tile_end;
      if (more) load_raw(t + 1);
      compute(t, buf);
      if (more) decode_store(t + 1, buf ^ 1);
      __syncthreads();
    }
  }

  // ---- epilogue -------------------------------------------------------------------
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int qi = q0 + wave * 64 + nb * 32 + l32;
    const float l_tot = l_run[nb] + __shfl_xor(l_run[nb], 32);
    if (g.n_splits == 1) {
      if (qi < n) {
        const float inv = 1.0f / l_tot;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const int c = cb * 32 + 8 * r4 + 4 * hf;
            const float x0 = o[cb][nb][4 * r4 + 0] * inv, x1 = o[cb][nb][4 * r4 + 1] * inv;
            const float x2 = o[cb][nb][4 * r4 + 2] * inv, x3 = o[cb][nb][4 * r4 + 3] * inv;
            const int64_t off = (int64_t)qi * g.out_tok_stride + (int64_t)h * g.out_head_stride + c;
            if (g.out_f32) {
              *reinterpret_cast<float4*>(reinterpret_cast<float*>(it.out) + off) = make_float4(x0, x1, x2, x3);
            } else {
              *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(it.out) + off) = make_uint2(pack_bf16(x0, x1), pack_bf16(x2, x3));
            }
          }
      }
    } else {
      const int slot = item_idx * g.n_splits + split;
      const int64_t row = ((int64_t)slot * g.H + h) * g.n_pad + qi;     // qi < n_pad always
      float* po = g.part_o + row * kHeadDim;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int c = cb * 32 + 8 * r4 + 4 * hf;
          *reinterpret_cast<float4*>(po + c) =
              make_float4(o[cb][nb][4 * r4 + 0], o[cb][nb][4 * r4 + 1], o[cb][nb][4 * r4 + 2], o[cb][nb][4 * r4 + 3]);
        }
      if (hf == 0) *reinterpret_cast<float2*>(g.part_ml + row * 2) = make_float2(m_run[nb], l_tot);
    }
  }
}

// Merge the split-KV partials: out = sum_s w_s O_s / sum_s w_s l_s, w_s = 2^(m_s - max m).
__global__ __launch_bounds__(256) void combine_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.z];
  const int h = blockIdx.y;
  const int qi = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int c = (threadIdx.x & 15) * 4;
  if (qi >= g.n) return;
  float m_max = kNegBig;
  for (int s = 0; s < g.n_splits; ++s) {
    const int64_t row = ((int64_t)(blockIdx.z * g.n_splits + s) * g.H + h) * g.n_pad + qi;
    m_max = fmaxf(m_max, g.part_ml[row * 2]);
  }
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float l = 0.f;
  for (int s = 0; s < g.n_splits; ++s) {
    const int64_t row = ((int64_t)(blockIdx.z * g.n_splits + s) * g.H + h) * g.n_pad + qi;
    const float2 ml = *reinterpret_cast<const float2*>(g.part_ml + row * 2);
    const float w = __builtin_amdgcn_exp2f(ml.x - m_max);
    const float4 po = *reinterpret_cast<const float4*>(g.part_o + row * kHeadDim + c);
    acc.x += w * po.x; acc.y += w * po.y; acc.z += w * po.z; acc.w += w * po.w;
    l += w * ml.y;
  }
  const float inv = 1.0f / l;
  const int64_t off = (int64_t)qi * g.out_tok_stride + (int64_t)h * g.out_head_stride + c;
  if (g.out_f32) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(it.out) + off) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
  } else {
    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(it.out) + off) =
        make_uint2(pack_bf16(acc.x * inv, acc.y * inv), pack_bf16(acc.z * inv, acc.w * inv));
  }
}

template <int KB, int VB>
static void launch_attn_t(const KvxBatch& b, hipStream_t st) {
  const Geometry& g = b.g;
  dim3 grid(g.n_pad / kQTile, g.H, b.n_items * g.n_splits);
  if (g.in_f32) hipLaunchKernelGGL((attn_kernel<KB, VB, true>), grid, dim3(256), 0, st, b);
  else hipLaunchKernelGGL((attn_kernel<KB, VB, false>), grid, dim3(256), 0, st, b);
}

void launch_attention(const KvxBatch& b, int /*max_tiles*/, hipStream_t st) {
  const int kb = b.g.uncompressed ? 4 : b.g.k_bits, vb = b.g.uncompressed ? 4 : b.g.v_bits;
#define KVX_CASE(K, V) if (kb == K && vb == V) { launch_attn_t<K, V>(b, st); return; }
  KVX_CASE(4, 4) KVX_CASE(8, 8) KVX_CASE(2, 4) KVX_CASE(2, 2) KVX_CASE(4, 8) KVX_CASE(8, 4) KVX_CASE(4, 2) KVX_CASE(2, 8) KVX_CASE(8, 2)
#undef KVX_CASE
}

void launch_combine(const KvxBatch& b, hipStream_t st) {
  const Geometry& g = b.g;
  if (g.n_splits <= 1) return;
  dim3 grid((g.n + 15) / 16, g.H, b.n_items);
  hipLaunchKernelGGL(combine_kernel, grid, dim3(256), 0, st, b);
}

}  // namespace kvx
