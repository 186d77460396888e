// Attention of one frame's queries over [de-quantised cache ; the frame's own K/V]
// (paper Sec. 3.1 Eq. 1 with the de-quantisation of Sec. 3.3 Eq. 10 fused in).
//
// Work decomposition: a workgroup of 4 waves owns 256 query rows of one head and a
// contiguous range of 64-key tiles (split-KV); each wave owns 64 query rows.  Per tile
// the 256 threads de-quantise the K and V codes once into LDS (K row-major, V
// transposed), then every wave runs S^T = K Q^T and O^T += V^T P^T on the matrix cores
// with an online softmax in registers.  Computing the transposed products puts a query
// in a lane and its keys in that lane's registers, so the probabilities feed the second
// MFMA straight from registers (the key order inside a 16-key step is a permutation
// shared by V^T's LDS layout) and the row statistics stay in the lane.
//
// Precision.  A de-quantised key s * (code - z) is an fp32 value; rounding it to 8
// significand bits perturbs the logits of the dominant key channels by ~1e-2, far above
// the output tolerance.  K~ is therefore held as a bf16 pair hi + lo (hi = truncation,
// lo = truncated remainder, together 16 significand bits) and S^T takes two bf16 MFMAs
// (v_mfma_f32_32x32x16_bf16) against the exact bf16 queries.  P and V~ go through the
// f16 MFMA (v_mfma_f32_32x32x16_f16, 11 significand bits, same rate).  fp32 inputs are
// split the same way (queries too).
//
// Softmax.  The softmax scale times log2(e) is folded into the keys as they are staged,
// so S^T is already in log2 units.  Each query keeps a reference m that is raised only
// when a key exceeds it by more than kRescaleGap (then O and l are rescaled, a rare,
// wave-uniform branch); otherwise p = 2^(s - m) <= 2^kRescaleGap needs no rescale.
//
// Schedule.  A wave issues instructions in order, so MFMAs only overlap vector work that
// sits between them in program order: the 32-key halves of a tile are software-pipelined
// (QK of the second half with the softmax of the first, PV of the first with the softmax
// of the second, PV of the second followed by the staging of the next tile) and
// sched_barrier fences keep that interleaving.
#include "kvx_dev.h"

namespace kvx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kLdsRow = 72;                       // 16-bit elements per LDS row: 64 + 8 pad (144 B)
constexpr int kTileElems = kTileK * kLdsRow;      // one K or V^T tile
constexpr float kNegBig = -1.0e30f;
constexpr float kRescaleGap = 8.0f;               // log2 units

#define KVX_FENCE() __builtin_amdgcn_sched_barrier(0)

__device__ __forceinline__ int swap23(int x) { return (x & ~0xC) | ((x & 4) << 1) | ((x & 8) >> 1); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2 x = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}
// Two fp32 values -> packed f16, round to nearest even (v_cvt_pk_f16_f32).
__device__ __forceinline__ uint32_t pack_f16(float a, float b) {
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
    const uint2 t = *reinterpret_cast<const uint2*>(p);
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
  uint4 ok[2], ov[2];                                     // packed bf16
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
  const float sc = g.scale_log2;
  // a wave whose 64 query rows all lie past the frame only helps with staging
  const bool wave_active = (q0 + wave * 64) < n;

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

  f32x16 o[2][2];                     // [channel block][query block]
  float m_ref[2], l_run[2];           // per query block; lanes l and l + 32 hold the same m_ref
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    m_ref[nb] = kNegBig;
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
      const float4 s0 = sp[0], s1 = sp[1];
      const int4 z0 = zp[0], z1 = zp[1];
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

  // K: row (key_a + i) gets 8 channels of hi and lo as one 16-byte store each; the values
  // carry the softmax scale.  V: rows are channels; the two keys land side by side as one
  // 4-byte store per channel.
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

  // De-quantise / convert the raw registers of `tile` into LDS buffer `buf`.
  auto decode_store = [&](int tile, int buf) {
    if (tile < ntc && compressed) {
      const int ja = tile * kTileK + key_a;
      const bool full = (tile + 1) * kTileK <= t_c;
      float sk[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) sk[e] = raw.ks[e] * sc;
      float va[8], vb[8];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          x[e] = sk[e] * (float)(code_at<KB>(raw.kc[i], e) - raw.kz[e]);
          const float vd = raw.vm[i].s * (float)(code_at<VB>(raw.vc[i], e) - raw.vm[i].z);
          if (i == 0) va[e] = vd; else vb[e] = vd;
        }
        if (!full && (ja + i) >= t_c) {
#pragma unroll
          for (int e = 0; e < 8; ++e) { x[e] = 0.f; if (i == 0) va[e] = 0.f; else vb[e] = 0.f; }
        }
        store_k_split(buf, i, x);
      }
      store_v_pair(buf, va, vb);
    } else {
      int base_row, limit;
      if (tile < ntc) { base_row = tile * kTileK; limit = t_c; } else { base_row = (tile - ntc) * kTileK; limit = n; }
      if (F32IN && tile >= ntc) {
        if constexpr (F32IN) {
          float x0[8], x1[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) { x0[e] = raw.ok32[0][e] * sc; x1[e] = raw.ok32[1][e] * sc; }   // rows past the end are zeros
          store_k_split(buf, 0, x0);
          store_k_split(buf, 1, x1);
          store_v_pair(buf, raw.ov32[0], raw.ov32[1]);
        }
      } else {
        float va[8], vb[8];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          uint4 kk = raw.ok[i], vv = raw.ov[i];
          if (base_row + key_a + i >= limit) { kk = make_uint4(0, 0, 0, 0); vv = make_uint4(0, 0, 0, 0); }
          const uint32_t k4[4] = {kk.x, kk.y, kk.z, kk.w};
          float x[8];
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) { x[2 * e2] = bf16lo_to_f32(k4[e2]) * sc; x[2 * e2 + 1] = bf16hi_to_f32(k4[e2]) * sc; }
          store_k_split(buf, i, x);
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

  // ---- pieces of the per-tile pipeline ---------------------------------------------
  f32x16 s[2][2];                     // [key half][query block], log2-domain logits
  f16x8 pb[2][2][2];                  // [key half][query block][16-key step]: P^T as B operand

  // Mask the keys past `valid` (ragged last tile) and raise the references if needed.
  auto pre_softmax = [&](int mb, int valid) {
    if (valid < kTileK) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = mb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
        if (key >= valid) {
          s[mb][0][r] = kNegBig;
          s[mb][1][r] = kNegBig;
        }
      }
    }
    float mx[2];
    bool need = false;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      float a = fmaxf(fmaxf(s[mb][nb][0], s[mb][nb][1]), s[mb][nb][2]);
#pragma unroll
      for (int r = 3; r < 15; r += 2) a = fmaxf(fmaxf(a, s[mb][nb][r]), s[mb][nb][r + 1]);
      a = fmaxf(a, s[mb][nb][15]);
      mx[nb] = a;
      need |= a > m_ref[nb] + kRescaleGap;
    }
    if (__any(need)) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const float mq = fmaxf(mx[nb], __shfl_xor(mx[nb], 32));      // both halves of a query agree
        const float m_new = (mq > m_ref[nb] + kRescaleGap) ? mq : m_ref[nb];
        const float alpha = __builtin_amdgcn_exp2f(m_ref[nb] - m_new);
        m_ref[nb] = m_new;
        l_run[nb] *= alpha;
        if (mb == 1) {
          // the first half's probabilities are already packed relative to the old reference
          // and not yet multiplied into O: bring them to the new reference too
          const _Float16 ah = (_Float16)alpha;
          pb[0][nb][0] = pb[0][nb][0] * ah;
          pb[0][nb][1] = pb[0][nb][1] * ah;
        }
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[cb][nb][r] *= alpha;
      }
    }
  };

  // Elements [r0, r0 + cnt) of half mb, query block nb: p = 2^(s - m), packed to f16, summed.
  const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
  auto softmax_part = [&](int mb, int nb, int r0, int cnt, uint32_t* pk) {
#pragma unroll
    for (int r = r0; r < r0 + cnt; r += 2) {
      const float p0 = __builtin_amdgcn_exp2f(s[mb][nb][r] - m_ref[nb]);
      const float p1 = __builtin_amdgcn_exp2f(s[mb][nb][r + 1] - m_ref[nb]);
      const uint32_t w = pack_f16(p0, p1);
      pk[r >> 1] = w;
      l_run[nb] = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), ones, l_run[nb], false);
    }
  };
  auto finish_p = [&](int mb, int nb, const uint32_t* pk) {
    pb[mb][nb][0] = __builtin_bit_cast(f16x8, make_uint4(pk[0], pk[1], pk[2], pk[3]));
    pb[mb][nb][1] = __builtin_bit_cast(f16x8, make_uint4(pk[4], pk[5], pk[6], pk[7]));
  };

  // O^T += V^T[:, 16 keys] P^T[16 keys] for one channel block and both query blocks.
  auto pv_step = [&](int buf, int mb, int kk, int cb) {
    const f16x8 a = *reinterpret_cast<const f16x8*>(lds_v[buf] + (cb * 32 + l32) * kLdsRow + (mb * 2 + kk) * 16 + hf * 8);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) o[cb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[mb][nb][kk], o[cb][nb], 0, 0, 0);
  };

  // ---- tile loop --------------------------------------------------------------------
  if (tile_begin < tile_end) {
    load_raw(tile_begin);
    decode_store(tile_begin, 0);
    __syncthreads();
    for (int t = tile_begin; t < tile_end; ++t) {
      const int buf = (t - tile_begin) & 1;
      const bool more = (t + 1) < tile_end;
      if (more && !(g.ablate & 2)) load_raw(t + 1);
      if (wave_active && !(g.ablate & 32)) {
        int valid;
        if (t < ntc) valid = min(kTileK, t_c - t * kTileK); else valid = min(kTileK, n - (t - ntc) * kTileK);
        uint32_t pk0[2][8], pk1[2][8];

        // S^T of the first 32 keys
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[0][nb][r] = 0.f;
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int aoff = l32 * kLdsRow + ks * 16 + hf * 8;
          const bf16x8 ah = *reinterpret_cast<const bf16x8*>(lds_khi[buf] + aoff);
          const bf16x8 al = *reinterpret_cast<const bf16x8*>(lds_klo[buf] + aoff);
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            s[0][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, qf[nb][ks], s[0][nb], 0, 0, 0);
            s[0][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, qf[nb][ks], s[0][nb], 0, 0, 0);
            if constexpr (F32IN) s[0][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, qlo[nb][ks], s[0][nb], 0, 0, 0);
          }
        }
        __builtin_amdgcn_s_setprio(0);
        pre_softmax(0, valid);
        KVX_FENCE();

        // S^T of the second 32 keys, interleaved with the softmax of the first.  Each
        // empty asm below takes the next MFMA's LDS operand, the next softmax chunk's
        // inputs and the previous chunk's outputs as read-write operands; volatile asms
        // keep their order, so between two of them sit exactly one MFMA and one chunk
        // of six vector instructions.
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[1][nb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int aoff = (32 + l32) * kLdsRow + ks * 16 + hf * 8;
          bf16x8 ah = *reinterpret_cast<const bf16x8*>(lds_khi[buf] + aoff);
          bf16x8 al = *reinterpret_cast<const bf16x8*>(lds_klo[buf] + aoff);
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            asm volatile("" : "+v"(ah), "+v"(s[0][nb]), "+v"(l_run[nb]));
            s[1][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, qf[nb][ks], s[1][nb], 0, 0, 0);
            softmax_part(0, nb, ks * 4, 2, pk0[nb]);
            asm volatile("" : "+v"(al), "+v"(s[0][nb]), "+v"(l_run[nb]), "+v"(pk0[nb][ks * 2]));
            s[1][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, qf[nb][ks], s[1][nb], 0, 0, 0);
            softmax_part(0, nb, ks * 4 + 2, 2, pk0[nb]);
            asm volatile("" : "+v"(l_run[nb]), "+v"(pk0[nb][ks * 2 + 1]));
            if constexpr (F32IN) s[1][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, qlo[nb][ks], s[1][nb], 0, 0, 0);
          }
        }
        finish_p(0, 0, pk0[0]);
        finish_p(0, 1, pk0[1]);
        KVX_FENCE();
        pre_softmax(1, valid);
        KVX_FENCE();

        // PV of the first half, interleaved with the softmax of the second: one MFMA and
        // one chunk of twelve vector instructions between consecutive asms.
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
          for (int cb = 0; cb < 2; ++cb) {
            const int step = kk * 2 + cb;
            f16x8 a = *reinterpret_cast<const f16x8*>(lds_v[buf] + (cb * 32 + l32) * kLdsRow + kk * 16 + hf * 8);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
              asm volatile("" : "+v"(a), "+v"(s[1][nb]), "+v"(l_run[nb]));
              o[cb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[0][nb][kk], o[cb][nb], 0, 0, 0);
              softmax_part(1, nb, step * 4, 4, pk1[nb]);
              asm volatile("" : "+v"(l_run[nb]), "+v"(pk1[nb][step * 2]), "+v"(pk1[nb][step * 2 + 1]));
            }
          }
        finish_p(1, 0, pk1[0]);
        finish_p(1, 1, pk1[1]);
        KVX_FENCE();

        // PV of the second half; the staging of the next tile follows
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
          for (int cb = 0; cb < 2; ++cb) pv_step(buf, 1, kk, cb);
        __builtin_amdgcn_s_setprio(0);
      }
      if (more && !(g.ablate & 1)) decode_store(t + 1, buf ^ 1);
      if (!(g.ablate & 16)) __syncthreads();
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
    } else if (qi < n) {
      const int slot = item_idx * g.n_splits + split;
      const int64_t row = ((int64_t)slot * g.H + h) * g.n_pad + qi;
      float* po = g.part_o + row * kHeadDim;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int c = cb * 32 + 8 * r4 + 4 * hf;
          *reinterpret_cast<float4*>(po + c) =
              make_float4(o[cb][nb][4 * r4 + 0], o[cb][nb][4 * r4 + 1], o[cb][nb][4 * r4 + 2], o[cb][nb][4 * r4 + 3]);
        }
      if (hf == 0) *reinterpret_cast<float2*>(g.part_ml + row * 2) = make_float2(m_ref[nb], l_tot);
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
