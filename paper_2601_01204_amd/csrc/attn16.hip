// Attention of one frame's queries over [de-quantised cache ; the frame's own K/V] (paper Sec. 3.1
// Eq. 1 with the de-quantisation of Sec. 3.3 Eq. 10 fused in) for caches whose quantiser metadata
// is in the 16-bit format: per key group and channel the logit-domain scale a = s * softmax scale *
// log2(e) as a half with 7 significant bits and zz = 1024 + z as a half; per value token and channel
// group a half scale and zz.
//
// What the format buys.  A de-quantised key times the logit factor is a * (code - z), a 7-bit number
// times an integer of at most 16 in magnitude: exact in the 11-bit significand of a half.  bf16
// queries are halves exactly.  So S^T = K Q^T is ONE f16 matrix instruction per 32 x 32 x 16 step
// with exact operands (the fp32-metadata kernel needs two, a bf16 hi and lo key), and the keys are
// de-quantised by two packed-half instructions per pair of values: the code word is spread into
// halves 1024 + code by masks (0x6400 | code), zz is subtracted exactly, the difference is multiplied
// by a.  The frame's own keys are bf16 values, exact as halves too, but their product with the logit
// factor is not, so their tiles run the first product unscaled from a zero accumulator and the logit
// factor and the softmax reference are applied to the 32 x 64 logits by one fused operation each.
//
// Work decomposition, softmax and schedule are those of the fp32-metadata kernel: a workgroup owns up
// to 12 32-row query blocks of one head, one per wave, and a contiguous range of 64-key tiles
// (split-KV, merged by combine_kernel); per tile waves 0-3 de-quantise K and waves 4-7 V into LDS (K
// row-major, V transposed; within every eight channels a K row holds them in the order 0 4 1 5 2 6 3
// 7, the order the masks produce, and the query fragments are permuted the same way once per wave);
// every wave then runs S^T = K Q^T and O^T += V^T P^T on the matrix cores (v_mfma_f32_32x32x16_f16),
// the transposed products keeping a query in a lane and its keys in that lane's registers; p = 2^(s - m)
// is formed without a prior maximum, an overflow of the half range shows in the row sum and only then
// (rare, wave-uniform) is m raised and the tile redone.
//
// Domain: |k * softmax scale * log2 e| and |v| below 65504 (the half range), finite inputs.
#include "kvx_dev.h"

#include <hip/hip_ext.h>

#include <type_traits>
#include <utility>

namespace kvx {
namespace a16 {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kLdsRow = 72;                       // halves per LDS row: 64 + 8 pad (144 B)
constexpr int kTileElems = kTileK * kLdsRow;      // one K or V^T tile
constexpr float kNegBig = -1.0e30f;
constexpr float kRescaleGap = 8.0f;               // log2 units
constexpr int kAttnMaxWaves = 12;                 // waves (= 32-row query blocks) per workgroup, three per SIMD
constexpr float kSumLimit = 1.0e37f;              // a row sum at or above this (or NaN) saw a half overflow
constexpr uint32_t kBias = 0x64006400u;           // two halves of 1024

__device__ __forceinline__ int swap23(int x) { return (x & ~0xC) | ((x & 4) << 1) | ((x & 8) >> 1); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2 x = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}
__device__ __forceinline__ uint32_t pack_f16(float a, float b) {
  const f32x2 x = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, f16x2));
}
__device__ __forceinline__ f16x2 as_h2(uint32_t w) { return __builtin_bit_cast(f16x2, w); }
__device__ __forceinline__ uint32_t as_u(f16x2 h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Eight bf16 values (channels 0..7 of an octet, two per word) as four half pairs in the octet order
// (0,4) (1,5) (2,6) (3,7).  bf16 -> half is exact inside the half range.
__device__ __forceinline__ uint4 bf16_octet_to_half_pairs(const uint4& r) {
  return make_uint4(pack_f16(bf16lo_to_f32(r.x), bf16lo_to_f32(r.z)), pack_f16(bf16hi_to_f32(r.x), bf16hi_to_f32(r.z)),
                    pack_f16(bf16lo_to_f32(r.y), bf16lo_to_f32(r.w)), pack_f16(bf16hi_to_f32(r.y), bf16hi_to_f32(r.w)));
}

// The codes of eight consecutive channels of one row: 2, 4 or 8 bytes.
template <int B> struct Octet;
template <> struct Octet<2> { typedef uint16_t type; };
template <> struct Octet<4> { typedef uint32_t type; };
template <> struct Octet<8> { typedef uint2 type; };

// The same eight codes as four pairs of halves 1024 + code.  2- and 4-bit codes: pairs (0,4) (1,5)
// (2,6) (3,7); bytes: (0,2) (1,3) (4,6) (5,7).
template <int B>
__device__ __forceinline__ void octet_pairs(const typename Octet<B>::type& w, uint32_t (&p)[4]) {
  if constexpr (B == 4) {
    p[0] = (w & 0x000F000Fu) | kBias;
    p[1] = ((w >> 4) & 0x000F000Fu) | kBias;
    p[2] = ((w >> 8) & 0x000F000Fu) | kBias;
    p[3] = ((w >> 12) & 0x000F000Fu) | kBias;
  } else if constexpr (B == 2) {
    const uint32_t t = (uint32_t)w | ((uint32_t)w << 8);      // code e at bits 2e, code e + 4 also at bits 16 + 2e
    p[0] = (t & 0x00030003u) | kBias;
    p[1] = ((t >> 2) & 0x00030003u) | kBias;
    p[2] = ((t >> 4) & 0x00030003u) | kBias;
    p[3] = ((t >> 6) & 0x00030003u) | kBias;
  } else {
    p[0] = (w.x & 0x00FF00FFu) | kBias;
    p[1] = ((w.x >> 8) & 0x00FF00FFu) | kBias;
    p[2] = (w.y & 0x00FF00FFu) | kBias;
    p[3] = ((w.y >> 8) & 0x00FF00FFu) | kBias;
  }
}
// Channel (within the octet) of the low / high half of pair j.
template <int B> __device__ __forceinline__ constexpr int pair_lo_channel(int j) { return B == 8 ? (j & 1) + 4 * (j >> 1) : j; }
template <int B> __device__ __forceinline__ constexpr int pair_hi_channel(int j) { return B == 8 ? (j & 1) + 4 * (j >> 1) + 2 : j + 4; }

// Staging registers of one thread: two rows x eight channels of K (waves 0-3) or of V (waves 4-7) as
// loaded, before decoding.  Every tile fills the same registers with the same straight-line sequence
// of loads, whatever the tile holds (only the addresses are selected), so the loads of a later tile
// stay in flight across the barriers.
//   cached K tile : c = the two rows' codes, a[0] = the eight channels' scales, a[1] = their 1024 + z
//   cached V tile : c = codes, m = the two rows' (scale, 1024 + z)
//   own frame     : a[0], a[1] = the two bf16 rows
// Registers a tile does not use are loaded from a valid dummy address.
template <int B>
struct TileRaw {
  uint4 a[2];
  typename Octet<B>::type c[2];
  uint32_t m[2];
};

template <int Mask, int N>
__device__ __forceinline__ void sched_group() {
  if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(Mask, N, 0);
}
// Step i of the first product (i = 2 * channel slice + key half): the K read for step i + AHEAD and,
// on even steps, the query read for two slices on, then the step's MFMA.  0x100 = LDS read, 0x008 = MFMA.
template <int AHEAD, int... I>
__device__ __forceinline__ void pin_qk_steps(std::integer_sequence<int, I...>) {
  ((sched_group<0x100, ((I + AHEAD < 8) ? 1 : 0) + (((I & 1) == 0 && (I >> 1) + 2 < 4) ? 1 : 0)>(), sched_group<0x008, 1>()), ...);
}

// Linear block id -> (column, query tile), column = (item, split, head).  Workgroups go to the 8 XCDs round-robin by
// id and each XCD has its own L2, so the query tiles of one column, which read the same K/V codes, get ids that are
// multiples of 8 apart and next to each other in dispatch order: they run on one XCD at about the same time and the
// second and third read of a tile is served by that XCD's L2 instead of HBM.  Columns are taken in groups of 8 (the
// last group may be smaller): id = group * 8 * n_qtiles + qt * group_size + (column within the group).
__device__ __forceinline__ void decode_block(int bid, int n_cols, int n_qtiles, int& col, int& qt) {
  const int per_group = 8 * n_qtiles;
  const int grp = bid / per_group;
  const int rest = bid - grp * per_group;
  const int gsize = min(8, n_cols - grp * 8);
  qt = rest / gsize;
  col = grp * 8 + (rest - qt * gsize);
}

template <int KB, int VB>
__global__ __launch_bounds__(kAttnMaxWaves * 64) void attn16_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  int bid, qt;
  decode_block(blockIdx.x, g.H * g.n_splits * b.n_items, g.n_qtiles, bid, qt);
  const int h = bid % g.H; bid /= g.H;
  const int split = bid % g.n_splits; bid /= g.n_splits;
  const int item_idx = bid;
  const Item it = b.items[item_idx];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hf = lane >> 5;

  __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][kTileElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][kTileElems];
  __shared__ uint4 lds_q[kAttnMaxWaves * 4 * 64];          // waves x 4 channel steps x 64 lanes

  const int n = g.n_new;                                  // query rows = the call's own keys: one frame, or a chunk of frames
  const int t_c = it.t_c;
  const int ntc = (t_c + kTileK - 1) / kTileK;            // cache tiles
  const int nto = g.own_tiles ? (n + kTileK - 1) / kTileK : 0;   // tiles of the call's own keys (none when they are in the cache already)
  const int nt = ntc + nto;
  const int tile_begin = (int)(((int64_t)nt * split) / g.n_splits);
  const int tile_end = (int)(((int64_t)nt * (split + 1)) / g.n_splits);

  const uint8_t* half = cache_half(g, it.cache, it.cur);
  const float sc = g.scale_log2;
  const int row0 = (qt * g.q_blocks + wave) * 32;
  const int nblk = (wave < g.q_blocks && row0 < n) ? 1 : 0;
  // Frame-wise causal mask inside the call's own keys (Sec. 3.1): a query of frame a sees own keys 0 .. (a + 1) n_frame - 1.
  // own_limit: that count for this lane's query; own_limit_wave: the largest over the wave's rows (uniform).
  const int own_limit = (min(row0 + l32, n - 1) / g.n + 1) * g.n;
  const int own_limit_wave = (min(row0 + 31, n - 1) / g.n + 1) * g.n;
  bool started = false;                                   // this wave has computed a tile (the first one sets m)

  // ---- this wave's query fragments (B operand of S^T = K Q^T), halves, octets permuted ----
  uint4* qbase = lds_q + (wave * 4) * 64 + lane;
  auto stage_q = [&]() __attribute__((always_inline)) {
    if (!nblk) return;
    const int qi = min(row0 + l32, n - 1);
    const uint8_t* qrow = reinterpret_cast<const uint8_t*>(it.q) + ((int64_t)qi * g.tok_stride + (int64_t)h * g.head_stride + hf * 8) * 2;
    const uint4 q0 = *reinterpret_cast<const uint4*>(qrow), q1 = *reinterpret_cast<const uint4*>(qrow + 32);
    const uint4 q2 = *reinterpret_cast<const uint4*>(qrow + 64), q3 = *reinterpret_cast<const uint4*>(qrow + 96);
    qbase[0 * 64] = bf16_octet_to_half_pairs(q0);
    qbase[1 * 64] = bf16_octet_to_half_pairs(q1);
    qbase[2 * 64] = bf16_octet_to_half_pairs(q2);
    qbase[3 * 64] = bf16_octet_to_half_pairs(q3);
  };

  f32x16 o[2];                        // [channel block]
  // The reference m (lanes l and l + 32 hold the same value), the running row sum, and a 16-register
  // block filled with -m that the first MFMA of a cached tile takes as its accumulator input.
  f32x16 negm;
  float m_ref = 0.f, l_run = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    negm[r] = 0.f;
    o[0][r] = 0.f;
    o[1][r] = 0.f;
  }
  asm volatile("" : "+v"(negm));

  // staging role of this thread: rows (key_a, key_a + 1) of the tile, channels [8 co, 8 co + 8)
  const int st = tid & 255;
  const int kp = st & 31;
  const int co = st >> 5;
  const int key_a = swap23(2 * kp);
  constexpr int kKRow = 8 * KB;     // bytes per cached key row
  constexpr int kVRow = 8 * VB;
  const int ngv = kHeadDim / g.v_group;
  const int k_shift = g.k_group == 64 ? 6 : 5;
  const int v_shift = g.v_group == 64 ? 6 : 5;

  const uint32_t lo_kc = (uint32_t)(key_a * kKRow + co * KB);                         // K codes, first row
  const uint32_t lo_km = (uint32_t)((((key_a >> k_shift) * kHeadDim) + co * 8) * 2);  // K scales / zero-points (halves)
  const uint32_t lo_vc = (uint32_t)(key_a * kVRow + co * VB);                         // V codes, first row
  const uint32_t lo_vr = (uint32_t)(key_a * kVRow);                                   // start of that V code row
  const uint32_t lo_vm = (uint32_t)((key_a * ngv + ((co * 8) >> v_shift)) * 4);       // V metadata word

  auto load_raw = [&](auto rolec, auto& raw, int tile) __attribute__((always_inline)) {
    constexpr bool ROLE_K = decltype(rolec)::value;
    constexpr int B = ROLE_K ? KB : VB;
    typedef typename Octet<B>::type CodeT;
    const uint8_t *bc, *ba, *bz, *bm;          // uniform bases: codes, a[0], a[1], m
    uint32_t oc0, oc1, oa0, oa1, om0, om1;
    if (tile < ntc) {
      const int64_t row0t = (int64_t)h * g.t_cap + tile * kTileK;
      if constexpr (ROLE_K) {
        bc = half + g.lay.k_codes + row0t * kKRow;
        oc0 = lo_kc; oc1 = lo_kc + kKRow;
        const int64_t moff = ((int64_t)h * g.g_cap + ((tile * kTileK) >> k_shift)) * (kHeadDim * 2);
        ba = half + g.lay.k_scale + moff;
        bz = half + g.lay.k_zero + moff;
        oa0 = oa1 = lo_km;
        bm = ba; om0 = om1 = lo_km;
      } else {
        bc = half + g.lay.v_codes + row0t * kVRow;
        oc0 = lo_vc; oc1 = lo_vc + kVRow;
        bm = half + g.lay.v_meta + row0t * ngv * 4;
        om0 = lo_vm; om1 = lo_vm + ngv * 4;
        ba = bz = bc; oa0 = oa1 = lo_vr;
      }
    } else {
      const int trow = (tile - ntc) * kTileK;
      const int lim = n - 1 - trow;                                   // rows past the frame are zeroed when decoded
      const uint32_t r0 = (uint32_t)min(key_a, lim), r1 = (uint32_t)min(key_a + 1, lim);
      ba = reinterpret_cast<const uint8_t*>(ROLE_K ? it.k : it.v) + ((int64_t)trow * g.tok_stride + (int64_t)h * g.head_stride) * 2;
      const uint32_t ts = (uint32_t)g.tok_stride;
      oa0 = (r0 * ts + co * 8) * 2;
      oa1 = (r1 * ts + co * 8) * 2;
      bz = bc = bm = ba;
      oc0 = oc1 = om0 = om1 = oa0;
    }
    raw.c[0] = *reinterpret_cast<const CodeT*>(bc + oc0);
    raw.c[1] = *reinterpret_cast<const CodeT*>(bc + oc1);
    raw.a[0] = *reinterpret_cast<const uint4*>(ba + oa0);
    raw.a[1] = *reinterpret_cast<const uint4*>(bz + oa1);
    if constexpr (!ROLE_K) {
      raw.m[0] = *reinterpret_cast<const uint32_t*>(bm + om0);
      raw.m[1] = *reinterpret_cast<const uint32_t*>(bm + om1);
    }
  };

  // V: rows of the tile in LDS are channels; the two keys of a thread land side by side as one 4-byte
  // store per channel, column 2 kp (the key order inside a 16-key step is the permutation swap23, which
  // the probabilities' register order shares).
  auto store_v_word = [&](int buf, int ch, uint32_t w) {
    *reinterpret_cast<uint32_t*>(lds_v[buf] + (co * 8 + ch) * kLdsRow + 2 * kp) = w;
  };

  auto decode_store = [&](auto rolec, const auto& raw, int tile, int buf) __attribute__((always_inline)) {
    constexpr bool ROLE_K = decltype(rolec)::value;
    if (tile < ntc) {
      if constexpr (ROLE_K) {
        // (1024 + code) - (1024 + z) is exact; times a: exact up to |code - z| = 16.  Rows past the
        // cache's end hold finite stale values; their logits are masked.
        const uint32_t aw[4] = {raw.a[0].x, raw.a[0].y, raw.a[0].z, raw.a[0].w};
        const uint32_t zw[4] = {raw.a[1].x, raw.a[1].y, raw.a[1].z, raw.a[1].w};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          uint32_t p[4], x[4];
          octet_pairs<KB>(raw.c[i], p);
#pragma unroll
          for (int j = 0; j < 4; ++j) x[j] = as_u((as_h2(p[j]) - as_h2(zw[j])) * as_h2(aw[j]));
          *reinterpret_cast<uint4*>(lds_k[buf] + (key_a + i) * kLdsRow + co * 8) = make_uint4(x[0], x[1], x[2], x[3]);
        }
      } else {
        // rows past the cache's end become zeros (scale zero): their probabilities are zero too
        const int ja = tile * kTileK + key_a;
        const bool full = (tile + 1) * kTileK <= t_c;       // uniform; only a cache's last tile can be ragged
        const uint32_t m0 = (full || ja < t_c) ? raw.m[0] : 0x64000000u, m1 = (full || ja + 1 < t_c) ? raw.m[1] : 0x64000000u;
        const uint32_t s0 = __builtin_amdgcn_perm(m0, m0, 0x01000100u), z0 = __builtin_amdgcn_perm(m0, m0, 0x03020302u);
        const uint32_t s1 = __builtin_amdgcn_perm(m1, m1, 0x01000100u), z1 = __builtin_amdgcn_perm(m1, m1, 0x03020302u);
        uint32_t pa[4], pc[4];
        octet_pairs<VB>(raw.c[0], pa);
        octet_pairs<VB>(raw.c[1], pc);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t xa = as_u((as_h2(pa[j]) - as_h2(z0)) * as_h2(s0));
          const uint32_t xc = as_u((as_h2(pc[j]) - as_h2(z1)) * as_h2(s1));
          store_v_word(buf, pair_lo_channel<VB>(j), __builtin_amdgcn_perm(xc, xa, 0x05040100u));
          store_v_word(buf, pair_hi_channel<VB>(j), __builtin_amdgcn_perm(xc, xa, 0x07060302u));
        }
      }
    } else {
      const int base_row = (tile - ntc) * kTileK;
      uint4 r0 = raw.a[0], r1 = raw.a[1];
      if (!(base_row + key_a < n)) r0 = make_uint4(0, 0, 0, 0);
      if (!(base_row + key_a + 1 < n)) r1 = make_uint4(0, 0, 0, 0);
      if constexpr (ROLE_K) {
        *reinterpret_cast<uint4*>(lds_k[buf] + key_a * kLdsRow + co * 8) = bf16_octet_to_half_pairs(r0);
        *reinterpret_cast<uint4*>(lds_k[buf] + (key_a + 1) * kLdsRow + co * 8) = bf16_octet_to_half_pairs(r1);
      } else {
        const uint32_t a4[4] = {r0.x, r0.y, r0.z, r0.w}, b4[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          store_v_word(buf, 2 * e2, pack_f16(bf16lo_to_f32(a4[e2]), bf16lo_to_f32(b4[e2])));
          store_v_word(buf, 2 * e2 + 1, pack_f16(bf16hi_to_f32(a4[e2]), bf16hi_to_f32(b4[e2])));
        }
      }
    }
  };

  // ---- one tile: S^T, then softmax and O^T ---------------------------------------------
  const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
  auto compute = [&](int t, int kbuf, int vbuf, bool first) __attribute__((always_inline)) {
    f32x16 s[2];                                   // [key half], log2-domain logits minus m
    constexpr int kAhead = 3;
    f16x8 ak[8], qf[4];
    auto read_k = [&](int i) __attribute__((always_inline)) {
      const int ks = i >> 1, mb = i & 1;
      ak[i] = *reinterpret_cast<const f16x8*>(lds_k[kbuf] + (mb * 32 + l32) * kLdsRow + ks * 16 + hf * 8);
    };
    auto read_q = [&](int ks) __attribute__((always_inline)) { qf[ks] = __builtin_bit_cast(f16x8, qbase[ks * 64]); };
    const bool own = t >= ntc;                     // the frame's own keys: unscaled, from a zero accumulator
    read_q(0);
#pragma unroll
    for (int i = 0; i < kAhead; ++i) read_k(i);
    read_q(1);
    __builtin_amdgcn_s_setprio(1);
    if (!own) {
      // cached keys carry the logit factor: the accumulator starts at -m, so S^T leaves the matrix core as s - m
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int ks = i >> 1, mb = i & 1;
        if (i + kAhead < 8) read_k(i + kAhead);
        if (mb == 0 && ks + 2 < 4) read_q(ks + 2);
        if (ks == 0) s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ak[i], qf[ks], negm, 0, 0, 0);
        else s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ak[i], qf[ks], s[mb], 0, 0, 0);
      }
      pin_qk_steps<kAhead>(std::make_integer_sequence<int, 8>{});
      __builtin_amdgcn_s_setprio(0);
    } else {
      f32x16 zero;
#pragma unroll
      for (int r = 0; r < 16; ++r) zero[r] = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int ks = i >> 1, mb = i & 1;
        if (i + kAhead < 8) read_k(i + kAhead);
        if (mb == 0 && ks + 2 < 4) read_q(ks + 2);
        if (ks == 0) s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ak[i], qf[ks], zero, 0, 0, 0);
        else s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ak[i], qf[ks], s[mb], 0, 0, 0);
      }
      pin_qk_steps<kAhead>(std::make_integer_sequence<int, 8>{});
      __builtin_amdgcn_s_setprio(0);
      const float nm = -m_ref;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[mb][r] = __builtin_fmaf(s[mb][r], sc, nm);
    }

    // keys this lane's query may see in the tile: a cache tile's valid rows (ragged last tile), or the own keys up
    // to the end of the query's frame (frame-wise causal mask; also covers the ragged end of the call's rows)
    const int valid = (t < ntc) ? t_c - t * kTileK : own_limit - (t - ntc) * kTileK;
    if (__any(valid < kTileK)) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = mb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key >= valid) s[mb][r] = kNegBig;
        }
    }
    f16x8 pb[4];                      // [16-key step]
    float l_new;
    f16x8 vf[4][2];
    auto read_v = [&](int kk) __attribute__((always_inline)) {
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        vf[kk][cb] = *reinterpret_cast<const f16x8*>(lds_v[vbuf] + (cb * 32 + l32) * kLdsRow + kk * 16 + hf * 8);
    };
    read_v(0);
    read_v(1);
    auto probabilities = [&]() __attribute__((always_inline)) {
      float l = l_run;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int mb = kk >> 1, r0 = (kk & 1) * 8;
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(s[mb][r0 + 2 * e]);
          const float p1 = __builtin_amdgcn_exp2f(s[mb][r0 + 2 * e + 1]);
          w[e] = pack_f16(p0, p1);
          l = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w[e]), ones, l, false);
        }
        pb[kk] = __builtin_bit_cast(f16x8, make_uint4(w[0], w[1], w[2], w[3]));
      }
      l_new = l;
    };
    bool redo = first;                // the first tile sets m from its own keys (m starts at 0)
    if (!first) {
      probabilities();
      redo |= !(l_new < kSumLimit);
    }
    if (__any(redo)) {
      float a = fmaxf(s[0][0], s[1][0]);
#pragma unroll
      for (int r = 1; r < 16; ++r) a = fmaxf(fmaxf(a, s[0][r]), s[1][r]);
      const float mq = fmaxf(a, __shfl_xor(a, 32));                // both halves of a query agree
      // a query that sees none of the tile's keys (all masked) keeps its reference
      const float delta = ((first && mq > 0.5f * kNegBig) || mq > kRescaleGap) ? mq : 0.f;
      const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(-delta);   // nothing accumulated before the first tile
      m_ref += delta;
      l_run *= alpha;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[cb][r] *= alpha;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[mb][r] -= delta;
#pragma unroll
      for (int r = 0; r < 16; ++r) negm[r] = -m_ref;
      asm volatile("" : "+v"(negm));     // opaque: the block stays in its registers, it is the accumulator input of every cached tile
      probabilities();
    }
    l_run = l_new;
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk + 2 < 4) read_v(kk + 2);
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[kk][cb], pb[kk], o[cb], 0, 0, 0);
    }
    sched_group<0x100, 4>();
    sched_group<0x008, 2>();
    sched_group<0x100, 4>();
    sched_group<0x008, 6>();
    __builtin_amdgcn_s_setprio(0);
  };
  // a tile of own keys that lies wholly behind the frames of this wave's queries is skipped (wave-uniform)
  auto run_compute = [&](int t, int buf) __attribute__((always_inline)) {
    if (nblk && !(t >= ntc && (t - ntc) * kTileK >= own_limit_wave)) {
      compute(t, buf, buf, !started);
      started = true;
    }
  };

  // ---- tile loop --------------------------------------------------------------------
  // Between two workgroup barriers waves 0-3 (K stagers) compute tile t and then stage tile t+1,
  // waves 4-7 (V stagers) stage first and then compute, the others only compute.  A tile's raw data
  // is loaded one interval before it is decoded.
  auto tile_loop = [&](auto rolec) __attribute__((always_inline)) {
    constexpr bool ROLE_K = decltype(rolec)::value;
    TileRaw<ROLE_K ? KB : VB> raw;
    const int last = tile_end - 1;
    load_raw(rolec, raw, tile_begin);
    stage_q();
    decode_store(rolec, raw, tile_begin, 0);
    load_raw(rolec, raw, min(tile_begin + 1, last));
    __syncthreads();
    for (int t = tile_begin; t < tile_end; ++t) {
      const int buf = (t - tile_begin) & 1;
      const bool more = t < last;
      if constexpr (ROLE_K) {
        run_compute(t, buf);
        if (more) decode_store(rolec, raw, t + 1, buf ^ 1);
        load_raw(rolec, raw, min(t + 2, last));
      } else {
        if (more) decode_store(rolec, raw, t + 1, buf ^ 1);
        load_raw(rolec, raw, min(t + 2, last));
        run_compute(t, buf);
      }
      __syncthreads();
    }
  };
  if (tile_begin < tile_end) {
    if (wave < 4) {
      tile_loop(std::true_type{});
    } else if (wave < 8) {
      tile_loop(std::false_type{});
    } else {
      stage_q();
      __syncthreads();
      for (int t = tile_begin; t < tile_end; ++t) {
        run_compute(t, (t - tile_begin) & 1);
        __syncthreads();
      }
    }
  }

  // ---- epilogue -------------------------------------------------------------------
  if (!started) m_ref = kNegBig;     // an empty (or wholly masked) key range weighs nothing in the merge
  const int qi = nblk ? row0 + l32 : n;
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (g.n_splits == 1) {
    if (qi < n) {
      const float inv = 1.0f / l_tot;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int c = cb * 32 + 8 * r4 + 4 * hf;
          const float x0 = o[cb][4 * r4 + 0] * inv, x1 = o[cb][4 * r4 + 1] * inv;
          const float x2 = o[cb][4 * r4 + 2] * inv, x3 = o[cb][4 * r4 + 3] * inv;
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
        *reinterpret_cast<float4*>(po + c) = make_float4(o[cb][4 * r4 + 0], o[cb][4 * r4 + 1], o[cb][4 * r4 + 2], o[cb][4 * r4 + 3]);
      }
    // a query that saw no key in this range (all masked) has l = 0: its reference must not raise the merge's maximum
    if (hf == 0) *reinterpret_cast<float2*>(g.part_ml + row * 2) = make_float2(l_tot > 0.f ? m_ref : kNegBig, l_tot);
  }
}

template <int KB, int VB>
static void launch_t(const KvxBatch& b, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const Geometry& g = b.g;
  dim3 grid(g.n_qtiles * g.H * b.n_items * g.n_splits);
  const dim3 block(64 * (g.q_blocks > 8 ? g.q_blocks : 8));      // a wave per query block, at least the 8 staging waves
  if (ev_start) hipExtLaunchKernelGGL((attn16_kernel<KB, VB>), grid, block, 0, st, ev_start, ev_stop, 0, b);
  else hipLaunchKernelGGL((attn16_kernel<KB, VB>), grid, block, 0, st, b);
}

}  // namespace a16

void launch_attention16(const KvxBatch& b, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const int kb = b.g.k_bits, vb = b.g.v_bits;
#define KVX_CASE(K, V) if (kb == K && vb == V) { a16::launch_t<K, V>(b, st, ev_start, ev_stop); return; }
  KVX_CASE(4, 4) KVX_CASE(2, 4) KVX_CASE(4, 2) KVX_CASE(2, 2) KVX_CASE(4, 8) KVX_CASE(2, 8)
#undef KVX_CASE
}

}  // namespace kvx
