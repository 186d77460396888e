// Attention of one frame's queries over [de-quantised cache ; the frame's own K/V]
// (paper Sec. 3.1 Eq. 1 with the de-quantisation of Sec. 3.3 Eq. 10 fused in).
//
// Work decomposition: a workgroup owns a tile of up to 12 32-row query blocks of one head
// (the frame's blocks cut evenly over tiles), one block per wave, so 8 to 12 waves, and a
// contiguous range of 64-key tiles (split-KV).  Per tile waves 0-3 de-quantise the K
// codes and waves 4-7 the V codes once into LDS (K row-major, V transposed), then every
// wave runs S^T = K Q^T and O^T += V^T P^T on the matrix cores with an online softmax in
// registers.  Computing the transposed products puts a query in a lane and its keys in
// that lane's registers, so the probabilities feed the second MFMA straight from
// registers (the key order inside a 16-key step is a permutation shared by V^T's LDS
// layout) and the row statistics stay in the lane.
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
// so S^T is already in log2 units.  Each query keeps a reference m and p = 2^(s - m) is
// formed without looking at the tile's maximum first: f16 holds p up to 2^16, and a key
// further above m than that makes p, and so the row sum, infinite.  Only then (a rare,
// wave-uniform branch) is m raised for every row whose largest key exceeds it by more
// than kRescaleGap, O and l are rescaled and the tile's probabilities are formed again.
//
// Schedule.  A wave issues in order.  Measured on gfx950, its independent vector
// instructions do run under its own MFMAs, but every 16-byte LDS operand read holds the
// wave for about as long as it holds the SIMD's LDS return path (16 cycles), so a single
// wave that interleaves its reads, MFMAs and softmax arithmetic gains little over doing
// them one after the other; the overlap has to come from different waves of a SIMD being
// in different phases.  A SIMD holds up to three waves of the workgroup (w, w + 4, w + 8),
// each with the same matrix work; waves 0-3 compute a tile and then stage K of the next
// one, waves 4-7 stage V first and then compute, waves 8-11 only compute, so their MFMA and
// vector stretches fall at different times between two barriers.
#include "kvx_dev.h"

#include <hip/hip_ext.h>

#include <type_traits>
#include <utility>

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
constexpr int kAttnMaxWaves = 12;                 // waves (= 32-row query blocks) per workgroup, three per SIMD
constexpr float kSumLimit = 1.0e37f;              // a row sum at or above this (or NaN) saw an f16 overflow

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
  hi = __builtin_amdgcn_perm(ub, ua, 0x07060302u);          // the upper halves of a (low) and b (high)
  const float ra = a - __uint_as_float(ua & 0xFFFF0000u), rb = b - __uint_as_float(ub & 0xFFFF0000u);
  lo = __builtin_amdgcn_perm(__float_as_uint(rb), __float_as_uint(ra), 0x07060302u);
}
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// The codes of eight consecutive channels of one row: 2, 4 or 8 bytes.
template <int B> struct Octet;
template <> struct Octet<2> { typedef uint16_t type; };
template <> struct Octet<4> { typedef uint32_t type; };
template <> struct Octet<8> { typedef uint2 type; };

template <int B>
__device__ __forceinline__ int octet_code(const typename Octet<B>::type& w, int e) {
  if constexpr (B == 4) return (int)((w >> (4 * e)) & 0xFu);
  else if constexpr (B == 2) return (int)(((uint32_t)w >> (2 * e)) & 0x3u);
  else return (int)(((e < 4 ? w.x : w.y) >> (8 * (e & 3))) & 0xFFu);
}

// The same eight codes as floats.  Bytes convert in one instruction each, so 4-bit codes
// are first spread into the bytes of two words (even and odd channels).
// Byte K of a word as a float (v_cvt_f32_ubyteK; written out because the compiler would
// otherwise merge the nibble masks below back into one bit-field extract per value).
template <int K>
__device__ __forceinline__ float byte_to_float(uint32_t w) {
  float f;
  if constexpr (K == 0) asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(f) : "v"(w));
  else if constexpr (K == 1) asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(f) : "v"(w));
  else if constexpr (K == 2) asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(f) : "v"(w));
  else asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(f) : "v"(w));
  return f;
}
template <int B>
__device__ __forceinline__ void octet_floats(const typename Octet<B>::type& w, float (&f)[8]) {
  if constexpr (B == 8) {
    f[0] = byte_to_float<0>(w.x); f[1] = byte_to_float<1>(w.x); f[2] = byte_to_float<2>(w.x); f[3] = byte_to_float<3>(w.x);
    f[4] = byte_to_float<0>(w.y); f[5] = byte_to_float<1>(w.y); f[6] = byte_to_float<2>(w.y); f[7] = byte_to_float<3>(w.y);
  } else if constexpr (B == 4) {
    const uint32_t ev = w & 0x0F0F0F0Fu, od = (w >> 4) & 0x0F0F0F0Fu;
    f[0] = byte_to_float<0>(ev); f[2] = byte_to_float<1>(ev); f[4] = byte_to_float<2>(ev); f[6] = byte_to_float<3>(ev);
    f[1] = byte_to_float<0>(od); f[3] = byte_to_float<1>(od); f[5] = byte_to_float<2>(od); f[7] = byte_to_float<3>(od);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (float)(((uint32_t)w >> (2 * e)) & 0x3u);
  }
}

// Staging registers of one thread: two rows x eight channels of K (waves 0-3) or of V
// (waves 4-7) as loaded, before decoding.  Every tile fills the same registers with the
// same straight-line sequence of loads, whatever the tile holds (only the addresses are
// selected), so the loads of a later tile stay in flight across the barriers.
//   cached K tile : c = the two rows' codes, a[0..1] = the channels' scales, a[2..3] = zero-points
//   cached V tile : c = codes, m = the two rows' (scale, zero-point)
//   bf16 rows     : a[0], a[1] = the two rows (own frame, uncompressed cache)
//   fp32 rows     : a[0..1] = first row, a[2..3] = second row (own frame)
// Registers a tile does not use are loaded from a valid dummy address.
template <int B>
struct TileRaw {
  uint4 a[4];
  typename Octet<B>::type c[2];
  uint2 m[2];
};

// Scheduling groups (the compiler keeps the groups of a basic block in the order given):
// Mask 0x008 = MFMA, 0x100 = LDS read.
template <int Mask, int N>
__device__ __forceinline__ void sched_group() {
  if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(Mask, N, 0);
}
// Step i of the first product (i = 2 * channel slice + key half): the K reads for step
// i + AHEAD and, on even steps, the query reads for two slices on, then the step's MFMAs.
template <int NB, bool F32, int AHEAD, int... I>
__device__ __forceinline__ void pin_qk_steps(std::integer_sequence<int, I...>) {
  ((sched_group<0x100, ((I + AHEAD < 8) ? 2 : 0) + (((I & 1) == 0 && (I >> 1) + 2 < 4) ? NB + (F32 ? 1 : 0) : 0)>(),
    sched_group<0x008, (F32 ? 3 : 2) * NB>()), ...);
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

template <int KB, int VB, bool F32IN>
__global__ __launch_bounds__(kAttnMaxWaves * 64) void attn_kernel(const KvxBatch b) {
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

  __shared__ __attribute__((aligned(16))) uint16_t lds_khi[2][kTileElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_klo[2][kTileElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][kTileElems];
  constexpr int kQSets = F32IN ? 2 : 1;                   // bf16 queries: one fragment set; fp32: hi and lo
  __shared__ uint4 lds_q[kAttnMaxWaves * kQSets * 4 * 64];   // waves x sets x 4 channel steps x 64 lanes

  const int n = g.n_new;                                  // query rows = the call's own keys: one frame, or a chunk of frames
  const int t_c = it.t_c;
  const int ntc = (t_c + kTileK - 1) / kTileK;            // cache tiles
  const int nto = g.own_tiles ? (n + kTileK - 1) / kTileK : 0;   // tiles of the call's own keys (none when they are in the cache already)
  const int nt = ntc + nto;
  // contiguous, near-equal tile ranges per split
  const int tile_begin = (int)(((int64_t)nt * split) / g.n_splits);
  const int tile_end = (int)(((int64_t)nt * (split + 1)) / g.n_splits);

  const uint8_t* half = cache_half(g, it.cache, it.cur);
  const bool compressed = !g.uncompressed;
  const float sc = g.scale_log2;
  // Query rows of this wave: block `wave` of the tile's q_blocks 32-row blocks; a wave
  // without rows (fewer than 8 blocks in the tile, or a ragged last tile) only stages.
  constexpr int NB = 1;
  const int row0 = (qt * g.q_blocks + wave) * 32;
  const int nblk = (wave < g.q_blocks && row0 < n) ? 1 : 0;
  // Frame-wise causal mask inside the call's own keys (Sec. 3.1): a query of frame a sees own keys 0 .. (a + 1) n_frame - 1.
  // own_limit: that count for this lane's query; own_limit_wave: the largest over the wave's rows (uniform).
  const int own_limit = (min(row0 + l32, n - 1) / g.n + 1) * g.n;
  const int own_limit_wave = (min(row0 + 31, n - 1) / g.n + 1) * g.n;
  bool started = false;                                   // this wave has computed a tile (the first one sets m)

  // ---- this wave's query fragments (B operand of S^T = K Q^T) ---------------------
  // They live in a private LDS region of the wave, one 16-byte entry per lane and
  // 16-channel step (fp32 input: a second set for the lo parts), and are re-read every
  // tile: the registers they would occupy hold the -m block below instead.
  // They are loaded together with the first tile's raw data, so that the two global
  // latencies overlap (rows past the frame repeat its last row; their output is not stored).
  uint4* qbase = lds_q + (wave * kQSets * 4) * 64 + lane;
  auto stage_q = [&]() __attribute__((always_inline)) {
    if (!nblk) return;
    const int qi = min(row0 + l32, n - 1);
    const uint8_t* qrow = reinterpret_cast<const uint8_t*>(it.q) +
                          ((int64_t)qi * g.tok_stride + (int64_t)h * g.head_stride + hf * 8) * (F32IN ? 4 : 2);
    if constexpr (F32IN) {
      uint4 a[4], c[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        a[ks] = *reinterpret_cast<const uint4*>(qrow + ks * 64);
        c[ks] = *reinterpret_cast<const uint4*>(qrow + ks * 64 + 16);
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const float x[8] = {__uint_as_float(a[ks].x), __uint_as_float(a[ks].y), __uint_as_float(a[ks].z), __uint_as_float(a[ks].w),
                            __uint_as_float(c[ks].x), __uint_as_float(c[ks].y), __uint_as_float(c[ks].z), __uint_as_float(c[ks].w)};
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split_bf16(x[2 * e], x[2 * e + 1], hi[e], lo[e]);
        qbase[(0 * 4 + ks) * 64] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        qbase[(1 * 4 + ks) * 64] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
      }
    } else {
      const uint4 q0 = *reinterpret_cast<const uint4*>(qrow), q1 = *reinterpret_cast<const uint4*>(qrow + 32);
      const uint4 q2 = *reinterpret_cast<const uint4*>(qrow + 64), q3 = *reinterpret_cast<const uint4*>(qrow + 96);
      qbase[0 * 64] = q0;
      qbase[1 * 64] = q1;
      qbase[2 * 64] = q2;
      qbase[3 * 64] = q3;
    }
  };

  f32x16 o[2][NB];                    // [channel block][query block]
  // Per query block (one here): the reference m (lanes l and l + 32 hold the same value), the running
  // row sum, and a 16-register block filled with -m that the first MFMA of every tile
  // takes as its accumulator input, so S^T leaves the matrix core as s - m.
  f32x16 negm[NB];
  float m_ref[NB], l_run[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m_ref[nb] = 0.f;
    l_run[nb] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[nb][r] = 0.f;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[cb][nb][r] = 0.f;
  }

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

  // Every raw load is addressed as a workgroup-uniform base (scalar registers, advanced per
  // tile by the scalar unit) plus a 32-bit offset of the lane.  For cache tiles the lane
  // offsets never change; they are computed here once.
  const uint32_t lo_kc = (uint32_t)(key_a * kKRow + co * KB);                        // K codes, first row
  const uint32_t lo_km = (uint32_t)((((key_a >> k_shift) * kHeadDim) + co * 8) * 4);  // K scales / zero-points
  const uint32_t lo_vc = (uint32_t)(key_a * kVRow + co * VB);                        // V codes, first row
  const uint32_t lo_vr = (uint32_t)(key_a * kVRow);                                  // start of that V code row
  const uint32_t lo_vm = (uint32_t)((key_a * ngv + ((co * 8) >> v_shift)) * (int)sizeof(VMeta));
  const uint32_t lo_un = (uint32_t)((key_a * kHeadDim + co * 8) * 2);                // row of an uncompressed cache

  // The loads of tile `tile`'s raw data for this thread.  `tile` may be any tile of the
  // range (a tile past the end is clamped by the caller and simply not decoded).
  auto load_raw = [&](auto rolec, auto& raw, int tile) __attribute__((always_inline)) {
    constexpr bool ROLE_K = decltype(rolec)::value;
    constexpr int B = ROLE_K ? KB : VB;
    typedef typename Octet<B>::type CodeT;
    const uint8_t *bc, *ba, *bz, *bm;          // uniform bases: codes, a[0..1], a[2..3], m
    uint32_t oc0, oc1, oa0, oa1, oa2, oa3, om0, om1;
    if (tile < ntc && compressed) {
      const int64_t row0t = (int64_t)h * g.t_cap + tile * kTileK;
      if constexpr (ROLE_K) {
        bc = half + g.lay.k_codes + row0t * kKRow;
        oc0 = lo_kc; oc1 = lo_kc + kKRow;
        const int64_t moff = ((int64_t)h * g.g_cap + ((tile * kTileK) >> k_shift)) * (kHeadDim * 4);
        ba = half + g.lay.k_scale + moff;
        bz = half + g.lay.k_zero + moff;
        oa0 = lo_km; oa1 = lo_km + 16; oa2 = lo_km; oa3 = lo_km + 16;
        bm = ba; om0 = om1 = lo_km;
      } else {
        bc = half + g.lay.v_codes + row0t * kVRow;
        oc0 = lo_vc; oc1 = lo_vc + kVRow;
        bm = half + g.lay.v_meta + row0t * ngv * (int64_t)sizeof(VMeta);
        om0 = lo_vm; om1 = lo_vm + ngv * (int)sizeof(VMeta);
        ba = bz = bc; oa0 = oa1 = oa2 = oa3 = lo_vr;
      }
    } else {
      if (tile < ntc) {
        // uncompressed bf16 cache: rows of 64 bf16; the row after a tile's last valid one is in bounds
        ba = half + (ROLE_K ? g.lay.k_codes : g.lay.v_codes) + ((int64_t)h * g.t_cap + tile * kTileK) * (kHeadDim * 2);
        oa0 = lo_un; oa1 = lo_un + kHeadDim * 2;
        oa2 = oa3 = oa0;
      } else {
        const int trow = (tile - ntc) * kTileK;
        const int lim = n - 1 - trow;                                   // rows past the frame are zeroed when decoded
        const uint32_t r0 = (uint32_t)min(key_a, lim), r1 = (uint32_t)min(key_a + 1, lim);
        constexpr uint32_t elt = F32IN ? 4 : 2;
        ba = reinterpret_cast<const uint8_t*>(ROLE_K ? it.k : it.v) + ((int64_t)trow * g.tok_stride + (int64_t)h * g.head_stride) * elt;
        const uint32_t ts = (uint32_t)g.tok_stride;
        const uint32_t q0 = (r0 * ts + co * 8) * elt, q1 = (r1 * ts + co * 8) * elt;
        if constexpr (F32IN) {
          oa0 = q0; oa1 = q0 + 16; oa2 = q1; oa3 = q1 + 16;
        } else {
          oa0 = q0; oa1 = q1; oa2 = oa3 = q0;
        }
      }
      bz = bc = bm = ba;
      oc0 = oc1 = om0 = om1 = oa0;
    }
    raw.c[0] = *reinterpret_cast<const CodeT*>(bc + oc0);
    raw.c[1] = *reinterpret_cast<const CodeT*>(bc + oc1);
    raw.a[0] = *reinterpret_cast<const uint4*>(ba + oa0);
    raw.a[1] = *reinterpret_cast<const uint4*>(ba + oa1);
    if constexpr (ROLE_K || F32IN) {
      raw.a[2] = *reinterpret_cast<const uint4*>(bz + oa2);
      raw.a[3] = *reinterpret_cast<const uint4*>(bz + oa3);
    }
    if constexpr (!ROLE_K) {
      raw.m[0] = *reinterpret_cast<const uint2*>(bm + om0);
      raw.m[1] = *reinterpret_cast<const uint2*>(bm + om1);
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
  auto decode_store = [&](auto rolec, const auto& raw, int tile, int buf) __attribute__((always_inline)) {
    constexpr bool ROLE_K = decltype(rolec)::value;
    if (tile < ntc && compressed) {
      // s * (code - z) evaluated as fma(code, s, -z * s): one conversion and one fused
      // operation per value (the result differs from Eq. 10's by a rounding of z * s, far
      // below what the bf16 pair or the f16 value keeps)
      const int ja = tile * kTileK + key_a;
      const bool full = (tile + 1) * kTileK <= t_c;       // uniform; only a cache's last tile can be ragged
      if constexpr (ROLE_K) {
        const uint32_t sw[8] = {raw.a[0].x, raw.a[0].y, raw.a[0].z, raw.a[0].w, raw.a[1].x, raw.a[1].y, raw.a[1].z, raw.a[1].w};
        const uint32_t zw[8] = {raw.a[2].x, raw.a[2].y, raw.a[2].z, raw.a[2].w, raw.a[3].x, raw.a[3].y, raw.a[3].z, raw.a[3].w};
        float sk[8], nz[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          sk[e] = __uint_as_float(sw[e]) * sc;
          nz[e] = -(float)(int32_t)zw[e] * sk[e];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          float f[8], x[8];
          octet_floats<KB>(raw.c[i], f);
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(f[e], sk[e], nz[e]);
          store_k_split(buf, i, x);        // rows past the cache's end hold finite stale values; their logits are masked
        }
      } else {
        // rows past the cache's end become zeros (scale and offset zero): their probabilities are zero too
        const bool ok0 = full || ja < t_c, ok1 = full || ja + 1 < t_c;
        const float s0 = ok0 ? __uint_as_float(raw.m[0].x) : 0.f, s1 = ok1 ? __uint_as_float(raw.m[1].x) : 0.f;
        const float nz0 = -(float)(int32_t)raw.m[0].y * s0, nz1 = -(float)(int32_t)raw.m[1].y * s1;
        float fa[8], fb[8], va[8], vb[8];
        octet_floats<VB>(raw.c[0], fa);
        octet_floats<VB>(raw.c[1], fb);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          va[e] = __builtin_fmaf(fa[e], s0, nz0);
          vb[e] = __builtin_fmaf(fb[e], s1, nz1);
        }
        store_v_pair(buf, va, vb);
      }
    } else {
      int base_row, limit;
      if (tile < ntc) { base_row = tile * kTileK; limit = t_c; } else { base_row = (tile - ntc) * kTileK; limit = n; }
      const bool ok0 = base_row + key_a < limit, ok1 = base_row + key_a + 1 < limit;
      float x0[8], x1[8];
      if (F32IN && tile >= ntc) {
        if constexpr (F32IN) {
          const uint32_t r0[8] = {raw.a[0].x, raw.a[0].y, raw.a[0].z, raw.a[0].w, raw.a[1].x, raw.a[1].y, raw.a[1].z, raw.a[1].w};
          const uint32_t r1[8] = {raw.a[2].x, raw.a[2].y, raw.a[2].z, raw.a[2].w, raw.a[3].x, raw.a[3].y, raw.a[3].z, raw.a[3].w};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            x0[e] = ok0 ? __uint_as_float(r0[e]) : 0.f;
            x1[e] = ok1 ? __uint_as_float(r1[e]) : 0.f;
          }
        }
      } else {
        uint4 r0 = raw.a[0], r1 = raw.a[1];
        if (!ok0) r0 = make_uint4(0, 0, 0, 0);
        if (!ok1) r1 = make_uint4(0, 0, 0, 0);
        const uint32_t a4[4] = {r0.x, r0.y, r0.z, r0.w}, b4[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          x0[2 * e2] = bf16lo_to_f32(a4[e2]); x0[2 * e2 + 1] = bf16hi_to_f32(a4[e2]);
          x1[2 * e2] = bf16lo_to_f32(b4[e2]); x1[2 * e2 + 1] = bf16hi_to_f32(b4[e2]);
        }
      }
      if constexpr (ROLE_K) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { x0[e] *= sc; x1[e] *= sc; }
        store_k_split(buf, 0, x0);
        store_k_split(buf, 1, x1);
      } else {
        store_v_pair(buf, x0, x1);
      }
    }
  };

  // ---- one tile: S^T, then softmax and O^T ---------------------------------------------
  const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
  auto compute = [&](int t, int kbuf, int vbuf, bool first) __attribute__((always_inline)) {
    f32x16 s[2][NB];                               // [key half][query block], log2-domain logits minus m
    // The operands come from LDS a few steps ahead of the MFMAs that use them (a step =
    // one key half of one 16-channel slice: the K hi and lo fragments).
    constexpr int kAhead = 3;
    bf16x8 ah[8], al[8], qh[4][NB], ql[4];
    auto read_k = [&](int i) __attribute__((always_inline)) {
      const int ks = i >> 1, mb = i & 1;
      const int aoff = (mb * 32 + l32) * kLdsRow + ks * 16 + hf * 8;
      ah[i] = *reinterpret_cast<const bf16x8*>(lds_khi[kbuf] + aoff);
      al[i] = *reinterpret_cast<const bf16x8*>(lds_klo[kbuf] + aoff);
    };
    auto read_q = [&](int ks) __attribute__((always_inline)) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) qh[ks][nb] = __builtin_bit_cast(bf16x8, qbase[ks * 64]);
      if constexpr (F32IN) ql[ks] = __builtin_bit_cast(bf16x8, qbase[(1 * 4 + ks) * 64]);
    };
    read_q(0);
#pragma unroll
    for (int i = 0; i < kAhead; ++i) read_k(i);
    read_q(1);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int ks = i >> 1, mb = i & 1;
      if (i + kAhead < 8) read_k(i + kAhead);
      if (mb == 0 && ks + 2 < 4) read_q(ks + 2);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        if (ks == 0) s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], qh[ks][nb], negm[nb], 0, 0, 0);
        else s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], qh[ks][nb], s[mb][nb], 0, 0, 0);
        s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], qh[ks][nb], s[mb][nb], 0, 0, 0);
        if constexpr (F32IN) s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], ql[ks], s[mb][nb], 0, 0, 0);
      }
    }
    // pin the order: the initial reads, then per step the reads issued for later steps and its MFMAs
    sched_group<0x100, 2 * kAhead + 2 * NB + (F32IN ? 2 : 0)>();
    pin_qk_steps<NB, F32IN, kAhead>(std::make_integer_sequence<int, 8>{});
    __builtin_amdgcn_s_setprio(0);

    // keys this lane's query may see in the tile: a cache tile's valid rows (ragged last tile), or the own keys up
    // to the end of the query's frame (frame-wise causal mask; also covers the ragged end of the call's rows)
    const int valid = (t < ntc) ? t_c - t * kTileK : own_limit - (t - ntc) * kTileK;
    if (__any(valid < kTileK)) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = mb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key >= valid) {
            s[mb][0][r] = kNegBig;
          }
        }
    }
    // p = 2^(s - m), packed to f16 as the B operand of the second product, summed into l.
    // The reference m is not checked beforehand: a key that exceeds it by more than the
    // f16 range allows turns its p, and with it the row sum, into infinity; only then
    // (rare, wave-uniform), and on the wave's first tile, are the references raised and
    // the probabilities formed again.
    f16x8 pb[NB][4];                  // [query block][16-key step]
    float l_new[NB];
    // V^T fragments of the first two 16-key steps are requested now, the rest while the
    // second product runs
    f16x8 vf[4][2];
    auto read_v = [&](int kk) __attribute__((always_inline)) {
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        vf[kk][cb] = *reinterpret_cast<const f16x8*>(lds_v[vbuf] + (cb * 32 + l32) * kLdsRow + kk * 16 + hf * 8);
    };
    read_v(0);
    read_v(1);
    auto probabilities = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        float l = l_run[nb];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const int mb = kk >> 1, r0 = (kk & 1) * 8;
          uint32_t w[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p0 = __builtin_amdgcn_exp2f(s[mb][nb][r0 + 2 * e]);
            const float p1 = __builtin_amdgcn_exp2f(s[mb][nb][r0 + 2 * e + 1]);
            w[e] = pack_f16(p0, p1);
            l = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w[e]), ones, l, false);
          }
          pb[nb][kk] = __builtin_bit_cast(f16x8, make_uint4(w[0], w[1], w[2], w[3]));
        }
        l_new[nb] = l;
      }
    };
    bool redo = first;                // the first tile sets m from its own keys (m starts at 0)
    if (!first) {
      probabilities();
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) redo |= !(l_new[nb] < kSumLimit);
    }
    if (__any(redo)) {
      // raise the references of the rows whose largest key exceeds them by more than the gap
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        float a = fmaxf(s[0][nb][0], s[1][nb][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) a = fmaxf(fmaxf(a, s[0][nb][r]), s[1][nb][r]);
        const float mq = fmaxf(a, __shfl_xor(a, 32));                // both halves of a query agree
        // a query that sees none of the tile's keys (all masked) keeps its reference
        const float delta = ((first && mq > 0.5f * kNegBig) || mq > kRescaleGap) ? mq : 0.f;
        const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(-delta);   // nothing accumulated before the first tile
        m_ref[nb] += delta;
        l_run[nb] *= alpha;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[cb][nb][r] *= alpha;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[mb][nb][r] -= delta;
#pragma unroll
        for (int r = 0; r < 16; ++r) negm[nb][r] = -m_ref[nb];
      }
      probabilities();
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) l_run[nb] = l_new[nb];
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk + 2 < 4) read_v(kk + 2);
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) o[cb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[kk][cb], pb[nb][kk], o[cb][nb], 0, 0, 0);
    }
    sched_group<0x100, 4>();
    sched_group<0x008, 2 * NB>();
    sched_group<0x100, 4>();
    sched_group<0x008, 6 * NB>();
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
  // Between two workgroup barriers waves 0-3 (K stagers) compute tile t and then stage tile
  // t+1, waves 4-7 (V stagers) stage first and then compute, the others only compute.  A
  // tile's raw data is loaded one interval before it is decoded.
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
  if (!started) m_ref[0] = kNegBig;     // an empty (or wholly masked) key range weighs nothing in the merge
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int qi = (nb < nblk) ? row0 + nb * 32 + l32 : n;
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
      // a query that saw no key in this range (all masked) has l = 0: its reference must not raise the merge's maximum
      if (hf == 0) *reinterpret_cast<float2*>(g.part_ml + row * 2) = make_float2(l_tot > 0.f ? m_ref[nb] : kNegBig, l_tot);
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
  if (qi >= g.n_new) return;
  // all partials are requested before any is used
  const int64_t row0 = ((int64_t)blockIdx.z * g.n_splits * g.H + h) * g.n_pad + qi;
  const int64_t row_step = (int64_t)g.H * g.n_pad;
  float2 ml[kMaxSplits];
  float4 po[kMaxSplits];
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s) {
    if (s < g.n_splits) {
      const int64_t row = row0 + s * row_step;
      ml[s] = *reinterpret_cast<const float2*>(g.part_ml + row * 2);
      po[s] = *reinterpret_cast<const float4*>(g.part_o + row * kHeadDim + c);
    }
  }
  float m_max = kNegBig;
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s)
    if (s < g.n_splits) m_max = fmaxf(m_max, ml[s].x);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float l = 0.f;
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s) {
    if (s < g.n_splits) {
      const float w = __builtin_amdgcn_exp2f(ml[s].x - m_max);
      acc.x += w * po[s].x; acc.y += w * po[s].y; acc.z += w * po[s].z; acc.w += w * po[s].w;
      l += w * ml[s].y;
    }
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
static void launch_attn_t(const KvxBatch& b, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const Geometry& g = b.g;
  dim3 grid(g.n_qtiles * g.H * b.n_items * g.n_splits);
  const dim3 block(64 * (g.q_blocks > 8 ? g.q_blocks : 8));      // a wave per query block, at least the 8 staging waves
  // with events: the runtime stamps them at the kernel's own start and end (what a kernel trace reports)
  if (ev_start) {
    if (g.in_f32) hipExtLaunchKernelGGL((attn_kernel<KB, VB, true>), grid, block, 0, st, ev_start, ev_stop, 0, b);
    else hipExtLaunchKernelGGL((attn_kernel<KB, VB, false>), grid, block, 0, st, ev_start, ev_stop, 0, b);
  } else {
    if (g.in_f32) hipLaunchKernelGGL((attn_kernel<KB, VB, true>), grid, block, 0, st, b);
    else hipLaunchKernelGGL((attn_kernel<KB, VB, false>), grid, block, 0, st, b);
  }
}

void launch_attention(const KvxBatch& b, int /*max_tiles*/, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const int kb = b.g.uncompressed ? 4 : b.g.k_bits, vb = b.g.uncompressed ? 4 : b.g.v_bits;
#define KVX_CASE(K, V) if (kb == K && vb == V) { launch_attn_t<K, V>(b, st, ev_start, ev_stop); return; }
  KVX_CASE(4, 4) KVX_CASE(8, 8) KVX_CASE(2, 4) KVX_CASE(2, 2) KVX_CASE(4, 8) KVX_CASE(8, 4) KVX_CASE(4, 2) KVX_CASE(2, 8) KVX_CASE(8, 2)
#undef KVX_CASE
}

void launch_combine(const KvxBatch& b, hipStream_t st) {
  const Geometry& g = b.g;
  if (g.n_splits <= 1) return;
  dim3 grid((g.n_new + 15) / 16, g.H, b.n_items);
  hipLaunchKernelGGL(combine_kernel, grid, dim3(256), 0, st, b);
}

}  // namespace kvx
