// Shared declarations between the host side of libkvx and its HIP kernels.
// Everything a kernel needs arrives by value in one KvxBatch kernel argument:
// the common geometry plus one small record per cache being stepped.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvx {

constexpr int kHeadDim = 64;        // d; the kernels are written for 64 channels per head
constexpr int kTileK = 64;          // keys per attention tile / tokens per rebuild block
constexpr int kQTileMax = 384;      // most query rows per attention workgroup (12 waves x 32)
constexpr int kMaxItems = 48;       // caches per launch (bounded by the kernel-argument size)
constexpr int kMaxSplits = 16;      // key-range splits per attention workgroup column

struct VMeta {                      // per (head, token, channel group) value metadata
  float s;
  int32_t z;
};

// Byte offsets of the parts of one half of a cache's double buffer.
struct CacheLayout {
  int64_t k_codes;    // [H][t_cap][d * k_bits / 8]
  int64_t k_scale;    // [H][g_cap][d] float
  int64_t k_zero;     // [H][g_cap][d] int32
  int64_t k_att;      // [H][g_cap][kAttBlock bytes]: the key metadata in the form the attention kernel consumes (see below)
  int64_t v_codes;    // [H][t_cap][d * v_bits / 8]
  int64_t v_meta;     // [H][t_cap][d / v_group] VMeta
  int64_t ids;        // [t_cap] int32
  int64_t half_bytes; // size of one half
  int64_t cache_bytes;// both halves
};

// Byte offsets inside one cache's private scratch.
struct ScratchLayout {
  int64_t qbar;       // [n_pooled][64] float: head-mean pooled query rows
  int64_t qt;         // [64] float: mean of the pooled rows
  int64_t dots;       // [H][t_cap] float: per-head q~ . K~
  int64_t scores;     // [t_cap] float: importance score of middle tokens (index = cache position - n)
  int64_t keys;       // [t_cap] uint32: order-preserving image of the scores
  int64_t keep;       // [t_cap] int32: kept positions, ascending
  int64_t sel;        // [16] int32: [0] first dropped position, [1] first rebuilt key group, [2] groups rebuilt (running), [3] kept middle tokens, [4] pooled-row blocks finished
  int64_t bytes;
};

struct Geometry {
  uint8_t* arena;         // caches: arena + cache * lay.cache_bytes + half * lay.half_bytes + offset
  uint8_t* scratch;       // per-cache scratch: scratch + cache * sl.bytes + offset
  float* part_o;          // attention partials [slot][H][n_pad][64], slot = item * n_splits + split
  float* part_ml;         // [slot][H][n_pad][2]: running max (log2 units) and sum
  CacheLayout lay;
  ScratchLayout sl;
  int64_t tok_stride;     // q/k/v strides in elements
  int64_t head_stride;
  int64_t out_tok_stride; // out strides in elements of the output dtype
  int64_t out_head_stride;
  int32_t H;
  int32_t n;              // tokens per frame
  int32_t n_special;
  int32_t pool_group;
  int32_t n_pooled;
  int32_t budget;
  int32_t t_cap;          // token capacity of a cache half (multiple of 64)
  int32_t g_cap;          // key-group capacity
  int32_t k_bits, k_group, v_bits, v_group;
  int32_t in_f32;         // 1: q/k/v are fp32, 0: bf16
  int32_t out_f32;        // 1: out is fp32, 0: bf16
  int32_t uncompressed;   // 1: bf16 cache without pruning or quantisation
  int32_t n_splits;
  int32_t n_pad;          // query rows padded to n_qtiles * q_blocks * 32
  int32_t n_qtiles;       // query tiles (attention workgroups per head and key split)
  int32_t q_blocks;       // 32-row query blocks per tile (<= 12, one per wave)
  float scale_log2;       // softmax scale * log2(e)
};

struct Item {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  int32_t cache;     // cache index = stream * n_layers + layer
  int32_t t_c;       // cache length before this step
  int32_t cur;       // which half holds the cache now (the step writes the other)
  int32_t prune;     // 1 if t_c + n > budget
  int32_t frame;     // index of this frame within its stream (for token ids)
  int32_t g0_host;   // first key group to rebuild when not pruning
  int32_t pad0, pad1;
};

struct KvxBatch {
  Geometry g;
  int32_t n_items;
  int32_t pad;
  Item items[kMaxItems];
};

// ---- key metadata for attention ---------------------------------------------------
// A cached key is s * (code - z) (Sec. 3.3 Eq. 10).  With m = code - z a small integer and
// sk = s * (softmax scale * log2 e) split as sk = a + b, a = the top kAttSplitBits
// significant bits of sk, the product m * a is exact in f16 and m * b is a small correction,
// so the attention kernel forms the key as an f16 pair (m * a, m * b) with packed f16
// arithmetic.  Per (head, group) a block of kAttBlock bytes holds three planes of 64 f16
// (a, b and 1024 + z per channel) and a 16-byte tail whose first word is nonzero if some
// channel of the group cannot take that path (zero-point out of range, scale outside f16's
// normal range).  The channels of a plane are stored in the order the attention kernel
// keeps them in LDS: codes that sit 16 bits apart in a code word become the two halves of
// one packed value.
constexpr int kAttBlock = 3 * kHeadDim * 2 + 16;
constexpr int kAttSplitBits = 6;          // significant bits of a: |m| < 32 keeps m * a within f16's 11
constexpr int kAttZMin = -16, kAttZMax = 31;
// position (0..15) of channel i (0..15) of a 16-channel slice in the stored order
template <int B>
__host__ __device__ constexpr int k_att_pos(int i) {
  if (B == 4) return (i & 8) | (((i & 3) << 1) | ((i >> 2) & 1));     // per octet: 0,4,1,5,2,6,3,7
  if (B == 2) return ((i & 7) << 1) | (i >> 3);                       // per slice: 0,8,1,9,...,7,15
  return i;
}
// channel (0..15) held at stored position p (0..15)
template <int B>
__host__ __device__ constexpr int k_att_chan(int p) {
  if (B == 4) return (p & 8) | ((p & 7) >> 1) | ((p & 1) << 2);
  if (B == 2) return (p >> 1) | ((p & 1) << 3);
  return p;
}

// ---- device-side address helpers ------------------------------------------------
__device__ __forceinline__ uint8_t* cache_half(const Geometry& g, int cache, int half) {
  return g.arena + (int64_t)cache * g.lay.cache_bytes + (int64_t)half * g.lay.half_bytes;
}
__device__ __forceinline__ uint8_t* cache_scratch(const Geometry& g, int cache) {
  return g.scratch + (int64_t)cache * g.sl.bytes;
}

// ---- launchers (each enqueues on `st`, never synchronises) ----------------------
void launch_attention(const KvxBatch& b, int max_tiles, hipStream_t st);
void launch_combine(const KvxBatch& b, hipStream_t st);
void launch_pool(const KvxBatch& b, hipStream_t st);
void launch_score(const KvxBatch& b, int max_tc, hipStream_t st);
void launch_select(const KvxBatch& b, int max_tc, hipStream_t st);
void launch_rebuild_k(const KvxBatch& b, int max_tnew, hipStream_t st);
void launch_rebuild_v(const KvxBatch& b, int max_tnew, hipStream_t st);
void launch_append_bf16(const KvxBatch& b, hipStream_t st);

}  // namespace kvx
