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

struct VMeta {                      // per (head, token, channel group) value metadata, fp32 metadata format
  float s;
  int32_t z;
};
// 16-bit metadata format.  Keys: two arrays of halfs, the logit-domain scale a = s * scale_log2 (7 significant
// bits) and zz = 1024 + z; within every eight channels the halfs are stored in the order 0 4 1 5 2 6 3 7 (the
// order in which the attention kernel's packed unpacking of a code word produces channel pairs).  Values: one
// 32-bit word per (head, token, channel group), low half the scale s, high half zz = 1024 + z.
constexpr float kMeta16ScaleMin = 0x1p-14f;   // smallest normal half
constexpr float kMeta16ScaleMax = 2048.0f;
constexpr int kMeta16ZMin = -1024, kMeta16ZMax = 1023;
__host__ __device__ __forceinline__ int meta16_pos(int c) { return (c & ~7) | ((c & 3) << 1) | ((c >> 2) & 1); }

// Byte offsets of the parts of one half of a cache's double buffer.
struct CacheLayout {
  int64_t k_codes;    // [H][t_cap][d * k_bits / 8]
  int64_t k_scale;    // [H][g_cap][d] float (16-bit metadata: half, logit-domain scale)
  int64_t k_zero;     // [H][g_cap][d] int32 (16-bit metadata: half, 1024 + z)
  int64_t v_codes;    // [H][t_cap][d * v_bits / 8]
  int64_t v_meta;     // [H][t_cap][d / v_group] VMeta (16-bit metadata: uint32)
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
  int64_t newtok;     // [t_cap] int32, slot layout: index of the call's token a slot receives, -1 for a slot whose token stays
  int64_t assign;     // [tokens of the largest call] int32, slot layout: slot of the call's i-th token
  int64_t sel;        // [16] int32: [0] first dropped position, [1] first rebuilt key group, [2] groups rebuilt (running), [3] kept middle tokens, [5] groups quantised with a zero-point beyond +-2^20 (running), [6] non-finite input seen (debug checks)
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
  int32_t n_new;          // tokens this call brings: n_frames * n (query rows, own keys, appended tokens)
  int32_t own_tiles;      // 1: attention reads the call's K/V from the inputs behind the cache; 0: they are in the cache already
                          //    (update-first order: items then name the updated half and its length)
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
  int32_t n_pad;          // query rows of this call padded to n_qtiles * q_blocks * 32
  int32_t n_qtiles;       // query tiles (attention workgroups per head and key split)
  int32_t q_blocks;       // 32-row query blocks per tile (<= 12, one per wave)
  float scale_log2;       // softmax scale * log2(e)
  float inv_scale_log2;   // fp32(1 / scale_log2): s = a * inv_scale_log2 in the 16-bit metadata format
  int32_t meta16;         // 1: 16-bit scales and zero-points
  int32_t slots;          // 1: slot-stable layout (one buffer, tokens never move), 0: compacting double buffer
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

// ---- device-side address helpers ------------------------------------------------
__device__ __forceinline__ uint8_t* cache_half(const Geometry& g, int cache, int half) {
  return g.arena + (int64_t)cache * g.lay.cache_bytes + (int64_t)half * g.lay.half_bytes;
}
__device__ __forceinline__ uint8_t* cache_scratch(const Geometry& g, int cache) {
  return g.scratch + (int64_t)cache * g.sl.bytes;
}

// ---- launchers (each enqueues on `st`, never synchronises) ----------------------
void launch_attention(const KvxBatch& b, int max_tiles, hipStream_t st, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
void launch_attention16(const KvxBatch& b, hipStream_t st, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
void launch_combine(const KvxBatch& b, hipStream_t st);
void launch_pool(const KvxBatch& b, hipStream_t st);
void launch_score(const KvxBatch& b, int max_tc, hipStream_t st);
void launch_select(const KvxBatch& b, int max_tc, hipStream_t st);
void launch_rebuild_k(const KvxBatch& b, int max_tnew, hipStream_t st);
void launch_rebuild_v(const KvxBatch& b, int max_tnew, hipStream_t st);
void launch_append_bf16(const KvxBatch& b, hipStream_t st);
void launch_check_finite(const KvxBatch& b, hipStream_t st);

constexpr int32_t kZeroPointWarn = 1 << 20;   // |z| beyond this is counted by kv_stats (zp_range_warnings)

}  // namespace kvx
