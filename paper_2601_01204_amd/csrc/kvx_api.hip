// Host side of libkvx: configuration checks, the one-time device arena, per-cache
// bookkeeping (lengths are a function of the frame count, so the host never reads
// anything back during a step) and the launch sequence of a step.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/kvx.h"
#include "kvx_dev.h"

using namespace kvx;

namespace {

struct CacheState {
  int32_t frames = 0;
  int32_t t_c = 0;
  int32_t cur = 0;
  int32_t last_pruned = 0;
  int32_t last_scores_len = 0;
  int64_t dropped = 0;
};

struct TimedLaunch {
  hipEvent_t start, stop;
  int kernel;
};

thread_local std::string g_init_error;

// Partial results of the attention kernel's key-range splits for kv_step_static, the entry point that
// must not allocate.  Every GPU the library runs on holds its own copy of this array until the process
// ends.  In host code the name is only a stand-in for the symbol: the address a kernel can use is taken
// once per device with hipGetSymbolAddress (static_scratch_address below) and passed on as a pointer.
constexpr size_t kStaticScratchBytes = (size_t)KV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices] = {};
std::mutex g_static_scratch_lock;

// The address of `scratch` on `device`, which must be the current device.
hipError_t static_scratch_address(int device, void** out) {
  *out = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_static_scratch_lock);
  if (!g_static_scratch[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_static_scratch[device] = p;
  }
  *out = g_static_scratch[device];
  return hipSuccess;
}

int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// IEEE half <-> float on the host, for the 16-bit metadata format in kv_export / kv_import.  Every value that
// crosses here is a normal half that the float holds exactly (scales in [2^-14, 2048], integers up to 2047).
float half_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16, e = (h >> 10) & 0x1Fu, m = h & 0x3FFu;
  uint32_t u;
  if (e == 0) {
    if (m == 0) {
      u = sign;
    } else {                       // subnormal half: value m * 2^-24
      const float v = (float)m * 0x1p-24f;
      memcpy(&u, &v, 4);
      u |= sign;
    }
  } else if (e == 31) {
    u = sign | 0x7F800000u | (m << 13);
  } else {
    u = sign | ((e + 112u) << 23) | (m << 13);
  }
  float f;
  memcpy(&f, &u, 4);
  return f;
}
// Exact conversion or failure: true and *out set when f is a normal half (or zero).
bool float_to_half_exact(float f, uint16_t* out) {
  uint32_t u;
  memcpy(&u, &f, 4);
  const uint32_t sign = (u >> 16) & 0x8000u, e = (u >> 23) & 0xFFu, m = u & 0x7FFFFFu;
  if (e == 0 && m == 0) { *out = (uint16_t)sign; return true; }
  if (e < 113 || e > 142 || (m & 0x1FFFu)) return false;
  *out = (uint16_t)(sign | ((e - 112u) << 10) | (m >> 13));
  return true;
}

}  // namespace

struct kv_handle {
  kv_config cfg{};
  Geometry geo{};
  std::vector<CacheState> caches;
  std::vector<int32_t> stream_n;       // tokens per frame of each stream (kv_set_stream_tokens; default: tokens_per_frame)
  std::vector<int64_t> seen_in_call;   // per cache: the step call that last named it (duplicate check without a per-call allocation)
  int64_t call_id = 0;
  uint8_t* arena = nullptr;
  uint8_t* work = nullptr;             // per-cache working memory (pooled query, dots, scores, keep list, counters)
  void* static_scratch = nullptr;      // this device's address of the file-scope `scratch` array (kv_step_static)
  float* part_o = nullptr;
  float* part_ml = nullptr;
  int64_t bytes_arena = 0, bytes_scratch = 0, bytes_part = 0;
  int64_t part_rows_cap = 0;  // (cache, split) slots x padded query rows the partial-result buffers hold
  int32_t splits_override = 0;
  int32_t n_cus = 256;        // compute units of the device (an attention workgroup occupies one by itself)
  int32_t target_wgs = 192;   // three quarters of the CUs: the rest runs the cache-update chain beside attention
  bool target_explicit = false;   // set through "attention_target_workgroups": used as given
  int device = 0;
  // second stream for the score / prune / re-quantise chain, which is independent of the
  // attention launches of the same step (both only read the current cache half)
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  int32_t f_max = 1;          // most frames per call
  int32_t n_pad_max = 0;      // padded query rows of the largest call (sizes the partial-result buffers)
  int32_t overlap = 1;
  int32_t debug_checks = 0;
  std::string err;
  // timing
  uint32_t timing_mask = 0;
  int32_t timing_every = 1;     // bracket the launches of every n-th kv_step / kv_step_batched call only
  int64_t step_calls = 0;
  bool timing_now = false;      // this call is one of them
  std::vector<TimedLaunch> timed;
  std::vector<TimedLaunch> free_events;
};

namespace {

int fail(kv_handle* h, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (h) h->err = buf; else g_init_error = buf;
  return code;
}

bool is_bits(int b) { return b == 2 || b == 4 || b == 8; }

// Query tiling of a call that brings `rows` query rows: an attention workgroup holds up to 12 waves, one 32-row
// query block each; the blocks are spread evenly over the fewest workgroups.
void set_query_tiling(Geometry& g, int rows) {
  const int nblocks = (rows + 31) / 32;
  const int tile_blocks = 12;
  g.n_new = rows;
  g.n_qtiles = (nblocks + tile_blocks - 1) / tile_blocks;
  g.q_blocks = (nblocks + g.n_qtiles - 1) / g.n_qtiles;
  g.n_pad = g.n_qtiles * g.q_blocks * 32;
}

int validate(const kv_config* c) {
  if (!c) return fail(nullptr, KV_E_INVAL, "kv_init: cfg is NULL");
  if (c->n_streams < 1 || c->n_layers < 1) return fail(nullptr, KV_E_INVAL, "kv_init: n_streams and n_layers must be >= 1");
  if ((int64_t)c->n_streams * c->n_layers > (1 << 20)) return fail(nullptr, KV_E_RANGE, "kv_init: too many caches");
  if (c->n_heads < 1 || c->n_heads > 64) return fail(nullptr, KV_E_INVAL, "kv_init: n_heads must be in [1, 64]");
  if (c->head_dim != kHeadDim) return fail(nullptr, KV_E_INVAL, "kv_init: head_dim must be 64");
  if (c->tokens_per_frame < 1 || c->tokens_per_frame > (1 << 20)) return fail(nullptr, KV_E_INVAL, "kv_init: tokens_per_frame out of range");
  if (c->n_special < 0 || c->n_special > c->tokens_per_frame) return fail(nullptr, KV_E_INVAL, "kv_init: n_special must be in [0, tokens_per_frame]");
  if (c->pool_group < 1) return fail(nullptr, KV_E_INVAL, "kv_init: pool_group must be >= 1");
  if (c->in_dtype != KV_BF16 && c->in_dtype != KV_F32) return fail(nullptr, KV_E_INVAL, "kv_init: in_dtype must be KV_BF16 or KV_F32");
  if (c->out_dtype != KV_BF16 && c->out_dtype != KV_F32) return fail(nullptr, KV_E_INVAL, "kv_init: out_dtype must be KV_BF16 or KV_F32");
  if (!(c->softmax_scale >= 0.f) || !std::isfinite(c->softmax_scale)) return fail(nullptr, KV_E_INVAL, "kv_init: softmax_scale must be finite and >= 0");
  if (c->meta_format != KV_META_F32 && c->meta_format != KV_META_F16) return fail(nullptr, KV_E_INVAL, "kv_init: meta_format must be KV_META_F32 or KV_META_F16");
  if (c->meta_format == KV_META_F16) {
    if (c->mode != KV_COMPRESSED) return fail(nullptr, KV_E_INVAL, "kv_init: KV_META_F16 applies to the compressed cache only");
    if (c->k_bits != 2 && c->k_bits != 4) return fail(nullptr, KV_E_INVAL, "kv_init: KV_META_F16 needs k_bits of 2 or 4 (the key products are exact in half precision up to 4-bit codes)");
    if (c->in_dtype != KV_BF16) return fail(nullptr, KV_E_INVAL, "kv_init: KV_META_F16 needs in_dtype KV_BF16");
  }
  if (c->layout != KV_LAYOUT_COMPACT && c->layout != KV_LAYOUT_SLOTS) return fail(nullptr, KV_E_INVAL, "kv_init: layout must be KV_LAYOUT_COMPACT or KV_LAYOUT_SLOTS");
  if (c->layout == KV_LAYOUT_SLOTS && c->mode != KV_COMPRESSED) return fail(nullptr, KV_E_INVAL, "kv_init: KV_LAYOUT_SLOTS applies to the compressed cache");
  if (c->order != KV_ATTEND_THEN_PRUNE && c->order != KV_PRUNE_THEN_ATTEND) return fail(nullptr, KV_E_INVAL, "kv_init: order must be KV_ATTEND_THEN_PRUNE or KV_PRUNE_THEN_ATTEND");
  if (c->max_frames_per_step < 0 || c->max_frames_per_step > 64) return fail(nullptr, KV_E_INVAL, "kv_init: max_frames_per_step must be in [0, 64]");
  if (c->order == KV_PRUNE_THEN_ATTEND && (c->mode != KV_COMPRESSED || c->max_frames_per_step > 1))
    return fail(nullptr, KV_E_INVAL, "kv_init: KV_PRUNE_THEN_ATTEND applies to the compressed cache with one frame per call");
  if (c->mode == KV_COMPRESSED) {
    if ((int64_t)c->budget_tokens < (1 + (int64_t)std::max(1, c->max_frames_per_step)) * (int64_t)c->tokens_per_frame)
      return fail(nullptr, KV_E_INVAL, "kv_init: budget_tokens must be >= (1 + max_frames_per_step) * tokens_per_frame (the first frame and the current frames are always kept)");
    if (c->budget_tokens > 32768) return fail(nullptr, KV_E_RANGE, "kv_init: budget_tokens above 32768 is not supported");
    if (!is_bits(c->k_bits) || !is_bits(c->v_bits)) return fail(nullptr, KV_E_INVAL, "kv_init: k_bits and v_bits must be 2, 4 or 8");
    if (c->k_group != 32 && c->k_group != 64) return fail(nullptr, KV_E_INVAL, "kv_init: k_group must be 32 or 64");
    if (c->v_group != 32 && c->v_group != 64) return fail(nullptr, KV_E_INVAL, "kv_init: v_group must be 32 or 64");
  } else if (c->mode == KV_UNCOMPRESSED_BF16) {
    if (c->max_frames < 1) return fail(nullptr, KV_E_INVAL, "kv_init: max_frames must be >= 1 in KV_UNCOMPRESSED_BF16 mode");
    if ((int64_t)c->max_frames * c->tokens_per_frame > (1ll << 28)) return fail(nullptr, KV_E_RANGE, "kv_init: max_frames * tokens_per_frame too large");
  } else {
    return fail(nullptr, KV_E_INVAL, "kv_init: unknown mode");
  }
  return KV_OK;
}

// Key-range splits per (item, head, query tile) column.  A workgroup occupies a compute
// unit by itself, so a launch runs in rounds of `target_wgs` workgroups; the estimate below
// is rounds x (tiles per workgroup + a fixed per-workgroup cost of about three tiles for the
// first loads and the partial-result store), and the split count with the smallest
// estimate wins (fewer splits on ties: less merge traffic).
int pick_splits(const kv_handle* h, const Geometry& g, int n_items, int min_tiles, int target_wgs) {
  int s;
  if (h->splits_override > 0) {
    s = h->splits_override;
  } else {
    const int64_t base = (int64_t)n_items * g.H * g.n_qtiles;
    const int tiles = std::max(1, std::min(min_tiles, 1 << 20));
    // up to two rounds' worth of workgroups, and at least four splits to choose from
    const int cap = (int)std::min<int64_t>(kMaxSplits, std::max<int64_t>(4, (2 * (int64_t)target_wgs) / base));
    double best = 0.0;
    s = 1;
    for (int c = 1; c <= cap; ++c) {
      const int64_t rounds = (base * c + target_wgs - 1) / target_wgs;
      const double cost = (double)rounds * ((double)tiles / c + 3.0) + (c > 1 ? 1.0 : 0.0);
      if (c == 1 || cost < best * 0.98) { best = cost; s = c; }
    }
  }
  s = std::max(1, std::min(s, (int)kMaxSplits));
  s = std::min(s, std::max(1, min_tiles));
  return s;
}

void record(kv_handle* h, int kernel, bool start, hipStream_t st) {
  if (!h->timing_now || !(h->timing_mask & (1u << kernel))) return;
  if (start) {
    TimedLaunch t;
    if (!h->free_events.empty()) {
      t = h->free_events.back();
      h->free_events.pop_back();
    } else {
      if (h->timed.size() >= 16384) return;
      if (hipEventCreate(&t.start) != hipSuccess) return;
      if (hipEventCreate(&t.stop) != hipSuccess) { hipEventDestroy(t.start); return; }
    }
    t.kernel = kernel;
    hipEventRecord(t.start, st);
    h->timed.push_back(t);
  } else {
    if (h->timed.empty() || h->timed.back().kernel != kernel) return;
    hipEventRecord(h->timed.back().stop, st);
  }
}

// An event pair for a launch that stamps its own events (nothing is recorded here).
void timed_pair(kv_handle* h, int kernel, hipEvent_t* start, hipEvent_t* stop) {
  *start = *stop = nullptr;
  if (!h->timing_now || !(h->timing_mask & (1u << kernel))) return;
  TimedLaunch t;
  if (!h->free_events.empty()) {
    t = h->free_events.back();
    h->free_events.pop_back();
  } else {
    if (h->timed.size() >= 16384) return;
    if (hipEventCreate(&t.start) != hipSuccess) return;
    if (hipEventCreate(&t.stop) != hipSuccess) { hipEventDestroy(t.start); return; }
  }
  t.kernel = kernel;
  h->timed.push_back(t);
  *start = t.start;
  *stop = t.stop;
}

}  // namespace

extern "C" {

int kv_init(const kv_config* cfg, kv_handle** out) {
  if (!out) return fail(nullptr, KV_E_INVAL, "kv_init: out is NULL");
  *out = nullptr;
  int rc = validate(cfg);
  if (rc != KV_OK) return rc;
  kv_handle* h = new (std::nothrow) kv_handle();
  if (!h) return fail(nullptr, KV_E_NOMEM, "kv_init: host allocation failed");
  h->cfg = *cfg;
  const kv_config& c = h->cfg;
  Geometry& g = h->geo;
  const bool unc = c.mode == KV_UNCOMPRESSED_BF16;
  g.H = c.n_heads;
  g.n = c.tokens_per_frame;
  g.n_special = c.n_special;
  g.pool_group = c.pool_group;
  g.n_pooled = c.n_special + (c.tokens_per_frame - c.n_special + c.pool_group - 1) / c.pool_group;
  g.budget = unc ? c.max_frames * c.tokens_per_frame : c.budget_tokens;
  g.t_cap = (int32_t)align_up(g.budget, 64);
  g.k_bits = unc ? 16 : c.k_bits;
  g.v_bits = unc ? 16 : c.v_bits;
  g.k_group = unc ? 64 : c.k_group;
  g.v_group = unc ? 64 : c.v_group;
  g.g_cap = g.t_cap / g.k_group;
  g.in_f32 = c.in_dtype == KV_F32;
  g.out_f32 = c.out_dtype == KV_F32;
  g.uncompressed = unc;
  g.meta16 = c.meta_format == KV_META_F16;
  g.slots = c.layout == KV_LAYOUT_SLOTS;
  h->f_max = std::max(1, c.max_frames_per_step);
  g.own_tiles = 1;
  // buffers are sized for the largest call; n_pad only grows with the row count
  int n_pad_max = 0;
  for (int f = 1; f <= h->f_max; ++f) {
    set_query_tiling(g, f * g.n);
    n_pad_max = std::max(n_pad_max, g.n_pad);
  }
  set_query_tiling(g, g.n);
  const float scale = c.softmax_scale > 0.f ? c.softmax_scale : 1.0f / std::sqrt((float)kHeadDim);
  g.scale_log2 = scale * 1.4426950408889634f;
  g.inv_scale_log2 = 1.0f / g.scale_log2;

  // one half of a cache
  CacheLayout& L = g.lay;
  int64_t off = 0;
  const int64_t k_row = (int64_t)kHeadDim * g.k_bits / 8, v_row = (int64_t)kHeadDim * g.v_bits / 8;
  L.k_codes = off; off = align_up(off + (int64_t)g.H * g.t_cap * k_row, 256);
  const int64_t k_meta_elt = g.meta16 ? 2 : 4, v_meta_elt = g.meta16 ? 4 : (int64_t)sizeof(VMeta);
  L.k_scale = off; off = align_up(off + (unc ? 0 : (int64_t)g.H * g.g_cap * kHeadDim * k_meta_elt), 256);
  L.k_zero = off;  off = align_up(off + (unc ? 0 : (int64_t)g.H * g.g_cap * kHeadDim * k_meta_elt), 256);
  L.v_codes = off; off = align_up(off + (int64_t)g.H * g.t_cap * v_row, 256);
  L.v_meta = off;  off = align_up(off + (unc ? 0 : (int64_t)g.H * g.t_cap * (kHeadDim / g.v_group) * v_meta_elt), 256);
  L.ids = off;     off = align_up(off + (int64_t)g.t_cap * 4, 256);
  L.half_bytes = off;
  L.cache_bytes = (unc || g.slots) ? off : 2 * off;

  ScratchLayout& S = g.sl;
  off = 0;
  S.qbar = off;   off = align_up(off + (int64_t)g.n_pooled * h->f_max * kHeadDim * 4, 256);
  S.qt = off;     off = align_up(off + kHeadDim * 4, 256);
  S.dots = off;   off = align_up(off + (unc ? 0 : (int64_t)g.H * g.t_cap * 4), 256);
  S.scores = off; off = align_up(off + (unc ? 0 : (int64_t)g.t_cap * 4), 256);
  S.keys = off;   off = align_up(off + (unc ? 0 : (int64_t)g.t_cap * 4), 256);
  S.keep = off;   off = align_up(off + (unc ? 0 : (int64_t)g.t_cap * 4), 256);
  S.newtok = off; off = align_up(off + (g.slots ? (int64_t)g.t_cap * 4 : 0), 256);
  S.assign = off; off = align_up(off + (g.slots ? (int64_t)h->f_max * g.n * 4 : 0), 256);
  S.sel = off;    off = align_up(off + 64, 256);
  S.bytes = off;

  int cus = 0;
  if (hipGetDevice(&h->device) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device) != hipSuccess || cus < 1) {
    rc = fail(nullptr, KV_E_HIP, "kv_init: no HIP device: %s", hipGetErrorString(hipGetLastError()));
    delete h;
    return rc;
  }
  h->n_cus = cus;
  h->target_wgs = std::max(1, cus * 3 / 4);
  {
    const hipError_t e = static_scratch_address(h->device, &h->static_scratch);
    if (e != hipSuccess) {
      rc = fail(nullptr, KV_E_HIP, "kv_init: address of the static scratch array: %s", hipGetErrorString(e));
      (void)hipGetLastError();
      delete h;
      return rc;
    }
  }

  const int64_t n_caches = (int64_t)c.n_streams * c.n_layers;
  h->caches.assign((size_t)n_caches, CacheState());
  h->seen_in_call.assign((size_t)n_caches, 0);
  h->stream_n.assign((size_t)c.n_streams, c.tokens_per_frame);
  // Partial results of the key-range splits: room for the largest (caches per launch) x (splits) x (padded query rows)
  // the automatic choice can reach, found by running it over every launch shape this handle can see.
  int64_t rows_cap = 0;
  for (int f = 1; f <= h->f_max; ++f) {
    Geometry gf = g;
    set_query_tiling(gf, f * g.n);
    const int tiles_max = (g.t_cap + kTileK - 1) / kTileK + (gf.n_new + kTileK - 1) / kTileK;
    for (int items = 1; items <= std::min<int64_t>(kMaxItems, n_caches); ++items)
      for (int tiles = tiles_max; tiles >= 1; tiles = tiles > 1 ? (tiles + 1) / 2 : 0)
        for (int target : {h->target_wgs, cus}) {
          const int sp = pick_splits(h, gf, items, tiles, target);
          rows_cap = std::max(rows_cap, (int64_t)items * sp * gf.n_pad);
        }
  }
  set_query_tiling(g, g.n);
  h->part_rows_cap = rows_cap;
  h->bytes_arena = n_caches * L.cache_bytes;
  h->bytes_scratch = n_caches * S.bytes;
  h->n_pad_max = n_pad_max;
  const int64_t part_o_bytes = rows_cap * g.H * kHeadDim * 4;
  const int64_t part_ml_bytes = rows_cap * g.H * 2 * 4;
  h->bytes_part = part_o_bytes + part_ml_bytes;

  hipError_t e1 = hipMalloc((void**)&h->arena, (size_t)h->bytes_arena);
  hipError_t e2 = e1 == hipSuccess ? hipMalloc((void**)&h->work, (size_t)h->bytes_scratch) : e1;
  hipError_t e3 = e2 == hipSuccess ? hipMalloc((void**)&h->part_o, (size_t)part_o_bytes) : e2;
  hipError_t e4 = e3 == hipSuccess ? hipMalloc((void**)&h->part_ml, (size_t)part_ml_bytes) : e3;
  if (e4 != hipSuccess) {
    rc = fail(nullptr, e4 == hipErrorOutOfMemory ? KV_E_NOMEM : KV_E_HIP, "kv_init: device allocation of %lld bytes failed: %s",
              (long long)(h->bytes_arena + h->bytes_scratch + h->bytes_part), hipGetErrorString(e4));
    (void)hipGetLastError();
    kv_destroy(h);
    return rc;
  }
  if (hipMemset(h->arena, 0, (size_t)h->bytes_arena) != hipSuccess || hipMemset(h->work, 0, (size_t)h->bytes_scratch) != hipSuccess ||
      hipDeviceSynchronize() != hipSuccess) {
    rc = fail(nullptr, KV_E_HIP, "kv_init: clearing the arena failed: %s", hipGetErrorString(hipGetLastError()));
    kv_destroy(h);
    return rc;
  }
  if (hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking) != hipSuccess || hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&h->ev_join, hipEventDisableTiming) != hipSuccess) {
    rc = fail(nullptr, KV_E_HIP, "kv_init: creating the side stream failed: %s", hipGetErrorString(hipGetLastError()));
    kv_destroy(h);
    return rc;
  }
  g.arena = h->arena;
  g.scratch = h->work;
  g.part_o = h->part_o;
  g.part_ml = h->part_ml;
  *out = h;
  return KV_OK;
}

}  // extern "C"

namespace {

// One set of launches per group of up to kMaxItems caches.  part_o / part_ml: where the attention
// kernel's key-range splits leave their partial results, room for rows_cap rows: (cache, split) pairs x padded query rows.
// with_timing = false: no event is created or recorded by this call.
int step_impl(kv_handle* h, int32_t n_items, const kv_step_item* items, int32_t n_frames, int64_t tok_stride, int64_t head_stride,
              void* hip_stream, float* part_o, float* part_ml, int64_t rows_cap, bool with_timing) {
  if (n_items < 1 || !items) return fail(h, KV_E_INVAL, "kv_step: no items");
  const kv_config& c = h->cfg;
  if (n_frames < 1 || n_frames > h->f_max) return fail(h, KV_E_RANGE, "kv_step: %d frames in one call, the handle takes 1..%d (max_frames_per_step)", n_frames, h->f_max);
  Geometry g0 = h->geo;
  {
    // the frame size of this call: that of the items' streams, which must agree
    const int n_call = (items[0].stream >= 0 && items[0].stream < c.n_streams) ? h->stream_n[(size_t)items[0].stream] : g0.n;
    for (int i = 1; i < n_items; ++i)
      if (items[i].stream >= 0 && items[i].stream < c.n_streams && h->stream_n[(size_t)items[i].stream] != n_call)
        return fail(h, KV_E_INVAL, "kv_step: item %d: its stream has %d tokens per frame, item 0's has %d; one call carries frames of one size",
                    i, h->stream_n[(size_t)items[i].stream], n_call);
    g0.n = n_call;
    g0.n_pooled = g0.n_special + (n_call - g0.n_special + g0.pool_group - 1) / g0.pool_group;
  }
  set_query_tiling(g0, n_frames * g0.n);
  const int n_new = g0.n_new;
  const bool update_first = c.order == KV_PRUNE_THEN_ATTEND;
  const int64_t elt = g0.in_f32 ? 4 : 2;
  if (head_stride < kHeadDim || tok_stride < kHeadDim) return fail(h, KV_E_INVAL, "kv_step: strides must be >= head_dim");
  const int64_t oelt = g0.out_f32 ? 4 : 2;
  if ((tok_stride * elt) % 16 || (head_stride * elt) % 16 || (tok_stride * oelt) % 16 || (head_stride * oelt) % 16)
    return fail(h, KV_E_INVAL, "kv_step: strides must keep rows 16-byte aligned");
  const int64_t call = ++h->call_id;
  for (int i = 0; i < n_items; ++i) {
    const kv_step_item& it = items[i];
    if (it.stream < 0 || it.stream >= c.n_streams || it.layer < 0 || it.layer >= c.n_layers)
      return fail(h, KV_E_RANGE, "kv_step: item %d: stream %d / layer %d out of range", i, it.stream, it.layer);
    if (!it.q || !it.k || !it.v || !it.out) return fail(h, KV_E_INVAL, "kv_step: item %d: NULL pointer", i);
    if (((uintptr_t)it.q | (uintptr_t)it.k | (uintptr_t)it.v | (uintptr_t)it.out) & 15)
      return fail(h, KV_E_INVAL, "kv_step: item %d: pointers must be 16-byte aligned", i);
    const size_t ci = (size_t)it.stream * c.n_layers + it.layer;
    if (h->seen_in_call[ci] == call) return fail(h, KV_E_INVAL, "kv_step: cache (stream %d, layer %d) appears twice in one batch", it.stream, it.layer);
    h->seen_in_call[ci] = call;
    if (g0.uncompressed && h->caches[ci].frames + n_frames > c.max_frames)
      return fail(h, KV_E_STATE, "kv_step: cache (stream %d, layer %d) cannot take %d more frames (max_frames %d)", it.stream, it.layer, n_frames, c.max_frames);
  }
  hipStream_t st = (hipStream_t)hip_stream;
  h->timing_now = with_timing && h->timing_mask != 0 && (h->step_calls % h->timing_every) == 0;
  h->step_calls += 1;

  for (int base = 0; base < n_items; base += kMaxItems) {
    const int cnt = std::min<int>(kMaxItems, n_items - base);
    KvxBatch b;
    b.g = g0;
    b.g.tok_stride = tok_stride;
    b.g.head_stride = head_stride;
    b.g.out_tok_stride = tok_stride;
    b.g.out_head_stride = head_stride;
    b.n_items = cnt;
    b.pad = 0;
    int max_tc = 0, max_tnew = 0, min_tiles = 1 << 30;
    bool any_prune = false;
    for (int i = 0; i < cnt; ++i) {
      const kv_step_item& src = items[base + i];
      const size_t ci = (size_t)src.stream * c.n_layers + src.layer;
      const CacheState& cs = h->caches[ci];
      Item& it = b.items[i];
      it.q = src.q; it.k = src.k; it.v = src.v; it.out = src.out;
      it.cache = (int32_t)ci;
      it.t_c = cs.t_c;
      it.cur = cs.cur;
      it.prune = (!g0.uncompressed && cs.t_c + n_new > g0.budget) ? 1 : 0;
      it.frame = cs.frames;
      it.g0_host = cs.t_c / g0.k_group;
      it.pad0 = it.pad1 = 0;
      any_prune |= it.prune != 0;
      max_tc = std::max(max_tc, cs.t_c);
      const int t_after = std::min(cs.t_c + n_new, g0.budget);
      max_tnew = std::max(max_tnew, t_after);
      const int tiles = update_first ? (t_after + kTileK - 1) / kTileK : (cs.t_c + kTileK - 1) / kTileK + (n_new + kTileK - 1) / kTileK;
      min_tiles = std::min(min_tiles, tiles);
    }
    b.g.part_o = part_o;
    b.g.part_ml = part_ml;
    // The cache-update chain runs next to attention on the library's second stream when attention alone cannot fill
    // the chip (fewer workgroup columns than compute units: one or a few caches per call).  The attention workgroups
    // of a launch that fills the chip hold every vector register of their compute units, so another kernel's
    // workgroups only get a unit between two of them: there the chain follows attention on the caller's stream
    // unless "overlap_update" 2 asks for the second stream at any size.  The slot layout's writers always follow
    // attention (they update the buffer it reads); "overlap_update" 0, the uncompressed baseline and the update-first
    // order (attention reads what the update wrote) keep everything in order on the caller's stream.
    const bool may_overlap = h->overlap != 0 && h->side && !g0.uncompressed && !update_first;
    const bool small_launch = (int64_t)cnt * g0.H * g0.n_qtiles <= (int64_t)h->n_cus;
    const bool beside = may_overlap && (h->overlap == 2 || small_launch);
    // a small launch leaves a quarter of the compute units to the chain next to it
    b.g.n_splits = pick_splits(h, b.g, cnt, min_tiles, ((beside && small_launch) || h->target_explicit) ? h->target_wgs : h->n_cus);
    // never more splits than the partial-result buffers hold (an explicit "attention_splits" may ask for more)
    b.g.n_splits = (int32_t)std::max<int64_t>(1, std::min<int64_t>(b.g.n_splits, rows_cap / ((int64_t)cnt * b.g.n_pad)));

    hipStream_t sb = st;          // stream of the cache-update chain
    if (beside) {
      hipEventRecord(h->ev_fork, st);
      hipStreamWaitEvent(h->side, h->ev_fork, 0);
      sb = h->side;
    }
    // the slot layout is updated in place: its writers follow attention, which reads the same buffer
    const bool rebuild_after = g0.slots && !update_first;
    if (!g0.uncompressed) {
      if (any_prune) {
        record(h, KV_K_POOL, true, sb);
        launch_pool(b, sb);
        record(h, KV_K_POOL, false, sb);
        record(h, KV_K_SCORE, true, sb);
        launch_score(b, max_tc, sb);
        record(h, KV_K_SCORE, false, sb);
        record(h, KV_K_SELECT, true, sb);
        launch_select(b, max_tc, sb);
        record(h, KV_K_SELECT, false, sb);
      }
      if (!rebuild_after) {
        record(h, KV_K_REBUILD_K, true, sb);
        launch_rebuild_k(b, max_tnew, sb);
        record(h, KV_K_REBUILD_K, false, sb);
        record(h, KV_K_REBUILD_V, true, sb);
        launch_rebuild_v(b, max_tnew, sb);
        record(h, KV_K_REBUILD_V, false, sb);
      }
    }
    if (h->debug_checks) launch_check_finite(b, st);
    {
      // the attention kernel is timed by events the runtime stamps at the kernel's own start
      // and end, so the figure is the kernel's duration as a kernel trace reports it
      hipEvent_t e0 = nullptr, e1 = nullptr;
      timed_pair(h, KV_K_ATTENTION, &e0, &e1);
      if (update_first) {
        // the update above ran on this stream; attention reads the half it wrote, which already holds the frame
        KvxBatch ba = b;
        ba.g.own_tiles = 0;
        for (int i = 0; i < cnt; ++i) {
          if (!g0.slots) ba.items[i].cur ^= 1;
          ba.items[i].t_c = std::min(b.items[i].t_c + n_new, g0.budget);
        }
        if (g0.meta16) launch_attention16(ba, st, e0, e1);
        else launch_attention(ba, 0, st, e0, e1);
      } else if (g0.meta16) {
        launch_attention16(b, st, e0, e1);
      } else {
        launch_attention(b, 0, st, e0, e1);
      }
    }
    record(h, KV_K_COMBINE, true, st);
    launch_combine(b, st);
    record(h, KV_K_COMBINE, false, st);
    if (g0.uncompressed) {
      record(h, KV_K_REBUILD_V, true, st);
      launch_append_bf16(b, st);
      record(h, KV_K_REBUILD_V, false, st);
    }
    if (sb != st) {
      hipEventRecord(h->ev_join, sb);
      hipStreamWaitEvent(st, h->ev_join, 0);
    }
    if (rebuild_after) {
      record(h, KV_K_REBUILD_K, true, st);
      launch_rebuild_k(b, max_tnew, st);
      record(h, KV_K_REBUILD_K, false, st);
      record(h, KV_K_REBUILD_V, true, st);
      launch_rebuild_v(b, max_tnew, st);
      record(h, KV_K_REBUILD_V, false, st);
    }
    hipError_t le = hipGetLastError();
    if (le != hipSuccess) return fail(h, KV_E_HIP, "kv_step: launch failed: %s", hipGetErrorString(le));

    for (int i = 0; i < cnt; ++i) {
      CacheState& cs = h->caches[(size_t)b.items[i].cache];
      const int t_all = cs.t_c + n_new;
      cs.last_pruned = b.items[i].prune;
      cs.last_scores_len = b.items[i].prune ? cs.t_c - g0.n : 0;
      if (b.items[i].prune) cs.dropped += t_all - g0.budget;
      cs.t_c = std::min(t_all, g0.budget);
      cs.frames += n_frames;
      if (!g0.uncompressed && !g0.slots) cs.cur ^= 1;
    }
  }
  return KV_OK;
}

}  // namespace

extern "C" {

int kv_step_batched(kv_handle* h, int32_t n_items, const kv_step_item* items, int64_t tok_stride, int64_t head_stride, void* hip_stream) {
  if (!h) return KV_E_INVAL;
  return step_impl(h, n_items, items, 1, tok_stride, head_stride, hip_stream, h->part_o, h->part_ml, h->part_rows_cap, true);
}

int kv_step_frames(kv_handle* h, int32_t stream, int32_t layer, int32_t n_frames, const void* q, const void* k, const void* v,
                   int64_t tok_stride, int64_t head_stride, void* out, void* hip_stream) {
  if (!h) return KV_E_INVAL;
  kv_step_item it;
  it.stream = stream;
  it.layer = layer;
  it.q = q;
  it.k = k;
  it.v = v;
  it.out = out;
  return step_impl(h, 1, &it, n_frames, tok_stride, head_stride, hip_stream, h->part_o, h->part_ml, h->part_rows_cap, true);
}

int kv_step_static(kv_handle* h, int32_t stream, int32_t layer, const void* q, const void* k, const void* v, int64_t tok_stride,
                   int64_t head_stride, void* out, void* hip_stream) {
  if (!h) return KV_E_INVAL;
  const Geometry& g = h->geo;      // its query tiling is that of one frame
  // one (cache, split) slot: [H][n_pad][64] fp32 partial outputs + [H][n_pad][2] fp32 (max, sum), the two parts 256-byte aligned
  const int64_t slot_o = (int64_t)g.H * g.n_pad * kHeadDim * 4, slot_ml = (int64_t)g.H * g.n_pad * 2 * 4;
  const int64_t slots = std::min<int64_t>((int64_t)kStaticScratchBytes / (slot_o + slot_ml + 512), kMaxSplits);
  if (slots < 2)
    return fail(h, KV_E_RANGE, "kv_step_static: n_heads x tokens_per_frame = %d x %d needs %lld bytes for the partial results of two key-range "
                "splits, above the static scratch of %lld bytes", g.H, g.n, (long long)(2 * (slot_o + slot_ml)), (long long)kStaticScratchBytes);
  if (!h->static_scratch) return fail(h, KV_E_STATE, "kv_step_static: the static scratch array has no address on this device");
  float* part_o = reinterpret_cast<float*>(h->static_scratch);
  float* part_ml = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(h->static_scratch) + align_up(slots * slot_o, 256));
  kv_step_item it;
  it.stream = stream;
  it.layer = layer;
  it.q = q;
  it.k = k;
  it.v = v;
  it.out = out;
  return step_impl(h, 1, &it, 1, tok_stride, head_stride, hip_stream, part_o, part_ml, slots * g.n_pad, false);
}

int kv_step(kv_handle* h, int32_t stream, int32_t layer, const void* q, const void* k, const void* v, int64_t tok_stride,
            int64_t head_stride, void* out, void* hip_stream) {
  kv_step_item it;
  it.stream = stream;
  it.layer = layer;
  it.q = q;
  it.k = k;
  it.v = v;
  it.out = out;
  return kv_step_batched(h, 1, &it, tok_stride, head_stride, hip_stream);
}

int kv_stats(kv_handle* h, kv_stats_t* s) {
  if (!h) return KV_E_INVAL;
  if (!s) return fail(h, KV_E_INVAL, "kv_stats: stats is NULL");
  if (hipDeviceSynchronize() != hipSuccess) return fail(h, KV_E_HIP, "kv_stats: %s", hipGetErrorString(hipGetLastError()));
  const Geometry& g = h->geo;
  const int64_t nc = (int64_t)h->caches.size();
  const int64_t halves = (g.uncompressed || g.slots) ? 1 : 2;
  memset(s, 0, sizeof *s);
  s->bytes_allocated = h->bytes_arena + h->bytes_scratch + h->bytes_part;
  s->bytes_k_codes = nc * halves * ((int64_t)g.H * g.t_cap * kHeadDim * g.k_bits / 8);
  const int64_t meta_bytes = g.meta16 ? 4 : 8;      // scale + zero-point of one group
  s->bytes_k_meta = g.uncompressed ? 0 : nc * halves * ((int64_t)g.H * g.g_cap * (kHeadDim * meta_bytes));
  s->bytes_v_codes = nc * halves * ((int64_t)g.H * g.t_cap * kHeadDim * g.v_bits / 8);
  s->bytes_v_meta = g.uncompressed ? 0 : nc * halves * ((int64_t)g.H * g.t_cap * (kHeadDim / g.v_group) * meta_bytes);
  s->bytes_ids = nc * halves * (int64_t)g.t_cap * 4;
  s->bytes_scratch = h->bytes_scratch + h->bytes_part;
  s->n_caches = (int32_t)nc;
  int32_t mn = INT32_MAX, mx = 0;
  for (size_t i = 0; i < h->caches.size(); ++i) {
    const CacheState& cs = h->caches[i];
    s->frames_seen_total += cs.frames;
    s->tokens_dropped_total += cs.dropped;
    mn = std::min(mn, cs.t_c);
    mx = std::max(mx, cs.t_c);
    if (!g.uncompressed) {
      int32_t sel[8];
      if (hipMemcpy(sel, h->work + (int64_t)i * g.sl.bytes + g.sl.sel, sizeof sel, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(h, KV_E_HIP, "kv_stats: %s", hipGetErrorString(hipGetLastError()));
      s->k_groups_rebuilt_total += sel[2];
      s->zp_range_warnings += sel[5];
      s->nonfinite_flag |= sel[6] != 0;
    }
  }
  s->cache_len_min = mn;
  s->cache_len_max = mx;
  const int64_t T = mx;
  if (g.uncompressed) {
    s->bytes_live_per_cache = 2 * (int64_t)g.H * T * kHeadDim * 2;
  } else {
    const int64_t groups = (T + g.k_group - 1) / g.k_group;
    s->bytes_live_per_cache = (int64_t)g.H * T * kHeadDim * g.k_bits / 8 + (int64_t)g.H * groups * (kHeadDim * meta_bytes) +
                              (int64_t)g.H * T * kHeadDim * g.v_bits / 8 + (int64_t)g.H * T * (kHeadDim / g.v_group) * meta_bytes + T * 4;
  }
  return KV_OK;
}

int kv_export(kv_handle* h, int32_t stream, int32_t layer, kv_export_t* x) {
  if (!h) return KV_E_INVAL;
  if (!x) return fail(h, KV_E_INVAL, "kv_export: bufs is NULL");
  const kv_config& c = h->cfg;
  if (stream < 0 || stream >= c.n_streams || layer < 0 || layer >= c.n_layers) return fail(h, KV_E_RANGE, "kv_export: stream/layer out of range");
  const Geometry& g = h->geo;
  if (g.uncompressed) return fail(h, KV_E_STATE, "kv_export: not available in KV_UNCOMPRESSED_BF16 mode");
  const size_t ci = (size_t)stream * c.n_layers + layer;
  const CacheState& cs = h->caches[ci];
  const int T = cs.t_c;
  if (x->capacity_tokens < T) return fail(h, KV_E_RANGE, "kv_export: capacity_tokens %d < cache length %d", x->capacity_tokens, T);
  if (hipDeviceSynchronize() != hipSuccess) return fail(h, KV_E_HIP, "kv_export: %s", hipGetErrorString(hipGetLastError()));
  x->cache_len = T;
  x->frames_seen = cs.frames;
  x->last_keep_len = cs.last_pruned ? g.budget : 0;
  x->last_scores_len = cs.last_scores_len;
  const uint8_t* half = h->arena + (int64_t)ci * g.lay.cache_bytes + (int64_t)cs.cur * g.lay.half_bytes;
  const uint8_t* sc = h->work + (int64_t)ci * g.sl.bytes;
  const int H = g.H;
  const int G = (T + g.k_group - 1) / g.k_group;
  const int ngv = kHeadDim / g.v_group;
  auto d2h = [&](void* dst, const void* src, size_t bytes) { return bytes == 0 || hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost) == hipSuccess; };
  bool ok = true;
  if (x->ids) ok &= d2h(x->ids, half + g.lay.ids, (size_t)T * 4);
  auto unpack = [&](uint8_t* dst, int64_t lay_off, int bits) {
    const int row = kHeadDim * bits / 8;
    std::vector<uint8_t> tmp((size_t)T * row);
    for (int hh = 0; hh < H && ok; ++hh) {
      ok &= d2h(tmp.data(), half + lay_off + (int64_t)hh * g.t_cap * row, tmp.size());
      for (int j = 0; j < T; ++j)
        for (int ch = 0; ch < kHeadDim; ++ch) {
          const int bit = ch * bits;
          dst[((int64_t)hh * T + j) * kHeadDim + ch] = (uint8_t)((tmp[(size_t)j * row + (bit >> 3)] >> (bit & 7)) & ((1 << bits) - 1));
        }
    }
  };
  if (x->k_codes) unpack(x->k_codes, g.lay.k_codes, g.k_bits);
  if (x->v_codes) unpack(x->v_codes, g.lay.v_codes, g.v_bits);
  if (g.meta16) {
    // halfs in the device order of every eight channels; s = a * fp32(1 / scale_log2), z = zz - 1024
    std::vector<uint16_t> tmp((size_t)G * kHeadDim);
    for (int hh = 0; hh < H && ok; ++hh) {
      if (x->k_scale) {
        ok &= d2h(tmp.data(), half + g.lay.k_scale + (int64_t)hh * g.g_cap * kHeadDim * 2, tmp.size() * 2);
        for (int gi = 0; gi < G; ++gi)
          for (int ch = 0; ch < kHeadDim; ++ch)
            x->k_scale[((int64_t)hh * G + gi) * kHeadDim + ch] = half_to_float(tmp[(size_t)gi * kHeadDim + meta16_pos(ch)]) * g.inv_scale_log2;
      }
      if (x->k_zero) {
        ok &= d2h(tmp.data(), half + g.lay.k_zero + (int64_t)hh * g.g_cap * kHeadDim * 2, tmp.size() * 2);
        for (int gi = 0; gi < G; ++gi)
          for (int ch = 0; ch < kHeadDim; ++ch)
            x->k_zero[((int64_t)hh * G + gi) * kHeadDim + ch] = (int32_t)half_to_float(tmp[(size_t)gi * kHeadDim + meta16_pos(ch)]) - 1024;
      }
    }
    if (x->v_scale || x->v_zero) {
      std::vector<uint32_t> vt((size_t)T * ngv);
      for (int hh = 0; hh < H && ok; ++hh) {
        ok &= d2h(vt.data(), half + g.lay.v_meta + (int64_t)hh * g.t_cap * ngv * 4, vt.size() * 4);
        for (size_t i = 0; i < vt.size(); ++i) {
          if (x->v_scale) x->v_scale[(size_t)hh * T * ngv + i] = half_to_float((uint16_t)(vt[i] & 0xFFFFu));
          if (x->v_zero) x->v_zero[(size_t)hh * T * ngv + i] = (int32_t)half_to_float((uint16_t)(vt[i] >> 16)) - 1024;
        }
      }
    }
  } else {
  for (int hh = 0; hh < H && ok; ++hh) {
    if (x->k_scale) ok &= d2h(x->k_scale + (int64_t)hh * G * kHeadDim, half + g.lay.k_scale + (int64_t)hh * g.g_cap * kHeadDim * 4, (size_t)G * kHeadDim * 4);
    if (x->k_zero) ok &= d2h(x->k_zero + (int64_t)hh * G * kHeadDim, half + g.lay.k_zero + (int64_t)hh * g.g_cap * kHeadDim * 4, (size_t)G * kHeadDim * 4);
  }
  if (x->v_scale || x->v_zero) {
    std::vector<VMeta> tmp((size_t)T * ngv);
    for (int hh = 0; hh < H && ok; ++hh) {
      ok &= d2h(tmp.data(), half + g.lay.v_meta + (int64_t)hh * g.t_cap * ngv * sizeof(VMeta), tmp.size() * sizeof(VMeta));
      for (size_t i = 0; i < tmp.size(); ++i) {
        if (x->v_scale) x->v_scale[(size_t)hh * T * ngv + i] = tmp[i].s;
        if (x->v_zero) x->v_zero[(size_t)hh * T * ngv + i] = tmp[i].z;
      }
    }
  }
  }
  if (cs.last_pruned) {
    if (x->last_keep) ok &= d2h(x->last_keep, sc + g.sl.keep, (size_t)g.budget * 4);
    if (x->last_scores) ok &= d2h(x->last_scores, sc + g.sl.scores, (size_t)cs.last_scores_len * 4);
  }
  if (!ok) return fail(h, KV_E_HIP, "kv_export: copy failed: %s", hipGetErrorString(hipGetLastError()));
  return KV_OK;
}

int kv_import(kv_handle* h, int32_t stream, int32_t layer, const kv_export_t* x) {
  if (!h) return KV_E_INVAL;
  if (!x) return fail(h, KV_E_INVAL, "kv_import: bufs is NULL");
  const kv_config& c = h->cfg;
  if (stream < 0 || stream >= c.n_streams || layer < 0 || layer >= c.n_layers) return fail(h, KV_E_RANGE, "kv_import: stream/layer out of range");
  const Geometry& g = h->geo;
  if (g.uncompressed) return fail(h, KV_E_STATE, "kv_import: not available in KV_UNCOMPRESSED_BF16 mode");
  if (!x->ids || !x->k_codes || !x->k_scale || !x->k_zero || !x->v_codes || !x->v_scale || !x->v_zero)
    return fail(h, KV_E_INVAL, "kv_import: ids, codes, scales and zero-points must all be given");
  const int T = x->cache_len;
  if (x->frames_seen < 0 || T < 0 || T > g.budget) return fail(h, KV_E_RANGE, "kv_import: cache_len %d / frames_seen %d out of range", T, x->frames_seen);
  const int64_t n_stream = h->stream_n[(size_t)stream];
  if ((int64_t)T != std::min<int64_t>((int64_t)x->frames_seen * n_stream, g.budget))
    return fail(h, KV_E_INVAL, "kv_import: cache_len %d is not min(frames_seen * tokens_per_frame, budget_tokens)", T);
  const int H = g.H;
  const int G = (T + g.k_group - 1) / g.k_group;
  const int ngv = kHeadDim / g.v_group;
  // pack the codes into rows of d * bits / 8 bytes, as the kernels store them
  auto pack = [&](const uint8_t* src, int bits, std::vector<uint8_t>& dst) -> bool {
    const int row = kHeadDim * bits / 8;
    dst.assign((size_t)H * T * row, 0);
    for (int64_t r = 0; r < (int64_t)H * T; ++r)
      for (int ch = 0; ch < kHeadDim; ++ch) {
        const uint8_t code = src[r * kHeadDim + ch];
        if (code >> bits) return false;
        const int bit = ch * bits;
        dst[(size_t)r * row + (bit >> 3)] |= (uint8_t)(code << (bit & 7));
      }
    return true;
  };
  std::vector<uint8_t> kc, vc;
  if (!pack(x->k_codes, g.k_bits, kc)) return fail(h, KV_E_INVAL, "kv_import: a key code does not fit %d bits", g.k_bits);
  if (!pack(x->v_codes, g.v_bits, vc)) return fail(h, KV_E_INVAL, "kv_import: a value code does not fit %d bits", g.v_bits);
  std::vector<VMeta> vm;
  std::vector<uint16_t> ka, kz;       // 16-bit metadata format: halfs in device order
  std::vector<uint32_t> vm16;
  if (g.meta16) {
    // the stored half scale is recovered from the fp32 scale the export gave: a = s * scale_log2 to the nearest
    // 7-bit value, accepted only if it reproduces s exactly
    ka.assign((size_t)H * G * kHeadDim, 0);
    kz.assign((size_t)H * G * kHeadDim, 0);
    for (int hh = 0; hh < H; ++hh)
      for (int gi = 0; gi < G; ++gi)
        for (int ch = 0; ch < kHeadDim; ++ch) {
          const size_t src = ((size_t)hh * G + gi) * kHeadDim + ch, dst = ((size_t)hh * G + gi) * kHeadDim + meta16_pos(ch);
          const float sv = x->k_scale[src];
          float a = sv * g.scale_log2;
          uint32_t u;
          memcpy(&u, &a, 4);
          u = (u + 0x10000u) & 0xFFFE0000u;               // nearest value with 7 significant bits
          memcpy(&a, &u, 4);
          const int32_t z = x->k_zero[src];
          if (!(a >= kMeta16ScaleMin && a <= kMeta16ScaleMax) || a * g.inv_scale_log2 != sv || !float_to_half_exact(a, &ka[dst]) ||
              z < kMeta16ZMin || z > kMeta16ZMax || !float_to_half_exact((float)(1024 + z), &kz[dst]))
            return fail(h, KV_E_INVAL, "kv_import: key scale or zero-point (head %d, group %d, channel %d) is not a value of the 16-bit metadata format", hh, gi, ch);
        }
    vm16.assign((size_t)H * T * ngv, 0);
    for (size_t i = 0; i < vm16.size(); ++i) {
      uint16_t hs, hz;
      const int32_t z = x->v_zero[i];
      if (!(x->v_scale[i] >= kMeta16ScaleMin && x->v_scale[i] <= kMeta16ScaleMax) || !float_to_half_exact(x->v_scale[i], &hs) ||
          z < kMeta16ZMin || z > kMeta16ZMax || !float_to_half_exact((float)(1024 + z), &hz))
        return fail(h, KV_E_INVAL, "kv_import: value scale or zero-point %lld is not a value of the 16-bit metadata format", (long long)i);
      vm16[i] = (uint32_t)hs | ((uint32_t)hz << 16);
    }
  } else {
    vm.assign((size_t)H * T * ngv, VMeta());
    for (size_t i = 0; i < vm.size(); ++i) {
      vm[i].s = x->v_scale[i];
      vm[i].z = x->v_zero[i];
    }
  }
  if (hipDeviceSynchronize() != hipSuccess) return fail(h, KV_E_HIP, "kv_import: %s", hipGetErrorString(hipGetLastError()));
  const size_t ci = (size_t)stream * c.n_layers + layer;
  uint8_t* half = h->arena + (int64_t)ci * g.lay.cache_bytes;        // the cache restarts in its first half
  auto h2d = [&](void* dst, const void* src, size_t bytes) { return bytes == 0 || hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice) == hipSuccess; };
  bool ok = h2d(half + g.lay.ids, x->ids, (size_t)T * 4);
  const int krow = kHeadDim * g.k_bits / 8, vrow = kHeadDim * g.v_bits / 8;
  for (int hh = 0; hh < H && ok; ++hh) {
    ok &= h2d(half + g.lay.k_codes + (int64_t)hh * g.t_cap * krow, kc.data() + (size_t)hh * T * krow, (size_t)T * krow);
    ok &= h2d(half + g.lay.v_codes + (int64_t)hh * g.t_cap * vrow, vc.data() + (size_t)hh * T * vrow, (size_t)T * vrow);
    if (g.meta16) {
      ok &= h2d(half + g.lay.k_scale + (int64_t)hh * g.g_cap * kHeadDim * 2, ka.data() + (size_t)hh * G * kHeadDim, (size_t)G * kHeadDim * 2);
      ok &= h2d(half + g.lay.k_zero + (int64_t)hh * g.g_cap * kHeadDim * 2, kz.data() + (size_t)hh * G * kHeadDim, (size_t)G * kHeadDim * 2);
      ok &= h2d(half + g.lay.v_meta + (int64_t)hh * g.t_cap * ngv * 4, vm16.data() + (size_t)hh * T * ngv, (size_t)T * ngv * 4);
    } else {
      ok &= h2d(half + g.lay.k_scale + (int64_t)hh * g.g_cap * kHeadDim * 4, x->k_scale + (int64_t)hh * G * kHeadDim, (size_t)G * kHeadDim * 4);
      ok &= h2d(half + g.lay.k_zero + (int64_t)hh * g.g_cap * kHeadDim * 4, x->k_zero + (int64_t)hh * G * kHeadDim, (size_t)G * kHeadDim * 4);
      ok &= h2d(half + g.lay.v_meta + (int64_t)hh * g.t_cap * ngv * sizeof(VMeta), vm.data() + (size_t)hh * T * ngv, (size_t)T * ngv * sizeof(VMeta));
    }
  }
  if (!ok) {
    h->caches[ci] = CacheState();       // partly written: the cache is empty rather than inconsistent
    return fail(h, KV_E_HIP, "kv_import: copy failed: %s", hipGetErrorString(hipGetLastError()));
  }
  CacheState cs;
  cs.t_c = T;
  cs.cur = 0;
  cs.frames = x->frames_seen;
  cs.dropped = (int64_t)x->frames_seen * n_stream - T;
  h->caches[ci] = cs;
  return KV_OK;
}

int kv_reset(kv_handle* h, int32_t stream, int32_t layer) {
  if (!h) return KV_E_INVAL;
  const kv_config& c = h->cfg;
  if (stream == -1 && layer == -1) {
    for (auto& cs : h->caches) cs = CacheState();
    return KV_OK;
  }
  if (stream < 0 || stream >= c.n_streams || layer < 0 || layer >= c.n_layers) return fail(h, KV_E_RANGE, "kv_reset: stream/layer out of range");
  h->caches[(size_t)stream * c.n_layers + layer] = CacheState();
  return KV_OK;
}

int kv_set_stream_tokens(kv_handle* h, int32_t stream, int32_t tokens_per_frame) {
  if (!h) return KV_E_INVAL;
  const kv_config& c = h->cfg;
  if (stream < 0 || stream >= c.n_streams) return fail(h, KV_E_RANGE, "kv_set_stream_tokens: stream out of range");
  if (tokens_per_frame < 1 || tokens_per_frame > c.tokens_per_frame || tokens_per_frame < c.n_special)
    return fail(h, KV_E_RANGE, "kv_set_stream_tokens: tokens_per_frame must be in [max(1, n_special), %d]", c.tokens_per_frame);
  for (int l = 0; l < c.n_layers; ++l)
    if (h->caches[(size_t)stream * c.n_layers + l].frames != 0)
      return fail(h, KV_E_STATE, "kv_set_stream_tokens: stream %d has frames in its caches; kv_reset it first", stream);
  h->stream_n[(size_t)stream] = tokens_per_frame;
  return KV_OK;
}

void kv_destroy(kv_handle* h) {
  if (!h) return;
  for (auto& t : h->timed) { hipEventDestroy(t.start); hipEventDestroy(t.stop); }
  for (auto& t : h->free_events) { hipEventDestroy(t.start); hipEventDestroy(t.stop); }
  if (h->side) { hipStreamSynchronize(h->side); hipStreamDestroy(h->side); }
  if (h->ev_fork) hipEventDestroy(h->ev_fork);
  if (h->ev_join) hipEventDestroy(h->ev_join);
  if (h->arena) hipFree(h->arena);
  if (h->work) hipFree(h->work);
  if (h->part_o) hipFree(h->part_o);
  if (h->part_ml) hipFree(h->part_ml);
  delete h;
}

const char* kv_last_error(kv_handle* h) { return h ? h->err.c_str() : g_init_error.c_str(); }

int kv_set_timing(kv_handle* h, uint32_t kernel_mask) {
  if (!h) return KV_E_INVAL;
  h->timing_mask = kernel_mask;
  return KV_OK;
}

int kv_read_timing(kv_handle* h, float* total_ms, int32_t* launches) {
  if (!h) return KV_E_INVAL;
  if (!total_ms || !launches) return fail(h, KV_E_INVAL, "kv_read_timing: NULL output");
  for (int i = 0; i < KV_K_COUNT; ++i) { total_ms[i] = 0.f; launches[i] = 0; }
  for (auto& t : h->timed) {
    float ms = 0.f;
    if (hipEventSynchronize(t.stop) == hipSuccess && hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) {
      total_ms[t.kernel] += ms;
      launches[t.kernel] += 1;
    } else {
      (void)hipGetLastError();
    }
    h->free_events.push_back(t);
  }
  h->timed.clear();
  return KV_OK;
}

int kv_set_option(kv_handle* h, const char* name, int64_t value) {
  if (!h) return KV_E_INVAL;
  if (!name) return fail(h, KV_E_INVAL, "kv_set_option: name is NULL");
  if (!strcmp(name, "attention_splits")) {
    if (value < 0 || value > kMaxSplits) return fail(h, KV_E_RANGE, "kv_set_option: attention_splits must be in [0, %d]", (int)kMaxSplits);
    h->splits_override = (int32_t)value;
    return KV_OK;
  }
  if (!strcmp(name, "timing_every")) {
    if (value < 1 || value > (1 << 20)) return fail(h, KV_E_RANGE, "kv_set_option: timing_every must be in [1, 2^20]");
    h->timing_every = (int32_t)value;
    return KV_OK;
  }
  if (!strcmp(name, "debug_checks")) {
    h->debug_checks = value != 0;
    return KV_OK;
  }
  if (!strcmp(name, "overlap_update")) {
    if (value < 0 || value > 2) return fail(h, KV_E_RANGE, "kv_set_option: overlap_update takes 0..2");
    h->overlap = (int32_t)value;
    h->target_wgs = h->overlap ? std::max(1, h->n_cus * 3 / 4) : h->n_cus;
    return KV_OK;
  }
  if (!strcmp(name, "attention_target_workgroups")) {
    if (value < 1 || value > 65536) return fail(h, KV_E_RANGE, "kv_set_option: attention_target_workgroups out of range");
    h->target_wgs = (int32_t)value;
    h->target_explicit = true;
    return KV_OK;
  }
  return fail(h, KV_E_INVAL, "kv_set_option: unknown option '%s'", name);
}

}  // extern "C"
