// Driver of the sanitizer build: walks the host code of the library (no kernel runs; see hip/hip_runtime.h here).
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../include/kvx.h"

#define CHECK(cond)                                                                   \
  do {                                                                                \
    if (!(cond)) {                                                                    \
      std::fprintf(stderr, "host_check: line %d: %s failed\n", __LINE__, #cond);      \
      std::exit(1);                                                                   \
    }                                                                                 \
  } while (0)

namespace {

struct Bufs {
  std::vector<int32_t> ids, kz, vz, keep;
  std::vector<uint8_t> kc, vc;
  std::vector<float> ks, vs, scores;
  kv_export_t x;
  Bufs(int H, int cap, int kg, int vg) {
    const int G = (cap + kg - 1) / kg, ngv = 64 / vg;
    ids.assign(cap, -1); kc.assign((size_t)H * cap * 64, 0xEE); vc.assign((size_t)H * cap * 64, 0xEE);
    ks.assign((size_t)H * G * 64, -1.f); kz.assign((size_t)H * G * 64, -1);
    vs.assign((size_t)H * cap * ngv, -1.f); vz.assign((size_t)H * cap * ngv, -1);
    keep.assign(cap, -1); scores.assign(cap, -1.f);
    std::memset(&x, 0, sizeof x);
    x.ids = ids.data(); x.k_codes = kc.data(); x.k_scale = ks.data(); x.k_zero = kz.data();
    x.v_codes = vc.data(); x.v_scale = vs.data(); x.v_zero = vz.data();
    x.last_keep = keep.data(); x.last_scores = scores.data(); x.capacity_tokens = cap;
  }
};

kv_config base_config(int meta, int layout, int kb, int kg, int vb, int vg) {
  kv_config c;
  std::memset(&c, 0, sizeof c);
  c.n_streams = 2; c.n_layers = 2; c.n_heads = 3; c.head_dim = 64;
  c.tokens_per_frame = 37; c.n_special = 5; c.pool_group = 16; c.budget_tokens = 160;
  c.k_bits = kb; c.k_group = kg; c.v_bits = vb; c.v_group = vg;
  c.in_dtype = KV_BF16; c.out_dtype = KV_BF16; c.mode = KV_COMPRESSED; c.max_frames = 0;
  c.softmax_scale = 0.f; c.meta_format = meta; c.max_frames_per_step = 2; c.order = KV_ATTEND_THEN_PRUNE; c.layout = layout;
  return c;
}

// A cache state that is a value of the format: codes below 2^bits, metadata representable.
void fill_state(Bufs& b, const kv_config& c, int frames, std::mt19937& rng) {
  const int T = std::min(frames * c.tokens_per_frame, c.budget_tokens), H = c.n_heads;
  const int G = (T + c.k_group - 1) / c.k_group, ngv = 64 / c.v_group;
  b.x.cache_len = T; b.x.frames_seen = frames;
  for (int i = 0; i < T; ++i) b.ids[i] = i;
  for (size_t i = 0; i < (size_t)H * T * 64; ++i) { b.kc[i] = rng() % (1u << c.k_bits); b.vc[i] = rng() % (1u << c.v_bits); }
  const float c_log2 = 0.125f * 1.4426950408889634f, inv = 1.0f / c_log2;
  for (size_t i = 0; i < (size_t)H * G * 64; ++i) {
    if (c.meta_format == KV_META_F16) {
      const float a = std::ldexp((float)(64 + rng() % 64) / 128.f, (int)(rng() % 12) - 8);      // 7 significant bits
      b.ks[i] = a * inv;
      b.kz[i] = (int)(rng() % 2048) - 1024;
    } else {
      b.ks[i] = std::ldexp(1.0f + (float)(rng() % 4096) / 4096.f, (int)(rng() % 20) - 10);
      b.kz[i] = (int)(rng() % 200001) - 100000;
    }
  }
  for (size_t i = 0; i < (size_t)H * T * ngv; ++i) {
    if (c.meta_format == KV_META_F16) {
      b.vs[i] = std::ldexp((float)(1024 + rng() % 1024) / 2048.f, (int)(rng() % 12) - 8);       // 11 significant bits
      b.vz[i] = (int)(rng() % 2048) - 1024;
    } else {
      b.vs[i] = std::ldexp(1.0f + (float)(rng() % 4096) / 4096.f, (int)(rng() % 20) - 10);
      b.vz[i] = (int)(rng() % 200001) - 100000;
    }
  }
}

void same_state(const Bufs& a, const Bufs& b, const kv_config& c) {
  const int T = a.x.cache_len, H = c.n_heads, G = (T + c.k_group - 1) / c.k_group, ngv = 64 / c.v_group;
  CHECK(a.x.cache_len == b.x.cache_len && a.x.frames_seen == b.x.frames_seen);
  CHECK(!std::memcmp(a.ids.data(), b.ids.data(), (size_t)T * 4));
  CHECK(!std::memcmp(a.kc.data(), b.kc.data(), (size_t)H * T * 64));
  CHECK(!std::memcmp(a.vc.data(), b.vc.data(), (size_t)H * T * 64));
  CHECK(!std::memcmp(a.ks.data(), b.ks.data(), (size_t)H * G * 64 * 4));
  CHECK(!std::memcmp(a.kz.data(), b.kz.data(), (size_t)H * G * 64 * 4));
  CHECK(!std::memcmp(a.vs.data(), b.vs.data(), (size_t)H * T * ngv * 4));
  CHECK(!std::memcmp(a.vz.data(), b.vz.data(), (size_t)H * T * ngv * 4));
}

void one_format(int meta, int layout, int kb, int kg, int vb, int vg) {
  std::mt19937 rng(17 + meta * 2 + layout + kb * 10 + vg);
  const kv_config c = base_config(meta, layout, kb, kg, vb, vg);
  kv_handle *h = nullptr, *h2 = nullptr;
  CHECK(kv_init(&c, &h) == KV_OK && h);
  CHECK(kv_init(&c, &h2) == KV_OK && h2);
  const int n = c.tokens_per_frame, H = c.n_heads;
  // frame buffers stand in for device memory (nothing reads them here), two frames' worth for the chunk call
  std::vector<uint16_t> q((size_t)2 * n * H * 64), k(q.size()), v(q.size()), o(q.size());
  const int64_t ts = (int64_t)H * 64, hs = 64;

  // bookkeeping over a stream that crosses the budget: lengths, drops, flat allocation
  kv_stats_t st0, st;
  CHECK(kv_stats(h, &st0) == KV_OK);
  for (int f = 0; f < 7; ++f) {
    CHECK(kv_step(h, 0, 0, q.data(), k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_OK);
    CHECK(kv_stats(h, &st) == KV_OK);
    CHECK(st.cache_len_max == std::min((f + 1) * n, c.budget_tokens));
    CHECK(st.bytes_allocated == st0.bytes_allocated);
  }
  CHECK(st.tokens_dropped_total == 7 * n - c.budget_tokens);
  CHECK(kv_step_frames(h, 0, 1, 2, q.data(), k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_OK);
  CHECK(kv_step_frames(h, 0, 1, 3, q.data(), k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_E_RANGE);
  CHECK(kv_step_static(h, 1, 0, q.data(), k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_OK);
  {
    kv_step_item items[4];
    for (int i = 0; i < 4; ++i) { items[i].stream = i / 2; items[i].layer = i % 2; items[i].q = q.data(); items[i].k = k.data(); items[i].v = v.data(); items[i].out = o.data(); }
    CHECK(kv_set_timing(h, 0x7F) == KV_OK);
    CHECK(kv_step_batched(h, 4, items, ts, hs, nullptr) == KV_OK);
    float ms[16]; int32_t cnt[16];
    CHECK(kv_read_timing(h, ms, cnt) == KV_OK);
    CHECK(kv_set_timing(h, 0) == KV_OK);
    items[3] = items[0];
    CHECK(kv_step_batched(h, 4, items, ts, hs, nullptr) == KV_E_INVAL);      // one cache twice
    items[3].layer = 9;
    CHECK(kv_step_batched(h, 4, items, ts, hs, nullptr) == KV_E_RANGE);
  }
  // error paths leave the handle usable
  CHECK(kv_step(h, 0, 0, nullptr, k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_E_INVAL);
  CHECK(kv_step(h, 0, 0, (const char*)q.data() + 2, k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_E_INVAL);
  CHECK(kv_step(h, 0, 0, q.data(), k.data(), v.data(), 32, hs, o.data(), nullptr) == KV_E_INVAL);
  CHECK(kv_step(h, 2, 0, q.data(), k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_E_RANGE);
  CHECK(std::strlen(kv_last_error(h)) > 0);
  CHECK(kv_set_stream_tokens(h, 0, 21) == KV_E_STATE);                       // caches of stream 0 are not empty
  CHECK(kv_set_option(h, "no_such_option", 1) == KV_E_INVAL);
  CHECK(kv_set_option(h, "overlap_update", 0) == KV_OK && kv_set_option(h, "attention_splits", 3) == KV_OK);
  CHECK(kv_step(h, 0, 0, q.data(), k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_OK);

  // export of whatever the arena holds (no kernel wrote it: zeros) stays inside the caller's buffers
  Bufs e0(H, c.budget_tokens, c.k_group, c.v_group);
  CHECK(kv_export(h, 0, 0, &e0.x) == KV_OK);
  CHECK(e0.x.cache_len == c.budget_tokens);
  Bufs small(H, 64, c.k_group, c.v_group);
  CHECK(kv_export(h, 0, 0, &small.x) == KV_E_RANGE);                          // capacity below the cache length

  // import -> export -> import into a second handle -> export: the packing and its inverse, every part of the state
  for (int frames : {1, 3, 9}) {
    Bufs a(H, c.budget_tokens, c.k_group, c.v_group), b(H, c.budget_tokens, c.k_group, c.v_group), d(H, c.budget_tokens, c.k_group, c.v_group);
    fill_state(a, c, frames, rng);
    CHECK(kv_import(h, 1, 1, &a.x) == KV_OK);
    CHECK(kv_export(h, 1, 1, &b.x) == KV_OK);
    same_state(a, b, c);
    CHECK(kv_import(h2, 0, 1, &b.x) == KV_OK);
    CHECK(kv_export(h2, 0, 1, &d.x) == KV_OK);
    same_state(a, d, c);
    CHECK(kv_step(h2, 0, 1, q.data(), k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_OK);    // the stream goes on
    // inconsistent buffers are refused and leave the cache as it was
    a.kc[5] = (uint8_t)(1u << c.k_bits);
    if (c.k_bits < 8) CHECK(kv_import(h, 1, 1, &a.x) < 0);
    a.kc[5] = 0;
    a.x.cache_len -= 1;
    CHECK(kv_import(h, 1, 1, &a.x) < 0);
    a.x.cache_len += 1;
    if (c.meta_format == KV_META_F16) {
      a.kz[0] = 5000;
      CHECK(kv_import(h, 1, 1, &a.x) == KV_E_INVAL);
    }
    CHECK(kv_export(h, 1, 1, &d.x) == KV_OK);
    same_state(b, d, c);
  }
  CHECK(kv_reset(h, -1, -1) == KV_OK);
  CHECK(kv_set_stream_tokens(h, 0, 21) == KV_OK);
  CHECK(kv_set_stream_tokens(h, 0, 38) == KV_E_RANGE);
  CHECK(kv_step(h, 0, 0, q.data(), k.data(), v.data(), ts, hs, o.data(), nullptr) == KV_OK);
  CHECK(kv_stats(h, &st) == KV_OK && st.cache_len_max == 21);
  kv_destroy(h);
  kv_destroy(h2);
}

}  // namespace

int main() {
  for (int meta : {KV_META_F32, KV_META_F16})
    for (int layout : {KV_LAYOUT_COMPACT, KV_LAYOUT_SLOTS}) {
      one_format(meta, layout, 4, 64, 4, 64);
      one_format(meta, layout, 2, 32, 4, 32);
      if (meta == KV_META_F32) one_format(meta, layout, 8, 32, 8, 64);
    }
  // configurations that kv_init must refuse
  {
    kv_handle* h = nullptr;
    kv_config c = base_config(KV_META_F32, KV_LAYOUT_COMPACT, 4, 64, 4, 64);
    c.budget_tokens = 2 * c.tokens_per_frame - 1;
    CHECK(kv_init(&c, &h) < 0 && !h && std::strlen(kv_last_error(nullptr)) > 0);
    c = base_config(KV_META_F16, KV_LAYOUT_COMPACT, 8, 64, 4, 64);
    CHECK(kv_init(&c, &h) < 0 && !h);                                        // 8-bit codes have no 16-bit metadata format
    c = base_config(KV_META_F32, KV_LAYOUT_COMPACT, 3, 64, 4, 64);
    CHECK(kv_init(&c, &h) < 0 && !h);
    c = base_config(KV_META_F32, KV_LAYOUT_COMPACT, 4, 64, 4, 64);
    c.mode = KV_UNCOMPRESSED_BF16; c.max_frames = 4;
    CHECK(kv_init(&c, &h) == KV_OK && h);
    std::vector<uint16_t> q((size_t)c.tokens_per_frame * c.n_heads * 64), o(q.size());
    for (int f = 0; f < 4; ++f) CHECK(kv_step(h, 0, 0, q.data(), q.data(), q.data(), c.n_heads * 64, 64, o.data(), nullptr) == KV_OK);
    CHECK(kv_step(h, 0, 0, q.data(), q.data(), q.data(), c.n_heads * 64, 64, o.data(), nullptr) == KV_E_STATE);
    Bufs e(c.n_heads, 160, 64, 64);
    CHECK(kv_import(h, 0, 0, &e.x) == KV_E_STATE);
    kv_destroy(h);
    kv_destroy(nullptr);
  }
  std::printf("host checks passed\n");
  return 0;
}
