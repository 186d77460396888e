// Debug check of a step's inputs (switched on with kv_set_option "debug_checks"): one pass
// over q, k and v of every item that raises a flag in the cache's scratch when it meets an
// infinity or a NaN.  The step itself runs unchanged; kv_stats reports the flag.
#include "kvx_dev.h"

namespace kvx {

__global__ __launch_bounds__(256) void check_finite_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.z];
  const void* src = blockIdx.y == 0 ? it.q : (blockIdx.y == 1 ? it.k : it.v);
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;      // 8 channels of one (token, head) row
  const int64_t row = idx >> 3;
  if (row >= (int64_t)g.n_new * g.H) return;
  const int tok = (int)(row / g.H), h = (int)(row % g.H), c0 = (int)(idx & 7) * 8;
  const int64_t off = (int64_t)tok * g.tok_stride + (int64_t)h * g.head_stride + c0;
  bool bad = false;
  if (g.in_f32) {
    const uint4* p = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(src) + off);
    const uint4 a = p[0], c = p[1];
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, c.x, c.y, c.z, c.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) bad |= (w[e] & 0x7F800000u) == 0x7F800000u;       // exponent all ones
  } else {
    const uint4 a = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(src) + off);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) bad |= (w[e] & 0x7F80u) == 0x7F80u || (w[e] & 0x7F800000u) == 0x7F800000u;
  }
  if (bad) atomicOr(reinterpret_cast<int32_t*>(cache_scratch(g, it.cache) + g.sl.sel) + 6, 1);
}

void launch_check_finite(const KvxBatch& b, hipStream_t st) {
  const int64_t lanes = (int64_t)b.g.n_new * b.g.H * 8;
  hipLaunchKernelGGL(check_finite_kernel, dim3((unsigned)((lanes + 255) / 256), 3, b.n_items), dim3(256), 0, st, b);
}

}  // namespace kvx
