// Token-importance scoring (paper Sec. 3.2, Eq. 2-6).
//
// Eq. 5-6 average the rows of Qbar Kbar^T, which by linearity equals q~ . Kbar_j with
// q~ the mean of the pooled, head-averaged query rows.  Every value here feeds top-k,
// so each kernel evaluates in fp32 with one rounding per operation and the fixed order
// of additions stated at the kernel (compiled without FMA contraction).
#include "kvx_dev.h"

namespace kvx {

// Eq. 2-3: one block per pooled row, one thread per (head, channel).  Per (head, channel):
// add the row's tokens in ascending order starting from the first, divide by the group
// size; then per channel add heads 0..H-1 in order starting from zero, divide by H.
__global__ __launch_bounds__(1024) void pool_rows_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.y];
  if (!it.prune) return;
  const int row = blockIdx.x;
  int a, e;
  if (row < g.n_special) {
    a = row;
    e = row + 1;
  } else {
    a = g.n_special + (row - g.n_special) * g.pool_group;
    e = min(a + g.pool_group, g.n);
  }
  __shared__ float pooled[64][kHeadDim];     // up to 64 heads
  const int c = threadIdx.x & 63;
  for (int h = threadIdx.x >> 6; h < g.H; h += 16) {
    float acc;
    if (g.in_f32) {
      const float* q = reinterpret_cast<const float*>(it.q);
      acc = q[(int64_t)a * g.tok_stride + (int64_t)h * g.head_stride + c];
#pragma unroll 8
      for (int t = a + 1; t < e; ++t) acc = acc + q[(int64_t)t * g.tok_stride + (int64_t)h * g.head_stride + c];
    } else {
      const uint16_t* q = reinterpret_cast<const uint16_t*>(it.q);
      acc = __uint_as_float((uint32_t)q[(int64_t)a * g.tok_stride + (int64_t)h * g.head_stride + c] << 16);
#pragma unroll 8
      for (int t = a + 1; t < e; ++t)
        acc = acc + __uint_as_float((uint32_t)q[(int64_t)t * g.tok_stride + (int64_t)h * g.head_stride + c] << 16);
    }
    pooled[h][c] = acc / (float)(e - a);
  }
  __syncthreads();
  if (threadIdx.x < 64) {
    float acc = 0.f;
    for (int h = 0; h < g.H; ++h) acc = acc + pooled[h][c];
    reinterpret_cast<float*>(cache_scratch(g, it.cache) + g.sl.qbar)[row * kHeadDim + c] = acc / (float)g.H;
  }
}

// The row mean of Eq. 6 pulled inside the product: q~ = (pooled rows added in ascending
// order from zero) / N_pooled, one thread per channel.  A kernel of its own, so that the
// pooled rows reach it through the kernel boundary and no block has to fence.
__global__ __launch_bounds__(64) void pool_mean_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.x];
  if (!it.prune) return;
  uint8_t* sc = cache_scratch(g, it.cache);
  const float* qbar = reinterpret_cast<const float*>(sc + g.sl.qbar);
  const int c = threadIdx.x;
  float acc = 0.f;
#pragma unroll 16
  for (int i = 0; i < g.n_pooled; ++i) acc = acc + qbar[i * kHeadDim + c];
  reinterpret_cast<float*>(sc + g.sl.qt)[c] = acc / (float)g.n_pooled;
}

template <int B>
__device__ __forceinline__ int row_code(const uint32_t* w, int c) {
  if constexpr (B == 4) return (int)((w[c >> 3] >> (4 * (c & 7))) & 0xFu);
  if constexpr (B == 2) return (int)((w[c >> 4] >> (2 * (c & 15))) & 0x3u);
  return (int)((w[c >> 2] >> (8 * (c & 3))) & 0xFFu);
}

// Per head and cached token: D[h, j] = q~ . K~[h, j, :] with K~ = s * (code - z) (Eq. 10),
// p[c] = q~[c] * K~[c], then the stride-halving pairwise tree p[c] += p[c + m] for
// m = 32, 16, ..., 1.  One thread holds one token's 64 channels; a block covers 256
// consecutive cache positions of one head and stages their groups' (s, z) and q~ in LDS.
template <int B>
__global__ __launch_bounds__(256) void score_dots_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.z];
  if (!it.prune) return;
  const int h = blockIdx.y;
  const int j0 = blockIdx.x * 256;
  if (j0 >= it.t_c) return;
  const uint8_t* half = cache_half(g, it.cache, it.cur);
  constexpr int kRowWords = 2 * B;                 // 64 channels * B bits / 32
  __shared__ __attribute__((aligned(16))) float s_s[8][kHeadDim];
  __shared__ __attribute__((aligned(16))) int32_t s_z[8][kHeadDim];
  __shared__ __attribute__((aligned(16))) float s_q[kHeadDim];

  const int k_shift = g.k_group == 64 ? 6 : 5;      // groups of 64 or 32 tokens
  const int groups_in_block = 256 >> k_shift;      // 4 or 8
  const int grp0 = j0 >> k_shift;
  for (int i = threadIdx.x; i < groups_in_block * kHeadDim; i += 256) {
    const int gi = i >> 6, c = i & 63;
    const int grp = grp0 + gi;
    if (grp < g.g_cap) {
      const int64_t moff = ((int64_t)h * g.g_cap + grp) * kHeadDim + c;
      s_s[gi][c] = reinterpret_cast<const float*>(half + g.lay.k_scale)[moff];
      s_z[gi][c] = reinterpret_cast<const int32_t*>(half + g.lay.k_zero)[moff];
    }
  }
  if (threadIdx.x < 64) s_q[threadIdx.x] = reinterpret_cast<const float*>(cache_scratch(g, it.cache) + g.sl.qt)[threadIdx.x];
  __syncthreads();

  const int j = j0 + threadIdx.x;
  if (j >= it.t_c) return;
  uint32_t w[kRowWords];
  const uint32_t* src = reinterpret_cast<const uint32_t*>(half + g.lay.k_codes + ((int64_t)h * g.t_cap + j) * (8 * B));
#pragma unroll
  for (int i = 0; i < kRowWords; ++i) w[i] = src[i];
  const int gi = (j - j0) >> k_shift;
  float p[kHeadDim];
#pragma unroll
  for (int c = 0; c < kHeadDim; ++c) {
    const float kd = s_s[gi][c] * (float)(row_code<B>(w, c) - s_z[gi][c]);
    p[c] = s_q[c] * kd;
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
#pragma unroll
    for (int c = 0; c < m; ++c) p[c] = p[c] + p[c + m];
  }
  reinterpret_cast<float*>(cache_scratch(g, it.cache) + g.sl.dots)[(int64_t)h * g.t_cap + j] = p[0];
}

void launch_pool(const KvxBatch& b, hipStream_t st) {
  hipLaunchKernelGGL(pool_rows_kernel, dim3(b.g.n_pooled, b.n_items), dim3(1024), 0, st, b);
  hipLaunchKernelGGL(pool_mean_kernel, dim3(b.n_items), dim3(64), 0, st, b);
}

void launch_score(const KvxBatch& b, int max_tc, hipStream_t st) {
  dim3 grid((max_tc + 255) / 256, b.g.H, b.n_items);
  switch (b.g.k_bits) {
    case 2: hipLaunchKernelGGL(score_dots_kernel<2>, grid, dim3(256), 0, st, b); break;
    case 4: hipLaunchKernelGGL(score_dots_kernel<4>, grid, dim3(256), 0, st, b); break;
    default: hipLaunchKernelGGL(score_dots_kernel<8>, grid, dim3(256), 0, st, b); break;
  }
}

}  // namespace kvx
