// Token-importance scoring (paper Sec. 3.2, Eq. 2-6).
//
// Eq. 5-6 average the rows of Qbar Kbar^T, which by linearity equals q~ . Kbar_j with
// q~ the mean of the pooled, head-averaged query rows.  Every value here feeds top-k,
// so each kernel evaluates in fp32 with one rounding per operation and the fixed order
// of additions stated at the kernel (compiled without FMA contraction).
#include "kvx_dev.h"

#include <algorithm>

namespace kvx {

// Eq. 2-3: one block per pooled row, eight lanes per head, eight channels per lane.  Per
// (head, channel): add the row's tokens in ascending order starting from the first, divide
// by the group size; then per channel add heads 0..H-1 in order starting from zero, divide
// by H.  A group's tokens are requested sixteen at a time before any is added, so a row
// costs one memory round trip.
constexpr int kPoolBatch = 16;
__global__ __launch_bounds__(512) void pool_rows_kernel(const KvxBatch b) {
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
  __shared__ __attribute__((aligned(16))) float pooled[64][kHeadDim];     // up to 64 heads
  const int h = threadIdx.x >> 3, c0 = (threadIdx.x & 7) * 8;
  if (h < g.H) {
    float acc[8];
    for (int t0 = a; t0 < e; t0 += kPoolBatch) {
      float v[kPoolBatch][8];
#pragma unroll
      for (int k = 0; k < kPoolBatch; ++k) {
        const int t = min(t0 + k, e - 1);                  // clamped: a repeated token is loaded but not added
        const int64_t off = (int64_t)t * g.tok_stride + (int64_t)h * g.head_stride + c0;
        if (g.in_f32) {
          const float4* q = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(it.q) + off);
          const float4 x0 = q[0], x1 = q[1];
          v[k][0] = x0.x; v[k][1] = x0.y; v[k][2] = x0.z; v[k][3] = x0.w;
          v[k][4] = x1.x; v[k][5] = x1.y; v[k][6] = x1.z; v[k][7] = x1.w;
        } else {
          const uint4 x = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(it.q) + off);
          const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            v[k][2 * j] = __uint_as_float(w[j] << 16);
            v[k][2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
          }
        }
      }
#pragma unroll
      for (int k = 0; k < kPoolBatch; ++k) {
        if (t0 + k < e) {
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[j] = (t0 + k == a) ? v[k][j] : acc[j] + v[k][j];
        }
      }
    }
    const float cnt = (float)(e - a);
#pragma unroll
    for (int j = 0; j < 8; ++j) pooled[h][c0 + j] = acc[j] / cnt;
  }
  __syncthreads();
  if (threadIdx.x < 64) {
    const int c = threadIdx.x;
    float acc = 0.f;
    for (int hh = 0; hh < g.H; ++hh) acc = acc + pooled[hh][c];
    reinterpret_cast<float*>(cache_scratch(g, it.cache) + g.sl.qbar)[row * kHeadDim + c] = acc / (float)g.H;
  }
}

// The row mean of Eq. 6 pulled inside the product: q~ = (pooled rows added in ascending
// order from zero) / N_pooled.  A kernel of its own, so that the pooled rows reach it
// through the kernel boundary and no block has to fence.  The rows are brought into LDS
// 128 at a time by the whole block (one memory round trip per 128 rows), then one thread
// per channel adds them in order.
constexpr int kMeanRows = 128;
__global__ __launch_bounds__(1024) void pool_mean_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.x];
  if (!it.prune) return;
  uint8_t* sc = cache_scratch(g, it.cache);
  const float4* qbar = reinterpret_cast<const float4*>(sc + g.sl.qbar);
  __shared__ __attribute__((aligned(16))) float rows[kMeanRows][kHeadDim];
  const int tid = threadIdx.x;
  float acc = 0.f;
  for (int r0 = 0; r0 < g.n_pooled; r0 += kMeanRows) {
    const int cnt = min(kMeanRows, g.n_pooled - r0);
    // 16 float4 per row: threads 0..1023 cover 64 rows per step
#pragma unroll
    for (int k = 0; k < kMeanRows / 64; ++k) {
      const int r = k * 64 + (tid >> 4);
      if (r < cnt) *reinterpret_cast<float4*>(&rows[r][(tid & 15) * 4]) = qbar[(int64_t)(r0 + r) * 16 + (tid & 15)];
    }
    __syncthreads();
    if (tid < kHeadDim) {
      for (int r = 0; r < cnt; ++r) acc = acc + rows[r][tid];
    }
    __syncthreads();
  }
  if (tid < kHeadDim) reinterpret_cast<float*>(sc + g.sl.qt)[tid] = acc / (float)g.n_pooled;
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
      if (g.meta16) {
        // halfs: logit-domain scale a (s = a * fp32(1 / scale_log2)) and 1024 + z, channels of an octet in the order 0 4 1 5 2 6 3 7
        const int64_t moff = ((int64_t)h * g.g_cap + grp) * kHeadDim + meta16_pos(c);
        s_s[gi][c] = (float)__builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t*>(half + g.lay.k_scale)[moff]) * g.inv_scale_log2;
        s_z[gi][c] = (int32_t)(float)__builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t*>(half + g.lay.k_zero)[moff]) - 1024;
      } else {
        const int64_t moff = ((int64_t)h * g.g_cap + grp) * kHeadDim + c;
        s_s[gi][c] = reinterpret_cast<const float*>(half + g.lay.k_scale)[moff];
        s_z[gi][c] = reinterpret_cast<const int32_t*>(half + g.lay.k_zero)[moff];
      }
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
  hipLaunchKernelGGL(pool_rows_kernel, dim3(b.g.n_pooled, b.n_items), dim3(std::max(64, 8 * b.g.H)), 0, st, b);
  hipLaunchKernelGGL(pool_mean_kernel, dim3(b.n_items), dim3(1024), 0, st, b);
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
