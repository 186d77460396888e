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
  // pooled row -> (frame of the call, row within the frame): every frame is pooled by itself
  const int row = blockIdx.x;
  const int fr = row / g.n_pooled, rr = row - fr * g.n_pooled;
  int a, e;
  if (rr < g.n_special) {
    a = fr * g.n + rr;
    e = a + 1;
  } else {
    a = fr * g.n + g.n_special + (rr - g.n_special) * g.pool_group;
    e = min(a + g.pool_group, (fr + 1) * g.n);
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
  const int n_rows = g.n_pooled * (g.n_new / g.n);          // the pooled rows of all the call's frames, in frame order
  for (int r0 = 0; r0 < n_rows; r0 += kMeanRows) {
    const int cnt = min(kMeanRows, n_rows - r0);
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
  if (tid < kHeadDim) reinterpret_cast<float*>(sc + g.sl.qt)[tid] = acc / (float)n_rows;
}

// One row's codes as floats, channel by channel, through byte conversions (v_cvt_f32_ubyteN): 4-bit codes are
// first spread into the bytes of two words per eight channels (even and odd channels), 2-bit codes into four.
template <int K>
__device__ __forceinline__ float byte_as_float(uint32_t w) {
  float f;
  if constexpr (K == 0) asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(f) : "v"(w));
  else if constexpr (K == 1) asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(f) : "v"(w));
  else if constexpr (K == 2) asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(f) : "v"(w));
  else asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(f) : "v"(w));
  return f;
}
// f[0..7] = codes of channels 8 o .. 8 o + 7 of a row whose words are w
template <int B>
__device__ __forceinline__ void octet_as_floats(const uint32_t* w, int o, float (&f)[8]) {
  if constexpr (B == 8) {
    const uint32_t x = w[2 * o], y = w[2 * o + 1];
    f[0] = byte_as_float<0>(x); f[1] = byte_as_float<1>(x); f[2] = byte_as_float<2>(x); f[3] = byte_as_float<3>(x);
    f[4] = byte_as_float<0>(y); f[5] = byte_as_float<1>(y); f[6] = byte_as_float<2>(y); f[7] = byte_as_float<3>(y);
  } else if constexpr (B == 4) {
    const uint32_t x = w[o], ev = x & 0x0F0F0F0Fu, od = (x >> 4) & 0x0F0F0F0Fu;
    f[0] = byte_as_float<0>(ev); f[2] = byte_as_float<1>(ev); f[4] = byte_as_float<2>(ev); f[6] = byte_as_float<3>(ev);
    f[1] = byte_as_float<0>(od); f[3] = byte_as_float<1>(od); f[5] = byte_as_float<2>(od); f[7] = byte_as_float<3>(od);
  } else {
    const uint32_t x = (w[o >> 1] >> (16 * (o & 1))) & 0xFFFFu;          // eight 2-bit codes
    const uint32_t t = x | (x << 16);                                     // codes 0..3 in bits 0..7, codes 4..7 in bits 24..31
    const uint32_t lo = t & 0x03000003u, m1 = (t >> 2) & 0x03000003u, m2 = (t >> 4) & 0x03000003u, m3 = (t >> 6) & 0x03000003u;
    // byte 0 of each word holds code k, byte 3 holds code k + 4
    f[0] = byte_as_float<0>(lo); f[4] = byte_as_float<3>(lo);
    f[1] = byte_as_float<0>(m1); f[5] = byte_as_float<3>(m1);
    f[2] = byte_as_float<0>(m2); f[6] = byte_as_float<3>(m2);
    f[3] = byte_as_float<0>(m3); f[7] = byte_as_float<3>(m3);
  }
}

// Per head and middle token: D[h, j] = sum over channels of q~[c] K~[h, j, c], K~ = s (code - z) (Eq. 10), evaluated
// with the per-group factors pulled out of the per-token work: a = q~[c] * s[c] and b = -float(z[c]) * a once per
// (head, key group, channel), p[c] = fma(float(code[c]), a[c], b[c]) per token, then the stride-halving pairwise tree
// p[c] += p[c + m] for m = 32, 16, ..., 1.  One thread holds one token's 64 channels; a block covers 256 consecutive
// cache positions of one head, starting behind the first frame (whose tokens are never scored), and stages a and b of
// the key groups it touches in LDS.
constexpr int kScoreGroupsMax = 256 / 32 + 1;
template <int B>
__global__ __launch_bounds__(256) void score_dots_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.z];
  if (!it.prune) return;
  const int h = blockIdx.y;
  const int j0 = g.n + blockIdx.x * 256;
  if (j0 >= it.t_c) return;
  const uint8_t* half = cache_half(g, it.cache, it.cur);
  constexpr int kRowWords = 2 * B;                 // 64 channels * B bits / 32
  __shared__ __attribute__((aligned(16))) float s_a[kScoreGroupsMax][kHeadDim];
  __shared__ __attribute__((aligned(16))) float s_b[kScoreGroupsMax][kHeadDim];

  // the token's code row is requested first, so that its latency runs beside the staging of the group factors
  const int j = j0 + threadIdx.x;
  uint32_t w[kRowWords];
  {
    const int jl = min(j, it.t_c - 1);
    const uint32_t* src = reinterpret_cast<const uint32_t*>(half + g.lay.k_codes + ((int64_t)h * g.t_cap + jl) * (8 * B));
#pragma unroll
    for (int i = 0; i < kRowWords; ++i) w[i] = src[i];
  }
  const int k_shift = g.k_group == 64 ? 6 : 5;      // groups of 64 or 32 tokens
  const int grp0 = j0 >> k_shift;
  const int groups_in_block = ((min(j0 + 255, it.t_c - 1)) >> k_shift) - grp0 + 1;      // <= 5 or 9
  const float* qt = reinterpret_cast<const float*>(cache_scratch(g, it.cache) + g.sl.qt);
  for (int i = threadIdx.x; i < groups_in_block * kHeadDim; i += 256) {
    const int gi = i >> 6, c = i & 63;
    const int grp = grp0 + gi;
    float sv, zf;
    if (g.meta16) {
      // halves: logit-domain scale a16 (s = a16 * fp32(1 / scale_log2)) and 1024 + z, channels of an octet in the order 0 4 1 5 2 6 3 7
      const int64_t moff = ((int64_t)h * g.g_cap + grp) * kHeadDim + meta16_pos(c);
      sv = (float)__builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t*>(half + g.lay.k_scale)[moff]) * g.inv_scale_log2;
      zf = (float)__builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t*>(half + g.lay.k_zero)[moff]) - 1024.0f;
    } else {
      const int64_t moff = ((int64_t)h * g.g_cap + grp) * kHeadDim + c;
      sv = reinterpret_cast<const float*>(half + g.lay.k_scale)[moff];
      zf = (float)reinterpret_cast<const int32_t*>(half + g.lay.k_zero)[moff];
    }
    const float a = qt[c] * sv;
    s_a[gi][c] = a;
    s_b[gi][c] = (-zf) * a;
  }
  __syncthreads();

  if (j >= it.t_c) return;
  const int gi = (j >> k_shift) - grp0;
  float p[kHeadDim];
#pragma unroll
  for (int o = 0; o < 8; ++o) {
    float f[8];
    octet_as_floats<B>(w, o, f);
    const float4 a0 = *reinterpret_cast<const float4*>(&s_a[gi][8 * o]), a1 = *reinterpret_cast<const float4*>(&s_a[gi][8 * o + 4]);
    const float4 b0 = *reinterpret_cast<const float4*>(&s_b[gi][8 * o]), b1 = *reinterpret_cast<const float4*>(&s_b[gi][8 * o + 4]);
    p[8 * o + 0] = __builtin_fmaf(f[0], a0.x, b0.x);
    p[8 * o + 1] = __builtin_fmaf(f[1], a0.y, b0.y);
    p[8 * o + 2] = __builtin_fmaf(f[2], a0.z, b0.z);
    p[8 * o + 3] = __builtin_fmaf(f[3], a0.w, b0.w);
    p[8 * o + 4] = __builtin_fmaf(f[4], a1.x, b1.x);
    p[8 * o + 5] = __builtin_fmaf(f[5], a1.y, b1.y);
    p[8 * o + 6] = __builtin_fmaf(f[6], a1.z, b1.z);
    p[8 * o + 7] = __builtin_fmaf(f[7], a1.w, b1.w);
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
#pragma unroll
    for (int c = 0; c < m; ++c) p[c] = p[c] + p[c + m];
  }
  reinterpret_cast<float*>(cache_scratch(g, it.cache) + g.sl.dots)[(int64_t)h * g.t_cap + j] = p[0];
}

void launch_pool(const KvxBatch& b, hipStream_t st) {
  hipLaunchKernelGGL(pool_rows_kernel, dim3(b.g.n_pooled * (b.g.n_new / b.g.n), b.n_items), dim3(std::max(64, 8 * b.g.H)), 0, st, b);
  hipLaunchKernelGGL(pool_mean_kernel, dim3(b.n_items), dim3(1024), 0, st, b);
}

void launch_score(const KvxBatch& b, int max_tc, hipStream_t st) {
  dim3 grid((std::max(max_tc - b.g.n, 1) + 255) / 256, b.g.H, b.n_items);      // the middle tokens: behind the first frame
  switch (b.g.k_bits) {
    case 2: hipLaunchKernelGGL(score_dots_kernel<2>, grid, dim3(256), 0, st, b); break;
    case 4: hipLaunchKernelGGL(score_dots_kernel<4>, grid, dim3(256), 0, st, b); break;
    default: hipLaunchKernelGGL(score_dots_kernel<8>, grid, dim3(256), 0, st, b); break;
  }
}

}  // namespace kvx
