// Top-k selection and keep list (paper Sec. 3.2): keep the first frame, the k best
// middle tokens (k = L_max - T_first - T_current) and the current frame, in ascending
// position order.  Integer work throughout: scores are compared through an
// order-preserving uint32 image of their fp32 bits, equal scores keep the lower
// position, so the result is unique and bit-exact.
//
// One workgroup of 1024 threads per cache.  Each thread keeps its share of the keys in
// registers (element i of thread t is position t + 1024 i, so the loads coalesce); a
// 3-pass most-significant-digit-first radix select (12, 10 and 10 bits) over an LDS
// histogram finds the key of the last token to drop; keep flags go to LDS and a block scan
// over contiguous chunks compacts the survivors in position order.  The first digit takes
// sign, exponent and three mantissa bits, so scores of one magnitude still spread over
// several bins and the LDS atomics of a wave rarely pile onto one address; after it only
// the keys of one bin remain candidates.
#include "kvx_dev.h"

namespace kvx {

constexpr int kSelThreads = 1024;
constexpr int kSelPerThread = 32;                              // keys held in registers per thread
constexpr int kSelMaxM = kSelThreads * kSelPerThread;          // 32768 middle tokens

__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum of one int per thread over a 1024-thread block.
__device__ __forceinline__ int block_scan_excl(int v, int* wave_sums, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
  __syncthreads();                 // wave_sums may still be read from a previous call
  if (lane == 63) wave_sums[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int s = wave_sums[w];
    if (w < wave) base += s;
    tot += s;
  }
  total = tot;
  return base + inc - v;
}

// S_j = (D[0,j] + D[1,j] + ... + D[H-1,j]) / H for the middle tokens, heads added in order
// (Eq. 4-6), and the order-preserving key of each score.  One thread per token, the H
// loads of a token independent of each other.
__global__ __launch_bounds__(256) void score_sum_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.y];
  if (!it.prune) return;
  const int n = g.n, H = g.H;
  const int M = it.t_c - n;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= M) return;
  uint8_t* sc = cache_scratch(g, it.cache);
  const float* d0 = reinterpret_cast<const float*>(sc + g.sl.dots) + n + i;
  float acc = d0[0];
  int h = 1;
  for (; h + 7 < H; h += 8) {
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = d0[(int64_t)(h + k) * g.t_cap];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc = acc + v[k];
  }
  for (; h < H; ++h) acc = acc + d0[(int64_t)h * g.t_cap];
  const float s = acc / (float)H;
  reinterpret_cast<float*>(sc + g.sl.scores)[i] = s;
  reinterpret_cast<uint32_t*>(sc + g.sl.keys)[i] = order_key(s);
}

constexpr int kSelBins = 4096;

__global__ __launch_bounds__(kSelThreads) void select_kernel(const KvxBatch b) {
  const Geometry& g = b.g;
  const Item it = b.items[blockIdx.x];
  if (!it.prune) return;
  const int n = g.n, t_c = it.t_c;
  const int n_cur = g.n_new;             // the call's tokens: always kept
  const int M = t_c - n;                 // middle tokens: cache positions n .. t_c - 1
  const int T = t_c + n_cur;
  const int n_drop = T - g.budget;       // >= 1
  const int k_keep = M - n_drop;         // = budget - n - n_cur
  uint8_t* sc = cache_scratch(g, it.cache);
  const uint32_t* keys = reinterpret_cast<const uint32_t*>(sc + g.sl.keys);
  int32_t* keep = reinterpret_cast<int32_t*>(sc + g.sl.keep);
  int32_t* sel = reinterpret_cast<int32_t*>(sc + g.sl.sel);
  const int tid = threadIdx.x;
  const int used = (M + kSelThreads - 1) / kSelThreads;      // keys per thread actually present (<= kSelPerThread)

  __shared__ int hist[kSelBins];
  __shared__ int wave_sums[16];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_remaining;
  __shared__ int sh_p0;
  __shared__ int sh_eq;
  __shared__ uint8_t flags[kSelMaxM];

  uint32_t key[kSelPerThread];
#pragma unroll
  for (int k = 0; k < kSelPerThread; ++k) {
    const int i = tid + k * kSelThreads;
    key[k] = (k < used && i < M) ? keys[i] : 0u;
  }
  if (tid == 0) {
    sh_prefix = 0u;
    sh_remaining = n_drop;
    sh_p0 = T;
  }
  __syncthreads();

  // Key of the n_drop-th smallest element, digit by digit.
  uint32_t mask = 0u;
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
    const int bins = pass == 0 ? 4096 : 1024;
    for (int i = tid; i < bins; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
#pragma unroll
    for (int k = 0; k < kSelPerThread; ++k) {
      if (k < used) {
        const int i = tid + k * kSelThreads;
        if (i < M && (key[k] & mask) == prefix) atomicAdd(&hist[(key[k] >> shift) & (uint32_t)(bins - 1)], 1);
      }
    }
    __syncthreads();
    {
      // the bin holding the rem-th smallest candidate: each thread owns bins / 1024 consecutive
      // bins, counts before each thread's bins by a block scan
      const int per = bins / kSelThreads;                   // 4 or 1
      int c4[4] = {0, 0, 0, 0};
      int cnt = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < per) { c4[j] = hist[tid * per + j]; cnt += c4[j]; }
      int tot_unused;
      int before = block_scan_excl(cnt, wave_sums, tot_unused);
      const int rem = sh_remaining;
      __syncthreads();
      if (before < rem && before + cnt >= rem) {           // exactly one thread
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (j < per) {
            if (before < rem && before + c4[j] >= rem) {
              sh_remaining = rem - before;
              sh_prefix = prefix | ((uint32_t)(tid * per + j) << shift);
              sh_eq = c4[j];                                // after the last pass: keys equal to the threshold
              before = rem;                                 // no later bin matches
            } else {
              before += c4[j];
            }
          }
        }
      }
    }
    mask |= (uint32_t)(bins - 1) << shift;
    __syncthreads();
  }
  const uint32_t thr = sh_prefix;
  const int need_eq = sh_remaining;              // equal-keyed tokens to drop (highest positions first)
  const int total_eq = sh_eq;
  const int eq_keep = total_eq - need_eq;        // equal-keyed tokens kept: the eq_keep lowest positions

  // Keep flags: 1 = keep, 0 = drop, 2 = equal to the threshold (resolved by position below).
#pragma unroll
  for (int k = 0; k < kSelPerThread; ++k) {
    const int i = tid + k * kSelThreads;
    if (k < used && i < M) flags[i] = key[k] > thr ? 1 : (key[k] == thr ? (eq_keep == 0 ? 0 : 2) : 0);
  }
  __syncthreads();

  // Contiguous chunk of middle positions per thread, so prefix sums follow position order.
  const int chunk = (M + kSelThreads - 1) / kSelThreads;
  const int c0 = min(tid * chunk, M), c1 = min(c0 + chunk, M);
  int tot;
  if (eq_keep > 0) {                              // ties straddle the cut: the lowest positions stay
    int eq_cnt = 0;
    for (int i = c0; i < c1; ++i) eq_cnt += (flags[i] == 2);
    int eq_rank = block_scan_excl(eq_cnt, wave_sums, tot);
    for (int i = c0; i < c1; ++i)
      if (flags[i] == 2) {
        flags[i] = eq_rank < eq_keep ? 1 : 0;
        ++eq_rank;
      }
  }
  int kept_cnt = 0;
  for (int i = c0; i < c1; ++i) kept_cnt += flags[i];
  int out = block_scan_excl(kept_cnt, wave_sums, tot);
  int first_drop = T;
  // slot layout: the freed slots in ascending order, then the never-used tail, take the call's tokens in order
  int32_t* newtok = reinterpret_cast<int32_t*>(sc + g.sl.newtok);
  int32_t* assign = reinterpret_cast<int32_t*>(sc + g.sl.assign);
  for (int i = c0; i < c1; ++i) {
    if (flags[i]) {
      keep[n + out] = n + i;
      if (g.slots) newtok[n + i] = -1;
      ++out;
    } else {
      if (first_drop == T) first_drop = n + i;
      if (g.slots) {
        const int d = i - out;             // dropped tokens before this one
        assign[d] = n + i;
        newtok[n + i] = d;
      }
    }
  }
  if (g.slots) {
    for (int i = tid; i < n; i += kSelThreads) newtok[i] = -1;
    for (int sl = t_c + tid; sl < g.budget; sl += kSelThreads) {
      const int d = n_drop + (sl - t_c);
      assign[d] = sl;
      newtok[sl] = d;
    }
  }
  if (first_drop < T) atomicMin(&sh_p0, first_drop);
  // the first frame and the call's own tokens are always kept
  for (int i = tid; i < n; i += kSelThreads) keep[i] = i;
  for (int i = tid; i < n_cur; i += kSelThreads) keep[n + k_keep + i] = t_c + i;
  __syncthreads();
  if (tid == 0) {
    sel[0] = sh_p0;
    sel[1] = sh_p0 / g.k_group;
    sel[3] = tot;                                 // survivors among the middle tokens (= k)
  }
}

void launch_select(const KvxBatch& b, int max_tc, hipStream_t st) {
  hipLaunchKernelGGL(score_sum_kernel, dim3((max_tc + 255) / 256, b.n_items), dim3(256), 0, st, b);
  hipLaunchKernelGGL(select_kernel, dim3(b.n_items), dim3(kSelThreads), 0, st, b);
}

}  // namespace kvx
