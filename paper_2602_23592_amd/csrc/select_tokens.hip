// Token-granularity selection (the comparison scheme of Section 3 and Section 4.2, "System advantage"):
// keep the k tokens whose recomputed K/V state deviates most from the cached one.
//
// Rank-based top-k, so the result is a pure function of the deviations: candidate i is kept iff fewer than k
// candidates come before it in the order (deviation descending, index ascending).  The ranks are counted by
// all workgroups (n^2 comparisons, the deviations streamed through LDS); one workgroup then compacts the
// kept indices in ascending order and appends the tail (instruction rows).
#include "keep_internal.h"

namespace keep {

constexpr int TR_THREADS = 256;
constexpr int TR_TILE = 2048;

__global__ void __launch_bounds__(TR_THREADS)
    k_token_rank(const float* __restrict__ dev, int n, int k, int32_t* __restrict__ flags) {
  __shared__ float tile[TR_TILE];
  const int i = blockIdx.x * TR_THREADS + threadIdx.x;
  const float v = i < n ? dev[i] : 0.f;
  int rank = 0;
  for (int j0 = 0; j0 < n; j0 += TR_TILE) {
    const int cnt = min(TR_TILE, n - j0);
    for (int t = threadIdx.x; t < cnt; t += TR_THREADS) tile[t] = dev[j0 + t];
    __syncthreads();
    // candidates before i win ties, candidates after i do not: split the tile at i
    const int split = min(max(i - j0, 0), cnt);
    for (int t = 0; t < split; ++t) rank += tile[t] >= v;
    for (int t = split; t < cnt; ++t) rank += tile[t] > v;  // (t == i - j0 compares v > v: false)
    __syncthreads();
  }
  if (i < n) flags[i] = rank < k;
}

// one workgroup: exclusive prefix sum of the flags, kept indices written in ascending order, then the tail
__global__ void __launch_bounds__(1024)
    k_token_compact(const int32_t* __restrict__ flags, int n, int n_tail, int32_t* __restrict__ list) {
  __shared__ int s_wave[16];
  __shared__ int s_base;
  if (threadIdx.x == 0) s_base = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i0 = 0; i0 < n; i0 += 1024) {
    const int i = i0 + threadIdx.x;
    const int f = i < n ? flags[i] : 0;
    // inclusive scan inside the wave
    int x = f;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(x, o, 64);
      if (lane >= o) x += y;
    }
    if (lane == 63) s_wave[wave] = x;
    __syncthreads();
    int before = s_base;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    if (f) list[before + x - 1] = i;
    __syncthreads();
    if (threadIdx.x == 1023) s_base = before + x;
    __syncthreads();
  }
  const int kept = s_base;
  for (int t = threadIdx.x; t < n_tail; t += 1024) list[kept + t] = n + t;
}

void launch_select_tokens(const float* d_deviation, int32_t n, int32_t k, int32_t n_tail, int32_t* d_flags,
                          int32_t* d_list, hipStream_t s) {
  if (n > 0)
    hipLaunchKernelGGL(k_token_rank, dim3((n + TR_THREADS - 1) / TR_THREADS), dim3(TR_THREADS), 0, s, d_deviation, n, k,
                       d_flags);
  hipLaunchKernelGGL(k_token_compact, dim3(1), dim3(1024), 0, s, d_flags, n, n_tail, d_list);
}

}  // namespace keep
