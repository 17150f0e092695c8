// Multi-hop importance propagation and selection (Section 4.2 of the paper:
// initialisation, importance propagation, convergence check) on the device.
//
// One workgroup.  Every floating-point value that decides the selection is
// computed in binary32 in a fixed order (sums over candidates in ascending
// order, one division each), so the result is a pure function of S.
#include "keep_internal.h"

namespace keep {

constexpr int SEL_THREADS = 1024;

// rank every candidate by (importance descending, index ascending) and mark the
// ones taken: the first k of the order (count mode) or a walk of the order that
// takes a memory iff it still fits the token budget (token mode).  All arrays in LDS.
// `imp` is consumed: in token mode its storage holds the lengths in rank order, then the walk's decisions.
__device__ void take(float* imp, int m, const int32_t* len, int k_count, int token_budget, int mode,
                     int32_t* order, int32_t* taken) {
  int my_rank[6];  // ranks of this thread's candidates (m <= 6000, 1024 threads)
  int n_mine = 0;
  for (int b = threadIdx.x; b < m; b += SEL_THREADS) {
    const float v = imp[b];
    int rank = 0;
    for (int c = 0; c < m; ++c) {
      const float u = imp[c];
      rank += (u > v) || (u == v && c < b);
    }
    my_rank[n_mine++] = rank;
    order[rank] = b;
    if (mode == KEEP_BUDGET_GROUP_COUNT) taken[b] = rank < k_count;
  }
  __syncthreads();  // every importance has been read, every rank is known
  if (mode != KEEP_BUDGET_GROUP_COUNT) {
    // The walk itself is sequential (a memory that does not fit is skipped, the next one may fit), so it is
    // given the lengths in rank order and writes its decisions back in place: one LDS read and one write per
    // step with independent addresses; the scatter to `taken` is parallel again.
    int32_t* olen = reinterpret_cast<int32_t*>(imp);
    n_mine = 0;
    for (int b = threadIdx.x; b < m; b += SEL_THREADS) olen[my_rank[n_mine++]] = len[b];
    __syncthreads();
    if (threadIdx.x == 0) {
      int used = 0;
      for (int i = 0; i < m; ++i) {
        const int l = olen[i];
        const int fits = used + l <= token_budget;
        olen[i] = fits;
        used += fits ? l : 0;
      }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < m; i += SEL_THREADS) taken[order[i]] = olen[i];
    __syncthreads();
  }
}

// The normalised score of (a, b) is S[a, b] / total_a with total_a the sum of row a in ascending order
// (0 where the row is empty); it is formed where it is used, only the row totals are kept.
__global__ void __launch_bounds__(SEL_THREADS)
    k_select(const float* __restrict__ S, int m, const int32_t* __restrict__ cand_len, int k_count, int token_budget,
             int mode, int hops, int set_only, int tile_rows, float* __restrict__ work, int32_t* __restrict__ iwork,
             int32_t* __restrict__ out, const int32_t* __restrict__ cand_total, const int32_t* __restrict__ id_map) {
  extern __shared__ float sel_smem[];
  float* tot = sel_smem;                                   // [m + 1] row totals
  float* imp = tot + (m + 1);                              // [m]
  int32_t* order = reinterpret_cast<int32_t*>(imp + m);    // [m]
  int32_t* rel = order + m;                                // [m]
  int32_t* rel2 = rel + m;                                 // [m]
  int32_t* len = rel2 + m;                                 // [m]
  __shared__ int s_same, s_cnt;
  (void)work;
  (void)iwork;
  // Callers that could not classify the budget on the host pass the candidates' token total: a budget that
  // takes every candidate or none is settled here without a selection (0 selections run), as the host does
  // for the other callers.
  if (cand_total) {
    const bool all = m > 0 && (mode == KEEP_BUDGET_GROUP_COUNT ? k_count >= m : token_budget >= *cand_total);
    const bool none = m == 0 || (mode == KEEP_BUDGET_GROUP_COUNT ? k_count == 0 : token_budget <= 0);
    if (all || none) {
      const int n = all ? m : 0;
      for (int a = threadIdx.x; a < n; a += SEL_THREADS) out[2 + a] = id_map ? id_map[a] : a;
      if (threadIdx.x == 0) {
        out[0] = n;
        out[1] = 0;
      }
      return;
    }
  }

  if (tile_rows > 0) {
    // Row totals, each still summed one element after the other in ascending order, but read through LDS:
    // blocks of tile_rows rows x 32 columns are fetched with consecutive threads on consecutive columns
    // (a thread walking its own row of S directly touches a new cache line at every step).
    float* tile = reinterpret_cast<float*>(len + m);  // [tile_rows][33]
    for (int a0 = 0; a0 <= m; a0 += tile_rows) {
      const int rows = min(tile_rows, m + 1 - a0);
      float total = 0.f;
      for (int b0 = 0; b0 < m; b0 += 32) {
        const int cols = min(32, m - b0);
        for (int i = threadIdx.x; i < rows * 32; i += SEL_THREADS) {
          const int r = i >> 5, j = i & 31;
          if (j < cols) tile[r * 33 + j] = S[(size_t)(a0 + r) * m + b0 + j];
        }
        __syncthreads();
        if ((int)threadIdx.x < rows)
          for (int j = 0; j < cols; ++j) total = total + tile[threadIdx.x * 33 + j];
        __syncthreads();
      }
      if ((int)threadIdx.x < rows) tot[a0 + threadIdx.x] = total;
    }
  } else {
    for (int a = threadIdx.x; a <= m; a += SEL_THREADS) {
      const float* row = S + (size_t)a * m;
      float total = 0.f;
      for (int b = 0; b < m; ++b) total = total + row[b];
      tot[a] = total;
    }
  }
  for (int b = threadIdx.x; b < m; b += SEL_THREADS) len[b] = cand_len[b];
  __syncthreads();
  const float tq = tot[m];
  for (int b = threadIdx.x; b < m; b += SEL_THREADS) imp[b] = tq > 0.f ? S[(size_t)m * m + b] / tq : 0.f;
  __syncthreads();
  take(imp, m, len, k_count, token_budget, mode, order, rel);
  int runs = 1;
  const int max_runs = hops > 1 ? hops : 1;
  while (runs < max_runs) {
    if (threadIdx.x == 0) s_cnt = 0;
    __syncthreads();
    {
      int c = 0;  // (integer count: the order of the additions does not matter)
      for (int a = threadIdx.x; a < m; a += SEL_THREADS) c += rel[a];
      if (c) atomicAdd(&s_cnt, c);
    }
    __syncthreads();
    // sources of the propagation: the query and the relevant set, or (set_only: the section's wording taken
    // literally) the relevant set alone; an empty source set leaves the importance at zero
    const int n_src = (set_only ? 0 : 1) + s_cnt;
    const float denom = (float)n_src;
    for (int b = threadIdx.x; b < m; b += SEL_THREADS) {
      float acc = (!set_only && tq > 0.f) ? S[(size_t)m * m + b] / tq : 0.f;
      for (int a = 0; a < m; ++a)
        if (rel[a]) {
          const float ta = tot[a];
          acc = acc + (ta > 0.f ? S[(size_t)a * m + b] / ta : 0.f);
        }
      imp[b] = n_src > 0 ? acc / denom : acc;
    }
    __syncthreads();
    take(imp, m, len, k_count, token_budget, mode, order, rel2);
    ++runs;
    if (threadIdx.x == 0) s_same = 1;
    __syncthreads();
    {
      int differs = 0;
      for (int a = threadIdx.x; a < m; a += SEL_THREADS) differs |= (rel[a] != rel2[a]);
      if (differs) s_same = 0;  // (every writer writes the same value)
    }
    __syncthreads();
    const int same = s_same;
    __syncthreads();
    if (same) break;
    for (int b = threadIdx.x; b < m; b += SEL_THREADS) rel[b] = rel2[b];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    int n = 0;
    for (int a = 0; a < m; ++a)
      if (rel[a]) out[2 + n++] = id_map ? id_map[a] : a;
    out[0] = n;
    out[1] = runs;
  }
}

void launch_select(const float* S, int32_t m, const int32_t* d_cand_len, int32_t k_count, int32_t token_budget,
                   int32_t mode, int32_t hops, float* d_work, int32_t* d_iwork, int32_t* d_out, hipStream_t s,
                   bool set_only, const int32_t* d_cand_total, const int32_t* d_id_map) {
  size_t sh = ((size_t)(m + 1) + m) * sizeof(float) + (size_t)4 * m * sizeof(int32_t);  // <= 160 KB: m <= 6000
  // room for the staging tile of the row totals (256 rows x 33 floats) unless the arrays leave none
  int tile_rows = 0;
  if (sh + (size_t)256 * 33 * sizeof(float) <= (size_t)160 * 1024 - 256) {
    tile_rows = 256;
    sh += (size_t)256 * 33 * sizeof(float);
  }
  static std::atomic<uint64_t> attr_done{0};
  set_max_dyn_smem_once(attr_done, reinterpret_cast<const void*>(k_select), 160 * 1024 - 256);
  hipLaunchKernelGGL(k_select, dim3(1), dim3(SEL_THREADS), sh, s, S, m, d_cand_len, k_count, token_budget, mode, hops,
                     set_only ? 1 : 0, tile_rows, d_work, d_iwork, d_out, d_cand_total, d_id_map);
}

}  // namespace keep
