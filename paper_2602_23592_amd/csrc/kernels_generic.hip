// Generic (scalar-FMA, fp32-accumulate) kernels: the kernel family used for fp32
// storage and for shapes the MFMA kernels do not take.  LDS-tiled GEMM, one-row
// flash-style attention, per-row group-score reduction.
#include "keep_internal.h"

namespace keep {

// ---------------------------------------------------------------------------
// C[M,N] = A[M,K] . W[N,K]^T, 64x64 tile, 16-deep K slices, 4x4 outputs per thread
// ---------------------------------------------------------------------------
struct BRows {
  const void* ptr[3];
  int32_t begin[4];  // first global column of each part, begin[n_parts] = N
  int32_t n_parts;
};

template <typename T, int EPI>
__global__ void __launch_bounds__(256)
    k_gemm_generic(const T* __restrict__ A, int M, int K, BRows B, const T* __restrict__ B2, int N,
                   const T* __restrict__ residual, void* __restrict__ Cv) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 1];
  __shared__ float Bs[BK][BN + 1];
  __shared__ float Bs2[EPI == EPI_SWIGLU_STORE ? BK : 1][BN + 1];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int lrow = tid >> 2, lk = (tid & 3) * 4;  // 64 rows x 4 chunks of 4 k
  const int tx = tid & 15, ty = tid >> 4;         // 16 x 16 threads, 4x4 outputs each
  float acc[4][4] = {}, acc2[4][4] = {};

  // resolve this thread's B row once
  const int bn = n0 + lrow;
  const T* brow = nullptr;
  if (bn < N) {
    const void* base = B.ptr[0];
    int first = 0;
    if (B.n_parts > 1 && bn >= B.begin[1]) {
      base = B.ptr[1];
      first = B.begin[1];
    }
    if (B.n_parts > 2 && bn >= B.begin[2]) {
      base = B.ptr[2];
      first = B.begin[2];
    }
    brow = reinterpret_cast<const T*>(base) + (size_t)(bn - first) * K;
  }
  const T* brow2 = (EPI == EPI_SWIGLU_STORE && bn < N) ? B2 + (size_t)bn * K : nullptr;
  const int am = m0 + lrow;
  const T* arow = am < M ? A + (size_t)am * K : nullptr;

  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int k = k0 + lk + e;
      As[lk + e][lrow] = (arow && k < K) ? ldf(arow + k) : 0.f;
      Bs[lk + e][lrow] = (brow && k < K) ? ldf(brow + k) : 0.f;
      if (EPI == EPI_SWIGLU_STORE) Bs2[lk + e][lrow] = (brow2 && k < K) ? ldf(brow2 + k) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4], b2[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
      if (EPI == EPI_SWIGLU_STORE) {
#pragma unroll
        for (int j = 0; j < 4; ++j) b2[j] = Bs2[kk][tx * 4 + j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] += a[i] * b[j];
          if (EPI == EPI_SWIGLU_STORE) acc2[i][j] += a[i] * b2[j];
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      const size_t idx = (size_t)m * N + n;
      if (EPI == EPI_STORE_F32) {
        reinterpret_cast<float*>(Cv)[idx] = acc[i][j];
      } else if (EPI == EPI_RESIDUAL_STORE) {
        stf(reinterpret_cast<T*>(Cv) + idx, ldf(residual + idx) + acc[i][j]);
      } else {
        const float g = acc[i][j];
        stf(reinterpret_cast<T*>(Cv) + idx, g / (1.0f + expf(-g)) * acc2[i][j]);
      }
    }
  }
}

template <typename T>
void launch_gemm_generic(const T* A, int32_t M, int32_t K, const GemmB& B, const void* B2, int32_t N, int epilogue,
                         const T* residual, void* C, hipStream_t s) {
  if (M <= 0 || N <= 0) return;
  BRows br;
  br.n_parts = B.n_parts;
  int acc = 0;
  for (int p = 0; p < 3; ++p) {
    br.ptr[p] = p < B.n_parts ? B.ptr[p] : nullptr;
    br.begin[p] = acc;
    if (p < B.n_parts) acc += B.n_rows[p];
  }
  br.begin[3] = acc;
  dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
  const T* b2 = reinterpret_cast<const T*>(B2);
  switch (epilogue) {
    case EPI_STORE_F32:
      hipLaunchKernelGGL((k_gemm_generic<T, EPI_STORE_F32>), grid, block, 0, s, A, M, K, br, b2, N, residual, C);
      break;
    case EPI_RESIDUAL_STORE:
      hipLaunchKernelGGL((k_gemm_generic<T, EPI_RESIDUAL_STORE>), grid, block, 0, s, A, M, K, br, b2, N, residual, C);
      break;
    default:
      hipLaunchKernelGGL((k_gemm_generic<T, EPI_SWIGLU_STORE>), grid, block, 0, s, A, M, K, br, b2, N, residual, C);
      break;
  }
}

// ---------------------------------------------------------------------------
// attention of one recomputed row and one query head over the cache rows 0..p
// (online softmax over chunks of 256 keys)
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
    k_attn_generic(const T* __restrict__ q, const T* __restrict__ k_cache, const T* __restrict__ v_cache,
                   const int32_t* __restrict__ row_pos, const int32_t* __restrict__ row_lo, int n_q_heads,
                   int n_kv_heads, int head_dim, T* __restrict__ o, float* __restrict__ lse) {
  extern __shared__ float smem[];
  float* s_q = smem;              // [head_dim]
  float* s_p = s_q + head_dim;    // [256]
  float* s_red = s_p + 256;       // [8]
  float* s_acc = s_red + 8;       // [256] cross-part reduction of the output
  const int r = blockIdx.x, h = blockIdx.y;
  const int hk = h / (n_q_heads / n_kv_heads);
  const int p_row = row_pos[r];
  const int p_lo = row_lo ? row_lo[r] : 0;  // first visible key (a unit cached on its own sees only itself)
  const int kv_dim = n_kv_heads * head_dim;
  const int tid = threadIdx.x;
  const float scale = 1.0f / sqrtf((float)head_dim);
  for (int d = tid; d < head_dim; d += 256) s_q[d] = ldf(q + ((size_t)r * n_q_heads + h) * head_dim + d);
  __syncthreads();
  // threads split as (part, d): part strides over the keys of a chunk, d is the output dim
  const int n_parts = 256 / head_dim > 0 ? 256 / head_dim : 1;
  const int part = tid / head_dim, d_out = tid - part * head_dim;
  const bool pv_active = part < n_parts && head_dim <= 256;
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int c0 = p_lo; c0 <= p_row; c0 += 256) {
    const int key = c0 + tid;
    float sc = -INFINITY;
    if (key <= p_row) {
      const T* kr = k_cache + (size_t)key * kv_dim + hk * head_dim;
      float dot = 0.f;
      for (int d = 0; d < head_dim; ++d) dot += s_q[d] * ldf(kr + d);
      sc = dot * scale;
    }
    // chunk max
    float mx = sc;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if ((tid & 63) == 0) s_red[tid >> 6] = mx;
    __syncthreads();
    const float m_new = fmaxf(m_run, fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3])));
    const float pj = key <= p_row ? expf(sc - m_new) : 0.f;
    s_p[tid] = pj;
    float sm = pj;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sm += __shfl_xor(sm, off, 64);
    if ((tid & 63) == 0) s_red[4 + (tid >> 6)] = sm;
    __syncthreads();
    const float alpha = expf(m_run - m_new);  // 0 on the first chunk (m_run = -inf)
    l_run = l_run * alpha + (s_red[4] + s_red[5] + s_red[6] + s_red[7]);
    m_run = m_new;
    if (pv_active) {
      acc *= alpha;
      const int kmax = min(256, p_row + 1 - c0);
      for (int j = part; j < kmax; j += n_parts)
        acc += s_p[j] * ldf(v_cache + (size_t)(c0 + j) * kv_dim + hk * head_dim + d_out);
    }
    __syncthreads();
  }
  s_acc[tid] = pv_active ? acc : 0.f;
  __syncthreads();
  if (tid < head_dim) {
    float t = 0.f;
    for (int pp = 0; pp < n_parts; ++pp) t += s_acc[pp * head_dim + tid];
    stf(o + ((size_t)r * n_q_heads + h) * head_dim + tid, t / l_run);
  }
  if (tid == 0) lse[(size_t)r * n_q_heads + h] = m_run + logf(l_run);
}

template <typename T>
void launch_attn_generic(const T* q, const T* k_cache, const T* v_cache, const int32_t* d_row_pos, int32_t n_rows,
                         int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, T* o, float* lse, hipStream_t s,
                         const int32_t* d_row_lo) {
  if (n_rows <= 0) return;
  const size_t sh = (size_t)(head_dim + 256 + 8 + 256) * sizeof(float);
  hipLaunchKernelGGL(k_attn_generic<T>, dim3(n_rows, n_q_heads), dim3(256), sh, s, q, k_cache, v_cache, d_row_pos,
                     d_row_lo, n_q_heads, n_kv_heads, head_dim, o, lse);
}

// ---------------------------------------------------------------------------
// attention mass of one recomputed row towards each candidate memory
//   rowmass[t, j] = sum_h sum_{s in block j, s <= t} exp(q_t,h . k_s / sqrt(dh) - lse[t,h])
// Rows and candidate keys are both in compact (prompt) order, so causality is s <= t.
// One wave per candidate block, lanes stride over its keys, fixed-order reductions.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
    k_score_rows_generic(const T* __restrict__ q, const T* __restrict__ k_compact, const float* __restrict__ lse,
                         const int32_t* __restrict__ row_start, int m, int n_q_heads, int n_kv_heads, int head_dim,
                         float* __restrict__ rowmass) {
  extern __shared__ float smem[];
  float* s_q = smem;                         // [n_q_heads * head_dim]
  float* s_lse = s_q + n_q_heads * head_dim;  // [n_q_heads]
  const int t = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int q_dim = n_q_heads * head_dim, kv_dim = n_kv_heads * head_dim;
  const int rep = n_q_heads / n_kv_heads;
  const float scale = 1.0f / sqrtf((float)head_dim);
  for (int i = tid; i < q_dim; i += 256) s_q[i] = ldf(q + (size_t)t * q_dim + i);
  for (int i = tid; i < n_q_heads; i += 256) s_lse[i] = lse[(size_t)t * n_q_heads + i];
  __syncthreads();
  // own block of row t
  int own = 0;
  {
    int lo = 0, hi = m;  // blocks 0..m (m = instruction)
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      if (row_start[mid] <= t)
        lo = mid;
      else
        hi = mid - 1;
    }
    own = lo;
  }
  for (int j = wave; j < m; j += 4) {
    float sum = 0.f;
    if (j != own) {
      const int s0 = row_start[j];
      const int s1 = min(row_start[j + 1], t + 1);
      for (int s = s0 + lane; s < s1; s += 64) {
        const T* kr = k_compact + (size_t)s * kv_dim;
        for (int h = 0; h < n_q_heads; ++h) {
          const T* kh = kr + (h / rep) * head_dim;
          const float* qh = s_q + h * head_dim;
          float dot = 0.f;
          for (int d = 0; d < head_dim; ++d) dot += qh[d] * ldf(kh + d);
          sum += expf(dot * scale - s_lse[h]);
        }
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) rowmass[(size_t)t * m + j] = sum;
  }
}

template <typename T>
void launch_score_rows_generic(const T* q, const T* k_compact, const float* lse, const int32_t* d_row_start, int32_t m,
                               int32_t n_rows, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                               float* rowmass, hipStream_t s) {
  if (n_rows <= 0 || m <= 0) return;
  const size_t sh = (size_t)(n_q_heads * head_dim + n_q_heads) * sizeof(float);
  hipLaunchKernelGGL(k_score_rows_generic<T>, dim3(n_rows), dim3(256), sh, s, q, k_compact, lse, d_row_start, m,
                     n_q_heads, n_kv_heads, head_dim, rowmass);
}

// S[a, b] = (sum over the rows t of block a, ascending, of rowmass[t, b]) / (heads * len_a * len_b); S[a, a] = 0
__global__ void k_score_finish(const float* __restrict__ rowmass, const int32_t* __restrict__ row_start, int m,
                               int n_q_heads, float* __restrict__ S) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  const int a = blockIdx.y;
  if (b >= m) return;
  float v = 0.f;
  if (a != b) {
    const int t0 = row_start[a], t1 = row_start[a + 1];
    float sum = 0.f;
    for (int t = t0; t < t1; ++t) sum += rowmass[(size_t)t * m + b];
    const float len_a = (float)(t1 - t0), len_b = (float)(row_start[b + 1] - row_start[b]);
    v = sum / ((float)n_q_heads * len_a * len_b);
  }
  S[(size_t)a * m + b] = v;
}

void launch_score_finish(const float* rowmass, const int32_t* d_row_start, int32_t m, int32_t n_q_heads, float* S,
                         hipStream_t s) {
  if (m <= 0) return;
  hipLaunchKernelGGL(k_score_finish, dim3((m + 255) / 256, m + 1), dim3(256), 0, s, rowmass, d_row_start, m, n_q_heads,
                     S);
}

#define INST(T)                                                                                                    \
  template void launch_gemm_generic<T>(const T*, int32_t, int32_t, const GemmB&, const void*, int32_t, int,       \
                                       const T*, void*, hipStream_t);                                              \
  template void launch_attn_generic<T>(const T*, const T*, const T*, const int32_t*, int32_t, int32_t, int32_t,   \
                                       int32_t, T*, float*, hipStream_t, const int32_t*);                          \
  template void launch_score_rows_generic<T>(const T*, const T*, const float*, const int32_t*, int32_t, int32_t,  \
                                             int32_t, int32_t, int32_t, float*, hipStream_t);
INST(float)
INST(bf16_t)
#undef INST

}  // namespace keep
