// HBM-bound kernels of the selective-recompute layer: row bookkeeping, gathers,
// RoPE re-alignment + concatenation of cached groups, RMSNorm, RoPE + scatter of
// refreshed K/V.  All move 16-byte vectors per lane; arithmetic is fp32.
#include "keep_internal.h"

namespace keep {

// ---------------------------------------------------------------------------
// 16-byte vectors of the storage type
// ---------------------------------------------------------------------------
template <typename T>
struct Vec;
template <>
struct Vec<float> {
  static constexpr int N = 4;
  __device__ static void unpack(const uint4& u, float* f) {
    f[0] = __uint_as_float(u.x);
    f[1] = __uint_as_float(u.y);
    f[2] = __uint_as_float(u.z);
    f[3] = __uint_as_float(u.w);
  }
  __device__ static uint4 pack(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};
template <>
struct Vec<bf16_t> {
  static constexpr int N = 8;
  __device__ static void unpack(const uint4& u, float* f) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static uint4 pack(const float* f) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
};

__device__ inline int find_block(const int32_t* starts, int n_blocks, int row) {
  // largest b in [0, n_blocks) with starts[b] <= row  (starts ascending, starts[0] = 0)
  int lo = 0, hi = n_blocks - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (starts[mid] <= row)
      lo = mid;
    else
      hi = mid - 1;
  }
  return lo;
}

// ---------------------------------------------------------------------------
// positions and block slots of the recomputed rows
// ---------------------------------------------------------------------------
__global__ void k_build_rows(const int32_t* __restrict__ set_off, const int32_t* __restrict__ row_start, int m,
                             int instr_off, int n_rows, int32_t* __restrict__ row_pos,
                             int32_t* __restrict__ row_slot) {
  int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_rows) return;
  int slot = find_block(row_start, m + 1, r);
  int base = slot < m ? set_off[slot] : instr_off;
  row_pos[r] = base + (r - row_start[slot]);
  row_slot[r] = slot;
}

void launch_build_rows(const int32_t* d_set_off, const int32_t* d_row_start, int32_t m, int32_t instr_off,
                       int32_t n_rows, int32_t* d_row_pos, int32_t* d_row_slot, hipStream_t s) {
  if (n_rows <= 0) return;
  hipLaunchKernelGGL(k_build_rows, dim3((n_rows + 255) / 256), dim3(256), 0, s, d_set_off, d_row_start, m, instr_off,
                     n_rows, d_row_pos, d_row_slot);
}

// ---------------------------------------------------------------------------
// gathers
// ---------------------------------------------------------------------------
template <typename T>
__global__ void k_embed_gather(const T* __restrict__ embed, const int32_t* __restrict__ token_ids,
                               const int32_t* __restrict__ row_pos, int hidden, T* __restrict__ x) {
  const int r = blockIdx.x;
  const int tok = token_ids[row_pos[r]];
  const uint4* src = reinterpret_cast<const uint4*>(embed + (size_t)tok * hidden);
  uint4* dst = reinterpret_cast<uint4*>(x + (size_t)r * hidden);
  const int nv = hidden / Vec<T>::N;
  for (int i = threadIdx.x; i < nv; i += blockDim.x) dst[i] = src[i];
}

template <typename T>
void launch_embed_gather(const T* embed, const int32_t* d_token_ids, const int32_t* d_row_pos, int32_t n_rows,
                         int32_t hidden, T* x, hipStream_t s) {
  if (n_rows <= 0) return;
  hipLaunchKernelGGL(k_embed_gather<T>, dim3(n_rows), dim3(256), 0, s, embed, d_token_ids, d_row_pos, hidden, x);
}

template <typename T>
__global__ void k_rows_gather(const T* __restrict__ x_src, const int32_t* __restrict__ src_start,
                              const int32_t* __restrict__ dst_start, int n_blocks, int hidden, T* __restrict__ x_dst) {
  const int r = blockIdx.x;
  __shared__ int s_src;
  if (threadIdx.x == 0) {
    int b = find_block(dst_start, n_blocks, r);
    s_src = src_start[b] + (r - dst_start[b]);
  }
  __syncthreads();
  const uint4* src = reinterpret_cast<const uint4*>(x_src + (size_t)s_src * hidden);
  uint4* dst = reinterpret_cast<uint4*>(x_dst + (size_t)r * hidden);
  const int nv = hidden / Vec<T>::N;
  for (int i = threadIdx.x; i < nv; i += blockDim.x) dst[i] = src[i];
}

template <typename T>
void launch_rows_gather(const T* x_src, const int32_t* d_src_start, const int32_t* d_dst_start, int32_t n_blocks_sel,
                        int32_t n_rows_dst, int32_t hidden, T* x_dst, hipStream_t s) {
  if (n_rows_dst <= 0) return;
  hipLaunchKernelGGL(k_rows_gather<T>, dim3(n_rows_dst), dim3(256), 0, s, x_src, d_src_start, d_dst_start,
                     n_blocks_sel, hidden, x_dst);
}

// ---------------------------------------------------------------------------
// re-alignment + concatenation of cached groups
//   K_hat[off_g + j] = Rot(off_g) K_cached[g][j],  V_hat[off_g + j] = V_cached[g][j]
// A cached key sits at group-local position j; rotating it on by the group's start
// offset puts it at global position off_g + j, because rotations add.
// Works in place when a source block already lies at its destination.
// ---------------------------------------------------------------------------
constexpr int REALIGN_ROWS = 4;

template <typename T>
__global__ void k_realign(const RealignSeg* __restrict__ segs, int n_segs, int total_rows, int n_kv_heads,
                          int head_dim, const float* __restrict__ rope_cos, const float* __restrict__ rope_sin,
                          T* __restrict__ k_cache, T* __restrict__ v_cache) {
  constexpr int VN = Vec<T>::N;
  __shared__ int s_seg[REALIGN_ROWS];
  const int row0 = blockIdx.x * REALIGN_ROWS;
  if (threadIdx.x < REALIGN_ROWS) {
    int r = row0 + threadIdx.x;
    int lo = 0, hi = n_segs - 1;
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      if (segs[mid].row_start <= r)
        lo = mid;
      else
        hi = mid - 1;
    }
    s_seg[threadIdx.x] = lo;
  }
  __syncthreads();
  const int half = head_dim / 2;
  const int kv_per_head = half / VN;               // vector pairs per head (K)
  const int k_items = n_kv_heads * kv_per_head;    // per row
  const int v_items = n_kv_heads * head_dim / VN;  // per row
  const int items = k_items + v_items;
  const int row_elems = n_kv_heads * head_dim;
  for (int it = threadIdx.x; it < REALIGN_ROWS * items; it += blockDim.x) {
    const int lr = it / items;
    const int r = row0 + lr;
    if (r >= total_rows) break;
    const RealignSeg sg = segs[s_seg[lr]];
    const int j = r - sg.row_start;  // local position inside the group
    const int i = it - lr * items;
    const size_t dst_row = (size_t)(sg.dst_off + j) * row_elems;
    if (i < k_items) {
      const int h = i / kv_per_head, c = (i - h * kv_per_head) * VN;
      const T* src = reinterpret_cast<const T*>(sg.k_src) + (size_t)j * row_elems + h * head_dim;
      uint4 ulo = *reinterpret_cast<const uint4*>(src + c);
      uint4 uhi = *reinterpret_cast<const uint4*>(src + half + c);
      float lo[VN], hi[VN], olo[VN], ohi[VN];
      Vec<T>::unpack(ulo, lo);
      Vec<T>::unpack(uhi, hi);
      const float* cs = rope_cos + (size_t)sg.dst_off * half + c;
      const float* sn = rope_sin + (size_t)sg.dst_off * half + c;
#pragma unroll
      for (int e = 0; e < VN; ++e) {
        const float cc = cs[e], ss = sn[e];
        olo[e] = lo[e] * cc - hi[e] * ss;
        ohi[e] = hi[e] * cc + lo[e] * ss;
      }
      T* dst = k_cache + dst_row + h * head_dim;
      *reinterpret_cast<uint4*>(dst + c) = Vec<T>::pack(olo);
      *reinterpret_cast<uint4*>(dst + half + c) = Vec<T>::pack(ohi);
    } else {
      const int e0 = (i - k_items) * VN;
      const T* src = reinterpret_cast<const T*>(sg.v_src) + (size_t)j * row_elems + e0;
      T* dst = v_cache + dst_row + e0;
      if (src != dst) *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
    }
  }
}

template <typename T>
void launch_realign(const RealignSeg* d_segs, int32_t n_segs, int32_t total_rows, int32_t n_kv_heads, int32_t head_dim,
                    const float* rope_cos, const float* rope_sin, T* k_cache, T* v_cache, hipStream_t s) {
  if (total_rows <= 0 || n_segs <= 0) return;
  const int blocks = (total_rows + REALIGN_ROWS - 1) / REALIGN_ROWS;
  hipLaunchKernelGGL(k_realign<T>, dim3(blocks), dim3(256), 0, s, d_segs, n_segs, total_rows, n_kv_heads, head_dim,
                     rope_cos, rope_sin, k_cache, v_cache);
}

// ---------------------------------------------------------------------------
// RMSNorm:  y = x / sqrt(mean(x^2) + eps) * w
// ---------------------------------------------------------------------------
__device__ inline float block_sum_256(float v, float* s_red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) s_red[w] = v;
  __syncthreads();
  float t = s_red[0] + s_red[1] + s_red[2] + s_red[3];
  __syncthreads();
  return t;
}

template <typename T>
__global__ void __launch_bounds__(256) k_rmsnorm(const T* __restrict__ x, const T* __restrict__ w, int hidden, float eps,
                                                 T* __restrict__ y) {
  constexpr int VN = Vec<T>::N;
  __shared__ float s_red[4];
  const size_t base = (size_t)blockIdx.x * hidden;
  const int nv = hidden / VN;
  float ss = 0.f;
  for (int i = threadIdx.x; i < nv; i += 256) {
    float f[VN];
    Vec<T>::unpack(*reinterpret_cast<const uint4*>(x + base + (size_t)i * VN), f);
#pragma unroll
    for (int e = 0; e < VN; ++e) ss += f[e] * f[e];
  }
  const float tot = block_sum_256(ss, s_red);
  const float inv = 1.0f / sqrtf(tot / (float)hidden + eps);
  for (int i = threadIdx.x; i < nv; i += 256) {
    float f[VN], g[VN];
    Vec<T>::unpack(*reinterpret_cast<const uint4*>(x + base + (size_t)i * VN), f);
    Vec<T>::unpack(*reinterpret_cast<const uint4*>(w + (size_t)i * VN), g);
#pragma unroll
    for (int e = 0; e < VN; ++e) f[e] = f[e] * inv * g[e];
    *reinterpret_cast<uint4*>(y + base + (size_t)i * VN) = Vec<T>::pack(f);
  }
}

template <typename T>
void launch_rmsnorm(const T* x, const T* w, int32_t n_rows, int32_t hidden, float eps, T* y, hipStream_t s) {
  if (n_rows <= 0) return;
  hipLaunchKernelGGL(k_rmsnorm<T>, dim3(n_rows), dim3(256), 0, s, x, w, hidden, eps, y);
}

// ---------------------------------------------------------------------------
// bias + RoPE at the global position + scatter
//   q[r]            <- Rot(p_r)(q_raw + bq)
//   k_compact[r], K_hat[p_r] <- Rot(p_r)(k_raw + bk)
//   V_hat[p_r]      <- v_raw + bv
// qkv_raw is the fp32 output of the fused QKV GEMM, [n_rows, q_dim + 2 kv_dim].
// ---------------------------------------------------------------------------
template <typename T>
__device__ inline void store4(T* p, const float* f);
template <>
__device__ inline void store4<float>(float* p, const float* f) {
  *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
}
template <>
__device__ inline void store4<bf16_t>(bf16_t* p, const float* f) {
  uint2 u;
  u.x = pack_bf16x2(f[0], f[1]);
  u.y = pack_bf16x2(f[2], f[3]);
  *reinterpret_cast<uint2*>(p) = u;
}

// sum over 4 elements of (value as it will sit in the cache - value in the cache now)^2
template <typename T>
__device__ inline float sq_dist4(const T* old, const float* f);
template <>
__device__ inline float sq_dist4<float>(const float* old, const float* f) {
  const float4 o = *reinterpret_cast<const float4*>(old);
  const float d0 = f[0] - o.x, d1 = f[1] - o.y, d2 = f[2] - o.z, d3 = f[3] - o.w;
  return d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
}
template <>
__device__ inline float sq_dist4<bf16_t>(const bf16_t* old, const float* f) {
  const uint2 o = *reinterpret_cast<const uint2*>(old);
  const uint32_t n0 = pack_bf16x2(f[0], f[1]), n1 = pack_bf16x2(f[2], f[3]);  // the stored (rounded) new values
  const float d0 = __uint_as_float(n0 << 16) - __uint_as_float(o.x << 16);
  const float d1 = __uint_as_float(n0 & 0xffff0000u) - __uint_as_float(o.x & 0xffff0000u);
  const float d2 = __uint_as_float(n1 << 16) - __uint_as_float(o.y << 16);
  const float d3 = __uint_as_float(n1 & 0xffff0000u) - __uint_as_float(o.y & 0xffff0000u);
  return d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
}

template <typename T>
__global__ void __launch_bounds__(256)
    k_rope_scatter(const float* __restrict__ qkv_raw, const T* __restrict__ bq, const T* __restrict__ bk,
                   const T* __restrict__ bv, const int32_t* __restrict__ row_pos, const int32_t* __restrict__ row_lo,
                   int n_q_heads, int n_kv_heads, int head_dim, const float* __restrict__ rope_cos,
                   const float* __restrict__ rope_sin,
                   T* __restrict__ q, T* __restrict__ k_compact, T* __restrict__ k_cache, T* __restrict__ v_cache,
                   float* __restrict__ dev_out) {
  __shared__ float s_red[4];
  float dev = 0.f;  // squared distance of this thread's refreshed K/V elements from the cache rows they replace
  const int r = blockIdx.x;
  const int pos = row_pos[r];
  const int half = head_dim / 2;
  const int q_dim = n_q_heads * head_dim, kv_dim = n_kv_heads * head_dim;
  const int ld = q_dim + 2 * kv_dim;
  const float* raw = qkv_raw + (size_t)r * ld;
  const int per_head = half / 4;
  const int rot_items = (n_q_heads + n_kv_heads) * per_head;
  const int v_items = kv_dim / 4;
  // a unit cached on its own is rotated at its local positions: cache row minus the unit's first row
  const int rpos = pos - (row_lo ? row_lo[r] : 0);
  const float* cs = rope_cos + (size_t)rpos * half;
  const float* sn = rope_sin + (size_t)rpos * half;
  for (int it = threadIdx.x; it < rot_items + v_items; it += 256) {
    if (it < rot_items) {
      const int h = it / per_head, c = (it - h * per_head) * 4;
      const bool is_q = h < n_q_heads;
      const int col = is_q ? h * head_dim : q_dim + (h - n_q_heads) * head_dim;
      float4 a = *reinterpret_cast<const float4*>(raw + col + c);
      float4 b = *reinterpret_cast<const float4*>(raw + col + half + c);
      float lo[4] = {a.x, a.y, a.z, a.w}, hi[4] = {b.x, b.y, b.z, b.w};
      const T* bias = is_q ? bq : bk;
      if (bias) {
        const int bcol = is_q ? h * head_dim : (h - n_q_heads) * head_dim;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          lo[e] += ldf(bias + bcol + c + e);
          hi[e] += ldf(bias + bcol + half + c + e);
        }
      }
      float olo[4], ohi[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float cc = cs[c + e], ss = sn[c + e];
        olo[e] = lo[e] * cc - hi[e] * ss;
        ohi[e] = hi[e] * cc + lo[e] * ss;
      }
      if (is_q) {
        T* dst = q + (size_t)r * q_dim + h * head_dim;
        store4<T>(dst + c, olo);
        store4<T>(dst + half + c, ohi);
      } else {
        const int hk = h - n_q_heads;
        T* d1 = k_compact + (size_t)r * kv_dim + hk * head_dim;
        T* d2 = k_cache + (size_t)pos * kv_dim + hk * head_dim;
        if (dev_out) dev += sq_dist4<T>(d2 + c, olo) + sq_dist4<T>(d2 + half + c, ohi);
        store4<T>(d1 + c, olo);
        store4<T>(d1 + half + c, ohi);
        store4<T>(d2 + c, olo);
        store4<T>(d2 + half + c, ohi);
      }
    } else {
      const int c = (it - rot_items) * 4;
      float4 a = *reinterpret_cast<const float4*>(raw + q_dim + kv_dim + c);
      float f[4] = {a.x, a.y, a.z, a.w};
      if (bv) {
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] += ldf(bv + c + e);
      }
      if (dev_out) dev += sq_dist4<T>(v_cache + (size_t)pos * kv_dim + c, f);
      store4<T>(v_cache + (size_t)pos * kv_dim + c, f);
    }
  }
  if (dev_out) {  // (uniform branch: every thread of the block takes part in the sum)
    const float tot = block_sum_256(dev, s_red);
    if (threadIdx.x == 0) dev_out[r] = tot;
  }
}

template <typename T>
void launch_rope_scatter(const float* qkv_raw, const T* bq, const T* bk, const T* bv, const int32_t* d_row_pos,
                         int32_t n_rows, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                         const float* rope_cos, const float* rope_sin, T* q, T* k_compact, T* k_cache, T* v_cache,
                         hipStream_t s,
                         const int32_t* d_row_lo, float* d_deviation) {
  if (n_rows <= 0) return;
  hipLaunchKernelGGL(k_rope_scatter<T>, dim3(n_rows), dim3(256), 0, s, qkv_raw, bq, bk, bv, d_row_pos, d_row_lo,
                     n_q_heads, n_kv_heads, head_dim, rope_cos, rope_sin, q, k_compact, k_cache, v_cache, d_deviation);
}

// x_dst[r] = x_src[idx[r]] for r < n_rows_dst (rows of `width` elements, a multiple of the 16-byte vector)
template <typename T>
__global__ void k_rows_gather_list(const T* __restrict__ x_src, const int32_t* __restrict__ idx, int width,
                                   T* __restrict__ x_dst) {
  const int r = blockIdx.x;
  const uint4* src = reinterpret_cast<const uint4*>(x_src + (size_t)idx[r] * width);
  uint4* dst = reinterpret_cast<uint4*>(x_dst + (size_t)r * width);
  const int nv = width / Vec<T>::N;
  for (int i = threadIdx.x; i < nv; i += blockDim.x) dst[i] = src[i];
}

template <typename T>
void launch_rows_gather_list(const T* x_src, const int32_t* d_idx, int32_t n_rows_dst, int32_t width, T* x_dst,
                             hipStream_t s) {
  if (n_rows_dst <= 0) return;
  hipLaunchKernelGGL(k_rows_gather_list<T>, dim3(n_rows_dst), dim3(256), 0, s, x_src, d_idx, width, x_dst);
}

// Greedy choice over one row of logits: the largest value, the lowest index among equal ones.
// One workgroup; every thread scans a strided slice (ascending, so it keeps the first of equal
// values), then a fixed tree over (value, index) pairs.
__global__ void __launch_bounds__(1024) k_argmax(const float* __restrict__ logits, int n, int32_t* __restrict__ out) {
  __shared__ float s_v[1024];
  __shared__ int s_i[1024];
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = threadIdx.x; i < n; i += 1024) {
    const float v = logits[i];
    if (v > best || bi == 0x7fffffff) {
      best = v;
      bi = i;
    }
  }
  s_v[threadIdx.x] = best;
  s_i[threadIdx.x] = bi;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      const float v2 = s_v[threadIdx.x + w];
      const int i2 = s_i[threadIdx.x + w];
      const float v1 = s_v[threadIdx.x];
      const int i1 = s_i[threadIdx.x];
      if (i2 != 0x7fffffff && (i1 == 0x7fffffff || v2 > v1 || (v2 == v1 && i2 < i1))) {
        s_v[threadIdx.x] = v2;
        s_i[threadIdx.x] = i2;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = s_i[0];
}

void launch_argmax(const float* logits, int32_t n, int32_t* out, hipStream_t s) {
  hipLaunchKernelGGL(k_argmax, dim3(1), dim3(1024), 0, s, logits, n, out);
}

// explicit instantiations
#define INST(T)                                                                                                       \
  template void launch_embed_gather<T>(const T*, const int32_t*, const int32_t*, int32_t, int32_t, T*, hipStream_t); \
  template void launch_rows_gather<T>(const T*, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, T*,       \
                                      hipStream_t);                                                                   \
  template void launch_realign<T>(const RealignSeg*, int32_t, int32_t, int32_t, int32_t, const float*, const float*, \
                                  T*, T*, hipStream_t);                                                               \
  template void launch_rmsnorm<T>(const T*, const T*, int32_t, int32_t, float, T*, hipStream_t);                     \
  template void launch_rope_scatter<T>(const float*, const T*, const T*, const T*, const int32_t*, int32_t, int32_t, \
                                       int32_t, int32_t, const float*, const float*, T*, T*, T*, T*, hipStream_t,   \
                                       const int32_t*, float*);                                                      \
  template void launch_rows_gather_list<T>(const T*, const int32_t*, int32_t, int32_t, T*, hipStream_t);
INST(float)
INST(bf16_t)
#undef INST

}  // namespace keep
