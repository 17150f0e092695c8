// Group-to-group attention scores on the matrix cores (bf16, head_dim 128).
//
//   mass[a, b] = sum over heads h, rows t of block a, keys s of block b, s <= t, of
//                exp(q_t,h . k_s / sqrt(dh) - lse[t, h])
//   S[a, b]    = mass / (heads * len_a * len_b),  S[a, a] = 0
//
// Rows (the recomputed tokens) and candidate keys (the recomputed memory tokens) are the
// same compact, position-ordered list, so the keys are read from the compact K buffer the
// QKV projection just wrote and causality is "key index <= row index".
//
// Pass 1 (MFMA): a wave owns a tile of <= 32 rows of ONE block and a chunk of 1024 keys.
// It forms S = Q . K^T tiles (lane = key column, registers = rows), turns them into
// probabilities with the rows' log-sum-exp and adds them over its rows and over all heads
// into per-key column sums kept in LDS; these go to colmass[tile, key].
// Pass 2: per (row tile, key block) sum of colmass over the block's keys (one wave, fixed
// butterfly).  Pass 3: per (a, b) sum over a's row tiles in order, then the division.
// No atomics anywhere: the result is reproducible bit for bit.
#include "keep_internal.h"

namespace keep {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int SDH = 128;
constexpr int S_KEYS = 64;      // keys per LDS tile
constexpr int S_CHUNK = 1024;   // keys per workgroup
constexpr int S_KSTRIDE = 136;  // bf16 per K row in LDS

struct RowTile {
  int32_t row0, nrows, slot;
};

static inline int32_t max_row_tiles(int32_t max_rows, int32_t max_groups) { return max_rows / 32 + max_groups + 2; }

size_t score_mfma_scratch_bytes(int32_t max_rows, int32_t max_groups) {
  const size_t rt = (size_t)max_row_tiles(max_rows, max_groups);
  size_t b = 0;
  b += (rt * 3 + (size_t)max_groups + 2) * sizeof(int32_t);  // tile table, tile_start per slot
  b = (b + 255) & ~(size_t)255;
  b += rt * (size_t)max_rows * sizeof(float);                // colmass
  b += rt * (size_t)(max_groups > 0 ? max_groups : 1) * sizeof(float);  // rtmass
  return b + 512;
}
size_t score_mfma_stage_ints(int32_t max_rows, int32_t max_groups) {
  return (size_t)max_row_tiles(max_rows, max_groups) * 3 + (size_t)max_groups + 2;
}

template <int CH>
__global__ void __launch_bounds__(256, 2)
    k_score_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc, const float* __restrict__ lse,
                 const RowTile* __restrict__ tiles, int n_rt, int n_keys, int n_q_heads, int n_kv_heads,
                 int hk_per_slice, float scale_log2e, float* __restrict__ colmass, int col_ld) {
  __shared__ __attribute__((aligned(16))) uint16_t s_k[2 * S_KEYS * S_KSTRIDE];
  __shared__ float s_col[4][S_CHUNK];
  __shared__ __attribute__((aligned(16))) float s_l2[4][CH][32];  // rows' log-sum-exp, log2 domain
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, lq = lane & 31;
  const int rep = n_q_heads / n_kv_heads;
  const int c0 = blockIdx.y * S_CHUNK;
  const int c1 = min(c0 + S_CHUNK, n_keys);
  // rows of the workgroup's last tile bound the keys that can be visible
  const int rt_last = min(n_rt, (int)blockIdx.x * 4 + 4) - 1;
  const int blk_last_row = tiles[rt_last].row0 + tiles[rt_last].nrows - 1;
  if (c0 > blk_last_row) return;
  const int key_end = min(c1, blk_last_row + 1);
  const int n_kt = (key_end - c0 + S_KEYS - 1) / S_KEYS;

  const int rt = blockIdx.x * 4 + wave;
  const bool has_tile = rt < n_rt;
  const RowTile tl = tiles[has_tile ? rt : rt_last];
  const int q_row = tl.row0 + min(lq, tl.nrows - 1);  // A operand row of this lane (clamped)
  const int tile_last_row = tl.row0 + tl.nrows - 1;

  for (int i = tid; i < 4 * S_CHUNK; i += 256) (&s_col[0][0])[i] = 0.f;

  const int ld_row = tid >> 4, ld_c = tid & 15;
  uint4 kreg0, kreg1, kreg2, kreg3;
  const int kv_dim = n_kv_heads * SDH;
#define SC_GLOAD1(KR, I, KT)                                                                     \
  {                                                                                              \
    const int key_ = min(c0 + (KT) * S_KEYS + ld_row + 16 * (I), n_keys - 1);                    \
    KR = *reinterpret_cast<const uint4*>(kc + (size_t)key_ * kv_dim + hk * SDH + ld_c * 8);      \
  }
#define SC_GLOAD(KT) SC_GLOAD1(kreg0, 0, KT) SC_GLOAD1(kreg1, 1, KT) SC_GLOAD1(kreg2, 2, KT) SC_GLOAD1(kreg3, 3, KT)
#define SC_SSTORE1(KR, I, BUFI) \
  *reinterpret_cast<uint4*>(&s_k[(BUFI) * S_KEYS * S_KSTRIDE + (ld_row + 16 * (I)) * S_KSTRIDE + ld_c * 8]) = KR;
#define SC_SSTORE(BUFI) SC_SSTORE1(kreg0, 0, BUFI) SC_SSTORE1(kreg1, 1, BUFI) SC_SSTORE1(kreg2, 2, BUFI) SC_SSTORE1(kreg3, 3, BUFI)

  // blockIdx.z selects a slice of the KV heads (small problems are spread over more workgroups;
  // the slices' column sums are added in slice order by the next pass)
  const int hk_begin = blockIdx.z * hk_per_slice;
  const int hk_end = min(n_kv_heads, hk_begin + hk_per_slice);
  for (int hk = hk_begin; hk < hk_end; ++hk) {
    for (int hc = 0; hc < rep; hc += CH) {
      const int nch = min(CH, rep - hc);  // heads in this pass (the last pass may be short)
      // Q operand for up to CH heads; the rows' log-sum-exp goes to LDS (+inf for rows past the tile's end)
      bf16x8 qf[CH][8];
#pragma unroll
      for (int j = 0; j < CH; ++j) {
        const int head = hk * rep + min(hc + j, rep - 1);
        const bf16_t* qp = q + ((size_t)q_row * n_q_heads + head) * SDH + g * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[j][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
      }
      __syncthreads();  // previous users of the K buffers and of s_l2 are done
      if (g == 0) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
          const int head = hk * rep + min(hc + j, rep - 1);
          s_l2[wave][j][lq] = (has_tile && lq < tl.nrows && j < nch)
                                  ? lse[(size_t)(tl.row0 + lq) * n_q_heads + head] * 1.4426950408889634f
                                  : INFINITY;
        }
      }
      SC_GLOAD(0)
      SC_SSTORE(0)
      __syncthreads();
      for (int kt = 0; kt < n_kt; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < n_kt) { SC_GLOAD(kt + 1) }
        const int k0 = c0 + kt * S_KEYS;
        if (has_tile && k0 <= tile_last_row) {
#pragma unroll
          for (int st = 0; st < 2; ++st) {
            const int key = k0 + st * 32 + lq;  // this lane's key column
            bf16x8 kf[8];
            const uint16_t* krow = &s_k[cur * S_KEYS * S_KSTRIDE + (st * 32 + lq) * S_KSTRIDE + g * 8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) kf[ks] = *reinterpret_cast<const bf16x8*>(krow + ks * 16);
            // only tiles that touch the diagonal (or the end of the key list) need the per-element test
            const bool need_mask = (k0 + S_KEYS - 1 > tl.row0) || (k0 + S_KEYS > n_keys);
            const bool key_ok = key < n_keys;
            float csum = 0.f;
#pragma unroll
            for (int j = 0; j < CH; ++j) {
              if (j >= nch) break;
              f32x16 acc;
#pragma unroll
              for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
              for (int ks = 0; ks < 8; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[j][ks], kf[ks], acc, 0, 0, 0);
#pragma unroll
              for (int e4 = 0; e4 < 4; ++e4) {
                // registers 4*e4 .. 4*e4+3 are rows 8*e4 + 4*g + {0..3} of the tile
                const float4 l4 = *reinterpret_cast<const float4*>(&s_l2[wave][j][8 * e4 + 4 * g]);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  const int row = tl.row0 + 8 * e4 + 4 * g + i;
                  const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[4 * e4 + i], scale_log2e, -lv[i]));
                  csum += (!need_mask || (key <= row && key_ok)) ? p : 0.f;
                }
              }
            }
            csum += __shfl_xor(csum, 32, 64);
            if (g == 0) s_col[wave][kt * S_KEYS + st * 32 + lq] += csum;
          }
        }
        if (kt + 1 < n_kt) { SC_SSTORE(cur ^ 1) }
        __syncthreads();
      }
    }
  }
#undef SC_GLOAD
#undef SC_GLOAD1
#undef SC_SSTORE
#undef SC_SSTORE1
  // column sums of this wave's row tile for the keys of the chunk
  if (has_tile) {
    float* dst = colmass + ((size_t)blockIdx.z * n_rt + rt) * col_ld + c0;
    for (int i = lane; i < key_end - c0; i += 64) dst[i] = s_col[wave][i];
  }
}

// rtmass[rt, b] = sum of colmass[rt, keys of block b that the tile can see], for b before the tile's block
__global__ void __launch_bounds__(256)
    k_score_rt_reduce(const float* __restrict__ colmass, int col_ld, int n_slices, const RowTile* __restrict__ tiles,
                      int n_rt, const int32_t* __restrict__ row_start, int m, float* __restrict__ rtmass) {
  const int lane = threadIdx.x & 63;
  const long w = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= (long)n_rt * m) return;
  const int rt = (int)(w / m), b = (int)(w % m);
  const RowTile tl = tiles[rt];
  float sum = 0.f;
  if (b < tl.slot) {
    const int last = tl.row0 + tl.nrows - 1;
    const int s0 = row_start[b], s1 = min(row_start[b + 1], last + 1);
    for (int z = 0; z < n_slices; ++z) {
      const float* src = colmass + ((size_t)z * n_rt + rt) * col_ld;
      for (int s = s0 + lane; s < s1; s += 64) sum += src[s];
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
  if (lane == 0) rtmass[(size_t)rt * m + b] = sum;
}

__global__ void k_score_finish_tiles(const float* __restrict__ rtmass, const int32_t* __restrict__ tile_start,
                                     const int32_t* __restrict__ row_start, int m, int n_q_heads,
                                     float* __restrict__ S) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  const int a = blockIdx.y;
  if (b >= m) return;
  float v = 0.f;
  if (b < a) {
    float sum = 0.f;
    for (int rt = tile_start[a]; rt < tile_start[a + 1]; ++rt) sum += rtmass[(size_t)rt * m + b];
    const float len_a = (float)(row_start[a + 1] - row_start[a]), len_b = (float)(row_start[b + 1] - row_start[b]);
    v = sum / ((float)n_q_heads * len_a * len_b);
  }
  S[(size_t)a * m + b] = v;
}

void launch_score_mfma(const bf16_t* q, const bf16_t* kc, const float* lse, const int32_t* h_row_start,
                       const int32_t* d_row_start, int32_t m, int32_t n_rows, int32_t n_q_heads, int32_t n_kv_heads,
                       int32_t* h_stage, void* d_scratch, int32_t max_rows, int32_t max_groups, float* S,
                       hipStream_t s) {
  if (m <= 0) return;
  // row tiles: <= 32 rows, never across a block boundary; blocks 0..m-1 memories, m the instruction
  const int32_t cap = max_row_tiles(max_rows, max_groups);
  RowTile* ht = reinterpret_cast<RowTile*>(h_stage);
  int32_t* h_tile_start = h_stage + (size_t)cap * 3;
  int n_rt = 0;
  for (int a = 0; a <= m; ++a) {
    h_tile_start[a] = n_rt;
    for (int t0 = h_row_start[a]; t0 < h_row_start[a + 1]; t0 += 32) {
      ht[n_rt].row0 = t0;
      ht[n_rt].nrows = std::min(32, h_row_start[a + 1] - t0);
      ht[n_rt].slot = a;
      ++n_rt;
    }
  }
  h_tile_start[m + 1] = n_rt;
  char* base = reinterpret_cast<char*>(d_scratch);
  RowTile* d_tiles = reinterpret_cast<RowTile*>(base);
  int32_t* d_tile_start = reinterpret_cast<int32_t*>(base) + (size_t)cap * 3;
  size_t off = ((size_t)cap * 3 + (size_t)max_groups + 2) * sizeof(int32_t);
  off = (off + 255) & ~(size_t)255;
  float* colmass = reinterpret_cast<float*>(base + off);
  float* rtmass = colmass + (size_t)cap * max_rows;
  (void)hipMemcpyAsync(d_tiles, ht, (size_t)n_rt * sizeof(RowTile), hipMemcpyHostToDevice, s);
  (void)hipMemcpyAsync(d_tile_start, h_tile_start, (size_t)(m + 2) * sizeof(int32_t), hipMemcpyHostToDevice, s);

  const int n_keys = h_row_start[m];
  const int rep = n_q_heads / n_kv_heads;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)SDH);
  // KV-head slices: as many as it takes to have ~1024 workgroups, within the column-sum scratch
  int n_slices = 1;
  const long base_blocks = (long)((n_rt + 3) / 4) * ((n_keys + S_CHUNK - 1) / S_CHUNK);
  while (n_slices < n_kv_heads && base_blocks * n_slices < 1024 && (long)(2 * n_slices) * n_rt <= cap &&
         n_kv_heads % (2 * n_slices) == 0)
    n_slices *= 2;
  const int hk_per_slice = n_kv_heads / n_slices;
  const dim3 grid((n_rt + 3) / 4, (n_keys + S_CHUNK - 1) / S_CHUNK, n_slices);
#define GO(CH)                                                                                                      \
  hipLaunchKernelGGL(k_score_mfma<CH>, grid, dim3(256), 0, s, q, kc, lse, d_tiles, n_rt, n_keys, n_q_heads,         \
                     n_kv_heads, hk_per_slice, scale_log2e, colmass, max_rows)
  // up to three query heads per pass keep two workgroups resident per CU (VALU of one overlaps MFMA of the other)
  if (rep >= 3)
    GO(3);
  else if (rep == 2)
    GO(2);
  else
    GO(1);
#undef GO
  const long waves = (long)n_rt * m;
  hipLaunchKernelGGL(k_score_rt_reduce, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, colmass, max_rows,
                     n_slices, d_tiles, n_rt, d_row_start, m, rtmass);
  hipLaunchKernelGGL(k_score_finish_tiles, dim3((m + 255) / 256, m + 1), dim3(256), 0, s, rtmass, d_tile_start,
                     d_row_start, m, n_q_heads, S);
}

}  // namespace keep
