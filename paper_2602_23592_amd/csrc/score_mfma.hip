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
constexpr int S_CHUNK = 1024;   // keys per workgroup at most (launches with few row tiles take shorter chunks)

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

typedef const void __attribute__((address_space(1))) * sc_gptr_t;
typedef void __attribute__((address_space(3))) * sc_lptr_t;

struct ScoreWave {       // wave-uniform state of one row tile
  int row0, nrows, last_row;
  bool has_tile;
};

// One pass over the chunk's keys for NCH query heads of KV head hk (heads hk*rep + hc ...).
// K tiles stream global -> LDS with global_load_lds_dwordx4 (lane l's 16 bytes land at base + 16 l:
// one instruction fills 4 rows of 256 B).  Chunk c of row r is kept at c ^ (r % 16), which makes the
// 16-byte operand reads of 16 consecutive rows hit all 64 banks; the lane fetches the matching chunk.
template <int NCH>
__device__ __forceinline__ void score_pass(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc,
                                           const float* __restrict__ lse, uint16_t* s_k, float* s_colw, float* s_l2w,
                                           const ScoreWave sw, int q_row, int hk, int head0, int n_q_heads, int kv_dim,
                                           int c0, int n_kt, int n_keys, float scale_log2e) {
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, lq = lane & 31;
  const int ld_row = wave * 16 + (lane >> 4);  // + 4 i, i < 4
  const int ld_pc = lane & 15;
#define SC_STAGE(KT, BUFI)                                                                       \
  {                                                                                              \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                              \
      const int row_ = ld_row + 4 * i;                                                           \
      const int key_ = min(c0 + (KT) * S_KEYS + row_, n_keys - 1);                               \
      __builtin_amdgcn_global_load_lds(                                                          \
          (sc_gptr_t)(kc + (size_t)key_ * kv_dim + hk * SDH + ((ld_pc ^ (row_ & 15)) << 3)),     \
          (sc_lptr_t)(s_k + (BUFI) * S_KEYS * SDH + (wave * 16 + 4 * i) * SDH), 16, 0, 0);       \
    }                                                                                            \
  }
  int koff[8];  // K row lq, logical chunk 2 ks + g
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) koff[ks] = lq * SDH + (((2 * ks + g) ^ (lq & 15)) << 3);

  bf16x8 qf[NCH][8];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const bf16_t* qp = q + ((size_t)q_row * n_q_heads + head0 + j) * SDH + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[j][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }
  __syncthreads();  // previous users of the K buffers and of the log-sum-exp rows are done
  if (g == 0) {     // +inf for rows past the tile's end: their probabilities come out as 0
#pragma unroll
    for (int j = 0; j < NCH; ++j)
      s_l2w[j * 32 + lq] = (sw.has_tile && lq < sw.nrows)
                               ? lse[(size_t)(sw.row0 + lq) * n_q_heads + head0 + j] * 1.4426950408889634f
                               : INFINITY;
  }
  SC_STAGE(0, 0)
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tile has landed
  __syncthreads();
  for (int kt = 0; kt < n_kt; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < n_kt) SC_STAGE(kt + 1, cur ^ 1)
    const int k0 = c0 + kt * S_KEYS;
    if (sw.has_tile && k0 <= sw.last_row) {
      const uint16_t* sk = s_k + cur * S_KEYS * SDH;
      // only tiles that touch the diagonal (or the end of the key list) need the per-element test
      const bool need_mask = (k0 + S_KEYS - 1 > sw.row0) || (k0 + S_KEYS > n_keys);
      bf16x8 kf[8];  // K operands of a 32-key half
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) kf[ks] = *reinterpret_cast<const bf16x8*>(sk + koff[ks]);
      // The tile is 2 * NCH units (32-key half, head).  The MFMAs of unit u + 1 are issued between the
      // exponentials of unit u, so the matrix pipe and the vector ALU of this wave run side by side.
      // registers 4*e4 .. 4*e4+3 of a unit are its rows 8*e4 + 4*g + {0..3}
      constexpr int NU = 2 * NCH;
      f32x16 acc[2];
#define SC_ISSUE(UN)                                                                                          \
  {                                                                                                           \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) acc[(UN) & 1][e] = 0.f;                                    \
    _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) acc[(UN) & 1] =                                          \
        __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[(UN) % NCH][ks], kf[ks], acc[(UN) & 1], 0, 0, 0);          \
    if ((UN) == NCH - 1) { /* last use of the first half's operands: fetch the second half's */               \
      _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) kf[ks] =                                               \
          *reinterpret_cast<const bf16x8*>(sk + 32 * SDH + koff[ks]);                                         \
    }                                                                                                         \
  }
      SC_ISSUE(0)
      float csum = 0.f;
      if (!need_mask) {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
          const int j = u % NCH;
          if (u + 1 < NU) SC_ISSUE(u + 1)
          float4 l4[4];
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) l4[e4] = *reinterpret_cast<const float4*>(&s_l2w[j * 32 + 8 * e4 + 4 * g]);
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            csum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[u & 1][4 * e4 + 0], scale_log2e, -l4[e4].x));
            csum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[u & 1][4 * e4 + 1], scale_log2e, -l4[e4].y));
            csum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[u & 1][4 * e4 + 2], scale_log2e, -l4[e4].z));
            csum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[u & 1][4 * e4 + 3], scale_log2e, -l4[e4].w));
          }
          if (u + 1 < NU) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
              __builtin_amdgcn_sched_group_barrier(0x402, 6, 0);  // six vector ALU / transcendental
            }
          }
          if (j == NCH - 1) {  // all heads of this half are in: add the lane's key column to the chunk's sums
            csum += __shfl_xor(csum, 32, 64);
            if (g == 0) s_colw[kt * S_KEYS + (u / NCH) * 32 + lq] += csum;
            csum = 0.f;
          }
        }
      } else {
#pragma unroll
        for (int u = 0; u < NU; ++u) {
          const int j = u % NCH;
          if (u + 1 < NU) SC_ISSUE(u + 1)
          const int key = k0 + (u / NCH) * 32 + lq;  // this lane's key column
          // first tile-relative row that may see the key (none past the end of the key list)
          const int first = (key < n_keys ? key - sw.row0 : 64) - 4 * g;
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const float4 l4 = *reinterpret_cast<const float4*>(&s_l2w[j * 32 + 8 * e4 + 4 * g]);
            const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[u & 1][4 * e4 + i], scale_log2e, -lv[i]));
              csum += (8 * e4 + i >= first) ? p : 0.f;
            }
          }
          if (j == NCH - 1) {
            csum += __shfl_xor(csum, 32, 64);
            if (g == 0) s_colw[kt * S_KEYS + (u / NCH) * 32 + lq] += csum;
            csum = 0.f;
          }
        }
      }
#undef SC_ISSUE
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the next tile has landed
    __syncthreads();
  }
#undef SC_STAGE
}

template <int CH>
__global__ void __launch_bounds__(256, 2)
    k_score_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc, const float* __restrict__ lse,
                 const RowTile* __restrict__ tiles, int n_rt, int n_keys, int n_q_heads, int n_kv_heads,
                 int hk_per_slice, int chunk, float scale_log2e, float* __restrict__ colmass, int col_ld) {
  __shared__ __attribute__((aligned(16))) uint16_t s_k[2 * S_KEYS * SDH];
  __shared__ float s_col[4][S_CHUNK];
  __shared__ __attribute__((aligned(16))) float s_l2[4][CH * 32];  // rows' log-sum-exp, log2 domain
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31;
  const int rep = n_q_heads / n_kv_heads;
  const int c0 = blockIdx.y * chunk;
  const int c1 = min(c0 + chunk, n_keys);
  // rows of the workgroup's last tile bound the keys that can be visible
  const int rt_last = min(n_rt, (int)blockIdx.x * 4 + 4) - 1;
  const int blk_last_row = tiles[rt_last].row0 + tiles[rt_last].nrows - 1;
  if (c0 > blk_last_row) return;
  const int key_end = min(c1, blk_last_row + 1);
  const int n_kt = (key_end - c0 + S_KEYS - 1) / S_KEYS;

  const int rt = blockIdx.x * 4 + wave;
  ScoreWave sw;
  sw.has_tile = rt < n_rt;
  const RowTile tl = tiles[sw.has_tile ? rt : rt_last];
  sw.row0 = __builtin_amdgcn_readfirstlane(tl.row0);   // the tile is the wave's: keep it in scalar registers
  sw.nrows = __builtin_amdgcn_readfirstlane(tl.nrows);
  sw.last_row = sw.row0 + sw.nrows - 1;
  const int q_row = sw.row0 + min(lq, sw.nrows - 1);  // A operand row of this lane (clamped)

  for (int i = tid; i < 4 * chunk; i += 256) s_col[i / chunk][i % chunk] = 0.f;

  // blockIdx.z selects a slice of the KV heads (small problems are spread over more workgroups;
  // the slices' column sums are added in slice order by the next pass)
  const int kv_dim = n_kv_heads * SDH;
  const int hk_begin = blockIdx.z * hk_per_slice;
  const int hk_end = min(n_kv_heads, hk_begin + hk_per_slice);
  for (int hk = hk_begin; hk < hk_end; ++hk) {
    for (int hc = 0; hc < rep; hc += CH) {
      const int nch = min(CH, rep - hc);  // heads in this pass (the last pass may be short)
      const int head0 = hk * rep + hc;
      if (nch == CH)
        score_pass<CH>(q, kc, lse, s_k, s_col[wave], s_l2[wave], sw, q_row, hk, head0, n_q_heads, kv_dim, c0, n_kt,
                       n_keys, scale_log2e);
      else if (nch == 2)
        score_pass<2>(q, kc, lse, s_k, s_col[wave], s_l2[wave], sw, q_row, hk, head0, n_q_heads, kv_dim, c0, n_kt,
                      n_keys, scale_log2e);
      else
        score_pass<1>(q, kc, lse, s_k, s_col[wave], s_l2[wave], sw, q_row, hk, head0, n_q_heads, kv_dim, c0, n_kt,
                      n_keys, scale_log2e);
    }
  }
  // column sums of this wave's row tile for the keys of the chunk
  if (sw.has_tile) {
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
                                     float* __restrict__ S, int only_rows_with_tiles) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  const int a = blockIdx.y;
  if (b >= m) return;
  // rows of blocks that were left out of this pass keep what an earlier pass wrote
  if (only_rows_with_tiles && tile_start[a] == tile_start[a + 1]) return;
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
                       hipStream_t s, const uint8_t* h_want) {
  if (m <= 0) return;
  // row tiles: <= 32 rows, never across a block boundary; blocks 0..m-1 memories, m the instruction
  const int32_t cap = max_row_tiles(max_rows, max_groups);
  RowTile* ht = reinterpret_cast<RowTile*>(h_stage);
  int32_t* h_tile_start = h_stage + (size_t)cap * 3;
  // h_want (NULL = every block): the source blocks a whose rows S[a, .] are wanted.  The other blocks get no
  // row tiles and their rows of S are left as they are.  Everything that shapes the arithmetic (the slice
  // count below) is derived from the full tile count, so a row comes out bit-identical either way.
  int n_rt = 0, full_n_rt = 0;
  for (int a = 0; a <= m; ++a) {
    h_tile_start[a] = n_rt;
    full_n_rt += (h_row_start[a + 1] - h_row_start[a] + 31) / 32;
    if (h_want && !h_want[a]) continue;
    for (int t0 = h_row_start[a]; t0 < h_row_start[a + 1]; t0 += 32) {
      ht[n_rt].row0 = t0;
      ht[n_rt].nrows = std::min(32, h_row_start[a + 1] - t0);
      ht[n_rt].slot = a;
      ++n_rt;
    }
  }
  h_tile_start[m + 1] = n_rt;
  if (n_rt == 0) return;
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
  const long base_blocks = (long)((full_n_rt + 3) / 4) * ((n_keys + S_CHUNK - 1) / S_CHUNK);
  while (n_slices < n_kv_heads && base_blocks * n_slices < 1024 && (long)(2 * n_slices) * full_n_rt <= cap &&
         n_kv_heads % (2 * n_slices) == 0)
    n_slices *= 2;
  const int hk_per_slice = n_kv_heads / n_slices;
  // Keys per workgroup.  A key's column sum is formed by one wave over its rows and heads in a fixed order
  // whatever the chunk, so the chunk length shapes the launch only, never a result.  Every pass over a chunk
  // starts with exposed loads of the rows' Q, so long chunks are the efficient ones (measured: 256-key chunks
  // cost 20 % more time on a launch that fills the chip either way); shorter ones are taken only while the
  // workgroups with visible keys would not even occupy the chip once (a few hundred rows against a long
  // key list: 0.61 -> 0.18 ms for the 256 instruction rows of the 33 024-token workload).
  int chunk = S_CHUNK;
  for (; chunk > 2 * S_KEYS; chunk /= 2) {
    long active = 0;
    for (int x = 0; x < (n_rt + 3) / 4; ++x) {
      const RowTile& lt = ht[std::min(4 * x + 3, n_rt - 1)];
      active += std::min((n_keys + chunk - 1) / chunk, (lt.row0 + lt.nrows - 1) / chunk + 1);
    }
    if (active * n_slices >= 512) break;
  }
  const dim3 grid((n_rt + 3) / 4, (n_keys + chunk - 1) / chunk, n_slices);
#define GO(CH)                                                                                                      \
  hipLaunchKernelGGL(k_score_mfma<CH>, grid, dim3(256), 0, s, q, kc, lse, d_tiles, n_rt, n_keys, n_q_heads,         \
                     n_kv_heads, hk_per_slice, chunk, scale_log2e, colmass, max_rows)
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
                     d_row_start, m, n_q_heads, S, h_want ? 1 : 0);
}

}  // namespace keep
