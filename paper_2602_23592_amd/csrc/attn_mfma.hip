// Sparse-row causal attention over the joined cache on the gfx950 matrix cores
// (bf16 operands, fp32 accumulate, head_dim 128, grouped-query heads).
//
// Each of the n_rows recomputed rows attends to cache rows 0..p (its global position),
// whatever lies between the recomputed rows.  A workgroup owns one KV head and 128
// "query rows" (a recomputed row paired with one of the query heads of that KV head);
// each of its 4 waves owns 32 of them.  K/V tiles of 64 keys are staged through LDS
// (two buffers; the next tile streams global -> LDS while the current one is used).
//
// The scores are computed transposed, S^T = K . Q^T, so that a lane owns one query row
// (column l % 32 of the 32x32 MFMA result) and the keys sit in its registers: row max and
// row sum are register reductions plus one exchange between the two lane halves.  Those
// registers are, as they stand, the B operand of O^T = V^T . P^T; V^T's A operand comes
// straight from the row-major V tile through the LDS transpose read (ds_read_b64_tr_b16).
// The softmax statistics therefore stay per lane from the first tile to the final divide.
//
// Work list.  With few recomputed rows there are few (tile, KV head) pairs and the longest
// ones (instruction rows see the whole cache) would run alone on a few CUs.  The host
// therefore cuts long key ranges into chunks: a work item is (tile, key-tile range); items of
// a cut tile write un-normalised partial sums (fp32) with their running max and sum, and
// k_attn_combine merges them per row in chunk order (no atomics, reproducible).
#include <algorithm>
#include <vector>

#include "keep_internal.h"

namespace keep {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int DH = 128;
constexpr int KT_KEYS = 64;
constexpr int ATT_BUF = 2 * KT_KEYS * DH;  // elements per LDS buffer: K tile then V tile

typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ bf16x8 cat4(s16x4 a, s16x4 b) {
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}

constexpr float M_FLOOR = -1.0e30f;  // running max starts here (finite, so a fully masked tile gives alpha = 1, p = 0)
constexpr int PART_FLOATS = 128 * DH;  // partial O of one (item, KV head): [dh/4][q 128][4]

__global__ void __launch_bounds__(256, 2)
    k_attn_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k_cache, const bf16_t* __restrict__ v_cache,
                const int32_t* __restrict__ row_pos, const int32_t* __restrict__ row_lo,
                const int32_t* __restrict__ row_list, int n_rows, int n_total,
                int n_q_heads, int n_kv_heads, const int4* __restrict__ items, float scale_log2e,
                bf16_t* __restrict__ o, float* __restrict__ lse, float* __restrict__ part_o,
                float* __restrict__ part_ml) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, lq = lane & 31;
  const int rep = n_q_heads / n_kv_heads;
  const int hk = blockIdx.x % n_kv_heads;
  const int4 item = items[blockIdx.x / n_kv_heads];  // {tile, first key tile, end key tile, partial slot or -1}
  const int tile = item.x;
  const int QR = n_rows * rep;
  const int kv_dim = n_kv_heads * DH;

  // this lane's query row
  const int x = tile * 128 + wave * 32 + lq;
  const bool valid = x < QR;
  // n_rows counts the listed rows when a list is given: entry x / rep names the row of q / o / lse / row_pos
  const int r = valid ? (row_list ? row_list[x / rep] : x / rep) : 0;
  const int head = hk * rep + (valid ? x % rep : 0);
  const int pos = valid ? row_pos[r] : 0;
  const int lo = (valid && row_lo) ? row_lo[r] : 0;  // first key the row may see
  int wmax = pos, wmin = pos, wlo_max = lo, wlo_min = valid ? lo : 0x7fffffff;
#pragma unroll
  for (int off = 16; off > 0; off >>= 1) {
    wmax = max(wmax, __shfl_xor(wmax, off, 64));
    wmin = min(wmin, __shfl_xor(wmin, off, 64));
    wlo_max = max(wlo_max, __shfl_xor(wlo_max, off, 64));
    wlo_min = min(wlo_min, __shfl_xor(wlo_min, off, 64));
  }
  // (the butterflies cover 32 lanes; fold the two halves and keep the wave's bounds in scalar registers,
  // so that the tests on them below are uniform branches)
  wmax = __builtin_amdgcn_readfirstlane(max(wmax, __shfl_xor(wmax, 32, 64)));
  wmin = __builtin_amdgcn_readfirstlane(min(wmin, __shfl_xor(wmin, 32, 64)));
  wlo_max = __builtin_amdgcn_readfirstlane(max(wlo_max, __shfl_xor(wlo_max, 32, 64)));
  wlo_min = __builtin_amdgcn_readfirstlane(min(wlo_min, __shfl_xor(wlo_min, 32, 64)));
  const int kt0 = item.y, n_kt = item.z;

  // Q^T operand: 8 k-steps of 16 head-dim elements
  bf16x8 qf[8];
  {
    const bf16_t* qp = q + ((size_t)r * n_q_heads + head) * DH + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }

  f32x16 oacc[4];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[nt][e] = 0.f;
  float m_run = M_FLOOR, l_run = 0.f;

  // ---- LDS tiles: per buffer K [64 keys][256 B] then V [64 keys][256 B], no padding; 16-byte chunks are
  // XOR-swizzled so that operand reads are bank-conflict free: K chunk c of row r sits at c ^ (r % 16)
  // (16 consecutive rows x one 16-byte chunk = all 64 banks), V chunk c of row r at c ^ (4 (r % 4))
  // (a transpose read is served half a wave at a time: its 4 rows x 4 chunks then sit in 16 different chunks,
  // all 64 banks once; with a row term that moves rows by fewer than 4 chunks two rows share banks and every
  // V read takes twice as long, which the bank-conflict counter showed as a third of all LDS cycles).
  // Global -> LDS goes through global_load_lds_dwordx4 (lane l's 16 bytes land at base + 16 l, so one
  // instruction fills 4 rows); the swizzle is applied to the global address each lane fetches.
  typedef const void __attribute__((address_space(1))) * gptr_t;
  typedef void __attribute__((address_space(3))) * lptr_t;
  typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
  const int ld_row = wave * 16 + (lane >> 4);  // + 4 i, i < 4
  const int ld_pc = lane & 15;
#define ATT_STAGE(KT, BUFI)                                                                                     \
  {                                                                                                             \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                             \
      const int row_ = ld_row + 4 * i;                                                                          \
      const int key_ = min((KT) * KT_KEYS + row_, n_total - 1);                                                 \
      const size_t g_ = ((size_t)key_ * n_kv_heads + hk) * DH;                                                  \
      uint16_t* l_ = smem + (BUFI) * ATT_BUF + (wave * 16 + 4 * i) * DH;                                        \
      __builtin_amdgcn_global_load_lds((gptr_t)(k_cache + g_ + ((ld_pc ^ (row_ & 15)) << 3)), (lptr_t)l_, 16, 0, 0); \
      __builtin_amdgcn_global_load_lds((gptr_t)(v_cache + g_ + ((ld_pc ^ ((row_ & 3) << 2)) << 3)),             \
                                       (lptr_t)(l_ + KT_KEYS * DH), 16, 0, 0);                                  \
    }                                                                                                           \
  }
  // element offsets of this lane's operand chunks inside a tile
  int koff[8];  // K row lq, logical chunk 2 ks + g
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) koff[ks] = lq * DH + (((2 * ks + g) ^ (lq & 15)) << 3);
  int voff[4];  // V row 4 g + (lane % 16) / 4 of a 16-key step, 8 bytes of head-dim tile nt
  {
    const int vr = 4 * g + ((lane & 15) >> 2);
    const int cl = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) voff[nt] = vr * DH + (((4 * nt + cl) ^ ((vr & 3) << 2)) << 3) + 4 * (lane & 1);
  }

  ATT_STAGE(kt0, 0)
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tile has landed in LDS
  __syncthreads();

  for (int kt = kt0; kt < n_kt; ++kt) {
    const int cur = (kt - kt0) & 1;
    const int k0 = kt * KT_KEYS;
    // every wave finished reading the other buffer before the barrier that ended the last iteration
    if (kt + 1 < n_kt) ATT_STAGE(kt + 1, cur ^ 1)
    if (k0 <= wmax && k0 + KT_KEYS > wlo_min) {
      const uint16_t* sk = smem + cur * ATT_BUF;
      const uint16_t* sv = sk + KT_KEYS * DH;
      // ---- S^T = K . Q^T for the two 32-key halves; K operands are read four k-steps ahead
      f32x16 sacc[2];
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[st][e] = 0.f;
      bf16x8 kfa[4], kfb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) kfa[i] = *reinterpret_cast<const bf16x8*>(sk + koff[i]);
#pragma unroll
      for (int i = 0; i < 4; ++i) kfb[i] = *reinterpret_cast<const bf16x8*>(sk + koff[4 + i]);
#pragma unroll
      for (int i = 0; i < 4; ++i) sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfa[i], qf[i], sacc[0], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) kfa[i] = *reinterpret_cast<const bf16x8*>(sk + 32 * DH + koff[i]);
#pragma unroll
      for (int i = 0; i < 4; ++i) sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfb[i], qf[4 + i], sacc[0], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) kfb[i] = *reinterpret_cast<const bf16x8*>(sk + 32 * DH + koff[4 + i]);
#pragma unroll
      for (int i = 0; i < 4; ++i) sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfa[i], qf[i], sacc[1], 0, 0, 0);
      // V^T operands of the first 16-key step: in flight during the softmax arithmetic
      s16x4 vlo[2][4], vhi[2][4];
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        vlo[0][nt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(sv + voff[nt]));
        vhi[0][nt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(sv + 8 * DH + voff[nt]));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfb[i], qf[4 + i], sacc[1], 0, 0, 0);

      // ---- causal mask, running max (raw scores; the scale is folded into the exponent's fma)
      const bool need_mask = k0 + KT_KEYS - 1 > wmin || k0 < wlo_max;
      if (need_mask) {
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int key = k0 + st * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
            sacc[st][e] = (key <= pos && key >= lo) ? sacc[st][e] : -INFINITY;
          }
      }
      float tmax = -INFINITY;
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, sacc[st][e]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m_run, tmax * scale_log2e);  // log2 domain
      // rescale the running sums only when some row's max moved (after the first tiles it rarely does)
      if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[nt][e] *= alpha;
        m_run = m_new;
      }
      float psum = 0.f;
      uint32_t pk[2][8];
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[st][e], scale_log2e, -m_new));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[st][e + 1], scale_log2e, -m_new));
          psum += p0 + p1;
          pk[st][e >> 1] = pack_bf16x2(p0, p1);
        }
      l_run += psum;
      // ---- O^T += V^T . P^T : 4 k-steps of 16 keys, 4 head-dim tiles of 32; the V^T operands of step
      // s+1 are read while step s multiplies.  A operand slot (g, i) holds key base + 8*(i/4) + 4*g + i%4:
      // exactly the keys of P^T's registers, so P needs no shuffle.
#pragma unroll
      for (int step = 0; step < 4; ++step) {
        const int st = step >> 1, hh = step & 1, vc = step & 1, vn = vc ^ 1;
        if (step + 1 < 4) {
          const uint16_t* vb = sv + (step + 1) * 16 * DH;
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) {
            vlo[vn][nt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vb + voff[nt]));
            vhi[vn][nt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vb + 8 * DH + voff[nt]));
          }
        }
        u32x4 pu;
#pragma unroll
        for (int i = 0; i < 4; ++i) pu[i] = pk[st][hh * 4 + i];
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pu);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
          oacc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cat4(vlo[vc][nt], vhi[vc][nt]), pf, oacc[nt], 0, 0, 0);
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the next tile has landed
    __syncthreads();
  }
#undef ATT_STAGE

  // ---- finish: combine the two lane halves' sums, then either normalise and write O and LSE, or
  // (cut tile) store the un-normalised partial with its max and sum for k_attn_combine
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (item.w < 0) {
    if (valid) {
      const float inv = 1.0f / l_tot;
      bf16_t* op = o + ((size_t)r * n_q_heads + head) * DH;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int e = 0; e < 16; e += 4) {
          const int d = nt * 32 + 8 * (e >> 2) + 4 * g;
          uint2 u;
          u.x = pack_bf16x2(oacc[nt][e] * inv, oacc[nt][e + 1] * inv);
          u.y = pack_bf16x2(oacc[nt][e + 2] * inv, oacc[nt][e + 3] * inv);
          *reinterpret_cast<uint2*>(op + d) = u;
        }
      if (g == 0) lse[(size_t)r * n_q_heads + head] = 0.6931471805599453f * (m_run + log2f(l_tot));
    }
  } else if (valid) {  // rows past the end of the list are never read back
    const size_t slot = (size_t)item.w * n_kv_heads + hk;
    float* po = part_o + slot * PART_FLOATS;
    const int ql = wave * 32 + lq;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int e = 0; e < 16; e += 4) {
        const int d4 = (nt * 32 + 8 * (e >> 2) + 4 * g) >> 2;
        *reinterpret_cast<float4*>(po + ((size_t)d4 * 128 + ql) * 4) =
            make_float4(oacc[nt][e], oacc[nt][e + 1], oacc[nt][e + 2], oacc[nt][e + 3]);
      }
    if (g == 0) {
      part_ml[slot * 256 + ql] = m_run;
      part_ml[slot * 256 + 128 + ql] = l_tot;
    }
  }
}

// Merge the partials of one cut tile and one KV head, chunks in key order.  A thread owns one query row
// and 4 of the 128 output dimensions (blockIdx.y picks which), so that even a tile with a single valid
// row (decoding) spreads over 32 threads and the loop over chunks is a stream of independent loads.
__global__ void __launch_bounds__(256)
    k_attn_combine(const int4* __restrict__ splits, const float* __restrict__ part_o, const float* __restrict__ part_ml,
                   const int32_t* __restrict__ row_list, int n_rows, int n_q_heads, int n_kv_heads,
                   bf16_t* __restrict__ o, float* __restrict__ lse) {
  const int hk = blockIdx.x % n_kv_heads;
  const int4 sp = splits[blockIdx.x / n_kv_heads];  // {tile, first slot, chunks, -}
  const int rep = n_q_heads / n_kv_heads;
  const int ql = threadIdx.x & 127;
  const int d4 = blockIdx.y * 2 + (threadIdx.x >> 7);  // 0..31
  const int x = sp.x * 128 + ql;
  if (x >= n_rows * rep) return;
  const int r = row_list ? row_list[x / rep] : x / rep, head = hk * rep + x % rep;
  const float* ml = part_ml + ((size_t)sp.y * n_kv_heads + hk) * 256 + ql;
  const size_t ml_step = (size_t)n_kv_heads * 256;
  float m_all = M_FLOOR;
#pragma unroll 8
  for (int c = 0; c < sp.z; ++c) m_all = fmaxf(m_all, ml[c * ml_step]);
  float l_all = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* po = part_o + ((size_t)sp.y * n_kv_heads + hk) * PART_FLOATS + ((size_t)d4 * 128 + ql) * 4;
  const size_t po_step = (size_t)n_kv_heads * PART_FLOATS;
#pragma unroll 8
  for (int c = 0; c < sp.z; ++c) {
    const float w = __builtin_amdgcn_exp2f(ml[c * ml_step] - m_all);
    l_all += ml[c * ml_step + 128] * w;
    const float4 v = *reinterpret_cast<const float4*>(po + c * po_step);
    acc.x += w * v.x;
    acc.y += w * v.y;
    acc.z += w * v.z;
    acc.w += w * v.w;
  }
  const float inv = 1.0f / l_all;
  uint2 u;
  u.x = pack_bf16x2(acc.x * inv, acc.y * inv);
  u.y = pack_bf16x2(acc.z * inv, acc.w * inv);
  *reinterpret_cast<uint2*>(o + ((size_t)r * n_q_heads + head) * DH + d4 * 4) = u;
  if (d4 == 0) lse[(size_t)r * n_q_heads + head] = 0.6931471805599453f * (m_all + log2f(l_all));
}

// The same merge for tiles cut into many chunks (a few rows streaming a long cache: decoding, a short instruction
// over a reused prompt).  A workgroup of 512 threads owns 4 of the 128 output dimensions (blockIdx.y) of one cut
// tile and KV head; thread t takes query row t % 128 and every fourth chunk starting at t / 128, so that a load
// instruction reads the 16-byte entries of consecutive query rows (contiguous in the partial's [dh/4][row][4]
// layout) and four chunk streams are in flight at once; the four streams' maxima and weighted sums are joined
// through LDS in stream order (reproducible).
__global__ void __launch_bounds__(512)
    k_attn_combine_wide(const int4* __restrict__ splits, const float* __restrict__ part_o,
                        const float* __restrict__ part_ml, const int32_t* __restrict__ row_list, int n_rows,
                        int n_q_heads, int n_kv_heads, bf16_t* __restrict__ o, float* __restrict__ lse) {
  __shared__ float s_m[4][128];
  __shared__ float s_l[4][128];
  __shared__ float4 s_acc[4][128];
  const int hk = blockIdx.x % n_kv_heads;
  const int4 sp = splits[blockIdx.x / n_kv_heads];  // {tile, first slot, chunks, -}
  const int rep = n_q_heads / n_kv_heads;
  const int ql = threadIdx.x & 127, sub = threadIdx.x >> 7;
  const int d4 = blockIdx.y;  // 0..31
  const int x = sp.x * 128 + ql;
  const bool valid = x < n_rows * rep;
  const float* ml = part_ml + ((size_t)sp.y * n_kv_heads + hk) * 256 + ql;
  const size_t ml_step = (size_t)n_kv_heads * 256;
  float m_sub = M_FLOOR;
  if (valid) {
#pragma unroll 4
    for (int c = sub; c < sp.z; c += 4) m_sub = fmaxf(m_sub, ml[c * ml_step]);
  }
  s_m[sub][ql] = m_sub;
  __syncthreads();
  const float m_all = fmaxf(fmaxf(s_m[0][ql], s_m[1][ql]), fmaxf(s_m[2][ql], s_m[3][ql]));
  float l_sub = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (valid) {
    const float* po = part_o + ((size_t)sp.y * n_kv_heads + hk) * PART_FLOATS + ((size_t)d4 * 128 + ql) * 4;
    const size_t po_step = (size_t)n_kv_heads * PART_FLOATS;
#pragma unroll 4
    for (int c = sub; c < sp.z; c += 4) {
      const float w = __builtin_amdgcn_exp2f(ml[c * ml_step] - m_all);
      l_sub += ml[c * ml_step + 128] * w;
      const float4 v = *reinterpret_cast<const float4*>(po + c * po_step);
      acc.x += w * v.x;
      acc.y += w * v.y;
      acc.z += w * v.z;
      acc.w += w * v.w;
    }
  }
  s_l[sub][ql] = l_sub;
  s_acc[sub][ql] = acc;
  __syncthreads();
  if (sub != 0 || !valid) return;
  float l_all = s_l[0][ql];
  float4 a = s_acc[0][ql];
#pragma unroll
  for (int z = 1; z < 4; ++z) {
    l_all += s_l[z][ql];
    const float4 v = s_acc[z][ql];
    a.x += v.x;
    a.y += v.y;
    a.z += v.z;
    a.w += v.w;
  }
  const int r = row_list ? row_list[x / rep] : x / rep, head = hk * rep + x % rep;
  const float inv = 1.0f / l_all;
  uint2 u;
  u.x = pack_bf16x2(a.x * inv, a.y * inv);
  u.y = pack_bf16x2(a.z * inv, a.w * inv);
  *reinterpret_cast<uint2*>(o + ((size_t)r * n_q_heads + head) * DH + d4 * 4) = u;
  if (d4 == 0) lse[(size_t)r * n_q_heads + head] = 0.6931471805599453f * (m_all + log2f(l_all));
}

// The same merge for tiles with many chunks and very few query rows (decoding: one row, a handful of heads):
// 16 lanes share one (query row, 4 output dimensions) item and take the chunks 16 apart,
// so the partials of 16 chunks are in flight at once instead of one after the other; the lanes' maxima and
// weighted sums are joined by a fixed butterfly (reproducible).  blockIdx.y * 16 + threadIdx.x / 16 = item
// = query row * 32 + dimension group.
__global__ void __launch_bounds__(256)
    k_attn_combine_spread(const int4* __restrict__ splits, const float* __restrict__ part_o,
                        const float* __restrict__ part_ml, const int32_t* __restrict__ row_list, int n_rows,
                        int n_q_heads, int n_kv_heads, bf16_t* __restrict__ o, float* __restrict__ lse) {
  const int hk = blockIdx.x % n_kv_heads;
  const int4 sp = splits[blockIdx.x / n_kv_heads];  // {tile, first slot, chunks, -}
  const int rep = n_q_heads / n_kv_heads;
  const int item = blockIdx.y * 16 + (threadIdx.x >> 4);
  const int cl = threadIdx.x & 15;
  const int ql = item >> 5, d4 = item & 31;
  const int x = sp.x * 128 + ql;
  if (ql >= 128 || x >= n_rows * rep) return;  // (whole 16-lane groups leave together)
  const int r = row_list ? row_list[x / rep] : x / rep, head = hk * rep + x % rep;
  const float* ml = part_ml + ((size_t)sp.y * n_kv_heads + hk) * 256 + ql;
  const size_t ml_step = (size_t)n_kv_heads * 256;
  float m_all = M_FLOOR;
  for (int c = cl; c < sp.z; c += 16) m_all = fmaxf(m_all, ml[c * ml_step]);
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, off, 64));
  float l_all = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* po = part_o + ((size_t)sp.y * n_kv_heads + hk) * PART_FLOATS + ((size_t)d4 * 128 + ql) * 4;
  const size_t po_step = (size_t)n_kv_heads * PART_FLOATS;
  for (int c = cl; c < sp.z; c += 16) {
    const float w = __builtin_amdgcn_exp2f(ml[c * ml_step] - m_all);
    l_all += ml[c * ml_step + 128] * w;
    const float4 v = *reinterpret_cast<const float4*>(po + c * po_step);
    acc.x += w * v.x;
    acc.y += w * v.y;
    acc.z += w * v.z;
    acc.w += w * v.w;
  }
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) {
    l_all += __shfl_xor(l_all, off, 64);
    acc.x += __shfl_xor(acc.x, off, 64);
    acc.y += __shfl_xor(acc.y, off, 64);
    acc.z += __shfl_xor(acc.z, off, 64);
    acc.w += __shfl_xor(acc.w, off, 64);
  }
  if (cl != 0) return;
  const float inv = 1.0f / l_all;
  uint2 u;
  u.x = pack_bf16x2(acc.x * inv, acc.y * inv);
  u.y = pack_bf16x2(acc.z * inv, acc.w * inv);
  *reinterpret_cast<uint2*>(o + ((size_t)r * n_q_heads + head) * DH + d4 * 4) = u;
  if (d4 == 0) lse[(size_t)r * n_q_heads + head] = 0.6931471805599453f * (m_all + log2f(l_all));
}

// ---- host-side work list ---------------------------------------------------
constexpr int ATT_MAX_SLOTS = 4096;      // partial buffers (cut items x KV heads) the scratch can hold
constexpr int ATT_SLOTS = 512;           // resident workgroups: 2 per CU x 256 CUs
constexpr int ATT_MIN_CHUNK = 16;        // never cut below 16 key tiles (1024 keys) ...
constexpr int ATT_MIN_CHUNK_SMALL = 4;   // ... unless the whole launch is small (a few rows over a long cache)

static inline int att_max_tiles(int max_rows, int rep) { return (int)(((long)max_rows * rep + 127) / 128); }

size_t attn_mfma_stage_ints(int32_t max_rows, int32_t n_q_heads, int32_t n_kv_heads) {
  const int mt = att_max_tiles(max_rows, n_q_heads / n_kv_heads);
  return (size_t)4 * (mt + ATT_MAX_SLOTS) + (size_t)4 * mt;  // items then splits
}
size_t attn_mfma_scratch_bytes(int32_t max_rows, int32_t n_q_heads, int32_t n_kv_heads) {
  return attn_mfma_stage_ints(max_rows, n_q_heads, n_kv_heads) * sizeof(int32_t) + 256 +
         (size_t)ATT_MAX_SLOTS * (PART_FLOATS + 256) * sizeof(float);
}

// The two launches, given a work list that is already in d_scratch.
static void launch_attn_planned(const bf16_t* q, const bf16_t* k_cache, const bf16_t* v_cache, const int32_t* d_row_pos,
                                const int32_t* d_row_lo, const int32_t* d_row_list, int32_t n_rows, int32_t n_total, int32_t n_q_heads,
                                int32_t n_kv_heads, int32_t max_rows, void* d_scratch, int n_items, int n_splits,
                                bool wide_combine, bf16_t* o, float* lse, hipStream_t s) {
  const int rep = n_q_heads / n_kv_heads;
  const int mt = att_max_tiles(max_rows, rep);
  char* base = reinterpret_cast<char*>(d_scratch);
  int4* d_items = reinterpret_cast<int4*>(base);
  int4* d_splits = d_items + (mt + ATT_MAX_SLOTS);
  size_t off = attn_mfma_stage_ints(max_rows, n_q_heads, n_kv_heads) * sizeof(int32_t);
  off = (off + 255) & ~(size_t)255;
  float* part_o = reinterpret_cast<float*>(base + off);
  float* part_ml = part_o + (size_t)ATT_MAX_SLOTS * PART_FLOATS;
  const size_t sh = (size_t)2 * ATT_BUF * sizeof(uint16_t);
  static std::atomic<uint64_t> attr_done{0};
  set_max_dyn_smem_once(attr_done, reinterpret_cast<const void*>(k_attn_mfma), (int)sh);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)DH);
  hipLaunchKernelGGL(k_attn_mfma, dim3(n_items * n_kv_heads), dim3(256), sh, s, q, k_cache, v_cache, d_row_pos, d_row_lo,
                     d_row_list, n_rows, n_total, n_q_heads, n_kv_heads, d_items, scale_log2e, o, lse, part_o, part_ml);
  if (n_splits && wide_combine) {
    const int pairs = std::min(128, n_rows * rep);  // query rows of the fullest tile
    if (pairs < 32)  // too few rows to fill the row-major kernel's lanes: spread the chunks over lanes instead
      hipLaunchKernelGGL(k_attn_combine_spread, dim3(n_splits * n_kv_heads, (pairs * 32 + 15) / 16), dim3(256), 0, s,
                         d_splits, part_o, part_ml, d_row_list, n_rows, n_q_heads, n_kv_heads, o, lse);
    else
      hipLaunchKernelGGL(k_attn_combine_wide, dim3(n_splits * n_kv_heads, 32), dim3(512), 0, s, d_splits, part_o,
                         part_ml, d_row_list, n_rows, n_q_heads, n_kv_heads, o, lse);
  } else if (n_splits) {
    hipLaunchKernelGGL(k_attn_combine, dim3(n_splits * n_kv_heads, 16), dim3(256), 0, s, d_splits, part_o, part_ml,
                       d_row_list, n_rows, n_q_heads, n_kv_heads, o, lse);
  }
}

void launch_attn_mfma(const bf16_t* q, const bf16_t* k_cache, const bf16_t* v_cache, const int32_t* d_row_pos,
                      const int32_t* h_row_start, const int32_t* h_set_off, int32_t m, int32_t instr_off,
                      int32_t n_rows, int32_t n_total, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_rows,
                      int32_t* h_stage, void* d_scratch, bf16_t* o, float* lse, hipStream_t s,
                      const int32_t* h_row_lo, const int32_t* d_row_lo, AttnPlan* plan, const int32_t* h_row_list,
                      const int32_t* d_row_list, int32_t n_list, const int32_t* h_row_pos) {
  // With a row list only the listed rows (ascending ids into q / o / lse / row_pos) are attended; n_rows then
  // stands for the length of the list everywhere below.
  const int32_t n_all_rows = n_rows;
  (void)n_all_rows;
  if (h_row_list) n_rows = n_list;
  if (n_rows <= 0) return;
  if (plan && plan->valid) {  // same row layout as the launch that made the plan: the work list is on the device
    launch_attn_planned(q, k_cache, v_cache, d_row_pos, d_row_lo, d_row_list, n_rows, n_total, n_q_heads, n_kv_heads, max_rows,
                        d_scratch, plan->n_items, plan->n_splits, plan->wide_combine, o, lse, s);
    return;
  }
  const int rep = n_q_heads / n_kv_heads;
  const int n_tiles = (n_rows * rep + 127) / 128;
  const int mt = att_max_tiles(max_rows, rep);
  // key tiles each query tile needs: up to the position of its last row
  auto pos_of_row = [&](int r) {
    if (h_row_list) r = h_row_list[r];
    if (h_row_pos) return h_row_pos[r];  // the caller has the positions as a plain list (token rows)
    int lo = 0, hi = m;  // blocks 0..m
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (h_row_start[mid] <= r)
        lo = mid;
      else
        hi = mid - 1;
    }
    return (lo < m ? h_set_off[lo] : instr_off) + (r - h_row_start[lo]);
  };
  int4* h_items = reinterpret_cast<int4*>(h_stage);
  int4* h_splits = reinterpret_cast<int4*>(h_stage + (size_t)4 * (mt + ATT_MAX_SLOTS));
  long total_steps = 0;
  // steps of tile t are kept in h_splits[t].w for the second pass (overwritten afterwards is fine: separate array)
  // tile t needs the key tiles [first[t], steps[t]): from the first key its first row may see (0 unless
  // h_row_lo says otherwise; bounds do not decrease along the rows) to the position of its last row
  static thread_local std::vector<int> steps, first;
  steps.resize(n_tiles);
  first.resize(n_tiles);
  for (int t = 0; t < n_tiles; ++t) {
    const int x_last = std::min(n_rows * rep, (t + 1) * 128) - 1;
    steps[t] = pos_of_row(x_last / rep) / KT_KEYS + 1;
    first[t] = h_row_lo ? h_row_lo[(t * 128) / rep] / KT_KEYS : 0;
    total_steps += steps[t] - first[t];
  }
  // Two workgroups fit on each of the 256 CUs: 512 slots.  A key range longer than a slot's average
  // share of the work would leave the chip waiting for it at the end (instruction rows see the whole
  // cache while most recomputed memories sit early in the prompt), so such ranges are cut into chunks
  // of about that length (never below ATT_MIN_CHUNK key tiles); everything shorter runs whole.
  // A launch with less work than 16 key tiles per slot (decoding: one row over the whole cache) streams the
  // cache once and is bound by memory: it is cut finer (down to 4 key tiles), still into one round of items.
  const bool small = total_steps * n_kv_heads < (long)ATT_MIN_CHUNK * ATT_SLOTS;
  int chunk = (int)std::max<long>(small ? ATT_MIN_CHUNK_SMALL : ATT_MIN_CHUNK,
                                  (total_steps * n_kv_heads + ATT_SLOTS - 1) / ATT_SLOTS);
  for (;;) {
    long slots = 0;
    for (int t = 0; t < n_tiles; ++t) {
      const int nc = (steps[t] - first[t] + chunk - 1) / chunk;
      if (nc > 1) slots += nc;
    }
    if (slots * n_kv_heads <= ATT_MAX_SLOTS) break;
    chunk *= 2;
  }
  int n_items = 0, n_splits = 0, slot = 0;
  int min_steps = steps[0];
  for (int t = 1; t < n_tiles; ++t) min_steps = std::min(min_steps, steps[t]);
  if (!h_row_lo && n_tiles > 1 && (long)min_steps * 10 >= (long)steps[n_tiles - 1] * 9) {
    // Every query tile reads (nearly) the whole cache: a few instruction rows over a long prompt.  Items go
    // out chunk by chunk on one grid of key ranges, so the query tiles that read the same K/V range are
    // neighbours in the launch order, run at the same time on the XCD of their KV head and find the range
    // in its L2 instead of fetching it once per query tile.
    int max_nc = 1;
    static thread_local std::vector<int> slot_base;
    slot_base.resize(n_tiles);
    for (int t = n_tiles - 1; t >= 0; --t) {
      const int nc = (steps[t] + chunk - 1) / chunk;
      max_nc = std::max(max_nc, nc);
      slot_base[t] = -1;
      if (nc > 1) {
        h_splits[n_splits++] = make_int4(t, slot, nc, 0);
        slot_base[t] = slot;
        slot += nc;
      }
    }
    for (int c = 0; c < max_nc; ++c)
      for (int t = n_tiles - 1; t >= 0; --t) {
        if (c * chunk >= steps[t]) continue;
        h_items[n_items++] = make_int4(t, c * chunk, std::min(steps[t], (c + 1) * chunk),
                                       slot_base[t] < 0 ? -1 : slot_base[t] + c);
      }
  } else {
    for (int t = n_tiles - 1; t >= 0; --t) {  // longest key ranges first, each cut into equal pieces
      const int span = steps[t] - first[t];
      const int nc = (span + chunk - 1) / chunk;
      if (nc <= 1) {
        h_items[n_items++] = make_int4(t, first[t], steps[t], -1);
      } else {
        const int len = (span + nc - 1) / nc;
        h_splits[n_splits++] = make_int4(t, slot, nc, 0);
        for (int c = 0; c < nc; ++c)
          h_items[n_items++] = make_int4(t, first[t] + c * len, std::min(steps[t], first[t] + (c + 1) * len), slot + c);
        slot += nc;
      }
    }
  }
  char* base = reinterpret_cast<char*>(d_scratch);
  int4* d_items = reinterpret_cast<int4*>(base);
  int4* d_splits = d_items + (mt + ATT_MAX_SLOTS);
  // one upload: the item list, or (when tiles were cut) everything up to the end of the split list, which
  // sits behind the item area in both buffers
  (void)d_splits;
  const size_t up_bytes = n_splits ? ((size_t)(mt + ATT_MAX_SLOTS) + n_splits) * sizeof(int4) : (size_t)n_items * sizeof(int4);
  (void)hipMemcpyAsync(d_items, h_items, up_bytes, hipMemcpyHostToDevice, s);
  // tiles cut into many chunks are merged with the chunks spread over lanes
  bool wide = false;
  for (int i = 0; i < n_splits; ++i) wide |= h_splits[i].z >= 16;
  if (plan) {
    plan->valid = true;
    plan->n_items = n_items;
    plan->n_splits = n_splits;
    plan->wide_combine = wide;
  }
  launch_attn_planned(q, k_cache, v_cache, d_row_pos, d_row_lo, d_row_list, n_rows, n_total, n_q_heads, n_kv_heads,
                      max_rows, d_scratch, n_items, n_splits, wide, o, lse, s);
}

}  // namespace keep
