// bf16 GEMM on the gfx950 matrix cores:  C[M,N] = A[M,K] . W[N,K]^T  (fp32 accumulate)
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_16x16x32_bf16 wants:
// lane l supplies 8 consecutive k of row (l % 16), k-block (l / 16).  (Of the two bf16 shapes this one
// sustains the higher rate under the chip's power limit: a register-only loop on random operands runs at
// 2.03 PFLOP/s against 1.78 PFLOP/s for 32x32x16, and the whole kernel gains 4 %; operand bytes read from
// LDS per flop are the same for both.)  A workgroup owns a
// BM x BN tile of C; K is walked in 64-deep slices staged through LDS (two buffers, one
// barrier per slice, next slice streamed global -> LDS by global_load_lds_dwordx4 while the
// current one is multiplied; operand fragments of the next step are read while a step multiplies).  LDS
// rows are 128 B; their 16-byte chunks are XOR-swizzled by the row index so that the
// 16-byte operand reads of consecutive rows spread over all banks.  Workgroups are mapped
// to tiles XCD by XCD so that the tiles resident on one XCD share slices through its L2.
//
// Epilogues: plain fp32 store, residual add (output and down projections),
// SwiGLU: the B tile interleaves rows of W_gate and W_up so that one lane holds
// gate[m, n] and up[m, n] in matching accumulator registers, and the fused QKV epilogue (bias, RoPE,
// compact q / k rows, scatter of K and V into the cache).
#include <algorithm>

#include "keep_internal.h"

namespace keep {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // 16-byte register vector (native, so arrays of it stay in VGPRs)

struct MfmaB {
  const bf16_t* ptr[3];
  int32_t begin[4];
  int32_t n_parts;
};

// Element offset of 16-byte chunk `chunk` of row `row` in a [rows][GBK] bf16 tile.  LDS has 64 four-byte
// banks (256 B per bank line); a row is GBK*2 bytes, so 256/(GBK*2) rows share a line.  The chunk index
// is XOR-ed with (row / rows-per-line) % chunks-per-row: 16 consecutive rows then cover all 64 banks
// exactly once for the 16-byte operand reads.
template <int GBK>
__device__ __forceinline__ int lds_off(int row, int chunk) {
  constexpr int CPR = GBK / 8, RPL = 128 / GBK;
  return row * GBK + ((chunk ^ ((row / RPL) & (CPR - 1))) << 3);
}

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
__device__ __forceinline__ constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

// Position t of the tile list -> tile coordinates: panels of GM tile rows, walked column by column.
template <int BM>
__device__ __forceinline__ void gemm_tile_of(int t, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
  constexpr int GM = (BM >= 256) ? 4 : 8;
  const int panel = t / (GM * tiles_n);
  const int panel_rows = min(GM, tiles_m - panel * GM);
  const int within = t - panel * GM * tiles_n;
  tile_m = panel * GM + within % panel_rows;
  tile_n = within / panel_rows;
}

template <int BM, int BN, int WM, int WN, int EPI, int GBK, int NST>
__global__ void __launch_bounds__(WM* WN * 64)
    k_gemm_mfma(const bf16_t* __restrict__ A, int M, int K, MfmaB B, const bf16_t* __restrict__ B2, int N,
                const bf16_t* __restrict__ residual, void* __restrict__ Cv, int tiles_m, int tiles_n,
                int full_per_xcd, int split_s, float* __restrict__ part, QkvEpilogue qe) {
  constexpr int T = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int MI = TM / 16, NI = TN / 16;  // 16x16 accumulator tiles per wave
  static_assert(NI % 4 == 0, "a wave's columns are walked in groups of four 16-column tiles");
  static_assert(EPI != EPI_SWIGLU_STORE || (NI % 2 == 0), "SwiGLU needs an even number of N tiles per wave");

  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int BUF = (BM + BN) * GBK;  // elements per buffer: A tile then B tile

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  // Workgroup -> tile.  Consecutive workgroup ids go round-robin to the 8 XCDs, each with its own L2.
  // XCD x therefore takes the x-th eighth of the tile list, and the list walks panels of GM tile rows
  // column by column, so the ~32 workgroups resident on one XCD cover a GM x (32/GM) patch of C and
  // share their A and B slices through that XCD's L2.
  //
  // The tail of each XCD's list, the tiles that would form a last, partly filled round of workgroups,
  // is cut along K instead: split_s workgroups share a tile, each multiplies its slice of K and writes
  // an fp32 partial tile; k_gemm_fixup adds the slices in order and applies the epilogue.
  const int n_tiles = tiles_m * tiles_n;
  const int per_xcd = (n_tiles + 7) >> 3;
  const int xcd = (int)(blockIdx.x & 7), j_x = (int)(blockIdx.x >> 3);
  int tl = j_x, piece = 0, pieces = 1;
  if (j_x >= full_per_xcd) {
    tl = full_per_xcd + (j_x - full_per_xcd) / split_s;
    piece = (j_x - full_per_xcd) % split_s;
    pieces = split_s;
  }
  const int t = xcd * per_xcd + tl;
  if (tl >= per_xcd || t >= n_tiles) return;
  int tile_m, tile_n;
  gemm_tile_of<BM>(t, tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;  // in B-tile rows (for SwiGLU: BN/2 output columns per block)

  // ---- global -> LDS staging without registers: global_load_lds_dwordx4 writes lane l's 16 bytes at
  // (wave-uniform LDS base) + 16 l, so one instruction fills 8 consecutive 128-byte tile rows.  The
  // XOR swizzle is applied on the global side: the lane whose bytes land in physical chunk pc of row r
  // fetches logical chunk pc ^ ((r / 2) % 8) of that row.
  constexpr int NW = WM * WN;
  constexpr int CPR = GBK / 8;      // 16-byte chunks per tile row
  constexpr int RPL = 128 / GBK;    // tile rows per 256-byte LDS bank line
  constexpr int RPI = 64 / CPR;     // tile rows filled by one wave-wide load instruction (1 KiB)
  constexpr int KS = GBK / 32;      // MFMA k-steps (32 deep) per slice
  constexpr int A_LD = BM / RPI / NW, B_LD = BN / RPI / NW;  // load instructions per wave per slice
  constexpr int LD = A_LD + B_LD;
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile rows must split evenly over the waves");
  typedef const void __attribute__((address_space(1))) * gptr_t;
  typedef void __attribute__((address_space(3))) * lptr_t;
  const bf16_t* a_src[A_LD];
  const bf16_t* b_src[B_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    const int r = (wave * A_LD + i) * RPI + lane / CPR, c = (lane % CPR) ^ ((r / RPL) & (CPR - 1));
    const int gm = min(m0 + r, M - 1);
    a_src[i] = A + (size_t)gm * K + c * 8;
  }
#pragma unroll
  for (int i = 0; i < B_LD; ++i) {
    const int r = (wave * B_LD + i) * RPI + lane / CPR, c = (lane % CPR) ^ ((r / RPL) & (CPR - 1));
    const bf16_t* row;
    if (EPI == EPI_SWIGLU_STORE) {
      // tile row r -> wave column block, gate/up half, column inside the half
      const int w = r / TN, within = r % TN, half = within / (TN / 2), col = within % (TN / 2);
      const int gn = (n0 / 2) + w * (TN / 2) + col;
      row = (half ? B2 : B.ptr[0]) + (size_t)gn * K;
    } else {
      const int gn = n0 + r;
      // (selects, not indexed loads: a dynamically indexed kernel-argument array goes to scratch)
      const bf16_t* base = B.ptr[0];
      int first = 0;
      if (B.n_parts > 1 && gn >= B.begin[1]) {
        base = B.ptr[1];
        first = B.begin[1];
      }
      if (B.n_parts > 2 && gn >= B.begin[2]) {
        base = B.ptr[2];
        first = B.begin[2];
      }
      row = base + (size_t)(gn - first) * K;
    }
    b_src[i] = row + c * 8;
  }
  // issue the loads of K-slice `slice` into LDS stage `stage`
#define GEMM_STAGE(slice, stage)                                                                               \
  {                                                                                                            \
    uint16_t* sa_ = smem + (stage) * BUF + (wave * A_LD) * RPI * GBK;                                          \
    uint16_t* sb_ = smem + (stage) * BUF + BM * GBK + (wave * B_LD) * RPI * GBK;                               \
    _Pragma("unroll") for (int i = 0; i < A_LD; ++i)                                                           \
        __builtin_amdgcn_global_load_lds((gptr_t)(a_src[i] + (size_t)(slice) * GBK), (lptr_t)(sa_ + i * RPI * GBK), 16, 0, 0); \
    _Pragma("unroll") for (int i = 0; i < B_LD; ++i)                                                           \
        __builtin_amdgcn_global_load_lds((gptr_t)(b_src[i] + (size_t)(slice) * GBK), (lptr_t)(sb_ + i * RPI * GBK), 16, 0, 0); \
  }

  // Fused QKV epilogue: once the K loop is over the operand tiles in LDS are dead, and the cos / sin rows of the
  // tile's BM rows (64 + 64 floats each, picked by the row's rotation position) are staged there, with the
  // rows' cache positions behind them, so that the epilogue's loads are LDS reads that no global store can
  // delay.  Wave w stages rows 32 w .. 32 w + 31; a load instruction fills two rows (lanes 0-15 / 32-47 the cos
  // chunks, lanes 16-31 / 48-63 the sin chunks).  Tiles that hold only value columns need no table.
#define QKV_STAGE_TABLES                                                                                          \
  {                                                                                                               \
    __syncthreads();                                                                                              \
    float* tab_ = reinterpret_cast<float*>(smem);                                                                 \
    int32_t* spos_ = reinterpret_cast<int32_t*>(smem) + BM * 128;                                                 \
    const int r_ = wave * (BM / NW) + (lane & 31);                                                                \
    const int gmr_ = min(m0 + r_, M - 1);                                                                         \
    const int p_ = qe.row_pos[gmr_];                                                                              \
    const int rp_ = p_ - (qe.row_lo ? qe.row_lo[gmr_] : 0);                                                       \
    if (lane < 32) {                                                                                              \
      spos_[r_] = p_;                                                                                             \
      spos_[BM + r_] = rp_;                                                                                       \
    }                                                                                                             \
    if (n0 < qe.q_dim + qe.kv_dim) {                                                                              \
      _Pragma("unroll") for (int i_ = 0; i_ < 16; ++i_) {                                                         \
        const int rp2_ = __shfl(rp_, 2 * i_ + (lane >> 5), 64);                                                   \
        const int ch_ = lane & 31;                                                                                \
        const float* src_ = (ch_ < 16 ? qe.rope_cos : qe.rope_sin) + (size_t)rp2_ * 64 + (ch_ & 15) * 4;          \
        __builtin_amdgcn_global_load_lds((gptr_t)src_, (lptr_t)(tab_ + (wave * (BM / NW) + 2 * i_) * 128), 16, 0, 0); \
      }                                                                                                           \
    }                                                                                                             \
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));                                                                     \
    __syncthreads();                                                                                              \
  }

  f32x4 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  // NST LDS stages: slices kt+1 .. kt+NST-1 are in flight (or landed) while slice kt is multiplied
  const int kt_begin = (int)((long)piece * (K / GBK) / pieces);
  const int KT = (int)((long)(piece + 1) * (K / GBK) / pieces);  // end of this workgroup's K slices
  // All NST stages are kept in flight: slice kt+NST is requested as soon as the barrier inside iteration kt
  // has shown that every wave is done reading the current stage (its last operands are in registers by
  // then), so the loads get NST-1 whole iterations to land.
#pragma unroll
  for (int p = 0; p < NST; ++p) GEMM_STAGE(min(kt_begin + p, KT - 1), p)
  __builtin_amdgcn_s_waitcnt(vmcnt_imm((NST - 1) * LD));  // slice 0 has landed in LDS
  __syncthreads();

  // A wave whose rows all lie past M (the last, partly filled row of tiles) has nothing to multiply: it keeps
  // doing its share of the staging and takes part in every barrier, but issues no operand reads and no MFMAs,
  // which leaves the SIMD's matrix pipe (and its power) to the wave it shares the SIMD with.
  if (m0 + wm * TM >= M) {
    int st_ = 0;
    for (int kt = kt_begin; kt < KT; ++kt) {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm((NST - 2) * LD));
      __syncthreads();
      GEMM_STAGE(min(kt + NST, KT - 1), st_)
      st_ = st_ + 1 == NST ? 0 : st_ + 1;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    if constexpr (EPI == EPI_QKV_ROPE) {
      if (pieces == 1) QKV_STAGE_TABLES  // (its two barriers are the workgroup's: every wave takes part)
    }
    return;
  }

  const int a_row0 = wm * TM + (lane & 15);
  const int b_row0 = wn * TN + (lane & 15);
  const int kg = lane >> 4;
  // LDS element offsets of this lane's operand chunks per k-step (rows differ by multiples of 16,
  // which leaves the swizzle term unchanged, so one offset per k-step serves every row tile)
  int a_off[KS], b_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    a_off[ks] = lds_off<GBK>(a_row0, ks * 4 + kg);
    b_off[ks] = BM * GBK + lds_off<GBK>(b_row0, ks * 4 + kg);
  }

  // A slice is walked in steps (k-step, group of four 16-column tiles): MI x 4 MFMAs each.  The A fragments
  // of a k-step serve all its groups; the B fragments of the next step (and, at the end of a k-step, the next
  // k-step's A fragments) are read while a step multiplies.
  constexpr int NG = NI / 4;        // column groups per k-step
  constexpr int STEPS = KS * NG;    // steps per slice
  static_assert(KS % 2 == 0, "the A fragments' two buffers alternate by k-step and must come out even over a slice");
  bf16x8 af[2][MI], bfr[2][4];
#pragma unroll
  for (int i = 0; i < MI; ++i) af[0][i] = *reinterpret_cast<const bf16x8*>(smem + a_off[0] + i * 16 * GBK);
#pragma unroll
  for (int j = 0; j < 4; ++j) bfr[0][j] = *reinterpret_cast<const bf16x8*>(smem + b_off[0] + j * 16 * GBK);

  int stage = 0;
  for (int kt = kt_begin; kt < KT; ++kt) {
    // (Past the end the last slice is fetched again into the stage just freed: harmless, and it keeps the
    // loop body one straight-line block for the instruction scheduler.)
    const int next_stage = stage + 1 == NST ? 0 : stage + 1;
    const uint16_t* cbuf = smem + stage * BUF;
    const uint16_t* nbuf = smem + next_stage * BUF;
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      const int ks = st / NG, g = st % NG;
      const int bc = st & 1, bn = bc ^ 1, ac = ks & 1, an = ac ^ 1;
      // (KS is even, so both buffer parities come out even over a slice and carry over to the next one)
      bool new_a;
      if (st + 1 < STEPS) {
        const int ks1 = (st + 1) / NG, g1 = (st + 1) % NG;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          bfr[bn][j] = *reinterpret_cast<const bf16x8*>(cbuf + b_off[ks1] + (g1 * 4 + j) * 16 * GBK);
        new_a = g1 == 0;
        if (new_a) {
#pragma unroll
          for (int i = 0; i < MI; ++i) af[an][i] = *reinterpret_cast<const bf16x8*>(cbuf + a_off[ks1] + i * 16 * GBK);
        }
      } else {
        // Last step of the slice: its operands are already in registers, so the workgroup waits for
        // slice kt+1 and synchronises BEFORE these MFMAs; the first operand reads of the next slice
        // are then in flight while they run.
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NST - 2) * LD));
        __syncthreads();
        GEMM_STAGE(min(kt + NST, KT - 1), stage)
#pragma unroll
        for (int j = 0; j < 4; ++j) bfr[bn][j] = *reinterpret_cast<const bf16x8*>(nbuf + b_off[0] + j * 16 * GBK);
#pragma unroll
        for (int i = 0; i < MI; ++i) af[an][i] = *reinterpret_cast<const bf16x8*>(nbuf + a_off[0] + i * 16 * GBK);
        new_a = true;
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][g * 4 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ac][i], bfr[bc][j], acc[i][g * 4 + j], 0, 0, 0);
      // interleave the operand reads issued above with the first half of the step's MFMAs (the second half
      // covers the latency of the last read)
      if (new_a) {
#pragma unroll
        for (int r = 0; r < 4 + MI; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
    }
    stage = next_stage;
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // no LDS write of this workgroup may outlive it

  // ---- epilogue.  acc[i][j][e]: row = i*16 + 4*(lane/16) + e, col = j*16 + lane%16
  const int col_l = lane & 15;
  const int row_l = 4 * (lane >> 4);
  if (pieces > 1) {  // partial tile [BM][BN] in tile coordinates
    const int rem_per_xcd = per_xcd - full_per_xcd;
    float* pt = part + ((size_t)(xcd * rem_per_xcd + (tl - full_per_xcd)) * split_s + piece) * (BM * BN);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = wm * TM + i * 16 + row_l + e;
#pragma unroll
        for (int j = 0; j < NI; ++j) pt[(size_t)r * BN + wn * TN + j * 16 + col_l] = acc[i][j][e];
      }
    return;
  }
  if constexpr (EPI == EPI_QKV_ROPE) {
    // The wave's TN = 128 columns are one head: query head, key head or value head by where they start.
    // RoPE pairs column c with c + 64: accumulator tiles j and j + 4, same lane, same register.
    static_assert(EPI != EPI_QKV_ROPE || (TN == 128 && NI == 8 && BM / NW == 32),
                  "the fused QKV epilogue needs one head per wave and 32 staged rows per wave");
    QKV_STAGE_TABLES
    const float* tab = reinterpret_cast<const float*>(smem);
    const int32_t* spos = reinterpret_cast<const int32_t*>(smem) + BM * 128;
    const int col0 = n0 + wn * TN;
    const int kind = col0 < qe.q_dim ? 0 : (col0 < qe.q_dim + qe.kv_dim ? 1 : 2);
    const int hcol = kind == 0 ? col0 : (kind == 1 ? col0 - qe.q_dim : col0 - qe.q_dim - qe.kv_dim);  // column inside q / k / v
    const bf16_t* bias = reinterpret_cast<const bf16_t*>(qe.bias[kind]);
    float bl[4] = {0.f, 0.f, 0.f, 0.f}, bh[4] = {0.f, 0.f, 0.f, 0.f};
    if (bias) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bl[j] = bf16_bits_to_f32(bias[hcol + j * 16 + col_l].bits);
        bh[j] = bf16_bits_to_f32(bias[hcol + 64 + j * 16 + col_l].bits);
      }
    }
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int rt = wm * TM + i * 16 + row_l + e;  // row inside the tile
        const int gm = m0 + rt;
        if (gm >= M) continue;
        const int pos = spos[rt];
        if (kind == 2) {
          bf16_t* dst = reinterpret_cast<bf16_t*>(qe.v_cache) + (size_t)pos * qe.kv_dim + hcol;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            dst[j * 16 + col_l].bits = f32_to_bf16_bits(acc[i][j][e] + bl[j]);
            dst[64 + j * 16 + col_l].bits = f32_to_bf16_bits(acc[i][j + 4][e] + bh[j]);
          }
        } else {
          const float* cs = tab + rt * 128;
          const float* sn = cs + 64;
          bf16_t* d1 = kind == 0 ? reinterpret_cast<bf16_t*>(qe.q) + (size_t)gm * qe.q_dim + hcol
                                 : reinterpret_cast<bf16_t*>(qe.k_compact) + (size_t)gm * qe.kv_dim + hcol;
          bf16_t* d2 = reinterpret_cast<bf16_t*>(qe.k_cache) + (size_t)pos * qe.kv_dim + hcol;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int c = j * 16 + col_l;
            const float lo = acc[i][j][e] + bl[j], hi = acc[i][j + 4][e] + bh[j];
            const float cc = cs[c], ss = sn[c];
            const uint16_t olo = f32_to_bf16_bits(lo * cc - hi * ss), ohi = f32_to_bf16_bits(hi * cc + lo * ss);
            d1[c].bits = olo;
            d1[64 + c].bits = ohi;
            if (kind == 1) {
              d2[c].bits = olo;
              d2[64 + c].bits = ohi;
            }
          }
        }
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int gm = m0 + wm * TM + i * 16 + row_l + e;
      if (gm >= M) continue;
      if (EPI == EPI_SWIGLU_STORE) {
        const int n_out = N;  // N = ffn_dim (output width)
#pragma unroll
        for (int j = 0; j < NI / 2; ++j) {
          const int gn = (n0 / 2) + wn * (TN / 2) + j * 16 + col_l;
          const float g = acc[i][j][e], u = acc[i][j + NI / 2][e];
          const float v = g / (1.0f + __expf(-g)) * u;
          reinterpret_cast<bf16_t*>(Cv)[(size_t)gm * n_out + gn].bits = f32_to_bf16_bits(v);
        }
      } else {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          const int gn = n0 + wn * TN + j * 16 + col_l;
          const size_t idx = (size_t)gm * N + gn;
          if (EPI == EPI_STORE_F32) {
            reinterpret_cast<float*>(Cv)[idx] = acc[i][j][e];
          } else {
            const float r = bf16_bits_to_f32(residual[idx].bits);
            reinterpret_cast<bf16_t*>(Cv)[idx].bits = f32_to_bf16_bits(r + acc[i][j][e]);
          }
        }
      }
    }
  }
}

#undef GEMM_STAGE
#undef QKV_STAGE_TABLES

// Epilogue of the tiles that were cut along K: partial slices added in slice order (reproducible).
template <int BM, int BN, int WM, int WN, int EPI>
__global__ void __launch_bounds__(256)
    k_gemm_fixup(const float* __restrict__ part, int M, int N, const bf16_t* __restrict__ residual,
                 void* __restrict__ Cv, int tiles_m, int tiles_n, int full_per_xcd, int split_s) {
  constexpr int TN = BN / WN;
  constexpr int OUT_N = EPI == EPI_SWIGLU_STORE ? BN / 2 : BN;  // output columns per tile
  const int n_tiles = tiles_m * tiles_n;
  const int per_xcd = (n_tiles + 7) >> 3;
  const int rem_per_xcd = per_xcd - full_per_xcd;
  const int xcd = blockIdx.x / rem_per_xcd, ri = blockIdx.x % rem_per_xcd;
  const int t = xcd * per_xcd + full_per_xcd + ri;
  if (t >= n_tiles) return;
  int tile_m, tile_n;
  gemm_tile_of<BM>(t, tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const float* pt = part + (size_t)blockIdx.x * split_s * (BM * BN);
  // one thread per 4 consecutive output columns of one row; the slices' loads are independent
  const int i = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (i >= BM * OUT_N) return;
  const int r = i / OUT_N, c = i % OUT_N;
  const int gm = m0 + r;
  if (gm >= M) return;
  if (EPI == EPI_SWIGLU_STORE) {
    // output column c of the tile: gate in tile column w*TN + col, up in w*TN + TN/2 + col
    const int w = c / (TN / 2), col = c % (TN / 2);
    const float* p = pt + (size_t)r * BN + w * TN + col;
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
#pragma unroll 4
    for (int z = 0; z < split_s; ++z) {
      const float4 gz = *reinterpret_cast<const float4*>(p + (size_t)z * (BM * BN));
      const float4 uz = *reinterpret_cast<const float4*>(p + (size_t)z * (BM * BN) + TN / 2);
      g.x += gz.x; g.y += gz.y; g.z += gz.z; g.w += gz.w;
      u.x += uz.x; u.y += uz.y; u.z += uz.z; u.w += uz.w;
    }
    uint2 o;
    o.x = pack_bf16x2(g.x / (1.0f + __expf(-g.x)) * u.x, g.y / (1.0f + __expf(-g.y)) * u.y);
    o.y = pack_bf16x2(g.z / (1.0f + __expf(-g.z)) * u.z, g.w / (1.0f + __expf(-g.w)) * u.w);
    *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(Cv) + (size_t)gm * N + n0 / 2 + c) = o;
  } else {
    const float* p = pt + (size_t)r * BN + c;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int z = 0; z < split_s; ++z) {
      const float4 v = *reinterpret_cast<const float4*>(p + (size_t)z * (BM * BN));
      a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    }
    const size_t idx = (size_t)gm * N + n0 + c;
    if (EPI == EPI_STORE_F32) {
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(Cv) + idx) = a;
    } else {
      const uint2 rv = *reinterpret_cast<const uint2*>(residual + idx);
      uint2 o;
      o.x = pack_bf16x2(bf16_bits_to_f32((uint16_t)(rv.x & 0xffff)) + a.x, bf16_bits_to_f32((uint16_t)(rv.x >> 16)) + a.y);
      o.y = pack_bf16x2(bf16_bits_to_f32((uint16_t)(rv.y & 0xffff)) + a.z, bf16_bits_to_f32((uint16_t)(rv.y >> 16)) + a.w);
      *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(Cv) + idx) = o;
    }
  }
}

// The same for the fused QKV epilogue: a thread owns 4 consecutive columns c.. of the low half of a head and their
// partners c + 64.. (RoPE pairs), of one row.
template <int BM, int BN>
__global__ void __launch_bounds__(256)
    k_gemm_fixup_qkv(const float* __restrict__ part, int M, int tiles_m, int tiles_n, int full_per_xcd, int split_s,
                     QkvEpilogue qe) {
  const int n_tiles = tiles_m * tiles_n;
  const int per_xcd = (n_tiles + 7) >> 3;
  const int rem_per_xcd = per_xcd - full_per_xcd;
  const int xcd = blockIdx.x / rem_per_xcd, ri = blockIdx.x % rem_per_xcd;
  const int t = xcd * per_xcd + full_per_xcd + ri;
  if (t >= n_tiles) return;
  int tile_m, tile_n;
  gemm_tile_of<BM>(t, tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const float* pt = part + (size_t)blockIdx.x * split_s * (BM * BN);
  constexpr int HEADS = BN / 128;               // heads per tile
  constexpr int ITEMS = BM * HEADS * 16;        // (row, head, group of 4 low columns)
  const int it = blockIdx.y * 256 + threadIdx.x;
  if (it >= ITEMS) return;
  const int r = it / (HEADS * 16), hh = (it / 16) % HEADS, c = (it % 16) * 4;
  const int gm = m0 + r;
  if (gm >= M) return;
  const float* p = pt + (size_t)r * BN + hh * 128 + c;
  float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
#pragma unroll 4
  for (int z = 0; z < split_s; ++z) {
    const float4 a = *reinterpret_cast<const float4*>(p + (size_t)z * (BM * BN));
    const float4 b = *reinterpret_cast<const float4*>(p + (size_t)z * (BM * BN) + 64);
    lo.x += a.x; lo.y += a.y; lo.z += a.z; lo.w += a.w;
    hi.x += b.x; hi.y += b.y; hi.z += b.z; hi.w += b.w;
  }
  float l4[4] = {lo.x, lo.y, lo.z, lo.w}, h4[4] = {hi.x, hi.y, hi.z, hi.w};
  const int col0 = n0 + hh * 128;
  const int kind = col0 < qe.q_dim ? 0 : (col0 < qe.q_dim + qe.kv_dim ? 1 : 2);
  const int hcol = kind == 0 ? col0 : (kind == 1 ? col0 - qe.q_dim : col0 - qe.q_dim - qe.kv_dim);
  const bf16_t* bias = reinterpret_cast<const bf16_t*>(qe.bias[kind]);
  if (bias) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      l4[e] += bf16_bits_to_f32(bias[hcol + c + e].bits);
      h4[e] += bf16_bits_to_f32(bias[hcol + 64 + c + e].bits);
    }
  }
  const int pos = qe.row_pos[gm];
  uint2 olo, ohi;
  if (kind == 2) {
    olo.x = pack_bf16x2(l4[0], l4[1]); olo.y = pack_bf16x2(l4[2], l4[3]);
    ohi.x = pack_bf16x2(h4[0], h4[1]); ohi.y = pack_bf16x2(h4[2], h4[3]);
    bf16_t* dst = reinterpret_cast<bf16_t*>(qe.v_cache) + (size_t)pos * qe.kv_dim + hcol;
    *reinterpret_cast<uint2*>(dst + c) = olo;
    *reinterpret_cast<uint2*>(dst + 64 + c) = ohi;
    return;
  }
  const int rpos = pos - (qe.row_lo ? qe.row_lo[gm] : 0);
  const float4 cs = *reinterpret_cast<const float4*>(qe.rope_cos + (size_t)rpos * 64 + c);
  const float4 sn = *reinterpret_cast<const float4*>(qe.rope_sin + (size_t)rpos * 64 + c);
  const float c4[4] = {cs.x, cs.y, cs.z, cs.w}, s4[4] = {sn.x, sn.y, sn.z, sn.w};
  float ol[4], oh[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    ol[e] = l4[e] * c4[e] - h4[e] * s4[e];
    oh[e] = h4[e] * c4[e] + l4[e] * s4[e];
  }
  olo.x = pack_bf16x2(ol[0], ol[1]); olo.y = pack_bf16x2(ol[2], ol[3]);
  ohi.x = pack_bf16x2(oh[0], oh[1]); ohi.y = pack_bf16x2(oh[2], oh[3]);
  bf16_t* d1 = kind == 0 ? reinterpret_cast<bf16_t*>(qe.q) + (size_t)gm * qe.q_dim + hcol
                         : reinterpret_cast<bf16_t*>(qe.k_compact) + (size_t)gm * qe.kv_dim + hcol;
  *reinterpret_cast<uint2*>(d1 + c) = olo;
  *reinterpret_cast<uint2*>(d1 + 64 + c) = ohi;
  if (kind == 1) {
    bf16_t* d2 = reinterpret_cast<bf16_t*>(qe.k_cache) + (size_t)pos * qe.kv_dim + hcol;
    *reinterpret_cast<uint2*>(d2 + c) = olo;
    *reinterpret_cast<uint2*>(d2 + 64 + c) = ohi;
  }
}

constexpr size_t GEMM_SPLIT_WS_BYTES = (size_t)256 * 256 * 256 * sizeof(float);  // 256 partial tiles of 256 x 256

template <int BM, int BN, int WM, int WN, int GBK, int NST>
static void launch_cfg(const bf16_t* A, int M, int K, const MfmaB& b, const bf16_t* B2, int N, int epilogue,
                       const bf16_t* residual, void* C, hipStream_t s, void* ws, const QkvEpilogue& qe) {
  // operand stages; the fused QKV epilogue re-uses them for BM rows of cos / sin (512 B each) and needs 2 BM
  // ints more for the rows' positions
  const size_t sh_ops = (size_t)NST * (BM + BN) * GBK * sizeof(uint16_t);
  const size_t sh = epilogue == EPI_QKV_ROPE ? std::max(sh_ops, (size_t)BM * 512) + (size_t)BM * 8 : sh_ops;
  const dim3 block(WM * WN * 64);
  const int n_tile_rows = epilogue == EPI_SWIGLU_STORE ? 2 * N : N;  // B-tile rows to cover
  const int tiles_n = n_tile_rows / BN, tiles_m = (M + BM - 1) / BM;
  const int per_xcd = (tiles_m * tiles_n + 7) / 8;
  // Workgroups resident per XCD (32 CUs): one per CU for the 256 x 256 tile (128 KB of LDS), two otherwise.
  // What would be a last, partly filled round is cut along K so that it fills the XCD once.
  const int slots = sh_ops > 80 * 1024 ? 32 : 64;
  int full = per_xcd, split = 1;
  if (ws && BM >= 128) {
    const int f = per_xcd / slots * slots, rem = per_xcd - f;
    if (rem > 0) {
      int sp = std::min(16, slots / rem);
      sp = std::min(sp, (K / GBK) / 4);  // at least four K slices per workgroup
      if (sp >= 2 && (size_t)8 * rem * sp * BM * BN * sizeof(float) <= GEMM_SPLIT_WS_BYTES) {
        full = f;
        split = sp;
      }
    }
  }
  const int rem = per_xcd - full;
  const dim3 grid(8 * (full + rem * split));
  float* part = reinterpret_cast<float*>(ws);
#define GO(E)                                                                                              \
  do {                                                                                                     \
    auto kern = k_gemm_mfma<BM, BN, WM, WN, E, GBK, NST>;                                                  \
    static std::atomic<uint64_t> attr_done{0};                                                             \
    set_max_dyn_smem_once(attr_done, reinterpret_cast<const void*>(kern), (int)sh);                        \
    hipLaunchKernelGGL(kern, grid, block, sh, s, A, M, K, b, B2, N, residual, C, tiles_m, tiles_n, full, split, part, qe); \
    if (split > 1 && E != EPI_QKV_ROPE)                                                                    \
      hipLaunchKernelGGL((k_gemm_fixup<BM, BN, WM, WN, E>), dim3(8 * rem, BM * BN / 1024), dim3(256), 0, s, part, M, N, \
                         residual, C, tiles_m, tiles_n, full, split);                                      \
  } while (0)
  if (epilogue == EPI_STORE_F32)
    GO(EPI_STORE_F32);
  else if (epilogue == EPI_RESIDUAL_STORE)
    GO(EPI_RESIDUAL_STORE);
  else if (epilogue == EPI_SWIGLU_STORE)
    GO(EPI_SWIGLU_STORE);
  else if constexpr (BN / WN == 128) {  // one head per wave
    GO(EPI_QKV_ROPE);
    if (split > 1)
      hipLaunchKernelGGL((k_gemm_fixup_qkv<BM, BN>), dim3(8 * rem, (BM * (BN / 128) * 16 + 255) / 256), dim3(256), 0, s,
                         part, M, tiles_m, tiles_n, full, split, qe);
  }
#undef GO
}

size_t gemm_ws_bytes() { return std::max(GEMM_SPLIT_WS_BYTES, gemm_skinny_ws_bytes()); }

// 256x256 tiles (8 waves, 64x128 each) unless the launch is so small that their start-up cost shows
// (fewer than ~10000 tile K-slices in all); 128x128 tiles then, and where the row counts are not
// multiples of 256.  A last, partly filled round of workgroups is cut along K in either case.
static bool big_tiles(int32_t M, int32_t K, const GemmB& B, int32_t rows) {
  int acc = 0;
  for (int p = 0; p < B.n_parts; ++p) {
    acc += B.n_rows[p];
    if (acc % 256) return false;
  }
  const long tiles256 = (long)((M + 255) / 256) * (rows / 256);
  return rows % 256 == 0 && tiles256 * (K / 64) >= 10000;
}

bool gemm_mfma_fuses_qkv(int32_t M, int32_t K, const GemmB& B, int32_t N, bool have_ws) {
  if (M <= 0 || N <= 0 || B.n_parts != 3) return false;
  if (have_ws && gemm_skinny_fits(M, K, B, N, EPI_STORE_F32)) return false;
  // every part a whole number of 128-column heads, so that a wave's columns never straddle q / k / v
  return big_tiles(M, K, B, N) && B.n_rows[0] % 128 == 0 && B.n_rows[1] % 128 == 0 && B.n_rows[2] % 128 == 0;
}

void launch_gemm_mfma(const bf16_t* A, int32_t M, int32_t K, const GemmB& B, const void* B2, int32_t N, int epilogue,
                      const bf16_t* residual, void* C, hipStream_t s, void* skinny_ws, const QkvEpilogue* qkv) {
  if (M <= 0 || N <= 0) return;
  if (epilogue != EPI_QKV_ROPE && skinny_ws && gemm_skinny_fits(M, K, B, N, epilogue)) {
    launch_gemm_skinny(A, M, K, B, B2, N, epilogue, residual, C, skinny_ws, s);
    return;
  }
  MfmaB b;
  b.n_parts = B.n_parts;
  int acc = 0;
  for (int p = 0; p < 3; ++p) {
    b.ptr[p] = p < B.n_parts ? reinterpret_cast<const bf16_t*>(B.ptr[p]) : nullptr;
    b.begin[p] = acc;
    if (p < B.n_parts) acc += B.n_rows[p];
  }
  b.begin[3] = acc;
  const bf16_t* b2 = reinterpret_cast<const bf16_t*>(B2);
  const int rows = epilogue == EPI_SWIGLU_STORE ? 2 * N : N;
  const QkvEpilogue qe = qkv ? *qkv : QkvEpilogue{};
  if (big_tiles(M, K, B, rows))
    launch_cfg<256, 256, 4, 2, 64, 2>(A, M, K, b, b2, N, epilogue, residual, C, s, skinny_ws, qe);
  else if (rows % 128 == 0)
    launch_cfg<128, 128, 2, 2, 64, 2>(A, M, K, b, b2, N, epilogue, residual, C, s, skinny_ws, qe);
  else
    launch_cfg<64, 64, 1, 1, 64, 2>(A, M, K, b, b2, N, epilogue, residual, C, s, skinny_ws, qe);
}

}  // namespace keep
