// Internal declarations shared by the HIP translation units of libkeep_hip.so.
// Not part of the public ABI (that is include/keep.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "keep.h"

namespace keep {

// ---------------------------------------------------------------------------
// storage types
// ---------------------------------------------------------------------------
struct bf16_t {
  uint16_t bits;
};

__host__ __device__ inline float bf16_bits_to_f32(uint16_t b) {
  union {
    uint32_t u;
    float f;
  } c;
  c.u = (uint32_t)b << 16;
  return c.f;
}
// round-to-nearest-even; NaN stays NaN (quiet).  On the device this is the hardware conversion
// (v_cvt_pk_bf16_f32 on gfx950): no branches in the kernels' inner loops.
__host__ __device__ inline uint16_t f32_to_bf16_bits(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_bit_cast(uint16_t, (__bf16)f);
#else
  union {
    uint32_t u;
    float f;
  } c;
  c.f = f;
  if ((c.u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((c.u >> 16) | 0x0040u);
  c.u += 0x7fffu + ((c.u >> 16) & 1u);
  return (uint16_t)(c.u >> 16);
#endif
}
// two floats -> packed bf16 pair (low half = a)
__device__ inline uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ inline float ldf(const float* p) { return *p; }
__device__ inline float ldf(const bf16_t* p) { return bf16_bits_to_f32(p->bits); }
__device__ inline void stf(float* p, float v) { *p = v; }
__device__ inline void stf(bf16_t* p, float v) { p->bits = f32_to_bf16_bits(v); }

// Raises a kernel's dynamic shared-memory limit once per device (bit d of `done` = done on device d);
// safe when several host threads launch at the same time: a second call with the same value is harmless.
inline void set_max_dyn_smem_once(std::atomic<uint64_t>& done, const void* fn, int bytes) {
  int dev = 0;
  (void)hipGetDevice(&dev);
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return;
  (void)hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  done.fetch_or(bit, std::memory_order_release);
}

// ---------------------------------------------------------------------------
// per-layer row bookkeeping that lives on the device
// ---------------------------------------------------------------------------
// Segment of rows to re-align: one memory group outside the relevant set.
struct RealignSeg {
  const void* k_src;  // [len, Hkv, dh], rotated at local positions
  const void* v_src;
  int32_t dst_off;    // first global position
  int32_t len;
  int32_t row_start;  // prefix sum of len over the segments of this launch
  int32_t pad;
};

enum GemmEpilogue {
  EPI_STORE_F32 = 0,      // C (fp32) = acc
  EPI_RESIDUAL_STORE = 1, // C (T) = residual (T) + acc
  EPI_SWIGLU_STORE = 2,   // C (T) = silu(acc_gate) * acc_up   (B = gate rows, B2 = up rows)
  EPI_QKV_ROPE = 3,       // fused QKV projection: bias, RoPE at the row's position, q / compact k written, K and V
                          // scattered into the cache rows (matrix-core path, 256 x 256 tiles, head_dim 128)
};

// Where the fused QKV epilogue reads positions and writes its results (device pointers).
struct QkvEpilogue {
  const int32_t* row_pos;  // [M] cache row (global position) of each projected row
  const int32_t* row_lo;   // [M] or NULL: first row of the unit a row belongs to (rotation at pos - row_lo)
  const float* rope_cos;   // [positions, 64]
  const float* rope_sin;
  const void* bias[3];     // q, k, v biases or NULL
  void* q;                 // [M, q_dim]
  void* k_compact;         // [M, kv_dim]
  void* k_cache;           // [N, kv_dim]
  void* v_cache;
  int32_t q_dim, kv_dim;
};

// One B operand made of up to three row blocks stacked along N (Wq | Wk | Wv).
struct GemmB {
  const void* ptr[3];
  const void* bias[3];  // unused by the GEMM itself
  int32_t n_rows[3];
  int32_t n_parts;
  // INT4 form of the same parts (codes, scale/zero words) and of the second operand of the SwiGLU
  // epilogue; read instead of `ptr` by the launches that stream the weights (at most 48 rows)
  bool has_w4;
  const void* w4_codes[3];
  const void* w4_scale_zero[3];
  const void* w4_codes_b2;
  const void* w4_scale_zero_b2;
};

// ---------------------------------------------------------------------------
// launchers (every one validates nothing: api.hip checks shapes first)
// ---------------------------------------------------------------------------
// rows bookkeeping: row_pos[n_rows], row_slot[n_rows] from the set
void launch_build_rows(const int32_t* d_set_off /*[m] global offset of each selected group*/,
                       const int32_t* d_row_start /*[m+2] compact prefix, last two: instr start, n_rows*/,
                       int32_t m, int32_t instr_off, int32_t n_rows, int32_t* d_row_pos, int32_t* d_row_slot,
                       hipStream_t s);

template <typename T>
void launch_embed_gather(const T* embed, const int32_t* d_token_ids /*[N]*/, const int32_t* d_row_pos,
                         int32_t n_rows, int32_t hidden, T* x, hipStream_t s);
template <typename T>
void launch_rows_gather(const T* x_src, const int32_t* d_src_start /*[m'+1]*/, const int32_t* d_dst_start /*[m'+2]*/,
                        int32_t n_blocks_sel, int32_t n_rows_dst, int32_t hidden, T* x_dst, hipStream_t s);
template <typename T>
void launch_realign(const RealignSeg* d_segs, int32_t n_segs, int32_t total_rows, int32_t n_kv_heads,
                    int32_t head_dim, const float* rope_cos, const float* rope_sin, T* k_cache, T* v_cache,
                    hipStream_t s);
template <typename T>
void launch_rmsnorm(const T* x, const T* w, int32_t n_rows, int32_t hidden, float eps, T* y, hipStream_t s);
// bias + RoPE + write q/k/v compact + scatter K,V into the cache rows row_pos[]
template <typename T>
void launch_rope_scatter(const float* qkv_raw /*[n_rows, q_dim + 2 kv_dim]*/, const T* bq, const T* bk, const T* bv,
                         const int32_t* d_row_pos, int32_t n_rows, int32_t n_q_heads, int32_t n_kv_heads,
                         int32_t head_dim, const float* rope_cos, const float* rope_sin, T* q, T* k_compact,
                         T* k_cache, T* v_cache, hipStream_t s, const int32_t* d_row_lo = nullptr,
                         float* d_deviation = nullptr);
// d_deviation [n_rows] or NULL: per row, the squared distance between the refreshed K/V (as stored) and the
// cache rows they overwrite, summed in a fixed order (token-granularity selection).
template <typename T>
void launch_rows_gather_list(const T* x_src, const int32_t* d_idx, int32_t n_rows_dst, int32_t width, T* x_dst,
                             hipStream_t s);
// Token-granularity selection: the k of the n candidates with the largest deviation (ties: lower index), as an
// ascending list in d_list[0..k), followed by the n_tail indices n, n+1, ... (the instruction rows);
// d_flags: [n] scratch.
void launch_select_tokens(const float* d_deviation, int32_t n, int32_t k, int32_t n_tail, int32_t* d_flags,
                          int32_t* d_list, hipStream_t s);

// out[0] = index of the largest of logits[0..n), the lowest index among equal values
void launch_argmax(const float* logits, int32_t n, int32_t* out, hipStream_t s);

// generic (scalar FMA) kernels
template <typename T>
void launch_gemm_generic(const T* A, int32_t M, int32_t K, const GemmB& B, const void* B2, int32_t N, int epilogue,
                         const T* residual, void* C, hipStream_t s);
template <typename T>
void launch_attn_generic(const T* q, const T* k_cache, const T* v_cache, const int32_t* d_row_pos, int32_t n_rows,
                         int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, T* o, float* lse, hipStream_t s,
                         const int32_t* d_row_lo = nullptr);
// rowmass[t, j] = sum over heads and over the keys s of candidate j (compact rows
// key_start[j]..key_start[j+1]) with s <= t of exp(q_t.k_s/sqrt(dh) - lse[t,h])
template <typename T>
void launch_score_rows_generic(const T* q, const T* k_compact, const float* lse, const int32_t* d_row_start,
                               int32_t m, int32_t n_rows, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                               float* rowmass /*[n_rows, m]*/, hipStream_t s);
// S[(m+1), m] from rowmass: sum rows of each block in order, divide by heads*len_a*len_b, zero diagonal
void launch_score_finish(const float* rowmass, const int32_t* d_row_start, int32_t m, int32_t n_q_heads, float* S,
                         hipStream_t s);

// MFMA (bf16, head_dim 128) kernels
// skinny_ws: device scratch of gemm_ws_bytes(): partials of the weight-streaming kernel for launches of at
// most 48 rows, and of the tiles that are cut along K to fill the last round of workgroups.  NULL: neither.
size_t gemm_ws_bytes();
void launch_gemm_mfma(const bf16_t* A, int32_t M, int32_t K, const GemmB& B, const void* B2, int32_t N, int epilogue,
                      const bf16_t* residual, void* C, hipStream_t s, void* skinny_ws = nullptr,
                      const QkvEpilogue* qkv = nullptr);
// true where launch_gemm_mfma would run this QKV projection on 256 x 256 tiles, the configuration that has the
// fused epilogue (EPI_QKV_ROPE; a wave's 128 columns are one head); elsewhere the caller projects to fp32
// (EPI_STORE_F32) and runs the RoPE/scatter kernel.
bool gemm_mfma_fuses_qkv(int32_t M, int32_t K, const GemmB& B, int32_t N, bool have_ws);
// bf16 expansion of an INT4 matrix: out[rows, K] = bf16((code - zero) * scale)
void launch_dequant_int4(const void* codes, const void* scale_zero, int32_t rows, int32_t K, void* out, hipStream_t s);
size_t gemm_skinny_ws_bytes();
bool gemm_skinny_fits(int32_t M, int32_t K, const GemmB& B, int32_t N, int epilogue);
void launch_gemm_skinny(const bf16_t* A, int32_t M, int32_t K, const GemmB& B, const void* B2, int32_t N, int epilogue,
                        const bf16_t* residual, void* C, void* ws, hipStream_t s);
// h_row_start / h_set_off / m / instr_off: the host copy of the layer's row layout (as for
// launch_build_rows), from which the work list is planned; h_stage: pinned host ints
// (attn_mfma_stage_ints), d_scratch: device bytes (attn_mfma_scratch_bytes).
size_t attn_mfma_stage_ints(int32_t max_rows, int32_t n_q_heads, int32_t n_kv_heads);
size_t attn_mfma_scratch_bytes(int32_t max_rows, int32_t n_q_heads, int32_t n_kv_heads);
// A work list already uploaded to d_scratch: launches with the same row layout (the layers of one decode
// step) pass the same AttnPlan and skip the planning and the upload after the first.
struct AttnPlan {
  bool valid = false;
  int n_items = 0, n_splits = 0;
  bool wide_combine = false;  // some tile is cut into 16 or more chunks: merge with the chunks spread over lanes
};
void launch_attn_mfma(const bf16_t* q, const bf16_t* k_cache, const bf16_t* v_cache, const int32_t* d_row_pos,
                      const int32_t* h_row_start, const int32_t* h_set_off, int32_t m, int32_t instr_off,
                      int32_t n_rows, int32_t n_total, int32_t n_q_heads, int32_t n_kv_heads, int32_t max_rows,
                      int32_t* h_stage, void* d_scratch, bf16_t* o, float* lse, hipStream_t s,
                      const int32_t* h_row_lo = nullptr, const int32_t* d_row_lo = nullptr, AttnPlan* plan = nullptr,
                      const int32_t* h_row_list = nullptr, const int32_t* d_row_list = nullptr, int32_t n_list = 0,
                      const int32_t* h_row_pos = nullptr);
// h_row_pos: HOST [n_rows] positions of the rows (ascending), used for planning instead of the block layout
// (h_row_start / h_set_off / m / instr_off are then ignored).
// h_row_list / d_row_list (host and device copies) of n_list ascending row ids: attend only these rows.
// h_row_lo / d_row_lo (host and device copies, both or neither): first key each row may see (default 0);
// used where several units are cached in one pass, each attending to itself only.
// group-score matrix S[(m+1), m] of the layer whose q / compact k / lse are given.
// h_stage: pinned host ints (score_mfma_stage_ints of them), d_scratch: device bytes
// (score_mfma_scratch_bytes), both sized with the same max_rows / max_groups.
size_t score_mfma_scratch_bytes(int32_t max_rows, int32_t max_groups);
size_t score_mfma_stage_ints(int32_t max_rows, int32_t max_groups);
void launch_score_mfma(const bf16_t* q, const bf16_t* k_compact, const float* lse, const int32_t* h_row_start,
                       const int32_t* d_row_start, int32_t m, int32_t n_rows, int32_t n_q_heads, int32_t n_kv_heads,
                       int32_t* h_stage, void* d_scratch, int32_t max_rows, int32_t max_groups, float* S,
                       hipStream_t s, const uint8_t* h_want = nullptr);
// h_want: HOST [m + 1] flags or NULL: compute only the rows S[a, .] of the flagged source blocks (block m is
// the instruction); the other rows of S are left untouched.

// multi-hop selection on the device; d_out: [0] = n_next, [1] = hops_run, [2..] = slots kept (ascending)
void launch_select(const float* S, int32_t m, const int32_t* d_cand_len, int32_t k_count, int32_t token_budget,
                   int32_t mode, int32_t hops, float* d_work /*[(m+1)*m + 2m]*/, int32_t* d_iwork /*[4m]*/,
                   int32_t* d_out /*[m+2]*/, hipStream_t s, bool set_only = false,
                   const int32_t* d_cand_total = nullptr, const int32_t* d_id_map = nullptr);
// d_cand_total (device scalar or NULL): sum of d_cand_len; when given, the kernel itself settles budgets that
// keep all or none of the candidates (hops_run 0).  d_id_map (device [m] or NULL): ids written instead of slots.
// set_only: the propagation averages the normalised rows of the relevant set alone (the query's row
// only initialises the importance); default: the query stays a source at every hop.

}  // namespace keep
