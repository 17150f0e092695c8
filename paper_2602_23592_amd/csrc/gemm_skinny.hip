// Skinny GEMM for launches of a few rows, up to 64 (bf16 in, fp32 accumulate): C[M, N] = A[M, K] . B[N, K]^T.
//
// With so few rows the work is reading the weights once: the kernel is bound by HBM, not by the
// matrix cores.  It is used where a memory unit is cached on its own (Section 4.1: one dynamic
// segment of a few dozen tokens goes through all the projections of every layer).
//
// Work split: a workgroup owns 64 weight rows (output columns) and one of S slices of K; its four
// waves take the slice's 64-wide K steps round-robin.  Nothing is shared between waves, so operands
// go global -> registers directly (no LDS staging): a lane reads 64 contiguous bytes of one weight
// row and 64 of one activation row per step, the two half-waves together consume whole 128-byte
// lines.  Which K index feeds which MFMA slot is free as long as A and B agree, so the lane's 32
// K values are simply its four 16-byte chunks in order.  The four waves' partial tiles are added
// through LDS and written as fp32 partials [S][M][ld]; a second kernel adds the S slices in
// order (no atomics: reproducible) and applies the epilogue.  (Letting the workgroup that finishes a
// column tile last do that sum instead, found by a ticket counter, was measured and dropped: the
// device-wide release each workgroup then needs before it draws its ticket writes back the XCD's L2,
// which made a one-row launch 3x slower.)
#include <algorithm>

#include "keep_internal.h"

namespace keep {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct SkinnyB {
  const bf16_t* ptr[3];
  int32_t begin[4];  // first output column of each part; begin[n_parts] = total rows
};

constexpr int SK_BN = 64;       // weight rows per workgroup
constexpr int SK_KSTEP = 64;    // K per wave step
constexpr size_t SK_MAX_PART_FLOATS = (size_t)64 * 65536;  // capacity of the partials workspace

size_t gemm_skinny_ws_bytes() { return SK_MAX_PART_FLOATS * sizeof(float); }

struct SkinnyEpi {       // what the finishing pass needs
  int epilogue;          // GemmEpilogue
  int N;                 // output columns (SwiGLU: gate and up each have N)
  const bf16_t* residual;
  void* C;
};

// One output element from the S slices, summed in slice order.
__device__ __forceinline__ void skinny_store(const float* __restrict__ part, int n_splits, int ld, int M, int m, int n,
                                             const SkinnyEpi& e) {
  float s0 = 0.f, s1 = 0.f;
  for (int z = 0; z < n_splits; ++z) {
    const float* p = part + ((size_t)z * M + m) * ld;
    s0 += p[n];
    if (e.epilogue == EPI_SWIGLU_STORE) s1 += p[e.N + n];
  }
  const size_t idx = (size_t)m * e.N + n;
  if (e.epilogue == EPI_STORE_F32) {
    reinterpret_cast<float*>(e.C)[idx] = s0;
  } else if (e.epilogue == EPI_RESIDUAL_STORE) {
    reinterpret_cast<bf16_t*>(e.C)[idx].bits = f32_to_bf16_bits(bf16_bits_to_f32(e.residual[idx].bits) + s0);
  } else {
    reinterpret_cast<bf16_t*>(e.C)[idx].bits = f32_to_bf16_bits(s0 / (1.0f + __expf(-s0)) * s1);
  }
}

template <int MT>
__global__ void __launch_bounds__(256, 2)
    k_gemm_skinny(const bf16_t* __restrict__ A, int M, int K, SkinnyB B, int n_rows_b, int n_splits,
                  float* __restrict__ part, int ld) {
  __shared__ float s_red[4][MT * 32][SK_BN + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, lq = lane & 31;
  const int n0 = blockIdx.x * SK_BN;
  const int z = blockIdx.y;
  const int steps = K / SK_KSTEP;
  const int s_begin = (int)((long)z * steps / n_splits), s_end = (int)((long)(z + 1) * steps / n_splits);

  // this lane's weight rows (one per 32-column tile) and activation rows (one per 32-row tile)
  const bf16_t* bp[2];
#pragma unroll
  for (int ct = 0; ct < 2; ++ct) {
    const int n = min(n0 + ct * 32 + lq, n_rows_b - 1);
    const bf16_t* base = B.ptr[0];
    int first = 0;
    if (n >= B.begin[1]) { base = B.ptr[1]; first = B.begin[1]; }
    if (n >= B.begin[2]) { base = B.ptr[2]; first = B.begin[2]; }
    bp[ct] = base + (size_t)(n - first) * K + 32 * g;
  }
  const bf16_t* ap[MT];
#pragma unroll
  for (int rt = 0; rt < MT; ++rt) ap[rt] = A + (size_t)min(rt * 32 + lq, M - 1) * K + 32 * g;

  f32x16 acc[MT][2];
#pragma unroll
  for (int rt = 0; rt < MT; ++rt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[rt][ct][e] = 0.f;

  // B (the HBM stream) is double-buffered in registers; A comes from L2 and, with two row tiles, is
  // single-buffered: the second set of A registers would not fit beside 64 accumulators.
  constexpr int AB = MT == 1 ? 2 : 1;
  bf16x8 a[AB][MT][4], b[2][2][4];
#define SK_LOAD_B(BUF, STEP)                                                                           \
  {                                                                                                    \
    const int k_ = (STEP) * SK_KSTEP;                                                                  \
    _Pragma("unroll") for (int ct = 0; ct < 2; ++ct) _Pragma("unroll") for (int c = 0; c < 4; ++c)     \
        b[BUF][ct][c] = *reinterpret_cast<const bf16x8*>(bp[ct] + k_ + 8 * c);                         \
  }
#define SK_LOAD_A(BUF, STEP)                                                                           \
  {                                                                                                    \
    const int k_ = (STEP) * SK_KSTEP;                                                                  \
    _Pragma("unroll") for (int rt = 0; rt < MT; ++rt) _Pragma("unroll") for (int c = 0; c < 4; ++c)    \
        a[(BUF) % AB][rt][c] = *reinterpret_cast<const bf16x8*>(ap[rt] + k_ + 8 * c);                  \
  }
#define SK_MFMA(BUF)                                                                                   \
  {                                                                                                    \
    _Pragma("unroll") for (int c = 0; c < 4; ++c) _Pragma("unroll") for (int rt = 0; rt < MT; ++rt)    \
        _Pragma("unroll") for (int ct = 0; ct < 2; ++ct) acc[rt][ct] =                                 \
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(BUF) % AB][rt][c], b[BUF][ct][c], acc[rt][ct], 0, 0, 0); \
  }
  int st = s_begin + wave;
  if (st < s_end) {
    SK_LOAD_B(0, st)
    SK_LOAD_A(0, st)
  }
  while (st < s_end) {  // two steps per trip so that the register buffers keep fixed names
    if (st + 4 < s_end) {
      SK_LOAD_B(1, st + 4)
      if (AB == 2) SK_LOAD_A(1, st + 4)
    }
    SK_MFMA(0)
    st += 4;
    if (st >= s_end) break;
    if (AB == 1) SK_LOAD_A(1, st)
    if (st + 4 < s_end) {
      SK_LOAD_B(0, st + 4)
      if (AB == 2) SK_LOAD_A(0, st + 4)
    }
    SK_MFMA(1)
    st += 4;
    if (AB == 1 && st < s_end) SK_LOAD_A(0, st)
  }
#undef SK_LOAD_A
#undef SK_LOAD_B
#undef SK_MFMA

  // add the four waves' tiles.  acc[rt][ct][e]: row rt*32 + 8*(e/4) + 4*g + e%4, column ct*32 + lq
#pragma unroll
  for (int rt = 0; rt < MT; ++rt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int e = 0; e < 16; ++e) s_red[wave][rt * 32 + 8 * (e >> 2) + 4 * g + (e & 3)][ct * 32 + lq] = acc[rt][ct][e];
  __syncthreads();
  float* dst = part + (size_t)z * M * ld;
  for (int i = tid; i < MT * 32 * SK_BN; i += 256) {
    const int r = i / SK_BN, cidx = i % SK_BN;
    const float v = (s_red[0][r][cidx] + s_red[1][r][cidx]) + (s_red[2][r][cidx] + s_red[3][r][cidx]);
    if (r < M && n0 + cidx < n_rows_b) dst[(size_t)r * ld + n0 + cidx] = v;
  }
}

// C = epilogue(sum over the K slices, in slice order)
__global__ void __launch_bounds__(256)
    k_skinny_finish(const float* __restrict__ part, int n_splits, int ld, int M, SkinnyEpi e) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  const int m = blockIdx.y;
  if (n >= e.N || m >= M) return;
  skinny_store(part, n_splits, ld, M, m, n, e);
}

// ---------------------------------------------------------------------------------------------
// INT4 weight-only variant (Section 6.1: the 32B model runs with INT4 weight-only quantisation).
// The weights the model computes with are  w = bf16((q - z) * s)  per group of 128 input features
// (codes q and zero z of 4 bits, scale s in bf16).  Launches of a few dozen rows are bound by
// reading the weights, so they read the 4-bit form (a quarter of the bytes) and expand it in
// registers to exactly those bf16 values; launches with many rows are bound by the matrix cores
// and use a bf16 copy expanded once by k_dequant_int4.
//
// Storage (rows a multiple of 32): codes in blocks of 32 rows x 128 features, ordered by (row block, feature
// group), 2048 bytes each; inside a block 64 bytes per row; within a run of 8 features byte t holds feature t
// (low nibble) and feature t + 4 (high nibble).  One 32-bit word per (row, group): scale bits | zero << 16,
// in the same block order, 32 words per block.  A wave step of the GEMM below reads one such block per row
// tile: one contiguous 2 KB request for the codes, one 128-byte request for the words.
// ---------------------------------------------------------------------------------------------
constexpr int W4_GROUP = 128;
constexpr int W4_ROWS = 32;                          // rows per storage block
constexpr int W4_BLOCK_BYTES = W4_ROWS * W4_GROUP / 2;  // 2048

// Eight weights of one code word -> 8 bf16 (4 packed words), in feature order.
// (q - z) * s has <= 13 significant bits, so fma(q, s, -z*s) is exact and the only rounding is the
// conversion to bf16 (round to nearest even).
// byte N of a word as a float (v_cvt_f32_ubyteN: the shift, the mask and the conversion in one instruction)
#define W4_UBYTE(N, DST, SRC) asm("v_cvt_f32_ubyte" #N " %0, %1" : "=v"(DST) : "v"(SRC))
__device__ __forceinline__ void w4_expand8(uint32_t d, float sc, float nzs, uint32_t out[4]) {
  const uint32_t lo = d & 0x0F0F0F0Fu, hi = (d >> 4) & 0x0F0F0F0Fu;  // features 0..3 and 4..7 as bytes
  float f[8];
  W4_UBYTE(0, f[0], lo); W4_UBYTE(1, f[1], lo); W4_UBYTE(2, f[2], lo); W4_UBYTE(3, f[3], lo);
  W4_UBYTE(0, f[4], hi); W4_UBYTE(1, f[5], hi); W4_UBYTE(2, f[6], hi); W4_UBYTE(3, f[7], hi);
#pragma unroll
  for (int t = 0; t < 8; ++t) f[t] = __builtin_fmaf(f[t], sc, nzs);
#pragma unroll
  for (int t = 0; t < 4; ++t) out[t] = pack_bf16x2(f[2 * t], f[2 * t + 1]);
}
#undef W4_UBYTE

__device__ __forceinline__ void w4_scale_zero(uint32_t word, float& sc, float& nzs) {
  sc = __uint_as_float(word << 16);
  nzs = -(float)((word >> 16) & 0xFu) * sc;  // exact: 4 bits times 8 bits
}

// one code word (8 features of one row) per thread, in storage order
__global__ void __launch_bounds__(256)
    k_dequant_int4(const uint32_t* __restrict__ codes, const uint32_t* __restrict__ scale_zero, long n_words,
                   int groups, int K, uint4* __restrict__ out) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_words) return;
  const long block = i / (W4_BLOCK_BYTES / 4);                 // (row block, group)
  const int within = (int)(i - block * (W4_BLOCK_BYTES / 4));  // word inside the block: row * 16 + run of 8
  const int r = within >> 4, run = within & 15;
  const long rb = block / groups;
  const int kg = (int)(block - rb * groups);
  float sc, nzs;
  w4_scale_zero(scale_zero[block * W4_ROWS + r], sc, nzs);
  uint32_t o[4];
  w4_expand8(codes[i], sc, nzs, o);
  const size_t row = (size_t)rb * W4_ROWS + r;
  out[(row * K + (size_t)kg * W4_GROUP + 8 * run) / 8] = make_uint4(o[0], o[1], o[2], o[3]);
}

void launch_dequant_int4(const void* codes, const void* scale_zero, int32_t rows, int32_t K, void* out, hipStream_t s) {
  const long n_words = (long)rows * (K / 8);
  if (n_words <= 0) return;
  hipLaunchKernelGGL(k_dequant_int4, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<const uint32_t*>(codes), reinterpret_cast<const uint32_t*>(scale_zero), n_words,
                     K / W4_GROUP, K, reinterpret_cast<uint4*>(out));
}

struct SkinnyW4 {
  const uint8_t* codes[3];
  const uint32_t* sz[3];
  int32_t begin[4];  // first output column of each part; unused parts never match
};

// Same work split as k_gemm_skinny, but a wave step covers one quantisation group (128 input features):
// the half-wave g reads the 32 code bytes of features 64 g .. 64 g + 63 of each of its two weight rows
// (two 16-byte loads per row) and one scale/zero word per row; a row tile's 32 rows are one storage block.
template <int MT>
__global__ void __launch_bounds__(256, 2)
    k_gemm_skinny_w4(const bf16_t* __restrict__ A, int M, int K, SkinnyW4 B, int n_rows_b, int n_splits,
                     float* __restrict__ part, int ld) {
  __shared__ float s_red[4][MT * 32][SK_BN + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, lq = lane & 31;
  const int n0 = blockIdx.x * SK_BN;
  const int z = blockIdx.y;
  const int steps = K / W4_GROUP;
  const int s_begin = (int)((long)z * steps / n_splits), s_end = (int)((long)(z + 1) * steps / n_splits);

  const uint8_t* cp[2];
  const uint32_t* zp[2];
#pragma unroll
  for (int ct = 0; ct < 2; ++ct) {
    const int n = min(n0 + ct * 32 + lq, n_rows_b - 1);
    int p = 0;
    if (n >= B.begin[1]) p = 1;
    if (n >= B.begin[2]) p = 2;
    // row r of the part: block row r / 32, row r % 32 inside the block; step s of the wave is block (r / 32, s)
    const size_t r = (size_t)(n - B.begin[p]);
    const size_t blk0 = (r / W4_ROWS) * (size_t)steps;
    cp[ct] = B.codes[p] + blk0 * W4_BLOCK_BYTES + (r % W4_ROWS) * (W4_GROUP / 2) + 32 * g;
    zp[ct] = B.sz[p] + blk0 * W4_ROWS + (r % W4_ROWS);
  }
  const bf16_t* ap[MT];
#pragma unroll
  for (int rt = 0; rt < MT; ++rt) ap[rt] = A + (size_t)min(rt * 32 + lq, M - 1) * K + 64 * g;

  f32x16 acc[MT][2];
#pragma unroll
  for (int rt = 0; rt < MT; ++rt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[rt][ct][e] = 0.f;

  // Code words (the HBM stream) and, with one row tile, the activations are requested one step ahead in
  // two register buffers; with two row tiles the activations (from L2) are single-buffered and requested
  // before the next step's codes, so that waiting for them leaves the code loads in flight.
  constexpr int AB = MT == 1 ? 2 : 1;
  uint4 cw[2][2][2];   // [buffer][weight row][half of the 32 bytes]
  uint32_t zw[2][2];   // scale / zero words
  bf16x8 a[AB][MT][8];
#define W4_LOAD_B(BUF, STEP)                                                                        \
  {                                                                                                 \
    _Pragma("unroll") for (int ct = 0; ct < 2; ++ct) {                                              \
      const uint4* src_ = reinterpret_cast<const uint4*>(cp[ct] + (size_t)(STEP) * W4_BLOCK_BYTES); \
      cw[BUF][ct][0] = src_[0];                                                                     \
      cw[BUF][ct][1] = src_[1];                                                                     \
      zw[BUF][ct] = zp[ct][(size_t)(STEP) * W4_ROWS];                                               \
    }                                                                                               \
  }
#define W4_LOAD_A(BUF, STEP)                                                                        \
  {                                                                                                 \
    _Pragma("unroll") for (int rt = 0; rt < MT; ++rt) _Pragma("unroll") for (int c = 0; c < 8; ++c) \
        a[(BUF) % AB][rt][c] = *reinterpret_cast<const bf16x8*>(ap[rt] + (size_t)(STEP) * W4_GROUP + 8 * c); \
  }
#define W4_COMPUTE(BUF)                                                                             \
  {                                                                                                 \
    _Pragma("unroll") for (int ct = 0; ct < 2; ++ct) {                                              \
      float sc_, nzs_;                                                                              \
      w4_scale_zero(zw[BUF][ct], sc_, nzs_);                                                        \
      const uint32_t d_[8] = {cw[BUF][ct][0].x, cw[BUF][ct][0].y, cw[BUF][ct][0].z, cw[BUF][ct][0].w, \
                              cw[BUF][ct][1].x, cw[BUF][ct][1].y, cw[BUF][ct][1].z, cw[BUF][ct][1].w}; \
      _Pragma("unroll") for (int c = 0; c < 8; ++c) {                                               \
        uint32_t o_[4];                                                                             \
        w4_expand8(d_[c], sc_, nzs_, o_);                                                           \
        typedef uint32_t u32x4_ __attribute__((ext_vector_type(4)));                                \
        const u32x4_ ov_ = {o_[0], o_[1], o_[2], o_[3]};                                            \
        const bf16x8 b_ = __builtin_bit_cast(bf16x8, ov_);                                          \
        _Pragma("unroll") for (int rt = 0; rt < MT; ++rt) acc[rt][ct] =                             \
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(BUF) % AB][rt][c], b_, acc[rt][ct], 0, 0, 0); \
      }                                                                                             \
    }                                                                                               \
  }
  // This wave's steps: s_begin + wave, + 4, ... (n_i of them).  Every request is issued unconditionally
  // (past the end the last step is requested again and never used): with no branch around the loads the
  // compiler's wait counts are exact, and a step waits for its own operands only, not for the newer requests.
  const int first = s_begin + wave;
  const int n_i = first < s_end ? (s_end - first + 3) / 4 : 0;
  if (n_i > 0) {
    const int last = first + 4 * (n_i - 1);
    int st = first;
    W4_LOAD_A(0, st)
    W4_LOAD_B(0, st)
    for (int i = 0; i < n_i; i += 2) {  // two steps per trip so that the register buffers keep fixed names
      int nx = min(st + 4, last);
      if (AB == 2) W4_LOAD_A(1, nx)
      W4_LOAD_B(1, nx)
      W4_COMPUTE(0)
      if (i + 1 >= n_i) break;
      st = nx;
      if (AB == 1) W4_LOAD_A(1, st)
      nx = min(st + 4, last);
      if (AB == 2) W4_LOAD_A(0, nx)
      W4_LOAD_B(0, nx)
      W4_COMPUTE(1)
      st = nx;
      if (AB == 1) W4_LOAD_A(0, st)
    }
  }
#undef W4_LOAD_A
#undef W4_LOAD_B
#undef W4_COMPUTE

#pragma unroll
  for (int rt = 0; rt < MT; ++rt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int e = 0; e < 16; ++e) s_red[wave][rt * 32 + 8 * (e >> 2) + 4 * g + (e & 3)][ct * 32 + lq] = acc[rt][ct][e];
  __syncthreads();
  float* dst = part + (size_t)z * M * ld;
  for (int i = tid; i < MT * 32 * SK_BN; i += 256) {
    const int r = i / SK_BN, cidx = i % SK_BN;
    const float v = (s_red[0][r][cidx] + s_red[1][r][cidx]) + (s_red[2][r][cidx] + s_red[3][r][cidx]);
    if (r < M && n0 + cidx < n_rows_b) dst[(size_t)r * ld + n0 + cidx] = v;
  }
}

bool gemm_skinny_fits(int32_t M, int32_t K, const GemmB& B, int32_t N, int epilogue) {
  const long rows = epilogue == EPI_SWIGLU_STORE ? 2L * N : N;
  const long ld = (rows + SK_BN - 1) / SK_BN * SK_BN;
  if (B.has_w4) {  // whole groups along K; every part a whole number of column tiles (two storage blocks)
    if (K % W4_GROUP) return false;
    for (int p = 0; p < B.n_parts; ++p)
      if (B.n_rows[p] % SK_BN) return false;
    if (epilogue == EPI_SWIGLU_STORE && N % SK_BN) return false;
  }
  // Where streaming the weights once stops paying (measured on unit caching at the 14B shape, 48 layers): with
  // bf16 weights the matrix-core tiles are as fast at 16 rows and faster from there on (32 rows: 8.3 ms against
  // 8.9 ms here, 64 rows: 8.8 against 11.0); the 4-bit form moves a quarter of the bytes and wins up to 48 rows
  // (33 rows: 7.3 ms against 8.4 ms, 48: 8.5 against 8.6, 64: 9.5 against 8.8).
  const int max_rows = B.has_w4 ? 48 : 16;
  return M >= 1 && M <= max_rows && K % SK_KSTEP == 0 && K >= SK_KSTEP && rows < (1L << 24) &&
         (size_t)M * (size_t)ld <= SK_MAX_PART_FLOATS && (epilogue != EPI_SWIGLU_STORE || B.n_parts == 1);
}

void launch_gemm_skinny(const bf16_t* A, int32_t M, int32_t K, const GemmB& B, const void* B2, int32_t N, int epilogue,
                        const bf16_t* residual, void* C, void* ws, hipStream_t s) {
  SkinnyB b;
  int acc = 0;
  for (int p = 0; p < 3; ++p) {
    b.ptr[p] = p < B.n_parts ? reinterpret_cast<const bf16_t*>(B.ptr[p]) : nullptr;
    b.begin[p] = acc;
    if (p < B.n_parts) acc += B.n_rows[p];
  }
  b.begin[3] = acc;
  if (epilogue == EPI_SWIGLU_STORE) {  // gate rows, then up rows
    b.ptr[1] = reinterpret_cast<const bf16_t*>(B2);
    b.begin[1] = N;
    acc = 2 * N;
  }
  for (int p = (epilogue == EPI_SWIGLU_STORE ? 2 : B.n_parts); p < 4; ++p) b.begin[p] = acc;  // unused parts never match
  const int rows = acc;
  const int tiles = (rows + SK_BN - 1) / SK_BN;
  const int ld = tiles * SK_BN;
  const int mt = M <= 32 ? 1 : 2;
  const int steps = B.has_w4 ? K / W4_GROUP : K / SK_KSTEP;
  // K slices: the chip holds 512 workgroups at a time (two per CU), and a count just above a multiple of 512
  // leaves most of it idle during the last round.  Among the slice counts that keep at least 4 steps per
  // workgroup and fit the workspace, take the one with the least estimated time, in bytes at the streaming
  // rate: per round of 512 workgroups their share of the weight bytes plus a fixed cost (a round's start-up
  // and its reduction through LDS, ~2 us), plus the partials written and read back.
  int smax = std::max(1, steps / 4);
  smax = (int)std::min<long>(smax, (long)(SK_MAX_PART_FLOATS / ((size_t)M * ld)));
  smax = std::max(1, std::min(smax, 64));
  const double w_bytes = (double)rows * K * (B.has_w4 ? 0.53 : 2.0);
  int splits = 1;
  double best = 0.0;
  for (int sp = 1; sp <= smax; ++sp) {
    const long wgs = (long)tiles * sp;
    const double est = (double)((wgs + 511) / 512) * (512.0 * (w_bytes / wgs) + 9.0e6) + 2.0 * M * (double)ld * sp * 4.0;
    if (sp == 1 || est < best) {
      best = est;
      splits = sp;
    }
  }
  float* part = reinterpret_cast<float*>(ws);
  const dim3 grid(tiles, splits);
  SkinnyEpi e;
  e.epilogue = epilogue;
  e.N = N;
  e.residual = residual;
  e.C = C;
  if (B.has_w4) {
    SkinnyW4 q;
    for (int p = 0; p < 3; ++p) {
      q.codes[p] = reinterpret_cast<const uint8_t*>(B.w4_codes[p]);
      q.sz[p] = reinterpret_cast<const uint32_t*>(B.w4_scale_zero[p]);
      q.begin[p] = b.begin[p];
    }
    q.begin[3] = b.begin[3];
    if (epilogue == EPI_SWIGLU_STORE) {  // the up rows are the second part
      q.codes[1] = reinterpret_cast<const uint8_t*>(B.w4_codes_b2);
      q.sz[1] = reinterpret_cast<const uint32_t*>(B.w4_scale_zero_b2);
    }
    if (mt == 1)
      hipLaunchKernelGGL(k_gemm_skinny_w4<1>, grid, dim3(256), 0, s, A, M, K, q, rows, splits, part, ld);
    else
      hipLaunchKernelGGL(k_gemm_skinny_w4<2>, grid, dim3(256), 0, s, A, M, K, q, rows, splits, part, ld);
  } else if (mt == 1)
    hipLaunchKernelGGL(k_gemm_skinny<1>, grid, dim3(256), 0, s, A, M, K, b, rows, splits, part, ld);
  else
    hipLaunchKernelGGL(k_gemm_skinny<2>, grid, dim3(256), 0, s, A, M, K, b, rows, splits, part, ld);
  const dim3 fgrid((N + 255) / 256, M);
  hipLaunchKernelGGL(k_skinny_finish, fgrid, dim3(256), 0, s, part, splits, ld, M, e);
}

}  // namespace keep
