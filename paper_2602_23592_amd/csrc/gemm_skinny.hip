// Skinny GEMM for launches of at most 64 rows (bf16 in, fp32 accumulate): C[M, N] = A[M, K] . B[N, K]^T.
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
// order (no atomics: reproducible) and applies the epilogue.
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
template <int EPI>
__global__ void __launch_bounds__(256)
    k_skinny_finish(const float* __restrict__ part, int n_splits, int ld, int M, int N,
                    const bf16_t* __restrict__ residual, void* __restrict__ Cv) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  const int m = blockIdx.y;
  if (n >= N || m >= M) return;
  float s0 = 0.f, s1 = 0.f;
  for (int z = 0; z < n_splits; ++z) {
    const float* p = part + ((size_t)z * M + m) * ld;
    s0 += p[n];
    if (EPI == EPI_SWIGLU_STORE) s1 += p[N + n];
  }
  const size_t idx = (size_t)m * N + n;
  if (EPI == EPI_STORE_F32) {
    reinterpret_cast<float*>(Cv)[idx] = s0;
  } else if (EPI == EPI_RESIDUAL_STORE) {
    reinterpret_cast<bf16_t*>(Cv)[idx].bits = f32_to_bf16_bits(bf16_bits_to_f32(residual[idx].bits) + s0);
  } else {
    reinterpret_cast<bf16_t*>(Cv)[idx].bits = f32_to_bf16_bits(s0 / (1.0f + __expf(-s0)) * s1);
  }
}

bool gemm_skinny_fits(int32_t M, int32_t K, const GemmB& B, int32_t N, int epilogue) {
  const long rows = epilogue == EPI_SWIGLU_STORE ? 2L * N : N;
  const long ld = (rows + SK_BN - 1) / SK_BN * SK_BN;
  return M >= 1 && M <= 64 && K % SK_KSTEP == 0 && K >= SK_KSTEP && rows < (1L << 24) &&
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
  const int steps = K / SK_KSTEP;
  // enough K slices for ~2048 waves (8 per CU), at least 4 steps per workgroup, partials within the workspace
  int splits = (512 + tiles - 1) / tiles;
  splits = std::min(splits, std::max(1, steps / 4));
  splits = std::min<long>(splits, (long)(SK_MAX_PART_FLOATS / ((size_t)M * ld)));
  splits = std::max(splits, 1);
  float* part = reinterpret_cast<float*>(ws);
  const dim3 grid(tiles, splits);
  if (mt == 1)
    hipLaunchKernelGGL(k_gemm_skinny<1>, grid, dim3(256), 0, s, A, M, K, b, rows, splits, part, ld);
  else
    hipLaunchKernelGGL(k_gemm_skinny<2>, grid, dim3(256), 0, s, A, M, K, b, rows, splits, part, ld);
  const dim3 fgrid((N + 255) / 256, M);
  if (epilogue == EPI_STORE_F32)
    hipLaunchKernelGGL(k_skinny_finish<EPI_STORE_F32>, fgrid, dim3(256), 0, s, part, splits, ld, M, N, residual, C);
  else if (epilogue == EPI_RESIDUAL_STORE)
    hipLaunchKernelGGL(k_skinny_finish<EPI_RESIDUAL_STORE>, fgrid, dim3(256), 0, s, part, splits, ld, M, N, residual, C);
  else
    hipLaunchKernelGGL(k_skinny_finish<EPI_SWIGLU_STORE>, fgrid, dim3(256), 0, s, part, splits, ld, M, N, residual, C);
}

}  // namespace keep
