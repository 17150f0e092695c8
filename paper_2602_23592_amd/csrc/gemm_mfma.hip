// bf16 GEMM on the gfx950 matrix cores:  C[M,N] = A[M,K] . W[N,K]^T  (fp32 accumulate)
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants:
// lane l supplies 8 consecutive k of row (l % 32), k-block (l / 32).  A workgroup owns a
// BM x BN tile of C; K is walked in 64-deep slices staged through LDS (two buffers, one
// barrier per slice, next slice prefetched into registers while the current one is
// multiplied).  LDS rows are 128 B; their 16-byte chunks are XOR-swizzled by the row
// index so that the 16-byte operand reads of 32 consecutive rows spread over all banks.
//
// Epilogues: plain fp32 store (QKV), residual add (output and down projections), and
// SwiGLU: the B tile interleaves rows of W_gate and W_up so that one lane holds
// gate[m, n] and up[m, n] in matching accumulator registers.
#include "keep_internal.h"

namespace keep {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // 16-byte register vector (native, so arrays of it stay in VGPRs)

struct MfmaB {
  const bf16_t* ptr[3];
  int32_t begin[4];
  int32_t n_parts;
};

constexpr int GBK = 64;  // K slice

__device__ __forceinline__ int lds_off(int row, int chunk) {
  // element offset of 16-byte chunk `chunk` (0..7) of row `row` in a [rows][64] bf16 tile
  return row * GBK + ((chunk ^ (row & 7)) << 3);
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ void __launch_bounds__(WM* WN * 64)
    k_gemm_mfma(const bf16_t* __restrict__ A, int M, int K, MfmaB B, const bf16_t* __restrict__ B2, int N,
                const bf16_t* __restrict__ residual, void* __restrict__ Cv) {
  constexpr int T = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int A_CH = BM * 8 / T, B_CH = BN * 8 / T;  // 16-byte chunks per thread per slice
  static_assert(BM * 8 % T == 0 && BN * 8 % T == 0, "tile / thread mismatch");
  static_assert(EPI != EPI_SWIGLU_STORE || (NI % 2 == 0), "SwiGLU needs an even number of N tiles per wave");

  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int BUF = (BM + BN) * GBK;  // elements per buffer: A tile then B tile

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int m0 = blockIdx.y * BM;
  const int n0 = blockIdx.x * BN;  // in B-tile rows (for SwiGLU: BN/2 output columns per block)

  // ---- global source pointers of this thread's chunks
  const u32x4* a_src[A_CH];
  const u32x4* b_src[B_CH];
  int a_dst[A_CH], b_dst[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int q = tid + i * T, r = q >> 3, c = q & 7;
    const int gm = min(m0 + r, M - 1);
    a_src[i] = reinterpret_cast<const u32x4*>(A + (size_t)gm * K + c * 8);
    a_dst[i] = lds_off(r, c);
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int q = tid + i * T, r = q >> 3, c = q & 7;
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
    b_src[i] = reinterpret_cast<const u32x4*>(row + c * 8);
    b_dst[i] = lds_off(r, c);
  }

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 a_reg[A_CH], b_reg[B_CH];
  const int KT = K / GBK;
  // prologue: slice 0 -> LDS buffer 0
#pragma unroll
  for (int i = 0; i < A_CH; ++i) a_reg[i] = a_src[i][0];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) b_reg[i] = b_src[i][0];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) *reinterpret_cast<u32x4*>(smem + a_dst[i]) = a_reg[i];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) *reinterpret_cast<u32x4*>(smem + BM * GBK + b_dst[i]) = b_reg[i];
  __syncthreads();

  const int a_row0 = wm * TM + (lane & 31);
  const int b_row0 = wn * TN + (lane & 31);
  const int kg = lane >> 5;

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      const int ko = (kt + 1) * (GBK / 8);  // in 16-byte units
#pragma unroll
      for (int i = 0; i < A_CH; ++i) a_reg[i] = a_src[i][ko];
#pragma unroll
      for (int i = 0; i < B_CH; ++i) b_reg[i] = b_src[i][ko];
    }
    const uint16_t* cA = smem + cur * BUF;
    const uint16_t* cB = cA + BM * GBK;
#pragma unroll
    for (int ks = 0; ks < GBK / 16; ++ks) {
      bf16x8 af[MI], bfr[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(cA + lds_off(a_row0 + i * 32, ks * 2 + kg));
#pragma unroll
      for (int j = 0; j < NI; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8*>(cB + lds_off(b_row0 + j * 32, ks * 2 + kg));
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      uint16_t* nA = smem + (cur ^ 1) * BUF;
      uint16_t* nB = nA + BM * GBK;
#pragma unroll
      for (int i = 0; i < A_CH; ++i) *reinterpret_cast<u32x4*>(nA + a_dst[i]) = a_reg[i];
#pragma unroll
      for (int i = 0; i < B_CH; ++i) *reinterpret_cast<u32x4*>(nB + b_dst[i]) = b_reg[i];
    }
    __syncthreads();
  }

  // ---- epilogue.  acc[i][j][e]: row = i*32 + 8*(e/4) + 4*(lane/32) + e%4, col = j*32 + lane%32
  const int col_l = lane & 31;
  const int row_l = 4 * (lane >> 5);
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int gm = m0 + wm * TM + i * 32 + 8 * (e >> 2) + row_l + (e & 3);
      if (gm >= M) continue;
      if (EPI == EPI_SWIGLU_STORE) {
        const int n_out = N;  // N = ffn_dim (output width)
#pragma unroll
        for (int j = 0; j < NI / 2; ++j) {
          const int gn = (n0 / 2) + wn * (TN / 2) + j * 32 + col_l;
          const float g = acc[i][j][e], u = acc[i][j + NI / 2][e];
          const float v = g / (1.0f + __expf(-g)) * u;
          reinterpret_cast<bf16_t*>(Cv)[(size_t)gm * n_out + gn].bits = f32_to_bf16_bits(v);
        }
      } else {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          const int gn = n0 + wn * TN + j * 32 + col_l;
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

template <int BM, int BN, int WM, int WN>
static void launch_cfg(const bf16_t* A, int M, int K, const MfmaB& b, const bf16_t* B2, int N, int epilogue,
                       const bf16_t* residual, void* C, hipStream_t s) {
  const size_t sh = (size_t)2 * (BM + BN) * GBK * sizeof(uint16_t);
  const dim3 block(WM * WN * 64);
  const int n_tile_rows = epilogue == EPI_SWIGLU_STORE ? 2 * N : N;  // B-tile rows to cover
  const dim3 grid(n_tile_rows / BN, (M + BM - 1) / BM);
#define GO(E)                                                                                              \
  do {                                                                                                     \
    auto kern = k_gemm_mfma<BM, BN, WM, WN, E>;                                                            \
    static bool attr_set = false;                                                                          \
    if (!attr_set) {                                                                                       \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                (int)sh);                                                                  \
      attr_set = true;                                                                                     \
    }                                                                                                      \
    hipLaunchKernelGGL(kern, grid, block, sh, s, A, M, K, b, B2, N, residual, C);                          \
  } while (0)
  if (epilogue == EPI_STORE_F32)
    GO(EPI_STORE_F32);
  else if (epilogue == EPI_RESIDUAL_STORE)
    GO(EPI_RESIDUAL_STORE);
  else
    GO(EPI_SWIGLU_STORE);
#undef GO
}

void launch_gemm_mfma(const bf16_t* A, int32_t M, int32_t K, const GemmB& B, const void* B2, int32_t N, int epilogue,
                      const bf16_t* residual, void* C, hipStream_t s) {
  if (M <= 0 || N <= 0) return;
  MfmaB b;
  b.n_parts = B.n_parts;
  int acc = 0;
  bool aligned256 = true;
  for (int p = 0; p < 3; ++p) {
    b.ptr[p] = p < B.n_parts ? reinterpret_cast<const bf16_t*>(B.ptr[p]) : nullptr;
    b.begin[p] = acc;
    if (p < B.n_parts) {
      acc += B.n_rows[p];
      if (acc % 256) aligned256 = false;
    }
  }
  b.begin[3] = acc;
  const bf16_t* b2 = reinterpret_cast<const bf16_t*>(B2);
  const int rows = epilogue == EPI_SWIGLU_STORE ? 2 * N : N;
  if (aligned256 && rows % 256 == 0 && M > 128)
    launch_cfg<256, 256, 2, 2>(A, M, K, b, b2, N, epilogue, residual, C, s);
  else if (rows % 128 == 0)
    launch_cfg<128, 128, 2, 2>(A, M, K, b, b2, N, epilogue, residual, C, s);
  else
    launch_cfg<64, 64, 1, 1>(A, M, K, b, b2, N, epilogue, residual, C, s);
}

}  // namespace keep
