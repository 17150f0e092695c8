// temporary: MFMA launchers not written yet
#include "keep_internal.h"
namespace keep {
void launch_gemm_mfma(const bf16_t*, int32_t, int32_t, const GemmB&, const void*, int32_t, int, const bf16_t*, void*, hipStream_t) {}
void launch_attn_mfma(const bf16_t*, const bf16_t*, const bf16_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, bf16_t*, float*, hipStream_t) {}
size_t score_mfma_scratch_bytes(int32_t, int32_t) { return 0; }
void launch_score_mfma(const bf16_t*, const bf16_t*, const float*, const int32_t*, const int32_t*, int32_t, int32_t, int32_t, int32_t, void*, float*, hipStream_t) {}
}
