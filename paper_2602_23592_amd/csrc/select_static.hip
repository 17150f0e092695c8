// keep_select_groups_static: the multi-hop selection for callers that cannot allocate.
//
// Same kernel as keep_select_groups (k_select).  That entry point keeps the candidates' lengths and the
// candidates' token total in the context's workspace (device memory the library allocated at keep_init);
// here they live in a file-scope device array, so the call needs no context, no workspace and makes no
// allocation of any kind.  Every GPU the library runs on holds its own copy of the array until the process
// ends; all calls on one GPU share it, so calls that overlap on one GPU race.
#include <math.h>

#include <algorithm>
#include <mutex>

#include "keep_internal.h"

namespace keep {
void set_init_error(const char* text);  // api.hip: message behind keep_last_error(NULL)
}

using namespace keep;

namespace {

// scratch: [0, KEEP_STATIC_MAX_CANDIDATES) lengths of the candidates, then one word: their sum
constexpr int SCRATCH_WORDS = KEEP_STATIC_MAX_CANDIDATES + 64;
static __device__ __align__(256) int32_t scratch[SCRATCH_WORDS];

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
int32_t* g_scratch_ptr[MAX_DEVICES] = {};  // device address of `scratch` on each GPU (its own copy at its own address)

// Lengths of the candidates in candidate order and their total.  One workgroup; indices are clamped into
// the length table so that a bad id cannot make the kernel read out of bounds.
__global__ void __launch_bounds__(1024)
    k_static_prepare(const int32_t* __restrict__ groups, int m, const int32_t* __restrict__ group_len, int n_groups,
                     int32_t* __restrict__ cand_len, int32_t* __restrict__ cand_total) {
  __shared__ int s_part[16];
  int sum = 0;
  for (int i = threadIdx.x; i < m; i += 1024) {
    const int g = min(max(groups[i], 0), n_groups - 1);
    const int len = group_len[g];
    cand_len[i] = len;
    sum += len;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < 16; ++w) t += s_part[w];
    *cand_total = t;  // written, not accumulated: nothing of an earlier call survives
  }
}

keep_status fail_static(keep_status st, const char* text) {
  set_init_error(text);
  return st;
}

}  // namespace

extern "C" keep_status keep_select_groups_static(const float* S, const int32_t* groups, int32_t n_sel,
                                                 const int32_t* group_len, int32_t n_groups_total, int32_t mem_tokens,
                                                 float ratio_next, int32_t hops, int32_t budget_mode,
                                                 int32_t propagation_sources, int32_t* result, void* stream) {
  if (!result || !group_len || (n_sel > 0 && (!S || !groups)))
    return fail_static(KEEP_ERR_INVALID_ARG, "keep_select_groups_static: a pointer argument is NULL");
  if (budget_mode != KEEP_BUDGET_GROUP_COUNT && budget_mode != KEEP_BUDGET_TOKENS)
    return fail_static(KEEP_ERR_INVALID_ARG, "keep_select_groups_static: unknown budget_mode");
  if (propagation_sources != KEEP_SOURCES_QUERY_AND_SET && propagation_sources != KEEP_SOURCES_SET_ONLY)
    return fail_static(KEEP_ERR_INVALID_ARG, "keep_select_groups_static: unknown propagation_sources");
  if (!(ratio_next >= 0.f && ratio_next <= 1.f))
    return fail_static(KEEP_ERR_INVALID_ARG, "keep_select_groups_static: ratio_next outside [0, 1]");
  if (hops < 1) return fail_static(KEEP_ERR_INVALID_ARG, "keep_select_groups_static: hops must be at least 1");
  if (n_groups_total < 1 || mem_tokens < n_groups_total)
    return fail_static(KEEP_ERR_INVALID_ARG, "keep_select_groups_static: n_groups_total must be at least 1 and "
                                             "mem_tokens at least n_groups_total (every memory has a token)");
  if (n_sel < 0 || n_sel > n_groups_total)
    return fail_static(KEEP_ERR_INVALID_ARG, "keep_select_groups_static: n_sel outside [0, n_groups_total]");
  if (n_sel > KEEP_STATIC_MAX_CANDIDATES)
    return fail_static(KEEP_ERR_WORKSPACE, "keep_select_groups_static: more than KEEP_STATIC_MAX_CANDIDATES (4096) "
                                           "candidates do not fit the static scratch array");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
    return fail_static(KEEP_ERR_HIP, "keep_select_groups_static: no current HIP device");
  int32_t* sp;
  {
    // first call on this device: ask the runtime where this device's copy of the array lives
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
        return fail_static(KEEP_ERR_HIP, "keep_select_groups_static: hipGetSymbolAddress(scratch) failed");
      g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    sp = g_scratch_ptr[dev];
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* cand_len = sp;
  int32_t* cand_total = sp + KEEP_STATIC_MAX_CANDIDATES;
  hipLaunchKernelGGL(k_static_prepare, dim3(1), dim3(1024), 0, s, groups, n_sel, group_len, n_groups_total, cand_len,
                     cand_total);
  // the two budgets, as keep_select_groups forms them on the host
  const int k_count = std::max(0, std::min<int>(n_sel, (int)ceil((double)ratio_next * (double)n_groups_total - 1.0e-3)));
  const int token_budget = (int)floor((double)ratio_next * (double)mem_tokens + 1.0e-3);
  launch_select(S, n_sel, cand_len, k_count, token_budget, budget_mode, hops, nullptr, nullptr, result, s,
                propagation_sources == KEEP_SOURCES_SET_ONLY, cand_total, groups);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_static(KEEP_ERR_HIP, hipGetErrorString(e));
  return KEEP_OK;
}
