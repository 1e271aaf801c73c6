// a3: greedy top-k of the per-path posterior (Sec. 3.2.3; Alg. 3).  One workgroup per prompt.
// Each path's rank is the number of paths that come before it in the order
// (score descending, index ascending, NaN last); paths with rank < k write kept[rank].
#include "sp_internal.h"

namespace sp {

// true when (a, ia) is ordered strictly before (b, ib)
__device__ __forceinline__ bool before(float a, int ia, float b, int ib) {
  const bool an = a != a, bn = b != b;
  if (an || bn) return (!an && bn) || (an && bn && ia < ib);
  return a > b || (a == b && ia < ib);
}

__global__ __launch_bounds__(256) void topk_kernel(const float *__restrict__ score,
                                                   const int32_t *__restrict__ path_off, int32_t k,
                                                   int32_t n_cap, int32_t *__restrict__ kept) {
  extern __shared__ float s_sc[];
  const int b = blockIdx.x;
  const int base = path_off[b];
  int n = path_off[b + 1] - base;
  n = n < 0 ? 0 : n;
  // a prompt with more paths than the caller's bound is still ranked completely: its scores are then
  // read from global memory instead of the LDS copy (slower, never truncated)
  const bool staged = n <= n_cap;
  const float *sc = score + base;
  if (staged)
    for (int i = threadIdx.x; i < n; i += blockDim.x) s_sc[i] = sc[i];
  for (int j = n + threadIdx.x; j < k; j += blockDim.x) kept[(int64_t)b * k + j] = -1;
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const float mine = staged ? s_sc[i] : sc[i];
    int rank = 0;
    if (staged) {
      for (int j = 0; j < n; ++j) rank += before(s_sc[j], j, mine, i) ? 1 : 0;
    } else {
      for (int j = 0; j < n; ++j) rank += before(sc[j], j, mine, i) ? 1 : 0;
    }
    if (rank < k) kept[(int64_t)b * k + rank] = i;
  }
}

hipError_t launch_topk(const float *score, const int32_t *path_off, int32_t n_prompts, int32_t n_paths_max,
                       int32_t k, int32_t *kept, hipStream_t s) {
  hipLaunchKernelGGL(topk_kernel, dim3(n_prompts), dim3(256), size_t(n_paths_max) * sizeof(float), s, score,
                     path_off, k, n_paths_max, kept);
  return hipGetLastError();
}

}  // namespace sp
