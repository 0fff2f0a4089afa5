// hs_tree_validate: structural check of packed draft trees, for debugging.  The other calls trust
// their callers for what this one tests: root first with parent -1, every other parent an earlier
// row of the same sequence, sibling tokens distinct, at most HS_MAX_CHILDREN children per node,
// offsets that start at 0 and do not decrease.
#include <limits.h>

#include "hs_common.h"

namespace hs {

constexpr int VAL_THREADS = 256;

__global__ void k_validate_begin(int32_t* report) {
  report[0] = 0;
  report[1] = INT_MAX;
}

__global__ __launch_bounds__(VAL_THREADS) void k_validate(const int32_t* __restrict__ parent,
                                                          const int32_t* __restrict__ token,
                                                          const int32_t* __restrict__ node_offsets, int B, int NN,
                                                          int32_t* report) {
  const int s = blockIdx.x, tid = threadIdx.x;
  // offsets: checked by every workgroup, reported by the first
  bool offsets_ok = node_offsets[0] == 0;
  for (int t = tid; t < B; t += VAL_THREADS) offsets_ok = offsets_ok && node_offsets[t + 1] >= node_offsets[t];
  if (!__syncthreads_and(offsets_ok ? 1 : 0) || node_offsets[B] != NN) {
    if (s == 0 && tid == 0) {
      report[0] = NN;
      report[1] = NN > 0 ? 0 : INT_MAX;
    }
    return;
  }
  const int o = node_offsets[s];
  const int n = node_offsets[s + 1] - o;
  for (int i = tid; i < n; i += VAL_THREADS) {
    const int p = parent[o + i];
    bool wrong = i == 0 ? p != -1 : !(p >= 0 && p < i);
    if (!wrong && i > 0) {
      const int x = token != nullptr ? token[o + i] : 0;
      int before = 0;  // earlier children of the same parent
      for (int j = 1; j < i && !wrong; ++j)
        if (parent[o + j] == p) {
          ++before;
          wrong = token != nullptr && token[o + j] == x;
        }
      wrong = wrong || before >= HS_MAX_CHILDREN;
    }
    if (wrong) {
      atomicAdd(&report[0], 1);
      atomicMin(&report[1], o + i);
    }
  }
}

__global__ void k_validate_end(int32_t* report) {
  if (report[1] == INT_MAX) report[1] = -1;
}

}  // namespace hs

extern "C" hs_status hs_tree_validate(const int32_t* parent, const int32_t* token, const int32_t* node_offsets,
                                      int32_t B, int32_t NN, int32_t* report, hs_stream stream) {
  hs::clear_error();
  HS_REQUIRE(B >= 0 && NN >= 0, HS_ERR_SHAPE, "hs_tree_validate: B=%d NN=%d", B, NN);
  HS_REQUIRE(report, HS_ERR_NULL, "hs_tree_validate: NULL report");
  HS_REQUIRE(B == 0 || node_offsets, HS_ERR_NULL, "hs_tree_validate: NULL node_offsets");
  HS_REQUIRE(NN == 0 || parent, HS_ERR_NULL, "hs_tree_validate: NULL parent");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(hs::k_validate_begin, dim3(1), dim3(1), 0, st, report);
  if (B > 0)
    hipLaunchKernelGGL(hs::k_validate, dim3((unsigned)B), dim3(hs::VAL_THREADS), 0, st, parent, token, node_offsets, B,
                       NN, report);
  hipLaunchKernelGGL(hs::k_validate_end, dim3(1), dim3(1), 0, st, report);
  return hs::launch_status("tree validate");
}
