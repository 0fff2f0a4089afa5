// hs_tree_prune: reranking of the draft tree by cumulative confidence (Section 2.2) under a depth
// cap, a threshold on the cumulative log-probability and a per-sequence node budget (Section 4.3).
//
// Nothing to stream: a few hundred nodes per sequence.  One workgroup per sequence keeps the tree in
// LDS (global scratch for very large trees), fills depth and the cumulative sums level by level so
// that every sum is the single float32 add the definition states, ranks the surviving candidates by
// counting, and scans the keep flags; a second launch turns per-sequence counts into packed offsets
// and emits the renumbered tree.
#include <limits.h>

#include "hs_common.h"

namespace hs {

constexpr int PR_THREADS = 256;
constexpr int PR_LDS_NODES = 4096;  // trees up to this size live in LDS

__device__ __forceinline__ int block_reduce_max(int v, int* red) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = max(v, __shfl_xor(v, off));
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  int r = red[0];
  for (int w = 1; w < PR_THREADS / 64; ++w) r = max(r, red[w]);
  __syncthreads();
  return r;
}

__device__ __forceinline__ int block_reduce_sum(int v, int* red) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  int r = 0;
  for (int w = 0; w < PR_THREADS / 64; ++w) r += red[w];
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(PR_THREADS) void k_prune_select(
    const int32_t* __restrict__ parent, const float* __restrict__ logc, const int32_t* __restrict__ node_offsets,
    const int32_t* __restrict__ d_max, const float* __restrict__ theta, const int32_t* __restrict__ max_nodes,
    int32_t* __restrict__ depth, float* __restrict__ cumlogp, uint8_t* __restrict__ keep,
    int32_t* __restrict__ ws_pos, int32_t* __restrict__ ws_count, int32_t* __restrict__ ws_flag) {
  __shared__ int l_par[PR_LDS_NODES];
  __shared__ int l_dep[PR_LDS_NODES];
  __shared__ float l_sum[PR_LDS_NODES];
  __shared__ int l_ok[PR_LDS_NODES];
  __shared__ int l_new[PR_LDS_NODES];
  __shared__ int red[PR_THREADS / 64];
  __shared__ int chunk_sum[PR_THREADS];

  const int s = blockIdx.x, tid = threadIdx.x;
  const int o = node_offsets[s];
  const int n = node_offsets[s + 1] - o;
  if (n <= 0) {
    if (tid == 0) ws_count[s] = 0;
    return;
  }
  const bool in_lds = n <= PR_LDS_NODES;
  // large trees use the output arrays and the workspace as their scratch
  int* par = in_lds ? l_par : const_cast<int*>(parent + o);
  int* dep = in_lds ? l_dep : depth + o;
  float* sum = in_lds ? l_sum : cumlogp + o;
  int* ok = in_lds ? l_ok : ws_flag + o;

  if (in_lds)
    for (int i = tid; i < n; i += PR_THREADS) par[i] = parent[o + i];
  __syncthreads();

  // depth: walk to the root
  int my_max = 0;
  for (int i = tid; i < n; i += PR_THREADS) {
    int d = 0;
    for (int j = par[i]; j >= 0; j = par[j]) ++d;
    dep[i] = d;
    my_max = max(my_max, d);
  }
  if (tid == 0) {
    sum[0] = 0.f;
    ok[0] = 1;
  }
  const int max_depth = block_reduce_max(my_max, red);

  // cumulative log-confidence and the path filter, one level at a time (parents are final first)
  const int dcap = d_max[s];
  const float th = theta[s];
  for (int level = 1; level <= max_depth; ++level) {
    for (int i = tid; i < n; i += PR_THREADS) {
      if (dep[i] == level) {
        const int p = par[i];
        const float v = sum[p] + fminf(logc[o + i], 0.f);
        sum[i] = v;
        ok[i] = (ok[p] != 0 && level <= dcap && v >= th) ? 1 : 0;
      }
    }
    __syncthreads();
  }

  // node budget: keep the first max_nodes candidates under (sum descending, index ascending)
  const int budget = max_nodes[s];
  int mine = 0;
  for (int i = tid; i < n; i += PR_THREADS) mine += (i >= 1 && ok[i]) ? 1 : 0;
  const int n_cand = block_reduce_sum(mine, red);
  if (budget > 0 && n_cand > budget) {
    int* nxt = in_lds ? l_new : ws_pos + o;  // ws_pos is not written before the last phase
    for (int i = tid; i < n; i += PR_THREADS) {
      int flag = ok[i];
      if (i >= 1 && flag) {
        const float v = sum[i];
        int r = 0;
        for (int j = 1; j < n; ++j) r += (ok[j] && better(sum[j], j, v, i)) ? 1 : 0;
        flag = r < budget ? 1 : 0;
      }
      nxt[i] = flag;
    }
    __syncthreads();
    for (int i = tid; i < n; i += PR_THREADS) ok[i] = nxt[i];
    __syncthreads();
  }

  // positions of the kept nodes: each thread owns a contiguous chunk, then a scan of chunk totals
  const int per = (n + PR_THREADS - 1) / PR_THREADS;
  const int lo = min(tid * per, n), hi = min(lo + per, n);
  int c = 0;
  for (int i = lo; i < hi; ++i) c += ok[i] ? 1 : 0;
  chunk_sum[tid] = c;
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int t = 0; t < PR_THREADS; ++t) {
      int x = chunk_sum[t];
      chunk_sum[t] = run;
      run += x;
    }
    ws_count[s] = run;
  }
  __syncthreads();
  int pos = chunk_sum[tid];
  for (int i = lo; i < hi; ++i) {
    const int k = ok[i] ? 1 : 0;
    ws_pos[o + i] = k ? pos : -1;
    keep[o + i] = (uint8_t)k;
    pos += k;
    if (in_lds) {
      depth[o + i] = dep[i];
      cumlogp[o + i] = sum[i];
    }
  }
}

__global__ __launch_bounds__(PR_THREADS) void k_prune_emit(const int32_t* __restrict__ parent,
                                                           const int32_t* __restrict__ node_offsets, int B,
                                                           const int32_t* __restrict__ ws_pos,
                                                           const int32_t* __restrict__ ws_count,
                                                           int32_t* __restrict__ out_offsets,
                                                           int32_t* __restrict__ out_src,
                                                           int32_t* __restrict__ out_parent) {
  __shared__ int red[PR_THREADS / 64];
  const int s = blockIdx.x, tid = threadIdx.x;
  int mine = 0;
  for (int t = tid; t < s; t += PR_THREADS) mine += ws_count[t];
  const int base = block_reduce_sum(mine, red);
  if (tid == 0) {
    out_offsets[s] = base;
    if (s == B - 1) out_offsets[B] = base + ws_count[s];
  }
  const int o = node_offsets[s];
  const int n = node_offsets[s + 1] - o;
  for (int i = tid; i < n; i += PR_THREADS) {
    const int p = ws_pos[o + i];
    if (p >= 0) {
      out_src[base + p] = i;
      out_parent[base + p] = (i == 0) ? -1 : ws_pos[o + parent[o + i]];
    }
  }
}

}  // namespace hs

extern "C" size_t hs_tree_prune_workspace(int32_t B, int32_t NN) {
  if (B <= 0 || NN < 0) return 0;
  return 2 * hs::align_up((size_t)(NN > 0 ? NN : 1) * sizeof(int32_t), 256) +
         hs::align_up((size_t)B * sizeof(int32_t), 256);
}

extern "C" hs_status hs_tree_prune(const int32_t* parent, const float* logc, const int32_t* node_offsets, int32_t B,
                                   int32_t NN, const int32_t* d_max, const float* theta, const int32_t* max_nodes,
                                   int32_t* depth, float* cumlogp, uint8_t* keep, int32_t* out_offsets,
                                   int32_t* out_src, int32_t* out_parent, void* workspace, size_t workspace_bytes,
                                   hs_stream stream) {
  hs::clear_error();
  HS_REQUIRE(B >= 0 && NN >= 0, HS_ERR_SHAPE, "hs_tree_prune: B=%d NN=%d", B, NN);
  if (B == 0) return HS_OK;
  HS_REQUIRE(node_offsets && d_max && theta && max_nodes && out_offsets, HS_ERR_NULL, "hs_tree_prune: NULL argument");
  HS_REQUIRE(NN == 0 || (parent && logc && depth && cumlogp && keep && out_src && out_parent), HS_ERR_NULL,
             "hs_tree_prune: NULL node array");
  const size_t need = hs_tree_prune_workspace(B, NN);
  HS_REQUIRE(workspace && workspace_bytes >= need && reinterpret_cast<uintptr_t>(workspace) % 256 == 0,
             HS_ERR_WORKSPACE, "hs_tree_prune: workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
             workspace_bytes);
  hs::Carver c(workspace);
  int32_t* ws_pos = c.take<int32_t>(NN > 0 ? NN : 1);
  int32_t* ws_flag = c.take<int32_t>(NN > 0 ? NN : 1);
  int32_t* ws_count = c.take<int32_t>(B);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(hs::k_prune_select, dim3(B), dim3(hs::PR_THREADS), 0, st, parent, logc, node_offsets, d_max,
                     theta, max_nodes, depth, cumlogp, keep, ws_pos, ws_count, ws_flag);
  hs_status r = hs::launch_status("prune select");
  if (r != HS_OK) return r;
  hipLaunchKernelGGL(hs::k_prune_emit, dim3(B), dim3(hs::PR_THREADS), 0, st, parent, node_offsets, B, ws_pos,
                     ws_count, out_offsets, out_src, out_parent);
  return hs::launch_status("prune emit");
}
