// hs_tree_expand: one level of Top-K growth of the draft trees, on the device (Section 2.2,
// Expansion; Section 4.3, Dynamic Extended Drafting: per-sequence depth limits).
//
// Nothing to stream: at most F * K new rows per sequence.  One workgroup per sequence appends the
// children of the frontier rows (their values are the single float32 add per node that the
// reranking step defines), ranks the new rows by counting under (value descending, row ascending)
// and lists the F best, in row order, as the next frontier.  The host never sees the tree: the
// calls of a step can be queued back to back, or captured in a graph.
#include <limits.h>

#include "hs_common.h"

namespace hs {

constexpr int EXP_THREADS = 256;
constexpr int EXP_MAX_NEW = 4096;  // F * K

struct ExpandArgs {
  int32_t* parent;
  int32_t* token;
  float* logc;
  float* cumlogp;
  int32_t* depth;
  float* ent;
  int32_t* n_nodes;
  int32_t* level;
  int32_t* frontier;
  int32_t* n_frontier;
  int32_t* frontier_rows;
  const int32_t* topk_idx;
  const float* topk_logp;
  const float* ent_topk;
  const int32_t* d_limit;
  int cap, F, K, first;
};

__global__ __launch_bounds__(EXP_THREADS) void k_tree_expand(ExpandArgs a) {
  __shared__ float cv[EXP_MAX_NEW];       // values of the new rows
  __shared__ int sel[EXP_MAX_NEW];        // 1 = among the F best
  __shared__ int fr_old[EXP_MAX_NEW];     // the frontier being expanded
  const int s = blockIdx.x, tid = threadIdx.x;
  const int F = a.F, K = a.K;
  const int64_t base = (int64_t)s * a.cap;
  int n, lvl, nf;
  if (a.first) {
    n = 1;
    lvl = 0;
    nf = 1;
    if (tid == 0) {
      a.parent[base] = -1;
      a.token[base] = -1;
      a.logc[base] = 0.f;
      a.cumlogp[base] = 0.f;
      a.depth[base] = 0;
      a.ent[base] = 0.f;
      fr_old[0] = 0;
    }
  } else {
    n = a.n_nodes[s];
    lvl = a.level[s];
    nf = a.n_frontier[s];
    nf = nf < 0 ? 0 : (nf > F ? F : nf);
    for (int j = tid; j < nf; j += EXP_THREADS) fr_old[j] = a.frontier[(int64_t)s * F + j];
  }
  const bool idle = nf == 0 || (a.d_limit != nullptr && lvl >= a.d_limit[s]);
  if (idle) {
    if (tid == 0) {
      a.n_frontier[s] = 0;
      if (a.first) {
        a.n_nodes[s] = 1;
        a.level[s] = 0;
      }
    }
    if (a.frontier_rows != nullptr)
      for (int j = tid; j < F; j += EXP_THREADS) a.frontier_rows[(int64_t)s * F + j] = (int32_t)base;
    return;
  }
  __syncthreads();  // fr_old is complete (and the root row written)

  // children of the frontier rows whose K children fit the capacity (a prefix of the frontier)
  int n_fit = (a.cap - n) / K;
  n_fit = n_fit > nf ? nf : n_fit;
  const int m = n_fit * K;
  for (int e = tid; e < m; e += EXP_THREADS) {
    const int j = e / K, k = e - j * K;
    const int f = fr_old[j];
    const int64_t src = ((int64_t)s * F + j) * K + k;
    const float lc = a.topk_logp[src];
    // the root's value is 0 by definition (on a first call its row may not be visible yet)
    const float up = (a.first || f == 0) ? 0.f : a.cumlogp[base + f];
    const float v = up + fminf(lc, 0.f);
    const int dep = (a.first || f == 0) ? 0 : a.depth[base + f];
    const int64_t row = base + n + e;
    a.parent[row] = f;
    a.token[row] = a.topk_idx[src];
    a.logc[row] = lc;
    a.cumlogp[row] = v;
    a.depth[row] = dep + 1;
    a.ent[row] = 0.f;
    cv[e] = v;
  }
  for (int j = tid; j < nf; j += EXP_THREADS) a.ent[base + fr_old[j]] = a.ent_topk[(int64_t)s * F + j];
  __syncthreads();

  // the F best new rows: rank by counting (the order is strict, so ranks are a permutation)
  for (int e = tid; e < m; e += EXP_THREADS) {
    const float v = cv[e];
    int r = 0;
    for (int o = 0; o < m; ++o) r += better(cv[o], o, v, e) ? 1 : 0;
    sel[e] = r < F ? 1 : 0;
  }
  __syncthreads();
  const int nf_new = m < F ? m : F;
  for (int e = tid; e < m; e += EXP_THREADS) {
    if (sel[e]) {
      int pos = 0;
      for (int o = 0; o < e; ++o) pos += sel[o];
      a.frontier[(int64_t)s * F + pos] = n + e;
      if (a.frontier_rows != nullptr) {
        a.frontier_rows[(int64_t)s * F + pos] = (int32_t)(base + n + e);
        if (pos == nf_new - 1)  // the last valid slot also fills the unused ones
          for (int j = nf_new; j < F; ++j) a.frontier_rows[(int64_t)s * F + j] = (int32_t)(base + n + e);
      }
    }
  }
  if (nf_new == 0 && a.frontier_rows != nullptr)
    for (int j = tid; j < F; j += EXP_THREADS) a.frontier_rows[(int64_t)s * F + j] = (int32_t)base;
  if (tid == 0) {
    a.n_nodes[s] = n + m;
    a.level[s] = lvl + 1;
    a.n_frontier[s] = nf_new;
  }
}

}  // namespace hs

using namespace hs;

extern "C" hs_status hs_tree_expand(int32_t* parent, int32_t* token, float* logc, float* cumlogp, int32_t* depth,
                                    float* ent, int32_t* n_nodes, int32_t* level, int32_t* frontier,
                                    int32_t* n_frontier, int32_t* frontier_rows, const int32_t* topk_idx,
                                    const float* topk_logp, const float* ent_topk, const int32_t* d_limit, int32_t B,
                                    int32_t cap, int32_t F, int32_t K, int32_t first, hs_stream stream) {
  clear_error();
  HS_REQUIRE(B >= 0, HS_ERR_SHAPE, "hs_tree_expand: B=%d", B);
  HS_REQUIRE(K >= 1 && K <= HS_MAX_TOPK, HS_ERR_SHAPE, "hs_tree_expand: K=%d must be in 1..%d", K, HS_MAX_TOPK);
  HS_REQUIRE(F >= 1 && (int64_t)F * K <= EXP_MAX_NEW, HS_ERR_SHAPE, "hs_tree_expand: F=%d, F * K must be in 1..%d", F,
             EXP_MAX_NEW);
  HS_REQUIRE(cap >= 1 + K, HS_ERR_SHAPE, "hs_tree_expand: cap=%d holds no level (K=%d)", cap, K);
  HS_REQUIRE((int64_t)B * cap < ((int64_t)1 << 31), HS_ERR_SHAPE, "hs_tree_expand: B * cap exceeds 2^31 rows");
  if (B == 0) return HS_OK;
  HS_REQUIRE(parent && token && logc && cumlogp && depth && ent && n_nodes && level && frontier && n_frontier &&
                 topk_idx && topk_logp && ent_topk,
             HS_ERR_NULL, "hs_tree_expand: NULL argument");
  ExpandArgs a{parent, token, logc, cumlogp, depth, ent, n_nodes, level, frontier, n_frontier, frontier_rows,
               topk_idx, topk_logp, ent_topk, d_limit, cap, F, K, first != 0 ? 1 : 0};
  hipLaunchKernelGGL(k_tree_expand, dim3((unsigned)B), dim3(EXP_THREADS), 0, static_cast<hipStream_t>(stream), a);
  return launch_status("tree expand");
}
