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

// (value, index) as one 45-bit key, index < 8192: larger key = better (larger value, then lower
// index); never 0.  The budget-th best key is found digit by digit, 6 bits at a time.
constexpr int KEY_BITS = 45;
constexpr int DIGIT_BITS = 6;
constexpr int N_DIGITS = (KEY_BITS + DIGIT_BITS - 1) / DIGIT_BITS;  // 8
__device__ __forceinline__ unsigned long long order_key(float v, int i) {
  unsigned u = __builtin_bit_cast(unsigned, v);
  u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;  // monotone map of float order onto unsigned order
  return ((unsigned long long)u << 13) | (unsigned)(8191 - i);
}

// The whole selection for one sequence; called once with LDS arrays and once with global scratch so
// that each copy is compiled for its own address space.
template <typename IP, typename FP>
__device__ __forceinline__ void prune_sequence(
    IP par, IP dep, FP sum, IP ok, IP nxt, unsigned long long* keys, int* digit_hist, int* red, int* chunk_sum, int n,
    int o,
    bool copy_out, FP lc, int dcap, float th, int budget, int32_t* __restrict__ depth,
    float* __restrict__ cumlogp, uint8_t* __restrict__ keep, int32_t* __restrict__ ws_pos,
    int32_t* __restrict__ ws_count, int s, bool emit, int32_t* __restrict__ out_offsets,
    int32_t* __restrict__ out_src, int32_t* __restrict__ out_parent, int NN) {
  const int tid = threadIdx.x, lane = tid & 63;
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
  for (int level = 1; level <= max_depth; ++level) {
    for (int i = tid; i < n; i += PR_THREADS) {
      if (dep[i] == level) {
        const int p = par[i];
        const float v = sum[p] + fminf(lc[i], 0.f);
        sum[i] = v;
        ok[i] = (ok[p] != 0 && level <= dcap && v >= th) ? 1 : 0;
      }
    }
    __syncthreads();
  }

  // node budget: keep the first max_nodes candidates under (sum descending, index ascending)
  int mine = 0;
  for (int i = tid; i < n; i += PR_THREADS) mine += (i >= 1 && ok[i]) ? 1 : 0;
  const int n_cand = block_reduce_sum(mine, red);
  if (budget > 0 && n_cand > budget) {
    if (keys != nullptr) {
      // The budget-th best key, digit by digit from the top.  Per digit: a 64-bin histogram of the
      // keys that match the digits fixed so far (LDS atomics, one histogram per round so that no
      // round waits for a reset), one barrier, then every wave finds, with a prefix sum over the
      // bins from the top, the largest digit d such that at least `need` matching keys have a digit
      // >= d; the keys above d are all in, the search goes on among those with digit d.  Keys are
      // distinct, so exactly `budget` candidates end up >= x.  Non-candidates carry key 0.
      for (int i = tid; i < n; i += PR_THREADS) keys[i] = (i >= 1 && ok[i]) ? order_key(sum[i], i) : 0ull;
      for (int b = tid; b < N_DIGITS * 64; b += PR_THREADS) digit_hist[b] = 0;
      __syncthreads();
      unsigned long long x = 0ull;  // digits fixed so far, in place
      int need = budget;
      for (int r = 0; r < N_DIGITS; ++r) {
        const int shift = (N_DIGITS - 1 - r) * DIGIT_BITS;
        int* hist = digit_hist + r * 64;
        for (int i = tid; i < n; i += PR_THREADS) {
          const unsigned long long k = keys[i];
          if (k != 0ull && (k >> (shift + DIGIT_BITS)) == (x >> (shift + DIGIT_BITS)))
            atomicAdd(&hist[(int)((k >> shift) & 63ull)], 1);
        }
        __syncthreads();
        const int mine_c = hist[63 - lane];            // lane l looks at digit 63 - l
        const int incl = wave_prefix_sum(mine_c);      // matching keys with digit >= 63 - l
        const int l_hit = __ffsll((long long)__ballot(incl >= need)) - 1;  // never empty: need <= matching keys
        const int above = __builtin_amdgcn_readlane(incl - mine_c, l_hit);
        const int here = __builtin_amdgcn_readlane(mine_c, l_hit);  // matching keys with exactly this digit
        need -= above;
        x |= (unsigned long long)(63 - l_hit) << shift;
        // all of them are wanted: the digits fixed so far, followed by zeros, already separate the kept
        // keys from the others (the same values in every thread: the workgroup leaves the loop together)
        if (here == need) break;
      }
      for (int i = tid; i < n; i += PR_THREADS) nxt[i] = (i == 0) ? 1 : ((keys[i] != 0ull && keys[i] >= x) ? 1 : 0);
    } else {
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
  if (tid < 64) {
    // exclusive scan of the PR_THREADS chunk totals by one wave: PR_THREADS / 64 per lane
    constexpr int PER = PR_THREADS / 64;
    int loc[PER], tot = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      loc[q] = tot;
      tot += chunk_sum[tid * PER + q];
    }
    int incl = tot;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const int excl = incl - tot;
#pragma unroll
    for (int q = 0; q < PER; ++q) chunk_sum[tid * PER + q] = excl + loc[q];
    if (tid == 63) {
      ws_count[s] = incl;
      red[0] = incl;  // (red is idle by now; read after the next barrier)
    }
  }
  __syncthreads();
  int pos = chunk_sum[tid];
  for (int i = lo; i < hi; ++i) {
    const int k = ok[i] ? 1 : 0;
    ws_pos[o + i] = k ? pos : -1;
    if (emit) nxt[i] = k ? pos : -1;
    keep[o + i] = (uint8_t)k;
    pos += k;
    if (copy_out) {
      depth[o + i] = dep[i];
      cumlogp[o + i] = sum[i];
    }
  }
  if (emit) {
    // a single sequence: its packed offset is 0, so the renumbered tree can be written right here
    __syncthreads();
    if (tid == 0) {
      out_offsets[0] = 0;
      out_offsets[1] = red[0];
    }
    for (int i = tid; i < n; i += PR_THREADS) {
      const int p = nxt[i];
      if (p >= 0) {
        out_src[p] = i;
        out_parent[p] = (i == 0) ? -1 : nxt[par[i]];
      }
    }
    // the unused tail of the output arrays: rows that hang off the root and repeat it
    for (int i = red[0] + tid; i < NN; i += PR_THREADS) {
      out_src[i] = 0;
      out_parent[i] = 0;
    }
  }
}

__global__ __launch_bounds__(PR_THREADS) void k_prune_select(
    const int32_t* __restrict__ parent, const float* __restrict__ logc, const int32_t* __restrict__ node_offsets,
    const int32_t* __restrict__ node_counts, const int32_t* __restrict__ d_max, const float* __restrict__ theta, const int32_t* __restrict__ max_nodes,
    int32_t* __restrict__ depth, float* __restrict__ cumlogp, uint8_t* __restrict__ keep,
    int32_t* __restrict__ ws_pos, int32_t* __restrict__ ws_count, int32_t* __restrict__ ws_flag,
    int32_t* __restrict__ out_offsets, int32_t* __restrict__ out_src, int32_t* __restrict__ out_parent, int NN) {
  __shared__ int l_par[PR_LDS_NODES];
  __shared__ int l_dep[PR_LDS_NODES];
  __shared__ float l_sum[PR_LDS_NODES];
  __shared__ int l_ok[PR_LDS_NODES];
  __shared__ int l_new[PR_LDS_NODES];
  __shared__ unsigned long long l_keys[PR_LDS_NODES];
  __shared__ int digit_hist[N_DIGITS * 64];
  __shared__ float l_logc[PR_LDS_NODES];
  __shared__ int red[PR_THREADS / 64];
  __shared__ int chunk_sum[PR_THREADS];

  const int s = blockIdx.x, tid = threadIdx.x;
  const int o = node_offsets[s];
  const int n = node_counts != nullptr ? node_counts[s] : node_offsets[s + 1] - o;
  if (n <= 0) {
    if (tid == 0) {
      ws_count[s] = 0;
      if (gridDim.x == 1) out_offsets[0] = out_offsets[1] = 0;
    }
    if (gridDim.x == 1)
      for (int i = tid; i < NN; i += PR_THREADS) {
        out_src[i] = 0;
        out_parent[i] = 0;
      }
    return;
  }
  if (n <= PR_LDS_NODES) {
    // one round trip to global memory for the whole tree; everything after runs out of LDS
    const int dcap = d_max[s], budget = max_nodes[s];
    const float th = theta[s];
    for (int i = tid; i < n; i += PR_THREADS) {
      l_par[i] = parent[o + i];
      l_logc[i] = logc[o + i];
    }
    __syncthreads();
    prune_sequence(l_par, l_dep, l_sum, l_ok, l_new, l_keys, digit_hist, red, chunk_sum, n, o, true, l_logc, dcap, th, budget, depth, cumlogp, keep, ws_pos, ws_count, s,
                   gridDim.x == 1, out_offsets, out_src, out_parent, NN);
  } else {
    // very large trees: the output arrays and the workspace are the scratch (ws_pos is not written
    // before the last phase, so it can hold the budget flags meanwhile)
    prune_sequence(const_cast<int32_t*>(parent + o), depth + o, cumlogp + o, ws_flag + o, ws_pos + o, (unsigned long long*)nullptr, digit_hist, red,
                   chunk_sum, n, o, false, const_cast<float*>(logc + o), d_max[s], theta[s], max_nodes[s], depth, cumlogp,
                   keep, ws_pos, ws_count, s, false, out_offsets, out_src, out_parent, NN);
  }
}

__global__ __launch_bounds__(PR_THREADS) void k_prune_emit(const int32_t* __restrict__ parent,
                                                           const int32_t* __restrict__ node_offsets,
                                                           const int32_t* __restrict__ node_counts, int B,
                                                           const int32_t* __restrict__ ws_pos,
                                                           const int32_t* __restrict__ ws_count,
                                                           int32_t* __restrict__ out_offsets,
                                                           int32_t* __restrict__ out_src,
                                                           int32_t* __restrict__ out_parent, int NN) {
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
  const int n = node_counts != nullptr ? node_counts[s] : node_offsets[s + 1] - o;
  for (int i = tid; i < n; i += PR_THREADS) {
    const int p = ws_pos[o + i];
    if (p >= 0) {
      out_src[base + p] = i;
      out_parent[base + p] = (i == 0) ? -1 : ws_pos[o + parent[o + i]];
    }
  }
  // the unused tail of the output arrays (last workgroup): rows that hang off a root and repeat it
  if (s == B - 1)
    for (int i = base + ws_count[s] + tid; i < NN; i += PR_THREADS) {
      out_src[i] = 0;
      out_parent[i] = 0;
    }
}

}  // namespace hs

extern "C" size_t hs_tree_prune_workspace(int32_t B, int32_t NN) {
  if (B <= 0 || NN < 0) return 0;
  return 2 * hs::align_up((size_t)(NN > 0 ? NN : 1) * sizeof(int32_t), 256) +
         hs::align_up((size_t)B * sizeof(int32_t), 256);
}

// Validation and the two launches; `workspace` is the caller's buffer or this library's static one.
static hs_status prune_impl(const char* who, const int32_t* parent, const float* logc, const int32_t* node_offsets,
                            const int32_t* node_counts, int32_t B, int32_t NN, const int32_t* d_max,
                            const float* theta, const int32_t* max_nodes, int32_t* depth, float* cumlogp,
                            uint8_t* keep, int32_t* out_offsets, int32_t* out_src, int32_t* out_parent,
                            void* workspace, hs_stream stream) {
  (void)who;
  hs::Carver c(workspace);
  int32_t* ws_pos = c.take<int32_t>(NN > 0 ? NN : 1);
  int32_t* ws_flag = c.take<int32_t>(NN > 0 ? NN : 1);
  int32_t* ws_count = c.take<int32_t>(B);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(hs::k_prune_select, dim3(B), dim3(hs::PR_THREADS), 0, st, parent, logc, node_offsets, node_counts,
                     d_max, theta, max_nodes, depth, cumlogp, keep, ws_pos, ws_count, ws_flag, out_offsets, out_src,
                     out_parent, NN);
  hs_status r = hs::launch_status("prune select");
  if (r != HS_OK) return r;
  // a single tree that fits LDS was emitted by the selecting workgroup itself
  if (B == 1 && NN <= hs::PR_LDS_NODES) return r;
  hipLaunchKernelGGL(hs::k_prune_emit, dim3(B), dim3(hs::PR_THREADS), 0, st, parent, node_offsets, node_counts, B,
                     ws_pos, ws_count, out_offsets, out_src, out_parent, NN);
  return hs::launch_status("prune emit");
}

#define HS_PRUNE_CHECK_ARGS(who)                                                                                      \
  HS_REQUIRE(B >= 0 && NN >= 0, HS_ERR_SHAPE, who ": B=%d NN=%d", B, NN);                                             \
  if (B == 0) return HS_OK;                                                                                           \
  HS_REQUIRE(node_offsets && d_max && theta && max_nodes && out_offsets, HS_ERR_NULL, who ": NULL argument");         \
  HS_REQUIRE(NN == 0 || (parent && logc && depth && cumlogp && keep && out_src && out_parent), HS_ERR_NULL,           \
             who ": NULL node array")

extern "C" hs_status hs_tree_prune_counted(const int32_t* parent, const float* logc, const int32_t* node_offsets,
                                           const int32_t* node_counts, int32_t B, int32_t NN, const int32_t* d_max,
                                           const float* theta, const int32_t* max_nodes, int32_t* depth,
                                           float* cumlogp, uint8_t* keep, int32_t* out_offsets, int32_t* out_src,
                                           int32_t* out_parent, void* workspace, size_t workspace_bytes,
                                           hs_stream stream) {
  hs::clear_error();
  HS_PRUNE_CHECK_ARGS("hs_tree_prune");
  const size_t need = hs_tree_prune_workspace(B, NN);
  HS_REQUIRE(workspace && workspace_bytes >= need && reinterpret_cast<uintptr_t>(workspace) % 256 == 0,
             HS_ERR_WORKSPACE, "hs_tree_prune: workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
             workspace_bytes);
  return prune_impl("hs_tree_prune", parent, logc, node_offsets, node_counts, B, NN, d_max, theta, max_nodes, depth,
                    cumlogp, keep, out_offsets, out_src, out_parent, workspace, stream);
}

extern "C" hs_status hs_tree_prune(const int32_t* parent, const float* logc, const int32_t* node_offsets, int32_t B,
                                   int32_t NN, const int32_t* d_max, const float* theta, const int32_t* max_nodes,
                                   int32_t* depth, float* cumlogp, uint8_t* keep, int32_t* out_offsets,
                                   int32_t* out_src, int32_t* out_parent, void* workspace, size_t workspace_bytes,
                                   hs_stream stream) {
  return hs_tree_prune_counted(parent, logc, node_offsets, nullptr, B, NN, d_max, theta, max_nodes, depth, cumlogp,
                               keep, out_offsets, out_src, out_parent, workspace, workspace_bytes, stream);
}

// ---- hs_tree_prune_static: the same call for callers that cannot allocate (code under HIP graph
// capture, serving loops, harnesses that forbid hipMalloc).  Its scratch is a device array of this
// library, one copy per GPU, resolved once per device with hipGetSymbolAddress; every call on a GPU
// uses that GPU's copy, so calls that overlap on one GPU race.  Nothing in it has to start at zero:
// both kernels write every scratch entry they later read.
namespace {
constexpr int PRUNE_STATIC_MAX_NN = HS_PRUNE_STATIC_MAX_NODES;
constexpr int PRUNE_STATIC_MAX_B = HS_PRUNE_STATIC_MAX_SEQS;
constexpr size_t PRUNE_STATIC_BYTES = 2 * ((size_t)PRUNE_STATIC_MAX_NN * 4) + (size_t)PRUNE_STATIC_MAX_B * 4;  // 540672
constexpr int PRUNE_MAX_DEVICES = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[PRUNE_STATIC_BYTES];
static void* scratch_of_device[PRUNE_MAX_DEVICES];  // the array's address on each GPU, once resolved

// The address of `scratch` on the current device (in host code the array's name is only a handle).
static hs_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= PRUNE_MAX_DEVICES)
    return hs::fail(HS_ERR_RUNTIME, "hs_tree_prune_static: no current device (%s)", hipGetErrorString(e));
  void* p = __atomic_load_n(&scratch_of_device[dev], __ATOMIC_ACQUIRE);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr)
      return hs::fail(HS_ERR_RUNTIME, "hs_tree_prune_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    __atomic_store_n(&scratch_of_device[dev], p, __ATOMIC_RELEASE);  // (two threads may both resolve it: same value)
  }
  *out = p;
  return HS_OK;
}

extern "C" hs_status hs_tree_prune_static(const int32_t* parent, const float* logc, const int32_t* node_offsets,
                                          int32_t B, int32_t NN, const int32_t* d_max, const float* theta,
                                          const int32_t* max_nodes, int32_t* depth, float* cumlogp, uint8_t* keep,
                                          int32_t* out_offsets, int32_t* out_src, int32_t* out_parent,
                                          hs_stream stream) {
  hs::clear_error();
  HS_PRUNE_CHECK_ARGS("hs_tree_prune_static");
  HS_REQUIRE(B <= PRUNE_STATIC_MAX_B && NN <= PRUNE_STATIC_MAX_NN, HS_ERR_UNSUPPORTED,
             "hs_tree_prune_static: B=%d NN=%d exceed the static scratch (at most %d sequences, %d nodes); "
             "use hs_tree_prune with a workspace", B, NN, PRUNE_STATIC_MAX_B, PRUNE_STATIC_MAX_NN);
  static_assert(PRUNE_STATIC_MAX_NN % 64 == 0 && PRUNE_STATIC_MAX_B % 64 == 0, "the carved pieces stay 256-byte aligned");
  void* ws = nullptr;
  hs_status r = static_scratch(&ws);
  if (r != HS_OK) return r;
  return prune_impl("hs_tree_prune_static", parent, logc, node_offsets, nullptr, B, NN, d_max, theta, max_nodes, depth,
                    cumlogp, keep, out_offsets, out_src, out_parent, ws, stream);
}
