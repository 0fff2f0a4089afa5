// hs_adaptive_control: complexity quantification of a draft tree and the decision that follows it
// (Section 4.1: cumulative meta-path Top-K entropy Phi of the operational path P*, Eq. 1;
// Section 4.2: entropy bins; Section 4.3: depth extension d' and node budget N').
//
// Nothing to stream: a few hundred nodes per sequence, one workgroup per sequence, no workspace.
// The parent pointers are staged in LDS (trees of up to 8192 rows; larger ones are walked in global
// memory).  Every node finds its depth by walking to the root; the nodes of the deepest level form their
// value root-first (the float32 add per node of the reranking step, so the choice of P* is taken
// on the same numbers as the pruning that follows); one 64-bit (value, row) key per node and a
// workgroup maximum pick P*; one thread then sums the path's entropies root-first in float32 and
// looks up the bin.
#include <limits.h>

#include "hs_common.h"

namespace hs {

constexpr int CTL_THREADS = 256;
constexpr int CTL_MAX_BINS = 64;
constexpr int CTL_MAX_LOW = 8;
constexpr int CTL_LDS_NODES = 8192;

struct ControlArgs {
  const int32_t* parent;
  const float* logc;
  const float* ent;
  const int32_t* node_offsets;
  const int32_t* node_counts;
  int n_edges, n_low, alpha, d_base, n_default, mode;
  float edges[CTL_MAX_BINS - 1];
  float gamma[CTL_MAX_LOW];
  float* phi;
  int32_t* pstar;
  int32_t* bin;
  int32_t* d_prime;
  int32_t* n_prime;
};

// What bin b means (Section 4.3): depth extension and node budget.  One definition for the kernel and
// for the host query hs_adaptive_policy.
__host__ __device__ inline void bin_policy(int b, int n_low, int alpha, int d_base, int n_default, const float* gamma,
                                           int* d_prime, int* n_prime) {
  int delta = 0, budget = n_default;
  if (b < n_low) {
    delta = alpha - b > 0 ? alpha - b : 0;
    budget = (int)floor((double)gamma[b] * (double)n_default + 0.5) + delta;
  }
  *d_prime = d_base + delta;
  *n_prime = budget;
}

// (value, row) as one key: larger key = larger value, then lower row; never 0 for a real node.
__device__ __forceinline__ unsigned long long control_key(float v, int i) {
  unsigned u = __builtin_bit_cast(unsigned, v);
  u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;  // monotone map of float order onto unsigned order
  return ((unsigned long long)u << 32) | (unsigned)(0x7fffffff - i);
}

// The ancestor of node i that is `up` levels above it.
template <typename IP>
__device__ __forceinline__ int ancestor(IP par, int i, int up) {
  for (; up > 0; --up) i = par[i];
  return i;
}

// The decision for one sequence; `par` points to LDS or to global memory.
template <typename IP>
__device__ __forceinline__ void control_sequence(const ControlArgs& a, int s, int n, IP par,
                                                 const float* __restrict__ lc, const float* __restrict__ ent,
                                                 int* red_i, unsigned long long* red_k) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // deepest level
  int my_max = 0;
  for (int i = tid; i < n; i += CTL_THREADS) {
    int d = 0;
    for (int j = par[i]; j >= 0; j = par[j]) ++d;
    my_max = max(my_max, d);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) my_max = max(my_max, __shfl_xor(my_max, off));
  if (lane == 0) red_i[wave] = my_max;
  __syncthreads();
  int D = red_i[0];
  for (int w = 1; w < CTL_THREADS / 64; ++w) D = max(D, red_i[w]);

  // best node of that level
  unsigned long long best = 0ull;
  for (int i = tid; i < n; i += CTL_THREADS) {
    int d = 0;
    for (int j = par[i]; j >= 0; j = par[j]) ++d;
    if (d != D) continue;
    float v;
    if (a.mode == 0) {
      v = 0.f;  // value of the root; then one float32 add per level, root first
      for (int t = 1; t <= D; ++t) v = v + fminf(lc[ancestor(par, i, D - t)], 0.f);
    } else {
      v = i == 0 ? 0.f : fminf(lc[i], 0.f);
    }
    const unsigned long long k = control_key(v, i);
    best = k > best ? k : best;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long other = __shfl_xor(best, off);
    best = other > best ? other : best;
  }
  if (lane == 0) red_k[wave] = best;
  __syncthreads();
  if (tid >= 64) return;  // the first wave finishes (no barrier from here on)
  for (int w = 1; w < CTL_THREADS / 64; ++w) best = red_k[w] > best ? red_k[w] : best;
  const int p = 0x7fffffff - (int)(unsigned)(best & 0xffffffffull);

  // Eq. 1 along the path to P*: the rows of its strict ancestors, root first.  The lanes fetch 64
  // path entries at a time side by side (one round trip instead of one per level); the float32 sum
  // still takes them one by one in path order.
  float acc = 0.f;
  for (int t0 = 0; t0 < D; t0 += 64) {
    const int t = t0 + lane;
    const float e = t < D ? ent[ancestor(par, p, D - t)] : 0.f;
    const int m = D - t0 < 64 ? D - t0 : 64;
    for (int l = 0; l < m; ++l) acc = acc + __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, e), l));
  }
  if (lane != 0) return;
  int b = 0;
  for (int e = 0; e < a.n_edges; ++e) b += acc >= a.edges[e] ? 1 : 0;
  int dp, np_;
  bin_policy(b, a.n_low, a.alpha, a.d_base, a.n_default, a.gamma, &dp, &np_);
  a.phi[s] = acc;
  a.pstar[s] = p;
  a.bin[s] = b;
  a.d_prime[s] = dp;
  a.n_prime[s] = np_;
}

__global__ __launch_bounds__(CTL_THREADS) void k_adaptive_control(ControlArgs a) {
  __shared__ int red_i[CTL_THREADS / 64];
  __shared__ unsigned long long red_k[CTL_THREADS / 64];
  __shared__ int par_lds[CTL_LDS_NODES];
  const int s = blockIdx.x, tid = threadIdx.x;
  const int o = a.node_offsets[s];
  const int n = a.node_counts != nullptr ? a.node_counts[s] : a.node_offsets[s + 1] - o;
  if (n <= 0) {
    if (tid == 0) {
      a.phi[s] = 0.f;
      a.pstar[s] = -1;
      a.bin[s] = 0;
      a.d_prime[s] = a.d_base;
      a.n_prime[s] = a.n_default;
    }
    return;
  }
  const float* __restrict__ lc = a.logc + o;
  const float* __restrict__ ent = a.ent + o;
  if (n <= CTL_LDS_NODES) {
    for (int i = tid; i < n; i += CTL_THREADS) par_lds[i] = a.parent[o + i];
    __syncthreads();
    control_sequence(a, s, n, (const int*)par_lds, lc, ent, red_i, red_k);
  } else {
    control_sequence(a, s, n, a.parent + o, lc, ent, red_i, red_k);
  }
}

}  // namespace hs

using namespace hs;

extern "C" hs_status hs_adaptive_control(const int32_t* parent, const float* logc, const float* ent,
                                         const int32_t* node_offsets, const int32_t* node_counts, int32_t B,
                                         int32_t NN, const float* host_bin_edges, int32_t n_bins, const float* host_gamma,
                                         int32_t n_low, int32_t alpha, int32_t d_base, int32_t n_default,
                                         hs_pstar_mode mode, float* phi, int32_t* pstar, int32_t* bin,
                                         int32_t* d_prime, int32_t* n_prime, hs_stream stream) {
  clear_error();
  HS_REQUIRE(B >= 0 && NN >= 0, HS_ERR_SHAPE, "hs_adaptive_control: B=%d NN=%d", B, NN);
  HS_REQUIRE(n_bins >= 1 && n_bins <= CTL_MAX_BINS, HS_ERR_SHAPE, "hs_adaptive_control: n_bins=%d must be in 1..%d",
             n_bins, CTL_MAX_BINS);
  HS_REQUIRE(n_low >= 0 && n_low <= CTL_MAX_LOW && n_low <= n_bins, HS_ERR_SHAPE,
             "hs_adaptive_control: n_low=%d must be in 0..min(%d, n_bins)", n_low, CTL_MAX_LOW);
  HS_REQUIRE(mode == HS_PSTAR_CUMULATIVE || mode == HS_PSTAR_LOCAL, HS_ERR_SHAPE, "hs_adaptive_control: mode %d",
             (int)mode);
  HS_REQUIRE(d_base >= 0 && n_default >= 0, HS_ERR_SHAPE, "hs_adaptive_control: d_base=%d n_default=%d", d_base,
             n_default);
  HS_REQUIRE((n_bins == 1 || host_bin_edges) && (n_low == 0 || host_gamma), HS_ERR_NULL,
             "hs_adaptive_control: NULL bin boundaries or gamma");
  for (int e = 0; e + 2 < n_bins; ++e)
    HS_REQUIRE(host_bin_edges[e] <= host_bin_edges[e + 1], HS_ERR_SHAPE,
               "hs_adaptive_control: bin boundaries must not decrease (entry %d)", e + 1);
  if (B == 0) return HS_OK;
  HS_REQUIRE(node_offsets && phi && pstar && bin && d_prime && n_prime, HS_ERR_NULL, "hs_adaptive_control: NULL argument");
  HS_REQUIRE(NN == 0 || (parent && logc && ent), HS_ERR_NULL, "hs_adaptive_control: NULL tree");
  ControlArgs a;
  a.parent = parent; a.logc = logc; a.ent = ent; a.node_offsets = node_offsets; a.node_counts = node_counts;
  a.n_edges = n_bins - 1; a.n_low = n_low; a.alpha = alpha; a.d_base = d_base; a.n_default = n_default;
  a.mode = (int)mode;
  for (int e = 0; e < CTL_MAX_BINS - 1; ++e) a.edges[e] = e < n_bins - 1 ? host_bin_edges[e] : 0.f;
  for (int e = 0; e < CTL_MAX_LOW; ++e) a.gamma[e] = e < n_low ? host_gamma[e] : 0.f;
  a.phi = phi; a.pstar = pstar; a.bin = bin; a.d_prime = d_prime; a.n_prime = n_prime;
  hipLaunchKernelGGL(k_adaptive_control, dim3((unsigned)B), dim3(CTL_THREADS), 0, static_cast<hipStream_t>(stream), a);
  return launch_status("adaptive control");
}

extern "C" hs_status hs_adaptive_policy(int32_t bin, const float* host_gamma, int32_t n_low, int32_t alpha,
                                        int32_t d_base, int32_t n_default, int32_t* host_d_prime,
                                        int32_t* host_n_prime) {
  clear_error();
  HS_REQUIRE(bin >= 0 && n_low >= 0 && n_low <= CTL_MAX_LOW && d_base >= 0 && n_default >= 0, HS_ERR_SHAPE,
             "hs_adaptive_policy: bin=%d n_low=%d d_base=%d n_default=%d", bin, n_low, d_base, n_default);
  HS_REQUIRE(host_d_prime && host_n_prime && (n_low == 0 || host_gamma), HS_ERR_NULL, "hs_adaptive_policy: NULL argument");
  int dp, np_;
  bin_policy(bin, n_low, alpha, d_base, n_default, host_gamma, &dp, &np_);
  *host_d_prime = dp;
  *host_n_prime = np_;
  return HS_OK;
}
