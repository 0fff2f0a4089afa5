// hs_verify_accept: the accept walk over a verified draft tree (Section 2.1 acceptance rule, applied
// to the children of each node in turn).
//
// Stage A (all rows in parallel, HBM-bound): the row scan finds every target row's argmax and
// softmax normaliser (and every draft row's normaliser in the stochastic modes).
// Stage B (one workgroup per sequence, latency-bound):
//   greedy      every node checks in parallel whether its whole root path is confirmed by the
//               target's argmax; the deepest confirmed node is the end of the accepted path.
//   stochastic  the walk is serial by nature, but what a node's children face is not: the state
//               after j rejections at a node depends on the node and j alone, not on the path that
//               led there.  Per rejection the normaliser of the residual distribution needs one
//               cooperative pass over the node's two vocabulary rows; the residual itself is never
//               materialised: after j rejections it is max(p(v) - beta_j q(v), 0) for every token
//               not yet rejected (beta_j a scalar that accumulates Z_i / (1 - sum of rejected q)),
//               and frozen at its value of the time for a rejected token.  So one workgroup per
//               node with children runs that node's chain of rejections ahead of the walk, all
//               nodes in parallel (k_accept_chain), and leaves each child's pair of current
//               probabilities; the walk itself (k_accept_walk, one workgroup per sequence) then
//               only compares uniforms with them, and draws the bonus token at the node where it
//               stops: an inverse-CDF search done as row sums of 64 tokens, a scan of the row sums,
//               and a scan inside the one row that is hit.
#include <limits.h>

#include "hs_common.h"

namespace hs {

constexpr int GR_THREADS = 256;
constexpr int AC_THREADS = 1024;
constexpr int AC_WAVES = AC_THREADS / 64;
constexpr int AC_MAX_KIDS = 256;    // children tried per node
constexpr int AC_MAX_ROWS = 8192;   // 64-token rows of the CDF search held in LDS (V <= 524288)
constexpr int AC_LIST_NODES = 4096; // calls with up to this many tree rows get a list of live tokens per row

// A node's list of live tokens holds one region per wave of its workgroup: the wave's share of the
// vocabulary (float4 index tid + k * AC_THREADS, plus a lane's token of the last V % 4).
static __host__ __device__ inline int64_t list_wave_cap(int V) {
  return (((int64_t)(V >> 2) + AC_THREADS - 1) / AC_THREADS) * 256 + 64;
}

// ----------------------------------------------------------------------------------- greedy
// With n_slices > 1 the target rows' argmax arrives as one (value, index) pair per row slice
// (the row scan's merge launch is folded into this kernel): the best pair under (value
// descending, index ascending) is the row's argmax, stored in `arg` for the walk.
__global__ __launch_bounds__(GR_THREADS) void k_accept_greedy(int32_t* __restrict__ arg,
                                                              const float* __restrict__ slice_val,
                                                              const int32_t* __restrict__ slice_idx, int n_slices,
                                                              const int32_t* __restrict__ token,
                                                              const int32_t* __restrict__ parent,
                                                              const int32_t* __restrict__ node_offsets,
                                                              int max_depth, int32_t* __restrict__ accept_len,
                                                              int32_t* __restrict__ accept_path,
                                                              int32_t* __restrict__ bonus_token) {
  __shared__ long long red[GR_THREADS / 64];
  const int s = blockIdx.x, tid = threadIdx.x;
  const int o = node_offsets[s];
  const int n = node_offsets[s + 1] - o;
  int32_t* path = accept_path + (int64_t)s * max_depth;
  for (int d = tid; d < max_depth; d += GR_THREADS) path[d] = -1;
  if (n <= 0) {
    if (tid == 0) {
      accept_len[s] = 0;
      bonus_token[s] = -1;
    }
    return;
  }
  if (n_slices > 1) {
    for (int i = tid; i < n; i += GR_THREADS) {
      const int64_t base = (int64_t)(o + i) * n_slices;
      float bv = slice_val[base];
      int bi = slice_idx[base];
      for (int q = 1; q < n_slices; ++q) {
        const float v = slice_val[base + q];
        const int x = slice_idx[base + q];
        if (better(v, x, bv, bi)) {
          bv = v;
          bi = x;
        }
      }
      arg[o + i] = bi;
    }
    __syncthreads();  // every row's argmax is visible to the workgroup
  }
  // key = depth of a fully confirmed node (higher wins), then lower index
  long long best = ((long long)0 << 32) | (unsigned)(INT_MAX - 0);  // the root: depth 0
  for (int i = tid; i < n; i += GR_THREADS) {
    bool ok = true;
    int d = 0;
    for (int j = i; j > 0;) {
      const int p = parent[o + j];
      ok = ok && (token[o + j] == arg[o + p]);
      j = p;
      ++d;
    }
    if (ok && d <= max_depth) {
      long long key = ((long long)d << 32) | (unsigned)(INT_MAX - i);
      best = key > best ? key : best;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    long long other = __shfl_xor(best, off);
    best = other > best ? other : best;
  }
  if ((tid & 63) == 0) red[tid >> 6] = best;
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < GR_THREADS / 64; ++w) best = red[w] > best ? red[w] : best;
    const int d = (int)(best >> 32);
    int node = INT_MAX - (int)(best & 0xffffffffll);
    accept_len[s] = d;
    bonus_token[s] = arg[o + node];
    for (int k = d - 1; k >= 0; --k) {
      path[k] = node;
      node = parent[o + node];
    }
  }
}

// ----------------------------------------------------------------------------------- stochastic
// A row of logits as probabilities: p(v) = exp((x[v] - m) / T + lz) with m the row's maximum and
// lz = -ln(sum exp((x - m) / T)), evaluated as exp2((x[v] - m) * c1 + c2): a subtraction, a fused
// multiply-add and the exponential instruction per token.
struct RowView {
  const float* x;  // logits row
  float m;         // its maximum
  float c1;        // log2(e) / T
  float c2;        // log2(e) * lz
  __device__ __forceinline__ RowView(const float* row, float max_logit, float lz, float inv_t)
      : x(row), m(max_logit), c1(inv_t * 1.4426950408889634f), c2(lz * 1.4426950408889634f) {}
  __device__ __forceinline__ float of(float logit) const { return exp2_fast(fmaf(logit - m, c1, c2)); }
  __device__ __forceinline__ float prob(int v) const { return of(x[v]); }
  __device__ __forceinline__ float4 of4(const float4 f) const { return make_float4(of(f.x), of(f.y), of(f.z), of(f.w)); }
  // tokens 4 i .. 4 i + 3 with one 16-byte load (the row must be 16-byte aligned)
  __device__ __forceinline__ float4 prob4(int i) const { return of4(reinterpret_cast<const float4*>(x)[i]); }
  __device__ __forceinline__ bool aligned16() const { return reinterpret_cast<uintptr_t>(x) % 16 == 0; }
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

__device__ __forceinline__ double wave_incl_scan(double v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    double o = __shfl_up(v, off);
    if (lane >= off) v += o;
  }
  return v;
}

// Sum of max(p(v) - beta q(v), 0) over the vocabulary, all threads of the workgroup; the result is
// the same in every thread.  Terms are formed in float32 (relative error 2^-24 of p(v)), summed in
// four float32 partial sums per thread over about V / (4 * threads) terms each, then in float64.
__device__ __forceinline__ double residual_mass(const RowView& p, const RowView& q, double beta, int V, double* red) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float bf = (float)beta;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  int v = tid;  // first token of the scalar part
  if (p.aligned16() && q.aligned16()) {
    // 16-byte loads, four of each row in flight per thread: a single compute unit streams the two
    // rows, so what is in flight bounds the pass
    const int n4 = V >> 2;
#pragma unroll 4
    for (int i = tid; i < n4; i += AC_THREADS) {
      const float4 pp = p.prob4(i), qq = q.prob4(i);
      a0 += fmaxf(fmaf(-bf, qq.x, pp.x), 0.f);
      a1 += fmaxf(fmaf(-bf, qq.y, pp.y), 0.f);
      a2 += fmaxf(fmaf(-bf, qq.z, pp.z), 0.f);
      a3 += fmaxf(fmaf(-bf, qq.w, pp.w), 0.f);
    }
    v = (n4 << 2) + tid;
  }
  for (; v < V; v += AC_THREADS) a0 += fmaxf(fmaf(-bf, q.prob(v), p.prob(v)), 0.f);
  double acc = wave_sum(((double)a0 + (double)a1) + ((double)a2 + (double)a3));
  __syncthreads();  // red is free
  if (lane == 0) red[wave] = acc;
  __syncthreads();
  double F = 0.0;
  for (int w = 0; w < AC_WAVES; ++w) F += red[w];
  return F;
}

// Sum over the workgroup of per-thread partial sums: four float32 partials per thread, then float64.
// The two barriers order LDS traffic only (they do not wait for global stores: a wave's list is
// read by that wave alone, and what thread 0 writes for the walk is read by a later kernel).
__device__ __forceinline__ double block_total(float a0, float a1, float a2, float a3, double* red) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  double acc = wave_sum(((double)a0 + (double)a1) + ((double)a2 + (double)a3));
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // red is free
  if (lane == 0) red[wave] = acc;
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  double F = 0.0;
  for (int w = 0; w < AC_WAVES; ++w) F += red[w];
  return F;
}

// A wave's list of live tokens in global memory, written through a ring of AC_RING pairs in LDS.
// A store instruction costs the same whether it carries 64 lanes or a few, so the pairs that pass
// are first packed in LDS and leave for global memory 128 at a time (16 bytes per lane).  Four
// pairs per lane are appended per call, without branches: one prefix sum over the lanes' counts
// gives each lane its first position, and a pair that does not pass is written to a slot of the
// lane's own behind the ring instead.  Order of the list: lane, then slot.
constexpr int AC_RING = 1024;
struct ListWriter {
  float2* __restrict__ wl;  // the wave's region
  float2* ring;             // the wave's ring in LDS: AC_RING pairs and 64 more, one per lane, that are never read
  int w;                    // pairs in global memory so far (a multiple of 128 until finish())
  int staged;               // pairs in the ring, from position w % AC_RING on (fewer than 128 between calls)
  bool keep;                // the whole list (at most AC_RING pairs) stays in the ring: nothing goes to global memory
  __device__ __forceinline__ void append4(const bool (&live)[4], const float (&pv)[4], const float (&qv)[4]) {
    const int lane = threadIdx.x & 63;
    int c[4];
    c[0] = live[0] ? 1 : 0;
#pragma unroll
    for (int k = 1; k < 4; ++k) c[k] = c[k - 1] + (live[k] ? 1 : 0);
    const int incl = wave_prefix_sum(c[3]);
    const int total = __builtin_amdgcn_readlane(incl, 63);
    const int first = w + staged + incl - c[3];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int at = (first + (k ? c[k - 1] : 0)) & (AC_RING - 1);
      ring[live[k] ? at : AC_RING + lane] = make_float2(pv[k], qv[k]);
    }
    staged += total;
    while (!keep && staged >= 128) {  // (the same decision in every lane; at most three rounds)
      __builtin_amdgcn_wave_barrier();
      const float4 v = *reinterpret_cast<const float4*>(&ring[(w & (AC_RING - 1)) + 2 * lane]);
      *reinterpret_cast<float4*>(&wl[w + 2 * lane]) = v;
      w += 128;
      staged -= 128;
    }
  }
  __device__ __forceinline__ void finish() {
    __builtin_amdgcn_wave_barrier();
    if (keep) return;
    for (int i = threadIdx.x & 63; i < staged; i += 64) wl[w + i] = ring[(w + i) & (AC_RING - 1)];
    w += staged;
    staged = 0;
  }
};

// residual_mass for the first rejection at a node that has more to come: the same sum, and every
// token whose term is positive leaves its pair (p(v), q(v)) in its wave's list.  beta only grows
// along a chain, so a token whose term has reached zero stays out of every later sum: the later
// passes (residual_mass_list) read the lists instead of the two vocabulary rows and evaluate no
// exponentials.  Both rows must be 16-byte aligned and V >= 4 * AC_THREADS.  The order of a list is
// fixed by the data (iteration, component, lane), so the sums are the same from run to run.
// The logits of the next four iterations are requested before the current four are worked on (all
// loads unconditional, out-of-range lanes re-read the last element): the stores into the list keep
// the compiler from moving loads, so the overlap has to be written out.
__device__ __forceinline__ double residual_mass_build(const RowView& p, const RowView& q, double beta, int V,
                                                      double* red, float2* __restrict__ wl, float2* ring,
                                                      int& wcount) {
  const int tid = threadIdx.x;
  const float bf = (float)beta;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  const int n4 = V >> 2;
  const int n_it = (n4 + AC_THREADS - 1) / AC_THREADS;  // the same for every thread: the ballots need whole waves
  const float4* __restrict__ px = reinterpret_cast<const float4*>(p.x);
  const float4* __restrict__ qx = reinterpret_cast<const float4*>(q.x);
  float4 fp[4], fq[4], np_[4], nq_[4];
  auto fetch = [&](int k0, float4 (&dp)[4], float4 (&dq)[4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = min(tid + (k0 + u) * AC_THREADS, n4 - 1);
      dp[u] = px[i];
      dq[u] = qx[i];
    }
  };
  ListWriter out{wl, ring, 0, 0, false};
  fetch(0, fp, fq);
  for (int k0 = 0; k0 < n_it; k0 += 4) {
    fetch(k0 + 4, np_, nq_);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (k0 + u < n_it) {
        const bool in = tid + (k0 + u) * AC_THREADS < n4;
        const float4 pp = p.of4(fp[u]), qq = q.of4(fq[u]);
        const float t0 = in ? fmaxf(fmaf(-bf, qq.x, pp.x), 0.f) : 0.f;
        const float t1 = in ? fmaxf(fmaf(-bf, qq.y, pp.y), 0.f) : 0.f;
        const float t2 = in ? fmaxf(fmaf(-bf, qq.z, pp.z), 0.f) : 0.f;
        const float t3 = in ? fmaxf(fmaf(-bf, qq.w, pp.w), 0.f) : 0.f;
        a0 += t0;
        a1 += t1;
        a2 += t2;
        a3 += t3;
        const bool live[4] = {t0 > 0.f, t1 > 0.f, t2 > 0.f, t3 > 0.f};
        const float pv[4] = {pp.x, pp.y, pp.z, pp.w}, qv[4] = {qq.x, qq.y, qq.z, qq.w};
        out.append4(live, pv, qv);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      fp[u] = np_[u];
      fq[u] = nq_[u];
    }
  }
  {  // the last V % 4 tokens
    const int v = (n4 << 2) + tid;
    float pv = 0.f, qv = 0.f, t = 0.f;
    if (v < V) {
      pv = p.prob(v);
      qv = q.prob(v);
      t = fmaxf(fmaf(-bf, qv, pv), 0.f);
    }
    a0 += t;
    const bool live[4] = {t > 0.f, false, false, false};
    const float pv4[4] = {pv, 0.f, 0.f, 0.f}, qv4[4] = {qv, 0.f, 0.f, 0.f};
    out.append4(live, pv4, qv4);
  }
  out.finish();
  wcount = out.w;
  return block_total(a0, a1, a2, a3, red);
}

// residual_mass over the lists that residual_mass_build left (two pairs per lane and load).  With
// `compact` the pairs whose term is still positive move to the front of the list, in place: a pair
// is written at or before the position it was read from, and the group of pairs that is read ahead
// lies behind every position written meanwhile.  A list of at most AC_RING pairs moves into the
// wave's ring in LDS and stays there (IN_LDS: it is read from the ring), which takes the round trips
// to memory out of the short passes at the end of a long chain.
// This is the wave's own part of the pass (a[] receives the lanes' four partial sums): waves of a
// workgroup may take different instantiations, so the workgroup's barriers stay with the caller.
template <bool IN_LDS>
__device__ __forceinline__ void residual_mass_list(double beta, float2* __restrict__ wl, float2* ring, int& wcount,
                                                   bool& in_lds, bool compact, float (&a)[4]) {
  constexpr int LU = 4;  // loads per lane and group: 512 pairs per wave
  const int lane = threadIdx.x & 63;
  const float bf = (float)beta;
  const int n = wcount;
  const int last2 = n > 1 ? (n - 1) >> 1 : 0;  // last float4 that holds a pair (list and ring hold 64 pairs at least)
  const float4* src = IN_LDS ? reinterpret_cast<const float4*>(ring) : reinterpret_cast<const float4*>(wl);
  float4 cur[LU], nxt[LU];
  auto fetch = [&](int base, float4 (&e)[LU]) {  // unconditional: lanes past the end re-read the last pairs
#pragma unroll
    for (int u = 0; u < LU; ++u) e[u] = src[min((base >> 1) + u * 64 + lane, last2)];
  };
  ListWriter out{wl, ring, 0, 0, n <= AC_RING};
  fetch(0, cur);
  for (int base = 0; base < n; base += LU * 128) {
    fetch(base + LU * 128, nxt);
#pragma unroll
    for (int u = 0; u < LU; u += 2) {
      const int i0 = base + u * 128 + 2 * lane, i1 = i0 + 128;
      const float t0 = i0 < n ? fmaxf(fmaf(-bf, cur[u].y, cur[u].x), 0.f) : 0.f;
      const float t1 = i0 + 1 < n ? fmaxf(fmaf(-bf, cur[u].w, cur[u].z), 0.f) : 0.f;
      const float t2 = i1 < n ? fmaxf(fmaf(-bf, cur[u + 1].y, cur[u + 1].x), 0.f) : 0.f;
      const float t3 = i1 + 1 < n ? fmaxf(fmaf(-bf, cur[u + 1].w, cur[u + 1].z), 0.f) : 0.f;
      a[0] += t0;
      a[1] += t1;
      a[2] += t2;
      a[3] += t3;
      if (compact) {
        const bool live[4] = {t0 > 0.f, t1 > 0.f, t2 > 0.f, t3 > 0.f};
        const float pv[4] = {cur[u].x, cur[u].z, cur[u + 1].x, cur[u + 1].z};
        const float qv[4] = {cur[u].y, cur[u].w, cur[u + 1].y, cur[u + 1].w};
        out.append4(live, pv, qv);
      }
    }
#pragma unroll
    for (int u = 0; u < LU; ++u) cur[u] = nxt[u];
  }
  if (compact) {
    out.finish();
    wcount = out.keep ? out.staged : out.w;
    in_lds = out.keep;
  }
}

// The same term for one token, as residual_mass forms it (used to take a frozen token's live term
// out of the sum again).
__device__ __forceinline__ double residual_term(const RowView& p, const RowView& q, double beta, int v) {
  return (double)fmaxf(fmaf(-(float)beta, q.prob(v), p.prob(v)), 0.f);
}
// Weight of token v in the distribution the bonus token is drawn from (frozen tokens aside).
__device__ __forceinline__ double token_weight(const RowView& p, const RowView& q, bool use_q, double beta, int v) {
  return use_q ? residual_term(p, q, beta, v) : (double)p.prob(v);
}

// Children of local row `cur` of a sequence of n rows, ascending, into kids_sorted; returns their
// number (at most AC_MAX_KIDS).  Called by all threads; ends with a barrier.
__device__ __forceinline__ int gather_children(const int32_t* __restrict__ parent, int o, int n, int cur, bool any,
                                               int* kids, int* kids_sorted, int* n_kids) {
  const int tid = threadIdx.x;
  if (tid == 0) *n_kids = 0;
  __syncthreads();
  if (any)
    for (int i = 1 + tid; i < n; i += AC_THREADS)
      if (parent[o + i] == cur) {
        int pos = atomicAdd(n_kids, 1);
        if (pos < AC_MAX_KIDS) kids[pos] = i;
      }
  __syncthreads();
  const int nk = *n_kids < AC_MAX_KIDS ? *n_kids : AC_MAX_KIDS;
  if (tid < nk) {
    int me = kids[tid], r = 0;
    for (int j = 0; j < nk; ++j) r += kids[j] < me ? 1 : 0;
    kids_sorted[r] = me;
  }
  __syncthreads();
  return nk;
}

// What the stochastic walk needs from a node's chain of rejections.
struct ChainOut {
  double* child_p;       // [NN] current target probability of the child's token when its turn comes
  double* child_q;       // [NN] current draft probability of it
  double* child_frozen;  // [NN] its weight in the residual after its own rejection
  double* node_beta;     // [NN] beta and normaliser after all of the node's children were rejected
  double* node_Z;
};

// One workgroup per tree row that has children (others leave at once): the chain of rejections at
// that node under the ratio rule, every child rejected in turn.
__global__ __launch_bounds__(AC_THREADS) void k_accept_chain(
    const float* __restrict__ target, const float* __restrict__ draft, int64_t row_stride,
    const int32_t* __restrict__ token, const int32_t* __restrict__ parent, const int32_t* __restrict__ node_offsets,
    int B, int V, float inv_t, int max_depth, const int32_t* __restrict__ t_arg, const float* __restrict__ t_lz,
    const int32_t* __restrict__ d_arg, const float* __restrict__ d_lz, ChainOut out, float2* __restrict__ lists) {
  __shared__ int kids[AC_MAX_KIDS];
  __shared__ int kids_sorted[AC_MAX_KIDS];
  __shared__ int n_kids;
  __shared__ double rej_w[AC_MAX_KIDS];
  __shared__ float kid_p[AC_MAX_KIDS], kid_q[AC_MAX_KIDS];  // p(x), q(x) of each child's token
  __shared__ __attribute__((aligned(16))) float2 rings[AC_WAVES][AC_RING + 64];  // see ListWriter
  __shared__ double red[AC_WAVES];
  const int g = blockIdx.x, tid = threadIdx.x;
  int lo = 0, hi = B;  // sequence of this row: last s with node_offsets[s] <= g
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (node_offsets[mid] <= g) lo = mid; else hi = mid;
  }
  const int o = node_offsets[lo];
  const int n = node_offsets[lo + 1] - o;
  const int cur = g - o;
  if (cur >= n) return;  // (an empty sequence before this row's: cannot happen, offsets are monotone)
  // (row statistics first: these loads do not depend on the tree)
  const float p_lz = t_lz[g], q_lz = d_lz[g];
  const int p_arg = t_arg[g], q_arg = d_arg[g];
  int depth = 0;
  for (int j = parent[o + cur]; j >= 0; j = parent[o + j]) ++depth;
  const int nk = gather_children(parent, o, n, cur, depth < max_depth, kids, kids_sorted, &n_kids);
  if (nk == 0) return;
  const float* p_row = target + (int64_t)g * row_stride;
  const float* q_row = draft + (int64_t)g * row_stride;
  const RowView p(p_row, p_row[p_arg], p_lz, inv_t);
  const RowView q(q_row, q_row[q_arg], q_lz, inv_t);
  // every child's token and its two probabilities, fetched side by side: the chain below is serial,
  // and a round trip to memory per step would dominate it
  if (tid < nk) {
    const int x = token[o + kids_sorted[tid]];
    kid_p[tid] = p.prob(x);
    kid_q[tid] = q.prob(x);
  }
  __syncthreads();
  // lists of live tokens (`lists` may be NULL): worth their stores when a second rejection follows
  const bool use_list = lists != nullptr && nk >= 2 && V >= 4 * AC_THREADS && p.aligned16() && q.aligned16();
  float2* __restrict__ wl = use_list ? lists + ((int64_t)g * AC_WAVES + (tid >> 6)) * list_wave_cap(V) : nullptr;
  float2* ring = rings[tid >> 6];
  int wcount = 0;
  bool in_lds = false;  // (per wave)
  double beta = 0.0, Z = 1.0, sumq = 0.0;
  for (int j = 0; j < nk; ++j) {
    const int c = kids_sorted[j];
    const double px = (double)kid_p[j];
    const double qx = (double)kid_q[j];
    const double pc = fmax(px - beta * qx, 0.0) / Z;  // current p(x)
    const double qc = qx / (1.0 - sumq);              // current q(x)
    // rejected: p <- norm(max(p - q, 0)), q(x) <- 0, q <- norm(q)
    beta += Z / (1.0 - sumq);
    sumq += qx;
    const double frozen = fmax(px - beta * qx, 0.0);
    if (tid == 0) {
      out.child_p[o + c] = pc;
      out.child_q[o + c] = qc;
      out.child_frozen[o + c] = frozen;
      rej_w[j] = frozen;
    }
    double F;  // (the barriers of a pass also publish rej_w)
    if (!use_list) F = residual_mass(p, q, beta, V, red);
    else if (j == 0) F = residual_mass_build(p, q, beta, V, red, wl, ring, wcount);
    else {
      float a[4] = {0.f, 0.f, 0.f, 0.f};
      if (__builtin_amdgcn_readfirstlane((int)in_lds)) residual_mass_list<true>(beta, wl, ring, wcount, in_lds, j + 1 < nk, a);
      else residual_mass_list<false>(beta, wl, ring, wcount, in_lds, j + 1 < nk, a);
      F = block_total(a[0], a[1], a[2], a[3], red);
    }
    // a rejected token's weight is frozen: its live term (as the passes form it) leaves the sum
    const float bf = (float)beta;
    for (int i = 0; i <= j; ++i) F += rej_w[i] - (double)fmaxf(fmaf(-bf, kid_q[i], kid_p[i]), 0.f);
    Z = F;
  }
  if (tid == 0) {
    out.node_beta[o + cur] = beta;
    out.node_Z[o + cur] = Z;
  }
}

__global__ __launch_bounds__(AC_THREADS) void k_accept_walk(
    const float* __restrict__ target, const float* __restrict__ draft, int64_t row_stride,
    const int32_t* __restrict__ token, const int32_t* __restrict__ parent, const int32_t* __restrict__ node_offsets,
    int NN, int V, int mode, float inv_t, const float* __restrict__ uniforms, int max_depth,
    const int32_t* __restrict__ t_arg, const float* __restrict__ t_lz, const int32_t* __restrict__ d_arg,
    const float* __restrict__ d_lz, ChainOut chain, int32_t* __restrict__ accept_len,
    int32_t* __restrict__ accept_path, int32_t* __restrict__ bonus_token) {
  __shared__ int kids[AC_MAX_KIDS];
  __shared__ int kids_sorted[AC_MAX_KIDS];
  __shared__ int n_kids;
  __shared__ int rej_tok[AC_MAX_KIDS];
  __shared__ double rej_w[AC_MAX_KIDS];  // frozen weight of each rejected token
  __shared__ float kid_u[AC_MAX_KIDS];    // the child's uniform
  __shared__ double kid_a[AC_MAX_KIDS], kid_b[AC_MAX_KIDS];  // its current p(x) (and q(x) under the ratio rule)
  __shared__ double rowsum[AC_MAX_ROWS];

  const int s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int o = node_offsets[s];
  const int n = node_offsets[s + 1] - o;
  int32_t* path = accept_path + (int64_t)s * max_depth;
  for (int d = tid; d < max_depth; d += AC_THREADS) path[d] = -1;
  if (n <= 0) {
    if (tid == 0) {
      accept_len[s] = 0;
      bonus_token[s] = -1;
    }
    return;
  }
  const bool ratio_mode = mode == HS_ACCEPT_STOCHASTIC;
  int cur = 0, len = 0;
  for (;;) {
    const int nk = gather_children(parent, o, n, cur, len < max_depth, kids, kids_sorted, &n_kids);

    const float* p_row = target + (int64_t)(o + cur) * row_stride;
    const RowView p(p_row, p_row[t_arg[o + cur]], t_lz[o + cur], inv_t);
    RowView q = p;
    const bool use_q = ratio_mode && nk > 0;
    if (use_q) {
      const float* q_row = draft + (int64_t)(o + cur) * row_stride;
      q = RowView(q_row, q_row[d_arg[o + cur]], d_lz[o + cur], inv_t);
    }

    // ---- what the tests of the children need, fetched side by side (a round trip to memory per
    // child would dominate the walk).  The rejected children are a prefix of the list, so entry i of
    // rej_tok / rej_w belongs to child i.
    if (tid < nk) {
      const int c = kids_sorted[tid];
      const int x = token[o + c];
      rej_tok[tid] = x;
      kid_u[tid] = uniforms[o + c];
      if (ratio_mode) {  // the node's chain of rejections was run ahead of the walk (k_accept_chain)
        kid_a[tid] = chain.child_p[o + c];
        kid_b[tid] = chain.child_q[o + c];
        rej_w[tid] = chain.child_frozen[o + c];
      } else {
        kid_a[tid] = (double)p.prob(x);
        rej_w[tid] = 0.0;
      }
    }
    __syncthreads();
    // ---- try the children in order (every thread runs the same scalar logic)
    double beta = 0.0, Z = 1.0, rem = 1.0;
    int n_rej = 0, accepted = -1;
    for (int j = 0; j < nk; ++j) {
      const double u = (double)kid_u[j];
      if (!ratio_mode) {
        const double px = kid_a[j];
        if (u * rem < px) {  // u < p(x) / rem
          accepted = kids_sorted[j];
          break;
        }
        rem -= px;
      } else {
        const double pc = kid_a[j], qc = kid_b[j];
        if (pc >= qc || u * qc < pc) {
          accepted = kids_sorted[j];
          break;
        }
      }
      ++n_rej;
    }
    if (ratio_mode && accepted < 0 && n_rej > 0) {
      beta = chain.node_beta[o + cur];
      Z = chain.node_Z[o + cur];
    }
    if (accepted >= 0) {
      if (tid == 0) path[len] = accepted;
      ++len;
      cur = accepted;
      continue;
    }

    // ---- no child accepted: draw the bonus token from the current distribution
    const bool sub_q = use_q && n_rej > 0;
    const double total = ratio_mode ? Z : rem;
    const double goal = (double)uniforms[NN + s] * total;
    const int n_rows = (V + 63) / 64;
    int first_row = 0;  // rows below it were summed with 16-byte loads
    if (p.aligned16() && (!sub_q || q.aligned16())) {
      // a lane takes four tokens, 16 lanes a row of 64, a wave four rows per trip
      const int full_rows = V >> 6;
      const int sub = lane >> 4, l16 = lane & 15;
      const float bf = (float)beta;
      for (int r0 = wave * 4; r0 < full_rows; r0 += AC_WAVES * 4) {
        const int r = r0 + sub;
        double w = 0.0;
        if (r < full_rows) {
          const float4 pp = p.prob4(r * 16 + l16);
          if (sub_q) {
            const float4 qq = q.prob4(r * 16 + l16);
            w = ((double)fmaxf(fmaf(-bf, qq.x, pp.x), 0.f) + (double)fmaxf(fmaf(-bf, qq.y, pp.y), 0.f)) +
                ((double)fmaxf(fmaf(-bf, qq.z, pp.z), 0.f) + (double)fmaxf(fmaf(-bf, qq.w, pp.w), 0.f));
          } else {
            w = ((double)pp.x + (double)pp.y) + ((double)pp.z + (double)pp.w);
          }
        }
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) w += __shfl_xor(w, off);
        if (l16 == 0 && r < full_rows) rowsum[r] = w;
      }
      first_row = full_rows;
    }
    for (int r = first_row + wave; r < n_rows; r += AC_WAVES) {
      const int v = r * 64 + lane;
      double w = v < V ? token_weight(p, q, sub_q, beta, v) : 0.0;
      w = wave_sum(w);
      if (lane == 0) rowsum[r] = w;
    }
    __syncthreads();
    if (tid == 0) {
      for (int i = 0; i < n_rej; ++i)
        rowsum[rej_tok[i] >> 6] += rej_w[i] - token_weight(p, q, sub_q, beta, rej_tok[i]);
    }
    __syncthreads();
    if (wave == 0) {
      double carry = 0.0;
      int row = -1, last_pos = -1;
      double excl = 0.0;
      for (int base = 0; base < n_rows && row < 0; base += 64) {
        const int r = base + lane;
        const double val = r < n_rows ? rowsum[r] : 0.0;
        const double incl = wave_incl_scan(val, lane) + carry;
        const unsigned long long hit = __ballot(r < n_rows && incl > goal);
        const unsigned long long pos = __ballot(r < n_rows && val > 0.0);
        if (hit != 0ull) {
          const int l = __ffsll((long long)hit) - 1;
          row = base + l;
          excl = __shfl(incl - val, l);
        } else {
          if (pos != 0ull) last_pos = base + 63 - __clzll((long long)pos);
          carry = __shfl(incl, 63);
        }
      }
      double row_goal = goal - excl;
      if (row < 0) {  // rounding left the goal at or above the total: take the last token with mass
        row = last_pos < 0 ? 0 : last_pos;
        row_goal = HS_INF;
      }
      const int v = row * 64 + lane;
      double w = v < V ? token_weight(p, q, sub_q, beta, v) : 0.0;
      for (int i = 0; i < n_rej; ++i)
        if (rej_tok[i] == v) w = rej_w[i];
      const double incl = wave_incl_scan(w, lane);
      const unsigned long long hit = __ballot(incl > row_goal);
      const unsigned long long pos = __ballot(w > 0.0);
      int l;
      if (hit != 0ull)
        l = __ffsll((long long)hit) - 1;
      else
        l = pos != 0ull ? 63 - __clzll((long long)pos) : 0;
      if (lane == 0) {
        accept_len[s] = len;
        int tok = row * 64 + l;
        bonus_token[s] = tok < V ? tok : V - 1;
      }
    }
    return;
  }
}

}  // namespace hs

extern "C" size_t hs_verify_accept_workspace(int32_t B, int32_t NN, int32_t V) {
  if (B <= 0 || NN <= 0 || V <= 0) return 0;
  // per row: argmax, -ln Z and an unused Top-1 entropy, for the target and for the draft rows
  const size_t per_set = 3 * hs::align_up((size_t)NN * sizeof(float), 256);
  // five doubles per row: what the rejection chains hand to the walk
  const size_t chain = 5 * hs::align_up((size_t)NN * sizeof(double), 256);
  // the rejection chains' lists of live tokens: a pair of floats per token and row
  const size_t lists = NN <= hs::AC_LIST_NODES
                           ? hs::align_up((size_t)NN * hs::AC_WAVES * hs::list_wave_cap(V) * sizeof(float2), 256)
                           : 0;
  return 2 * per_set + chain + lists + hs::row_topk_workspace(NN, V, 1);
}

extern "C" hs_status hs_verify_accept(const float* target_logits, const float* draft_logits, int64_t row_stride,
                                      const int32_t* token, const int32_t* parent, const int32_t* node_offsets,
                                      int32_t B, int32_t NN, int32_t V, hs_accept_mode mode, float temperature,
                                      const float* uniforms, int32_t max_depth, int32_t* accept_len,
                                      int32_t* accept_path, int32_t* bonus_token, void* workspace,
                                      size_t workspace_bytes, hs_stream stream) {
  hs::clear_error();
  HS_REQUIRE(B >= 0 && NN >= 0 && V >= 1, HS_ERR_SHAPE, "hs_verify_accept: B=%d NN=%d V=%d", B, NN, V);
  HS_REQUIRE(max_depth >= 1, HS_ERR_SHAPE, "hs_verify_accept: max_depth=%d must be at least 1", max_depth);
  HS_REQUIRE(row_stride >= V, HS_ERR_SHAPE, "hs_verify_accept: row_stride=%lld < V=%d", (long long)row_stride, V);
  HS_REQUIRE(mode == HS_ACCEPT_GREEDY || mode == HS_ACCEPT_STOCHASTIC || mode == HS_ACCEPT_STOCHASTIC_POINTMASS,
             HS_ERR_SHAPE, "hs_verify_accept: unknown mode %d", (int)mode);
  if (B == 0) return HS_OK;
  HS_REQUIRE(node_offsets && accept_len && accept_path && bonus_token, HS_ERR_NULL, "hs_verify_accept: NULL argument");
  const bool stochastic = mode != HS_ACCEPT_GREEDY;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (NN > 0) {
    HS_REQUIRE(target_logits && token && parent, HS_ERR_NULL, "hs_verify_accept: NULL node array");
    if (stochastic) {
      HS_REQUIRE(uniforms, HS_ERR_NULL, "hs_verify_accept: uniforms are required in the stochastic modes");
      HS_REQUIRE(mode != HS_ACCEPT_STOCHASTIC || draft_logits, HS_ERR_NULL,
                 "hs_verify_accept: draft_logits are required in mode HS_ACCEPT_STOCHASTIC");
      HS_REQUIRE(temperature > 0.f, HS_ERR_SHAPE, "hs_verify_accept: temperature must be positive");
      HS_REQUIRE((V + 63) / 64 <= hs::AC_MAX_ROWS, HS_ERR_UNSUPPORTED,
                 "hs_verify_accept: stochastic modes support V <= %d", hs::AC_MAX_ROWS * 64);
    }
  }
  const size_t need = hs_verify_accept_workspace(B, NN, V);
  HS_REQUIRE(need == 0 || (workspace && workspace_bytes >= need && reinterpret_cast<uintptr_t>(workspace) % 256 == 0),
             HS_ERR_WORKSPACE, "hs_verify_accept: workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
             workspace_bytes);
  int32_t *t_arg = nullptr, *d_arg = nullptr;
  float *t_lz = nullptr, *d_lz = nullptr;
  hs::ScanSlices slices{nullptr, nullptr, 1};
  hs::ChainOut chain{nullptr, nullptr, nullptr, nullptr, nullptr};
  float2* lists = nullptr;
  if (NN > 0) {
    hs::Carver c(workspace);
    t_arg = c.take<int32_t>(NN);
    t_lz = c.take<float>(NN);
    float* t_ent = c.take<float>(NN);
    d_arg = c.take<int32_t>(NN);
    d_lz = c.take<float>(NN);
    float* d_ent = c.take<float>(NN);
    chain.child_p = c.take<double>(NN);
    chain.child_q = c.take<double>(NN);
    chain.child_frozen = c.take<double>(NN);
    chain.node_beta = c.take<double>(NN);
    chain.node_Z = c.take<double>(NN);
    if (NN <= hs::AC_LIST_NODES) lists = c.take<float2>((size_t)NN * hs::AC_WAVES * hs::list_wave_cap(V));
    void* scan_ws = c.take<char>(0);
    const float T = stochastic ? temperature : 1.0f;
    // greedy: the merge of the row slices is done by the accept kernel (one launch less)
    hs_status r = hs::row_topk_launch(target_logits, row_stride, NN, V, 1, T, t_arg, t_lz, t_ent, nullptr, nullptr,
                                      scan_ws, st, stochastic ? nullptr : &slices);
    if (r != HS_OK) return r;
    if (mode == HS_ACCEPT_STOCHASTIC) {
      r = hs::row_topk_launch(draft_logits, row_stride, NN, V, 1, T, d_arg, d_lz, d_ent, nullptr, nullptr, scan_ws,
                              st);
      if (r != HS_OK) return r;
    }
  }
  if (!stochastic) {
    hipLaunchKernelGGL(hs::k_accept_greedy, dim3(B), dim3(hs::GR_THREADS), 0, st, t_arg, slices.val, slices.idx,
                       slices.count, token, parent, node_offsets, max_depth, accept_len, accept_path, bonus_token);
    return hs::launch_status("accept (greedy)");
  }
  if (mode == HS_ACCEPT_STOCHASTIC && NN > 0) {
    hipLaunchKernelGGL(hs::k_accept_chain, dim3(NN), dim3(hs::AC_THREADS), 0, st, target_logits, draft_logits,
                       row_stride, token, parent, node_offsets, B, V, 1.0f / temperature, max_depth, t_arg, t_lz,
                       d_arg, d_lz, chain, lists);
    hs_status r = hs::launch_status("accept (rejection chains)");
    if (r != HS_OK) return r;
  }
  hipLaunchKernelGGL(hs::k_accept_walk, dim3(B), dim3(hs::AC_THREADS), 0, st, target_logits, draft_logits, row_stride,
                     token, parent, node_offsets, NN, V, (int)mode, 1.0f / temperature, uniforms, max_depth, t_arg,
                     t_lz, d_arg, d_lz, chain, accept_len, accept_path, bonus_token);
  return hs::launch_status("accept (stochastic)");
}
