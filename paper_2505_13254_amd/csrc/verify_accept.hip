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
//               led there.  The residual itself is never materialised: after j rejections it is
//               max(p(v) - beta_j q(v), 0) for every token not yet rejected (beta_j a scalar that
//               accumulates Z_i / (1 - sum of rejected q)), and frozen at its value of the time
//               for a rejected token; only its normaliser is needed per rejection.  A node with
//               one child gets it from one cooperative pass over its two vocabulary rows; for a
//               node with several children the tokens with p > q are first sorted by p / q into
//               buckets with their sums (three kernels on the whole chip), after which every
//               normaliser of the chain is two suffix sums plus the tokens of three buckets.  One
//               workgroup per node with children runs that node's chain of rejections ahead of
//               the walk, all nodes in parallel (k_accept_chain), and leaves each child's pair of
//               current probabilities; the walk itself (k_accept_walk, one workgroup per sequence) then
//               only compares uniforms with them, and draws the bonus token at the node where it
//               stops: an inverse-CDF search done as row sums of 64 tokens, a scan of the row sums,
//               and a scan inside the one row that is hit.
#include <limits.h>

#include "hs_common.h"

namespace hs {

constexpr int GR_THREADS = 256;
constexpr int GR_LDS_ROWS = 1024;  // tree rows that the greedy walk stages in LDS
constexpr int AC_THREADS = 1024;
constexpr int AC_WAVES = AC_THREADS / 64;
constexpr int AC_MAX_KIDS = 256;    // children tried per node
constexpr int AC_MAX_ROWS = 8192;   // 64-token rows of the CDF search held in LDS (V <= 524288)
constexpr int BR_SLICES = 16;     // workgroups per tree row that sum the bonus distribution's rows ahead of the walk
constexpr int BR_THREADS = 512;
constexpr int BK_NODES = 4096;      // calls with up to this many tree rows get the sorted residual (below)
constexpr int BK_SLICES = 16;       // vocabulary slices per row in the kernels that build it
constexpr int BK_N = 256;           // buckets of the ratio p / q: BK_PER_OCTAVE per factor of two, from 1 upwards
constexpr int BK_THREADS = 256;     // (one thread per bucket in the scan)
constexpr float BK_PER_OCTAVE = 16.f;
constexpr float FIX_SCALE = 0x1p62f;   // probabilities are summed as 64-bit integers in units of 2^-62:
constexpr double FIX_UNIT = 0x1p-62;   // the sums do not depend on the order of their terms

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
  // Trees of up to GR_LDS_ROWS rows are staged in LDS (parents, tokens, the rows' argmax), all of their
  // global reads in one trip: the walks below are chains of dependent reads, one per tree level.
  __shared__ int l_par[GR_LDS_ROWS], l_tok[GR_LDS_ROWS], l_arg[GR_LDS_ROWS];
  const bool staged = n <= GR_LDS_ROWS;
  if (staged) {
    for (int i = tid; i < n; i += GR_THREADS) {
      l_par[i] = parent[o + i];
      l_tok[i] = token[o + i];
    }
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
      if (staged) l_arg[i] = bi;
    }
  } else if (staged) {
    for (int i = tid; i < n; i += GR_THREADS) l_arg[i] = arg[o + i];
  }
  __syncthreads();  // every row's argmax is visible to the workgroup
  // key = depth of a fully confirmed node (higher wins), then lower index
  long long best = ((long long)0 << 32) | (unsigned)(INT_MAX - 0);  // the root: depth 0
  for (int i = tid; i < n; i += GR_THREADS) {
    bool ok = true;
    int d = 0;
    if (staged) {
      for (int j = i; j > 0;) {
        const int p = l_par[j];
        ok = ok && (l_tok[j] == l_arg[p]);
        j = p;
        ++d;
      }
    } else {
      for (int j = i; j > 0;) {
        const int p = parent[o + j];
        ok = ok && (token[o + j] == arg[o + p]);
        j = p;
        ++d;
      }
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
    bonus_token[s] = staged ? l_arg[node] : arg[o + node];
    for (int k = d - 1; k >= 0; --k) {
      path[k] = node;
      node = staged ? l_par[node] : parent[o + node];
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
  __device__ __forceinline__ float arg(float logit) const { return fmaf(logit - m, c1, c2); }  // log2 p
  __device__ __forceinline__ float of(float logit) const { return exp2_fast(arg(logit)); }
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

// Sum over each row of 16 lanes; the row's last lane holds it.  DPP moves of the two halves of the
// double: a lane without a source takes 0.
__device__ __forceinline__ double row16_sum(double x) {
#define HS_DPP_ADD(ctrl, banks)                                                                              \
  x += __hiloint2double(__builtin_amdgcn_update_dpp(0, __double2hiint(x), ctrl, 0xf, banks, false),          \
                        __builtin_amdgcn_update_dpp(0, __double2loint(x), ctrl, 0xf, banks, false))
  HS_DPP_ADD(0x111, 0xf);  // row_shr:1
  HS_DPP_ADD(0x112, 0xf);  // row_shr:2
  HS_DPP_ADD(0x114, 0xe);  // row_shr:4
  HS_DPP_ADD(0x118, 0xc);  // row_shr:8
#undef HS_DPP_ADD
  return x;
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
// number (at most AC_MAX_KIDS: of a node with more children the AC_MAX_KIDS lowest rows are taken,
// whatever order the threads arrive in).  Called by all threads; ends with a barrier.
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
  if (*n_kids > AC_MAX_KIDS) {
    // more children than the lists hold (never with Top-k expansion): which of them the atomic
    // counter let in depends on arrival order, so the lists are made again by rank, each child
    // counting the children before it; the first AC_MAX_KIDS stay
    for (int i = 1 + tid; i < n; i += AC_THREADS)
      if (parent[o + i] == cur) {
        int r = 0;
        for (int j = 1; j < i && r < AC_MAX_KIDS; ++j) r += parent[o + j] == cur ? 1 : 0;
        if (r < AC_MAX_KIDS) kids_sorted[r] = i;
      }
    __syncthreads();
    return AC_MAX_KIDS;
  }
  const int nk = *n_kids;
  if (tid < nk) {
    int me = kids[tid], r = 0;
    for (int j = 0; j < nk; ++j) r += kids[j] < me ? 1 : 0;
    kids_sorted[r] = me;
  }
  __syncthreads();
  return nk;
}

// ------------------------------------------------------------------ the sorted residual
// Along a node's chain of rejections only beta changes: F(beta) = sum_v max(p(v) - beta q(v), 0),
// taken at an increasing sequence of beta >= 1 that is not known in advance.  A token contributes
// p - beta q while its ratio p / q exceeds beta and nothing afterwards.  So, for every node with
// at least two children, three small kernels that run on the whole chip sort the tokens with
// p > q by their ratio into BK_N buckets (a counting sort: count per vocabulary slice and bucket,
// scan, scatter) and keep, per bucket, the sums of p and of q.  F(beta) is then
//     sum over the buckets well above beta of (P_b - beta Q_b)      two suffix sums, read once
//   + sum over the tokens of the three buckets around beta of max(p - beta q, 0)
// which is what k_accept_chain evaluates per rejection: a few thousand pairs instead of two
// vocabulary rows.  A token's bucket is floor(BK_PER_OCTAVE * log2(p / q)), taken from the two
// exponent arguments (p = exp2(a_p)): the rounding of that difference is many orders below a
// bucket's width, and one bucket to either side of beta's own is still treated token by token, so
// no token is ever taken for live or dead by its bucket alone when it is not.  All sums are 64-bit
// integers in units of 2^-62 (LDS and per-slice partial sums), so neither the order in which the
// lanes' atomic additions arrive nor the order of the tokens inside a bucket changes a result.
struct BucketWs {
  uint32_t* count;            // [NN][BK_SLICES][BK_N] live tokens per (slice, bucket); after the scan: first position
  unsigned long long* psum;   // [NN][BK_SLICES][BK_N] their p, summed
  unsigned long long* qsum;   // [NN][BK_SLICES][BK_N] their q
  uint32_t* start;            // [NN][BK_N + 1] first position of a bucket in `pairs` (ascending ratio)
  unsigned long long* sp;     // [NN][BK_N + 1] sum of p over the buckets >= b
  unsigned long long* sq;     // [NN][BK_N + 1] sum of q over them
  float2* pairs;              // [NN][V] (p, q) of the live tokens, bucket by bucket
  int32_t* nk;                // [NN] number of children the chain will try
};

__device__ __forceinline__ int bucket_of(float ap, float aq) {
  return (int)fminf(fmaxf((ap - aq) * BK_PER_OCTAVE, 0.f), (float)(BK_N - 1));
}
__device__ __forceinline__ unsigned long long to_fixed(float x) { return (unsigned long long)(x * FIX_SCALE); }

// Sequence, local row and number of children to try of global row g (all threads; one barrier).
struct NodeRef {
  int o, n, cur, nk;
};
__device__ __forceinline__ NodeRef node_ref(int g, const int32_t* __restrict__ parent,
                                            const int32_t* __restrict__ node_offsets, int B, int max_depth,
                                            int* lds_count) {
  int lo = 0, hi = B;  // sequence of this row: last s with node_offsets[s] <= g
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (node_offsets[mid] <= g) lo = mid; else hi = mid;
  }
  NodeRef r;
  r.o = node_offsets[lo];
  r.n = node_offsets[lo + 1] - r.o;
  r.cur = g - r.o;
  r.nk = 0;
  if (r.cur >= r.n) return r;  // (an empty sequence before this row's: cannot happen, offsets are monotone)
  int depth = 0;
  for (int j = parent[r.o + r.cur]; j >= 0; j = parent[r.o + j]) ++depth;
  if (threadIdx.x == 0) *lds_count = 0;
  __syncthreads();
  if (depth < max_depth) {
    int c = 0;
    for (int i = 1 + threadIdx.x; i < r.n; i += blockDim.x) c += parent[r.o + i] == r.cur ? 1 : 0;
    if (c) atomicAdd(lds_count, c);
  }
  __syncthreads();
  r.nk = *lds_count < AC_MAX_KIDS ? *lds_count : AC_MAX_KIDS;
  return r;
}

// grid (BK_SLICES, NN).  SCATTER false: counts and sums of slice blockIdx.x of row blockIdx.y;
// SCATTER true (after k_bucket_scan): the same pass again, now placing every live pair.
template <bool SCATTER>
__global__ __launch_bounds__(BK_THREADS) void k_bucket_pass(
    const float* __restrict__ target, const float* __restrict__ draft, int64_t row_stride,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ node_offsets, int B, int V, float inv_t,
    int max_depth, const int32_t* __restrict__ t_arg, const float* __restrict__ t_lz,
    const int32_t* __restrict__ d_arg, const float* __restrict__ d_lz, BucketWs ws) {
  __shared__ unsigned cnt[BK_N];  // SCATTER: the next free position of each bucket
  __shared__ unsigned long long ps[BK_N], qs[BK_N];
  __shared__ int n_kids;
  const int slice = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;
  int nk;
  if (SCATTER) {
    nk = ws.nk[g];
  } else {
    nk = node_ref(g, parent, node_offsets, B, max_depth, &n_kids).nk;
    if (slice == 0 && tid == 0) ws.nk[g] = nk;
  }
  if (nk < 2) return;  // a single rejection is one plain pass of the chain kernel
  const int64_t slot = ((int64_t)g * BK_SLICES + slice) * BK_N;
  for (int b = tid; b < BK_N; b += BK_THREADS) {
    cnt[b] = SCATTER ? ws.count[slot + b] : 0u;
    ps[b] = 0ull;
    qs[b] = 0ull;
  }
  const float* p_row = target + (int64_t)g * row_stride;
  const float* q_row = draft + (int64_t)g * row_stride;
  const RowView p(p_row, p_row[t_arg[g]], t_lz[g], inv_t);
  const RowView q(q_row, q_row[d_arg[g]], d_lz[g], inv_t);
  float2* __restrict__ pairs = ws.pairs + (int64_t)g * V;
  __syncthreads();
  auto token = [&](float xp, float xq) {
    const float ap = p.arg(xp), aq = q.arg(xq);
    const float pv = exp2_fast(ap), qv = exp2_fast(aq);
    if (pv > qv) {  // live at beta = 1, where every chain starts
      const int b = bucket_of(ap, aq);
      if (SCATTER) {
        pairs[atomicAdd(&cnt[b], 1u)] = make_float2(pv, qv);
      } else {
        atomicAdd(&cnt[b], 1u);
        atomicAdd(&ps[b], to_fixed(pv));
        atomicAdd(&qs[b], to_fixed(qv));
      }
    }
  };
  const int n4 = V >> 2;
  const int per = (n4 + BK_SLICES - 1) / BK_SLICES;
  const int i1 = min(n4, (slice + 1) * per);
  const float4* __restrict__ px = reinterpret_cast<const float4*>(p_row);
  const float4* __restrict__ qx = reinterpret_cast<const float4*>(q_row);
#pragma unroll 2
  for (int i = slice * per + tid; i < i1; i += BK_THREADS) {
    const float4 fp = px[i], fq = qx[i];
    token(fp.x, fq.x);
    token(fp.y, fq.y);
    token(fp.z, fq.z);
    token(fp.w, fq.w);
  }
  if (slice == BK_SLICES - 1) {  // the last V % 4 tokens
    const int v = (n4 << 2) + tid;
    if (v < V) token(p_row[v], q_row[v]);
  }
  if (!SCATTER) {
    __syncthreads();
    for (int b = tid; b < BK_N; b += BK_THREADS) {
      ws.count[slot + b] = cnt[b];
      ws.psum[slot + b] = ps[b];
      ws.qsum[slot + b] = qs[b];
    }
  }
}

// grid NN, one thread per bucket: per-slice counts become first positions, bucket totals become
// the suffix sums the chain reads.
__global__ __launch_bounds__(BK_N) void k_bucket_scan(BucketWs ws) {
  __shared__ unsigned s_cnt[BK_N];
  __shared__ unsigned long long s_p[BK_N], s_q[BK_N];
  const int g = blockIdx.x, b = threadIdx.x;
  if (ws.nk[g] < 2) return;
  unsigned off[BK_SLICES], total = 0u;
  unsigned long long tp = 0ull, tq = 0ull;
#pragma unroll
  for (int sl = 0; sl < BK_SLICES; ++sl) {
    const int64_t at = ((int64_t)g * BK_SLICES + sl) * BK_N + b;
    off[sl] = total;
    total += ws.count[at];
    tp += ws.psum[at];
    tq += ws.qsum[at];
  }
  s_cnt[b] = total;
  s_p[b] = tp;
  s_q[b] = tq;
  __syncthreads();
  // inclusive prefix counts (ascending) and inclusive suffix sums (descending), log-step
  for (int d = 1; d < BK_N; d <<= 1) {
    const unsigned c = b >= d ? s_cnt[b - d] : 0u;
    const unsigned long long ap = b + d < BK_N ? s_p[b + d] : 0ull, aq = b + d < BK_N ? s_q[b + d] : 0ull;
    __syncthreads();
    s_cnt[b] += c;
    s_p[b] += ap;
    s_q[b] += aq;
    __syncthreads();
  }
  const unsigned first = s_cnt[b] - total;
#pragma unroll
  for (int sl = 0; sl < BK_SLICES; ++sl) ws.count[((int64_t)g * BK_SLICES + sl) * BK_N + b] = first + off[sl];
  const int64_t row = (int64_t)g * (BK_N + 1);
  ws.start[row + b] = first;
  ws.sp[row + b] = s_p[b];
  ws.sq[row + b] = s_q[b];
  if (b == BK_N - 1) {
    ws.start[row + BK_N] = first + total;
    ws.sp[row + BK_N] = 0ull;
    ws.sq[row + BK_N] = 0ull;
  }
}

// A row's bucket tables, staged in LDS once per chain (the chain is serial: what it reads per
// rejection should not be a round trip to memory).
struct BucketTables {
  unsigned start[BK_N + 1];
  unsigned long long sp[BK_N + 1], sq[BK_N + 1];
};
__device__ __forceinline__ void load_bucket_tables(const BucketWs& ws, int g, BucketTables& t) {
  const int64_t row = (int64_t)g * (BK_N + 1);
  for (int b = threadIdx.x; b <= BK_N; b += blockDim.x) {
    t.start[b] = ws.start[row + b];
    t.sp[b] = ws.sp[row + b];
    t.sq[b] = ws.sq[row + b];
  }
}

// What the first wave hands to the others for one rejection, and what they hand back.
struct BucketStep {
  double beta;
  int lo, hi;                          // positions in `pairs` of the tokens to take one by one
  unsigned long long part[AC_WAVES];   // their terms, summed per wave
};

// beta's own bucket with one bucket to either side: [b_lo, b_hi).  NaN and infinity end up at valid
// indices as well; float32 is enough to pick the bucket, as it is for the tokens' buckets.
__device__ __forceinline__ void near_buckets(double beta, int& b_lo, int& b_hi) {
  const int own = (int)fminf(fmaxf(__log2f((float)beta) * BK_PER_OCTAVE, 0.f), (float)(BK_N - 1));
  b_lo = own > 0 ? own - 1 : 0;
  b_hi = own + 2 < BK_N ? own + 2 : BK_N;
}

// The terms max(p - beta q, 0) of pairs [lo, hi), all threads of the workgroup, summed per wave into
// step.part.  They are formed in float64 and summed as integers in units of 2^-52 (the fraction
// bits of 1 + term, term < 1): the order of the pairs inside a bucket, which the scatter's atomic
// additions decide, does not reach the result.
__device__ __forceinline__ void near_terms(const float2* __restrict__ pairs, BucketStep& step) {
  const int tid = threadIdx.x;
  const double beta = step.beta;
  const int hi = step.hi;
  unsigned long long acc = 0ull;
#pragma unroll 4
  for (int i = step.lo + tid; i < hi; i += AC_THREADS) {
    const float2 e = pairs[i];
    const double term = fmin(fmax((double)e.x - beta * (double)e.y, 0.0), 0x1.fffffffffffffp-1);
    acc += (unsigned long long)__double_as_longlong(1.0 + term) & 0xfffffffffffffull;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  if ((tid & 63) == 0) step.part[tid >> 6] = acc;
}

// One workgroup per sequence: the rows the scan of [target rows ; draft rows] has to read: every
// target row (wanted[row] = 1) and the draft rows of the rows that are somebody's parent
// (has_child = wanted + NN; nobody reads the draft row of a row without children).
__global__ __launch_bounds__(GR_THREADS) void k_mark_parents(const int32_t* __restrict__ parent,
                                                             const int32_t* __restrict__ node_offsets, int NN,
                                                             uint8_t* __restrict__ wanted) {
  const int s = blockIdx.x, tid = threadIdx.x;
  const int o = node_offsets[s];
  const int n = node_offsets[s + 1] - o;
  uint8_t* __restrict__ has_child = wanted + NN;
  for (int i = tid; i < n; i += GR_THREADS) {
    wanted[o + i] = 1;
    has_child[o + i] = 0;
  }
  __syncthreads();
  for (int i = 1 + tid; i < n; i += GR_THREADS) has_child[o + parent[o + i]] = 1;
}

// What the stochastic walk needs from a node's chain of rejections.
struct ChainOut {
  double* child_p;       // [NN] current target probability of the child's token when its turn comes
  double* child_q;       // [NN] current draft probability of it
  double* child_frozen;  // [NN] its weight in the residual after its own rejection
  double* node_beta;     // [NN] beta and normaliser after all of the node's children were rejected
  double* node_Z;
  int32_t* n_tried;      // [NN] number of children the node's chain tried (0: the node's residual is p itself)
  double* bonus_rows;    // [NN][ceil(V / 64)] row sums of the residual a bonus token would be drawn from
                         // if the walk stopped at the node (NULL: the walk sums the rows of its stop node)
};

// Sums of the bonus distribution's weights over rows of 64 tokens, rows [r_begin, r_end) of a node,
// by all waves of the workgroup: dst[r] for each of them.  A lane takes four tokens, 16 lanes a row, a
// wave four rows per trip; the loads of four trips are requested together (lanes past the last row
// re-read it), and a row's 16 partial sums meet in its last lane by DPP moves.  Rows that are not
// whole, or rows of arrays that are not 16-byte aligned, are summed a token per lane.  A row's sum
// does not depend on who computes it: the walk and k_bonus_rows give the same bits.
__device__ __forceinline__ void bonus_row_sums(const RowView& p, const RowView& q, bool sub_q, double beta, int V,
                                               int r_begin, int r_end, double* __restrict__ dst) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
  int first_row = r_begin;  // rows below it were summed with 16-byte loads
  if (p.aligned16() && (!sub_q || q.aligned16()) && V >= 64) {
    constexpr int TRIPS = 4;
    const int full_end = min(V >> 6, r_end);
    const int sub = lane >> 4, l16 = lane & 15;
    const float bf = (float)beta;
    const float4* __restrict__ px = reinterpret_cast<const float4*>(p.x);
    const float4* __restrict__ qx = reinterpret_cast<const float4*>(q.x);
    for (int r0 = r_begin + wave * 4; r0 < full_end; r0 += n_waves * 4 * TRIPS) {
      float4 fp[TRIPS], fq[TRIPS];
#pragma unroll
      for (int u = 0; u < TRIPS; ++u) {
        const int r = min(r0 + u * n_waves * 4 + sub, full_end - 1);
        fp[u] = px[r * 16 + l16];
        fq[u] = sub_q ? qx[r * 16 + l16] : fp[u];
      }
#pragma unroll
      for (int u = 0; u < TRIPS; ++u) {
        const int r = r0 + u * n_waves * 4 + sub;
        const float4 pp = p.of4(fp[u]);
        double w;
        if (sub_q) {
          const float4 qq = q.of4(fq[u]);
          w = ((double)fmaxf(fmaf(-bf, qq.x, pp.x), 0.f) + (double)fmaxf(fmaf(-bf, qq.y, pp.y), 0.f)) +
              ((double)fmaxf(fmaf(-bf, qq.z, pp.z), 0.f) + (double)fmaxf(fmaf(-bf, qq.w, pp.w), 0.f));
        } else {
          w = ((double)pp.x + (double)pp.y) + ((double)pp.z + (double)pp.w);
        }
        w = row16_sum(w);
        if (l16 == 15 && r < full_end) dst[r] = w;
      }
    }
    first_row = max(full_end, r_begin);
  }
  for (int r = first_row + wave; r < r_end; r += n_waves) {
    const int v = r * 64 + lane;
    double w = v < V ? token_weight(p, q, sub_q, beta, v) : 0.0;
    w = wave_sum(w);
    if (lane == 0) dst[r] = w;
  }
}

// One workgroup per tree row that has children (others leave at once): the chain of rejections at
// that node under the ratio rule, every child rejected in turn.
__global__ __launch_bounds__(AC_THREADS) void k_accept_chain(
    const float* __restrict__ target, const float* __restrict__ draft, int64_t row_stride,
    const int32_t* __restrict__ token, const int32_t* __restrict__ parent, const int32_t* __restrict__ node_offsets,
    int B, int V, float inv_t, int max_depth, const int32_t* __restrict__ t_arg, const float* __restrict__ t_lz,
    const int32_t* __restrict__ d_arg, const float* __restrict__ d_lz, ChainOut out, BucketWs bk) {
  __shared__ int kids[AC_MAX_KIDS];
  __shared__ int kids_sorted[AC_MAX_KIDS];
  __shared__ int n_kids;
  __shared__ double rej_w[AC_MAX_KIDS];
  __shared__ float kid_p[AC_MAX_KIDS], kid_q[AC_MAX_KIDS];  // p(x), q(x) of each child's token
  __shared__ double red[AC_WAVES];
  __shared__ BucketTables tables;
  __shared__ BucketStep step;
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
  if (tid == 0) out.n_tried[g] = nk;
  const float* p_row = target + (int64_t)g * row_stride;
  const RowView p(p_row, p_row[p_arg], p_lz, inv_t);
  if (nk == 0) {
    // no chain to run: this workgroup sums the rows of p, the distribution a bonus token is drawn from
    // if the walk stops here (done long before the longest chain of the launch)
    const int n_rows = (V + 63) / 64;
    if (out.bonus_rows != nullptr) bonus_row_sums(p, p, false, 0.0, V, 0, n_rows, out.bonus_rows + (int64_t)g * n_rows);
    return;
  }
  const float* q_row = draft + (int64_t)g * row_stride;
  const RowView q(q_row, q_row[q_arg], q_lz, inv_t);
  // every child's token and its two probabilities, fetched side by side: the chain below is serial,
  // and a round trip to memory per step would dominate it
  // the sorted residual (bk.pairs may be NULL) exists for the rows with at least two children
  const bool sorted = bk.pairs != nullptr && nk >= 2;
  if (sorted) load_bucket_tables(bk, g, tables);
  if (tid < nk) {
    const int x = token[o + kids_sorted[tid]];
    kid_p[tid] = p.prob(x);
    kid_q[tid] = q.prob(x);
  }
  __syncthreads();
  const float2* __restrict__ pairs = sorted ? bk.pairs + (int64_t)g * V : nullptr;
  double beta = 0.0, Z = 1.0, sumq = 0.0;
  if (sorted) {
    // The first wave keeps the chain's scalars; the others only help with the tokens around beta.
    // (Sixteen waves that all repeat the scalar part take issue slots from one another: 4 us a step.)
    const bool lead = tid < 64;
    for (int j = 0; j < nk; ++j) {
      int b_hi = 0;
      if (lead) {
        const int c = kids_sorted[j];
        const double px = (double)kid_p[j];
        const double qx = (double)kid_q[j];
        const double pc = fmax(px - beta * qx, 0.0) / Z;  // current p(x)
        const double qc = qx / (1.0 - sumq);              // current q(x)
        beta += Z / (1.0 - sumq);
        sumq += qx;
        const double frozen = fmax(px - beta * qx, 0.0);
        int b_lo;
        near_buckets(beta, b_lo, b_hi);
        rej_w[j] = frozen;  // (every lane of the wave stores the same value; LDS keeps a wave's order)
        if (tid == 0) {
          out.child_p[o + c] = pc;
          out.child_q[o + c] = qc;
          out.child_frozen[o + c] = frozen;
          step.beta = beta;
          step.lo = (int)tables.start[b_lo];
          step.hi = (int)tables.start[b_hi];
        }
      }
      __syncthreads();
      near_terms(pairs, step);
      __syncthreads();
      if (lead) {
        unsigned long long near = 0ull;
        for (int w = 0; w < AC_WAVES; ++w) near += step.part[w];
        double F = ((double)tables.sp[b_hi] - beta * (double)tables.sq[b_hi]) * FIX_UNIT + (double)near * 0x1p-52;
        // a rejected token's weight is frozen: its live term leaves the sum
        for (int i = 0; i <= j; ++i) F += rej_w[i] - fmax((double)kid_p[i] - beta * (double)kid_q[i], 0.0);
        Z = F;
      }
    }
  } else {
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
      double F = residual_mass(p, q, beta, V, red);  // (its barriers also publish rej_w)
      // a rejected token's weight is frozen: its live term, as the pass formed it, leaves the sum
      const float bf = (float)beta;
      for (int i = 0; i <= j; ++i) F += rej_w[i] - (double)fmaxf(fmaf(-bf, kid_q[i], kid_p[i]), 0.f);
      Z = F;
    }
  }
  if (tid == 0) {
    out.node_beta[o + cur] = beta;
    out.node_Z[o + cur] = Z;
  }
}

// grid (BR_SLICES, NN), after the chains: the row sums the walk would need if it stopped at row
// blockIdx.y, for every row with children at once (the walk visits a few rows one after the other and
// knows its stop row last; summing that row's vocabulary on its single compute unit took 15 us).  The
// residual at a row is fixed before the walk: max(p - beta q, 0) with the chain's final beta where all
// children were rejected (summed here), p itself where no child is tried (summed by the row's own
// workgroup of k_accept_chain, which has nothing else to do); the rejected tokens' frozen weights are
// the walk's corrections, as before.
__global__ __launch_bounds__(BR_THREADS) void k_bonus_rows(const float* __restrict__ target,
                                                           const float* __restrict__ draft, int64_t row_stride, int V,
                                                           float inv_t, const int32_t* __restrict__ t_arg,
                                                           const float* __restrict__ t_lz,
                                                           const int32_t* __restrict__ d_arg,
                                                           const float* __restrict__ d_lz, ChainOut chain) {
  const int slice = blockIdx.x, g = blockIdx.y;
  const int n_rows = (V + 63) / 64;
  const int per = (n_rows + BR_SLICES - 1) / BR_SLICES;
  const int r_begin = slice * per, r_end = min(n_rows, r_begin + per);
  if (r_begin >= r_end || chain.n_tried[g] == 0) return;  // (a row without children: summed by its chain workgroup)
  const float* p_row = target + (int64_t)g * row_stride;
  const float* q_row = draft + (int64_t)g * row_stride;
  const RowView p(p_row, p_row[t_arg[g]], t_lz[g], inv_t);
  const RowView q(q_row, q_row[d_arg[g]], d_lz[g], inv_t);
  bonus_row_sums(p, q, true, chain.node_beta[g], V, r_begin, r_end, chain.bonus_rows + (int64_t)g * n_rows);
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
  __shared__ double chunk_tot[AC_MAX_ROWS / 64];  // sums of 64 rows
  __shared__ int chunk_last[AC_MAX_ROWS / 64];

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
    if (chain.bonus_rows != nullptr) {  // summed ahead of the walk, for every row (k_bonus_rows)
      const double* __restrict__ pre = chain.bonus_rows + (int64_t)(o + cur) * n_rows;
      for (int r = tid; r < n_rows; r += AC_THREADS) rowsum[r] = pre[r];
    } else {
      bonus_row_sums(p, q, sub_q, beta, V, 0, n_rows, rowsum);
    }
    __syncthreads();
    if (tid == 0) {
      for (int i = 0; i < n_rej; ++i)
        rowsum[rej_tok[i] >> 6] += rej_w[i] - token_weight(p, q, sub_q, beta, rej_tok[i]);
    }
    __syncthreads();
    // two levels: the sixteen waves sum chunks of 64 rows side by side, one wave then looks for the
    // chunk, the row inside it and the token inside the row
    const int n_chunks = (n_rows + 63) >> 6;
    for (int c = wave; c < n_chunks; c += AC_WAVES) {
      const int r = c * 64 + lane;
      const double val = r < n_rows ? rowsum[r] : 0.0;
      const double tot = wave_sum(val);
      const unsigned long long pos = __ballot(r < n_rows && val > 0.0);
      if (lane == 0) {
        chunk_tot[c] = tot;
        chunk_last[c] = pos != 0ull ? c * 64 + 63 - __clzll((long long)pos) : -1;  // its last row with mass
      }
    }
    __syncthreads();
    if (wave == 0) {
      double carry = 0.0, chunk_excl = 0.0;
      int chunk = -1, last_pos = -1;
      for (int cb = 0; cb < n_chunks && chunk < 0; cb += 64) {
        const int c = cb + lane;
        const double val = c < n_chunks ? chunk_tot[c] : 0.0;
        const int lp = c < n_chunks ? chunk_last[c] : -1;
        const double incl = wave_incl_scan(val, lane) + carry;
        const unsigned long long hit = __ballot(c < n_chunks && incl > goal);
        if (hit != 0ull) {
          const int l = __ffsll((long long)hit) - 1;
          chunk = cb + l;
          chunk_excl = __shfl(incl - val, l);
        } else {
          const unsigned long long pos = __ballot(lp >= 0);
          if (pos != 0ull) last_pos = __shfl(lp, 63 - __clzll((long long)pos));
          carry = __shfl(incl, 63);
        }
      }
      int row = -1;
      double excl = 0.0;
      if (chunk >= 0) {
        const int r = chunk * 64 + lane;
        const double val = r < n_rows ? rowsum[r] : 0.0;
        const double incl = wave_incl_scan(val, lane) + chunk_excl;
        const unsigned long long hit = __ballot(r < n_rows && incl > goal);
        if (hit != 0ull) {
          const int l = __ffsll((long long)hit) - 1;
          row = chunk * 64 + l;
          excl = __shfl(incl - val, l);
        } else {
          last_pos = chunk_last[chunk];  // (the two orders of summation differ by a rounding: the chunk's last row with mass)
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

// Bytes of the sorted residual's arrays for NN rows (0 beyond BK_NODES rows); with a carver, also
// takes them.
static size_t bucket_workspace(int NN, int V, Carver* c, BucketWs* ws) {
  if (NN > BK_NODES) return 0;
  const size_t n_sb = (size_t)NN * BK_SLICES * BK_N, n_b = (size_t)NN * (BK_N + 1);
  if (c != nullptr) {
    ws->count = c->take<uint32_t>(n_sb);
    ws->psum = c->take<unsigned long long>(n_sb);
    ws->qsum = c->take<unsigned long long>(n_sb);
    ws->start = c->take<uint32_t>(n_b);
    ws->sp = c->take<unsigned long long>(n_b);
    ws->sq = c->take<unsigned long long>(n_b);
    ws->pairs = c->take<float2>((size_t)NN * V);
    ws->nk = c->take<int32_t>(NN);
  }
  return align_up(n_sb * 4, 256) + 2 * align_up(n_sb * 8, 256) + align_up(n_b * 4, 256) + 2 * align_up(n_b * 8, 256) +
         align_up((size_t)NN * V * sizeof(float2), 256) + align_up((size_t)NN * 4, 256);
}

// Bytes of the row sums k_bonus_rows leaves for the walk (0 beyond BK_NODES rows: the walk then sums
// the rows of its stop node itself).
static size_t bonus_rows_bytes(int NN, int V) {
  return NN <= BK_NODES ? align_up((size_t)NN * ((V + 63) / 64) * sizeof(double), 256) : 0;
}

}  // namespace hs

extern "C" size_t hs_verify_accept_workspace_mode(int32_t B, int32_t NN, int32_t V, hs_accept_mode mode) {
  if (B <= 0 || NN <= 0 || V <= 0) return 0;
  // per row: argmax, -ln Z and an unused Top-1 entropy, for the target and for the draft rows (the
  // two sets back to back: the ratio rule scans [target rows ; draft rows] in one launch)
  const size_t sets = 3 * hs::align_up((size_t)2 * NN * sizeof(float), 256);
  // five doubles per row: what the rejection chains hand to the walk; two bytes per row: rows to scan
  const size_t chain = 5 * hs::align_up((size_t)NN * sizeof(double), 256) + hs::align_up((size_t)2 * NN, 256);
  // the sorted residual belongs to the ratio rule alone, and so does the scan of twice the rows
  const bool ratio = mode == HS_ACCEPT_STOCHASTIC;
  size_t sorted = ratio ? hs::bucket_workspace(NN, V, nullptr, nullptr) : 0;
  // the ratio rule's children counts, and the bonus distribution's row sums of every tree row
  if (ratio) sorted += hs::align_up((size_t)NN * sizeof(int32_t), 256) + hs::bonus_rows_bytes(NN, V);
  const size_t scan1 = hs::row_topk_workspace(NN, V, 1), scan2 = ratio ? hs::row_topk_workspace(2 * NN, V, 1) : 0;
  return sets + chain + sorted + (scan1 > scan2 ? scan1 : scan2);
}

extern "C" size_t hs_verify_accept_workspace(int32_t B, int32_t NN, int32_t V) {
  return hs_verify_accept_workspace_mode(B, NN, V, HS_ACCEPT_STOCHASTIC);  // the largest of the three
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
  const size_t need = hs_verify_accept_workspace_mode(B, NN, V, mode);
  HS_REQUIRE(need == 0 || (workspace && workspace_bytes >= need && reinterpret_cast<uintptr_t>(workspace) % 256 == 0),
             HS_ERR_WORKSPACE, "hs_verify_accept: workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
             workspace_bytes);
  int32_t *t_arg = nullptr, *d_arg = nullptr;
  float *t_lz = nullptr, *d_lz = nullptr;
  hs::ScanSlices slices{nullptr, nullptr, 1};
  slices.pairs_only = true;  // (the greedy walk needs the rows' argmax and nothing else)
  hs::ChainOut chain{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  hs::BucketWs bk{};  // (all NULL: no sorted residual)
  if (NN > 0) {
    hs::Carver c(workspace);
    t_arg = c.take<int32_t>(2 * (size_t)NN);
    t_lz = c.take<float>(2 * (size_t)NN);
    float* t_ent = c.take<float>(2 * (size_t)NN);
    d_arg = t_arg + NN;  // (the draft rows' results follow the target rows')
    d_lz = t_lz + NN;
    chain.child_p = c.take<double>(NN);
    chain.child_q = c.take<double>(NN);
    chain.child_frozen = c.take<double>(NN);
    chain.node_beta = c.take<double>(NN);
    chain.node_Z = c.take<double>(NN);
    uint8_t* wanted = c.take<uint8_t>(2 * (size_t)NN);
    if (mode == HS_ACCEPT_STOCHASTIC) {
      hs::bucket_workspace(NN, V, &c, &bk);
      chain.n_tried = c.take<int32_t>(NN);
      if (hs::bonus_rows_bytes(NN, V) > 0) chain.bonus_rows = c.take<double>((size_t)NN * ((V + 63) / 64));
    }
    void* scan_ws = c.take<char>(0);
    const float T = stochastic ? temperature : 1.0f;
    hs_status r;
    if (mode == HS_ACCEPT_STOCHASTIC) {
      // one scan over [target rows ; draft rows]; draft rows are read where a row has children, and
      // nowhere else
      hipLaunchKernelGGL(hs::k_mark_parents, dim3(B), dim3(hs::GR_THREADS), 0, st, parent, node_offsets, NN, wanted);
      r = hs::row_topk_launch(target_logits, row_stride, 2 * NN, V, 1, T, t_arg, t_lz, t_ent, nullptr, nullptr,
                              scan_ws, st, nullptr, wanted, nullptr, draft_logits, NN);
    } else {
      // greedy: the merge of the row slices is done by the accept kernel (one launch less)
      r = hs::row_topk_launch(target_logits, row_stride, NN, V, 1, T, t_arg, t_lz, t_ent, nullptr, nullptr, scan_ws,
                              st, stochastic ? nullptr : &slices);
    }
    if (r != HS_OK) return r;
  }
  if (!stochastic) {
    hipLaunchKernelGGL(hs::k_accept_greedy, dim3(B), dim3(hs::GR_THREADS), 0, st, t_arg, slices.val, slices.idx,
                       slices.count, token, parent, node_offsets, max_depth, accept_len, accept_path, bonus_token);
    return hs::launch_status("accept (greedy)");
  }
  if (mode == HS_ACCEPT_STOCHASTIC && NN > 0) {
    // the sorted residual pays from a few thousand tokens on and needs 16-byte aligned rows
    const bool sorted = bk.pairs != nullptr && V >= 4096 && row_stride % 4 == 0 &&
                        reinterpret_cast<uintptr_t>(target_logits) % 16 == 0 &&
                        reinterpret_cast<uintptr_t>(draft_logits) % 16 == 0;
    if (sorted) {
      const dim3 grid(hs::BK_SLICES, NN);
      hipLaunchKernelGGL(hs::k_bucket_pass<false>, grid, dim3(hs::BK_THREADS), 0, st, target_logits, draft_logits,
                         row_stride, parent, node_offsets, B, V, 1.0f / temperature, max_depth, t_arg, t_lz, d_arg,
                         d_lz, bk);
      hipLaunchKernelGGL(hs::k_bucket_scan, dim3(NN), dim3(hs::BK_N), 0, st, bk);
      hipLaunchKernelGGL(hs::k_bucket_pass<true>, grid, dim3(hs::BK_THREADS), 0, st, target_logits, draft_logits,
                         row_stride, parent, node_offsets, B, V, 1.0f / temperature, max_depth, t_arg, t_lz, d_arg,
                         d_lz, bk);
      hs_status r = hs::launch_status("accept (sorted residual)");
      if (r != HS_OK) return r;
    } else {
      bk.pairs = nullptr;
    }
    hipLaunchKernelGGL(hs::k_accept_chain, dim3(NN), dim3(hs::AC_THREADS), 0, st, target_logits, draft_logits,
                       row_stride, token, parent, node_offsets, B, V, 1.0f / temperature, max_depth, t_arg, t_lz,
                       d_arg, d_lz, chain, bk);
    hs_status r = hs::launch_status("accept (rejection chains)");
    if (r != HS_OK) return r;
    if (chain.bonus_rows != nullptr) {
      hipLaunchKernelGGL(hs::k_bonus_rows, dim3(hs::BR_SLICES, NN), dim3(hs::BR_THREADS), 0, st, target_logits,
                         draft_logits, row_stride, V, 1.0f / temperature, t_arg, t_lz, d_arg, d_lz, chain);
      r = hs::launch_status("accept (bonus rows)");
      if (r != HS_OK) return r;
    }
  }
  hipLaunchKernelGGL(hs::k_accept_walk, dim3(B), dim3(hs::AC_THREADS), 0, st, target_logits, draft_logits, row_stride,
                     token, parent, node_offsets, NN, V, (int)mode, 1.0f / temperature, uniforms, max_depth, t_arg,
                     t_lz, d_arg, d_lz, chain, accept_len, accept_path, bonus_token);
  return hs::launch_status("accept (stochastic)");
}
