// hs_draft_entropy_topk: one streaming pass over float32 logits rows.
//
// Computes, per row, the softmax statistics (max, sum of exponentials, entropy numerator) and the
// K best (logit, index) pairs (Section 4.1, Eq. 1; Section 2.2 Expansion).  HBM-bound: 4 bytes per
// logit, read once.
//
// One workgroup (four or sixteen waves, see below) scans a row (k_scan_rows), merges its waves'
// results and writes the outputs.  Only when there are too few rows to fill the chip is a row cut
// into slices for several workgroups; a small second kernel then merges the slices
// (k_scan_finalize).
//
// Top-K selection never sorts the data.  Each wave keeps its K best pairs as a sorted list in
// registers, entry l in lane l.  Per tile only the elements that are not worse than the list's K-th
// entry are looked at (one ballot per register); each of them is broadcast and inserted: the lanes
// whose entry it beats take their left neighbour's entry (or the new one), a shift by one lane done
// with a DPP move.  Before a list is full the threshold comes from the first tile: the K-th largest
// of the workgroup's wave maxima (of its 16-lane row maxima when it has fewer waves than K, of a
// wave's 64 lane maxima when even those are too few): K elements reach it, so no
// true Top-K member is ever filtered out, and only about K elements of the whole tile pass it.
// All decisions compare raw float32 logits under the strict order (value descending, index
// ascending), so the indices do not depend on how rows are split or reduced.
#include <limits.h>
#include <stdlib.h>

#include "hs_common.h"

namespace hs {

// The row scan is built for two workgroup sizes.  Sixteen waves: fewest slices to merge, best
// for a few dozen rows.  Four waves, several workgroups per compute unit: the workgroups' set-up,
// merge and write-out phases overlap with other workgroups' streaming, best for many rows (and
// for very few, where a row is cut into many short slices anyway).
constexpr int SCAN_BIG = 1024, SCAN_SMALL = 256;
constexpr int SCAN_VPT = 16;                        // values per thread per tile (4 x float4)
constexpr int scan_tile(int threads) { return threads * SCAN_VPT; }  // logits per workgroup tile
constexpr int FIN_THREADS = 256;
constexpr int FIN_CAP = HS_MAX_TOPK * HS_MAX_TOPK;  // candidates the merge of 64 slices can face
constexpr int MAX_SPLITS = 64;                       // slices per row (one list head per lane)
constexpr int SCAN_TARGET_WGS = 256;                 // rows are sliced until about one 16-wave workgroup per compute unit exists
constexpr float LOG2E = 1.4426950408889634f;

struct ScanPlan {
  int threads;       // workgroup size
  int splits;        // workgroups per row
  int tiles_per_wg;  // tiles each of them scans
};

static ScanPlan plan_scan(int R, int V) {
  ScanPlan p;
  p.threads = (R >= 256 || R <= 16) ? SCAN_SMALL : SCAN_BIG;  // measured on MI355X
  const int tile = scan_tile(p.threads);
  const int n_tiles = (V + tile - 1) / tile;
  // few rows: slice them until the chip is full (measured best)
  int want = SCAN_TARGET_WGS * (SCAN_BIG / p.threads) / (R > 0 ? R : 1);
  if (want > n_tiles) want = n_tiles;
  if (want > MAX_SPLITS) want = MAX_SPLITS;
  if (want < 1) want = 1;
  p.tiles_per_wg = (n_tiles + want - 1) / want;
  p.splits = (n_tiles + p.tiles_per_wg - 1) / p.tiles_per_wg;
  return p;
}

// Rank of this lane's pair among the pairs of lanes 0 .. n-1 (number of them holding a better pair).
__device__ __forceinline__ int wave_rank(float v, int i, int n) {
  int r = 0;
  for (int l = 0; l < n; ++l) {
    float ov = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
    int oi = __builtin_amdgcn_readlane(i, l);
    r += better(ov, oi, v, i) ? 1 : 0;
  }
  return r;
}

// The value of the lane to the left (lane 0 receives 0): a DPP move shifted by one lane across the wave.
__device__ __forceinline__ int from_left(int x) { return __builtin_amdgcn_update_dpp(0, x, 0x138, 0xf, 0xf, true); }

// Inserts the wave-uniform pair (xv, xi) into the sorted list held one entry per lane.
__device__ __forceinline__ void list_insert(float xv, int xi, float& lv, int& li) {
  const bool beats = better(xv, xi, lv, li);  // false ... false true ... true along the lanes
  const int left_beaten = from_left(beats ? 1 : 0);
  const float left_v = __builtin_bit_cast(float, from_left(__builtin_bit_cast(int, lv)));
  const int left_i = from_left(li);
  lv = beats ? (left_beaten ? left_v : xv) : lv;
  li = beats ? (left_beaten ? left_i : xi) : li;
}

// Maximum of each row of 16 lanes; lane 15 of a row holds it.
__device__ __forceinline__ float row16_max(float x) {
  const int id = __builtin_bit_cast(int, -HS_INF);
#define HS_DPP_STEP(ctrl, banks) \
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(id, __builtin_bit_cast(int, x), ctrl, 0xf, banks, false)))
  HS_DPP_STEP(0x111, 0xf);  // row_shr:1
  HS_DPP_STEP(0x112, 0xf);  // row_shr:2
  HS_DPP_STEP(0x114, 0xe);  // row_shr:4
  HS_DPP_STEP(0x118, 0xc);  // row_shr:8
#undef HS_DPP_STEP
  return x;
}

// Statistics of a wave's 64 lanes in one: the common maximum first, then plain sums of the lanes'
// terms rescaled to it.  The lowest lane that holds the maximum keeps its own maximum's unit out of
// s1 (as each lane did for itself); for every other lane that unit is an ordinary term.
__device__ __forceinline__ Stats stats_wave_sum(Stats a, float inv_t) {
  const float m = wave_max(a.m);
  if (m == -HS_INF) return stats_empty();
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((long long)__ballot(a.m == m)) - 1;
  float cs = 0.f, ct = 0.f;
  if (a.m != -HS_INF) {
    const float d = (a.m - m) * inv_t;  // <= 0
    const float e = exp2_fast(d * 1.4426950408889634f);
    const float w = 1.f + a.s1;
    cs = lane == leader ? a.s1 : e * w;
    ct = e * (a.t + d * w);
  }
  return Stats{m, wave_sum(cs), wave_sum(ct)};
}

// Scratch of the merges (shared memory).
template <int CAP>
struct MergeScratch {
  float cv[CAP];  // candidates
  int ci[CAP];
  int rank[CAP];
  float ov[HS_MAX_TOPK];  // the K best of them, in order
  int oi[HS_MAX_TOPK];
  int cnt;
  float thr_v;
  int thr_i;
  Stats total;
};

// Ranks the candidates sm.cv/ci[0, n) by counting (the order is strict: ranks are a permutation) and
// leaves those of rank < K, in order, in sm.ov / sm.oi.  With fewer candidates than threads a
// candidate's opponents are shared out among P threads, which add up their counts in LDS.
// Called by all `nthreads` threads (a power of two); sm.rank[0, n) must be zero on entry (a barrier
// before the call); ends with a barrier.
template <int CAP>
__device__ __forceinline__ void rank_candidates(MergeScratch<CAP>& sm, int n, int K, int tid, int nthreads) {
  int shift = 0;  // P = 2^shift threads per candidate
  while (n > 0 && (n << (shift + 1)) <= nthreads) ++shift;
  const int P = 1 << shift;
  const int chunk = (n + P - 1) >> shift;
  for (int base = 0; base < n; base += nthreads) {  // one trip unless n > nthreads
    const int a = base + (tid >> shift), part = tid & (P - 1);
    if (a < n) {
      const float av = sm.cv[a];
      const int ai = sm.ci[a];
      const int b0 = part * chunk, b1 = (b0 + chunk < n) ? b0 + chunk : n;
      int r = 0;
      for (int b = b0; b < b1; ++b) r += better(sm.cv[b], sm.ci[b], av, ai) ? 1 : 0;
      if (P > 1) atomicAdd(&sm.rank[a], r);
      else sm.rank[a] = r;
    }
  }
  __syncthreads();
  for (int a = tid; a < n; a += nthreads) {
    const int r = sm.rank[a];
    if (r < K) {
      sm.ov[r] = sm.cv[a];
      sm.oi[r] = sm.ci[a];
    }
  }
  __syncthreads();
}

// Loads and stores that are coherent across the chip's XCDs (each has an L2 of its own): relaxed
// atomics of device scope, which go past a stale or private cache line.  What workgroups of one
// launch use to hand their slices' results to each other: a fence that reaches the other XCDs
// would write back and invalidate a whole L2, and cost the scan several times its own duration.
__device__ __forceinline__ float ld_dev(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ int ld_dev(const int* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(int* p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Merges S <= 64 slices of a row: statistics st[s] (m, s1, t) and sorted K-lists pv/pi[s * K + k].
// COHERENT: the slices were written by other workgroups of the same launch (ld_dev).
// Leaves the row's statistics in sm.total and its K best pairs, in order, in sm.ov / sm.oi.
// Called by all `nthreads` threads of the workgroup (tid 0..nthreads-1); ends with a barrier.
// Everything the merge reads from memory is requested at once (one trip, which is most of its
// time when the slices come from other workgroups): the lists by all threads, the statistics by the
// last wave.  Then the K-th best list head becomes a threshold (with at least K lists), which only
// a few entries pass, and those are ranked by counting.
template <bool COHERENT, int CAP>
__device__ __forceinline__ void merge_slices(const float4* st, const float* pv, const int* pi, int S, int K,
                                             float inv_t, MergeScratch<CAP>& sm, int tid, int nthreads) {
  const int lane = tid & 63;
  __shared__ float head_v[MAX_SPLITS];
  __shared__ int head_i[MAX_SPLITS];
  constexpr int PER = 4;  // entries a thread keeps in registers (a trip covers PER x nthreads of the S x K)
  const int n_all = S * K;
  float ev[PER];
  int ei[PER];
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const int e = tid + q * nthreads;
    ev[q] = -HS_INF;
    ei[q] = INT_MAX;
    if (e < n_all) {
      ev[q] = COHERENT ? ld_dev(pv + e) : pv[e];
      ei[q] = COHERENT ? ld_dev(pi + e) : pi[e];
    }
  }
  Stats a = stats_empty();
  const bool stats_wave = tid >= nthreads - 64;
  if (stats_wave && lane < S) {
    if (COHERENT) {
      const float* sf = reinterpret_cast<const float*>(st + lane);
      a = Stats{ld_dev(sf), ld_dev(sf + 1), ld_dev(sf + 2)};
    } else {
      const float4 f = st[lane];
      a = Stats{f.x, f.y, f.z};
    }
  }
  for (int e = tid; e < n_all; e += nthreads) sm.rank[e] = 0;
  if (tid == 0) sm.cnt = 0;
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const int e = tid + q * nthreads;
    if (e < n_all && e % K == 0) {
      head_v[e / K] = ev[q];
      head_i[e / K] = ei[q];
    }
  }
  if (stats_wave) {
    a = stats_wave_sum(a, inv_t);
    if (lane == 0) sm.total = a;
  }
  __syncthreads();
  if (tid < 64) {
    // threshold: the K-th best list head when there are at least K lists, else "everything passes"
    float tv = -HS_INF;
    int ti = INT_MAX;
    if (S >= K) {
      const float hv = lane < S ? head_v[lane] : -HS_INF;
      const int hi = lane < S ? head_i[lane] : INT_MAX;
      int r = wave_rank(hv, hi, S);
      unsigned long long who = __ballot(r == K - 1 && lane < S);
      if (who != 0ull) {
        int src = __ffsll((long long)who) - 1;
        tv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, hv), src));
        ti = __builtin_amdgcn_readlane(hi, src);
      }
    }
    if (lane == 0) {
      sm.thr_v = tv;
      sm.thr_i = ti;
    }
  }
  __syncthreads();
  {
    const float tv = sm.thr_v;
    const int ti = sm.thr_i;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      if (ei[q] != INT_MAX && !better(tv, ti, ev[q], ei[q])) {  // (INT_MAX: an unused list entry, or none)
        int pos = atomicAdd(&sm.cnt, 1);  // order of arrival does not matter: ranks are computed below
        sm.cv[pos] = ev[q];               // (at most S * K <= CAP entries)
        sm.ci[pos] = ei[q];
      }
    }
    // (more entries than PER x nthreads: the rest in further trips)
    for (int e = tid + PER * nthreads; e < n_all; e += nthreads) {
      float v = COHERENT ? ld_dev(pv + e) : pv[e];
      int i = COHERENT ? ld_dev(pi + e) : pi[e];
      if (i != INT_MAX && !better(tv, ti, v, i)) {
        int pos = atomicAdd(&sm.cnt, 1);
        sm.cv[pos] = v;
        sm.ci[pos] = i;
      }
    }
  }
  __syncthreads();
  rank_candidates(sm, sm.cnt, K, tid, nthreads);
}

// Writes a row's results from its merged statistics and Top-K list (first wave of the workgroup).
template <int CAP>
__device__ __forceinline__ void write_row(const MergeScratch<CAP>& sm, int64_t row, int K, float inv_t,
                                          int32_t* __restrict__ topk_idx, float* __restrict__ topk_logp,
                                          float* __restrict__ ent_topk, float* __restrict__ ent_full,
                                          float* __restrict__ lse, int tid) {
  if (tid >= 64) return;
  const int lane = tid;
  const float m = sm.total.m, s1 = sm.total.s1, t = sm.total.t;
  const float l1p = log1pf(s1);
  if (lane < K) {
    topk_idx[row * K + lane] = sm.oi[lane];
    topk_logp[row * K + lane] = (sm.ov[lane] - m) * inv_t - l1p;
  }
  // Top-K probabilities renormalised over the K: weights relative to the best one (lane = entry);
  // entropy = ln(1 + sum w) - sum(w a) / (1 + sum w), every term of one sign
  float w = 0.f, wa = 0.f;
  if (lane >= 1 && lane < K) {
    const float a = (sm.ov[lane] - sm.ov[0]) * inv_t;
    if (a > -100.f) {
      w = expf(a);
      wa = w * a;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    w += __shfl_xor(w, off);
    wa += __shfl_xor(wa, off);
  }
  if (lane == 0) {
    ent_topk[row] = log1pf(w) - wa / (1.f + w);
    if (ent_full) ent_full[row] = l1p - t / (1.f + s1);
    if (lse) lse[row] = m * inv_t + l1p;
  }
}

// grid (S, R): slice `blockIdx.x` of row `blockIdx.y`.  S == 1: the outputs are written here;
// S > 1: the slice's statistics and K-list go to part_* for k_scan_finalize, or, FUSED, for the
// workgroup that finishes a row's last slice: every workgroup draws a ticket from the row's counter
// (`tickets`, zero before the launch), the one that draws S - 1 knows that all slices are written,
// puts the counter back to zero for the next launch, merges the slices and writes the row.
constexpr int FUSED_CAP = 1024;  // slices x K that the merging workgroup's scratch holds
constexpr size_t TICKET_BYTES = 65536 * sizeof(unsigned);  // a counter for each of the at most 65535 rows of a call
// STATS false: only the K best pairs are wanted (the greedy accept walk's argmax scan); the softmax
// statistics, most of the arithmetic of a tile, are left out and part_stats is not written.
template <bool VEC, int SCAN_THREADS, bool FUSED, int NBUF, bool STATS>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_rows(const float* __restrict__ logits, int64_t row_stride,
                                                            int V, int K, float inv_t, int tiles_per_wg,
                                                            float4* __restrict__ part_stats,
                                                            float* __restrict__ part_val, int* __restrict__ part_idx,
                                                            int32_t* __restrict__ topk_idx,
                                                            float* __restrict__ topk_logp,
                                                            float* __restrict__ ent_topk,
                                                            float* __restrict__ ent_full, float* __restrict__ lse,
                                                            const uint8_t* __restrict__ row_active,
                                                            const int32_t* __restrict__ row_index,
                                                            const float* __restrict__ logits2, int rows1,
                                                            unsigned* __restrict__ tickets) {
  if (row_active != nullptr && row_active[blockIdx.y] == 0) return;  // (the whole workgroup: a row nobody will read)
  // (both arms as int64: mixed with the unsigned block index a negative entry would turn positive)
  const int64_t src_row = row_index != nullptr ? (int64_t)row_index[blockIdx.y] : (int64_t)blockIdx.y;
  if (src_row < 0) return;
  constexpr int SCAN_WAVES = SCAN_THREADS / 64;
  constexpr int SCAN_GROUPS = SCAN_WAVES * 4 < 64 ? SCAN_WAVES * 4 : 64;  // rows of 16 lanes, at most one per lane
  constexpr int SCAN_TILE = scan_tile(SCAN_THREADS);
  // candidates the merge of the waves can face (and, FUSED, the merge of a row's slices)
  constexpr int SCAN_CAP = (FUSED && SCAN_WAVES * HS_MAX_TOPK < FUSED_CAP) ? FUSED_CAP : SCAN_WAVES * HS_MAX_TOPK;
  __shared__ float4 wave_st[SCAN_WAVES];
  __shared__ float group_maxima[SCAN_GROUPS];
  __shared__ MergeScratch<SCAN_CAP> sm;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x, S = gridDim.x, row = blockIdx.y;
  // (rows from rows1 on may lie in a second array)
  const float* __restrict__ x = (logits2 != nullptr && src_row >= rows1) ? logits2 + (src_row - rows1) * row_stride
                                                                         : logits + src_row * row_stride;

  // this wave's K best pairs so far, best first, entry l in lane l; the rest holds a pair that
  // loses against every real one
  float lv = -HS_INF;
  int li = INT_MAX;
  // statistics are kept in the log2 domain while scanning: y = (x - m) * c, c = log2(e) / T
  const float c = inv_t * LOG2E;
  float m = -HS_INF, s1 = 0.f, t2 = 0.f;
  float thr = -HS_INF;
  int thr_i = INT_MAX;  // among elements equal to thr only those with a lower index can still enter the list
  if (tid == 0) sm.cnt = 0;
  if (tid < HS_MAX_TOPK) {  // a slice with fewer than K elements leaves the rest of its list unused
    sm.ov[tid] = -HS_INF;
    sm.oi[tid] = INT_MAX;
  }
  __syncthreads();

  auto load_tile = [&](int tile, float (&v)[SCAN_VPT]) {
    const int tbase = (split * tiles_per_wg + tile) * SCAN_TILE;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i0 = tbase + (j * SCAN_THREADS + tid) * 4;
      if (VEC && i0 + 3 < V) {
        float4 f = *reinterpret_cast<const float4*>(x + i0);
        v[j * 4 + 0] = f.x;
        v[j * 4 + 1] = f.y;
        v[j * 4 + 2] = f.z;
        v[j * 4 + 3] = f.w;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[j * 4 + e] = (i0 + e < V) ? x[i0 + e] : -HS_INF;
      }
    }
  };
  // a tile that lies inside the row as a whole (aligned rows): four loads, no conditions, so the
  // compiler can count them when it waits for an older tile
  auto load_full_tile = [&](int tile, float (&v)[SCAN_VPT]) {
    const float* __restrict__ src = x + (int64_t)(split * tiles_per_wg + tile) * SCAN_TILE + tid * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float4 f = *reinterpret_cast<const float4*>(src + j * SCAN_THREADS * 4);
      v[j * 4 + 0] = f.x;
      v[j * 4 + 1] = f.y;
      v[j * 4 + 2] = f.z;
      v[j * 4 + 3] = f.w;
    }
  };
  // tiles this workgroup really has (uniform)
  int n_my = (V - split * tiles_per_wg * SCAN_TILE + SCAN_TILE - 1) / SCAN_TILE;
  n_my = n_my < 0 ? 0 : (n_my > tiles_per_wg ? tiles_per_wg : n_my);
  int n_full = VEC ? (V - split * tiles_per_wg * SCAN_TILE) / SCAN_TILE : 0;  // leading whole tiles
  n_full = n_full < 0 ? 0 : (n_full > n_my ? n_my : n_full);

  // One tile: statistics of this thread's 16 values, threshold, insertion of the few values that
  // reach it.
  auto process = [&](const float (&v)[SCAN_VPT], int tile) {
    const int tbase = (split * tiles_per_wg + tile) * SCAN_TILE;
#define HS_IDX(jj) (tbase + (((jj) >> 2) * SCAN_THREADS + tid) * 4 + ((jj)&3))

    // ---- softmax statistics of this thread's values
    float tm = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
    tm = fmaxf(tm, fmaxf(fmaxf(fmaxf(v[8], v[9]), fmaxf(v[10], v[11])), fmaxf(fmaxf(v[12], v[13]), fmaxf(v[14], v[15]))));
    int skip = -1;
    if (STATS && tm > m) {
#pragma unroll
      for (int jj = SCAN_VPT - 1; jj >= 0; --jj) skip = (v[jj] == tm) ? jj : skip;  // first instance of the max
      if (m != -HS_INF) {
        const float d2 = (m - tm) * c;
        const float e = exp2_fast(d2);
        const float w = 1.f + s1;
        t2 = e * (t2 + d2 * w);
        s1 = e * w;
      }
      m = tm;
    }
    if (STATS && tm != -HS_INF) {
#pragma unroll
      for (int jj = 0; jj < SCAN_VPT; ++jj) {
        // x - m first: exact near the maximum (an fma with a rounded m * c would leave the maximum's
        // own y slightly off zero and put that into t2); the clamp keeps 0 * -inf out of t2
        const float y = fmaxf((v[jj] - m) * c, -1e30f);
        const float e = exp2_fast(y);
        t2 = fmaf(e, y, t2);
        s1 += (jj == skip) ? 0.f : e;
      }
    }

    // ---- threshold (a value): no element below it can be among the row's K best.  First tile:
    // the K-th largest of the workgroup's group maxima (K elements of the tile reach it), or of
    // this wave's 64 lane maxima; afterwards also the wave's own K-th entry once its list is full.
    if (tile == 0) {
      if (K <= SCAN_GROUPS) {
        // maxima of the waves, or of their rows of 16 lanes when there are fewer waves than K
        const bool by_wave = K <= SCAN_WAVES;
        const int n_groups = by_wave ? SCAN_WAVES : SCAN_GROUPS;
        if (by_wave) {
          const float wm = wave_max(tm);
          if (lane == 0) group_maxima[wave] = wm;
        } else {
          const float rm = row16_max(tm);
          if ((lane & 15) == 15) group_maxima[wave * 4 + (lane >> 4)] = rm;
        }
        // an exchange through LDS only: the barrier must not wait for the next tiles' loads
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const float mine = lane < n_groups ? group_maxima[lane] : -HS_INF;
        const int r = wave_rank(mine, lane, n_groups);
        const unsigned long long who = __ballot(r == K - 1 && lane < n_groups);
        thr = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine), __ffsll((long long)who) - 1));
      } else {
        const int r = wave_rank(tm, lane, 64);
        const unsigned long long who = __ballot(r == K - 1);
        thr = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, tm), __ffsll((long long)who) - 1));
      }
    }
    // the wave's own K-th entry, once it is at least as good as the threshold, replaces it as a
    // (value, index) pair: an element that equals it in value enters only with a lower index
    // (rows of equal logits would otherwise send every element through the insertion)
    auto tighten = [&]() {
      const float kv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lv), K - 1));
      if (kv >= thr) {
        thr = kv;
        thr_i = __builtin_amdgcn_readlane(li, K - 1);  // INT_MAX while the list is not full
      }
    };
    tighten();

    // ---- insert the elements that reach the threshold (skipped when no lane's maximum does)
    if (__ballot(tm >= thr) != 0ull) {
#pragma unroll
      for (int jj = 0; jj < SCAN_VPT; ++jj) {
        if (__ballot(v[jj] >= thr) != 0ull) {
          const int idx = HS_IDX(jj);
          unsigned long long todo = __ballot(v[jj] > thr || (v[jj] == thr && idx < thr_i));
          while (todo != 0ull) {
            const int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1ull;
            const float xv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v[jj]), src));
            const int xi = __builtin_amdgcn_readlane(idx, src);
            list_insert(xv, xi, lv, li);
          }
          tighten();
        }
      }
    }
#undef HS_IDX
  };
  // NBUF register buffers, NBUF - 1 tiles in flight: the loads of tile t + NBUF - 1 are requested
  // before tile t is processed (what is in flight bounds the bandwidth).  The steady-state loop
  // requests without a condition, so that the wait before a tile's values counts exactly the younger
  // tiles; the last tiles run through the guarded copy below.
  float buf[NBUF][SCAN_VPT];
  // (whole tiles by the unconditional loads: the guarded ones wait for each other)
#pragma unroll
  for (int b = 0; b < NBUF - 1; ++b) {
    if (b < n_full) load_full_tile(b, buf[b]);
    else if (b < n_my) load_tile(b, buf[b]);
  }
  int tile = 0;
  for (; tile + 2 * NBUF - 2 < n_full; tile += NBUF) {
#pragma unroll
    for (int b = 0; b < NBUF; ++b) {
      load_full_tile(tile + b + NBUF - 1, buf[(b + NBUF - 1) % NBUF]);
      process(buf[b], tile + b);
    }
  }
  for (; tile < n_my; tile += NBUF) {
#pragma unroll
    for (int b = 0; b < NBUF; ++b) {
      if (tile + b < n_my) {
        if (tile + b + NBUF - 1 < n_my) load_tile(tile + b + NBUF - 1, buf[(b + NBUF - 1) % NBUF]);
        process(buf[b], tile + b);
      }
    }
  }

  // ---- the waves' statistics and the real entries of their lists meet in LDS
  if (STATS) {
    Stats st{m, s1, t2 * 0.6931471805599453f};  // back to natural-log units
    st = stats_wave_sum(st, inv_t);
    if (lane == 0) wave_st[wave] = make_float4(st.m, st.s1, st.t, 0.f);
  }
  {
    const bool real = lane < K && li != INT_MAX;  // a list's real entries come first
    const int n_w = __popcll(__ballot(real));
    int base = 0;
    if (lane == 0) base = atomicAdd(&sm.cnt, n_w);  // (zeroed at the start, a barrier ago)
    base = __builtin_amdgcn_readfirstlane(base);
    if (real) {
      sm.cv[base + lane] = lv;
      sm.ci[base + lane] = li;
      sm.rank[base + lane] = 0;
    }
  }
  __syncthreads();
  if (STATS && tid < 64) {
    Stats a = stats_empty();
    if (lane < SCAN_WAVES) {
      const float4 f = wave_st[lane];
      a = Stats{f.x, f.y, f.z};
    }
    a = stats_wave_sum(a, inv_t);
    if (lane == 0) sm.total = a;
  }
  rank_candidates(sm, sm.cnt, K, tid, SCAN_THREADS);  // (its first barrier also publishes sm.total)
  static_assert(STATS || !FUSED, "rows are finished by the caller of a scan without statistics");
  if (S == 1) {
    if (STATS) write_row(sm, row, K, inv_t, topk_idx, topk_logp, ent_topk, ent_full, lse, tid);
    else if (tid < K) topk_idx[row * K + tid] = sm.oi[tid];
  } else {
    const int64_t slot = (int64_t)row * S + split;
    if (!FUSED) {
      if (tid < K) {
        part_val[slot * K + tid] = sm.ov[tid];
        part_idx[slot * K + tid] = sm.oi[tid];
      }
      if (STATS && tid == 0) part_stats[slot] = make_float4(sm.total.m, sm.total.s1, sm.total.t, 0.f);
    } else {
      __shared__ int is_last;
      // The slice's results go out by the first wave alone, with stores that the other XCDs see; once
      // they are acknowledged (vmcnt) the ticket is drawn.  The workgroup that draws the last one
      // finds every slice of the row written.
      if (tid < 64) {
        if (tid < K) {
          st_dev(part_val + slot * K + tid, sm.ov[tid]);
          st_dev(part_idx + slot * K + tid, sm.oi[tid]);
        }
        if (tid < 3) st_dev(reinterpret_cast<float*>(part_stats + slot) + tid, tid == 0 ? sm.total.m : tid == 1 ? sm.total.s1 : sm.total.t);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (tid == 0) {
          const unsigned drawn = __hip_atomic_fetch_add(&tickets[row], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          is_last = drawn == (unsigned)(S - 1) ? 1 : 0;
          // (nobody else touches this row's counter any more: back to zero for the next launch)
          if (is_last) __hip_atomic_store(&tickets[row], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      __syncthreads();
      if (is_last) {
        merge_slices<true>(part_stats + (int64_t)row * S, part_val + (int64_t)row * S * K, part_idx + (int64_t)row * S * K,
                           S, K, inv_t, sm, tid, SCAN_THREADS);
        write_row(sm, row, K, inv_t, topk_idx, topk_logp, ent_topk, ent_full, lse, tid);
      }
    }
  }
}

// Clears a workspace (hs_workspace_prepare): a fill kernel, not a memset, so that it may be captured.
__global__ __launch_bounds__(256) void k_fill_zero(uint4* __restrict__ p, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

__global__ __launch_bounds__(FIN_THREADS) void k_scan_finalize(const float4* __restrict__ part_stats,
                                                               const float* __restrict__ part_val,
                                                               const int* __restrict__ part_idx, int S, int K,
                                                               float inv_t, int32_t* __restrict__ topk_idx,
                                                               float* __restrict__ topk_logp,
                                                               float* __restrict__ ent_topk,
                                                               float* __restrict__ ent_full,
                                                               float* __restrict__ lse,
                                                               const uint8_t* __restrict__ row_active,
                                                               const int32_t* __restrict__ row_index) {
  __shared__ MergeScratch<FIN_CAP> sm;
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  if (row_active != nullptr && row_active[row] == 0) return;
  if (row_index != nullptr && row_index[row] < 0) return;
  merge_slices<false>(part_stats + row * S, part_val + row * S * K, part_idx + row * S * K, S, K, inv_t, sm, tid, FIN_THREADS);
  write_row(sm, row, K, inv_t, topk_idx, topk_logp, ent_topk, ent_full, lse, tid);
}

size_t row_topk_workspace(int R, int V, int K) {
  if (R <= 0) return 0;
  ScanPlan p = plan_scan(R, V);
  size_t n = (size_t)R * p.splits;
  return TICKET_BYTES + align_up(n * sizeof(float4), 256) + 2 * align_up(n * K * sizeof(float), 256);
}

hs_status row_topk_launch(const float* logits, int64_t row_stride, int R, int V, int K, float temperature,
                          int32_t* topk_idx, float* topk_logp, float* ent_topk, float* ent_full, float* lse,
                          void* workspace, hipStream_t stream, ScanSlices* slices, const uint8_t* row_active,
                          const int32_t* row_index, const float* logits2, int rows1, bool prepared) {
  // (rows are the grid's second dimension)
  HS_REQUIRE(R <= 65535, HS_ERR_UNSUPPORTED, "row scan: %d rows in one call (at most 65535)", R);
  ScanPlan p = plan_scan(R, V);
  Carver c(workspace);
  size_t n = (size_t)R * p.splits;
  // one counter per row, zero in a prepared workspace and left at zero; always the same leading part
  // of the workspace, whatever the shape, so that calls of different shapes can share a prepared one
  unsigned* tickets = c.take<unsigned>(TICKET_BYTES / sizeof(unsigned));
  float4* part_stats = c.take<float4>(n);
  float* part_val = c.take<float>(n * K);
  int* part_idx = c.take<int>(n * K);
  const float inv_t = 1.0f / temperature;
  const bool vec = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 4 == 0) &&
                   (reinterpret_cast<uintptr_t>(logits2) % 16 == 0);
  dim3 grid(p.splits, R);
  // one launch: the rows' last slices merge (needs the zeroed counters of a prepared workspace)
  const bool fused = prepared && slices == nullptr && p.splits > 1 && p.splits * K <= FUSED_CAP;
#define HS_SCAN_LAUNCH(VEC, T, F, ST)                                                                                     \
  hipLaunchKernelGGL((k_scan_rows<VEC, T, F, 3, ST>), grid, dim3(T), 0, stream, logits, row_stride, V, K, inv_t, p.tiles_per_wg, \
                     part_stats, part_val, part_idx, topk_idx, topk_logp, ent_topk, ent_full, lse, row_active, row_index, logits2, rows1, tickets)
  if (slices != nullptr && slices->pairs_only) {
    if (p.threads == SCAN_BIG) {
      if (vec) HS_SCAN_LAUNCH(true, SCAN_BIG, false, false);
      else HS_SCAN_LAUNCH(false, SCAN_BIG, false, false);
    } else {
      if (vec) HS_SCAN_LAUNCH(true, SCAN_SMALL, false, false);
      else HS_SCAN_LAUNCH(false, SCAN_SMALL, false, false);
    }
  } else if (fused) {
    if (p.threads == SCAN_BIG) {
      if (vec) HS_SCAN_LAUNCH(true, SCAN_BIG, true, true);
      else HS_SCAN_LAUNCH(false, SCAN_BIG, true, true);
    } else {
      if (vec) HS_SCAN_LAUNCH(true, SCAN_SMALL, true, true);
      else HS_SCAN_LAUNCH(false, SCAN_SMALL, true, true);
    }
  } else if (p.threads == SCAN_BIG) {
    if (vec) HS_SCAN_LAUNCH(true, SCAN_BIG, false, true);
    else HS_SCAN_LAUNCH(false, SCAN_BIG, false, true);
  } else {
    if (vec) HS_SCAN_LAUNCH(true, SCAN_SMALL, false, true);
    else HS_SCAN_LAUNCH(false, SCAN_SMALL, false, true);
  }
#undef HS_SCAN_LAUNCH
  hs_status st = launch_status("row scan");
  if (slices != nullptr) {
    slices->val = part_val;
    slices->idx = part_idx;
    slices->count = p.splits;
  }
  if (st != HS_OK || p.splits == 1 || slices != nullptr || fused) return st;
  hipLaunchKernelGGL(k_scan_finalize, dim3(R), dim3(FIN_THREADS), 0, stream, part_stats, part_val, part_idx,
                     p.splits, K, inv_t, topk_idx, topk_logp, ent_topk, ent_full, lse, row_active, row_index);
  return launch_status("row scan merge");
}

}  // namespace hs

extern "C" size_t hs_draft_entropy_topk_workspace(int32_t R, int32_t V, int32_t K) {
  if (R <= 0 || V <= 0 || K <= 0 || K > HS_MAX_TOPK) return 0;
  return hs::row_topk_workspace(R, V, K);
}

static hs_status entropy_topk_impl(const float* logits, int64_t row_stride, const int32_t* row_index, int32_t R,
                                   int32_t V, int32_t K, float temperature, int32_t* topk_idx, float* topk_logp,
                                   float* ent_topk, float* ent_full, float* lse, void* workspace,
                                   size_t workspace_bytes, hs_stream stream, bool prepared = false) {
  hs::clear_error();
  HS_REQUIRE(R >= 0 && V >= 1, HS_ERR_SHAPE, "hs_draft_entropy_topk: R=%d V=%d", R, V);
  HS_REQUIRE(K >= 1 && K <= V, HS_ERR_SHAPE, "hs_draft_entropy_topk: K=%d must be in 1..V=%d", K, V);
  HS_REQUIRE(K <= HS_MAX_TOPK, HS_ERR_UNSUPPORTED, "hs_draft_entropy_topk: K=%d exceeds HS_MAX_TOPK=%d", K,
             HS_MAX_TOPK);
  HS_REQUIRE(row_stride >= V, HS_ERR_SHAPE, "hs_draft_entropy_topk: row_stride=%lld < V=%d", (long long)row_stride, V);
  HS_REQUIRE(temperature > 0.f, HS_ERR_SHAPE, "hs_draft_entropy_topk: temperature must be positive");
  if (R == 0) return HS_OK;
  HS_REQUIRE(logits && topk_idx && topk_logp && ent_topk, HS_ERR_NULL, "hs_draft_entropy_topk: NULL argument");
  size_t need = hs::row_topk_workspace(R, V, K);
  HS_REQUIRE(workspace && workspace_bytes >= need && reinterpret_cast<uintptr_t>(workspace) % 256 == 0,
             HS_ERR_WORKSPACE, "hs_draft_entropy_topk: workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
             workspace_bytes);
  return hs::row_topk_launch(logits, row_stride, R, V, K, temperature, topk_idx, topk_logp, ent_topk, ent_full, lse,
                             workspace, static_cast<hipStream_t>(stream), nullptr, nullptr, row_index, nullptr, 0, prepared);
}

extern "C" hs_status hs_draft_entropy_topk(const float* logits, int64_t row_stride, int32_t R, int32_t V, int32_t K,
                                           float temperature, int32_t* topk_idx, float* topk_logp, float* ent_topk,
                                           float* ent_full, float* lse, void* workspace, size_t workspace_bytes,
                                           hs_stream stream) {
  return entropy_topk_impl(logits, row_stride, nullptr, R, V, K, temperature, topk_idx, topk_logp, ent_topk, ent_full,
                           lse, workspace, workspace_bytes, stream);
}

extern "C" hs_status hs_draft_entropy_topk_rows(const float* logits, int64_t row_stride, const int32_t* row_index,
                                                int32_t R, int32_t V, int32_t K, float temperature,
                                                int32_t* topk_idx, float* topk_logp, float* ent_topk, float* ent_full,
                                                float* lse, void* workspace, size_t workspace_bytes,
                                                hs_stream stream) {
  HS_REQUIRE(R <= 0 || row_index != nullptr, HS_ERR_NULL, "hs_draft_entropy_topk_rows: row_index is NULL");
  return entropy_topk_impl(logits, row_stride, row_index, R, V, K, temperature, topk_idx, topk_logp, ent_topk,
                           ent_full, lse, workspace, workspace_bytes, stream);
}

extern "C" hs_status hs_draft_entropy_topk_fused(const float* logits, int64_t row_stride, const int32_t* row_index,
                                                 int32_t R, int32_t V, int32_t K, float temperature,
                                                 int32_t* topk_idx, float* topk_logp, float* ent_topk, float* ent_full,
                                                 float* lse, void* workspace, size_t workspace_bytes,
                                                 hs_stream stream) {
  return entropy_topk_impl(logits, row_stride, row_index, R, V, K, temperature, topk_idx, topk_logp, ent_topk,
                           ent_full, lse, workspace, workspace_bytes, stream, true);
}

extern "C" hs_status hs_workspace_prepare(void* workspace, size_t workspace_bytes, hs_stream stream) {
  hs::clear_error();
  if (workspace_bytes == 0) return HS_OK;
  HS_REQUIRE(workspace != nullptr, HS_ERR_NULL, "hs_workspace_prepare: NULL workspace");
  HS_REQUIRE(reinterpret_cast<uintptr_t>(workspace) % 256 == 0 && workspace_bytes % 16 == 0, HS_ERR_WORKSPACE,
             "hs_workspace_prepare: the workspace must be 256-byte aligned and a multiple of 16 bytes long (got %zu)",
             workspace_bytes);
  const size_t n16 = workspace_bytes / 16;
  HS_REQUIRE((n16 + 255) / 256 <= 0x7fffffffull, HS_ERR_UNSUPPORTED, "hs_workspace_prepare: %zu bytes", workspace_bytes);
  hipLaunchKernelGGL(hs::k_fill_zero, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<uint4*>(workspace), n16);
  return hs::launch_status("workspace prepare");
}
