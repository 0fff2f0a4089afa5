// hs_draft_entropy_topk: one streaming pass over float32 logits rows.
//
// Computes, per row, the softmax statistics (max, sum of exponentials, entropy numerator) and the
// K best (logit, index) pairs (Section 4.1, Eq. 1; Section 2.2 Expansion).  A row is cut into
// slices handled by different workgroups (k_scan_rows); a small second kernel merges the slices of
// a row and writes the results (k_scan_finalize).  HBM-bound: 4 bytes per logit, read once.
//
// Top-K selection never sorts the data.  Each wave keeps a running sorted list of its K best
// pairs; per 4096-element tile it compacts (ballot + popcount, deterministic positions) only the
// elements that are not worse than a threshold into LDS and re-ranks "list + candidates" by
// counting, which also sorts them.  The threshold is the list's K-th entry, or, for a wave's first
// tile, the K-th best of the 64 per-lane maxima (at least K elements are at or above it, so no
// true Top-K member is ever filtered out).  All decisions compare raw float32 logits under the
// strict order (value descending, index ascending), so the indices do not depend on how rows are
// split or reduced.
#include <limits.h>

#include "hs_common.h"

namespace hs {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_WAVES = SCAN_THREADS / 64;
constexpr int SCAN_VPT = 16;                        // values per thread per tile (4 x float4)
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_VPT;  // 4096 logits per workgroup tile
constexpr int CAND_CAP = 64 * SCAN_VPT + HS_MAX_TOPK;  // a wave's whole tile plus its list
constexpr int FIN_THREADS = 256;
constexpr int FIN_CAP = HS_MAX_TOPK * HS_MAX_TOPK;  // candidates the merge can face
constexpr int MAX_SPLITS = 64;                       // slices per row (one list head per lane)
constexpr float LOG2E = 1.4426950408889634f;

struct ScanPlan {
  int splits;        // workgroups per row
  int tiles_per_wg;  // tiles each of them scans
};

static ScanPlan plan_scan(int R, int V) {
  int n_tiles = (V + SCAN_TILE - 1) / SCAN_TILE;
  int want = 2048 / (R > 0 ? R : 1);  // aim at ~8 workgroups per compute unit
  if (want < 1) want = 1;
  if (want > n_tiles) want = n_tiles;
  if (want > MAX_SPLITS) want = MAX_SPLITS;
  int tpw = (n_tiles + want - 1) / want;
  int min_tpw = (n_tiles + MAX_SPLITS - 1) / MAX_SPLITS;
  if (tpw < min_tpw) tpw = min_tpw;
  ScanPlan p;
  p.tiles_per_wg = tpw;
  p.splits = (n_tiles + tpw - 1) / tpw;
  return p;
}

// Re-ranks entries [0, n) of (cv, ci) by counting and writes those of rank < K, in order, to (ov, oi).
// Called by `nthreads` cooperating threads (whole waves) with ids 0..nthreads-1; the caller
// synchronises around it.  The entries to compare against are held 64 at a time in registers and
// broadcast lane by lane, so the inner loop has no memory latency in it.
__device__ __forceinline__ void rank_select(const float* cv, const int* ci, int n, int K, float* ov, int* oi,
                                            int id, int nthreads) {
  const int lane = id & 63;
  for (int base = 0; base < n; base += nthreads) {  // uniform trip count
    const int a = base + id;
    float av = -HS_INF;
    int ai = INT_MAX;
    if (a < n) {
      av = cv[a];
      ai = ci[a];
    }
    int r = 0;
    for (int c0 = 0; c0 < n; c0 += 64) {
      float bv = -HS_INF;
      int bi = INT_MAX;
      if (c0 + lane < n) {
        bv = cv[c0 + lane];
        bi = ci[c0 + lane];
      }
      const int m = (n - c0) < 64 ? (n - c0) : 64;
      for (int j = 0; j < m; ++j) {
        const float xv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bv), j));
        const int xi = __builtin_amdgcn_readlane(bi, j);
        r += better(xv, xi, av, ai) ? 1 : 0;
      }
    }
    if (a < n && r < K) {
      ov[r] = av;
      oi[r] = ai;
    }
  }
}

// Orders this wave's LDS traffic: what lanes wrote before is visible to all lanes after.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Rank of this lane's pair among the 64 lanes' pairs (number of lanes holding a better pair).
__device__ __forceinline__ int wave_rank(float v, int i) {
  int r = 0;
#pragma unroll
  for (int l = 0; l < 64; ++l) {
    float ov = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
    int oi = __builtin_amdgcn_readlane(i, l);
    r += better(ov, oi, v, i) ? 1 : 0;
  }
  return r;
}

template <bool VEC>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_rows(const float* __restrict__ logits, int64_t row_stride,
                                                            int V, int K, float inv_t, int tiles_per_wg,
                                                            float4* __restrict__ part_stats,
                                                            float* __restrict__ part_val, int* __restrict__ part_idx) {
  __shared__ float cv[SCAN_WAVES][CAND_CAP];
  __shared__ int ci[SCAN_WAVES][CAND_CAP];
  __shared__ float lv[2][SCAN_WAVES][HS_MAX_TOPK];
  __shared__ int li[2][SCAN_WAVES][HS_MAX_TOPK];
  __shared__ Stats wstats[SCAN_WAVES];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x, S = gridDim.x, row = blockIdx.y;
  const float* __restrict__ x = logits + (int64_t)row * row_stride;

  // the list starts as K distinct "worse than anything" entries
  int cur = 0;
  if (lane < K) {
    lv[0][wave][lane] = -HS_INF;
    li[0][wave][lane] = INT_MAX - lane;
  }
  // statistics are kept in the log2 domain while scanning: y = (x - m) * c, c = log2(e) / T
  const float c = inv_t * LOG2E;
  float m = -HS_INF, s1 = 0.f, t2 = 0.f;
  bool first = true;
  wave_sync();

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
  // tiles this workgroup really has (uniform)
  int n_my = (V - split * tiles_per_wg * SCAN_TILE + SCAN_TILE - 1) / SCAN_TILE;
  n_my = n_my < 0 ? 0 : (n_my > tiles_per_wg ? tiles_per_wg : n_my);

  float v[SCAN_VPT], vn[SCAN_VPT];
  if (n_my > 0) load_tile(0, v);
  for (int tile = 0; tile < n_my; ++tile) {
    const int tbase = (split * tiles_per_wg + tile) * SCAN_TILE;
    if (tile + 1 < n_my) load_tile(tile + 1, vn);  // next tile's loads fly while this one is processed
#define HS_IDX(jj) (tbase + (((jj) >> 2) * SCAN_THREADS + tid) * 4 + ((jj)&3))

    // ---- softmax statistics of this thread's values
    float tm = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
    tm = fmaxf(tm, fmaxf(fmaxf(fmaxf(v[8], v[9]), fmaxf(v[10], v[11])), fmaxf(fmaxf(v[12], v[13]), fmaxf(v[14], v[15]))));
    int skip = -1;
    if (tm > m) {
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
    if (tm != -HS_INF) {
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

    // ---- threshold: the list's K-th entry, or for the first tile the K-th best of the lane maxima
    // (of the maxima of groups of four lanes when K <= 16: a quarter of the comparisons)
    float tv;
    int ti;
    if (first) {
      float bv = -HS_INF;
      int bi = INT_MAX;
#pragma unroll
      for (int jj = 0; jj < SCAN_VPT; ++jj) {
        int idx = HS_IDX(jj);
        if (better(v[jj], idx, bv, bi)) {
          bv = v[jj];
          bi = idx;
        }
      }
      int r;
      if (K <= 16) {
#pragma unroll
        for (int off = 1; off <= 2; off <<= 1) {
          const float ov = __shfl_xor(bv, off);
          const int oi = __shfl_xor(bi, off);
          if (better(ov, oi, bv, bi)) {
            bv = ov;
            bi = oi;
          }
        }
        r = 0;
#pragma unroll
        for (int l = 0; l < 64; l += 4) {
          const float ov = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bv), l));
          const int oi = __builtin_amdgcn_readlane(bi, l);
          r += better(ov, oi, bv, bi) ? 1 : 0;
        }
      } else {
        r = wave_rank(bv, bi);
      }
      unsigned long long who = __ballot(r == K - 1);
      int src = __ffsll((long long)who) - 1;  // never empty: the order is strict, ranks are a permutation
      tv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bv), src));
      ti = __builtin_amdgcn_readlane(bi, src);
      first = false;
    } else {
      tv = lv[cur][wave][K - 1];
      ti = li[cur][wave][K - 1];
    }

    // ---- compact the elements that are not worse than the threshold (skipped when no lane's
    // maximum reaches it), then re-rank list + candidates
    if (__ballot(tm >= tv) != 0ull) {
      int cnt = 0;
      const unsigned long long lt = (1ull << lane) - 1ull;
#pragma unroll
      for (int jj = 0; jj < SCAN_VPT; ++jj) {
        int idx = HS_IDX(jj);
        bool f = !better(tv, ti, v[jj], idx);
        unsigned long long mask = __ballot(f);
        if (f) {
          int pos = cnt + __popcll(mask & lt);
          cv[wave][pos] = v[jj];
          ci[wave][pos] = idx;
        }
        cnt += __popcll(mask);
      }
      if (lane < K) {
        cv[wave][cnt + lane] = lv[cur][wave][lane];
        ci[wave][cnt + lane] = li[cur][wave][lane];
      }
      wave_sync();
      rank_select(cv[wave], ci[wave], cnt + K, K, lv[cur ^ 1][wave], li[cur ^ 1][wave], lane, 64);
      cur ^= 1;
      wave_sync();
    }
#undef HS_IDX
#pragma unroll
    for (int jj = 0; jj < SCAN_VPT; ++jj) v[jj] = vn[jj];
  }
  Stats st{m, s1, t2 * 0.6931471805599453f};  // back to natural-log units
  // waves flip their list buffers independently (tiles without candidates are skipped per wave):
  // bring every wave's final list to buffer 0 before the lists are merged
  if (cur == 1 && lane < K) {
    lv[0][wave][lane] = lv[1][wave][lane];
    li[0][wave][lane] = li[1][wave][lane];
  }

  // ---- merge the four waves' lists and statistics, write this slice's partial result
  st = stats_wave_reduce(st, inv_t);
  if (lane == 0) wstats[wave] = st;
  __syncthreads();
  float* mv = &cv[1][0];  // scratch for the union of the four lists (4K <= 256 entries)
  int* mi = &ci[1][0];
  if (tid < SCAN_WAVES * K) {
    int w = tid / K, k = tid - w * K;
    mv[tid] = lv[0][w][k];
    mi[tid] = li[0][w][k];
  }
  __syncthreads();
  const int64_t pbase = ((int64_t)row * S + split) * K;
  rank_select(mv, mi, SCAN_WAVES * K, K, part_val + pbase, part_idx + pbase, tid, SCAN_THREADS);
  if (tid == 0) {
    Stats a = stats_merge(stats_merge(wstats[0], wstats[1], inv_t), stats_merge(wstats[2], wstats[3], inv_t), inv_t);
    part_stats[(int64_t)row * S + split] = make_float4(a.m, a.s1, a.t, 0.f);
  }
}

__global__ __launch_bounds__(FIN_THREADS) void k_scan_finalize(const float4* __restrict__ part_stats,
                                                               const float* __restrict__ part_val,
                                                               const int* __restrict__ part_idx, int S, int K,
                                                               float inv_t, int32_t* __restrict__ topk_idx,
                                                               float* __restrict__ topk_logp,
                                                               float* __restrict__ ent_topk,
                                                               float* __restrict__ ent_full,
                                                               float* __restrict__ lse) {
  __shared__ float cv[FIN_CAP];
  __shared__ int ci[FIN_CAP];
  __shared__ float ov[HS_MAX_TOPK];
  __shared__ int oi[HS_MAX_TOPK];
  __shared__ int cnt;
  __shared__ float thr_v;
  __shared__ int thr_i;
  __shared__ Stats total;

  const int tid = threadIdx.x, lane = tid & 63;
  const int row = blockIdx.x;
  const float* pv = part_val + (int64_t)row * S * K;
  const int* pi = part_idx + (int64_t)row * S * K;

  if (tid < 64) {
    Stats a = stats_empty();
    float hv = -HS_INF;
    int hi = INT_MAX;
    if (lane < S) {
      float4 f = part_stats[(int64_t)row * S + lane];
      a = Stats{f.x, f.y, f.z};
      hv = pv[lane * K];
      hi = pi[lane * K];
    }
    a = stats_wave_reduce(a, inv_t);
    // threshold: the K-th best list head when there are at least K lists, else "everything passes"
    float tv = -HS_INF;
    int ti = INT_MAX;
    if (S >= K) {
      int r = wave_rank(hv, hi);
      unsigned long long who = __ballot(r == K - 1 && lane < S);
      if (who != 0ull) {
        int src = __ffsll((long long)who) - 1;
        tv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, hv), src));
        ti = __builtin_amdgcn_readlane(hi, src);
      }
    }
    if (lane == 0) {
      total = a;
      thr_v = tv;
      thr_i = ti;
      cnt = 0;
    }
  }
  __syncthreads();
  {
    const float tv = thr_v;
    const int ti = thr_i;
    for (int e = tid; e < S * K; e += FIN_THREADS) {
      float v = pv[e];
      int i = pi[e];
      if (!better(tv, ti, v, i)) {
        int pos = atomicAdd(&cnt, 1);  // order of arrival does not matter: ranks are recomputed below
        if (pos < FIN_CAP) {
          cv[pos] = v;
          ci[pos] = i;
        }
      }
    }
  }
  __syncthreads();
  const int n = cnt < FIN_CAP ? cnt : FIN_CAP;
  rank_select(cv, ci, n, K, ov, oi, tid, FIN_THREADS);
  __syncthreads();

  const float m = total.m, s1 = total.s1, t = total.t;
  const float l1p = log1pf(s1);
  if (tid < K) {
    topk_idx[(int64_t)row * K + tid] = oi[tid];
    topk_logp[(int64_t)row * K + tid] = (ov[tid] - m) * inv_t - l1p;
  }
  if (tid < 64) {
    // Top-K probabilities renormalised over the K: weights relative to the best one (lane = entry);
    // entropy = ln(1 + sum w) - sum(w a) / (1 + sum w), every term of one sign
    float w = 0.f, wa = 0.f;
    if (lane >= 1 && lane < K) {
      const float a = (ov[lane] - ov[0]) * inv_t;
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
}

size_t row_topk_workspace(int R, int V, int K) {
  if (R <= 0) return 0;
  ScanPlan p = plan_scan(R, V);
  size_t n = (size_t)R * p.splits;
  return align_up(n * sizeof(float4), 256) + 2 * align_up(n * K * sizeof(float), 256);
}

hs_status row_topk_launch(const float* logits, int64_t row_stride, int R, int V, int K, float temperature,
                          int32_t* topk_idx, float* topk_logp, float* ent_topk, float* ent_full, float* lse,
                          void* workspace, hipStream_t stream) {
  ScanPlan p = plan_scan(R, V);
  Carver c(workspace);
  size_t n = (size_t)R * p.splits;
  float4* part_stats = c.take<float4>(n);
  float* part_val = c.take<float>(n * K);
  int* part_idx = c.take<int>(n * K);
  const float inv_t = 1.0f / temperature;
  const bool vec = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && (row_stride % 4 == 0);
  dim3 grid(p.splits, R);
  if (vec)
    hipLaunchKernelGGL(k_scan_rows<true>, grid, dim3(SCAN_THREADS), 0, stream, logits, row_stride, V, K, inv_t,
                       p.tiles_per_wg, part_stats, part_val, part_idx);
  else
    hipLaunchKernelGGL(k_scan_rows<false>, grid, dim3(SCAN_THREADS), 0, stream, logits, row_stride, V, K, inv_t,
                       p.tiles_per_wg, part_stats, part_val, part_idx);
  hs_status st = launch_status("row scan");
  if (st != HS_OK) return st;
  hipLaunchKernelGGL(k_scan_finalize, dim3(R), dim3(FIN_THREADS), 0, stream, part_stats, part_val, part_idx,
                     p.splits, K, inv_t, topk_idx, topk_logp, ent_topk, ent_full, lse);
  return launch_status("row scan merge");
}

}  // namespace hs

extern "C" size_t hs_draft_entropy_topk_workspace(int32_t R, int32_t V, int32_t K) {
  if (R <= 0 || V <= 0 || K <= 0 || K > HS_MAX_TOPK) return 0;
  return hs::row_topk_workspace(R, V, K);
}

extern "C" hs_status hs_draft_entropy_topk(const float* logits, int64_t row_stride, int32_t R, int32_t V, int32_t K,
                                           float temperature, int32_t* topk_idx, float* topk_logp, float* ent_topk,
                                           float* ent_full, float* lse, void* workspace, size_t workspace_bytes,
                                           hs_stream stream) {
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
                             workspace, static_cast<hipStream_t>(stream));
}
