// hs_tree_attention: tree-masked attention of the kept tree rows over the prefix KV cache
// (Section 2.2: the pruned tree is verified in one pass with tree-mask attention).
//
// This file holds the entry point, the launch planning, the float32 / any-shape kernel
// (k_attn_generic: vector ALU, K/V tiles staged through LDS, 16 rows per workgroup) and the
// split combine (k_attn_combine).  bfloat16 with head dimension 128 goes to the MFMA kernel in
// tree_attention_mfma.hip.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <functional>
#include <vector>

#include "attn_common.h"

namespace hs {

hs_status attn_mfma_launch(const AttnArgs& a, int max_tree_rows, hipStream_t stream, hipEvent_t ev_start,
                           hipEvent_t ev_stop);
bool attn_mfma_supported(int D, hs_dtype dt, int max_tree_rows, float scale);
size_t attn_mfma_table_bytes(int max_tree_rows, int64_t NN);

constexpr int GEN_THREADS = 256;
constexpr int GEN_ROWS = 16;  // rows per workgroup (4 per wave)
constexpr int GEN_TILE = 64;  // keys per tile (one per lane)
constexpr int MAX_TREE_ROWS = 1024;

template <typename T, int D>
__global__ __launch_bounds__(GEN_THREADS) void k_attn_generic(AttnArgs a) {
  __shared__ float Ks[GEN_TILE][D + 1];
  __shared__ float Vs[GEN_TILE][D];
  __shared__ float Qs[GEN_ROWS][D];
  __shared__ float Ps[GEN_THREADS / 64][4][GEN_TILE];
  __shared__ int par[MAX_TREE_ROWS];

  const int s = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = a.node_offsets[s];
  const int M = a.node_offsets[s + 1] - n0;
  const int64_t p0 = a.block_table != nullptr ? 0 : a.prefix_offsets[s];
  const int64_t L = prefix_len_of(a, s);
  if (M <= 0) return;
  const int G = a.G, Hkv = a.Hkv, Hq = a.Hq;
  const int R = G * M;
  const int n_rb = (R + GEN_ROWS - 1) / GEN_ROWS;
  const int n_sp = splits_of(L, a.split_len);
  int x = blockIdx.x;
  const int g = x % Hkv;
  x /= Hkv;
  const int rb = x % a.n_rb_max;
  const int sp = x / a.n_rb_max;
  if (rb >= n_rb || sp >= n_sp) return;

  const T* q = static_cast<const T*>(a.q);
  const bool paged = a.block_table != nullptr;  // prefix tiles are pages of GEN_TILE tokens
  const T* kp = static_cast<const T*>(a.k_prefix) + (paged ? 0 : p0) * Hkv * D;
  const T* vp = static_cast<const T*>(a.v_prefix) + (paged ? 0 : p0) * Hkv * D;
  const T* kt = static_cast<const T*>(a.k_tree) + (int64_t)n0 * Hkv * D;
  const T* vt = static_cast<const T*>(a.v_tree) + (int64_t)n0 * Hkv * D;

  for (int i = tid; i < M; i += GEN_THREADS) par[i] = a.parent[(a.tree_shared ? 0 : n0) + i];
  const int r0 = rb * GEN_ROWS;
  for (int e = tid; e < GEN_ROWS * D; e += GEN_THREADS) {
    const int rr = e / D, d = e - rr * D;
    const int r = r0 + rr;
    float v = 0.f;
    if (r < R) {
      const int i = r / G, gi = r - i * G;
      v = load_elem<T>(q + ((int64_t)(n0 + i) * Hq + g * G + gi) * D + d);
    }
    Qs[rr][d] = v;
  }

  constexpr int DPL = D / 64;  // output elements per lane
  float m_run[4], l_run[4], acc[4][DPL];
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    m_run[rr] = -HS_INF;
    l_run[rr] = 0.f;
#pragma unroll
    for (int dd = 0; dd < DPL; ++dd) acc[rr][dd] = 0.f;
  }

  const int64_t k_lo = (int64_t)sp * a.split_len;
  const int64_t k_hi = (sp == n_sp - 1) ? L : k_lo + a.split_len;
  const int n_prefix_tiles = (int)((k_hi - k_lo + GEN_TILE - 1) / GEN_TILE);
  const int n_tree_tiles = (sp == n_sp - 1) ? (M + GEN_TILE - 1) / GEN_TILE : 0;

  for (int t = 0; t < n_prefix_tiles + n_tree_tiles; ++t) {
    const bool tree = t >= n_prefix_tiles;
    const int64_t base = tree ? (int64_t)(t - n_prefix_tiles) * GEN_TILE : k_lo + (int64_t)t * GEN_TILE;
    const int64_t limit = tree ? M : k_hi;
    const T* ksrc = tree ? kt : kp;
    const T* vsrc = tree ? vt : vp;
    // where the tile's first key lives: in place, or in the page the block table names
    const int64_t where = (!tree && paged) ? (int64_t)a.block_table[(int64_t)s * a.max_blocks + base / GEN_TILE] * GEN_TILE
                                           : base;
    __syncthreads();  // previous tile fully consumed (and Qs / par written, first time)
    for (int e = tid; e < GEN_TILE * D; e += GEN_THREADS) {
      const int j = e / D, d = e - j * D;
      const int64_t key = base + j;
      float kv = 0.f, vv = 0.f;
      if (key < limit) {
        kv = load_elem<T>(ksrc + ((where + j) * Hkv + g) * D + d);
        vv = load_elem<T>(vsrc + ((where + j) * Hkv + g) * D + d);
      }
      Ks[j][d] = kv;
      Vs[j][d] = vv;
    }
    __syncthreads();

    // scores of this wave's 4 rows against the tile's 64 keys (lane = key)
    float sc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int d = 0; d < D; ++d) {
      const float kv = Ks[lane][d];
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) sc[rr] = fmaf(Qs[wave * 4 + rr][d], kv, sc[rr]);
    }
    const int64_t key = base + lane;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int r = r0 + wave * 4 + rr;
      bool ok = key < limit && r < R;
      if (ok && tree) ok = on_root_path(par, r / G, (int)key);
      const float sv = ok ? sc[rr] * a.scale : -HS_INF;
      float mx = sv;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      const float m_new = fmaxf(m_run[rr], mx);
      float pj = 0.f, alpha = 1.f;
      if (m_new != -HS_INF) {
        pj = __expf(sv - m_new);
        alpha = __expf(m_run[rr] - m_new);  // 0 when nothing was seen before
      }
      float ps = pj;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) ps += __shfl_xor(ps, off);
      l_run[rr] = l_run[rr] * alpha + ps;
      m_run[rr] = m_new;
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) acc[rr][dd] *= alpha;
      Ps[wave][rr][lane] = pj;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int j = 0; j < GEN_TILE; ++j) {
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) {
        const float vv = Vs[j][lane + 64 * dd];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) acc[rr][dd] = fmaf(Ps[wave][rr][j], vv, acc[rr][dd]);
      }
    }
  }

  // write the result (sequences with one split) or this split's partial record
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int r = r0 + wave * 4 + rr;
    if (r >= R) continue;
    const int i = r / G, gi = r - i * G;
    const int64_t row = (int64_t)(n0 + i) * Hq + g * G + gi;
    if (n_sp == 1) {
      T* out = static_cast<T*>(a.o) + row * D;
      const float inv = 1.f / l_run[rr];
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) store_elem<T>(out + lane + 64 * dd, acc[rr][dd] * inv);
      if (a.lse && lane == 0) a.lse[row] = m_run[rr] + __logf(l_run[rr]);
    } else {
      float* rec = a.part + (row * a.sp_max + sp) * (D + ATTN_REC_PAD);
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) rec[lane + 64 * dd] = acc[rr][dd];
      if (lane == 0) {
        rec[D] = m_run[rr];
        rec[D + 1] = l_run[rr];
      }
    }
  }
}

// Merges the splits of one (node, head) row: weights exp(m_sp - max m), splits taken in rising
// order.  One wave per row, lane l owns D / 64 adjacent output elements
constexpr int CMB_ROWS = 4;  // rows (waves) per workgroup
template <typename T, int D>
__global__ __launch_bounds__(64 * CMB_ROWS) void k_attn_combine(AttnArgs a, int64_t n_rows) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * CMB_ROWS + (threadIdx.x >> 6);  // node_global * Hq + h
  if (row >= n_rows) return;
  const int node = (int)(row / a.Hq);
  int n_sp;
  if (a.n_tbl > 0) {
    // the table entry whose row range holds this node
    n_sp = 1;
    for (int base = 0; base < a.n_tbl; base += 64) {
      const int idx = base + lane;
      bool mine = false;
      int cnt = 0;
      if (idx < a.n_tbl) {
        mine = node >= a.tbl[idx].n0 && node < a.tbl[idx].n0 + a.tbl[idx].M;
        cnt = a.tbl[idx].n_sp;
      }
      const unsigned long long hit = __ballot(mine);
      if (hit != 0ull) {
        n_sp = __builtin_amdgcn_readlane(cnt, __builtin_ctzll(hit));
        break;
      }
    }
  } else {
    // sequence of this node: last s with node_offsets[s] <= node
    int lo = 0, hi = a.B;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (a.node_offsets[mid] <= node) lo = mid; else hi = mid;
    }
    n_sp = splits_of(prefix_len_of(a, lo), a.split_len);
  }
  if (n_sp == 1) return;  // written directly by the attention kernel
  constexpr int REC = D + ATTN_REC_PAD;
  const float* rec = a.part + row * a.sp_max * REC;
  // lane sp holds split sp's reference maximum and denominator (at most 64 splits): one trip to memory
  // for all of them, then the splits' rows four at a time
  float mv = -HS_INF, lv = 0.f;
  if (lane < n_sp) {
    mv = rec[lane * REC + D];
    lv = rec[lane * REC + D + 1];
  }
  const float m = wave_max(mv);
  const float w = lane < n_sp ? __expf(mv - m) : 0.f;
  const float l = wave_sum(lv * w);
  constexpr int DPL = D / 64;
  float o[DPL];
#pragma unroll
  for (int dd = 0; dd < DPL; ++dd) o[dd] = 0.f;
  for (int sp0 = 0; sp0 < n_sp; sp0 += 4) {
    float v[4][DPL];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) v[u][dd] = sp0 + u < n_sp ? rec[(sp0 + u) * REC + lane * DPL + dd] : 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float wu = __shfl(w, (sp0 + u) & 63);  // (0 beyond the last split)
#pragma unroll
      for (int dd = 0; dd < DPL; ++dd) o[dd] = fmaf(v[u][dd], wu, o[dd]);
    }
  }
  const float inv = 1.f / l;
#pragma unroll
  for (int dd = 0; dd < DPL; ++dd) store_elem<T>(static_cast<T*>(a.o) + row * D + lane * DPL + dd, o[dd] * inv);
  if (a.lse && lane == 0) a.lse[row] = m + __logf(l);
}

struct AttnPlan {
  int split_len, sp_max, n_rb_max, max_rows;
  int64_t max_L;
  bool ok;
};

// Chooses the split length from the host copies of the offsets: enough workgroups to fill the
// chip, but splits long enough that partial records stay small next to the K/V they summarise.
static AttnPlan plan_attention(const int32_t* hno, const int64_t* hpo, const int64_t* hlens, int B, int Hq, int Hkv,
                               int rows_per_wg, int target_wgs) {
  AttnPlan p{};
  int max_M = 0;
  int64_t max_L = 0, sum_L = 0;
  for (int s = 0; s < B; ++s) {
    const int M = hno[s + 1] - hno[s];
    const int64_t L = hlens != nullptr ? hlens[s] : hpo[s + 1] - hpo[s];
    if (M > max_M) max_M = M;
    if (M > 0) {
      if (L > max_L) max_L = L;
      sum_L += L;
    }
  }
  p.max_rows = max_M;
  p.max_L = max_L;
  const int G = Hq / Hkv;
  p.n_rb_max = rows_per_wg > 0 ? (G * max_M + rows_per_wg - 1) / rows_per_wg : 1;
  if (p.n_rb_max < 1) p.n_rb_max = 1;
  // workgroups without splitting: one per (sequence, head, row block); split until the target is met
  const int64_t base_wgs = (int64_t)B * Hkv * p.n_rb_max;
  int64_t want = base_wgs > 0 ? (target_wgs + base_wgs - 1) / base_wgs : 1;  // splits per average sequence
  if (want < 1) want = 1;
  const int64_t mean_L = B > 0 ? sum_L / B : 0;
  int64_t len = (mean_L + want - 1) / want;
  len = (len + 255) / 256 * 256;   // multiple of 256 tokens
  if (len < 512) len = 512;        // never split finer than 512 tokens
  p.split_len = (int)len;
  p.sp_max = splits_of(max_L, p.split_len);
  p.ok = true;
  return p;
}

// ---- work-list plan for the matrix-core kernel.
// Every (sequence, split, row group, KV head) is one work item = one workgroup.  The hardware
// starts workgroups in index order as compute units free up, so listing the items by falling cost
// is longest-processing-time-first scheduling.  The cost model (microseconds, fitted to
// measurements on MI355X) only has to rank alternatives: an item costs a fixed part plus a
// per-tile part that grows with the number of waves that have rows.
constexpr int PLAN_CUS = 256;
constexpr float PLAN_ITEM_US = 10.f;
// Splits of at least 128 tokens (the workspace bound relies on it).  A launch of few workgroups is mostly an
// item's fixed cost: one layer of the 8B shape (32 tiles a head) takes 25.9 us cut into 4 x 8 tiles, 23.5 us
// into 8 x 4 or 16 x 2, combine launch included.
constexpr int PLAN_MIN_SPLIT_TILES = 2;
constexpr int PLAN_MIN_SPLIT_TOKENS = PLAN_MIN_SPLIT_TILES * 64;
static inline float plan_tile_us(int waves) { return 1.25f + 0.04f * (float)waves; }

struct ListPlan {
  float est_us;
  int target;
};

// Splits of a sequence of `tiles` prefix tiles when items should hold about `target` tiles.
static inline int plan_splits(int tiles, int target, int sp_cap, bool paged = false) {
  int n = (tiles + target / 2) / target;
  const int most = tiles / PLAN_MIN_SPLIT_TILES;
  if (n > most) n = most;
  if (n > sp_cap) n = sp_cap;
  if (paged && n < (tiles + 255) / 256) n = (tiles + 255) / 256;  // the kernel holds the pages of 256 tiles
  return n < 1 ? 1 : n;
}

// The cut itself: `per` tiles to a split, and as many splits as that takes (rounding `per` up can make
// the last of the splits asked for empty: they are dropped, every split starts inside the prefix).
static inline void plan_cut(int tiles, int target, int sp_cap, bool paged, int* nsp, int* per) {
  int n = plan_splits(tiles, target, sp_cap, paged);
  int p = (tiles + n - 1) / n;
  if (p < 1) p = 1;
  n = (tiles + p - 1) / p;
  *nsp = n < 1 ? 1 : n;
  *per = p;
}

// Fills a.tbl / a.n_tbl / a.n_items / a.sp_max.  Returns false when the batch does not fit the table.
static bool plan_worklist(AttnArgs& a, const int32_t* hno, const int64_t* hpo, const int64_t* hlens, int B,
                          int sp_cap) {
  struct Seq {
    int s, M, tiles, rg, waves0, waves_last, ttiles;
  };
  Seq seqs[ATTN_TBL];
  int n = 0;
  for (int s = 0; s < B; ++s) {
    const int M = hno[s + 1] - hno[s];
    const int64_t L = hlens != nullptr ? hlens[s] : hpo[s + 1] - hpo[s];
    if (M <= 0) continue;
    if (n == ATTN_TBL || L >= (int64_t)1 << 30) return false;
    const int blocks = (a.G * M + 31) / 32;  // 32-row wave blocks
    Seq q;
    q.s = s;
    q.M = M;
    q.tiles = (int)((L + 63) / 64);
    q.rg = (blocks + 7) / 8;
    q.waves0 = blocks < 8 ? blocks : 8;
    q.waves_last = blocks - 8 * (q.rg - 1);
    q.ttiles = (M + 63) / 64;
    seqs[n++] = q;
  }
  if (n == 0) return false;
  // Unequal items (a ragged batch): the makespan of each candidate is found by replaying the
  // hardware's dispatch, which hands the next workgroup in index order to the first compute unit
  // that falls free (list scheduling).  Equal items (the layers of one step) run in whole rounds.
  static const int targets[] = {1 << 20, 192, 160, 128, 112, 96, 80, 72, 64, 56, 48, 40, 32, 24, 16, 8, 4, 2};
  // Cuts finer than eight tiles are candidates only while eight-tile items would leave compute units idle
  // (a launch of one or two layers): such an item is mostly its fixed cost.
  int64_t coarse_items = 0;
  for (int i = 0; i < n; ++i) coarse_items += (int64_t)a.Hkv * seqs[i].rg * (seqs[i].tiles / 8 > 0 ? seqs[i].tiles / 8 : 1);
  const int n_targets = (int)(sizeof(targets) / sizeof(targets[0])) - (coarse_items < PLAN_CUS ? 0 : 2);
  ListPlan best{0.f, 0};
  static thread_local std::vector<float> item_cost, cu_free;  // (kept between calls: no allocation in the steady state)
  for (int ti = 0; ti < n_targets; ++ti) {
    const int target = targets[ti];
    double total = 0.0, rec_bytes = 0.0;
    float mx = 0.f, mn = 1e30f;
    int64_t items = 0;
    int ord[ATTN_TBL];
    float seq_cost[ATTN_TBL];
    for (int i = 0; i < n; ++i) {
      const Seq& q = seqs[i];
      int nsp, per;
      plan_cut(q.tiles, target, sp_cap, a.block_table != nullptr, &nsp, &per);
      const float big = PLAN_ITEM_US + (float)(per + q.ttiles) * plan_tile_us(q.waves0);
      const float one = PLAN_ITEM_US + (float)per * plan_tile_us(q.waves0);
      const float one_last = PLAN_ITEM_US + (float)per * plan_tile_us(q.waves_last);
      total += (double)a.Hkv * nsp * ((q.rg - 1) * one + one_last);
      items += (int64_t)a.Hkv * nsp * q.rg;
      if (big > mx) mx = big;
      if (one_last < mn) mn = one_last;
      if (nsp > 1) rec_bytes += (double)q.M * a.Hq * nsp * ((a.half ? 64 : 128) + ATTN_REC_PAD) * 4 * 2;  // written, then read
      ord[i] = i;
      seq_cost[i] = (float)per * plan_tile_us(q.waves0);
    }
    // (no schedule ends before the work divided by the compute units, nor before its longest item: a
    // candidate whose bound is no better than the best estimate so far needs no replay)
    const float combine_us = rec_bytes > 0.0 ? 4.f + (float)(rec_bytes / 2.5e6) : 0.f;  // the combine launch, ~2.5 TB/s
    {
      const float floor_us = (float)(total / PLAN_CUS) > mx ? (float)(total / PLAN_CUS) : mx;
      if (best.target != 0 && floor_us + combine_us >= best.est_us) continue;
    }
    float est;
    if (mx - mn <= 0.1f * mx || items > 8192) {
      est = (float)(total / PLAN_CUS) + 0.15f * mx;
      if (mx > est) est = mx;
      if (mx - mn <= 0.1f * mx) {  // equal items run in whole rounds
        const float rounds = (float)((items + PLAN_CUS - 1) / PLAN_CUS) * (float)(total / (double)items);
        if (rounds > est) est = rounds;
      }
    } else {
      // the items in dispatch order (as the table below lists them), then the replay
      std::stable_sort(ord, ord + n, [&](int x, int y) { return seq_cost[x] > seq_cost[y]; });
      item_cost.clear();
      for (int k = 0; k < n; ++k) {
        const Seq& q = seqs[ord[k]];
        int nsp, per;
        plan_cut(q.tiles, target, sp_cap, a.block_table != nullptr, &nsp, &per);
        for (int sp = 0; sp < nsp; ++sp) {
          int t = q.tiles - sp * per;
          t = t > per ? per : (t < 0 ? 0 : t);
          if (sp == nsp - 1) t += q.ttiles;
          for (int rg = 0; rg < q.rg; ++rg) {
            const float c = PLAN_ITEM_US + (float)t * plan_tile_us(rg == q.rg - 1 ? q.waves_last : q.waves0);
            for (int h = 0; h < a.Hkv; ++h) item_cost.push_back(c);
          }
        }
      }
      cu_free.assign(PLAN_CUS, 0.f);
      std::make_heap(cu_free.begin(), cu_free.end(), std::greater<float>());
      float end = 0.f;
      for (float c : item_cost) {
        std::pop_heap(cu_free.begin(), cu_free.end(), std::greater<float>());
        const float done = cu_free.back() + c;
        cu_free.back() = done;
        std::push_heap(cu_free.begin(), cu_free.end(), std::greater<float>());
        if (done > end) end = done;
      }
      est = end;
    }
    est += combine_us;
    if (best.target == 0 || est < best.est_us) best = ListPlan{est, target};
  }
  // the table: sequences by falling cost of an item
  int order[ATTN_TBL];
  float cost[ATTN_TBL];
  int nsp_of[ATTN_TBL], per_of[ATTN_TBL];
  for (int i = 0; i < n; ++i) {
    const Seq& q = seqs[i];
    plan_cut(q.tiles, best.target, sp_cap, a.block_table != nullptr, &nsp_of[i], &per_of[i]);
    cost[i] = (float)per_of[i] * plan_tile_us(q.waves0);
    order[i] = i;
  }
  std::stable_sort(order, order + n, [&](int x, int y) { return cost[x] > cost[y]; });
  int64_t first = 0;
  int sp_max = 1;
  for (int k = 0; k < n; ++k) {
    const int i = order[k];
    const Seq& q = seqs[i];
    SeqEntry& e = a.tbl[k];
    e.first_item = (int)first;
    e.n0 = hno[q.s];
    e.M = q.M;
    e.L = (int)(hlens != nullptr ? hlens[q.s] : hpo[q.s + 1] - hpo[q.s]);
    e.p0 = a.block_table != nullptr ? (long long)q.s * a.max_blocks : hpo[q.s];
    e.tiles_per_split = per_of[i];
    e.n_sp = (short)nsp_of[i];
    e.n_rg = (short)q.rg;
    first += (int64_t)a.Hkv * nsp_of[i] * q.rg;
    if (nsp_of[i] > sp_max) sp_max = nsp_of[i];
    if (first >= (int64_t)1 << 30) return false;
  }
  a.n_tbl = n;
  a.n_items = (int)first;
  a.sp_max = sp_max;
  return true;
}

// The plan depends on the host arrays and the head layout alone, and a model calls the attention of all its
// layers with the same ones: the last few plans are kept per thread.  (Planning a ragged batch of 16 sequences
// replays some twenty candidate cuts over hundreds of items each, a few hundred microseconds on the host:
// more than the launch itself takes on the GPU.)
struct PlanMemo {
  std::vector<int64_t> key;  // everything the plan is a function of; empty: unused slot
  bool ok;
  int n_tbl, n_items, sp_max;
  SeqEntry tbl[ATTN_TBL];
};
constexpr int PLAN_MEMO_SLOTS = 4;
constexpr int PLAN_MEMO_MAX_B = 1024;  // larger batches (at most 96 of their entries non-empty) are planned every time

static bool plan_worklist_memo(AttnArgs& a, const int32_t* hno, const int64_t* hpo, const int64_t* hlens, int B,
                               int sp_cap) {
  if (B > PLAN_MEMO_MAX_B) return plan_worklist(a, hno, hpo, hlens, B, sp_cap);
  static thread_local PlanMemo memo[PLAN_MEMO_SLOTS];
  static thread_local unsigned next_slot = 0;
  static thread_local std::vector<int64_t> key;
  key.clear();
  key.push_back(B);
  key.push_back(sp_cap);
  key.push_back(a.G);
  key.push_back(a.Hkv);
  key.push_back(a.half);
  key.push_back(a.block_table != nullptr ? 1 + (int64_t)a.max_blocks : 0);  // (paged: an entry's p0 is s * max_blocks)
  key.push_back((hpo != nullptr ? 1 : 0) + (hlens != nullptr ? 2 : 0));
  for (int s = 0; s <= B; ++s) key.push_back(hno[s]);
  if (hpo != nullptr)
    for (int s = 0; s <= B; ++s) key.push_back(hpo[s]);
  if (hlens != nullptr)
    for (int s = 0; s < B; ++s) key.push_back(hlens[s]);
  for (PlanMemo& m : memo)
    if (m.key == key) {
      if (m.ok) {
        a.n_tbl = m.n_tbl;
        a.n_items = m.n_items;
        a.sp_max = m.sp_max;
        memcpy(a.tbl, m.tbl, sizeof(SeqEntry) * (size_t)m.n_tbl);
      }
      return m.ok;
    }
  PlanMemo& m = memo[next_slot++ % PLAN_MEMO_SLOTS];
  m.ok = plan_worklist(a, hno, hpo, hlens, B, sp_cap);
  m.key = key;
  if (m.ok) {
    m.n_tbl = a.n_tbl;
    m.n_items = a.n_items;
    m.sp_max = a.sp_max;
    memcpy(m.tbl, a.tbl, sizeof(SeqEntry) * (size_t)a.n_tbl);
  }
  return m.ok;
}

}  // namespace hs

using namespace hs;

static size_t part_bytes(int64_t NN, int Hq, int D, int sp_max) {
  if (sp_max <= 1) return 0;
  return align_up((size_t)NN * Hq * sp_max * (D + ATTN_REC_PAD) * sizeof(float), 256);
}

extern "C" size_t hs_tree_attention_workspace(int32_t B, int32_t NN, int64_t total_prefix, int32_t Hq, int32_t Hkv,
                                              int32_t D, hs_dtype dt) {
  (void)dt;
  if (B <= 0 || NN <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || total_prefix < 0) return 0;
  // upper bound over every plan the launch may choose: splits are at least PLAN_MIN_SPLIT_TOKENS long
  const int64_t sp_bound = total_prefix / PLAN_MIN_SPLIT_TOKENS + 1;
  // (+ the ancestor table that trees of more than 256 rows keep there: such a tree needs NN > 256)
  return part_bytes(NN, Hq, D, (int)(sp_bound < 2 ? 2 : sp_bound > 64 ? 64 : sp_bound)) +
         align_up(attn_mfma_table_bytes(NN < MAX_TREE_ROWS ? NN : MAX_TREE_ROWS, NN), 256);
}

extern "C" hs_status hs_tree_attention(const void* q, const void* k_prefix, const void* v_prefix, const void* k_tree,
                                       const void* v_tree, const int32_t* parent, const int32_t* node_offsets,
                                       const int64_t* prefix_offsets, const int32_t* host_node_offsets,
                                       const int64_t* host_prefix_offsets, int32_t B, int32_t Hq, int32_t Hkv,
                                       int32_t D, hs_dtype dt, float scale, void* o, float* lse, void* workspace,
                                       size_t workspace_bytes, hs_stream stream) {
  return hs_tree_attention_lens(q, k_prefix, v_prefix, k_tree, v_tree, parent, node_offsets, prefix_offsets,
                                host_node_offsets, host_prefix_offsets, nullptr, nullptr, B, Hq, Hkv, D, dt, scale, o,
                                lse, workspace, workspace_bytes, stream);
}

// Events that hs_time_next_attention left for this thread's next attention call.
static thread_local hipEvent_t timing_start = nullptr, timing_stop = nullptr;
// Kernel that this thread's last attention call launched (hs_tree_attention_last_kernel).
static thread_local int last_kernel = 0;

extern "C" int32_t hs_tree_attention_last_kernel(void) { return last_kernel; }

extern "C" hs_status hs_time_next_attention(void* start_event, void* stop_event) {
  clear_error();
  HS_REQUIRE((start_event == nullptr) == (stop_event == nullptr), HS_ERR_NULL,
             "hs_time_next_attention: give both events or neither");
  timing_start = static_cast<hipEvent_t>(start_event);
  timing_stop = static_cast<hipEvent_t>(stop_event);
  return HS_OK;
}

// What hs_tree_attention_plan reports (host memory; per_seq may be NULL).
struct PlanReport {
  int64_t* totals;   // [6]
  int32_t* per_seq;  // [B][4]
};

// The three entry points in one: dense prefix regions (prefix_lens NULL), regions with spare
// capacity (prefix_lens given), pages (block_table given: k_prefix / v_prefix are the page pools,
// the offset arrays are absent).
static hs_status attention_impl(const void* q, const void* k_prefix, const void* v_prefix, const void* k_tree,
                                const void* v_tree, const int32_t* parent, const int32_t* node_offsets,
                                const int64_t* prefix_offsets, const int32_t* host_node_offsets,
                                const int64_t* host_prefix_offsets, const int64_t* prefix_lens,
                                const int64_t* host_prefix_lens, const int32_t* block_table, int32_t max_blocks,
                                int32_t B, int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt, float scale, void* o,
                                float* lse, void* workspace, size_t workspace_bytes, hs_stream stream,
                                bool tree_shared = false, const PlanReport* report = nullptr) {
  // report != NULL: plan only.  The host arrays are read and checked as in a real call, the device
  // pointers may be NULL, nothing is launched; the report says how the launch would be cut.
  const bool plan_only = report != nullptr;
  if (plan_only)
    for (int k = 0; k < 6; ++k) report->totals[k] = 0;
  const bool paged = block_table != nullptr;
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;
  if (!plan_only) {
    ev_start = timing_start;  // one-shot, whatever this call comes to
    ev_stop = timing_stop;
    timing_start = timing_stop = nullptr;
    last_kernel = 0;
  }
  HS_REQUIRE(B >= 0, HS_ERR_SHAPE, "hs_tree_attention: B=%d", B);
  HS_REQUIRE(Hq >= 1 && Hkv >= 1 && Hq % Hkv == 0, HS_ERR_SHAPE, "hs_tree_attention: Hq=%d must be a multiple of Hkv=%d",
             Hq, Hkv);
  HS_REQUIRE(D == 64 || D == 128, HS_ERR_UNSUPPORTED, "hs_tree_attention: head dimension %d (64 and 128 are built)", D);
  HS_REQUIRE(dt == HS_F32 || dt == HS_BF16, HS_ERR_SHAPE, "hs_tree_attention: unknown dtype %d", (int)dt);
  if (B == 0) return HS_OK;
  HS_REQUIRE(host_node_offsets && (paged || host_prefix_offsets) &&
                 (plan_only || (node_offsets && (paged || prefix_offsets))),
             HS_ERR_NULL, "hs_tree_attention: offset arrays (device and host copies) are required");
  HS_REQUIRE(host_node_offsets[0] == 0 && (paged || host_prefix_offsets[0] == 0), HS_ERR_SHAPE,
             "hs_tree_attention: offsets must start at 0");
  HS_REQUIRE(!paged || ((plan_only || prefix_lens) && host_prefix_lens && max_blocks >= 0), HS_ERR_NULL,
             "hs_tree_attention_paged: prefix lengths (device and host) are required");
  int64_t total_used = 0;
  for (int s = 0; s < B; ++s) {
    const int M = host_node_offsets[s + 1] - host_node_offsets[s];
    if (paged) {
      HS_REQUIRE(M >= 0, HS_ERR_SHAPE, "hs_tree_attention: offsets decrease at sequence %d", s);
      HS_REQUIRE(host_prefix_lens[s] >= 0 && host_prefix_lens[s] <= (int64_t)max_blocks * 64, HS_ERR_SHAPE,
                 "hs_tree_attention_paged: prefix length of sequence %d exceeds its %d blocks", s, max_blocks);
      // (a key split holds the pages of at most 256 tiles, a sequence has at most 64 splits)
      HS_REQUIRE(host_prefix_lens[s] <= (int64_t)64 * 256 * 64, HS_ERR_UNSUPPORTED,
                 "hs_tree_attention_paged: prefix of sequence %d is longer than %d tokens", s, 64 * 256 * 64);
      total_used += host_prefix_lens[s];
      HS_REQUIRE(M <= MAX_TREE_ROWS, HS_ERR_UNSUPPORTED, "hs_tree_attention: sequence %d has %d tree rows (limit %d)",
                 s, M, MAX_TREE_ROWS);
      continue;
    }
    HS_REQUIRE(M >= 0 && host_prefix_offsets[s + 1] >= host_prefix_offsets[s], HS_ERR_SHAPE,
               "hs_tree_attention: offsets decrease at sequence %d", s);
    HS_REQUIRE(M <= MAX_TREE_ROWS, HS_ERR_UNSUPPORTED, "hs_tree_attention: sequence %d has %d tree rows (limit %d)", s,
               M, MAX_TREE_ROWS);
    HS_REQUIRE(host_prefix_lens == nullptr ||
                   (host_prefix_lens[s] >= 0 && host_prefix_lens[s] <= host_prefix_offsets[s + 1] - host_prefix_offsets[s]),
               HS_ERR_SHAPE, "hs_tree_attention: prefix length of sequence %d exceeds its region", s);
  }
  HS_REQUIRE(plan_only || (prefix_lens == nullptr) == (host_prefix_lens == nullptr), HS_ERR_NULL,
             "hs_tree_attention: prefix_lens and host_prefix_lens go together");
  const int NN = host_node_offsets[B];
  const int64_t total_prefix = paged ? total_used : host_prefix_offsets[B];
  if (NN == 0) return HS_OK;
  HS_REQUIRE(plan_only || (q && k_tree && v_tree && parent && o), HS_ERR_NULL, "hs_tree_attention: NULL tensor");
  HS_REQUIRE(plan_only || total_prefix == 0 || (k_prefix && v_prefix), HS_ERR_NULL, "hs_tree_attention: NULL prefix cache");

  int max_M = 0;
  for (int s = 0; s < B; ++s) max_M = std::max(max_M, host_node_offsets[s + 1] - host_node_offsets[s]);
  auto aligned16 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  // (head-count limits: the matrix-core kernel numbers rows and lane offsets in narrow types)
  // D = 64: the matrix-core kernel takes the KV heads in pairs (their number must be even); a pair
  // then has twice the query heads
  const bool pairs = D == 64;
  const int kv_units = pairs ? Hkv / 2 : Hkv, g_unit = pairs ? 2 * (Hq / Hkv) : Hq / Hkv;
  const bool mfma = attn_mfma_supported(D, dt, max_M, scale) && (!pairs || Hkv % 2 == 0) && g_unit <= 128 &&
                    (int64_t)g_unit * max_M < 65536 && Hkv <= 4096 && aligned16(q) &&
                    aligned16(k_prefix) && aligned16(v_prefix) && aligned16(k_tree) && aligned16(v_tree) &&
                    aligned16(o);
  AttnArgs a;
  a.q = q; a.k_prefix = k_prefix; a.v_prefix = v_prefix; a.k_tree = k_tree; a.v_tree = v_tree;
  a.parent = parent; a.tree_shared = tree_shared ? 1 : 0; a.node_offsets = node_offsets; a.prefix_offsets = prefix_offsets; a.prefix_lens = prefix_lens;
  a.block_table = block_table; a.max_blocks = max_blocks;
  a.B = B; a.Hq = Hq; a.Hkv = mfma ? kv_units : Hkv; a.G = mfma ? g_unit : Hq / Hkv; a.half = mfma && pairs ? 1 : 0; a.scale = scale;
  a.o = o; a.lse = lse; a.part = static_cast<float*>(workspace);
  a.n_tbl = 0; a.n_items = 0; a.anc_tiles = nullptr;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the workspace query bounds the splits of a sequence the same way
  const int64_t sp_bound = total_prefix / PLAN_MIN_SPLIT_TOKENS + 1;
  const int sp_cap = (int)(sp_bound < 2 ? 2 : sp_bound > 64 ? 64 : sp_bound);

  AttnPlan plan{};
  if (!(mfma && plan_worklist_memo(a, host_node_offsets, host_prefix_offsets, host_prefix_lens, B, sp_cap))) {
    a.n_tbl = 0;
    plan = plan_attention(host_node_offsets, host_prefix_offsets, host_prefix_lens, B, Hq, a.Hkv, mfma ? 0 : GEN_ROWS, mfma ? 256 : 1024);
    while (plan.sp_max > sp_cap) {
      plan.split_len *= 2;
      plan.sp_max = splits_of(plan.max_L, plan.split_len);
    }
    if (paged && plan.split_len > 256 * 64) {  // the matrix-core kernel holds the pages of 256 tiles per split
      plan.split_len = 256 * 64;
      plan.sp_max = splits_of(plan.max_L, plan.split_len);
    }
    a.split_len = plan.split_len; a.sp_max = plan.sp_max; a.n_rb_max = plan.n_rb_max;
  } else {
    a.split_len = 0; a.n_rb_max = 1;
  }
  const size_t table_bytes = mfma ? align_up(attn_mfma_table_bytes(max_M, NN), 256) : 0;
  const size_t need = part_bytes(NN, Hq, D, a.sp_max) + table_bytes;
  if (table_bytes != 0 && workspace != nullptr)
    a.anc_tiles = reinterpret_cast<const unsigned*>(static_cast<const char*>(workspace) + part_bytes(NN, Hq, D, a.sp_max));
  if (plan_only) {
    const int n_rg_max = mfma ? (a.G * max_M + 255) / 256 : plan.n_rb_max;
    report->totals[0] = mfma ? 1 : 2;
    report->totals[1] = a.n_tbl > 0 ? a.n_items : (int64_t)a.Hkv * n_rg_max * a.sp_max * B;
    report->totals[2] = a.sp_max;
    report->totals[3] = a.split_len;
    report->totals[4] = (int64_t)need;
    report->totals[5] = a.sp_max > 1 ? 1 : 0;
    if (report->per_seq != nullptr) {
      for (int s = 0; s < B; ++s) {
        int32_t* r = report->per_seq + 4 * s;
        const int M = host_node_offsets[s + 1] - host_node_offsets[s];
        const int64_t L = host_prefix_lens != nullptr ? host_prefix_lens[s] : host_prefix_offsets[s + 1] - host_prefix_offsets[s];
        r[0] = M > 0 ? splits_of(L, a.split_len > 0 ? a.split_len : 1 << 30) : 0;
        r[1] = a.split_len / 64;
        r[2] = M > 0 ? (mfma ? (a.G * M + 255) / 256 : (a.G * M + GEN_ROWS - 1) / GEN_ROWS) : 0;
        r[3] = -1;
      }
      for (int k = 0; k < a.n_tbl; ++k) {  // work lists: the table's entries, found back by their first tree row
        const SeqEntry& e = a.tbl[k];
        for (int s = 0; s < B; ++s)
          if (host_node_offsets[s] == e.n0 && host_node_offsets[s + 1] - e.n0 == e.M && report->per_seq[4 * s + 3] < 0) {
            int32_t* r = report->per_seq + 4 * s;
            r[0] = e.n_sp; r[1] = e.tiles_per_split; r[2] = e.n_rg; r[3] = e.first_item;
            break;
          }
      }
    }
    return HS_OK;
  }
  HS_REQUIRE(need == 0 || (workspace && workspace_bytes >= need && reinterpret_cast<uintptr_t>(workspace) % 256 == 0),
             HS_ERR_WORKSPACE, "hs_tree_attention: workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
             workspace_bytes);

  if (mfma) {
    hs_status r = attn_mfma_launch(a, max_M, st, ev_start, ev_stop);
    if (r != HS_OK) return r;
    last_kernel = 1;
  } else {
    dim3 grid((unsigned)(Hkv * plan.n_rb_max * plan.sp_max), (unsigned)B);
    if (dt == HS_F32 && D == 64) hipLaunchKernelGGL((k_attn_generic<float, 64>), grid, dim3(GEN_THREADS), 0, st, a);
    else if (dt == HS_F32) hipLaunchKernelGGL((k_attn_generic<float, 128>), grid, dim3(GEN_THREADS), 0, st, a);
    else if (D == 64) hipLaunchKernelGGL((k_attn_generic<bf16_t, 64>), grid, dim3(GEN_THREADS), 0, st, a);
    else hipLaunchKernelGGL((k_attn_generic<bf16_t, 128>), grid, dim3(GEN_THREADS), 0, st, a);
    hs_status r = launch_status("tree attention");
    if (r != HS_OK) return r;
    last_kernel = 2;
  }
  if (a.sp_max > 1) {
    const int64_t n_rows = (int64_t)NN * Hq;
    dim3 grid((unsigned)((n_rows + CMB_ROWS - 1) / CMB_ROWS)), block(64 * CMB_ROWS);
    if (dt == HS_F32 && D == 64) hipLaunchKernelGGL((k_attn_combine<float, 64>), grid, block, 0, st, a, n_rows);
    else if (dt == HS_F32) hipLaunchKernelGGL((k_attn_combine<float, 128>), grid, block, 0, st, a, n_rows);
    else if (D == 64) hipLaunchKernelGGL((k_attn_combine<bf16_t, 64>), grid, block, 0, st, a, n_rows);
    else hipLaunchKernelGGL((k_attn_combine<bf16_t, 128>), grid, block, 0, st, a, n_rows);
    return launch_status("tree attention combine");
  }
  return HS_OK;
}

extern "C" hs_status hs_tree_attention_lens(const void* q, const void* k_prefix, const void* v_prefix,
                                            const void* k_tree, const void* v_tree, const int32_t* parent,
                                            const int32_t* node_offsets, const int64_t* prefix_offsets,
                                            const int32_t* host_node_offsets, const int64_t* host_prefix_offsets,
                                            const int64_t* prefix_lens, const int64_t* host_prefix_lens, int32_t B,
                                            int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt, float scale, void* o,
                                            float* lse, void* workspace, size_t workspace_bytes, hs_stream stream) {
  clear_error();
  return attention_impl(q, k_prefix, v_prefix, k_tree, v_tree, parent, node_offsets, prefix_offsets, host_node_offsets,
                        host_prefix_offsets, prefix_lens, host_prefix_lens, nullptr, 0, B, Hq, Hkv, D, dt, scale, o, lse,
                        workspace, workspace_bytes, stream);
}

extern "C" hs_status hs_tree_attention_shared_tree(const void* q, const void* k_prefix, const void* v_prefix,
                                                   const void* k_tree, const void* v_tree, const int32_t* parent,
                                                   const int32_t* node_offsets, const int64_t* prefix_offsets,
                                                   const int32_t* host_node_offsets,
                                                   const int64_t* host_prefix_offsets, int32_t B, int32_t Hq,
                                                   int32_t Hkv, int32_t D, hs_dtype dt, float scale, void* o, float* lse,
                                                   void* workspace, size_t workspace_bytes, hs_stream stream) {
  clear_error();
  if (B > 0 && host_node_offsets != nullptr) {
    const int M = host_node_offsets[1] - host_node_offsets[0];
    for (int s = 1; s < B; ++s)
      HS_REQUIRE(host_node_offsets[s + 1] - host_node_offsets[s] == M, HS_ERR_SHAPE,
                 "hs_tree_attention_shared_tree: entry %d has %d rows, entry 0 has %d", s,
                 host_node_offsets[s + 1] - host_node_offsets[s], M);
  }
  return attention_impl(q, k_prefix, v_prefix, k_tree, v_tree, parent, node_offsets, prefix_offsets, host_node_offsets,
                        host_prefix_offsets, nullptr, nullptr, nullptr, 0, B, Hq, Hkv, D, dt, scale, o, lse, workspace,
                        workspace_bytes, stream, true);
}

extern "C" hs_status hs_tree_attention_paged(const void* q, const void* k_pages, const void* v_pages,
                                             const void* k_tree, const void* v_tree, const int32_t* parent,
                                             const int32_t* node_offsets, const int32_t* host_node_offsets,
                                             const int32_t* block_table, int32_t max_blocks, int32_t page_tokens,
                                             const int64_t* prefix_lens, const int64_t* host_prefix_lens, int32_t B,
                                             int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt, float scale, void* o,
                                             float* lse, void* workspace, size_t workspace_bytes, hs_stream stream) {
  clear_error();
  HS_REQUIRE(page_tokens == 64, HS_ERR_UNSUPPORTED, "hs_tree_attention_paged: page_tokens=%d (pages of 64 tokens are built)",
             page_tokens);
  HS_REQUIRE(B == 0 || block_table, HS_ERR_NULL, "hs_tree_attention_paged: NULL block_table");
  return attention_impl(q, k_pages, v_pages, k_tree, v_tree, parent, node_offsets, nullptr, host_node_offsets, nullptr,
                        prefix_lens, host_prefix_lens, block_table, max_blocks, B, Hq, Hkv, D, dt, scale, o, lse,
                        workspace, workspace_bytes, stream);
}

extern "C" hs_status hs_tree_attention_plan(const int32_t* host_node_offsets, const int64_t* host_prefix_offsets,
                                            const int64_t* host_prefix_lens, int32_t paged, int32_t max_blocks,
                                            int32_t B, int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt,
                                            int64_t* totals, int32_t* per_seq) {
  clear_error();
  HS_REQUIRE(totals != nullptr, HS_ERR_NULL, "hs_tree_attention_plan: NULL totals");
  const PlanReport report{totals, per_seq};
  static const int32_t no_table = 0;  // (paged calls are told apart by their block table; none is read on the host)
  return attention_impl(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, host_node_offsets,
                        paged ? nullptr : host_prefix_offsets, nullptr, host_prefix_lens, paged ? &no_table : nullptr,
                        max_blocks, B, Hq, Hkv, D, dt, 1.0f, nullptr, nullptr, nullptr, 0, nullptr, false, &report);
}
