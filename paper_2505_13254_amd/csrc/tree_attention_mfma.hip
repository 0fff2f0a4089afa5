// bfloat16 tree attention on the matrix cores (head dimension 128).
//
// One workgroup = up to 256 query rows of one (sequence, KV head, key split); every wave owns
// 32 * QT rows and keeps their output accumulators in registers for the whole pass, so K and V are
// read from HBM once per workgroup and shared through LDS by all G x M rows of the KV head
// (Section 2.2: every tree row attends to the same prefix).
//
// Both products are computed transposed with v_mfma_f32_32x32x16_bf16:
//     S^T[key, row] = K[key, :] . Q[row, :]      A = K fragment (LDS), B = Q fragment (registers)
//     O^T[d,  row] += V^T[d, key] P^T[key, row]  A = V fragment (LDS), B = P (registers)
// In the S^T accumulator a lane holds 16 keys of ONE row, so the softmax maximum and sum are
// in-lane reductions plus one exchange between the two half-waves, and P^T is already laid out as
// the B operand of the second product: no transposition of P through LDS.  The contraction order of
// the keys inside a 16-key MFMA step is permuted to match that layout, and the V^T fragments are
// fetched from the row-major V tile with the transposing LDS read (ds_read_b64_tr_b16), which hands
// each lane four keys of one output column.
//
// Softmax runs in the log2 domain.  Q is pre-multiplied by scale * log2(e), and the first MFMA of a
// score block starts from an accumulator holding minus the row's reference maximum, so the matrix
// core delivers x - m directly and the only per-score vector work is exp2, the row sum and the
// conversion to bf16.  The reference maximum is updated lazily: accumulators are rescaled only when
// a score exceeds the reference by more than 2^8 (exact after the final division by the equally
// referenced denominator).  The check costs one compare per block: it rides on the row sum of the
// exponentials, which exceeds 2^8 whenever a score does, and only then is the exact maximum taken.
// The first product of block b+1 is issued together with the exponentials of block b, so matrix and
// vector instructions of independent blocks sit in the same scheduling region.
//
// The tree part (ancestor mask) is a bit table built in LDS from the parent pointers.
//
// K/V tiles go from HBM straight into LDS (global_load_lds_dwordx4, 16 bytes per lane, no staging
// registers) through a ring of four tile buffers: while one tile is multiplied and the next one is
// already being read for its scores, two more are on their way (64 KB per compute unit in flight).
// The XOR swizzle that keeps LDS reads conflict-free is applied on the global side: the lane that fills LDS slot c of a row fetches chunk c ^ swz_key(row).
// Waits are explicit (s_waitcnt vmcnt(n) counts this wave's younger tile loads) and the workgroup
// barrier carries no memory fence, so outstanding loads survive it.
#include "attn_common.h"

namespace hs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(3))) shortx4* lds_s4_ptr;

constexpr int MF_ROWS = 256;       // query rows per workgroup
constexpr int MF_TILE = 64;        // keys per LDS tile (two 32-key blocks)
constexpr int MF_NBUF = 4;         // LDS ring: two tiles in use, two on their way from HBM
constexpr int MF_MAX_M = 256;      // tree rows per sequence (ancestor bit table: M x 8 words)
constexpr int MF_ROW_BYTES = 256;  // one K or V row of a head: 128 bf16
constexpr int MF_TILE_BYTES = MF_TILE * MF_ROW_BYTES;
constexpr float MF_LOG2E = 1.4426950408889634f;
constexpr float MF_LN2 = 0.6931471805599453f;
constexpr float MF_LAZY = 8.0f;    // rescale only when the reference maximum is exceeded by 2^8

#ifndef HS_QT
#define HS_QT 1
#endif

bool attn_mfma_supported(int D, hs_dtype dt, int max_tree_rows, float scale) {
  return D == 128 && dt == HS_BF16 && max_tree_rows <= MF_MAX_M && scale > 0.f;
}

// 16-byte chunk c (0..15) of row r lives at chunk position c ^ swz_key(r).  The key takes 16
// different values over 16 consecutive rows (one K row per lane: conflict-free 16-byte reads) and
// its bits 1-2 are the row's low two bits (the four rows that a 16-lane group of the transposing V
// read touches land in four different 32-byte bank ranges).
__device__ __forceinline__ int swz_key(int row) { return ((row & 3) << 1) | ((row >> 2) & 1) | (row & 8); }
__device__ __forceinline__ int swz(int row, int chunk) { return row * MF_ROW_BYTES + ((chunk ^ swz_key(row)) << 4); }

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_addr + 16 i.
// lds_addr is a wave-uniform LDS byte address (placed in M0, which is saved and restored).
__device__ __forceinline__ void lds_dma16(const char* gptr, unsigned lds_addr) {
  const unsigned m = __builtin_amdgcn_readfirstlane(lds_addr);
  unsigned saved;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
      : "=&s"(saved)
      : "s"(m), "v"(gptr)
      : "memory");
}

struct TileSrc {
  const char* k;
  const char* v;
  int64_t base;   // first key of the tile (token index in the prefix, or tree row)
  int64_t limit;  // keys at or beyond it do not exist
  bool tree;
};

// QT = 32-row blocks per wave: 2 -> 4 waves of 64 rows, 1 -> 8 waves of 32 rows (two waves per SIMD).
template <int QT>
__global__ __launch_bounds__(512 / QT) void k_attn_mfma(AttnArgs a, int n_rg_max) {
  constexpr int THREADS = 512 / QT;
  constexpr int LOADS = 1024 / THREADS;  // 16-byte chunks of K (and of V) per thread per tile
  __shared__ __attribute__((aligned(16))) char lds_k[MF_NBUF][MF_TILE_BYTES];
  __shared__ __attribute__((aligned(16))) char lds_v[MF_NBUF][MF_TILE_BYTES];
  __shared__ unsigned anc[MF_MAX_M * 8];

  const int s = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int n0 = a.node_offsets[s];
  const int M = a.node_offsets[s + 1] - n0;
  const int64_t p0 = a.prefix_offsets[s];
  const int64_t L = a.prefix_offsets[s + 1] - p0;
  if (M <= 0) return;
  const int G = a.G, Hkv = a.Hkv, Hq = a.Hq;
  const int R = G * M;
  const int n_rg = (R + MF_ROWS - 1) / MF_ROWS;
  const int n_sp = splits_of(L, a.split_len);
  int x = blockIdx.x;
  const int g = x % Hkv;
  x /= Hkv;
  const int rg = x % n_rg_max;
  const int sp = x / n_rg_max;
  if (rg >= n_rg || sp >= n_sp) return;

  const char* kp = static_cast<const char*>(a.k_prefix) + (p0 * Hkv + g) * MF_ROW_BYTES;
  const char* vp = static_cast<const char*>(a.v_prefix) + (p0 * Hkv + g) * MF_ROW_BYTES;
  const char* kt = static_cast<const char*>(a.k_tree) + ((int64_t)n0 * Hkv + g) * MF_ROW_BYTES;
  const char* vt = static_cast<const char*>(a.v_tree) + ((int64_t)n0 * Hkv + g) * MF_ROW_BYTES;
  const int64_t tok_stride = (int64_t)Hkv * MF_ROW_BYTES;

  const bool last_split = sp == n_sp - 1;
  const int64_t k_lo = (int64_t)sp * a.split_len;
  const int64_t k_hi = last_split ? L : k_lo + a.split_len;
  const int n_ptiles = (int)((k_hi - k_lo + MF_TILE - 1) / MF_TILE);
  const int n_ttiles = last_split ? (M + MF_TILE - 1) / MF_TILE : 0;
  const int n_tiles = n_ptiles + n_ttiles;  // >= 1: a split holds prefix keys, or it is the last one

  auto tile_src = [&](int t) {
    TileSrc ts;
    ts.tree = t >= n_ptiles;
    if (ts.tree) {
      ts.k = kt; ts.v = vt; ts.base = (int64_t)(t - n_ptiles) * MF_TILE; ts.limit = M;
    } else {
      ts.k = kp; ts.v = vp; ts.base = k_lo + (int64_t)t * MF_TILE; ts.limit = k_hi;
    }
    return ts;
  };

  // ---- ancestor bit table: bit j of row i's words is set iff tree row j is on the root path of i
  if (last_split && tid < M) {
    unsigned w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = tid; j >= 0; j = a.parent[n0 + j]) {
#pragma unroll
      for (int q = 0; q < 8; ++q) w[q] |= ((j >> 5) == q) ? (1u << (j & 31)) : 0u;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) anc[tid * 8 + q] = w[q];
  }

  // ---- this wave's rows; Q fragments (B operand of the first product), pre-multiplied by
  // scale * log2(e) so that the scores come out of the MFMA in the log2 domain
  const float c2 = a.scale * MF_LOG2E;
  const int row_base = rg * MF_ROWS + wave * (32 * QT);
  const bool wave_active = row_base < R;
  bf16x8 qf[QT][8];
  int tree_row[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int r = row_base + qt * 32 + col;
    const int rc = r < R ? r : R - 1;
    const int i = rc / G, gi = rc - i * G;
    tree_row[qt] = i;
    const char* qrow = static_cast<const char*>(a.q) + ((int64_t)(n0 + i) * Hq + g * G + gi) * MF_ROW_BYTES;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      bf16x8 raw = {0, 0, 0, 0, 0, 0, 0, 0};
      if (r < R && wave_active) raw = *reinterpret_cast<const bf16x8*>(qrow + (2 * kk + half) * 16);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        floatx2 f = {(float)raw[2 * e] * c2, (float)raw[2 * e + 1] * c2};
        bf16x2 hb = __builtin_convertvector(f, bf16x2);
        qf[qt][kk][2 * e] = hb[0];
        qf[qt][kk][2 * e + 1] = hb[1];
      }
    }
  }

  floatx16 acc[QT][4];   // O^T: [d block of 32][16 values]: d = 32 tt + 8 (v / 4) + 4 half + v % 4
  floatx16 negm[QT];     // minus the reference maximum in all 16 slots: start value of a score block
  float m_ref[QT], l_sum[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m_ref[qt] = 0.f;
    l_sum[qt] = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) negm[qt][v] = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[qt][t][v] = 0.f;
  }

  // ---- tile loads.  Issued as inline assembly: the compiler then neither tracks them in its own
  // wait counters nor orders LDS reads of other ring slots behind them.
  const unsigned lds_k_addr = (unsigned)(uintptr_t)(lds_ptr)&lds_k[0][0];
  const unsigned lds_v_addr = (unsigned)(uintptr_t)(lds_ptr)&lds_v[0][0];
  // per-lane byte offsets inside a full prefix tile: fixed for the whole pass
  int64_t lane_off[LOADS];
  unsigned lane_lds[LOADS];
#pragma unroll
  for (int j = 0; j < LOADS; ++j) {
    const int c = j * THREADS + tid;  // LDS slot (16-byte units) this lane fills
    const int row = c >> 4, slot = c & 15;
    lane_off[j] = (int64_t)row * tok_stride + ((slot ^ swz_key(row)) << 4);
    lane_lds[j] = (unsigned)((j * THREADS + wave * 64) << 4);  // wave-uniform LDS byte offset
  }
  auto issue = [&](int t) {
    const unsigned ring = (unsigned)(t % MF_NBUF) * MF_TILE_BYTES;
    if (t < n_ptiles && k_lo + (int64_t)(t + 1) * MF_TILE <= k_hi) {
      // a full tile of prefix keys: one scalar base plus the fixed lane offsets
      const int64_t tile_off = (k_lo + (int64_t)t * MF_TILE) * tok_stride;
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        lds_dma16(kp + tile_off + lane_off[j], lds_k_addr + ring + lane_lds[j]);
        lds_dma16(vp + tile_off + lane_off[j], lds_v_addr + ring + lane_lds[j]);
      }
      return;
    }
    const TileSrc ts = tile_src(t);
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int c = j * THREADS + tid;
      const int row = c >> 4, slot = c & 15;
      int64_t key = ts.base + row;
      key = key < ts.limit ? key : ts.limit - 1;  // rows past the end repeat the last row (masked later)
      const int64_t off = key * tok_stride + ((slot ^ swz_key(row)) << 4);
      lds_dma16(ts.k + off, lds_k_addr + ring + lane_lds[j]);
      lds_dma16(ts.v + off, lds_v_addr + ring + lane_lds[j]);
    }
  };
  // Wait until this wave's loads of tile t have landed (only the loads of tile t+1 may still be
  // pending), then meet the other waves.  It is called while tile t-1 is still being multiplied, so
  // the slot that is free for a new load is the one of tile t-2: tile t+2 goes there.
  auto arrive = [&](int t) {
    if (t + 1 < n_tiles) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * LOADS) : "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (t + 2 < n_tiles) issue(t + 2);
  };

  // ---- S^T block = K[32 keys] Q^T, started from -m_ref
  auto qk = [&](int blk, floatx16 (&S)[QT]) {
    const char* kbuf = lds_k[(blk >> 1) % MF_NBUF];
    const int krow = (blk & 1) * 32 + col;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kbuf + swz(krow, 2 * kk + half));
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
        S[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qt][kk], kk == 0 ? negm[qt] : S[qt], 0, 0, 0);
    }
  };
  // ---- masks of a block's scores: tree keys off the row's root path, keys past the end of the
  // split.  Only the blocks from n_plain on need it (the partial prefix tail and the tree part).
  const int n_plain = (int)((k_hi - k_lo) >> 5);
  auto mask_block = [&](int blk, floatx16 (&S)[QT]) {
    const TileSrc ts = tile_src(blk >> 1);
    const int64_t bbase = ts.base + (blk & 1) * 32;
    if (ts.tree) {
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        const unsigned word = bbase < ts.limit ? anc[tree_row[qt] * 8 + (int)(bbase >> 5)] : 0u;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int bit = 8 * (v >> 2) + 4 * half + (v & 3);
          S[qt][v] = ((word >> bit) & 1u) ? S[qt][v] : -HS_INF;
        }
      }
    } else if (bbase + 32 > ts.limit) {
      const int valid = (int)(ts.limit - bbase);  // may be <= 0: the whole block is past the end
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 8 * (v >> 2) + 4 * half + (v & 3);
        if (key >= valid) {
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) S[qt][v] = -HS_INF;
        }
      }
    }
  };
  // exact maximum of a row's 32 scores of a block (both half-waves)
  auto row_max = [&](const floatx16& S) {
    float m4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) m4[c] = fmaxf(fmaxf(S[c], S[4 + c]), fmaxf(S[8 + c], S[12 + c]));
    const float mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
    return fmaxf(mx, __shfl_xor(mx, 32));
  };
  // moves the reference maximum of row block qt up by delta (>= 0 except at the very first block)
  auto move_reference = [&](int qt, float delta) {
    const float alpha = exp2_fast(-delta);
    m_ref[qt] += delta;
    l_sum[qt] *= alpha;
#pragma unroll
    for (int v = 0; v < 16; ++v) negm[qt][v] = -m_ref[qt];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[qt][tt][v] *= alpha;
  };
  // ---- P = exp2(S) as bf16 B operands; row sums.  The lazy reference check rides on the row sum:
  // a score above the reference by more than 2^8 makes the sum exceed 2^8 (so does an overflow), and
  // only then the exact maximum is taken, the reference moved and the block redone.  S_next (scores
  // of the following block, already started from the old reference) moves along.
  auto exps = [&](floatx16 (&S)[QT], bf16x8 (&P)[QT][2], floatx16 (&S_next)[QT], bool have_next) {
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      float p[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) p[v] = exp2_fast(S[qt][v]);
      float s4[4];  // four independent partial sums
#pragma unroll
      for (int c = 0; c < 4; ++c) s4[c] = (p[c] + p[4 + c]) + (p[8 + c] + p[12 + c]);
      float ps = (s4[0] + s4[1]) + (s4[2] + s4[3]);
      if (__ballot(!(ps <= 256.f)) != 0ull) {  // rare
        const float mx = row_max(S[qt]);
        const float delta = mx > 0.f ? mx : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          S[qt][v] -= delta;
          p[v] = exp2_fast(S[qt][v]);
          if (have_next) S_next[qt][v] -= delta;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) s4[c] = (p[c] + p[4 + c]) + (p[8 + c] + p[12 + c]);
        ps = (s4[0] + s4[1]) + (s4[2] + s4[3]);
        move_reference(qt, delta);
      }
      l_sum[qt] += ps;
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          floatx2 f = {p[8 * k2 + 2 * e], p[8 * k2 + 2 * e + 1]};
          bf16x2 hb = __builtin_convertvector(f, bf16x2);
          P[qt][k2][2 * e] = hb[0];
          P[qt][k2][2 * e + 1] = hb[1];
        }
    }
  };
  // ---- O^T += V^T P^T for one 32-key block.  The transposing read returns, to lane l of a 16-lane
  // group, element l % 4 of the 8-byte pieces addressed by lanes l / 4 + {0, 4, 8, 12} of the group:
  // lane (a = l % 4, j = l / 4) therefore addresses key j of the wanted four at columns 4a .. 4a+3.
  const int tr_a = lane & 3, tr_j = (lane >> 2) & 3, tr_dh = (lane >> 4) & 1;
  auto pv = [&](int blk, const bf16x8 (&P)[QT][2]) {
    const char* vbuf = lds_v[(blk >> 1) % MF_NBUF];
    const int kb = blk & 1;
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        bf16x8 vf;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          const int key = kb * 32 + 16 * k2 + 8 * r + 4 * half + tr_j;
          const int chunk = 4 * tt + 2 * tr_dh + (tr_a >> 1);
          const shortx4 got = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s4_ptr)(vbuf + swz(key, chunk) + (tr_a & 1) * 8));
          const bf16x4 gb = __builtin_bit_cast(bf16x4, got);
          vf[4 * r + 0] = gb[0];
          vf[4 * r + 1] = gb[1];
          vf[4 * r + 2] = gb[2];
          vf[4 * r + 3] = gb[3];
        }
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          acc[qt][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, P[qt][k2], acc[qt][tt], 0, 0, 0);
      }
    }
  };

  issue(0);
  if (n_tiles > 1) issue(1);
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // the ancestor table is complete

  const int n_blocks = 2 * n_tiles;
  floatx16 s_cur[QT], s_next[QT];
  bf16x8 pb[QT][2];
  arrive(0);
  if (wave_active) {
    qk(0, s_cur);
    mask_block(0, s_cur);
    // the first block always has a visible key (a prefix token, or the root): its exact maximum
    // becomes the first reference
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      const float mx = row_max(s_cur[qt]);
#pragma unroll
      for (int v = 0; v < 16; ++v) s_cur[qt][v] -= mx;
      move_reference(qt, mx);
    }
  }
  for (int blk = 0; blk + 1 < n_blocks; ++blk) {
    if (blk & 1) arrive((blk + 1) >> 1);  // the next block opens a new tile
    if (wave_active) {
      qk(blk + 1, s_next);              // matrix pipe: scores of the next block ...
      exps(s_cur, pb, s_next, true);    // ... vector pipe: exponentials of this one
      pv(blk, pb);                      // matrix pipe: second product of this block
      if (blk + 1 >= n_plain) mask_block(blk + 1, s_next);
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) s_cur[qt] = s_next[qt];
    }
  }
  if (wave_active) {
    exps(s_cur, pb, s_next, false);
    pv(n_blocks - 1, pb);
  }

  // ---- results: direct (single split everywhere) or this split's partial record
  if (!wave_active) return;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int r = row_base + qt * 32 + col;
    const float l_tot = l_sum[qt] + __shfl_xor(l_sum[qt], 32);
    if (r >= R) continue;
    const int i = r / G, gi = r - i * G;
    const int64_t row = (int64_t)(n0 + i) * Hq + g * G + gi;
    if (a.sp_max == 1) {
      const float inv = 1.f / l_tot;
      char* out = static_cast<char*>(a.o) + row * MF_ROW_BYTES;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int d0 = 32 * tt + 8 * b + 4 * half;
          floatx2 f01 = {acc[qt][tt][4 * b] * inv, acc[qt][tt][4 * b + 1] * inv};
          floatx2 f23 = {acc[qt][tt][4 * b + 2] * inv, acc[qt][tt][4 * b + 3] * inv};
          uint2 pk;
          pk.x = __builtin_bit_cast(unsigned, __builtin_convertvector(f01, bf16x2));
          pk.y = __builtin_bit_cast(unsigned, __builtin_convertvector(f23, bf16x2));
          *reinterpret_cast<uint2*>(out + d0 * 2) = pk;
        }
      if (a.lse && half == 0) a.lse[row] = (m_ref[qt] + __log2f(l_tot)) * MF_LN2;
    } else {
      float* rec = a.part + (row * a.sp_max + sp) * ATTN_REC;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int d0 = 32 * tt + 8 * b + 4 * half;
          float4 f = {acc[qt][tt][4 * b], acc[qt][tt][4 * b + 1], acc[qt][tt][4 * b + 2], acc[qt][tt][4 * b + 3]};
          *reinterpret_cast<float4*>(rec + d0) = f;
        }
      if (half == 0) {
        rec[128] = m_ref[qt] * MF_LN2;
        rec[129] = l_tot;
      }
    }
  }
}

hs_status attn_mfma_launch(const AttnArgs& a, int max_tree_rows, hipStream_t stream) {
  const int n_rg_max = (a.G * max_tree_rows + MF_ROWS - 1) / MF_ROWS;
  dim3 grid((unsigned)(a.Hkv * n_rg_max * a.sp_max), (unsigned)a.B);
  hipLaunchKernelGGL(k_attn_mfma<HS_QT>, grid, dim3(512 / HS_QT), 0, stream, a, n_rg_max);
  return launch_status("tree attention (mfma)");
}

}  // namespace hs
