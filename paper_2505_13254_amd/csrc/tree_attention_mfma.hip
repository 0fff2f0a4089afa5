// bfloat16 tree attention on the matrix cores (head dimension 128; head dimension 64 by taking
// the KV heads in pairs, see HALF below).
//
// One workgroup = up to 256 query rows of one (sequence, KV head, key split); each of its eight
// waves owns 32 rows and keeps their output accumulators in registers for the whole pass, so K and
// V are read from HBM once per workgroup and shared through LDS by all G x M rows of the KV head
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
// conversion to bf16.
//
// The reference maximum of a row is the exact maximum of its first 32-key block and then stays
// fixed: nothing is rescaled inside the loop.  P and the accumulators are floating point, so a later
// score above the reference only makes them larger, with the same relative precision; the result
// is exact after the final division by the equally referenced denominator.  Only an overflow (a
// score more than ~2^6 octaves above the reference) would break this; it shows in the denominator at
// the end of the pass, and the workgroup then repeats its pass with the classic block-by-block
// update of the maximum (rare, slow, same result).
//
// Schedule.  Each 32-key block passes through two windows of eight matrix instructions: its scores,
// then its second product.  A window also takes half of a block's exponentials (the second half of
// the block whose product comes next, or the first half of the block whose scores were just
// finished) and requests the LDS fragments that the matrix instructions three steps ahead will
// need, so matrix, vector and LDS pipes of a wave all have independent work at any time.
//
// The tree part (ancestor mask) is a bit table built in LDS from the parent pointers (trees of up
// to 256 rows).  Larger trees (BIG, up to 1024 rows) take the table from global memory, where
// k_anc_tiles has laid it out per 64-key tile before the launch: the slice of a tree tile (two words
// for each of the workgroup's 256 rows) travels into a ring in LDS together with the tile.
//
// K/V tiles go from HBM straight into LDS (global_load_lds_dwordx4, 16 bytes per lane, no staging
// registers) through a ring of four tile buffers: one tile is being multiplied, the next one has
// landed, two more are on their way (64 KB per compute unit in flight).  The XOR swizzle that keeps
// LDS reads conflict-free is applied on the global side: the lane that fills LDS slot c of a row
// fetches chunk c ^ swz_key(row).  Waits are explicit (s_waitcnt vmcnt(n) counts this wave's younger
// tile loads) and the workgroup barrier carries no memory fence, so outstanding loads survive it.
#include <type_traits>

#include <hip/hip_ext.h>

#include "attn_common.h"

namespace hs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(3))) shortx4* lds_s4_ptr;

constexpr int MF_ROWS = 256;       // query rows per workgroup
constexpr int MF_THREADS = 512;    // eight waves of 32 rows, two per SIMD
constexpr int MF_TILE = 64;        // keys per LDS tile (two 32-key blocks)
constexpr int MF_NBUF = 4;         // LDS ring: one tile in use, one landed, two on their way from HBM
constexpr int MF_MAX_M = 256;      // tree rows per sequence whose ancestor bit table (M x 8 words) is built in LDS
constexpr int MF_BIG_M = 1024;     // tree rows per sequence with the table in global memory
constexpr int MF_ANC_SLICE = 2 * MF_ROWS;  // words of a tree tile's mask slice: two per row of the workgroup
constexpr int MF_ROW_BYTES = 256;  // one K or V row of a head: 128 bf16
constexpr int MF_TILE_BYTES = MF_TILE * MF_ROW_BYTES;
constexpr int MF_BLOCK_BYTES = 32 * MF_ROW_BYTES;
constexpr int MF_LOADS = MF_TILE * 16 / MF_THREADS;  // 16-byte chunks of K (and of V) per thread per tile
constexpr int MF_AHEAD = 1;        // LDS fragments are requested this many steps (of two matrix instructions) ahead
constexpr float MF_LOG2E = 1.4426950408889634f;
constexpr float MF_LN2 = 0.6931471805599453f;
constexpr float MF_SUM_LIMIT = 0x1p64f;  // a denominator beyond it (or NaN) sends the pass to the exact path

// (D = 64: the caller also makes sure that the number of KV heads is even)
bool attn_mfma_supported(int D, hs_dtype dt, int max_tree_rows, float scale) {
  return (D == 128 || D == 64) && dt == HS_BF16 && max_tree_rows <= MF_BIG_M && scale > 0.f;
}

// Bytes of the ancestor table that launches with more than MF_MAX_M rows in a tree keep in the
// workspace: 16 tiles x two words for every tree row of the batch (0: no such table is needed).
size_t attn_mfma_table_bytes(int max_tree_rows, int64_t NN) {
  return max_tree_rows > MF_MAX_M ? (size_t)NN * (MF_BIG_M / MF_TILE) * 8 : 0;
}

// Ancestor table of large trees, one slice per 64-key tile: words (2 i, 2 i + 1) of tile tt hold bit
// j - 64 tt for every tree row j of [64 tt, 64 tt + 64) on the root path of tree row i (itself
// included).  The table of the sequence whose first row is n0 starts at word 32 n0; tile tt of a
// tree of M rows lies 2 M tt words further.  grid: (row chunks of 256, sequences).
__global__ __launch_bounds__(256) void k_anc_tiles(const int32_t* __restrict__ parent, const int32_t* __restrict__ node_offsets,
                                                   unsigned* __restrict__ table) {
  __shared__ int par[MF_BIG_M];
  const int s = blockIdx.y;
  const int n0 = node_offsets[s];
  int M = node_offsets[s + 1] - n0;
  if (M > MF_BIG_M) M = MF_BIG_M;  // (the host has refused larger trees)
  if ((int)blockIdx.x * 256 >= M) return;
  for (int i = threadIdx.x; i < M; i += 256) par[i] = parent[n0 + i];
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= M) return;
  unsigned* out = table + (size_t)n0 * 32;
  const int n_tt = (M + MF_TILE - 1) / MF_TILE;
  // the path is walked once, from the row towards the root: row numbers fall, and so do the tiles
  int j = i;
  for (int tt = n_tt - 1; tt >= 0; --tt) {
    const int lo = tt * MF_TILE;
    unsigned w0 = 0, w1 = 0;
    while (j >= lo) {
      const int b = j - lo;
      if (b < 32) w0 |= 1u << b;
      else if (b < 64) w1 |= 1u << (b - 32);
      const int up = par[j];
      j = up < j ? up : -1;  // (a malformed tree cannot keep the walk from ending)
    }
    uint2 w = {w0, w1};
    *reinterpret_cast<uint2*>(out + ((size_t)tt * M + i) * 2) = w;
  }
}

// 16-byte chunk c (0..15) of row r lives at chunk position c ^ swz_key(r).  The key takes 16
// different values over 16 consecutive rows (one K row per lane: conflict-free 16-byte reads) and
// its upper two bits are the row's low two bits: the four rows that a transposing V read touches
// within a half-wave land in four different 64-byte bank ranges.
__device__ __forceinline__ int swz_key(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int swz(int row, int chunk) { return row * MF_ROW_BYTES + ((chunk ^ swz_key(row)) << 4); }

// One tile from global memory straight into LDS: four loads of 16 bytes per lane (K and V, two row
// groups each).  A load lands at its wave-uniform LDS byte address (taken from M0, which is saved
// and restored) + 16 * lane; its source is a scalar base plus a 32-bit lane offset.
// ONCE: no other workgroup reads these keys, every head's rows fit one row group (a property of the
// launch, so that the hot loop has no branch for it).  The loads then carry the non-temporal hint, so that the stream does not push the data of
// the step's other kernels out of the caches (measured on the 32-layer launch: this kernel 1.5 us
// faster, the step's other kernels 3 us; 8 % on the 64-sequence batch).  With several row groups the
// later ones find the keys in L2, and the hint would cost that (3 % on the 1023-row workload).
#define MF_DMA_TILE(HINT)                                                                                  \
  asm volatile("s_mov_b32 %0, m0\n\t"                                                                      \
               "s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %5, %7" HINT "\n\t"                             \
               "s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %5, %8" HINT "\n\t"                             \
               "s_mov_b32 m0, %3\n\tglobal_load_lds_dwordx4 %6, %7" HINT "\n\t"                             \
               "s_mov_b32 m0, %4\n\tglobal_load_lds_dwordx4 %6, %8" HINT "\n\t"                             \
               "s_mov_b32 m0, %0"                                                                          \
               : "=&s"(saved)                                                                              \
               : "s"(lds_k0), "s"(lds_v0), "s"(lds_k1), "s"(lds_v1), "v"(off0), "v"(off1), "s"(kbase), "s"(vbase) \
               : "memory")
template <bool ONCE>
__device__ __forceinline__ void lds_dma_tile(const char* kbase, const char* vbase, unsigned off0, unsigned off1,
                                             unsigned lds_k0, unsigned lds_v0, unsigned lds_k1, unsigned lds_v1) {
  unsigned saved;
  if constexpr (ONCE) MF_DMA_TILE(" nt");
  else MF_DMA_TILE("");
}
#undef MF_DMA_TILE

// s_waitcnt on the LDS counter alone (vmcnt and expcnt fields at their maxima)
#define MF_WAIT_LDS_CONST(n) __builtin_amdgcn_s_waitcnt(0xC07F | ((n) << 8))
__device__ __forceinline__ void wait_lds(int n) {  // n is a constant once the windows are unrolled
  switch (n) {
    case 0: MF_WAIT_LDS_CONST(0); break;
    case 2: MF_WAIT_LDS_CONST(2); break;
    case 4: MF_WAIT_LDS_CONST(4); break;
    case 6: MF_WAIT_LDS_CONST(6); break;
    case 8: MF_WAIT_LDS_CONST(8); break;
    case 10: MF_WAIT_LDS_CONST(10); break;
    case 12: MF_WAIT_LDS_CONST(12); break;
    default: break;  // no hint: the compiler's own waits stand
  }
}

#define MF_PIN() __builtin_amdgcn_sched_barrier(0)

// PAGED: the prefix K/V live in pages of MF_TILE tokens ([page, token, Hkv, D]); a tile is a page.
// BIG: trees of more than MF_MAX_M rows may occur; the ancestor table comes from a.anc_tiles.
// HALF: head dimension 64.  Two neighbouring KV heads of a token are 256 contiguous bytes, i.e. one
// row of this kernel, and a.Hkv / a.G count such pairs and the 2 G query heads that read them.  A
// query row is widened to 128 elements with zeros on the other head's side, so its scores see its own
// KV head only; the second product yields both heads' values and the row's own half is stored.  The
// matrix cores do twice the arithmetic; K and V are still read once, in whole 256-byte rows.
template <bool PAGED, bool ONCE, bool BIG, bool HALF>
__global__ __launch_bounds__(MF_THREADS) void k_attn_mfma(AttnArgs a, int n_rg_max) {
  constexpr int Q_ROW_BYTES = HALF ? MF_ROW_BYTES / 2 : MF_ROW_BYTES;  // a row of Q and of O
  constexpr int Q_LOADS = HALF ? 4 : 8;                                 // 16-byte loads of a lane's part of it
  static_assert(!(BIG && ONCE), "more than 256 tree rows are several row groups");
  static_assert(MF_NBUF * MF_ANC_SLICE == MF_MAX_M * 8, "the slice ring of large trees takes the place of the table");
  __shared__ __attribute__((aligned(16))) char lds_k[MF_NBUF][MF_TILE_BYTES];
  __shared__ __attribute__((aligned(16))) char lds_v[MF_NBUF][MF_TILE_BYTES];
  __shared__ unsigned anc[MF_MAX_M * 8];
  __shared__ int par_lds[MF_MAX_M];
  __shared__ int exact_flag;
  __shared__ int page_lds[PAGED ? 256 : 1];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (uniform for the compiler too: scalar branches)
  const int col = lane & 31, half = lane >> 5;
  // The first 64 entries of the work-list table are requested before anything else (the table is
  // part of the kernel arguments, so entry `lane` exists whatever the launch), and every scalar
  // argument the kernel needs is fetched in one batch right behind: left to itself the compiler
  // fetches each argument where it is first used, one scalar-cache round trip after another.
  uintx4 t0_lo = *reinterpret_cast<const uintx4*>(&a.tbl[lane]);
  uintx4 t0_hi = *(reinterpret_cast<const uintx4*>(&a.tbl[lane]) + 1);
  const void* const h_q = a.q;
  const void* const h_k_prefix = a.k_prefix;
  const void* const h_v_prefix = a.v_prefix;
  const void* const h_k_tree = a.k_tree;
  const void* const h_v_tree = a.v_tree;
  const int32_t* const h_parent = a.parent;
  void* const h_o = a.o;
  const unsigned* const h_anc = a.anc_tiles;
  float* const h_lse = a.lse;
  float* const h_part = a.part;
  const float h_scale = a.scale;
  const int h_sp_max = a.sp_max, h_n_tbl = a.n_tbl, h_tree_shared = a.tree_shared;
  const int G = a.G, Hkv = a.Hkv, Hq = a.Hq;
  asm volatile("" : "+v"(t0_lo), "+v"(t0_hi));  // (keeps the request here instead of inside the branch that uses it)
  asm volatile("" ::"s"(h_q), "s"(h_k_prefix), "s"(h_v_prefix), "s"(h_k_tree), "s"(h_v_tree), "s"(h_parent), "s"(h_o),
               "s"(h_lse), "s"(h_part), "s"(h_scale), "s"(h_sp_max), "s"(h_n_tbl), "s"(G), "s"(Hkv), "s"(Hq),
               "s"(n_rg_max), "s"(h_tree_shared));
  int n0, M, g, rg, sp, n_sp, tiles_per_split;
  int64_t p0, L;
  if (h_n_tbl > 0) {
    // Work-list launch: the table of sequences sits in the kernel arguments; lane l fetches entry
    // l (and l + 64), a ballot finds the entry whose item range holds this workgroup, and its
    // fields are read from that lane: one memory round trip, no dependent offset loads.
    const int x = blockIdx.x;
    unsigned f[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int base = 0; base < h_n_tbl; base += 64) {
      const int idx = base + lane;
      uintx4 lo = {0x7fffffffu, 0, 0, 0}, hi = {0, 0, 0, 0};
      if (base == 0) {
        if (idx < h_n_tbl) {
          lo = t0_lo;
          hi = t0_hi;
        }
      } else if (idx < h_n_tbl) {
        lo = *reinterpret_cast<const uintx4*>(&a.tbl[idx]);
        hi = *(reinterpret_cast<const uintx4*>(&a.tbl[idx]) + 1);
      }
      const unsigned long long below = __ballot((int)lo[0] <= x);  // entries are in rising first_item order
      if (below == 0ull) break;
      const int e = __builtin_popcountll(below) - 1;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        f[k] = __builtin_amdgcn_readlane(lo[k], e);
        f[4 + k] = __builtin_amdgcn_readlane(hi[k], e);
      }
      if (below != ~0ull) break;
    }
    n0 = (int)f[1];
    M = (int)f[2];
    L = (int)f[3];
    p0 = (int64_t)(((unsigned long long)f[5] << 32) | f[4]);
    tiles_per_split = (int)f[6];
    n_sp = (int)(short)(f[7] & 0xffffu);
    const int n_rg = (int)(short)(f[7] >> 16);
    int local = x - (int)f[0];
    g = local % Hkv;
    local /= Hkv;
    rg = local % n_rg;
    sp = local / n_rg;
  } else {
    const int s = blockIdx.y;
    n0 = a.node_offsets[s];
    M = a.node_offsets[s + 1] - n0;
    p0 = PAGED ? (int64_t)s * a.max_blocks : a.prefix_offsets[s];
    L = prefix_len_of(a, s);
    if (M <= 0) return;
    n_sp = splits_of(L, a.split_len);
    tiles_per_split = a.split_len / MF_TILE;
    int x = blockIdx.x;
    g = x % Hkv;
    x /= Hkv;
    rg = x % n_rg_max;
    sp = x / n_rg_max;
    if (rg >= (G * M + MF_ROWS - 1) / MF_ROWS || sp >= n_sp) return;
  }
  const int R = G * M;

  const char* kp = static_cast<const char*>(h_k_prefix) + ((PAGED ? 0 : p0) * Hkv + g) * MF_ROW_BYTES;
  const char* vp = static_cast<const char*>(h_v_prefix) + ((PAGED ? 0 : p0) * Hkv + g) * MF_ROW_BYTES;
  const char* kt = static_cast<const char*>(h_k_tree) + ((int64_t)n0 * Hkv + g) * MF_ROW_BYTES;
  const char* vt = static_cast<const char*>(h_v_tree) + ((int64_t)n0 * Hkv + g) * MF_ROW_BYTES;
  const int64_t tok_stride = (int64_t)Hkv * MF_ROW_BYTES;

  const bool last_split = sp == n_sp - 1;
  const int64_t k_lo = (int64_t)sp * tiles_per_split * MF_TILE;
  const int64_t k_hi = last_split ? L : k_lo + (int64_t)tiles_per_split * MF_TILE;
  const int n_ptiles = (int)((k_hi - k_lo + MF_TILE - 1) / MF_TILE);
  // (large trees: tree rows behind the last row of this row group are on nobody's root path, their tiles are left out)
  int tree_keys = M;
  if constexpr (BIG)
    if ((rg + 1) * MF_ROWS < R) tree_keys = ((rg + 1) * MF_ROWS - 1) / G + 1;
  const int n_ttiles = last_split ? (tree_keys + MF_TILE - 1) / MF_TILE : 0;
  const int n_tiles = n_ptiles + n_ttiles;  // >= 1: a split holds prefix keys, or it is the last one
  const int n_full = (int)((k_hi - k_lo) / MF_TILE);  // leading tiles made of 64 prefix keys
  const int n_plain = (int)((k_hi - k_lo) >> 5);      // leading blocks that need no mask

  // ---- tile loads.  Issued as inline assembly: the compiler then neither tracks them in its own
  // wait counters nor orders LDS reads of other ring slots behind them.  The lane that fills the
  // 16-byte LDS slot c of a tile (row c / 16, position c % 16) fetches chunk (c % 16) ^ swz_key(row).
  static_assert(MF_LOADS == 2, "lds_dma_tile moves two row groups of K and of V");
  const unsigned lds_k_addr = (unsigned)(uintptr_t)(lds_ptr)&lds_k[0][0];
  const unsigned lds_v_addr = (unsigned)(uintptr_t)(lds_ptr)&lds_v[0][0];
  const unsigned wave_lds = __builtin_amdgcn_readfirstlane((unsigned)(wave * 64 * 16));  // this wave's 1 KB of a row group
  const int dma_row = tid >> 4;                                                        // + 32 for the second row group
  const unsigned dma_chunk = (unsigned)(((tid & 15) ^ swz_key(dma_row)) << 4);         // swz_key(row + 32) == swz_key(row)
  const unsigned lane_off0 = (unsigned)(dma_row * (int)tok_stride) + dma_chunk;        // inside a full tile: fixed
  const unsigned lane_off1 = lane_off0 + (unsigned)(32 * (int)tok_stride);
  // Large trees: lane l of wave w fetches word l % 2 of the workgroup's row 32 w + l / 2 (rows past
  // the end: of the last row) from a tile's slice of this sequence's table.
  const unsigned lds_anc_addr = (unsigned)(uintptr_t)(lds_ptr)&anc[0];
  const unsigned* anc_tbl = nullptr;
  unsigned anc_lane_off = 0;
  if constexpr (BIG) {
    anc_tbl = h_anc + (size_t)(h_tree_shared ? 0 : n0) * 32;
    int r = rg * MF_ROWS + wave * 32 + (lane >> 1);
    r = r < R ? r : R - 1;
    anc_lane_off = (unsigned)(((r / G) * 2 + (lane & 1)) * 4);
  }
  // Paged caches: the pages of this split's tiles (at most 256) are staged in LDS; the requests
  // go out here, before the Q rows are asked for, so that waiting for them waits for nothing else.
  // A tile's page is then one LDS read.  (That read is older than every fragment read requested
  // after it, so the windows' counted LDS waits at most wait for one fragment more than they need.)
  if (PAGED) {
    const int32_t* bt = a.block_table + p0 + k_lo / MF_TILE;
    if (tid < n_ptiles) page_lds[tid] = bt[tid];
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  }
  // byte offset, from kp / vp, of prefix tile t of this split
  auto prefix_tile = [&](int t) -> int64_t {
    if (!PAGED) return (k_lo + (int64_t)t * MF_TILE) * tok_stride;
    return (int64_t)__builtin_amdgcn_readfirstlane(page_lds[t]) * MF_TILE * tok_stride;
  };
  // a full tile of prefix keys into ring slot `slot`
  auto issue_full = [&](int t, int slot) {
    const int64_t tile_off = prefix_tile(t);
    const unsigned ring = (unsigned)slot * MF_TILE_BYTES + wave_lds;
    lds_dma_tile<ONCE>(kp + tile_off, vp + tile_off, lane_off0, lane_off1, lds_k_addr + ring, lds_v_addr + ring,
                 lds_k_addr + ring + MF_BLOCK_BYTES, lds_v_addr + ring + MF_BLOCK_BYTES);
  };
  // any tile: the last prefix tile may be partial, tree tiles come from the tree buffers; rows past
  // the end repeat the last row (their scores are masked)
  auto issue = [&](int t) {
    if (t < n_full) {
      issue_full(t, t % MF_NBUF);
      return;
    }
    const bool tree = t >= n_ptiles;
    const char* ks = tree ? kt : kp;
    const char* vs = tree ? vt : vp;
    const int64_t base = tree ? (int64_t)(t - n_ptiles) * MF_TILE : k_lo + (int64_t)t * MF_TILE;
    const int rows = (int)((tree ? (int64_t)M : k_hi) - base);  // >= 1 rows of this tile exist
    const int r0 = dma_row < rows ? dma_row : rows - 1;
    const int r1 = dma_row + 32 < rows ? dma_row + 32 : rows - 1;
    const unsigned ring = (unsigned)(t % MF_NBUF) * MF_TILE_BYTES + wave_lds;
    const int64_t off = tree ? base * tok_stride : prefix_tile(t);
    if constexpr (BIG) {
      // The tile's slice of the ancestor table goes first: one more load of this wave, older than the
      // tile's four, so a wait that leaves the four youngest loads pending has seen it land.
      if (tree) {
        const unsigned* src = anc_tbl + (size_t)(t - n_ptiles) * (2 * (size_t)M);
        const unsigned dst = lds_anc_addr + (unsigned)(t % MF_NBUF) * (MF_ANC_SLICE * 4) + (unsigned)(wave * 256);
        unsigned saved;
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dword %2, %3\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved)
                     : "s"(dst), "v"(anc_lane_off), "s"(src)
                     : "memory");
      }
    }
    lds_dma_tile<ONCE>(ks + off, vs + off, (unsigned)(r0 * (int)tok_stride) + dma_chunk,
                 (unsigned)(r1 * (int)tok_stride) + dma_chunk, lds_k_addr + ring, lds_v_addr + ring,
                 lds_k_addr + ring + MF_BLOCK_BYTES, lds_v_addr + ring + MF_BLOCK_BYTES);
  };
  // waits until at most n (a multiple of four, at most 16) of this wave's loads are pending
  auto wait_vm = [&](int n) {
    switch (n) {
      case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
      case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
      case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
      case 12: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
      default: asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
    }
  };
  // Start of a pass: tiles 0 and 1 are on their way; wait for this wave's part of tile 0, meet the
  // other waves, request tile 2.
  auto first_arrival = [&]() {
    if (n_tiles > 1) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * MF_LOADS) : "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (2 < n_tiles) issue(2);
  };
  // Middle of trip t (tile t is being multiplied): wait for this wave's part of tile t + 1 (tile
  // t + 2 may still be pending), meet the other waves, request tile t + 3.  Every wave has finished
  // tile t - 1 by then: its slot is the one that tile t + 3 goes to.
  auto next_arrival = [&](int t) {
    if (t + 2 < n_tiles) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * MF_LOADS) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    if (t + 3 < n_tiles) issue(t + 3);
  };

  // ---- set-up.  Its global reads (parent pointers, Q rows) are requested first and the first two
  // K/V tiles right behind them, so that HBM is busy while the ancestor table is built and Q is
  // converted.  (Loads return in order: waiting for the Q rows never waits for a tile.)
  const int row_base = rg * MF_ROWS + wave * 32;
  const bool wave_active = row_base < R;
  // r / G for a row number r < 2^16 without the integer-division sequence: (r + 0.5) / G is at least
  // 1 / (2 G) away from an integer, far more than the rounding of the float product
  const float inv_G = 1.0f / (float)G;
  auto div_G = [&](int r) { return (int)(((float)r + 0.5f) * inv_G); };
  // These loads are inline assembly like the tile loads: the compiler does not see the tile loads, so
  // a load of its own would be waited for with vmcnt(0), i.e. together with every tile requested
  // behind it.  Here the waits count the younger loads (wait_vm), and an empty asm statement that
  // "writes" the registers keeps their uses behind the wait.  Lanes without a row of their own load
  // a valid row (the last one; tree row 0) and zero it afterwards.
  int my_parent = 0;
  if constexpr (!BIG) {
    const int32_t* src = h_parent + (h_tree_shared ? 0 : n0) + (tid < M ? tid : 0);  // (one tree for all entries, or each its own)
    asm volatile("global_load_dword %0, %1, off" : "=v"(my_parent) : "v"(src) : "memory");
  }
  uintx4 qraw[8];
  int tree_row;
  bool row_real;
  bool q_upper = false;  // HALF: this row's query head reads the second KV head of the pair
  {
    const int r = row_base + col;
    const int rc = r < R ? r : R - 1;
    const int i = div_G(rc), gi = rc - i * G;
    tree_row = i;
    row_real = r < R;
    if constexpr (HALF) q_upper = 2 * gi >= G;
    const char* qrow = static_cast<const char*>(h_q) + ((int64_t)(n0 + i) * Hq + g * G + gi) * Q_ROW_BYTES + half * 16;
#pragma unroll
    for (int kk = 0; kk < Q_LOADS; ++kk)
      asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(qraw[kk]) : "v"(qrow), "n"(32 * kk) : "memory");
  }
  issue(0);
  if (n_tiles > 1) issue(1);
  // (large trees: a leading tree tile brings one load more; waiting for a multiple of four at most
  // as large as the count waits for no less)
  const int first_tile_loads = 2 * MF_LOADS * (n_tiles < 2 ? n_tiles : 2);
  if constexpr (!BIG) {
    wait_vm(Q_LOADS + first_tile_loads);  // the parent pointers are there (the Q loads and the tiles are younger)
    asm volatile("" : "+v"(my_parent));
  }

  // ---- ancestor bit table: bit j of row i's words is set iff tree row j is on the root path of i.
  // The parent pointers are staged in LDS and the paths are walked there.
  if (!BIG && last_split) {
    if (tid < M) par_lds[tid] = my_parent;
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (tid < M) {
      unsigned w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      for (int j = tid; j >= 0; j = par_lds[j]) {
#pragma unroll
        for (int q = 0; q < 8; ++q) w[q] |= ((j >> 5) == q) ? (1u << (j & 31)) : 0u;
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) anc[tid * 8 + q] = w[q];
    }
  }
  if (tid == 0) exact_flag = 0;

  // ---- Q fragments (B operand of the first product), pre-multiplied by scale * log2(e) so that
  // the scores come out of the MFMA in the log2 domain
  const float c2 = row_real ? h_scale * MF_LOG2E : 0.f;
  wait_vm(first_tile_loads);  // the Q rows are there (the tiles are younger)
  if constexpr (HALF) {
    asm volatile("" : "+v"(qraw[0]), "+v"(qraw[1]), "+v"(qraw[2]), "+v"(qraw[3]));
    const uintx4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {  // the row's 64 elements on its own head's side, zeros on the other
      qraw[4 + kk] = q_upper ? qraw[kk] : zero;
      qraw[kk] = q_upper ? zero : qraw[kk];
    }
  } else {
    asm volatile("" : "+v"(qraw[0]), "+v"(qraw[1]), "+v"(qraw[2]), "+v"(qraw[3]), "+v"(qraw[4]), "+v"(qraw[5]),
                 "+v"(qraw[6]), "+v"(qraw[7]));
  }
  bf16x8 qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    const bf16x8 raw = __builtin_bit_cast(bf16x8, qraw[kk]);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      floatx2 f = {(float)raw[2 * e] * c2, (float)raw[2 * e + 1] * c2};
      bf16x2 hb = __builtin_convertvector(f, bf16x2);
      qf[kk][2 * e] = hb[0];
      qf[kk][2 * e + 1] = hb[1];
    }
  }

  floatx16 acc[4];   // O^T: [d block of 32][16 values]: d = 32 tt + 8 (v / 4) + 4 half + v % 4
  floatx16 negm;     // minus the reference maximum in all 16 slots: start value of a score block
  float m_ref = 0.f, l_sum = 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) negm[v] = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

  // ---- LDS fragments.  Per-lane addresses for block 0 of ring slot 0; a block of slot s, parity b
  // lies s * MF_TILE_BYTES + b * MF_BLOCK_BYTES further (an immediate offset when s is static).
  // K: lane (col, half) reads chunk 2 kk + half of key row col.  V: the transposing read returns, to
  // lane l of a 16-lane group, element l % 4 of the 8-byte pieces addressed by lanes l / 4 + {0, 4,
  // 8, 12} of the group: lane (a = l % 4, j = l / 4) therefore addresses key j of the wanted four at
  // columns 4a .. 4a+3; fragment f = 4 k2 + tt holds the 16 keys of contraction step k2 for the 32
  // output columns of d block tt.
  const int tr_a = lane & 3, tr_j = (lane >> 2) & 3, tr_dh = (lane >> 4) & 1;
  const char* kl[8];
  const char* vl[8][2];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) kl[kk] = &lds_k[0][0] + swz(col, 2 * kk + half);
#pragma unroll
  for (int f = 0; f < 8; ++f)
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int key = 16 * (f >> 2) + 8 * r + 4 * half + tr_j;
      vl[f][r] = &lds_v[0][0] + swz(key, 4 * (f & 3) + 2 * tr_dh + (tr_a >> 1)) + (tr_a & 1) * 8;
    }
  auto ldk = [&](int off, int kk) { return *reinterpret_cast<const bf16x8*>(kl[kk] + off); };
  auto ldv = [&](int off, int f) {
    bf16x8 vf;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const shortx4 got = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(vl[f][r] + off));
      const bf16x4 gb = __builtin_bit_cast(bf16x4, got);
      vf[4 * r + 0] = gb[0];
      vf[4 * r + 1] = gb[1];
      vf[4 * r + 2] = gb[2];
      vf[4 * r + 3] = gb[3];
    }
    return vf;
  };
  // byte offset of block (slot, parity) inside a ring
  auto blk_off = [](int slot, int parity) { return slot * MF_TILE_BYTES + parity * MF_BLOCK_BYTES; };

  // ---- masks of a block's scores: tree keys off the row's root path, keys past the end of the
  // split.  Only the blocks from n_plain on need it (the partial prefix tail and the tree part).
  auto mask_block = [&](int blk, floatx16& S) {
    const int t = blk >> 1;
    if (t >= n_ptiles) {
      const int bbase = (t - n_ptiles) * MF_TILE + (blk & 1) * 32;
      unsigned word;
      if constexpr (BIG) word = bbase < M ? anc[(t % MF_NBUF) * MF_ANC_SLICE + (wave * 32 + col) * 2 + (blk & 1)] : 0u;
      else word = bbase < M ? anc[tree_row * 8 + (bbase >> 5)] : 0u;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int bit = 8 * (v >> 2) + 4 * half + (v & 3);
        S[v] = ((word >> bit) & 1u) ? S[v] : -HS_INF;
      }
    } else {
      const int64_t bbase = k_lo + (int64_t)t * MF_TILE + (blk & 1) * 32;
      if (bbase + 32 > k_hi) {
        const int valid = (int)(k_hi - bbase);  // may be <= 0: the whole block is past the end
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = 8 * (v >> 2) + 4 * half + (v & 3);
          S[v] = key < valid ? S[v] : -HS_INF;
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
  // moves the reference maximum up by delta (>= 0 except at the very first block)
  auto move_reference = [&](float delta) {
    const float alpha = exp2_fast(-delta);
    m_ref += delta;
    l_sum *= alpha;
#pragma unroll
    for (int v = 0; v < 16; ++v) negm[v] = -m_ref;
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tt][v] *= alpha;
  };
  // the first reference of a pass (denominator and accumulators are still zero: nothing to rescale,
  // and no 0 x 2^(-m) = 0 x inf for a first block whose scores are all hugely negative)
  auto set_reference = [&](float mx) {
    m_ref = mx;
#pragma unroll
    for (int v = 0; v < 16; ++v) negm[v] = -mx;
  };
  // the pieces of a window: two exponentials (keys 2j, 2j + 1 of half h of a block), and, one step
  // later, their bf16 pair; the two values also go into two running denominators
  float l0 = 0.f, l1 = 0.f;
  auto exp_pair = [&](const floatx16& S, int h, int j) {
    floatx2 pp = {exp2_fast(S[8 * h + 2 * j]), exp2_fast(S[8 * h + 2 * j + 1])};
    return pp;
  };
  auto pack_pair = [&](const floatx2& pp, uintx4& P, int j) {
    l0 += pp[0];
    l1 += pp[1];
    P[j] = __builtin_bit_cast(unsigned, __builtin_convertvector(pp, bf16x2));
  };
  // half h of a block outside the windows
  auto exp_half = [&](const floatx16& S, int h, uintx4& P) {
#pragma unroll
    for (int j = 0; j < 4; ++j) pack_pair(exp_pair(S, h, j), P, j);
  };

  bf16x8 kf[8], vf[8];  // fragment registers: four of each are alive at any time
  // Score window: S_out = K(block at oq) Q^T, started from -m_ref, in four steps of two matrix
  // instructions.  A step first requests the fragments of the next step (the window's last step:
  // the first two V fragments of the block at ov, whose product window follows), waits for its own,
  // and pairs its matrix instructions with two exponentials of half h of S_in.
  // Wave priority: the two waves of a SIMD compete for its issue slots.  A wave raises its priority
  // for a window (product windows above score windows) and drops it afterwards, so that whichever wave
  // is inside a window, and of two the one in its product window, issues first: 3 % on every shape
  // (paired A/B: -2.4 us of 78 on the 32-layer launch, -3.7 % on the 70B shape).  Toggling around each
  // matrix instruction instead was slower than no priorities at all.
  auto win_qk = [&](int oq, int ov, floatx16& S_out, const floatx16& S_in, int h, uintx4& P) {
    floatx2 pp[4];
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int sN = j + MF_AHEAD;  // the step whose fragments are requested now (4, 5: product window)
      if (sN < 4) {
        kf[2 * sN] = ldk(oq, 2 * sN);
        kf[2 * sN + 1] = ldk(oq, 2 * sN + 1);
      } else {
        vf[2 * (sN - 4)] = ldv(ov, 2 * (sN - 4));
        vf[2 * (sN - 4) + 1] = ldv(ov, 2 * (sN - 4) + 1);
      }
      int pending = 0;  // LDS reads requested after those of step j: K steps count 2, V steps 4
#pragma unroll
      for (int d = 1; d <= MF_AHEAD; ++d) pending += (j + d < 4) ? 2 : 4;
      wait_lds(pending);
      S_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[2 * j], qf[2 * j], j == 0 ? negm : S_out, 0, 0, 0);
      pp[j] = exp_pair(S_in, h, j);
      S_out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[2 * j + 1], qf[2 * j + 1], S_out, 0, 0, 0);
      if (j > 0) pack_pair(pp[j - 1], P, j - 1);
      MF_PIN();
    }
    pack_pair(pp[3], P, 3);
    __builtin_amdgcn_s_setprio(0);
  };
  // Product window: O^T += V^T(block at ov) P^T with P = (P0, P1), same step structure; its last
  // steps request the first K fragments of the block at oq, whose score window follows
  // (with_kf: there is such a block).  with_exp: exponentials of half h of S_in are taken.
  auto win_pv = [&](int ov, int oq, const uintx4& P0, const uintx4& P1, const floatx16& S_in, int h, uintx4& P,
                    auto with_exp, auto with_kf) {
    constexpr bool EXP = decltype(with_exp)::value, KF = decltype(with_kf)::value;
    __builtin_amdgcn_s_setprio(2);
    const bf16x8 b0 = __builtin_bit_cast(bf16x8, P0), b1 = __builtin_bit_cast(bf16x8, P1);
    floatx2 pp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int sN = j + MF_AHEAD;
      if (sN < 4) {
        vf[2 * sN] = ldv(ov, 2 * sN);
        vf[2 * sN + 1] = ldv(ov, 2 * sN + 1);
      } else if (KF) {
        kf[2 * (sN - 4)] = ldk(oq, 2 * (sN - 4));
        kf[2 * (sN - 4) + 1] = ldk(oq, 2 * (sN - 4) + 1);
      }
      if (KF) {
        int pending = 0;
#pragma unroll
        for (int d = 1; d <= MF_AHEAD; ++d) pending += (j + d < 4) ? 4 : 2;
        wait_lds(pending);
      }
      acc[(2 * j) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[2 * j], j < 2 ? b0 : b1, acc[(2 * j) & 3], 0, 0, 0);
      if (EXP) pp[j] = exp_pair(S_in, h, j);
      acc[(2 * j + 1) & 3] =
          __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[2 * j + 1], j < 2 ? b0 : b1, acc[(2 * j + 1) & 3], 0, 0, 0);
      if (EXP && j > 0) pack_pair(pp[j - 1], P, j - 1);
      MF_PIN();
    }
    if (EXP) pack_pair(pp[3], P, 3);
    __builtin_amdgcn_s_setprio(0);
  };
  const std::true_type YES{};
  const std::false_type NO{};

  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // the ancestor table is complete
  first_arrival();
  const int n_blocks = 2 * n_tiles;

  if (wave_active) {
    floatx16 sA, sB;    // scores of the even / odd block of the tile in hand
    uintx4 pa, pb, pc;  // halves of P (bf16 pairs): first half of the even block, a second half, first half of the odd block
    // ---- first block: it always has a visible key (a prefix token, or the root), and its exact
    // maximum is the reference of the whole pass
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kf[kk] = ldk(0, kk);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], kk == 0 ? negm : sA, 0, 0, 0);
    if (n_plain < 1) mask_block(0, sA);
    {
      const float mx = row_max(sA);
#pragma unroll
      for (int v = 0; v < 16; ++v) sA[v] -= mx;
      set_reference(mx);
      exp_half(sA, 0, pa);
    }
#pragma unroll
    for (int kk = 0; kk < 2 * MF_AHEAD; ++kk) kf[kk] = ldk(blk_off(0, 1), kk);
    // ---- one trip per tile t (blocks 2t and 2t + 1, ring slot s = t % 4); the barrier in its
    // middle lets tile t + 1 in
    //   window 1: scores of 2t+1      | second half of 2t
    //   window 2: product of 2t       | first half of 2t+1
    //   window 3: scores of 2t+2      | second half of 2t+1
    //   window 4: product of 2t+1     | first half of 2t+2
    // MASKED: blocks from n_plain on are masked and the tile that is requested may be any tile.
    auto trip = [&](int t, int s, auto masked) {
      constexpr bool MASKED = decltype(masked)::value;
      const int s1 = (s + 1) % MF_NBUF;
      win_qk(blk_off(s, 1), blk_off(s, 0), sB, sA, 1, pb);
      if (MASKED && 2 * t + 1 >= n_plain) mask_block(2 * t + 1, sB);
      if (MASKED) {
        next_arrival(t);
      } else {
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * MF_LOADS) : "memory");
        issue_full(t + 3, (s + 3) % MF_NBUF);
      }
      win_pv(blk_off(s, 0), blk_off(s1, 0), pa, pb, sB, 0, pc, YES, YES);
      win_qk(blk_off(s1, 0), blk_off(s, 1), sA, sB, 1, pb);
      if (MASKED && 2 * t + 2 >= n_plain) mask_block(2 * t + 2, sA);
      win_pv(blk_off(s, 1), blk_off(s1, 1), pc, pb, sA, 0, pa, YES, YES);
    };
    // Four tiles per round with the ring slots spelled out, while they and the tiles they request
    // (up to t + 6) are full prefix tiles: every LDS address is then a register plus an immediate.
    int t = 0;
    for (; t + 6 < n_full; t += 4) {
      trip(t, 0, NO);
      trip(t + 1, 1, NO);
      trip(t + 2, 2, NO);
      trip(t + 3, 3, NO);
    }
    for (; t + 1 < n_tiles; ++t) trip(t, t % MF_NBUF, YES);
    {  // last tile: nothing follows its odd block
      const int s = t % MF_NBUF;
      win_qk(blk_off(s, 1), blk_off(s, 0), sB, sA, 1, pb);
      if (2 * t + 1 >= n_plain) mask_block(2 * t + 1, sB);
      win_pv(blk_off(s, 0), 0, pa, pb, sB, 0, pc, YES, NO);
      exp_half(sB, 1, pb);
#pragma unroll
      for (int f = 0; f < 2 * MF_AHEAD; ++f) vf[f] = ldv(blk_off(s, 1), f);
      win_pv(blk_off(s, 1), 0, pc, pb, sB, 0, pa, NO, NO);
    }
    l_sum = l0 + l1;
  } else {
    // no rows: this wave only moves tiles and meets the barriers
    for (int t = 0; t + 1 < n_tiles; ++t) next_arrival(t);
  }

  // ---- did the fixed reference hold?  (denominator of both half-waves; NaN counts as no)
  float l_tot = l_sum + __shfl_xor(l_sum, 32);
  if (wave_active && __ballot(!(l_tot < MF_SUM_LIMIT)) != 0ull && lane == 0) exact_flag = 1;
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // also: every LDS read of the pass is done
  if (exact_flag != 0) {
    // ---- exact path (rare): the pass again, one block at a time, the reference following the
    // running maximum: classic online softmax, no overlap between the steps
    m_ref = 0.f;
    l_sum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) negm[v] = 0.f;
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tt][v] = 0.f;
    issue(0);
    if (n_tiles > 1) issue(1);
    first_arrival();
    for (int blk = 0; blk < n_blocks; ++blk) {
      // the barrier of next_arrival also keeps any wave from reading tile t + 1 before all of it is there
      if ((blk & 1) && blk + 1 < n_blocks) next_arrival(blk >> 1);
      if (!wave_active) continue;
      const int off = blk_off((blk >> 1) % MF_NBUF, blk & 1);
      floatx16 S;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ldk(off, kk), qf[kk], kk == 0 ? negm : S, 0, 0, 0);
      if (blk >= n_plain) mask_block(blk, S);
      const float mx = row_max(S);
      if (blk == 0 || __ballot(mx > 0.f) != 0ull) {
        const float delta = (blk == 0 || mx > 0.f) ? mx : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) S[v] -= delta;
        if (blk == 0) set_reference(delta);
        else move_reference(delta);
      }
      uintx4 P0, P1;
      l0 = 0.f;
      l1 = 0.f;
      exp_half(S, 0, P0);
      exp_half(S, 1, P1);
      l_sum += l0 + l1;
      const bf16x8 b0 = __builtin_bit_cast(bf16x8, P0), b1 = __builtin_bit_cast(bf16x8, P1);
#pragma unroll
      for (int f = 0; f < 8; ++f)
        acc[f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ldv(off, f), f < 4 ? b0 : b1, acc[f & 3], 0, 0, 0);
    }
    l_tot = l_sum + __shfl_xor(l_sum, 32);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  }
  if (!wave_active) return;

  if (n_sp == 1) {
    // ---- results, sequence with a single split: normalised rows go out as bf16.  Each wave turns its
    // 32 x 128 block around in LDS (the tile ring is free: every wave has passed the last barrier),
    // so that a lane stores 16 contiguous bytes and a store instruction covers four whole rows.
    constexpr int ST_ROW = MF_ROW_BYTES + 16;  // padded row: the 8-byte writes of 16 rows spread over all banks
    char* stage = wave < 4 ? lds_k[wave] : lds_v[wave - 4];
    const float inv = 1.f / l_tot;
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int d0 = 32 * tt + 8 * b + 4 * half;
        floatx2 f01 = {acc[tt][4 * b] * inv, acc[tt][4 * b + 1] * inv};
        floatx2 f23 = {acc[tt][4 * b + 2] * inv, acc[tt][4 * b + 3] * inv};
        uint2 pk;
        pk.x = __builtin_bit_cast(unsigned, __builtin_convertvector(f01, bf16x2));
        pk.y = __builtin_bit_cast(unsigned, __builtin_convertvector(f23, bf16x2));
        *reinterpret_cast<uint2*>(stage + col * ST_ROW + d0 * 2) = pk;
      }
    const int r = row_base + col;
    if (h_lse && half == 0 && r < R) {
      const int i = div_G(r), gi = r - i * G;
      h_lse[(int64_t)(n0 + i) * Hq + g * G + gi] = (m_ref + __log2f(l_tot)) * MF_LN2;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave's staging writes are in LDS
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int row_l = 4 * j + (lane >> 4), chunk = lane & 15;
      const int ro = row_base + row_l;
      const int i = div_G(ro < R ? ro : 0), gi = ro - i * G;
      // (HALF: the eight chunks on the side of the row's own KV head are its 64 output elements)
      if (ro < R && (!HALF || (chunk >> 3) == (2 * gi >= G ? 1 : 0))) {
        const uint4 val = *reinterpret_cast<const uint4*>(stage + row_l * ST_ROW + chunk * 16);
        char* dst = static_cast<char*>(h_o) + ((int64_t)(n0 + i) * Hq + g * G + gi) * Q_ROW_BYTES + (HALF ? chunk & 7 : chunk) * 16;
        // non-temporal: the rows start their way to memory now instead of waiting in L2 for the
        // write-back at the end of the kernel, when every workgroup's rows would go at once
        __builtin_nontemporal_store(__builtin_bit_cast(uintx4, val), reinterpret_cast<uintx4*>(dst));
      }
    }
  } else {
    // ---- this split's partial record: unnormalised accumulators, reference maximum, denominator
    const int r = row_base + col;
    if (r < R) {
      const int i = div_G(r), gi = r - i * G;
      const int64_t row = (int64_t)(n0 + i) * Hq + g * G + gi;
      constexpr int REC_D = HALF ? 64 : 128;  // a record: o[REC_D], m, l, two pad floats
      float* rec = h_part + (row * h_sp_max + sp) * (REC_D + ATTN_REC_PAD);
      const int own = 2 * gi >= G ? 1 : 0;  // HALF: the side of the row's own KV head
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int d0 = 32 * tt + 8 * b + 4 * half;
          float4 f = {acc[tt][4 * b], acc[tt][4 * b + 1], acc[tt][4 * b + 2], acc[tt][4 * b + 3]};
          if (!HALF) *reinterpret_cast<float4*>(rec + d0) = f;
          else if ((tt >> 1) == own) *reinterpret_cast<float4*>(rec + (d0 & 63)) = f;
        }
      if (half == 0) {
        rec[REC_D] = m_ref * MF_LN2;
        rec[REC_D + 1] = l_tot;
      }
    }
  }
}

// `ev_start` / `ev_stop` (may be NULL): HIP events attached to this dispatch; the runtime stamps them
// when the kernel begins and ends, so their elapsed time is the kernel's own duration.
hs_status attn_mfma_launch(const AttnArgs& a, int max_tree_rows, hipStream_t stream, hipEvent_t ev_start,
                           hipEvent_t ev_stop) {
  const int n_rg_max = (a.G * max_tree_rows + MF_ROWS - 1) / MF_ROWS;
  dim3 grid((unsigned)(a.Hkv * n_rg_max * a.sp_max), (unsigned)a.B);
  if (a.n_tbl > 0) grid = dim3((unsigned)a.n_items, 1u);
  const bool once = n_rg_max == 1;  // every (sequence, head) is one row group: its keys have one reader
  const bool big = max_tree_rows > MF_MAX_M;
  const dim3 block(MF_THREADS);
  if (big) {
    if (a.anc_tiles == nullptr) return fail(HS_ERR_WORKSPACE, "tree attention: trees of %d rows need the ancestor table", max_tree_rows);
    const dim3 tgrid((unsigned)((max_tree_rows + 255) / 256), (unsigned)(a.tree_shared ? 1 : a.B));
    hipLaunchKernelGGL(k_anc_tiles, tgrid, dim3(256), 0, stream, a.parent, a.node_offsets, const_cast<unsigned*>(a.anc_tiles));
    hs_status r = launch_status("tree attention (ancestor table)");
    if (r != HS_OK) return r;
  }
#define MF_LAUNCH(PAGED, ONCE, BIG)                                                                                        \
  do {                                                                                                                     \
    if (a.half)                                                                                                            \
      hipExtLaunchKernelGGL((k_attn_mfma<PAGED, ONCE, BIG, true>), grid, block, 0, stream, ev_start, ev_stop, 0, a, n_rg_max);  \
    else                                                                                                                   \
      hipExtLaunchKernelGGL((k_attn_mfma<PAGED, ONCE, BIG, false>), grid, block, 0, stream, ev_start, ev_stop, 0, a, n_rg_max); \
  } while (0)
  if (a.block_table != nullptr) {
    if (big) MF_LAUNCH(true, false, true);
    else if (once) MF_LAUNCH(true, true, false);
    else MF_LAUNCH(true, false, false);
  } else {
    if (big) MF_LAUNCH(false, false, true);
    else if (once) MF_LAUNCH(false, true, false);
    else MF_LAUNCH(false, false, false);
  }
#undef MF_LAUNCH
  return launch_status("tree attention (mfma)");
}

}  // namespace hs
