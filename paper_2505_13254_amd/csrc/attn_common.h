// Shared pieces of the tree-attention kernels (internal).
//
// Work decomposition, plain launches (float32 / any-shape kernel; matrix-core kernel when a batch
// has more sequences than the table below holds): grid.y = sequence, grid.x enumerates (key split, row block,
// KV head) of that sequence; workgroups whose indices fall outside their sequence's extent exit at
// once.  The prefix of sequence s is cut into n_sp = max(1, ceil(L_s / split_len)) splits; the last
// split also handles the tree rows themselves (the masked part).  Rows of one KV head g are
// r = i * G + gi for tree row i and group member gi (query head h = g * G + gi).
//
// Partial results (only when some sequence has more than one split): one record of D + 4 floats per
// (node, head, split): unnormalised output o[D], reference maximum m (in units of the scaled score),
// denominator l (relative to m) and two pad floats (records stay 16-byte aligned);
// slot = (node_global * Hq + h) * sp_max + split.
#pragma once
#include <cstddef>

#include "hs_common.h"

namespace hs {

typedef unsigned short bf16_t;  // raw bfloat16 bits

constexpr int ATTN_REC_PAD = 4;  // floats after o[D] in a partial record: m, l, pad, pad

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __builtin_bit_cast(float, (unsigned)b << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest, ties to even
  unsigned u = __builtin_bit_cast(unsigned, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T>
__device__ __forceinline__ float load_elem(const T* p);
template <>
__device__ __forceinline__ float load_elem<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_elem<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }

template <typename T>
__device__ __forceinline__ void store_elem(T* p, float v);
template <>
__device__ __forceinline__ void store_elem<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_elem<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// One sequence of the launch as the host planned it (work-list launches).  Its work items are
// numbered first_item + (split * n_rg + row_group) * Hkv + kv_head; entries are listed by falling
// cost of an item, so that the hardware's in-order dispatch starts the long items first.  The
// prefix is cut into n_sp splits of tiles_per_split 64-key tiles (the last one takes the rest and
// the tree rows).
struct SeqEntry {
  int first_item;
  int n0;               // first tree row of the sequence (global row number)
  int M;                // tree rows
  int L;                // prefix tokens
  long long p0;         // first prefix token (global); paged caches: first entry of the sequence's block-table row
  int tiles_per_split;
  short n_sp, n_rg;
};
static_assert(sizeof(SeqEntry) == 32, "eight dwords, fetched as two 16-byte loads per lane");
constexpr int ATTN_TBL = 96;  // entries that fit the kernel-argument segment next to the rest

struct AttnArgs {
  const void* q;
  const void* k_prefix;
  const void* v_prefix;
  const void* k_tree;
  const void* v_tree;
  const int32_t* parent;
  int tree_shared;  // 1: `parent` holds one tree that every batch entry uses (all entries have its row count)
  const int32_t* node_offsets;
  const int64_t* prefix_offsets;
  const int64_t* prefix_lens;  // used tokens of each sequence's prefix region; NULL: the whole region
  const int32_t* block_table;  // paged caches: page of each 64-token block, row s at s * max_blocks; else NULL
  int max_blocks;
  int B, Hq, Hkv, G;
  int half;        // 1 (matrix-core kernel, D = 64): Hkv counts pairs of KV heads and G the 2 Hq / Hkv query heads of a pair
  float scale;
  int split_len;   // prefix tokens per split (multiple of 64)
  int sp_max;      // largest split count of any sequence; 1 = results are written directly
  int n_rb_max;    // largest row-block count of any sequence (generic kernel)
  void* o;
  float* lse;
  float* part;
  const unsigned* anc_tiles;  // ancestor table of large trees (matrix-core kernel), in the workspace; else NULL
  int n_tbl;       // > 0: work-list launch (1-D grid over the items of tbl[0 .. n_tbl)); 0: grid.y = sequence
  int n_items;
  alignas(16) SeqEntry tbl[ATTN_TBL];  // (lanes fetch their entry with 16-byte loads)
};
static_assert(offsetof(AttnArgs, tbl) % 16 == 0, "16-byte loads of the table entries");

// Prefix length of sequence s (plain launches read it on the device).
__device__ __forceinline__ int64_t prefix_len_of(const AttnArgs& a, int s) {
  return a.prefix_lens != nullptr ? a.prefix_lens[s] : a.prefix_offsets[s + 1] - a.prefix_offsets[s];
}

__host__ __device__ __forceinline__ int splits_of(int64_t L, int split_len) {
  int n = (int)((L + split_len - 1) / split_len);
  return n < 1 ? 1 : n;
}

// Is tree row j on the root path of tree row i (j == i or an ancestor)?  par: local parents.
__device__ __forceinline__ bool on_root_path(const int* par, int i, int j) {
  int a = i;
  while (a > j) a = par[a];
  return a == j;
}

}  // namespace hs
