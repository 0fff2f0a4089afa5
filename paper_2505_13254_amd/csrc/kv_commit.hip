// hs_kv_commit: the accepted path joins the KV cache (Section 2.1: what an accepted path means for
// the context of the next step; rows of rejected nodes go nowhere).
//
// Per sequence the K/V rows of the tree's root and of the accepted rows, in path order, are copied
// behind the used part of the sequence's cache region and the used length grows by their number.
// A copy of a few kilobytes per sequence: one workgroup per sequence, 16 bytes per lane and step.
#include "hs_common.h"

namespace hs {

constexpr int KC_THREADS = 256;

// block_table == NULL: sequence s owns tokens cache_offsets[s] .. cache_offsets[s+1] of the caches.
// Otherwise the caches are pools of pages of `page_tokens` tokens and token t of sequence s lives in
// page block_table[s * max_blocks + t / page_tokens].
__global__ __launch_bounds__(KC_THREADS) void k_kv_commit(const char* __restrict__ k_tree,
                                                          const char* __restrict__ v_tree,
                                                          const int32_t* __restrict__ node_offsets,
                                                          const int32_t* __restrict__ accept_path,
                                                          const int32_t* __restrict__ accept_len, int max_depth,
                                                          char* __restrict__ k_cache, char* __restrict__ v_cache,
                                                          const int64_t* __restrict__ cache_offsets,
                                                          const int32_t* __restrict__ block_table, int max_blocks,
                                                          int page_tokens, int64_t* __restrict__ cache_lens,
                                                          int row_bytes) {
  const int s = blockIdx.x, tid = threadIdx.x;
  const int n0 = node_offsets[s];
  const int M = node_offsets[s + 1] - n0;
  if (M <= 0) return;
  const bool paged = block_table != nullptr;
  const int64_t c0 = paged ? 0 : cache_offsets[s];
  const int64_t used = cache_lens[s];
  const int64_t room = (paged ? (int64_t)max_blocks * page_tokens : cache_offsets[s + 1] - c0) - used;
  int n_acc = accept_len[s];
  n_acc = n_acc < 0 ? 0 : (n_acc > max_depth ? max_depth : n_acc);
  int64_t rows = 1 + n_acc;  // the root, then the accepted rows
  rows = rows > room ? (room > 0 ? room : 0) : rows;
  const int chunks = row_bytes / 16;  // 16-byte pieces of a token's K (or V) row
  for (int64_t e = tid; e < rows * chunks; e += KC_THREADS) {
    const int t = (int)(e / chunks), c = (int)(e - (int64_t)t * chunks);
    int r = t == 0 ? 0 : accept_path[(int64_t)s * max_depth + t - 1];
    r = r < 0 ? 0 : (r >= M ? M - 1 : r);  // (a path entry outside the tree would be a caller's error)
    const int64_t src = ((int64_t)(n0 + r)) * row_bytes + c * 16;
    int64_t pos = c0 + used + t;  // token position in the caches
    if (paged) {
      const int64_t tok = used + t;
      pos = (int64_t)block_table[(int64_t)s * max_blocks + tok / page_tokens] * page_tokens + tok % page_tokens;
    }
    const int64_t dst = pos * row_bytes + c * 16;
    *reinterpret_cast<uint4*>(k_cache + dst) = *reinterpret_cast<const uint4*>(k_tree + src);
    *reinterpret_cast<uint4*>(v_cache + dst) = *reinterpret_cast<const uint4*>(v_tree + src);
  }
  __syncthreads();  // every thread has read the old length
  if (tid == 0) cache_lens[s] = used + rows;
}

}  // namespace hs

using namespace hs;

static hs_status kv_commit_impl(const void* k_tree, const void* v_tree, const int32_t* node_offsets,
                                const int32_t* accept_path, const int32_t* accept_len, int32_t max_depth, void* k_cache,
                                void* v_cache, const int64_t* cache_offsets, const int32_t* block_table,
                                int32_t max_blocks, int32_t page_tokens, int64_t* cache_lens, int32_t B, int32_t Hkv,
                                int32_t D, hs_dtype dt, hs_stream stream) {
  HS_REQUIRE(B >= 0 && Hkv >= 1 && D >= 1 && max_depth >= 1, HS_ERR_SHAPE, "hs_kv_commit: B=%d Hkv=%d D=%d max_depth=%d",
             B, Hkv, D, max_depth);
  HS_REQUIRE(dt == HS_F32 || dt == HS_BF16, HS_ERR_SHAPE, "hs_kv_commit: unknown dtype %d", (int)dt);
  const int64_t row_bytes = (int64_t)Hkv * D * (dt == HS_F32 ? 4 : 2);
  HS_REQUIRE(row_bytes % 16 == 0 && row_bytes < ((int64_t)1 << 30), HS_ERR_UNSUPPORTED,
             "hs_kv_commit: a token's K row (%lld bytes) must be a multiple of 16 bytes", (long long)row_bytes);
  if (B == 0) return HS_OK;
  HS_REQUIRE(k_tree && v_tree && node_offsets && accept_path && accept_len && k_cache && v_cache &&
                 (cache_offsets || block_table) && cache_lens,
             HS_ERR_NULL, "hs_kv_commit: NULL argument");
  auto aligned16 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  HS_REQUIRE(aligned16(k_tree) && aligned16(v_tree) && aligned16(k_cache) && aligned16(v_cache), HS_ERR_UNSUPPORTED,
             "hs_kv_commit: tensors must be 16-byte aligned");
  hipLaunchKernelGGL(k_kv_commit, dim3((unsigned)B), dim3(KC_THREADS), 0, static_cast<hipStream_t>(stream),
                     static_cast<const char*>(k_tree), static_cast<const char*>(v_tree), node_offsets, accept_path,
                     accept_len, max_depth, static_cast<char*>(k_cache), static_cast<char*>(v_cache), cache_offsets,
                     block_table, max_blocks, page_tokens, cache_lens, (int)row_bytes);
  return launch_status("kv commit");
}

extern "C" hs_status hs_kv_commit(const void* k_tree, const void* v_tree, const int32_t* node_offsets,
                                  const int32_t* accept_path, const int32_t* accept_len, int32_t max_depth,
                                  void* k_cache, void* v_cache, const int64_t* cache_offsets, int64_t* cache_lens,
                                  int32_t B, int32_t Hkv, int32_t D, hs_dtype dt, hs_stream stream) {
  clear_error();
  HS_REQUIRE(B == 0 || cache_offsets, HS_ERR_NULL, "hs_kv_commit: NULL cache_offsets");
  return kv_commit_impl(k_tree, v_tree, node_offsets, accept_path, accept_len, max_depth, k_cache, v_cache,
                        cache_offsets, nullptr, 0, 1, cache_lens, B, Hkv, D, dt, stream);
}

extern "C" hs_status hs_kv_commit_paged(const void* k_tree, const void* v_tree, const int32_t* node_offsets,
                                        const int32_t* accept_path, const int32_t* accept_len, int32_t max_depth,
                                        void* k_pages, void* v_pages, const int32_t* block_table, int32_t max_blocks,
                                        int32_t page_tokens, int64_t* cache_lens, int32_t B, int32_t Hkv, int32_t D,
                                        hs_dtype dt, hs_stream stream) {
  clear_error();
  HS_REQUIRE(page_tokens >= 1 && max_blocks >= 0, HS_ERR_SHAPE, "hs_kv_commit_paged: page_tokens=%d max_blocks=%d",
             page_tokens, max_blocks);
  HS_REQUIRE(B == 0 || block_table, HS_ERR_NULL, "hs_kv_commit_paged: NULL block_table");
  return kv_commit_impl(k_tree, v_tree, node_offsets, accept_path, accept_len, max_depth, k_pages, v_pages, nullptr,
                        block_table, max_blocks, page_tokens, cache_lens, B, Hkv, D, dt, stream);
}
