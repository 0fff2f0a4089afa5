/*
 * heterospec.h - C ABI of the MI355X (gfx950) tree-verification library.
 *
 * One speculative-decoding verification step, as four asynchronous calls:
 *
 *   hs_draft_entropy_topk   vocabulary-wide softmax of draft logits, Top-K tokens with their
 *                           log-probabilities, Top-K entropy          (Section 4.1 Eq. 1; Section 2.2 Expansion)
 *   hs_tree_prune           cumulative-confidence reranking / pruning of the draft tree
 *                                                                      (Section 2.2 Reranking; Section 4.3 Top-N Pruning)
 *   hs_tree_attention       tree-masked attention of the kept rows over the prefix KV cache
 *                                                                      (Section 2.2: tree-mask attention)
 *   hs_verify_accept        greedy or stochastic accept walk           (Section 2.1 acceptance rule)
 *
 * and, around them, the device-side pieces of the adaptive step (no host round trip inside):
 *
 *   hs_tree_expand          one level of Top-K growth of the draft tree from the Top-K results of
 *                           the rows expanded last                     (Section 2.2 Expansion; Section 4.3
 *                                                                       Dynamic Extended Drafting)
 *   hs_adaptive_control     cumulative Top-K entropy of the operational path, its entropy bin, and
 *                           the depth extension and node budget of that bin (Section 4.1 Eq. 1; 4.2; 4.3)
 *   hs_tree_prune_counted   hs_tree_prune on trees stored with spare capacity
 *   hs_kv_commit            the accepted path's K/V rows join the KV cache (Section 2.1: decoding
 *                           resumes behind the last accepted token)
 *   hs_tree_attention_lens  hs_tree_attention on caches stored with spare capacity
 *   hs_tree_attention_paged, hs_kv_commit_paged   the same two on caches made of pages
 *   hs_tree_attention_shared_tree   hs_tree_attention on batch entries that all verify one tree
 *
 * Conventions that hold for every call
 *   - Pointers are DEVICE pointers unless the parameter name starts with host_.  The caller owns
 *     every buffer; the library allocates and frees nothing, and keeps nothing after a call.
 *   - Scratch memory comes from the caller: `workspace` must hold at least the bytes the matching
 *     *_workspace query returns for the same shape arguments and must be 256-byte aligned.
 *     A smaller or NULL workspace (when the query is non-zero) gives HS_ERR_WORKSPACE.
 *   - A call only enqueues kernels on `stream` (a hipStream_t; NULL = the default stream) and
 *     returns.  Results are valid once the caller has synchronised that stream.  No call
 *     synchronises the device, and none records a memset, so calls may be captured in a HIP graph.
 *   - Host-visible arguments are validated before anything is launched; on any error nothing is
 *     launched and hs_last_error() describes the problem.  Device-side data is trusted:
 *     parent[i] < i, offsets non-decreasing, sibling tokens distinct, no NaN logits.
 *   - All arrays are dense row-major.  Ragged batches are packed back to back and described by
 *     offset arrays with B+1 entries (first 0, last the total).
 *   - Same inputs give bit-identical outputs (no floating-point atomics).
 *   - Trees: row 0 of each sequence is the root (the last committed token), parent[root] = -1,
 *     parents are LOCAL indices within the sequence and parent[i] < i.
 *   - Trees with spare capacity: where a call takes node_counts [B], sequence s uses rows
 *     node_offsets[s] .. node_offsets[s] + node_counts[s] - 1 and the rows up to node_offsets[s+1]
 *     are unused capacity; node_counts == NULL means that every row is used.
 */
#ifndef HETEROSPEC_H_
#define HETEROSPEC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HS_OK = 0,
  HS_ERR_NULL = 1,        /* a required pointer is NULL                                  */
  HS_ERR_SHAPE = 2,       /* a size is negative, zero where it may not be, or inconsistent */
  HS_ERR_UNSUPPORTED = 3, /* a valid request this build has no kernel for                */
  HS_ERR_WORKSPACE = 4,   /* workspace NULL, misaligned or smaller than the query says   */
  HS_ERR_RUNTIME = 5      /* the HIP runtime refused a launch                            */
} hs_status;

typedef enum { HS_F32 = 0, HS_BF16 = 1 } hs_dtype;

typedef enum {
  HS_ACCEPT_GREEDY = 0,               /* temperature 0: follow the target's argmax                       */
  HS_ACCEPT_STOCHASTIC = 1,           /* accept x with prob min(1, p(x)/p_hat(x)); residual on rejection */
  HS_ACCEPT_STOCHASTIC_POINTMASS = 2  /* candidates treated as point-mass proposals: accept with p(x)    */
} hs_accept_mode;

typedef enum {
  HS_PSTAR_CUMULATIVE = 0, /* operational path = deepest-level node with the largest cumulative value */
  HS_PSTAR_LOCAL = 1       /* ... with the largest confidence of its own (final) token                 */
} hs_pstar_mode;

typedef void* hs_stream; /* a hipStream_t */

#define HS_MAX_TOPK 64
#define HS_MAX_CHILDREN 256 /* children of one node that the sampling accept rules try (see hs_verify_accept) */

/* Static description of a status code; never NULL, never freed. */
const char* hs_status_string(hs_status st);
/* Detail of the last error raised on the calling thread ("" if none). Valid until the next call
 * on this thread. */
const char* hs_last_error(void);
/* Library version, "major.minor". */
const char* hs_version(void);

/* ------------------------------------------------------------------------------------------------
 * hs_draft_entropy_topk  (Section 4.1, Eq. 1: the per-position term of the cumulative Top-K
 * entropy; Section 2.2, Expansion: Top-k tokens and their confidences c_j)
 *
 * For each of R rows x of draft logits over V tokens, with y = x / temperature:
 *   topk_idx [R,K]  int32  indices of the K largest logits, largest first; equal logits are
 *                          ordered by ascending index (decided on the raw float32 values)
 *   topk_logp[R,K]  float  log softmax(y) at those indices  (log of the confidence c)
 *   ent_topk [R]    float  -sum_i pt_i ln pt_i over the Top-K probabilities renormalised to sum 1
 *   ent_full [R]    float  entropy of softmax(y) over the whole vocabulary      (may be NULL)
 *   lse      [R]    float  ln sum_v exp(y_v)                                    (may be NULL)
 * logits: float32, row r starts at logits + r*row_stride (row_stride >= V, in elements).
 * -inf logits are allowed (probability 0).  Natural logarithms.
 * Requires 1 <= K <= min(V, HS_MAX_TOPK), temperature > 0, 0 <= R <= 65535 (R == 0 is a no-op;
 * more rows: HS_ERR_UNSUPPORTED, split the call).
 */
size_t hs_draft_entropy_topk_workspace(int32_t R, int32_t V, int32_t K);
hs_status hs_draft_entropy_topk(const float* logits, int64_t row_stride, int32_t R, int32_t V,
                                int32_t K, float temperature,
                                int32_t* topk_idx, float* topk_logp, float* ent_topk,
                                float* ent_full, float* lse,
                                void* workspace, size_t workspace_bytes, hs_stream stream);

/* hs_draft_entropy_topk_rows: the same, with the rows picked out of a larger array: result row r
 * (0 <= r < R) comes from logits row row_index[r] (device, int32 [R]; the rows a level-by-level
 * expansion wants next, as hs_tree_expand lists them in frontier_rows).  A negative entry leaves
 * the results of row r as they are.  The entries are trusted, like all device-side data. */
hs_status hs_draft_entropy_topk_rows(const float* logits, int64_t row_stride, const int32_t* row_index,
                                     int32_t R, int32_t V, int32_t K, float temperature,
                                     int32_t* topk_idx, float* topk_logp, float* ent_topk,
                                     float* ent_full, float* lse,
                                     void* workspace, size_t workspace_bytes, hs_stream stream);

/* hs_draft_entropy_topk_fused: hs_draft_entropy_topk / _rows (row_index may be NULL: every row) in ONE
 * kernel launch whatever the row count.  Few rows are cut into slices so that the whole chip reads
 * them; the plain calls then merge a row's slices with a second launch, this one lets the workgroup
 * that finishes a row's last slice do it, found by a counter per row at the start of the workspace.
 * The counters must be zero when the call starts and are zero again when it has completed, so the
 * workspace must be PREPARED: cleared once by hs_workspace_prepare and used since then only by
 * hs_draft_entropy_topk_fused calls that ran to completion (any number of them, of any shape the
 * workspace is large enough for).  Any other use of the memory, the plain calls included, ends that:
 * prepare it again.  On an unprepared workspace the results are undefined (no fault, no hang).
 * Same outputs as the plain calls, bit for bit.  Workspace size: hs_draft_entropy_topk_workspace. */
hs_status hs_draft_entropy_topk_fused(const float* logits, int64_t row_stride, const int32_t* row_index,
                                      int32_t R, int32_t V, int32_t K, float temperature,
                                      int32_t* topk_idx, float* topk_logp, float* ent_topk,
                                      float* ent_full, float* lse,
                                      void* workspace, size_t workspace_bytes, hs_stream stream);

/* hs_workspace_prepare: clears `workspace_bytes` bytes (a multiple of 16) of a 256-byte aligned
 * workspace with a fill kernel on `stream` (no memset: the call may be captured in a HIP graph).
 * What hs_draft_entropy_topk_fused asks of its workspace. */
hs_status hs_workspace_prepare(void* workspace, size_t workspace_bytes, hs_stream stream);

/* ------------------------------------------------------------------------------------------------
 * hs_tree_prune  (Section 2.2: the value of node i is the product of the confidences on the path
 * root -> i, and the best nodes by value form the verified subtree; Section 4.3: the node budget
 * N' varies per step)
 *
 * B candidate trees packed by node_offsets [B+1]; NN = node_offsets[B] (passed by the caller).
 * Per sequence s, with n = its node count and local indices:
 *   depth[0] = 0, depth[i] = depth[parent[i]] + 1
 *   cumlogp[0] = 0, cumlogp[i] = fl32(cumlogp[parent[i]] + min(logc[i], 0))   (one float add per node)
 *   node i >= 1 survives iff, for i and each of its ancestors j: depth[j] <= d_max[s] and
 *   cumlogp[j] >= theta[s]; and, when max_nodes[s] > 0 and more than max_nodes[s] nodes survive
 *   that test, i is among the first max_nodes[s] of them ordered by (cumlogp descending, index
 *   ascending).  The root always survives.  A filter is switched off by d_max = INT32_MAX,
 *   theta = -inf, max_nodes = 0.
 * Outputs: depth, cumlogp, keep (1 = survives) are indexed like the input [NN];
 *   out_offsets [B+1] packs the surviving rows; out_src [NN'] is each surviving row's LOCAL index in
 *   its candidate tree (ascending); out_parent [NN'] its parent as a LOCAL index among the surviving
 *   rows (-1 for the root).  out_src / out_parent must have room for NN entries.
 *   The entries of out_src / out_parent past the last surviving row (NN' .. NN-1) are set to 0: rows
 *   that hang off a root and repeat it, so that a consumer sized for a fixed node budget (a captured
 *   graph, say) reads a valid tree even when fewer nodes survive.
 * logc[i] is the log-confidence of node i (ignored for roots).  An empty sequence (n = 0) emits nothing.
 */
size_t hs_tree_prune_workspace(int32_t B, int32_t NN);
hs_status hs_tree_prune(const int32_t* parent, const float* logc, const int32_t* node_offsets,
                        int32_t B, int32_t NN,
                        const int32_t* d_max, const float* theta, const int32_t* max_nodes,
                        int32_t* depth, float* cumlogp, uint8_t* keep,
                        int32_t* out_offsets, int32_t* out_src, int32_t* out_parent,
                        void* workspace, size_t workspace_bytes, hs_stream stream);

/* hs_tree_prune_static: hs_tree_prune without a workspace argument, for callers that cannot allocate
 * device memory and have no buffer to lend: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The scratch is a device array inside the library (528 KiB per
 * GPU, held until the process ends); the call allocates and frees nothing.  Limits: B <=
 * HS_PRUNE_STATIC_MAX_SEQS and NN <= HS_PRUNE_STATIC_MAX_NODES, beyond them HS_ERR_UNSUPPORTED
 * (nothing launched).  Every call on a GPU uses that GPU's one array: calls that may overlap on
 * one GPU (different streams, different threads) race; calls on one stream are ordered.  The
 * first call on a device looks the array's address up (hipGetSymbolAddress), so make it outside a
 * stream capture.  Arguments, outputs and results are those of hs_tree_prune, bit for bit. */
#define HS_PRUNE_STATIC_MAX_SEQS 4096
#define HS_PRUNE_STATIC_MAX_NODES 65536
hs_status hs_tree_prune_static(const int32_t* parent, const float* logc, const int32_t* node_offsets,
                               int32_t B, int32_t NN,
                               const int32_t* d_max, const float* theta, const int32_t* max_nodes,
                               int32_t* depth, float* cumlogp, uint8_t* keep,
                               int32_t* out_offsets, int32_t* out_src, int32_t* out_parent,
                               hs_stream stream);

/* ------------------------------------------------------------------------------------------------
 * hs_tree_attention  (Section 2.2: the pruned tree is verified in one pass with tree-mask
 * attention)
 *
 * For sequence s, tree row i, query head h (KV head g = h / (Hq/Hkv)):
 *   o[i,h,:] = softmax_j( scale * <q[i,h,:], k[j,g,:]> ) . v[j,g,:]
 * over j = every prefix token of s, and every tree row of s on the root path of i (the root, the
 * ancestors of i, and i itself).  One attention layer; no positional encoding is applied.
 *   q [NN,Hq,D], o [NN,Hq,D]; k_prefix, v_prefix [total_prefix,Hkv,D]; k_tree, v_tree [NN,Hkv,D]
 *   all of element type dt (HS_BF16: bfloat16 storage, float32 softmax state and accumulation,
 *   output rounded once; HS_F32: float32 throughout).
 *   parent [NN] int32 local indices; node_offsets [B+1] int32; prefix_offsets [B+1] int64 (token units).
 *   host_node_offsets / host_prefix_offsets: HOST copies of the two offset arrays, read during the
 *   call to size the launch; they must equal the device arrays.  The host copies (and, in the _lens
 *   and _paged calls, host_prefix_lens) are what the launch is planned from: row counts, prefix
 *   lengths and key splits are fixed when the call returns, and a launch that was captured into a HIP
 *   graph keeps them on every replay.  Replaying it after the lengths have changed on the device (after
 *   hs_kv_commit, say) attends to the lengths of the capture; capture one graph per shape instead.
 *   lse [NN,Hq] float: ln of the softmax denominator (of the scaled scores); may be NULL.
 * Requires Hq % Hkv == 0, D in {64, 128}, at most 1024 tree rows per sequence.
 * bfloat16 runs on the matrix cores (D = 64: with an even number of KV heads, which the kernel takes in
 * pairs); when a sequence has more than 256 tree rows, a
 * small launch ahead of the attention kernel writes the trees' ancestor table into the workspace
 * (128 bytes per tree row, included in the workspace query).
 * Workspace: one partial record of D + 4 floats per (tree row, query head, key split); the query
 * returns the bound for min(64, total_prefix / 128 + 1) splits, more than any plan of that batch
 * uses (a batch whose keys are not cut needs none; hs_tree_attention_plan tells what a given batch needs).  The host keeps the last few plans per calling thread (a model's layers share theirs); the
 * calls stay re-entrant across threads and hold no device state.
 */
size_t hs_tree_attention_workspace(int32_t B, int32_t NN, int64_t total_prefix,
                                   int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt);
hs_status hs_tree_attention(const void* q, const void* k_prefix, const void* v_prefix,
                            const void* k_tree, const void* v_tree,
                            const int32_t* parent, const int32_t* node_offsets,
                            const int64_t* prefix_offsets,
                            const int32_t* host_node_offsets, const int64_t* host_prefix_offsets,
                            int32_t B, int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt, float scale,
                            void* o, float* lse,
                            void* workspace, size_t workspace_bytes, hs_stream stream);

/* hs_tree_attention_lens: hs_tree_attention on KV caches stored with spare capacity (what
 * hs_kv_commit grows): sequence s owns the token range prefix_offsets[s] .. prefix_offsets[s+1] of
 * k_prefix / v_prefix and prefix_lens[s] (int64 [B], device; host_prefix_lens the same on the host)
 * of it are in use.  Both NULL: the whole range, i.e. hs_tree_attention.  The workspace query takes
 * the total capacity as total_prefix. */
hs_status hs_tree_attention_lens(const void* q, const void* k_prefix, const void* v_prefix,
                                 const void* k_tree, const void* v_tree,
                                 const int32_t* parent, const int32_t* node_offsets,
                                 const int64_t* prefix_offsets,
                                 const int32_t* host_node_offsets, const int64_t* host_prefix_offsets,
                                 const int64_t* prefix_lens, const int64_t* host_prefix_lens,
                                 int32_t B, int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt, float scale,
                                 void* o, float* lse,
                                 void* workspace, size_t workspace_bytes, hs_stream stream);

/* hs_tree_attention_shared_tree: hs_tree_attention on B batch entries that verify the same tree, each
 * with its own Q, K and V: the decoder layers of one verification step (Section 2.2: one tree-mask
 * pass of the target model over the draft tree), or sequences that were given the same tree.
 * `parent` holds that one tree (int32 [M], device; e.g. hs_tree_prune's out_parent as it is); every
 * entry must have M rows (node_offsets[s+1] - node_offsets[s] == M for all s, checked on the host
 * copy: HS_ERR_SHAPE otherwise).  Everything else as hs_tree_attention. */
hs_status hs_tree_attention_shared_tree(const void* q, const void* k_prefix, const void* v_prefix,
                                        const void* k_tree, const void* v_tree,
                                        const int32_t* parent, const int32_t* node_offsets,
                                        const int64_t* prefix_offsets,
                                        const int32_t* host_node_offsets, const int64_t* host_prefix_offsets,
                                        int32_t B, int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt, float scale,
                                        void* o, float* lse,
                                        void* workspace, size_t workspace_bytes, hs_stream stream);

/* hs_tree_attention_paged: hs_tree_attention on paged KV caches.  k_pages / v_pages are pools
 * [n_pages, page_tokens, Hkv, D]; block_table (device, int32 [B, max_blocks]) names the page of each
 * block of page_tokens consecutive prefix tokens of a sequence; prefix_lens (device int64 [B]) and
 * host_prefix_lens (the same on the host) give the used tokens (at most max_blocks * page_tokens).
 * Pages of 64 tokens are built (one page is one tile of the matrix-core kernel); a prefix may
 * hold at most 1 048 576 tokens.  The workspace query takes the sum of the prefix lengths as
 * total_prefix.  Everything else as hs_tree_attention. */
hs_status hs_tree_attention_paged(const void* q, const void* k_pages, const void* v_pages,
                                  const void* k_tree, const void* v_tree,
                                  const int32_t* parent, const int32_t* node_offsets,
                                  const int32_t* host_node_offsets,
                                  const int32_t* block_table, int32_t max_blocks, int32_t page_tokens,
                                  const int64_t* prefix_lens, const int64_t* host_prefix_lens,
                                  int32_t B, int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt, float scale,
                                  void* o, float* lse,
                                  void* workspace, size_t workspace_bytes, hs_stream stream);

/* ------------------------------------------------------------------------------------------------
 * hs_verify_accept  (Section 2.1: a drafted token x is accepted with probability
 * min(1, p(x)/p_hat(x)); on rejection a token is drawn from the residual of p and later drafts are
 * dropped.  On a tree, the children of the current node are tried in ascending row index.)
 *
 * target_logits [NN,V] float: row i is the target model's logits after tree row i.
 * draft_logits  [NN,V] float: row i is the draft distribution the children of row i were proposed
 *   from (only rows that have children are read; NULL allowed in greedy mode).
 * token [NN] int32: the token of each row (root entry ignored).  parent / node_offsets as above.
 * uniforms [NN + B] float in [0,1): uniforms[node] decides that node's test, uniforms[NN + s]
 *   draws the bonus token of sequence s (NULL allowed in greedy mode).
 * Greedy: from the root, move to the child whose token equals argmax of the target row of the
 *   current node (ties -> lower index) until there is none; bonus = that argmax.
 * Stochastic: p = softmax(target/T), q = softmax(draft/T) at the current node; for each child c
 *   in order accept iff u_c < min(1, p(x_c)/q(x_c)); on rejection p <- norm(max(p - q, 0)),
 *   q(x_c) <- 0, q <- norm(q).  If no child is accepted the bonus token is the first index whose
 *   running sum of p exceeds u_bonus.  Point-mass variant: accept iff u_c < p(x_c); on rejection
 *   p(x_c) <- 0, p <- norm(p).
 * Outputs: accept_len [B] (number of accepted rows), accept_path [B,max_depth] local row indices
 *   padded with -1, bonus_token [B] (-1 for an empty sequence).  The walk stops after max_depth
 *   accepted rows.
 * Limits: the sampling rules try at most HS_MAX_CHILDREN children of a node, the lowest rows (Top-k
 *   expansion gives a node k <= HS_MAX_TOPK children; hs_tree_validate reports rows beyond the
 *   limit); NN <= 65535 rows in greedy mode and 32767 in the sampling modes (HS_ERR_UNSUPPORTED beyond).
 * Workspace: hs_verify_accept_workspace_mode gives what a call in `mode` needs; the query without
 *   a mode gives the largest of the three, that of HS_ACCEPT_STOCHASTIC: besides a few arrays of
 *   NN entries, a pair of floats per row and vocabulary entry, 80 KiB of bucket tables per row
 *   and a double per row and 64 vocabulary entries (about 8.2 * NN * V bytes; left out for
 *   NN > 4096, where every rejection re-reads the two rows and the walk sums the rows of its stop
 *   node itself).  Rows whose address is a multiple of 16 bytes (base and row_stride * 4) take
 *   the faster paths.
 */
size_t hs_verify_accept_workspace(int32_t B, int32_t NN, int32_t V);
size_t hs_verify_accept_workspace_mode(int32_t B, int32_t NN, int32_t V, hs_accept_mode mode);
hs_status hs_verify_accept(const float* target_logits, const float* draft_logits,
                           int64_t row_stride, const int32_t* token, const int32_t* parent,
                           const int32_t* node_offsets,
                           int32_t B, int32_t NN, int32_t V, hs_accept_mode mode, float temperature,
                           const float* uniforms, int32_t max_depth,
                           int32_t* accept_len, int32_t* accept_path, int32_t* bonus_token,
                           void* workspace, size_t workspace_bytes, hs_stream stream);

/* ------------------------------------------------------------------------------------------------
 * hs_tree_prune_counted: hs_tree_prune for trees stored with spare capacity (see the conventions):
 * node_counts [B] int32 gives the used rows of each sequence; depth / cumlogp / keep are written for
 * used rows only.  NN = node_offsets[B] (capacity).  node_counts == NULL is hs_tree_prune.
 */
hs_status hs_tree_prune_counted(const int32_t* parent, const float* logc, const int32_t* node_offsets,
                                const int32_t* node_counts, int32_t B, int32_t NN,
                                const int32_t* d_max, const float* theta, const int32_t* max_nodes,
                                int32_t* depth, float* cumlogp, uint8_t* keep,
                                int32_t* out_offsets, int32_t* out_src, int32_t* out_parent,
                                void* workspace, size_t workspace_bytes, hs_stream stream);

/* ------------------------------------------------------------------------------------------------
 * hs_tree_expand  (Section 2.2, Expansion: the tree grows one depth at a time; the nodes of the
 * newest depth with the largest value V, the product of the confidences on their root path, are
 * expanded with the Top-k tokens of their draft distribution.  Section 4.3, Dynamic Extended
 * Drafting: the number of levels may differ per sequence.)
 *
 * The draft trees of B sequences live in arrays with room for `cap` rows per sequence (sequence s
 * starts at row s * cap): parent, token, depth int32; logc, cumlogp, ent float.  n_nodes [B] counts
 * the used rows, level [B] the levels grown, frontier [B,F] lists the rows to expand now (local
 * indices, ascending) and n_frontier [B] how many of them there are.
 *
 * One call grows every sequence by one level from the results of hs_draft_entropy_topk on the
 * draft distributions of its frontier rows: result row s * F + j belongs to frontier[s,j].
 *   first != 0: the state is initialised first (root alone: parent -1, token -1, values 0; the
 *     frontier is the root, level 0), so the results are those of the roots' rows (j = 0).
 *   For each frontier row f (in order) and k < K: a new row with parent f, token topk_idx[.,k],
 *     logc = topk_logp[.,k], cumlogp = fl32(cumlogp[f] + min(logc, 0)), depth[f] + 1, ent 0;
 *     ent[f] = ent_topk[.].  A frontier row whose K children would exceed `cap` gets none.
 *   The next frontier is the F best new rows under (cumlogp descending, row ascending), listed in
 *     ascending row order; level += 1.
 *   A sequence with level >= d_limit[s] (d_limit may be NULL: no limit) or an empty frontier is
 *     left unchanged and its n_frontier becomes 0.
 * frontier_rows [B*F] int32 (may be NULL): global row (s * cap + local) of each frontier slot, for
 *   gathering the next draft inputs; slots past n_frontier repeat the sequence's last valid one
 *   (row s * cap when there is none).
 * Requires 1 <= K <= HS_MAX_TOPK, 1 <= F, F * K <= 4096, cap >= 1 + K.
 */
hs_status hs_tree_expand(int32_t* parent, int32_t* token, float* logc, float* cumlogp, int32_t* depth,
                         float* ent, int32_t* n_nodes, int32_t* level, int32_t* frontier,
                         int32_t* n_frontier, int32_t* frontier_rows,
                         const int32_t* topk_idx, const float* topk_logp, const float* ent_topk,
                         const int32_t* d_limit, int32_t B, int32_t cap, int32_t F, int32_t K,
                         int32_t first, hs_stream stream);

/* ------------------------------------------------------------------------------------------------
 * hs_adaptive_control  (Section 4.1, Eq. 1: Phi(P) = sum over the positions of path P of the
 * Top-K entropy of the draft distribution at that position, evaluated on the operational path P*
 * (defined below); Section 4.2: the trained decision
 * tree partitions Phi into entropy bins B_0 .. B_{n-1}, lowest entropy first; Section 4.3:
 * d'(B_i) = d_base + Delta(B_i), N'(B_i) = gamma_i * N_default + Delta(B_i), Delta(B_i) = alpha - i
 * for the low-entropy bins, nothing changes for the others.)
 *
 * Per sequence (trees as in hs_tree_prune, optionally with spare capacity):
 *   P*      the node of the deepest level present with the largest cumulative value (cumlogp as
 *           hs_tree_prune defines it; HS_PSTAR_LOCAL: the largest min(logc, 0)); ties -> lower row
 *   phi     sum of ent[a] over the strict ancestors a of P*, root first, in float32: ent[a] is the
 *           Top-K entropy of the draft distribution at a (hs_draft_entropy_topk's ent_topk of its row)
 *   bin     number of boundaries host_bin_edges[0 .. n_bins-2] (ascending) that phi has reached
 *   Delta   max(alpha - bin, 0) if bin < n_low, else 0
 *   d_prime = d_base + Delta
 *   n_prime = floor((double)host_gamma[bin] * n_default + 0.5) + Delta if bin < n_low, else n_default
 * Outputs phi float [B]; pstar (local row, -1 for an empty sequence), bin, d_prime, n_prime int32 [B]:
 * d_prime / n_prime can be handed to hs_tree_expand (d_limit) and hs_tree_prune (d_max, max_nodes)
 * without leaving the device.  host_bin_edges and host_gamma are HOST arrays, read during the call.
 * Requires 1 <= n_bins <= 64, 0 <= n_low <= min(8, n_bins).  No workspace.
 */
hs_status hs_adaptive_control(const int32_t* parent, const float* logc, const float* ent,
                              const int32_t* node_offsets, const int32_t* node_counts,
                              int32_t B, int32_t NN,
                              const float* host_bin_edges, int32_t n_bins,
                              const float* host_gamma, int32_t n_low,
                              int32_t alpha, int32_t d_base, int32_t n_default, hs_pstar_mode mode,
                              float* phi, int32_t* pstar, int32_t* bin, int32_t* d_prime,
                              int32_t* n_prime, hs_stream stream);

/* hs_adaptive_policy: what hs_adaptive_control decides for entropy bin `bin` (Section 4.3: Delta, d', N'
 * as defined above), computed on the host with the kernel's own formula and written to the two HOST
 * integers.  For callers that prepare one set of buffers or one captured graph per bin (Section 4.3,
 * Dynamic Computational Adaptation) and need each bin's shape beforehand.  No device work. */
hs_status hs_adaptive_policy(int32_t bin, const float* host_gamma, int32_t n_low, int32_t alpha,
                             int32_t d_base, int32_t n_default,
                             int32_t* host_d_prime, int32_t* host_n_prime);

/* ------------------------------------------------------------------------------------------------
 * hs_kv_commit  (Section 2.1: what an accepted path means for the next step's context)
 *
 * For each sequence with a tree, the K/V rows of the tree's root (the last committed token, whose
 * K/V is not in the cache yet) and of the accept_len[s] accepted rows accept_path[s, 0..] (local
 * rows, as hs_verify_accept writes them; row stride max_depth) are appended, in that order, to the
 * sequence's cache: token position cache_offsets[s] + cache_lens[s] onwards of k_cache / v_cache
 * [capacity, Hkv, D] (element type dt, as k_tree / v_tree [NN, Hkv, D]).  cache_lens[s] (int64,
 * device, in/out) grows by the number of rows written.  A sequence whose region
 * (cache_offsets[s+1] - cache_offsets[s] tokens) cannot take all its rows takes the leading ones
 * that fit; the caller sees that from cache_lens.  Rows of rejected tree nodes are not copied.
 * Requires Hkv * D * sizeof(element) to be a multiple of 16 and 16-byte aligned tensors.  No workspace.
 */
hs_status hs_kv_commit(const void* k_tree, const void* v_tree, const int32_t* node_offsets,
                       const int32_t* accept_path, const int32_t* accept_len, int32_t max_depth,
                       void* k_cache, void* v_cache, const int64_t* cache_offsets, int64_t* cache_lens,
                       int32_t B, int32_t Hkv, int32_t D, hs_dtype dt, hs_stream stream);

/* ------------------------------------------------------------------------------------------------
 * hs_tree_validate  (debugging aid; the tree conventions above are what every other call trusts)
 *
 * Checks B packed trees: node_offsets [B+1] start at 0, do not decrease and end at NN; in every
 * sequence row 0 has parent -1 and every other row's parent is an earlier row of the sequence; no
 * row has HS_MAX_CHILDREN or more earlier rows of the same parent; and, when token [NN] is given (may
 * be NULL), no row shares parent and token with an earlier row (siblings are distinct Top-k picks,
 * Section 2.2).
 * report (device, int32 [2]): the number of offending rows and the global index of the first one
 * (-1 if none); broken offsets count every row.  Valid after the stream is synchronised.
 * Quadratic in the rows of a sequence: not for the hot path.
 */
hs_status hs_tree_validate(const int32_t* parent, const int32_t* token, const int32_t* node_offsets,
                           int32_t B, int32_t NN, int32_t* report, hs_stream stream);

/* hs_kv_commit_paged: hs_kv_commit into paged caches (pools and block_table as in
 * hs_tree_attention_paged; any page_tokens >= 1).  The pages a sequence grows into must already be
 * in its block-table row; a sequence takes at most max_blocks * page_tokens tokens. */
hs_status hs_kv_commit_paged(const void* k_tree, const void* v_tree, const int32_t* node_offsets,
                             const int32_t* accept_path, const int32_t* accept_len, int32_t max_depth,
                             void* k_pages, void* v_pages, const int32_t* block_table, int32_t max_blocks,
                             int32_t page_tokens, int64_t* cache_lens,
                             int32_t B, int32_t Hkv, int32_t D, hs_dtype dt, hs_stream stream);

/* ------------------------------------------------------------------------------------------------
 * hs_time_next_attention  (measurement aid, not a step of the method)
 *
 * Hands two HIP events (hipEvent_t, created by the caller with timing enabled) to the next
 * hs_tree_attention / _lens / _paged call made on the calling thread.  That call attaches them to
 * the dispatch of its attention kernel: the runtime stamps `start_event` when the kernel begins to
 * execute and `stop_event` when it has ended, so hipEventElapsedTime(start, stop), once the stream
 * is synchronised, is that kernel's own duration, without the microseconds that events recorded
 * before and after a launch add to it.  The combine kernel that follows a launch with split keys
 * is not covered, nor is the scalar kernel that other shapes than bf16 take (the events then stay
 * as they were).  One-shot: the call consumes the pair whether it succeeds or not.  Both NULL
 * withdraws a pair not yet consumed; exactly one NULL gives HS_ERR_NULL.  The events stay the
 * caller's.
 */
hs_status hs_time_next_attention(void* start_event, void* stop_event);

/* hs_tree_attention_last_kernel  (debugging aid, not a step of the method)
 *
 * Which kernel the calling thread's last hs_tree_attention / _lens / _paged / _shared_tree call
 * launched: 1 = the matrix-core kernel (bfloat16; D = 128, or D = 64 with an even number of KV heads;
 * 16-byte aligned tensors; G * rows < 65536 for G = Hq / Hkv, twice that at D = 64),
 * 2 = the vector-ALU kernel (everything else),
 * 0 = none (no such call yet, an empty batch, or the call failed before its launch). */
int32_t hs_tree_attention_last_kernel(void);

/* hs_tree_attention_plan  (diagnostic, host only: no GPU is touched, nothing is launched)
 *
 * How hs_tree_attention / _lens (host_prefix_lens given) / _paged (paged != 0: host_prefix_offsets is
 * ignored, host_prefix_lens and max_blocks are required) would cut a batch of this shape into
 * workgroups, assuming 16-byte aligned tensors.  The host arrays are checked as in the real call
 * (same status codes).
 *   totals [6] (host, written): [0] kernel as in hs_tree_attention_last_kernel (0: nothing to launch),
 *     [1] workgroups of the attention launch, [2] largest number of key splits of a sequence,
 *     [3] tokens per split when all sequences are cut alike (0: each sequence has its own cut, see
 *     per_seq), [4] workspace bytes the call needs, [5] 1 if a combine launch follows.
 *   per_seq [B][4] (host, written; may be NULL): key splits, 64-key tiles per split, row groups
 *     (workgroups per KV head and split), number of the sequence's first workgroup in dispatch order
 *     (-1: the launch is a plain grid).
 */
hs_status hs_tree_attention_plan(const int32_t* host_node_offsets, const int64_t* host_prefix_offsets,
                                 const int64_t* host_prefix_lens, int32_t paged, int32_t max_blocks,
                                 int32_t B, int32_t Hq, int32_t Hkv, int32_t D, hs_dtype dt,
                                 int64_t* totals, int32_t* per_seq);

#ifdef __cplusplus
}
#endif
#endif /* HETEROSPEC_H_ */
