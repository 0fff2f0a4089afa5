"""Commit of the accepted path into the KV cache.

Follows Section 2.1: after verification the accepted draft tokens become part of the context,
later drafts are discarded, and decoding resumes behind the last accepted token.  For the
attention layer this means that the K/V rows of the tree's root (the last committed token, whose
K/V was not in the cache yet) and of the accepted rows, in path order, are appended to the
sequence's cache; the rows of rejected tree nodes go nowhere.  Test infrastructure only.

Caches with spare capacity: sequence s owns the token range cache_offsets[s] .. cache_offsets[s+1]
of k_cache / v_cache and uses the first cache_lens[s] of it.
"""
import numpy as np


def kv_commit(k_tree, v_tree, node_offsets, accept_path, accept_len, k_cache, v_cache, cache_offsets, cache_lens):
    """k_tree, v_tree [NN,Hkv,D]; node_offsets [B+1]; accept_path int [B,max_depth] (local rows, -1 padded),
    accept_len int [B]; k_cache, v_cache [capacity,Hkv,D] (same element type as the tree tensors);
    cache_offsets int64 [B+1]; cache_lens int64 [B].
    Returns (k_cache, v_cache, cache_lens) after the commit (copies).  A sequence whose region cannot
    take all its rows takes the leading ones that fit."""
    k_cache, v_cache = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    lens = np.array(cache_lens, dtype=np.int64, copy=True)
    B = len(node_offsets) - 1
    for s in range(B):
        n0, n1 = int(node_offsets[s]), int(node_offsets[s + 1])
        if n1 == n0:
            continue
        rows = [0] + [int(r) for r in accept_path[s][:int(accept_len[s])]]
        room = int(cache_offsets[s + 1]) - int(cache_offsets[s]) - int(lens[s])
        rows = rows[:max(room, 0)]
        for r in rows:
            assert 0 <= r < n1 - n0
            dst = int(cache_offsets[s]) + int(lens[s])
            k_cache[dst] = k_tree[n0 + r]
            v_cache[dst] = v_tree[n0 + r]
            lens[s] += 1
    return k_cache, v_cache, lens


def gather_pages(pages, block_table, lens, page_tokens=None):
    """Paged cache -> packed dense cache.  pages [n_pages, page_tokens, Hkv, D]; block_table int [B, max_blocks]
    (page of each block of page_tokens consecutive tokens of a sequence); lens [B] used tokens.
    Returns (dense [sum lens, Hkv, D], offsets int64 [B+1]): token t of sequence s is row
    t % page_tokens of page block_table[s, t // page_tokens]."""
    pages = np.asarray(pages)
    pt = pages.shape[1] if page_tokens is None else page_tokens
    rows, offs = [], [0]
    for s, n in enumerate(lens):
        for t in range(int(n)):
            rows.append(pages[int(block_table[s][t // pt]), t % pt])
        offs.append(offs[-1] + int(n))
    dense = np.stack(rows) if rows else np.zeros((0,) + pages.shape[2:], pages.dtype)
    return dense, np.asarray(offs, np.int64)


def kv_commit_paged(k_tree, v_tree, node_offsets, accept_path, accept_len, k_pages, v_pages, block_table, cache_lens):
    """kv_commit into paged caches: the same rows, appended at token positions cache_lens[s] onwards of
    sequence s, each landing in its page; a sequence takes at most max_blocks * page_tokens tokens."""
    k_pages, v_pages = np.array(k_pages, copy=True), np.array(v_pages, copy=True)
    lens = np.array(cache_lens, dtype=np.int64, copy=True)
    pt = k_pages.shape[1]
    for s in range(len(node_offsets) - 1):
        n0, n1 = int(node_offsets[s]), int(node_offsets[s + 1])
        if n1 == n0:
            continue
        rows = [0] + [int(r) for r in accept_path[s][:int(accept_len[s])]]
        room = len(block_table[s]) * pt - int(lens[s])
        for r in rows[:max(room, 0)]:
            t = int(lens[s])
            page = int(block_table[s][t // pt])
            k_pages[page, t % pt] = k_tree[n0 + r]
            v_pages[page, t % pt] = v_tree[n0 + r]
            lens[s] += 1
    return k_pages, v_pages, lens
