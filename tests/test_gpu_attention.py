"""GPU parity of hs_tree_attention against the CPU checker: max-abs 2e-2 for bfloat16 outputs,
1e-4 for float32; lse within 1e-3 / 1e-4."""
import numpy as np
import pytest

from synth import workloads as W
from oracle import tree_attention, pipeline as P

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _case(w, seed, parents, Ls, variant):
    """A packed attention problem for explicit trees and prefix lengths."""
    parts = [W.attention_inputs(w, seed, s, int(L), len(p), variant, parent=np.asarray(p))
             for s, (p, L) in enumerate(zip(parents, Ls))]
    q, kp, vp, kt, vt = (np.concatenate([x[i] for x in parts], axis=0) for i in range(5))
    no = np.concatenate([[0], np.cumsum([len(p) for p in parents])]).astype(np.int32)
    po = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int64)
    return dict(w=w, q=q, k_prefix=kp, v_prefix=vp, k_tree=kt, v_tree=vt,
                parent=np.concatenate([np.asarray(p, np.int32) for p in parents]),
                node_offsets=no, prefix_offsets=po, scale=1.0 / np.sqrt(w.D))


def _compare(G, step, dtype, big_scores=False):
    want_o, want_lse = P.attention_out(step)
    got_o, got_lse = G.run_attention(step)
    diff = np.abs(got_o.astype(np.float64) - want_o)
    err = diff.max()
    assert err <= TOL[dtype], err
    # bf16: the kernel folds scale * log2(e) into Q and rounds it to bf16 again, which perturbs each
    # score by at most 2^-8 * sum_d |q_d k_d| * scale; with few keys the log-sum-exp moves by as much,
    # so it gets the same 2e-2 bound as the outputs.  Where one planted score of size s dominates
    # (big_scores), sum_d |q_d k_d| * scale = s, and the log-sum-exp is that score: 2^-8 |lse| more.
    lse_err = float(np.abs(got_lse - want_lse).max())
    lse_tol = 1e-4 if dtype == "f32" else 2e-2
    if big_scores:
        lse_tol += 2.0 ** -8 * float(np.abs(want_lse).max())
    assert lse_err <= lse_tol, (lse_err, lse_tol)
    scale = np.abs(want_o).max()
    if dtype == "f32":
        assert err <= 1e-5 * max(scale, 1e-6) + 1e-7, (err, scale)
        return err
    # Besides the stated max-abs: every element within the bound that the kernel's arithmetic implies
    # (gpu_util.attention_error_bound: worst case of each rounding, element by element) ...
    bound = G.attention_error_bound(step, want_o)
    worst = float((diff / bound).max())
    assert worst <= 1.0, (worst, err, scale)
    # ... and, since the roundings are independent and rarely all at their worst, the largest error
    # within 1e-2 of the output scale: a weight's and the result's rounding are at most 2^-8 = 3.9e-3
    # each (2^-9 on average) and the re-rounded Q moves a score by about 2^-8 / sqrt(3) * scale *
    # |q . k|_2 = 2e-3 for unit-variance inputs.  (Not asked of big_scores: a score of size s carries
    # up to 2^-8 s there, which the element-wise bound above accounts for.)
    if not big_scores:
        assert err <= 1e-2 * max(scale, 1e-6) + 1e-7, (err, scale)
    return err


def _random_parents(rs, n, back=6):
    return [-1] + [int(rs.randint(max(0, i - back), i)) for i in range(1, n)]


@pytest.mark.parametrize("variant", ["config", "unit", "peaky"])
def test_workload1_float32(G, variant):
    w = W.WORKLOADS[1]
    par = W.tree_parents(w, 0)                               # the full 17-row tree
    _compare(G, _case(w, 0, [list(par)], [128], variant), "f32")
    st = P.build_step(w, 0, variant=variant)                 # and the pruned step as the pipeline builds it
    _compare(G, st, "f32")


@pytest.mark.parametrize("variant", ["config", "unit", "peaky"])
@pytest.mark.parametrize("wid,L,M", [(2, 700, 61), (3, 300, 129), (4, 1100, 97)])
def test_bf16_shapes_reduced_prefix(G, wid, L, M, variant):
    w = W.WORKLOADS[wid]
    rs = np.random.RandomState(wid)
    _compare(G, _case(w, 1, [_random_parents(rs, M)], [L], variant), "bf16")


@pytest.mark.parametrize("variant", ["unit_v", "peaky_v"])
@pytest.mark.parametrize("wid,L,M", [(2, 700, 61), (3, 300, 129), (4, 1100, 97), (5, 5000, 129)])
def test_outputs_of_order_one(G, wid, L, M, variant):
    """V drawn N(0,1) like Q and K: outputs reach several units (a planted key hands its V row through
    almost unchanged), so the stated 2e-2 max-abs is a real constraint here, not only the relative
    checks.  Also a ragged pair with a row group beyond 256 rows and a short prefix."""
    w = W.WORKLOADS[wid]
    rs = np.random.RandomState(70 + wid)
    _compare(G, _case(w, 9, [_random_parents(rs, M)], [L], variant), "bf16")
    _compare(G, _case(w, 10, [_random_parents(rs, 7), _random_parents(rs, M)], [3, L // 2], variant), "bf16")


@pytest.mark.parametrize("wid,L,M", [(2, 700, 61), (5, 2100, 33)])
def test_scores_that_overflow_a_fixed_reference(G, wid, L, M):
    """Planted scores 120+ above the rest, late in the prefix and in the tree: exp of the gap to the
    first block's maximum overflows float32, so the rows need the running-maximum treatment."""
    w = W.WORKLOADS[wid]
    rs = np.random.RandomState(40 + wid)
    _compare(G, _case(w, 6, [_random_parents(rs, M)], [L], "hot"), "bf16", big_scores=True)
    _compare(G, _case(w, 7, [_random_parents(rs, M), _random_parents(rs, 9)], [L, 70], "hot"), "bf16", big_scores=True)


def test_chain_star_and_no_prefix(G):
    w = W.WORKLOADS[2]
    chain = list(range(-1, 40))
    star = [-1] + [0] * 70
    for par, L in ((chain, 130), (star, 65), (chain, 0), ([-1], 0), ([-1], 3), (star, 1)):
        _compare(G, _case(w, 2, [par], [L], "unit"), "bf16")
    w1 = W.WORKLOADS[1]
    for par, L in ((chain, 70), ([-1], 0)):
        _compare(G, _case(w1, 2, [par], [L], "unit"), "f32")


def test_ragged_batch_with_empty_sequence(G):
    w = W.small(W.WORKLOADS[5])
    rs = np.random.RandomState(5)
    sizes = [9, 129, 0, 33, 64, 65, 1]
    Ls = [512, 37, 100, 2049, 0, 1300, 64]
    parents = [_random_parents(rs, n) if n else [] for n in sizes]
    _compare(G, _case(w, 3, parents, Ls, "peaky"), "bf16")


def test_split_and_unsplit_sequences_in_one_launch(G):
    """A long sequence is cut into key splits (merged by the combine kernel) while the short ones of
    the same launch are written directly by the attention kernel."""
    w = W.small(W.WORKLOADS[5])
    rs = np.random.RandomState(11)
    sizes, Ls = [33, 9, 70, 129, 5], [6000, 100, 3000, 9000, 511]
    _compare(G, _case(w, 8, [_random_parents(rs, n) for n in sizes], Ls, "peaky"), "bf16")


@pytest.mark.parametrize("B,D,big", [(70, 128, 40), (96, 128, 40), (100, 128, 40), (100, 128, 300), (100, 64, 40), (100, 64, 300)])
def test_batches_around_the_work_list_capacity(G, B, D, big):
    """More than 64 sequences need the second half of the kernel-argument table; more than 96 do
    not fit it and take the launch with one grid row per sequence: also with a tree past 256 rows in
    the batch and with head dimension 64."""
    w = W.small(W.WORKLOADS[5], D=D)
    rs = np.random.RandomState(B)
    sizes = [int(x) for x in rs.randint(0, 20, size=B)]
    Ls = [int(x) for x in rs.randint(0, 300, size=B)]
    Ls[B // 2] = 2500                                        # one sequence long enough to be split
    sizes[B // 2] = big
    parents = [_random_parents(rs, n) if n else [] for n in sizes]
    _compare(G, _case(w, 9, parents, Ls, "unit"), "bf16")


def test_many_splits_long_prefix(G):
    w = W.WORKLOADS[2]
    rs = np.random.RandomState(8)
    err = _compare(G, _case(w, 4, [_random_parents(rs, 61)], [16384 + 77], "unit"), "bf16")


def test_sibling_independence_and_determinism(G):
    w = W.WORKLOADS[2]
    rs = np.random.RandomState(9)
    par = _random_parents(rs, 40, back=4)
    st = _case(w, 5, [par], [300], "unit")
    a, _ = G.run_attention(st)
    b, _ = G.run_attention(st)
    assert np.array_equal(a, b)
    leaf = max(i for i in range(40) if i not in par)         # a leaf: nobody else may see it
    st2 = dict(st)
    kt = st["k_tree"].copy()
    kt[leaf] ^= np.uint16(0x0101)
    st2["k_tree"] = kt
    c, _ = G.run_attention(st2)
    others = [i for i in range(40) if i != leaf]
    assert np.array_equal(a[others], c[others]) and not np.array_equal(a[leaf], c[leaf])


def test_events_attached_to_the_attention_kernel(G):
    """hs_time_next_attention: the pair is consumed by one call, brackets the kernel alone, and leaves
    the result as it is."""
    import paper_2505_13254_amd as hs
    w = W.WORKLOADS[2]
    rs = np.random.RandomState(12)
    st = _case(w, 6, [_random_parents(rs, 61)], [4096 + 5], "unit")
    plain, _ = G.run_attention(st)
    e0, e1, f0, f1 = (torch.cuda.Event(enable_timing=True) for _ in range(4))
    for e in (e0, e1, f0, f1):
        e.record()
    torch.cuda.synchronize()
    hs.hs_time_next_attention(e0, e1)
    f0.record()
    timed, _ = G.run_attention(st)           # uploads, launches, synchronises, downloads
    f1.record()
    torch.cuda.synchronize()
    assert np.array_equal(plain, timed)
    own, around = e0.elapsed_time(e1), f0.elapsed_time(f1)
    assert 0.0 < own < around, (own, around)
    assert own < 5.0, own                    # milliseconds: one small kernel
    again, _ = G.run_attention(st)           # one-shot: this call leaves the pair alone
    torch.cuda.synchronize()
    assert e0.elapsed_time(e1) == own
    hs.hs_time_next_attention(e0, e1)
    hs.hs_time_next_attention(None, None)    # withdrawn
    G.run_attention(st)
    torch.cuda.synchronize()
    assert e0.elapsed_time(e1) == own
    import ctypes
    assert hs.lib().hs_time_next_attention(None, ctypes.c_void_p(e1.cuda_event)) != 0   # half a pair is refused


@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (16, 2)])
@pytest.mark.parametrize("M,L", [(256, 200), (257, 100), (1024, 70), (513, 0), (700, 1300)])
def test_tree_row_limits(G, M, L, hq, hkv):
    """Trees of up to 256 rows have their ancestor table built inside the attention kernel; larger ones
    (up to the limit of 1024 rows) take it from a table laid out per key tile by a launch of its own.
    Both run on the matrix cores.  G = 4, 1 and 8 query heads per KV head: up to 32 row groups; L = 0:
    the leading tiles are tree tiles."""
    import paper_2505_13254_amd as hs
    w = W.small(W.WORKLOADS[2], Hq=hq, Hkv=hkv)
    rs = np.random.RandomState(M)
    _compare(G, _case(w, 13, [_random_parents(rs, M, back=12)], [L], "unit"), "bf16")
    assert hs.hs_tree_attention_last_kernel() == 1


@pytest.mark.parametrize("shape", ["chain", "star", "deep_then_wide"])
def test_large_trees_of_extreme_shape(G, shape):
    """600 rows as one chain (every earlier row is an ancestor: all mask bits set below the diagonal), as a
    star (only the root and the row itself) and as a chain of 300 whose last node has 299 children."""
    import paper_2505_13254_amd as hs
    M = 600
    par = {"chain": [-1] + list(range(M - 1)), "star": [-1] + [0] * (M - 1),
           "deep_then_wide": [-1] + list(range(300)) + [300] * (M - 301)}[shape]
    w = W.small(W.WORKLOADS[2], Hq=8, Hkv=2)
    _compare(G, _case(w, 15, [par], [130], "peaky"), "bf16")
    assert hs.hs_tree_attention_last_kernel() == 1


@pytest.mark.parametrize("seed", [3, 4])
def test_ragged_batches_with_large_trees(G, seed):
    """Batches that mix trees of a few rows with trees beyond 256 rows, prefixes from nothing to several key
    splits, every input variant (planted large scores included)."""
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(seed)
    for it in range(8):
        hq, hkv = [(8, 2), (8, 8), (16, 2), (4, 1)][rs.randint(4)]
        w = W.small(W.WORKLOADS[2], Hq=hq, Hkv=hkv)
        B = int(rs.randint(2, 6))
        sizes = [int(rs.choice([0, 2, 61, 256, 257, 300, 640, 1024])) for _ in range(B)]
        sizes[int(rs.randint(B))] = int(rs.choice([257, 321, 777]))
        Ls = [int(rs.choice([0, 1, 63, 64, 500, 1300, 2049, 4100])) for _ in range(B)]
        parents = [_random_parents(rs, n, back=int(rs.choice([2, 6, 40]))) if n else [] for n in sizes]
        variant = ["config", "unit", "peaky", "hot"][rs.randint(4)]
        _compare(G, _case(w, 1000 * seed + it, parents, Ls, variant), "bf16", big_scores=variant == "hot")
        assert hs.hs_tree_attention_last_kernel() == 1


@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (16, 2), (12, 6)])
@pytest.mark.parametrize("M,L", [(61, 300), (129, 1000), (300, 70), (9, 0), (64, 2100)])
def test_head_dimension_64_in_bfloat16(G, M, L, hq, hkv):
    """bfloat16 with D = 64 runs on the matrix cores too: the kernel takes the KV heads in pairs (two heads of
    a token are one 256-byte row) and widens each query row with zeros on the other head's side.  One and
    several row groups, large trees, an empty prefix, a prefix cut into splits."""
    import paper_2505_13254_amd as hs
    w = W.small(W.WORKLOADS[2], Hq=hq, Hkv=hkv, D=64)
    rs = np.random.RandomState(M + hq)
    _compare(G, _case(w, 21, [_random_parents(rs, M, back=9)], [L], "unit"), "bf16")
    assert hs.hs_tree_attention_last_kernel() == 1


def test_head_dimension_64_ragged_batches(G):
    """D = 64 through the ragged work-list launch: several sequences, splits, all input variants; an odd
    number of KV heads cannot be paired and runs on the vector ALUs."""
    import paper_2505_13254_amd as hs
    rs = np.random.RandomState(64)
    for it in range(10):
        hq, hkv = [(8, 2), (8, 8), (16, 4), (4, 2), (3, 3)][rs.randint(5)]
        w = W.small(W.WORKLOADS[2], Hq=hq, Hkv=hkv, D=64)
        B = int(rs.randint(1, 6))
        sizes = [int(rs.choice([0, 1, 9, 33, 61, 64, 65, 129, 300])) for _ in range(B)]
        if sum(sizes) == 0:
            sizes[0] = 5
        Ls = [int(rs.choice([0, 1, 63, 64, 65, 500, 1300, 2049, 4100])) for _ in range(B)]
        parents = [_random_parents(rs, n) if n else [] for n in sizes]
        variant = ["config", "unit", "peaky", "hot", "unit_v"][rs.randint(5)]
        _compare(G, _case(w, 6400 + it, parents, Ls, variant), "bf16", big_scores=variant == "hot")
        assert hs.hs_tree_attention_last_kernel() == (2 if hkv % 2 else 1)


@pytest.mark.parametrize("hq,hkv,M,L", [(8, 2, 61, 300), (4, 2, 40, 700), (8, 2, 129, 64), (8, 8, 9, 2100)])
def test_first_keys_with_hugely_negative_scores(G, hq, hkv, M, L):
    """Two query rows score -150 on the first 64 prefix keys: the maximum of their first block is far below
    the range in which 2^(-m) is finite, and every later score is 150 above it (the exact pass)."""
    w = W.small(W.WORKLOADS[2], Hq=hq, Hkv=hkv)
    rs = np.random.RandomState(M)
    _compare(G, _case(w, 31, [_random_parents(rs, M)], [L], "cold"), "bf16", big_scores=True)


def test_a_long_prefix_cut_into_the_most_splits(G):
    """70 000 prefix tokens on two KV heads: the planner asks for the largest number of key splits (64); with
    18 tiles to a split 61 splits hold all 1094 tiles, and no split may start behind the prefix."""
    import paper_2505_13254_amd as hs
    w = W.small(W.WORKLOADS[2], Hq=8, Hkv=2)
    rs = np.random.RandomState(7)
    st = _case(w, 41, [_random_parents(rs, 33)], [70000], "unit")
    totals, per = hs.hs_tree_attention_plan(torch.from_numpy(st["node_offsets"]), torch.from_numpy(st["prefix_offsets"]),
                                            8, 2, 128, hs.HS_BF16)
    n_sp, per_split = int(per[0][0]), int(per[0][1])
    assert n_sp > 32 and (n_sp - 1) * per_split < 1094 <= n_sp * per_split
    _compare(G, st, "bf16")


def test_more_tree_rows_than_supported_is_an_error(G):
    import paper_2505_13254_amd as hs
    w = W.small(W.WORKLOADS[2], Hq=8, Hkv=2)
    rs = np.random.RandomState(1)
    st = _case(w, 14, [_random_parents(rs, 1025)], [10], "unit")
    with pytest.raises(hs.HsError) as e:
        G.run_attention(st)
    assert e.value.status == 3 and "1025" in str(e.value)    # HS_ERR_UNSUPPORTED, names the size


@pytest.mark.parametrize("seed", [1, 2])
def test_random_ragged_batches(G, seed):
    """Thirty random batches per seed: 1 to 8 sequences, tree sizes and prefix lengths drawn around the
    tile, row-group and split boundaries (empty trees and empty prefixes included), four head layouts."""
    rs = np.random.RandomState(seed)
    for it in range(30):
        hq, hkv = [(8, 2), (8, 8), (16, 2), (4, 1)][rs.randint(4)]
        w = W.small(W.WORKLOADS[2], Hq=hq, Hkv=hkv)
        B = int(rs.randint(1, 9))
        sizes = [int(rs.choice([0, 1, 2, 9, 33, 61, 64, 65, 129, 140])) for _ in range(B)]
        if sum(sizes) == 0:
            sizes[0] = 5
        Ls = [int(rs.choice([0, 1, 63, 64, 65, 500, 1300, 2049, 4100])) for _ in range(B)]
        parents = [_random_parents(rs, n) if n else [] for n in sizes]
        variant = ["config", "unit", "peaky"][rs.randint(3)]
        _compare(G, _case(w, 100 * seed + it, parents, Ls, variant), "bf16")


@pytest.mark.parametrize("wid,M,B", [(2, 61, 5), (2, 100, 3), (2, 300, 3), (1, 16, 4)])
def test_entries_that_share_one_tree(G, wid, M, B):
    """hs_tree_attention_shared_tree: B entries (different Q, K, V and prefix lengths) verify one tree
    passed once; the result equals the checker's on the tree repeated per entry, and bit for bit the
    ordinary call's on the repeated tree.  Matrix-core kernel with one and with several row groups,
    and the float32 kernel."""
    import paper_2505_13254_amd as hs
    w = W.WORKLOADS[wid]
    rs = np.random.RandomState(90 + M)
    tree = _random_parents(rs, M)
    Ls = [int(x) for x in rs.randint(0, 700, size=B)]
    st = _case(w, 8, [tree] * B, Ls, "unit")
    want_o, want_lse = P.attention_out(st)
    plain_o, plain_lse = G.run_attention(st)
    no, po = st["node_offsets"], st["prefix_offsets"]
    o, lse = hs.hs_tree_attention(G.dev_store(st["q"]), G.dev_store(st["k_prefix"]), G.dev_store(st["v_prefix"]),
                                  G.dev_store(st["k_tree"]), G.dev_store(st["v_tree"]),
                                  G.dev(np.asarray(tree, np.int32), torch.int32), G.dev(no), G.dev(po),
                                  torch.from_numpy(no), torch.from_numpy(po), float(st["scale"]), want_lse=True,
                                  shared_tree=True)
    o, lse = G.host(o), G.host(lse)
    dtype = "f32" if w.dtype == "f32" else "bf16"
    assert np.abs(o.astype(np.float64) - want_o).max() <= TOL[dtype]
    assert np.array_equal(o, plain_o) and np.array_equal(lse, plain_lse)


def test_shared_tree_needs_entries_of_equal_size(G):
    import paper_2505_13254_amd as hs
    w = W.WORKLOADS[2]
    rs = np.random.RandomState(3)
    st = _case(w, 8, [_random_parents(rs, 10), _random_parents(rs, 12)], [64, 64], "unit")
    no, po = st["node_offsets"], st["prefix_offsets"]
    with pytest.raises(RuntimeError, match="rows"):
        hs.hs_tree_attention(G.dev_store(st["q"]), G.dev_store(st["k_prefix"]), G.dev_store(st["v_prefix"]),
                             G.dev_store(st["k_tree"]), G.dev_store(st["v_tree"]),
                             G.dev(st["parent"][:10], torch.int32), G.dev(no), G.dev(po), torch.from_numpy(no),
                             torch.from_numpy(po), float(st["scale"]), shared_tree=True)
