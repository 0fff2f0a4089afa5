"""Host logic of hs_tree_attention, on the CPU: how a batch is cut into workgroups (hs_tree_attention_plan
runs the real call's validation and planning and launches nothing), checked for the properties every plan
must have, and the same code under AddressSanitizer / UndefinedBehaviorSanitizer."""
import os
import shutil
import subprocess

import numpy as np
import pytest
import torch

import paper_2505_13254_amd as hs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
W5_L = [856, 9850, 7619, 8510, 8308, 14995, 14506, 1572, 13592, 15067, 15126, 9243, 4415, 9633, 2862, 11678]
W5_M = [9, 26, 43, 60, 78, 95, 112, 129, 129, 112, 95, 78, 60, 43, 26, 9]


def _plan(Ms, Ls, Hq, Hkv, D=128, dt=None, lens=None, paged=False, max_blocks=0):
    no = torch.from_numpy(np.concatenate([[0], np.cumsum(Ms)]).astype(np.int32))
    po = None if paged else torch.from_numpy(np.concatenate([[0], np.cumsum(Ls)]).astype(np.int64))
    hl = None if lens is None else torch.from_numpy(np.asarray(lens, np.int64))
    t, p = hs.hs_tree_attention_plan(no, po, Hq, Hkv, D, hs.HS_BF16 if dt is None else dt, host_prefix_lens=hl,
                                     paged=paged, max_blocks=max_blocks)
    return t.numpy(), p.numpy()


def _check_work_list(Ms, Ls, Hq, Hkv, D, totals, per):
    """A work-list plan: every sequence with rows has its items, items are numbered without gaps in
    dispatch order, a sequence's splits cover its prefix tiles once, no split is shorter than 2 tiles."""
    kernel, n_items, sp_max, split_len, ws_bytes, combine = (int(x) for x in totals)
    units = Hkv // 2 if D == 64 else Hkv
    G = (Hq // Hkv) * (2 if D == 64 else 1)
    assert kernel == 1 and split_len == 0
    seqs = [s for s in range(len(Ms)) if Ms[s] > 0]
    order = sorted(seqs, key=lambda s: per[s][3])
    nxt = 0
    for s in order:
        n_sp, per_split, n_rg, first = (int(x) for x in per[s])
        tiles = (Ls[s] + 63) // 64
        assert first == nxt, (s, first, nxt)
        assert n_rg == (G * Ms[s] + 255) // 256
        assert 1 <= n_sp <= sp_max <= 64
        assert n_sp * per_split >= tiles and (n_sp - 1) * per_split < max(tiles, 1)
        if n_sp > 1:
            assert per_split >= 2
        nxt += units * n_sp * n_rg
    assert nxt == n_items
    for s in range(len(Ms)):
        if Ms[s] == 0:
            assert tuple(per[s]) == (0, 0, 0, -1)
    assert combine == (1 if sp_max > 1 else 0)
    # the long items first: the cost of an item never rises along the dispatch order
    waves = lambda s: min(8, (G * Ms[s] + 31) // 32)
    costs = [int(per[s][1]) * (1.25 + 0.04 * waves(s)) for s in order]
    assert all(a >= b - 1e-6 for a, b in zip(costs, costs[1:])), costs
    NN = int(sum(Ms))
    assert ws_bytes <= hs.lib().hs_tree_attention_workspace(len(Ms), NN, int(sum(Ls)), Hq, Hkv, D, int(hs.HS_BF16))


def test_the_bench_launch_is_one_workgroup_per_layer_and_head():
    totals, per = _plan([61] * 32, [2048] * 32, 32, 8)
    assert tuple(totals) == (1, 256, 1, 0, 0, 0)
    assert all(tuple(r[:3]) == (1, 32, 1) for r in per)
    _check_work_list([61] * 32, [2048] * 32, 32, 8, 128, totals, per)


def test_a_single_layer_is_cut_finer_than_a_launch_that_fills_the_chip():
    """One layer of the 8B shape is 8 (sequence, head) pairs for 256 compute units: its keys are cut into
    items of fewer than 8 tiles; four layers already take 8-tile items."""
    totals, per = _plan([61], [2048], 32, 8)
    _check_work_list([61], [2048], 32, 8, 128, totals, per)
    assert 2 <= per[0][1] < 8 and totals[1] == 8 * per[0][0] and totals[5] == 1
    totals4, per4 = _plan([61] * 4, [2048] * 4, 32, 8)
    _check_work_list([61] * 4, [2048] * 4, 32, 8, 128, totals4, per4)
    assert all(r[1] >= 8 for r in per4)


def test_plans_are_remembered_per_input_not_per_call_order():
    """The library keeps its last few plans: the same inputs give the same plan whatever was planned in
    between (more shapes than it keeps), and inputs that differ in one length, one tree size, the head layout,
    the used lengths or the offsets alone are not taken for each other."""
    base = ([61, 129, 9], [3000, 20000, 700], 32, 8)
    variants = [base,
                ([61, 129, 9], [3000, 20001, 700], 32, 8),
                ([61, 130, 9], [3000, 20000, 700], 32, 8),
                ([61, 129, 9], [3000, 20000, 700], 64, 8),
                ([61, 129, 9], [3000, 20000, 700], 32, 4),
                ([61, 129, 9], [3000, 20000, 764], 32, 8),
                ([61, 129, 9, 0], [3000, 20000, 700, 0], 32, 8)]
    first = [_plan(*v) for v in variants]
    for v, (t, p) in zip(variants, first):
        _check_work_list(v[0], v[1], v[2], v[3], 128, t, p)
    for rnd in range(3):
        for k in np.random.RandomState(rnd).permutation(len(variants)):
            t, p = _plan(*variants[k])
            assert np.array_equal(t, first[k][0]) and np.array_equal(p, first[k][1]), (rnd, k)
    # used lengths: same offsets, different lens; and the same lens behind different offsets
    t_a, p_a = _plan([61, 61], [20000, 20000], 32, 8, lens=[300, 20000])
    t_b, p_b = _plan([61, 61], [20000, 20000], 32, 8, lens=[20000, 300])
    t_c, p_c = _plan([61, 61], [20000, 20000], 32, 8)
    assert p_a[0][0] == 1 and p_b[1][0] == 1 and p_c[0][0] > 1 and p_c[1][0] > 1
    t_a2, p_a2 = _plan([61, 61], [20000, 20000], 32, 8, lens=[300, 20000])
    assert np.array_equal(t_a, t_a2) and np.array_equal(p_a, p_a2)


def test_plans_from_several_threads_at_once():
    """Planning state is per calling thread: four threads planning different batches at the same time (the
    foreign calls run without the interpreter lock) get what a single thread gets."""
    import threading
    rs = np.random.RandomState(5)
    shapes = []
    for _ in range(24):
        B = int(rs.randint(1, 30))
        shapes.append(([int(x) for x in rs.choice([1, 9, 61, 129, 300], size=B)],
                       [int(x) for x in rs.choice([0, 64, 700, 2048, 9000, 40000], size=B)], 32, 8))
    want = [_plan(*sh) for sh in shapes]
    errors = []

    def work(tid):
        try:
            for rep in range(6):
                for k in range(tid, len(shapes), 4):
                    t, p = _plan(*shapes[k])
                    assert np.array_equal(t, want[k][0]) and np.array_equal(p, want[k][1]), (tid, rep, k)
        except Exception as e:          # noqa: BLE001 (reported below, in the main thread)
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors


def test_the_ragged_batch_is_cut_into_comparable_items():
    totals, per = _plan(W5_M, W5_L, 32, 8)
    _check_work_list(W5_M, W5_L, 32, 8, 128, totals, per)
    assert totals[2] > 1 and 256 < totals[1] < 2048
    assert per[5][0] > per[0][0]                       # 14995 tokens are cut, 856 are not


@pytest.mark.parametrize("seed", range(6))
def test_random_batches_have_consistent_plans(seed):
    rs = np.random.RandomState(seed)
    for it in range(120):
        Hq, Hkv = [(32, 8), (8, 8), (64, 8), (4, 1), (12, 6)][rs.randint(5)]
        D = int(rs.choice([128, 64]))
        if D == 64 and Hkv % 2:
            continue
        B = int(rs.randint(1, 40))
        Ms = [int(rs.choice([0, 1, 9, 61, 64, 129, 257, 700])) for _ in range(B)]
        Ls = [int(rs.choice([0, 1, 63, 64, 500, 2048, 4100, 16384, 70000])) for _ in range(B)]
        if sum(Ms) == 0:
            Ms[0] = 3
        totals, per = _plan(Ms, Ls, Hq, Hkv, D)
        _check_work_list(Ms, Ls, Hq, Hkv, D, totals, per)
        again, per2 = _plan(Ms, Ls, Hq, Hkv, D)
        assert np.array_equal(totals, again) and np.array_equal(per, per2)


def test_used_lengths_not_capacities_decide_the_cut():
    Ms, caps = [61, 61], [20000, 20000]
    t_full, p_full = _plan(Ms, caps, 32, 8)
    t_used, p_used = _plan(Ms, caps, 32, 8, lens=[300, 20000])
    assert p_full[0][0] > 1 and p_used[0][0] == 1 and p_used[1][0] > 1
    _check_work_list(Ms, [300, 20000], 32, 8, 128, t_used, p_used)


def test_paged_caches_keep_a_split_within_256_pages():
    totals, per = _plan([61], None, 32, 8, lens=[64 * 256 * 3 + 5], paged=True, max_blocks=800)
    assert totals[0] == 1 and per[0][0] >= 4 and per[0][1] <= 256


def test_more_sequences_than_the_table_holds_take_a_plain_grid():
    B = 130
    totals, per = _plan([9] * B, [3000] * B, 32, 8)
    assert totals[0] == 1 and totals[3] >= 512 and totals[3] % 256 == 0
    assert all(int(r[3]) == -1 for r in per)
    assert totals[1] == 8 * 1 * totals[2] * B


def test_which_kernel_a_shape_gets():
    assert _plan([61], [300], 8, 2)[0][0] == 1
    assert _plan([61], [300], 8, 2, dt=hs.HS_F32)[0][0] == 2
    assert _plan([61], [300], 8, 2, D=64)[0][0] == 1          # pairs of KV heads
    assert _plan([61], [300], 3, 3, D=64)[0][0] == 2          # an odd number cannot be paired
    assert _plan([1024], [300], 8, 2)[0][0] == 1
    assert _plan([0, 0], [300, 5], 8, 2)[0][0] == 0           # nothing to launch


def test_bad_host_arrays_are_refused_as_in_the_real_call():
    with pytest.raises(hs.HsError) as e:
        _plan([1025], [10], 8, 2)
    assert e.value.status == 3
    no = torch.tensor([0, 5, 3], dtype=torch.int32)
    po = torch.tensor([0, 10, 20], dtype=torch.int64)
    with pytest.raises(hs.HsError):
        hs.hs_tree_attention_plan(no, po, 8, 2, 128, hs.HS_BF16)
    with pytest.raises(hs.HsError):
        _plan([5], [10], 8, 3)                                # Hq not a multiple of Hkv


def test_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The files that hold the call's validation and planning, compiled with the host-side sanitizers
    (device code is compiled as usual and never runs), linked with a driver that plans a few thousand
    random batches: dense, spare-capacity and paged, up to 130 sequences, all head layouts."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined"]
    common = [hipcc, "-O1", "-g", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip", "-Xclang",
              "-target-feature", "-Xclang", "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"),
              "-I" + os.path.join(ROOT, "paper_2505_13254_amd", "csrc"), "-Wno-unused-variable"] + san
    srcs = [os.path.join(ROOT, "paper_2505_13254_amd", "csrc", f)
            for f in ("tree_attention.hip", "tree_attention_mfma.hip", "api.cpp")]
    srcs.append(os.path.join(ROOT, "tests", "host", "plan_fuzz.cpp"))
    procs, objs = [], []
    for src in srcs:
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        objs.append(obj)
        procs.append(subprocess.Popen(common + ["-c", src, "-o", obj], stdout=subprocess.PIPE, stderr=subprocess.STDOUT))
    for p in procs:
        out, _ = p.communicate(timeout=600)
        assert p.returncode == 0, out.decode()[-2000:]
    exe = str(tmp_path / "plan_fuzz")
    # (host-side sanitizer runtimes only: no device code is instrumented anywhere in this test)
    link = subprocess.run([hipcc, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-o", exe] + objs,
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300)
    assert link.returncode == 0, link.stdout.decode()[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", LD_PRELOAD="")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300, env=env)
    assert run.returncode == 0 and run.stdout.decode().startswith("ok"), run.stdout.decode()[-3000:]
