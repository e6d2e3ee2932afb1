"""Metrics and curation rules (Equations 1-3, Sections 3.5, 4.2, 6): the plain-Python oracle is
pinned to hand-worked tables and to what the definitions fix, then the library's host functions
are compared with it exactly on a seeded synthetic record table (no GPU involved)."""
import os

import numpy as np
import pytest

from oracle import curation_oracle as ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(os.path.join(ROOT, "paper_2510_07356_amd", "libgqa_decode.so")):
        from paper_2510_07356_amd.build import build_library
        build_library()
    from paper_2510_07356_amd import binding
    return binding


def record_table(seed, tasks=1200, gens=5):
    """Synthetic stand-in for the paper's synthesis output: `gens` generations per task, about
    half correct, log-normal speedups with a thin tail above 5, reasoning lengths of a few
    thousand tokens that grow with task difficulty, a third of the tasks single-operator."""
    rng = np.random.Generator(np.random.PCG64([seed, 77]))
    n = tasks * gens
    task_id = np.repeat(rng.permutation(tasks) * 3 + 11, gens)
    difficulty = np.repeat(rng.lognormal(8.4, 0.5, tasks), gens)
    length = np.maximum(200, difficulty * rng.lognormal(0.0, 0.35, n)).astype(np.int32)
    correct = rng.random(n) < 0.55
    t_torch = rng.lognormal(0.0, 0.6, n)
    t_kernel = t_torch / rng.lognormal(0.1, 0.9, n)
    single = np.repeat(rng.random(tasks) < 0.33, gens)
    order = rng.permutation(n)                      # records of a task are not adjacent
    return dict(task_id=task_id[order], length=length[order], correct=correct[order].astype(np.uint8),
                t_torch=t_torch[order], t_kernel=t_kernel[order], single=single[order].astype(np.uint8))


# ---- pins of the oracle -----------------------------------------------------------------------
def test_speedup_and_fast_p_hand_table():
    s = ref.speedup([2.0, 3.0, 1.0, 4.0], [1.0, 6.0, 1.0, 0.5], [1, 1, 0, 1])
    assert s == [2.0, 0.5, 0.0, 8.0]                       # Equation 1; incorrect -> 0
    assert ref.fast_p(s, 0.0) == 0.75                      # fast_0 is the correctness rate
    assert ref.fast_p(s, 1.0) == 0.5
    assert ref.fast_p(s, 2.0) == 0.25                      # strict inequality
    assert ref.fast_p(s, 8.0) == 0.0


def test_fast_p_is_monotone_and_fast0_is_exec():
    t = record_table(1)
    s = ref.speedup(t["t_torch"], t["t_kernel"], t["correct"])
    assert ref.fast_p(s, 0.0) == t["correct"].mean()
    vals = [ref.fast_p(s, p) for p in (0.0, 0.5, 1.0, 2.0, 5.0, 50.0)]
    assert all(a >= b for a, b in zip(vals, vals[1:]))


def test_pass_at_k_hand_table():
    assert ref.exec_pass_at_k([[0, 0, 1], [0, 0, 0], [1, 1, 1], [0, 1, 0]]) == 0.75
    assert ref.fast1_pass_at_k([[0.0, 1.0, 0.9], [0.0, 1.01, 0.0]]) == 0.5     # speedup must exceed 1
    one = [[1], [0], [1], [1]]
    assert ref.exec_pass_at_k(one) == 0.75                 # k = 1 is the plain rate


def test_arl_and_bins():
    assert ref.arl([[1000, 3000], [5000, 7000]]) == 4000.0              # Equation 3
    assert ref.arl([[7]]) == 7.0
    # Section 6: easy below 4000, hard above 8500, the two thresholds themselves are medium
    assert [ref.difficulty_bin(x) for x in (0, 3999.9, 4000, 6000, 8500, 8500.1)] == [0, 0, 1, 1, 1, 2]


def test_selection_hand_table():
    #         task   speedup  length  single
    rows = [(1, 2.0, 100, 0),   # shortest of task 1 and fastest        -> (a)
            (1, 1.5, 200, 0),
            (2, 1.0, 100, 0),   # shortest of task 2 but not fastest    -> nothing
            (2, 6.0, 300, 0),   # > 5                                   -> (b)
            (3, 0.0, 50, 1),    # shortest of task 3 but incorrect      -> nothing
            (3, 1.2, 80, 1),    # correct single-operator, length 80    -> (c) first
            (3, 1.1, 60, 1),    # correct single-operator, length 60    -> (c) first
            (4, 7.0, 10, 1),    # shortest, fastest and > 5             -> (a) and (b)
            (4, 7.0, 20, 1),    # ties the best, > 5                    -> (b)
            (5, 3.0, 500, 1)]   # only generation of task 5             -> (a)
    t, s, l, o = (list(c) for c in zip(*rows))
    assert ref.select(t, s, l, o, 5.0, 1) == [1, 0, 0, 2, 0, 0, 4, 3, 2, 1]
    assert ref.select(t, s, l, o, 5.0, 5) == [1, 0, 0, 2, 0, 4, 4, 3, 2, 1]
    assert ref.select(t, s, l, o, 5.0, 0) == [1, 0, 0, 2, 0, 0, 0, 3, 2, 1]


def test_selection_invariants():
    t = record_table(2)
    s = ref.speedup(t["t_torch"], t["t_kernel"], t["correct"])
    flags = ref.select(t["task_id"], s, t["length"], t["single"], 5.0, 544)
    f = np.array(flags)
    sp = np.array(s)
    assert ((f & 1) != 0).sum() <= len(set(t["task_id"]))           # at most one (a) sample per task
    assert np.all(sp[f != 0] > 0)                                   # nothing incorrect is kept
    assert np.array_equal((f & 2) != 0, sp > 5.0)
    c = (f & 4) != 0
    assert c.sum() <= 544 and np.all(t["single"][c] == 1) and not np.any(f[c] & 3)
    # the three parts are disjoint and add up to the selection (as the counts of Section 3.5 do)
    a, b_only = ((f & 1) != 0).sum(), ((f & 3) == 2).sum()
    assert a + b_only + c.sum() == (f != 0).sum()


# ---- the library against the oracle -------------------------------------------------------------
@pytest.mark.parametrize("seed", [3, 4])
def test_library_matches_oracle(lib, seed):
    t = record_table(seed)
    s_ref = ref.speedup(t["t_torch"], t["t_kernel"], t["correct"])
    s = lib.concur_speedup(t["t_torch"], t["t_kernel"], t["correct"])
    assert s.tolist() == s_ref                                       # one IEEE division each: exact
    for p in (0.0, 0.5, 1.0, 2.0, 5.0):
        assert lib.concur_fast_p(s, p) == ref.fast_p(s_ref, p)
    tasks, gens = 1200, 5
    order = np.argsort(t["task_id"], kind="stable")
    corr = t["correct"][order].reshape(tasks, gens)
    sp = s[order].reshape(tasks, gens)
    L = t["length"][order].reshape(tasks, gens)
    assert lib.concur_exec_pass_at_k(corr) == ref.exec_pass_at_k(corr.tolist())
    assert lib.concur_fast1_pass_at_k(sp) == ref.fast1_pass_at_k(sp.tolist())
    assert lib.concur_arl(L) == ref.arl(L.tolist())
    task_arl = L.mean(axis=1)
    assert lib.concur_difficulty_bins(task_arl).tolist() == [ref.difficulty_bin(x) for x in task_arl]
    for quota in (0, 50, 544, 10**6):
        flags, counts = lib.concur_select(t["task_id"], s, t["length"], t["single"], 5.0, quota)
        want = ref.select(t["task_id"].tolist(), s_ref, t["length"].tolist(), t["single"].tolist(), 5.0, quota)
        assert flags.tolist() == want
        w = np.array(want)
        assert counts == (int(((w & 1) != 0).sum()), int(((w & 3) == 2).sum()), int(((w & 4) != 0).sum()))


def test_library_edge_cases(lib):
    assert np.isnan(lib.concur_fast_p([], 1.0))
    flags, counts = lib.concur_select([], [], [], [], 5.0, 544)
    assert flags.size == 0 and counts == (0, 0, 0)
    with pytest.raises(ValueError):
        lib.concur_speedup([1.0], [0.0], [1])                        # correct but no run time
    assert lib.concur_speedup([1.0], [0.0], [0]).tolist() == [0.0]
    with pytest.raises(ValueError):
        lib.concur_difficulty_bins([1.0], lo=9000.0, hi=4000.0)
    # ties in reasoning length: the earlier record is the shortest
    flags, _ = lib.concur_select([7, 7], [1.0, 2.0], [100, 100], [0, 0], 5.0, 0)
    assert flags.tolist() == [0, 0]
    flags, _ = lib.concur_select([7, 7], [2.0, 1.0], [100, 100], [0, 0], 5.0, 0)
    assert flags.tolist() == [1, 0]
