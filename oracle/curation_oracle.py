"""Plain-Python statement of the paper's metrics and curation rules (test infrastructure only).

Written from Equations 1-3, Section 3.5 (the three parts of the curated set), Section 4.2
(pass@k) and Section 6 (difficulty bins by average reasoning length), with loops and dicts and no
shared code with the library.  Where the paper is silent (ties, how the single-operator samples of
part (c) are picked) it takes the reading documented in include/concur_curation.h.
Pinned by tests/test_curation.py: hand-worked tables, the paper's own bin thresholds and counts'
arithmetic (3,934 + 414 + 544 = 4,892).
"""
import math


def speedup(t_torch, t_kernel, correct):                      # Equation 1
    return [tt / tk if c else 0.0 for tt, tk, c in zip(t_torch, t_kernel, correct)]


def fast_p(speedups, p):                                      # Equation 2
    return sum(1 for s in speedups if s > p) / len(speedups)


def exec_pass_at_k(correct_rows):                             # Section 4.2
    return sum(1 for row in correct_rows if any(row)) / len(correct_rows)


def fast1_pass_at_k(speedup_rows):
    return sum(1 for row in speedup_rows if any(s > 1.0 for s in row)) / len(speedup_rows)


def arl(length_rows):                                         # Equation 3
    n, m = len(length_rows), len(length_rows[0])
    return math.fsum(x for row in length_rows for x in row) / (n * m)


def difficulty_bin(task_arl, lo=4000.0, hi=8500.0):           # Section 6
    return 0 if task_arl < lo else (2 if task_arl > hi else 1)


def select(task_id, speedups, reasoning_len, single_op, threshold=5.0, quota=544):   # Section 3.5
    n = len(task_id)
    flags = [0] * n
    by_task = {}
    for i in range(n):
        by_task.setdefault(task_id[i], []).append(i)
    for members in by_task.values():
        shortest = min(members, key=lambda i: (reasoning_len[i], i))
        if speedups[shortest] > 0 and all(speedups[shortest] >= speedups[j] for j in members):
            flags[shortest] |= 1
    for i in range(n):
        if speedups[i] > threshold:
            flags[i] |= 2
    pool = sorted((i for i in range(n) if single_op[i] and speedups[i] > 0 and flags[i] == 0),
                  key=lambda i: (reasoning_len[i], i))
    for i in pool[:quota]:
        flags[i] |= 4
    return flags
