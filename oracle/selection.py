"""CPU oracle for the offline cluster-combination selection (paper Sec. 4.2, Algorithm 1) and for
longest-cached-prefix lookup (Sec. 2.3 / 4.2: reuse up to the first mismatch, cut the tail).
TEST INFRASTRUCTURE ONLY - never imported by the product path.

A data sample is the ordered tuple of clusters it activates (the order is the fixed, theme-based
one, so equal sets give equal tuples).  The cached set C holds cluster prefixes.  For a sample,
the number of hit clusters is the length of its longest prefix that is in C; coverage(D, C) is
the sum over the samples.  Each of the N rounds looks at every prefix of every sample that is a
single cluster or extends a member of C by one cluster, and adds the one whose addition raises
the coverage most.

Readings where the paper is silent: among candidates with equal gain the smallest tuple (ordinary
tuple comparison of cluster ids) wins; a candidate already in C is not a candidate; when no
candidate is left the selection stops early with fewer than N members.
"""
from __future__ import annotations


def coverage(samples, cached) -> int:
    """Sum over the samples of the length of the longest prefix of the sample that is cached."""
    cached = set(tuple(c) for c in cached)
    total = 0
    for s in samples:
        s = tuple(s)
        best = 0
        for n in range(1, len(s) + 1):
            if s[:n] in cached:
                best = n
        total += best
    return total


def select_combinations(samples, budget: int):
    """Algorithm 1.  Returns (list of chosen prefixes in the order chosen, coverage after each)."""
    samples = [tuple(int(c) for c in s) for s in samples]
    prefixes = set()
    for s in samples:
        for n in range(1, len(s) + 1):
            prefixes.add(s[:n])
    chosen, trace = [], []
    for _ in range(budget):
        have = set(chosen)
        options = [p for p in prefixes if p not in have and (len(p) == 1 or p[:-1] in have)]
        if not options:
            break
        base = coverage(samples, chosen)
        best, best_gain = None, -1
        for p in sorted(options):                  # ascending: the first of equal gains stays
            gain = coverage(samples, chosen + [p]) - base
            if gain > best_gain:
                best, best_gain = p, gain
        chosen.append(best)
        trace.append(base + best_gain)
    return chosen, trace


def longest_cached_prefix(cached_sequences, prompt):
    """(index of a cached token sequence sharing the longest common prefix with `prompt`, its
    length); the lowest index among equals; (-1, 0) when nothing matches."""
    best_i, best_n = -1, 0
    for i, seq in enumerate(cached_sequences):
        n = 0
        while n < len(seq) and n < len(prompt) and int(seq[n]) == int(prompt[n]):
            n += 1
        if n > best_n:
            best_i, best_n = i, n
    return best_i, best_n
