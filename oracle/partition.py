"""Exhaustive definition of the heterogeneity-aware pipeline partition (Sec. III-C, Eq. 3 and Eq. 4).

TEST INFRASTRUCTURE ONLY; the product never imports this.  No dynamic programming, no memo: Eq. 4's recursion is
evaluated over every split position and every prefix of the sorted processor list, which is the search space the
paper's heuristic keeps (a stage's processors are consecutive in the list sorted by capability).

Notation: L layers 0..L-1; t[a][l] time of layer l on processor a; p[l] parameter bytes of layer l; act[l] bytes
of the activation between layer l and l+1; bw bytes per second between processors; `gpus` the sorted list.

    Q(i, j, S) = (1/|S|) * ( max_{a in S} sum_{l=i..j} t[a][l]  +  2 (|S|-1) sum_{l=i..j} p[l] / bw )        (Eq. 3)
    C(i, j, S) = min( Q(i, j, S),
                      min_{i <= k < j} min_{proper non-empty prefixes S1 of S}
                          max( C(i, k, S1), act[k] / bw, Q(k+1, j, S \\ S1) ) )                               (Eq. 4)

The first alternative (the range as ONE replicated stage) is the data-parallel time Alg. 1 initialises its table
with.  Pinned by hand-worked values in tests/test_partition.py.
"""
from __future__ import annotations


def Q(t, p, bw, i, j, S):
    m = len(S)
    comp = max(sum(t[a][l] for l in range(i, j + 1)) for a in S)
    sync = 2.0 * (m - 1) * sum(p[l] for l in range(i, j + 1)) / bw
    return (comp + sync) / m


def C(t, p, act, bw, i, j, S):
    """Returns (time, stages) with stages = [(first layer, last layer, processors)], in pipeline order."""
    best = (Q(t, p, bw, i, j, S), [(i, j, list(S))])
    for k in range(i, j):
        for n in range(1, len(S)):
            left_t, left_stages = C(t, p, act, bw, i, k, S[:n])
            cand = max(left_t, act[k] / bw, Q(t, p, bw, k + 1, j, S[n:]))
            if cand < best[0]:
                best = (cand, left_stages + [(k + 1, j, list(S[n:]))])
    return best
