"""CPU oracle for group discovery (Sections 2.4.1-2.4.2) and for ordering an aggregate's result
(Section 2.5).

TEST INFRASTRUCTURE ONLY (same rules as lq_oracle): never imported by the GPU package.

group_domain follows the paper's procedure for finding the groups of one table: for a single
attribute the groups are its distinct values ("numerical unique"); for several attributes the
distinct tuples are found by sorting the tuples and keeping the first of every run of equal
neighbours (the sort-unique procedure the paper adopts).  Written out in those steps:
  1. order the rows lexicographically by their tuples (first column most significant)
  2. a row starts a new group iff its tuple differs from the previous row's in that order
  3. the running count of group starts, minus one, is the row's group code
so that group codes number the distinct tuples in ascending lexicographic order.  Because the codes
follow the sorted domain, a result indexed by them is already ordered by the grouping attributes:
that is how Section 2.5 folds sorting on keys into the matrix form.

order_groups is the relational definition of ORDER BY on the populated groups of a dense
aggregate result, with ties broken by ascending group index so that the answer is unique.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

KEY_GROUP_COLUMN = 0      # the code of grouping dimension `index` (position among the grouping dimensions)
KEY_SUM = 1               # sums[index][g]
KEY_COUNT = 2             # counts[g]


def group_domain(cols: Sequence[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (values [card x n_cols] int64, code [rows] int64)."""
    cols = [np.asarray(c).astype(np.int64).reshape(-1) for c in cols]
    r = len(cols[0])
    assert all(len(c) == r for c in cols)
    if r == 0:
        return np.zeros((0, len(cols)), dtype=np.int64), np.zeros((0,), dtype=np.int64)
    tuples = np.stack(cols, axis=1)
    order = np.lexsort(tuple(cols[::-1]))                 # step 1 (lexsort's last key is the primary one)
    sorted_t = tuples[order]
    starts = np.ones(r, dtype=bool)                       # step 2
    starts[1:] = np.any(sorted_t[1:] != sorted_t[:-1], axis=1)
    code_sorted = np.cumsum(starts) - 1                   # step 3
    code = np.empty(r, dtype=np.int64)
    code[order] = code_sorted
    return sorted_t[starts], code


def order_groups(group_card: Sequence[int], sums: np.ndarray, counts: np.ndarray,
                 keys: Sequence[Tuple[int, int, bool]]) -> np.ndarray:
    """Populated groups (counts > 0) ordered by `keys`, each (kind, index, descending); ties by group index.

    group_card lists the cardinalities of the grouping dimensions in order; group g decomposes as
    a mixed-radix number over them, last one fastest.
    """
    sums = np.asarray(sums, dtype=np.int64)
    counts = np.asarray(counts, dtype=np.int64)
    G = int(np.prod(group_card)) if len(group_card) else 1
    assert counts.shape == (G,)

    def digits(g):
        out = []
        for c in reversed(group_card):
            out.append(g % c)
            g //= c
        return out[::-1]

    def sort_key(g):
        k = []
        for kind, index, desc in keys:
            if kind == KEY_GROUP_COLUMN:
                v = digits(g)[index]
            elif kind == KEY_SUM:
                v = int(sums[index][g])
            else:
                v = int(counts[g])
            k.append(-v if desc else v)
        k.append(g)
        return tuple(k)

    populated = [g for g in range(G) if counts[g] > 0]
    return np.array(sorted(populated, key=sort_key), dtype=np.int64)
