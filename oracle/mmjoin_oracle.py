"""CPU oracle for the join that feeds the fused paths (Section 2.3): one key column per side, the
dimension side S holding unique keys.

TEST INFRASTRUCTURE ONLY (same rules as lq_oracle): never imported by the GPU package.

The oracle is the relational meaning of an equi-join, written out: fact row i matches dimension row j
exactly when their key values are equal (Section 2.3: the row-matching matrix has I[i, j] = 1 for
such pairs and nothing else).  With unique keys on S every fact row has at most one match, so I is
the vector fk[i] = the matching S row, or -1 when the key does not occur in S; rows without a match do
not appear in the join result (Section 2.3.2).  The row-mapping matrices I_R and I_S of Section 2.3.3
are the COO index vectors of I, aligned with the materialised rows m = 0 .. nnz-1 in ascending R row.

``row_matching_matrix`` is the same relation obtained the way the matrix-multiplication join obtains it
(Algorithm 1: positions in a common sorted key domain, one indicator matrix per side, their product).
It is not what the GPU results are compared with; the pins check that both forms give the same pairs.
"""
from __future__ import annotations

import numpy as np
import scipy.sparse as sp


def join_pairs(key_R, key_S):
    """All (i, j) with key_R[i] == key_S[j], ascending in (i, j); duplicates allowed on both sides."""
    key_R = np.asarray(key_R).reshape(-1)
    key_S = np.asarray(key_S).reshape(-1)
    rows_of = {}
    for j, k in enumerate(key_S.tolist()):
        rows_of.setdefault(k, []).append(j)
    return [(i, j) for i, k in enumerate(key_R.tolist()) for j in rows_of.get(k, ())]


def key_to_row(key_R, key_S):
    """fk[i] = row of S whose key equals key_R[i], -1 if none; plus the COO (rows, cols) of I in
    materialised-row order (ascending R row).  key_S must not contain duplicates."""
    key_R = np.asarray(key_R).reshape(-1)
    key_S = np.asarray(key_S).reshape(-1)
    row_of = {}
    for j, k in enumerate(key_S.tolist()):
        if k in row_of:
            raise ValueError("duplicate keys on the dimension side")
        row_of[k] = j
    fk = np.array([row_of.get(k, -1) for k in key_R.tolist()], dtype=np.int32).reshape(-1)
    rows = np.nonzero(fk >= 0)[0].astype(np.int64)
    cols = fk[rows].astype(np.int64)
    return fk, rows, cols


def row_matching_matrix(key_R, key_S):
    """(domain, I): the sorted common key domain and the row-matching matrix as the product of the two
    key-indicator matrices over that domain (Algorithm 1), in scipy COO form."""
    key_R = np.asarray(key_R).astype(np.int64).reshape(-1)
    key_S = np.asarray(key_S).astype(np.int64).reshape(-1)
    domain = np.union1d(key_R, key_S)

    def indicator(keys):
        position = np.searchsorted(domain, keys)
        return sp.csr_matrix((np.ones(len(keys), dtype=np.int64), (np.arange(len(keys)), position)),
                             shape=(len(keys), len(domain)))
    return domain, (indicator(key_R) @ indicator(key_S).T).tocoo()
