"""CPU oracle for the matrix-multiplication join (Section 2.3, Algorithm 1) restricted to what
feeds the fused paths: one key column per side, the dimension side S holding unique keys.

TEST INFRASTRUCTURE ONLY (same rules as lq_oracle): never imported by the GPU package.

The steps are Algorithm 1's, with numpy / scipy primitives for its set union, dictionary lookups,
CSR construction and sparse product:
  1. key_domain = sorted union of the two key columns; key_dict maps a key to its position
  2. MAT_R [r_R x |domain|] and MAT_S [r_S x |domain|]: one 1 per row, in the column of the row's key
  3. I = MAT_R * MAT_S^T, taken in COO form: I[i, j] = 1 iff row i of R matches row j of S
  4. row-mapping matrices of Section 2.3.3: the COO row and column index vectors, aligned with
     m = <0 .. nnz-1>, are I_R and I_S (materialised row m comes from R row rows[m], S row cols[m])
For a key column S without duplicates every row of I has at most one 1, so I is equivalently the
vector fk[i] = the matching S row, or -1 when the key of R row i does not occur in S (such rows do
not appear in the join result, Section 2.3.2).
"""
from __future__ import annotations

import numpy as np
import scipy.sparse as sp


def mmjoin(key_R, key_S):
    """Returns (domain, I) with I the scipy COO row-matching matrix of Algorithm 1."""
    key_R = np.asarray(key_R).astype(np.int64).reshape(-1)
    key_S = np.asarray(key_S).astype(np.int64).reshape(-1)
    domain = np.union1d(key_R, key_S)                               # line 1 (sorted, unique)
    col_R = np.searchsorted(domain, key_R)                          # key_dict[key] for every R row
    col_S = np.searchsorted(domain, key_S)
    MAT_R = sp.csr_matrix((np.ones(len(key_R), dtype=np.int64), (np.arange(len(key_R)), col_R)),
                          shape=(len(key_R), len(domain)))
    MAT_S = sp.csr_matrix((np.ones(len(key_S), dtype=np.int64), (np.arange(len(key_S)), col_S)),
                          shape=(len(key_S), len(domain)))
    I = (MAT_R @ MAT_S.T).tocoo()
    return domain, I


def key_to_row(key_R, key_S):
    """fk[i] = row of S whose key equals key_R[i], -1 if none; plus the COO (rows, cols) of I in
    materialised-row order (ascending R row).  key_S must not contain duplicates."""
    key_S = np.asarray(key_S).reshape(-1)
    if len(np.unique(key_S)) != len(key_S):
        raise ValueError("duplicate keys on the dimension side")
    _, I = mmjoin(key_R, key_S)
    order = np.lexsort((I.col, I.row))
    rows, cols = I.row[order].astype(np.int64), I.col[order].astype(np.int64)
    fk = np.full(len(np.asarray(key_R).reshape(-1)), -1, dtype=np.int32)
    fk[rows] = cols
    return fk, rows, cols
