"""Pins for the join oracle (Section 2.3): nested-loop equality join, the matrix form of Algorithm 1 (product
of the two key-indicator matrices over the common sorted domain) giving the same pairs, the paper's text
example (common key domain {0,1,2,3,4,7}), invariants of the row-matching matrix.  CPU only."""
import numpy as np
import pytest

from oracle import mmjoin_oracle as MJ


def _nested_loop(key_R, key_S):
    return [(i, j) for i, a in enumerate(key_R) for j, b in enumerate(key_S) if a == b]


def test_row_matching_matrix_equals_nested_loop_join_even_with_duplicates_on_both_sides():
    r = np.random.default_rng(1)
    key_R = r.integers(-5, 12, size=40)
    key_S = r.integers(-5, 12, size=15)              # duplicates: I may have several 1s per row
    _, I = MJ.row_matching_matrix(key_R, key_S)
    got = sorted(zip(I.row.tolist(), I.col.tolist()))
    assert got == sorted(_nested_loop(key_R, key_S))
    assert (I.data == 1).all()
    assert MJ.join_pairs(key_R, key_S) == sorted(_nested_loop(key_R, key_S))


def test_matrix_product_form_and_relational_form_are_the_same_relation():
    """Algorithm 1's product of indicator matrices against the dictionary match the GPU is compared with:
    same COO pairs, at most one 1 per row of I when the dimension keys are unique, row sums = match flags."""
    r = np.random.default_rng(3)
    key_S = r.permutation(np.arange(-400, 400, 3))[:150]
    key_R = np.concatenate([r.choice(key_S, size=500), r.integers(-1000, -500, size=40)])
    r.shuffle(key_R)
    fk, rows, cols = MJ.key_to_row(key_R, key_S)
    domain, I = MJ.row_matching_matrix(key_R, key_S)
    assert (np.diff(domain) > 0).all() and set(domain.tolist()) == set(key_R.tolist()) | set(key_S.tolist())
    order = np.lexsort((I.col, I.row))
    assert I.row[order].tolist() == rows.tolist() and I.col[order].tolist() == cols.tolist()
    per_row = np.asarray(I.tocsr().sum(axis=1)).reshape(-1)
    assert per_row.max() == 1 and (per_row == (fk >= 0)).all()


def test_paper_text_example_domain():
    """Section 2.3.1 step 1: the common domain of the running example is {0, 1, 2, 3, 4, 7}; the
    figure's tables are not available, so R and S here are ours, chosen to have that union."""
    key_R = np.array([2, 3, 0, 4, 7, 2, 1])
    key_S = np.array([7, 3, 2, 0, 4])
    domain, I = MJ.row_matching_matrix(key_R, key_S)
    assert domain.tolist() == [0, 1, 2, 3, 4, 7]
    fk, rows, cols = MJ.key_to_row(key_R, key_S)
    assert fk.tolist() == [2, 1, 3, 4, 0, 2, -1]      # by hand: position of each R key in S; key 1 has no match
    assert rows.tolist() == [0, 1, 2, 3, 4, 5] and cols.tolist() == [2, 1, 3, 4, 0, 2]


def test_key_to_row_is_dictionary_lookup_on_shuffled_sparse_keys():
    r = np.random.default_rng(2)
    key_S = r.permutation(np.arange(1000, 1000 + 37 * 300, 37))[:250]
    key_R = np.concatenate([r.choice(key_S, size=900), r.integers(0, 999, size=100)])   # 100 unmatched
    r.shuffle(key_R)
    fk, rows, cols = MJ.key_to_row(key_R, key_S)
    d = {int(k): j for j, k in enumerate(key_S)}
    assert fk.tolist() == [d.get(int(k), -1) for k in key_R]
    assert rows.tolist() == [i for i, k in enumerate(key_R) if int(k) in d]
    assert (cols == fk[rows]).all()
    assert len(rows) == (fk >= 0).sum()                 # nnz = rows of the materialised table
    with pytest.raises(ValueError):
        MJ.key_to_row(key_R, np.array([5, 6, 5]))
