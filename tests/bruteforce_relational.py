"""Brute-force relational evaluation used to pin the oracle on tiny inputs.

Tables are lists of Python tuples with explicit key values; joins are nested
loops on key equality.  Nothing here knows about row indices, indicator
matrices or the oracle.
"""
from __future__ import annotations


def star_join(fact_rows, dim_tables):
    """fact_rows: list of (features tuple, [key_0, key_1, ...]).
    dim_tables: list of lists of (pk, features tuple).
    Returns the joined tuples (fact features, then each dimension's features) in fact order;
    a fact row appears once per combination of matching dimension rows (inner join)."""
    out = []
    for feats, keys in fact_rows:
        partial = [tuple(feats)]
        for key, table in zip(keys, dim_tables):
            nxt = []
            for p in partial:
                for pk, dfeats in table:
                    if pk == key:
                        nxt.append(p + tuple(dfeats))
            partial = nxt
        out.extend(partial)
    return out


def mlp(t, weights, biases):
    """Plain-Python (ReLU-)MLP on one tuple; weights[j][q][o]."""
    a = list(t)
    for j, W in enumerate(weights):
        n_out = len(W[0])
        b = []
        for o in range(n_out):
            s = 0.0
            for q in range(len(a)):
                s += a[q] * W[q][o]
            if biases is not None and biases[j] is not None:
                s += biases[j][o]
            if j < len(weights) - 1:
                s = max(s, 0.0)
            b.append(s)
        a = b
    return a


def filter_join_group_sum(fact_rows, dim_tables, group_attr, predicates, n_measures):
    """SELECT group attrs, SUM(measure_m), COUNT(*) FROM fact JOIN dims WHERE preds GROUP BY attrs.

    fact_rows: list of ([key_0..], [measure_0..], fact_ok bool)
    dim_tables[k]: list of (pk, attrs dict)
    group_attr[k]: attribute name of dimension k to group by, or None
    predicates[k]: function(attrs) -> bool, or None
    Returns {group tuple: ([sums], count)} holding only non-empty groups."""
    res = {}
    for keys, meas, ok in fact_rows:
        if not ok:
            continue
        matches = [()]
        for k, (key, table) in enumerate(zip(keys, dim_tables)):
            nxt = []
            for g in matches:
                for pk, attrs in table:
                    if pk != key:
                        continue
                    if predicates[k] is not None and not predicates[k](attrs):
                        continue
                    nxt.append(g + ((attrs[group_attr[k]],) if group_attr[k] else ()))
            matches = nxt
        for g in matches:
            sums, cnt = res.get(g, ([0] * n_measures, 0))
            res[g] = ([s + int(m) for s, m in zip(sums, meas)], cnt + 1)
    return res
