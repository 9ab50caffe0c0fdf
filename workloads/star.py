"""Seeded synthetic star schemas shaped like the paper's workloads.

This module only draws inputs (tables, key columns, weights, masks, group
codes).  It holds none of the method's arithmetic and is the one module both
the CPU oracle's callers and the GPU library's callers may share.

Shapes follow the synthetic star schema and the SSB cardinalities of the
paper's experiment section (Tables 3-5): a large fact table, a few dimension
tables of 1e3..1e6 rows, a linear operator or small MLP on the joined width.
The SSB data itself is not available; these inputs stand in for it.

Every generator returns torch tensors (CPU by default; on ``device`` when one
is given, using a seeded ``torch.Generator`` there so that 1e8-row inputs never
cross PCIe).  CPU draws use ``numpy.random.default_rng(seed)``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
import torch

SEED0 = 230608367


@dataclass
class PredictWorkload:
    """Inputs of one fused join + predict problem."""
    name: str
    n: int
    X: Optional[torch.Tensor]            # [n x c_f] or None when c_f == 0
    dims: List[torch.Tensor]             # D_k [r_k x c_k]
    fks: List[torch.Tensor]              # int32 [n], values in [0, r_k)
    weights: List[torch.Tensor]          # W_j [in x out]; W_0 rows: fact cols, dim 0, dim 1, ...
    biases: List[Optional[torch.Tensor]]
    dtype: torch.dtype = torch.float32

    @property
    def c_f(self) -> int:
        return 0 if self.X is None else int(self.X.shape[1])

    @property
    def k(self) -> int:
        return self.c_f + sum(int(d.shape[1]) for d in self.dims)


@dataclass
class GroupByWorkload:
    """Inputs of one masked star-join group-by."""
    name: str
    n: int
    fks: List[torch.Tensor]              # int32 [n]
    dim_rows: List[int]
    dim_mask: List[Optional[torch.Tensor]]   # uint8 [r_k] or None
    dim_code: List[Optional[torch.Tensor]]   # int32 [r_k] or None
    group_card: List[int]                # 1 where dim_code is None
    fact_mask: Optional[torch.Tensor]    # uint8 [n] or None
    measures: List[torch.Tensor]         # int32 [n]
    attrs: dict = field(default_factory=dict)  # raw dimension attributes (for brute-force checks)

    @property
    def G(self) -> int:
        g = 1
        for c in self.group_card:
            g *= c
        return g


class _Draw:
    """Normal / integer draws on the CPU (numpy) or on a torch device."""

    def __init__(self, seed: int, device=None):
        self.device = None if device is None else torch.device(device)
        if self.device is None or self.device.type == "cpu":
            self.device = None
            self.rng = np.random.default_rng(seed)
        else:
            self.gen = torch.Generator(device=self.device)
            self.gen.manual_seed(seed)

    def normal(self, shape, sigma=1.0, dtype=torch.float32) -> torch.Tensor:
        if self.device is None:
            a = self.rng.standard_normal(size=shape, dtype=np.float32)
            t = torch.from_numpy(a)
        else:
            t = torch.randn(shape, generator=self.gen, device=self.device, dtype=torch.float32)
        if sigma != 1.0:
            t = t * float(sigma)
        return t.to(dtype).contiguous()

    def small_ints(self, shape, lo, hi, dtype=torch.float32) -> torch.Tensor:
        """Integer-valued floats in [lo, hi): exactly representable in bf16 when |v| <= 256."""
        return self.integers(shape, lo, hi).to(dtype).contiguous()

    def integers(self, shape, lo, hi) -> torch.Tensor:
        """int32 uniform in [lo, hi)."""
        if self.device is None:
            a = self.rng.integers(lo, hi, size=shape, dtype=np.int64).astype(np.int32)
            return torch.from_numpy(a)
        return torch.randint(lo, hi, shape, generator=self.gen, device=self.device,
                             dtype=torch.int32)

    def uniform(self, n) -> torch.Tensor:
        if self.device is None:
            return torch.from_numpy(self.rng.random(n))
        return torch.rand(n, generator=self.gen, device=self.device, dtype=torch.float64)

    def permutation(self, r) -> torch.Tensor:
        if self.device is None:
            return torch.from_numpy(self.rng.permutation(r).astype(np.int64))
        return torch.randperm(r, generator=self.gen, device=self.device)

    def zipf(self, n, r, s, permute=True) -> torch.Tensor:
        """Bounded Zipf(s) over ranks 1..r by inverse CDF; rank -> row through a fixed
        random permutation (or the identity, which keeps the hot rows contiguous)."""
        dev = self.device if self.device is not None else torch.device("cpu")
        w = torch.arange(1, r + 1, dtype=torch.float64, device=dev).pow(-float(s))
        cdf = torch.cumsum(w, 0)
        cdf = cdf / cdf[-1]
        perm = self.permutation(r) if permute else None
        out = torch.empty(n, dtype=torch.int32, device=dev)
        step = 1 << 24
        for lo in range(0, n, step):
            hi = min(n, lo + step)
            u = self.uniform(hi - lo).to(dev)
            rank = torch.searchsorted(cdf, u).clamp_(max=r - 1)
            out[lo:hi] = (perm[rank] if perm is not None else rank).to(torch.int32)
        return out


def make_predict(name: str, n: int, c_f: int, dim_rows: Sequence[int], dim_cols: Sequence[int],
                 layers: Sequence[int], *, seed: int, dtype=torch.float32, device=None,
                 w_sigma: Optional[Sequence[float]] = None, bias: bool = False,
                 fk_dist: str = "uniform", zipf_s: float = 1.1, zipf_permute: bool = True,
                 integer_valued: bool = False) -> PredictWorkload:
    """Generic star schema + (ReLU-)MLP of output widths ``layers``.

    ``integer_valued`` draws small integers instead of normals (features in
    [-4, 4], weights in [-2, 2]) so that every product and sum is exact in
    fp32 and fp64 alike.
    """
    d = _Draw(seed, device)
    k = c_f + sum(dim_cols)

    def feat(shape):
        return d.small_ints(shape, -4, 5, dtype) if integer_valued else d.normal(shape, 1.0, dtype)

    X = feat((n, c_f)) if c_f > 0 else None
    dims = [feat((int(r), int(c))) for r, c in zip(dim_rows, dim_cols)]
    fks = []
    for r in dim_rows:
        if fk_dist == "uniform":
            fks.append(d.integers((n,), 0, int(r)))
        elif fk_dist == "zipf":
            fks.append(d.zipf(n, int(r), zipf_s, zipf_permute))
        else:
            raise ValueError(fk_dist)
    widths = [k] + list(layers)
    weights, biases = [], []
    for j in range(len(layers)):
        sig = 1.0 if w_sigma is None else w_sigma[j]
        shape = (widths[j], widths[j + 1])
        weights.append(d.small_ints(shape, -2, 3, dtype) if integer_valued
                       else d.normal(shape, sig, dtype))
        biases.append((d.small_ints((widths[j + 1],), -2, 3, dtype) if integer_valued
                       else d.normal((widths[j + 1],), sig, dtype)) if bias else None)
    return PredictWorkload(name, n, X, dims, fks, weights, biases, dtype)


# --- the five named configurations (index = position in the baseline list) ---------------

def c1_tiny_linear(device=None, n: int = 10_000) -> PredictWorkload:
    """Linear regression (l = 1) over a 2-dimension star; launch-latency sized."""
    return make_predict("c1_tiny_linear", n, 4, (100, 50), (8, 8), (1,), seed=SEED0 + 0,
                        device=device)


def c2_mlp(device=None, n: int = 10_000_000) -> PredictWorkload:
    """2-layer MLP 100 -> 64 -> 1 over a 3-dimension star (setting-1-like cardinalities)."""
    return make_predict("c2_mlp", n, 4, (1_000, 10_000, 100_000), (32, 32, 32), (64, 1),
                        seed=SEED0 + 1, device=device, w_sigma=(0.1, 0.1))


def c4_skewed(device=None, n: int = 100_000_000, permute: bool = True) -> PredictWorkload:
    """Linear model with 4 outputs, 2 dimensions of 1e6 x 128, Zipf(1.1) keys."""
    return make_predict("c4_skewed" + ("" if permute else "_contig"), n, 8,
                        (1_000_000, 1_000_000), (128, 128), (4,), seed=SEED0 + 3, device=device,
                        fk_dist="zipf", zipf_s=1.1, zipf_permute=permute)


def c5_wide_bf16(device=None, n: int = 50_000_000) -> PredictWorkload:
    """bf16 MLP 1024 -> 256 -> 16, no fact columns, 4 dimensions of 1e4 x 256.
    Weights N(0, 1/fan_in) so activations stay O(1)."""
    return make_predict("c5_wide_bf16", n, 0, (10_000,) * 4, (256,) * 4, (256, 16),
                        seed=SEED0 + 4, device=device, dtype=torch.bfloat16,
                        w_sigma=(1.0 / 32.0, 1.0 / 16.0))


def c3_groupby(device=None, n: int = 6_000_000, variant: str = "A", n_measures: int = 1,
               dim_rows: Sequence[int] = (2_556, 30_000, 2_000, 200_000)) -> GroupByWorkload:
    """SSB-sf1-shaped aggregate: 4 joins, two mask dimensions, GROUP BY 7 x 25, SUM.

    dim0 carries a7 in 0..6; dims 1-3 carry a5 in 0..4 and b25 = 5*a5 + U{0..4}.
    Grouping: dim0.a7 x dim1.b25.  Variant A masks dim2.a5 == 2 (20 %) and
    dim3.b25 in {3, 11, 19} (12 %): about 2.4 % of fact rows survive.  Variant B
    adds dim1.a5 == 1, which leaves 35 of the 175 groups populated.
    """
    d = _Draw(SEED0 + 2 + (0 if variant == "A" else 100), device)
    dev = d.device if d.device is not None else torch.device("cpu")
    fks = [d.integers((n,), 0, int(r)) for r in dim_rows]
    a7 = d.integers((dim_rows[0],), 0, 7)
    a5 = [None] + [d.integers((dim_rows[k],), 0, 5) for k in (1, 2, 3)]
    b25 = [None] + [(a5[k] * 5 + d.integers((dim_rows[k],), 0, 5)).to(torch.int32) for k in (1, 2, 3)]
    measures = [d.integers((n,), 1, 100_001) for _ in range(n_measures)]
    m2 = (a5[2] == 2).to(torch.uint8)
    m3 = ((b25[3] == 3) | (b25[3] == 11) | (b25[3] == 19)).to(torch.uint8)
    m1 = (a5[1] == 1).to(torch.uint8) if variant == "B" else None
    return GroupByWorkload(
        name=f"c3_groupby_{variant}", n=n, fks=fks, dim_rows=[int(r) for r in dim_rows],
        dim_mask=[None, m1, m2, m3], dim_code=[a7, b25[1], None, None],
        group_card=[7, 25, 1, 1], fact_mask=None, measures=measures,
        attrs={"a7": a7, "a5": a5, "b25": b25, "device": str(dev)})


def sample_rows(n: int, head: int = 4096, stride: int = 9973) -> torch.Tensor:
    """Deterministic row sample for spot checks at sizes the oracle cannot sweep:
    the first and last ``head`` rows plus every ``stride``-th row."""
    idx = set(range(min(head, n))) | set(range(max(0, n - head), n)) | set(range(0, n, stride))
    return torch.tensor(sorted(idx), dtype=torch.int64)


def take_rows(w: PredictWorkload, rows: torch.Tensor) -> PredictWorkload:
    """The sub-problem made of the given fact rows (tables and model unchanged), on the CPU."""
    dev_rows = rows.to(w.fks[0].device)
    X = None if w.X is None else w.X[dev_rows].cpu()
    return PredictWorkload(w.name + "_sample", int(rows.numel()), X,
                           [d.cpu() for d in w.dims], [f[dev_rows].cpu() for f in w.fks],
                           [x.cpu() for x in w.weights],
                           [None if b is None else b.cpu() for b in w.biases], w.dtype)


# --- decision trees in matrix form (Section 3.3.1) ----------------------------------------

@dataclass
class TreeModel:
    """A binary decision tree both as a linked structure and in the matrix form of the paper."""
    feature: torch.Tensor        # int32 [p]   column of the joined table tested by node q
    threshold: torch.Tensor      # fp32  [p]   node q goes to its True side when value > threshold
    H: torch.Tensor              # int8  [p x l]  +1 / -1 / 0 path matrix
    true_child: List[int]        # >= 0: internal node, < 0: leaf -(id + 1)
    false_child: List[int]

    @property
    def n_nodes(self) -> int:
        return int(self.feature.shape[0])

    @property
    def n_leaves(self) -> int:
        return int(self.H.shape[1])


def make_tree(n_cols: int, n_leaves: int, seed: int, cols: Optional[Sequence[int]] = None,
              sigma: float = 0.7) -> TreeModel:
    """Random binary tree with ``n_leaves`` leaves over the columns ``cols`` (default: all
    ``n_cols`` columns of the joined table).  Internal nodes are numbered in creation order
    (root = 0), leaves left to right with the False side on the left."""
    if n_leaves < 2:
        raise ValueError("a tree needs at least two leaves")
    rng = np.random.default_rng(seed)
    cols = list(range(n_cols)) if cols is None else list(cols)
    # grow: every leaf is a slot (parent, side); splitting a slot creates a node with two slots
    true_child, false_child = [], []
    slots = [None]                      # root slot
    while len(slots) + len(true_child) < 2 * n_leaves - 1 or len(slots) < n_leaves:
        if len(slots) >= n_leaves:
            break
        s = slots.pop(int(rng.integers(0, len(slots))))
        q = len(true_child)
        true_child.append(None)
        false_child.append(None)
        if s is not None:
            parent, side = s
            (true_child if side else false_child)[parent] = q
        slots.append((q, 0))
        slots.append((q, 1))
    p = len(true_child)
    # number the leaves left to right (False side first) by a walk from the root
    leaf_of_slot = {}
    order = []

    def walk(q):
        for side, arr in ((0, false_child), (1, true_child)):
            if arr[q] is None:
                leaf_of_slot[(q, side)] = len(order)
                order.append((q, side))
            else:
                walk(arr[q])
    walk(0)
    for (q, side), leaf in leaf_of_slot.items():
        (true_child if side else false_child)[q] = -(leaf + 1)
    l = len(order)
    H = np.zeros((p, l), dtype=np.int8)

    def mark(q, path):
        for side, arr in ((0, false_child), (1, true_child)):
            step = path + [(q, 1 if side else -1)]
            if arr[q] < 0:
                for node, sign in step:
                    H[node, -arr[q] - 1] = sign
            else:
                mark(arr[q], step)
    mark(0, [])
    feature = rng.choice(np.asarray(cols), size=p).astype(np.int32)
    threshold = (rng.standard_normal(p) * sigma).astype(np.float32)
    return TreeModel(torch.from_numpy(feature), torch.from_numpy(threshold), torch.from_numpy(H),
                     [int(x) for x in true_child], [int(x) for x in false_child])
