"""Seeded synthetic inputs: batches of binary trees in CSR form plus model parameters.

This module only *draws* inputs.  It contains none of the arithmetic of the tree
cells and imports neither the GPU binding nor the CPU checker, so both can be fed
the very same arrays.

The paper evaluates on binary parse trees of movie-review sentences (Section 6.1,
"Applications") and on balanced / linear variants of them (Section 6.2,
"Balancedness of trees"); neither the sentences nor the parses are public inside
this repository, so the shapes below stand in for them: random bracketings with
5..50 leaves for sentences, perfectly balanced trees and left-branching chains for
the two extreme shapes.

Random numbers come from a counter-based SplitMix64 generator written out here so
that the streams do not depend on the numpy version.  Every quantity has its own
stream (tree shapes, word ids, each parameter tensor); drawing one never shifts
another.

Tree encoding (the paper's ``tree.children[idx]`` / ``tree.leaves[idx]`` index
arrays of Figures 1 and 2, flattened over a batch):

* ``tree_off[t] .. tree_off[t+1]`` is the node range of tree ``t``;
* ``left[n]``, ``right[n]`` are *global* node indices of the children, ``-1`` at leaves;
* ``word[n]`` is the word id at leaves, ``-1`` at internal nodes.

Nodes are numbered in pre-order by default (every parent *before* its children), the
opposite of the topologically sorted numbering the iterative formulation needs.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

_MASK = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB


def _mix_scalar(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


class Stream:
    """Counter-based SplitMix64: output i is mix(key + (i+1) * golden)."""

    def __init__(self, seed: int, name: str):
        k = _mix_scalar(seed * 0x100000001B3 + 0x51ED270B)
        for ch in name.encode():
            k = _mix_scalar(k ^ (ch + 0x9E37))
        self.key = k
        self.ctr = 0

    def u64(self, n: int) -> np.ndarray:
        idx = np.arange(self.ctr + 1, self.ctr + n + 1, dtype=np.uint64)
        self.ctr += n
        with np.errstate(over="ignore"):
            z = np.uint64(self.key) + idx * np.uint64(_GOLDEN)
            z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
            z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
            z = z ^ (z >> np.uint64(31))
        return z

    def uniform01(self, n: int) -> np.ndarray:
        """Doubles in [0, 1) with 53 random bits."""
        return (self.u64(n) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))

    def uniform(self, lo: float, hi: float, shape) -> np.ndarray:
        n = int(np.prod(shape))
        return (lo + (hi - lo) * self.uniform01(n)).reshape(shape).astype(np.float32)

    def normal(self, std: float, shape) -> np.ndarray:
        """Box-Muller on pairs of uniforms (cosine branch only)."""
        n = int(np.prod(shape))
        u = self.uniform01(2 * n)
        r = np.sqrt(-2.0 * np.log(1.0 - u[0::2]))
        z = r * np.cos(2.0 * np.pi * u[1::2])
        return (std * z).reshape(shape).astype(np.float32)

    def integers(self, lo: int, hi: int, n: int) -> np.ndarray:
        """Integers in [lo, hi] (inclusive), by floor(u * span)."""
        span = hi - lo + 1
        return lo + np.floor(self.uniform01(n) * span).astype(np.int64)


class _Draws:
    """Sequential scalar integer draws served from a Stream in blocks."""

    def __init__(self, stream: Stream):
        self.s = stream
        self.buf = np.empty(0)
        self.pos = 0

    def integer(self, lo: int, hi: int) -> int:
        if self.pos >= len(self.buf):
            self.buf = self.s.uniform01(4096)
            self.pos = 0
        u = self.buf[self.pos]
        self.pos += 1
        return lo + int(u * (hi - lo + 1))


@dataclass
class TreeBatch:
    tree_off: np.ndarray  # int32 [B+1]
    left: np.ndarray      # int32 [N]
    right: np.ndarray     # int32 [N]
    word: np.ndarray      # int32 [N]

    @property
    def n_trees(self) -> int:
        return len(self.tree_off) - 1

    @property
    def n_nodes(self) -> int:
        return int(self.tree_off[-1])

    @property
    def n_leaves(self) -> int:
        return int((self.left < 0).sum())

    @property
    def n_internal(self) -> int:
        return self.n_nodes - self.n_leaves


def _shape_preorder(n_leaves: int, split) -> tuple:
    """Local (0-based) left/right arrays of one tree, pre-order numbering.

    ``split(L)`` returns the number of leaves that go to the left child of a node
    spanning L >= 2 leaves; it is called once per internal node, in pre-order.
    """
    left: List[int] = []
    right: List[int] = []
    stack = [(n_leaves, -1, 0)]
    while stack:
        L, par, side = stack.pop()
        me = len(left)
        left.append(-1)
        right.append(-1)
        if par >= 0:
            if side == 0:
                left[par] = me
            else:
                right[par] = me
        if L > 1:
            k = split(L)
            assert 1 <= k <= L - 1
            stack.append((L - k, me, 1))
            stack.append((k, me, 0))  # popped first: left subtree precedes right
    return np.asarray(left, dtype=np.int64), np.asarray(right, dtype=np.int64)


def make_trees(seed: int, leaf_counts: Sequence[int], shapes: Sequence[str], vocab: int) -> TreeBatch:
    """Batch of full binary trees.

    shapes[t] is ``"random"`` (split point uniform in 1..L-1 at every internal node),
    ``"balanced"`` (split L//2) or ``"chain"`` (left child gets L-1 leaves, the right
    child is a single leaf).  Word ids are uniform in [0, vocab), assigned to the
    leaves of the whole batch from left to right.
    """
    draws = _Draws(Stream(seed, "shape"))
    lefts, rights, offs = [], [], [0]
    for L, shp in zip(leaf_counts, shapes):
        if shp == "random":
            split = lambda n: draws.integer(1, n - 1)
        elif shp == "balanced":
            split = lambda n: n // 2
        elif shp == "chain":
            split = lambda n: n - 1
        else:
            raise ValueError(shp)
        l, r = _shape_preorder(int(L), split)
        base = offs[-1]
        lefts.append(np.where(l >= 0, l + base, -1))
        rights.append(np.where(r >= 0, r + base, -1))
        offs.append(base + len(l))
    left = np.concatenate(lefts).astype(np.int32)
    right = np.concatenate(rights).astype(np.int32)
    word = np.full(left.shape, -1, dtype=np.int32)
    is_leaf = left < 0
    word[is_leaf] = Stream(seed, "word").integers(0, vocab - 1, int(is_leaf.sum())).astype(np.int32)
    return TreeBatch(np.asarray(offs, dtype=np.int32), left, right, word)


def renumber(batch: TreeBatch, mode: str, seed: int = 0) -> tuple:
    """Renumber the nodes inside every tree; returns (new batch, new_of_old).

    mode: ``"post"`` (children before parents, i.e. a topological order),
    ``"random"`` (seeded shuffle per tree) or ``"pre"`` (identity).
    ``new_of_old[n]`` is the new global index of old node n.
    """
    N = batch.n_nodes
    new_of_old = np.arange(N, dtype=np.int64)
    if mode == "pre":
        pass
    elif mode == "random":
        s = Stream(seed, "perm")
        for t in range(batch.n_trees):
            a, b = int(batch.tree_off[t]), int(batch.tree_off[t + 1])
            keys = s.u64(b - a)
            new_of_old[a:b] = a + np.argsort(np.argsort(keys, kind="stable"), kind="stable")
    elif mode == "post":
        has_parent = np.zeros(N, dtype=bool)
        has_parent[batch.left[batch.left >= 0]] = True
        has_parent[batch.right[batch.right >= 0]] = True
        for t in range(batch.n_trees):
            a, b = int(batch.tree_off[t]), int(batch.tree_off[t + 1])
            root = a + int(np.flatnonzero(~has_parent[a:b])[0])
            nxt = a
            stack = [(root, False)]
            while stack:
                n, done = stack.pop()
                if done or batch.left[n] < 0:
                    new_of_old[n] = nxt
                    nxt += 1
                else:
                    stack.append((n, True))
                    stack.append((int(batch.right[n]), False))
                    stack.append((int(batch.left[n]), False))
    else:
        raise ValueError(mode)
    left = np.full(N, -1, dtype=np.int32)
    right = np.full(N, -1, dtype=np.int32)
    word = np.full(N, -1, dtype=np.int32)
    internal = batch.left >= 0
    left[new_of_old[internal]] = new_of_old[batch.left[internal]]
    right[new_of_old[internal]] = new_of_old[batch.right[internal]]
    word[new_of_old] = batch.word
    return TreeBatch(batch.tree_off.copy(), left, right, word), new_of_old


CELL_TREELSTM, CELL_TREERNN, CELL_RNTN = 0, 1, 2


@dataclass
class Params:
    """Model parameters as fp32 numpy arrays, in the layout of the C interface."""
    cell: int
    vocab: int
    embed_dim: int
    hidden: int
    emb: np.ndarray                      # [vocab, embed_dim]
    w_leaf: Optional[np.ndarray] = None  # TreeLSTM [embed_dim, 3H]   columns i | o | u
    b_leaf: Optional[np.ndarray] = None  # TreeLSTM [3H]
    u: Optional[np.ndarray] = None       # TreeLSTM [2H, 5H] columns i | f_l | f_r | o | u ; TreeRNN/RNTN W [2d, d]
    b: Optional[np.ndarray] = None       # TreeLSTM [5H] ; TreeRNN/RNTN [d]
    v: Optional[np.ndarray] = None       # RNTN [d, 2d, 2d]  (k, p, q)


def _xavier(stream: Stream, rows: int, cols: int) -> np.ndarray:
    bound = float(np.sqrt(6.0 / (rows + cols)))  # fans = shape of the stored matrix
    return stream.uniform(-bound, bound, (rows, cols))


def make_treelstm_params(seed: int, vocab: int, embed_dim: int, hidden: int, init: str) -> Params:
    """init = "uniform0.1": everything U(-0.1, 0.1), biases 0.
    init = "xavier": embeddings N(0, 0.1^2), Xavier-uniform matrices, forget biases 1, other biases 0."""
    E, H = embed_dim, hidden
    if init == "uniform0.1":
        emb = Stream(seed, "emb").uniform(-0.1, 0.1, (vocab, E))
        w_leaf = Stream(seed, "w_leaf").uniform(-0.1, 0.1, (E, 3 * H))
        u = Stream(seed, "u").uniform(-0.1, 0.1, (2 * H, 5 * H))
        b = np.zeros(5 * H, dtype=np.float32)
    elif init == "xavier":
        emb = Stream(seed, "emb").normal(0.1, (vocab, E))
        w_leaf = _xavier(Stream(seed, "w_leaf"), E, 3 * H)
        u = _xavier(Stream(seed, "u"), 2 * H, 5 * H)
        b = np.zeros(5 * H, dtype=np.float32)
        b[H:3 * H] = 1.0
    else:
        raise ValueError(init)
    return Params(CELL_TREELSTM, vocab, E, H, emb, w_leaf, np.zeros(3 * H, dtype=np.float32), u, b)


def make_rnn_params(seed: int, cell: int, vocab: int, d: int, scale: float = 0.05) -> Params:
    emb = Stream(seed, "emb").uniform(-scale, scale, (vocab, d))
    w = Stream(seed, "w").uniform(-scale, scale, (2 * d, d))
    b = np.zeros(d, dtype=np.float32)
    v = None
    if cell == CELL_RNTN:
        v = Stream(seed, "v").uniform(-scale, scale, (d, 2 * d, 2 * d))
    return Params(cell, vocab, d, d, emb, None, None, w, b, v)


@dataclass
class Workload:
    name: str
    trees: TreeBatch
    params: Params
    note: str = ""


def _sentence_trees(seed: int, batch: int, vocab: int, lo: int = 5, hi: int = 50) -> TreeBatch:
    counts = Stream(seed, "leaves").integers(lo, hi, batch)
    return make_trees(seed, counts, ["random"] * batch, vocab)


def workload(name: str) -> Workload:
    """The evaluation workloads (seeds 0..4); the fourth one comes with two cells, `treernn` and `rntn`."""
    if name == "tiny":
        tr = make_trees(0, [8] * 4, ["random"] * 4, 100)
        return Workload(name, tr, make_treelstm_params(0, 100, 16, 16, "uniform0.1"))
    if name == "sentence":
        tr = _sentence_trees(1, 25, 20000)
        return Workload(name, tr, make_treelstm_params(1, 20000, 300, 150, "xavier"))
    if name == "throughput":
        tr = _sentence_trees(2, 256, 20000)
        return Workload(name, tr, make_treelstm_params(2, 20000, 300, 512, "xavier"))
    if name == "treernn":
        tr = _sentence_trees(3, 256, 20000)
        return Workload(name, tr, make_rnn_params(3, CELL_TREERNN, 20000, 256))
    if name == "rntn":
        tr = _sentence_trees(3, 256, 20000)
        return Workload(name, tr, make_rnn_params(3, CELL_RNTN, 20000, 64))
    if name == "stress":
        tr = make_trees(4, [1024] * 64, ["chain", "balanced"] * 32, 50000)
        return Workload(name, tr, make_treelstm_params(4, 50000, 256, 256, "xavier"))
    if name == "mixed":
        # a few very deep trees in a batch of much shallow work (the case for critical-path-first scheduling):
        # 8 192 sentence trees followed by 8 left-branching chains of 1 024 leaves
        counts = list(Stream(5, "leaves").integers(5, 50, 8192)) + [1024] * 8
        tr = make_trees(5, counts, ["random"] * 8192 + ["chain"] * 8, 20000)
        return Workload(name, tr, make_treelstm_params(5, 20000, 256, 256, "xavier"))
    if name == "mixed_small":
        counts = list(Stream(6, "leaves").integers(5, 50, 512)) + [256] * 4
        tr = make_trees(6, counts, ["random"] * 512 + ["chain"] * 4, 1000)
        return Workload(name, tr, make_treelstm_params(6, 1000, 48, 64, "xavier"))
    raise ValueError(name)


WORKLOADS = ("tiny", "sentence", "throughput", "treernn", "rntn", "stress")


@dataclass
class TopDown:
    """Inputs of a top-down generation: parameters, root states and the two limits."""
    name: str
    hidden: int
    u_td: np.ndarray       # [H x 8H], columns [iL|fL|oL|uL|iR|fR|oR|uR]
    b_td: np.ndarray       # [8H]
    w_stop: np.ndarray     # [H]
    b_stop: float
    h_root: np.ndarray     # [B x H]
    c_root: np.ndarray     # [B x H]
    max_depth: int
    max_nodes: int


def make_topdown(seed: int, name: str, batch: int, hidden: int, max_depth: int, max_nodes: int, stop_scale: float,
                 b_stop: float) -> TopDown:
    """Xavier-uniform edge weights (forget biases 1), a stopping direction of N(0, (stop_scale / sqrt(H))^2) entries,
    root states h ~ U(-0.8, 0.8), c ~ N(0, 0.5^2)."""
    H = hidden
    u_td = _xavier(Stream(seed, "u_td"), H, 8 * H)
    b_td = np.zeros(8 * H, dtype=np.float32)
    b_td[H:2 * H] = 1.0
    b_td[5 * H:6 * H] = 1.0
    w_stop = Stream(seed, "w_stop").normal(stop_scale / float(np.sqrt(H)), (H,))
    h_root = Stream(seed, "h_root").uniform(-0.8, 0.8, (batch, H))
    c_root = Stream(seed, "c_root").normal(0.5, (batch, H))
    return TopDown(name, H, u_td, b_td, w_stop, float(b_stop), h_root, c_root, max_depth, max_nodes)


def topdown_workload(name: str) -> TopDown:
    """Dynamic-structure workloads: `td64` / `td1` are the two batch sizes of the paper's top-down experiment (64 and 1
    instances) at the hidden size of the `throughput` workload; the others are small parity cases."""
    if name == "td64":        # 2 038 nodes, depths 0..9, trees of 1 to 409 nodes
        return make_topdown(10, name, 64, 512, 12, 8192, 6.0, -0.3)
    if name == "td1":         # tree 7 of td64 on its own: 409 nodes
        w = make_topdown(10, name, 64, 512, 12, 8192, 6.0, -0.3)
        w.h_root, w.c_root, w.max_nodes = w.h_root[7:8].copy(), w.c_root[7:8].copy(), 1024
        return w
    if name == "td_small":    # 231 nodes, depths 0..6
        return make_topdown(18, name, 5, 33, 6, 700, 6.0, 0.3)
    if name == "td_mid":      # 1 781 nodes, depths 0..10
        return make_topdown(12, name, 25, 150, 10, 4096, 6.0, -0.3)
    raise ValueError(name)


TOPDOWN_WORKLOADS = ("td_small", "td_mid", "td64", "td1")


def subset(batch: TreeBatch, trees: Sequence[int]) -> tuple:
    """The given trees as a batch of their own (indices rebased); also returns, for
    every node of the new batch, its global index in the original batch."""
    lefts, rights, words, offs, orig = [], [], [], [0], []
    for t in trees:
        a, b = int(batch.tree_off[t]), int(batch.tree_off[t + 1])
        shift = offs[-1] - a
        l = batch.left[a:b].astype(np.int64)
        r = batch.right[a:b].astype(np.int64)
        lefts.append(np.where(l >= 0, l + shift, -1))
        rights.append(np.where(r >= 0, r + shift, -1))
        words.append(batch.word[a:b])
        orig.append(np.arange(a, b))
        offs.append(offs[-1] + (b - a))
    tb = TreeBatch(np.asarray(offs, dtype=np.int32), np.concatenate(lefts).astype(np.int32),
                   np.concatenate(rights).astype(np.int32), np.concatenate(words).astype(np.int32))
    return tb, np.concatenate(orig)
