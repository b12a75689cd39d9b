"""CPU checker for the tree-network forward pass: ctypes front end of tree_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library and its Python binding never import
this package, and this package never imports them.  See the header of
tree_oracle.c for what is computed and how it is pinned (and what is not).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from .build import LIB, build

_lib = None
_F = ctypes.POINTER(ctypes.c_float)
_I = ctypes.POINTER(ctypes.c_int32)


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(LIB)
        lib.oracle_structure.restype = ctypes.c_int
        lib.oracle_structure.argtypes = [ctypes.c_int, ctypes.c_int, _I, _I, _I, _I, _I, _I]
        lib.oracle_backward.restype = ctypes.c_int
        lib.oracle_backward.argtypes = ([ctypes.c_int] * 3 + [_F] * 5 + [ctypes.c_int, ctypes.c_int] + [_I] * 4 + [_F] * 3
                                        + [_F] * 5)
        lib.oracle_backward_rntn.restype = ctypes.c_int
        lib.oracle_backward_rntn.argtypes = [ctypes.c_int, _F, _F, ctypes.c_int, ctypes.c_int] + [_I] * 3 + [_F] * 6
        lib.oracle_backward_rnn.restype = ctypes.c_int
        lib.oracle_backward_rnn.argtypes = [ctypes.c_int, _F, ctypes.c_int, ctypes.c_int] + [_I] * 3 + [_F] * 5
        lib.oracle_classify_backward.restype = ctypes.c_int
        lib.oracle_classify_backward.argtypes = ([ctypes.c_int] * 3 + [_F] * 3 + [_I] + [_F] * 3 + [ctypes.POINTER(ctypes.c_double)])
        lib.oracle_td_step.restype = None
        lib.oracle_td_step.argtypes = [ctypes.c_int] + [_F] * 3 + [ctypes.c_float] + [_F] * 5
        lib.oracle_td_generate.restype = ctypes.c_int
        lib.oracle_td_generate.argtypes = ([ctypes.c_int] + [_F] * 3 + [ctypes.c_float, ctypes.c_int] + [_F] * 2
                                           + [ctypes.c_int, ctypes.c_int] + [_I] * 4 + [_F] * 3 + [_I])
        lib.oracle_classify.restype = ctypes.c_int
        lib.oracle_classify.argtypes = [ctypes.c_int] * 3 + [_F] * 4
        lib.oracle_forward.restype = ctypes.c_int
        lib.oracle_forward.argtypes = ([ctypes.c_int] * 5 + [_F] * 6 + [ctypes.c_int, ctypes.c_int] + [_I] * 4
                                       + [ctypes.c_int, ctypes.c_int] + [_F] * 4)
        _lib = lib
    return _lib


def _f(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(_F)


def _i(a: np.ndarray):
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return a.ctypes.data_as(_I)


def to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bfloat16 (ties to even), kept in an fp32 array."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape)


def structure(tree_off, left, right):
    """(parent, root, height) by plain traversal; raises ValueError on a malformed batch."""
    lib = _load()
    n_trees, n_nodes = len(tree_off) - 1, len(left)
    parent = np.empty(max(n_nodes, 1), dtype=np.int32)
    height = np.zeros(max(n_nodes, 1), dtype=np.int32)
    root = np.empty(max(n_trees, 1), dtype=np.int32)
    rc = lib.oracle_structure(n_trees, n_nodes, _i(tree_off), _i(left), _i(right), _i(parent), _i(root), _i(height))
    if rc != 0:
        raise ValueError("malformed tree batch")
    return parent[:n_nodes], root[:n_trees], height[:n_nodes]


def forward(cell, vocab, embed_dim, hidden, emb, w_leaf, b_leaf, u, b, v,
            tree_off, left, right, word, order="recursive", n_threads=1, round_bf16=False):
    """Evaluate every node.  Returns dict(h, c, h_root, c_root) of fp32 arrays (c* None unless TreeLSTM)."""
    lib = _load()
    n_trees, n_nodes = len(tree_off) - 1, len(left)
    H = hidden
    h = np.zeros((n_nodes, H), dtype=np.float32)
    h_root = np.zeros((n_trees, H), dtype=np.float32)
    c = c_root = None
    if cell == 0:
        c = np.zeros((n_nodes, H), dtype=np.float32)
        c_root = np.zeros((n_trees, H), dtype=np.float32)
    rc = lib.oracle_forward(cell, vocab, embed_dim, H, int(bool(round_bf16)),
                            _f(emb), _f(w_leaf), _f(b_leaf), _f(u), _f(b), _f(v),
                            n_trees, n_nodes, _i(tree_off), _i(left), _i(right), _i(word),
                            {"recursive": 0, "topological": 1}[order], int(n_threads),
                            _f(h), _f(c), _f(h_root), _f(c_root))
    if rc != 0:
        raise ValueError("malformed tree batch")
    return {"h": h, "c": c, "h_root": h_root, "c_root": c_root}


def backward(params, trees, h, c, g_h):
    """Gradients of a loss with dL/dh[n] = g_h[n].  TreeLSTM: dict(d_u, d_b, d_w_leaf, d_b_leaf, d_x [N x E]);
    TreeRNN (c is ignored): dict(d_u [2H x H], d_b [H], d_x [N x H]); RNTN: the same plus d_v [H x 2H x 2H]."""
    lib = _load()
    if params.cell == 1:
        H = params.hidden
        n_trees, n_nodes = len(trees.tree_off) - 1, len(trees.left)
        out = {"d_u": np.zeros((2 * H, H), np.float32), "d_b": np.zeros(H, np.float32), "d_x": np.zeros((n_nodes, H), np.float32)}
        f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
        rc = lib.oracle_backward_rnn(H, _f(params.u), n_trees, n_nodes, _i(trees.tree_off), _i(trees.left), _i(trees.right),
                                     _f(f32(h)), _f(f32(g_h)), _f(out["d_u"]), _f(out["d_b"]), _f(out["d_x"]))
        if rc != 0:
            raise ValueError("malformed tree batch")
        return out
    if params.cell == 2:
        H = params.hidden
        n_trees, n_nodes = len(trees.tree_off) - 1, len(trees.left)
        out = {"d_u": np.zeros((2 * H, H), np.float32), "d_b": np.zeros(H, np.float32),
               "d_v": np.zeros((H, 2 * H, 2 * H), np.float32), "d_x": np.zeros((n_nodes, H), np.float32)}
        f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
        rc = lib.oracle_backward_rntn(H, _f(params.u), _f(params.v), n_trees, n_nodes, _i(trees.tree_off), _i(trees.left),
                                      _i(trees.right), _f(f32(h)), _f(f32(g_h)), _f(out["d_u"]), _f(out["d_b"]), _f(out["d_v"]),
                                      _f(out["d_x"]))
        if rc != 0:
            raise ValueError("malformed tree batch")
        return out
    assert params.cell == 0
    H, E = params.hidden, params.embed_dim
    n_trees, n_nodes = len(trees.tree_off) - 1, len(trees.left)
    out = {"d_u": np.zeros((2 * H, 5 * H), np.float32), "d_b": np.zeros(5 * H, np.float32),
           "d_w_leaf": np.zeros((E, 3 * H), np.float32), "d_b_leaf": np.zeros(3 * H, np.float32),
           "d_x": np.zeros((n_nodes, E), np.float32)}
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    rc = lib.oracle_backward(params.vocab, E, H, _f(params.emb), _f(params.w_leaf), _f(params.b_leaf), _f(params.u),
                             _f(params.b), n_trees, n_nodes, _i(trees.tree_off), _i(trees.left), _i(trees.right),
                             _i(trees.word), _f(f32(h)), _f(f32(c)), _f(f32(g_h)),
                             _f(out["d_u"]), _f(out["d_b"]), _f(out["d_w_leaf"]), _f(out["d_b_leaf"]), _f(out["d_x"]))
    if rc != 0:
        raise ValueError("malformed tree batch")
    return out


def classify(h, w_s, b_s):
    """Per-node class probabilities softmax(h W_s + b_s): h [N x H], w_s [H x C], b_s [C] -> [N x C] fp32."""
    lib = _load()
    h = np.ascontiguousarray(h, dtype=np.float32)
    w_s = np.ascontiguousarray(w_s, dtype=np.float32)
    b_s = np.ascontiguousarray(b_s, dtype=np.float32)
    n, H = h.shape
    C = w_s.shape[1]
    assert w_s.shape[0] == H and b_s.shape == (C,)
    probs = np.zeros((n, C), dtype=np.float32)
    if lib.oracle_classify(n, H, C, _f(h), _f(w_s), _f(b_s), _f(probs)) != 0:
        raise ValueError("bad classifier dimensions")
    return probs


def classify_backward(h, w_s, b_s, label):
    """Cross-entropy (summed over nodes with label >= 0) on top of classify(): dict(loss, g_h, d_w_s, d_b_s)."""
    lib = _load()
    h = np.ascontiguousarray(h, dtype=np.float32)
    w_s = np.ascontiguousarray(w_s, dtype=np.float32)
    b_s = np.ascontiguousarray(b_s, dtype=np.float32)
    label = np.ascontiguousarray(label, dtype=np.int32)
    n, H = h.shape
    C = w_s.shape[1]
    out = {"g_h": np.zeros((n, H), np.float32), "d_w_s": np.zeros((H, C), np.float32), "d_b_s": np.zeros(C, np.float32)}
    loss = ctypes.c_double(0.0)
    if lib.oracle_classify_backward(n, H, C, _f(h), _f(w_s), _f(b_s), _i(label), _f(out["g_h"]), _f(out["d_w_s"]),
                                    _f(out["d_b_s"]), ctypes.byref(loss)) != 0:
        raise ValueError("bad classifier dimensions or labels")
    out["loss"] = loss.value
    return out


def td_step(u_td, b_td, w_stop, b_stop, h, c):
    """One node of the top-down generator: (child_h [2 x H], child_c [2 x H], score) from the node's stored state."""
    lib = _load()
    h = np.ascontiguousarray(h, dtype=np.float32)
    c = np.ascontiguousarray(c, dtype=np.float32)
    H = h.shape[0]
    kh, kc = np.zeros((2, H), np.float32), np.zeros((2, H), np.float32)
    score = np.zeros(1, np.float32)
    lib.oracle_td_step(H, _f(u_td), _f(b_td), _f(w_stop), float(b_stop), _f(h), _f(c), _f(kh), _f(kc), _f(score))
    return kh, kc, float(score[0])


def td_generate(u_td, b_td, w_stop, b_stop, h_root, c_root, max_depth, max_nodes):
    """Top-down generation from the root states; dict(n_nodes, truncated, parent, left, right, depth, score, h, c),
    arrays cut to n_nodes rows, nodes in breadth-first order."""
    lib = _load()
    h_root = np.ascontiguousarray(h_root, dtype=np.float32)
    c_root = np.ascontiguousarray(c_root, dtype=np.float32)
    B, H = h_root.shape
    ints = [np.full(max_nodes, -1, np.int32) for _ in range(4)]
    score = np.zeros(max_nodes, np.float32)
    h, c = np.zeros((max_nodes, H), np.float32), np.zeros((max_nodes, H), np.float32)
    trunc = np.zeros(1, np.int32)
    n = lib.oracle_td_generate(H, _f(u_td), _f(b_td), _f(w_stop), float(b_stop), B, _f(h_root), _f(c_root), int(max_depth),
                               int(max_nodes), *[_i(a) for a in ints], _f(score), _f(h), _f(c), _i(trunc))
    if n < 0:
        raise ValueError("bad arguments")
    return {"n_nodes": n, "truncated": int(trunc[0]), "parent": ints[0][:n], "left": ints[1][:n], "right": ints[2][:n],
            "depth": ints[3][:n], "score": score[:n], "h": h[:n], "c": c[:n]}


def forward_params(params, trees, **kw):
    """Convenience: same as forward() for objects carrying the fields by name."""
    return forward(params.cell, params.vocab, params.embed_dim, params.hidden, params.emb, params.w_leaf,
                   params.b_leaf, params.u, params.b, params.v,
                   trees.tree_off, trees.left, trees.right, trees.word, **kw)
