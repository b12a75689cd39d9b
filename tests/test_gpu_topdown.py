"""GPU parity of the top-down generator (tl_td_generate) against the CPU checker, through the C ABI.

Row numbers of the generated nodes depend on timing, so nodes are compared by their path from the root (tree
number, then L / R per edge).  A decision `score > 0` whose score lies within MARGIN of zero may legitimately fall
either way (the GPU sums in fp32, the checker in fp64): trees that contain such a node are checked for validity node
by node (every child is the checker's step of its parent's stored state), the others must match the checker's trees
exactly, with states within |g - o| <= 1e-4 + 1e-3 |o| (errors of up to 12 chained fp32 cells).
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1809_00832_amd import binding, synth

pytestmark = pytest.mark.gpu
MARGIN = 1e-4
HERE = os.path.dirname(os.path.abspath(__file__))


def generate(w, **chg):
    a = dict(w_stop=w.w_stop, b_stop=w.b_stop, max_depth=w.max_depth, max_nodes=w.max_nodes)
    a.update(chg)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    ctx = binding.tl_td_create(w.hidden, dev(w.u_td), dev(w.b_td), dev(a["w_stop"]), a["b_stop"], a.get("spin_limit", 0))
    try:
        out = binding.tl_td_generate(ctx, dev(w.h_root), dev(w.c_root), a["max_nodes"], a["max_depth"])
        code = binding.tl_td_status(ctx)
        assert code == binding.TL_OK, binding.tl_strerror(code)
        counts = out["counts"].cpu().numpy()
        n = int(counts[0])
        res = {k: out[k][:n].cpu().numpy() for k in ("h", "c", "parent", "left", "right", "depth", "score")}
        res.update(n_nodes=n, truncated=int(counts[1]), frontiers=int(counts[2]))
        return res
    finally:
        binding.tl_td_destroy(ctx)


def paths(r, B):
    """Path key of every node; also checks that the links form B proper trees over rows 0 .. n-1."""
    n = r["n_nodes"]
    assert B <= n
    key = [None] * n
    for t in range(B):
        assert r["parent"][t] == -1 and r["depth"][t] == 0
        key[t] = (t, "")
    seen = np.zeros(n, bool)
    seen[:B] = True
    for v in range(n):
        l, rr = int(r["left"][v]), int(r["right"][v])
        assert (l < 0) == (rr < 0)
        if l < 0:
            continue
        assert rr == l + 1 and v < l and rr < n
        assert r["parent"][l] == v and r["parent"][rr] == v
        assert r["depth"][l] == r["depth"][v] + 1 and r["depth"][rr] == r["depth"][v] + 1
        assert not seen[l] and not seen[rr]
        seen[l] = seen[rr] = True
    assert seen.all()
    for v in range(B, n):                       # a child's row is always above its parent's
        p = int(r["parent"][v])
        key[v] = (key[p][0], key[p][1] + ("L" if int(r["left"][p]) == v else "R"))
    return key


def close(g, o, atol=1e-4, rtol=1e-3):
    return bool((np.abs(g.astype(np.float64) - o) <= atol + rtol * np.abs(o)).all())


def check_steps(w, r, nodes, w_stop=None, b_stop=None, max_depth=None):
    """Every listed node against the checker's single step from the node's stored state."""
    w_stop = w.w_stop if w_stop is None else w_stop
    b_stop = w.b_stop if b_stop is None else b_stop
    max_depth = w.max_depth if max_depth is None else max_depth
    undecided = 0
    for v in nodes:
        kh, kc, score = oracle.td_step(w.u_td, w.b_td, w_stop, b_stop, r["h"][v], r["c"][v])
        assert abs(float(r["score"][v]) - score) <= 1e-5 + 1e-4 * abs(score), (v, r["score"][v], score)
        expanded = r["left"][v] >= 0
        if abs(score) > MARGIN and r["truncated"] == 0:
            assert expanded == (score > 0 and r["depth"][v] < max_depth), (v, score)
        else:
            undecided += 1
        if expanded:
            for side, kid in enumerate((int(r["left"][v]), int(r["right"][v]))):
                assert close(r["h"][kid], kh[side]) and close(r["c"][kid], kc[side]), (v, side)
    return undecided


@pytest.mark.parametrize("name", ["td_small", "td_mid"])
def test_generated_trees_match_the_checker(name):
    print("case topdown", name, flush=True)
    w = synth.topdown_workload(name)
    B = w.h_root.shape[0]
    ref = oracle.td_generate(w.u_td, w.b_td, w.w_stop, w.b_stop, w.h_root, w.c_root, w.max_depth, w.max_nodes)
    got = generate(w)
    gk, rk = paths(got, B), paths(ref, B)
    assert np.array_equal(got["h"][:B], w.h_root) and np.array_equal(got["c"][:B], w.c_root)
    shaky = {rk[v][0] for v in range(ref["n_nodes"]) if abs(float(ref["score"][v])) <= MARGIN}
    gmap = {k: v for v, k in enumerate(gk)}
    rmap = {k: v for v, k in enumerate(rk)}
    firm = [t for t in range(B) if t not in shaky]
    assert len(firm) >= B - 3, "too many trees with a decision near zero: %s" % sorted(shaky)
    for t in firm:
        assert {k for k in gmap if k[0] == t} == {k for k in rmap if k[0] == t}, "tree %d has another shape" % t
    for k, v in rmap.items():
        if k[0] in shaky:
            continue
        g = gmap[k]
        assert close(got["h"][g], ref["h"][v]) and close(got["c"][g], ref["c"][v]), k
        assert got["depth"][g] == ref["depth"][v] and (got["left"][g] >= 0) == (ref["left"][v] >= 0)
    if not shaky:
        assert got["n_nodes"] == ref["n_nodes"] and got["frontiers"] == int(ref["depth"].max()) + 1
    undecided = check_steps(w, got, range(got["n_nodes"]))
    print("    nodes %d (checker %d), trees compared %d of %d, decisions within the margin %d" % (
        got["n_nodes"], ref["n_nodes"], len(firm), B, undecided), flush=True)


def test_full_size_batch_of_64():
    """H = 512, 64 roots (the batch size of the paper's top-down experiment): per-tree sizes against the stored
    result of the checker (tests/golden/topdown_td64.json, written by make_topdown_golden.py), every node
    against the checker's step, and identical trees bit for bit from run to run."""
    print("case topdown td64", flush=True)
    w = synth.topdown_workload("td64")
    B = w.h_root.shape[0]
    with open(os.path.join(HERE, "golden", "topdown_td64.json")) as fh:
        gold = json.load(fh)
    got = generate(w)
    gk = paths(got, B)
    sizes = np.bincount([k[0] for k in gk], minlength=B)
    depth = np.zeros(B, int)
    for v, k in enumerate(gk):
        depth[k[0]] = max(depth[k[0]], len(k[1]))
    compared = 0
    for t, tr in enumerate(gold["trees"]):
        if tr["min_abs_score"] > MARGIN:
            assert sizes[t] == tr["nodes"] and depth[t] == tr["depth"], (t, sizes[t], tr)
            compared += 1
    assert compared >= B - 4 and got["truncated"] == 0
    undecided = check_steps(w, got, range(got["n_nodes"]))        # every node against the checker's step
    again = generate(w)
    ak = paths(again, B)
    assert again["n_nodes"] == got["n_nodes"]
    amap = {k: v for v, k in enumerate(ak)}
    order = np.array([amap[k] for k in gk])
    assert np.array_equal(again["h"][order], got["h"]) and np.array_equal(again["c"][order], got["c"])
    assert np.array_equal(again["score"][order], got["score"])
    print("    nodes %d (checker %d), trees compared %d, decisions within the margin %d" % (
        got["n_nodes"], gold["n_nodes"], compared, undecided), flush=True)


@pytest.mark.parametrize("B", [1, 7, 32])
def test_small_batches_take_the_data_flow_form(B):
    """Batches of up to 32 roots at H = 512 grow without frontiers (deciders beside expanders, children computed while
    their parent is being scored): the B largest trees of the batch of 64 against the checker's trees (those without
    a decision near zero, at least half of them), node by node by
    path, every node against the checker's step, and the same bits from run to run although rows and tiles differ."""
    print("case topdown data-flow form", B, flush=True)
    w = synth.topdown_workload("td64")
    with open(os.path.join(HERE, "golden", "topdown_td64.json")) as fh:
        gold = json.load(fh)
    pick = sorted(range(64), key=lambda t: -gold["trees"][t]["nodes"])[:B]
    w.h_root, w.c_root = w.h_root[pick].copy(), w.c_root[pick].copy()
    ref = oracle.td_generate(w.u_td, w.b_td, w.w_stop, w.b_stop, w.h_root, w.c_root, w.max_depth, w.max_nodes)
    got = generate(w)
    gk, rk = paths(got, B), paths(ref, B)
    shaky = {rk[v][0] for v in range(ref["n_nodes"]) if abs(float(ref["score"][v])) <= MARGIN}
    gmap = {k: v for v, k in enumerate(gk)}
    rmap = {k: v for v, k in enumerate(rk)}
    assert 2 * len(shaky) <= B
    for t in range(B):
        if t not in shaky:
            assert {k for k in gmap if k[0] == t} == {k for k in rmap if k[0] == t}, "tree %d has another shape" % t
    for k, v in rmap.items():
        if k[0] not in shaky:
            g = gmap[k]
            assert close(got["h"][g], ref["h"][v]) and close(got["c"][g], ref["c"][v]), k
            assert got["depth"][g] == ref["depth"][v] and (got["left"][g] >= 0) == (ref["left"][v] >= 0)
    if not shaky:
        assert got["n_nodes"] == ref["n_nodes"] and got["frontiers"] == int(ref["depth"].max()) + 1
    assert got["truncated"] == 0
    check_steps(w, got, range(0, got["n_nodes"], 1 if B < 32 else 2))
    for _ in range(3):
        again = generate(w)
        amap = {k: v for v, k in enumerate(paths(again, B))}
        assert again["n_nodes"] == got["n_nodes"]
        order = np.array([amap[k] for k in gk])
        assert np.array_equal(again["h"][order], got["h"]) and np.array_equal(again["c"][order], got["c"])
        assert np.array_equal(again["score"][order], got["score"])
    print("    nodes %d (checker %d), trees with a decision within the margin %d" % (got["n_nodes"], ref["n_nodes"], len(shaky)),
          flush=True)


def test_data_flow_form_beyond_the_rows_marked_in_advance():
    """The data-flow form marks 16 MiB of rows as "not written" before it starts and later rows when they are reserved:
    full trees of 2 x 32 767 nodes at H = 64 (32 768 rows are marked in advance), closed forms and sampled steps; then
    the same with room for half of them."""
    print("case topdown rows marked when reserved", flush=True)
    B, H, D = 2, 64, 14
    full_n = B * (2 ** (D + 1) - 1)
    w = synth.make_topdown(77, "case", B, H, D, full_n + 5, 6.0, 0.0)
    zero = np.zeros_like(w.w_stop)
    full = generate(w, w_stop=zero, b_stop=1.0)
    assert full["n_nodes"] == full_n and full["truncated"] == 0 and full["frontiers"] == D + 1
    assert np.array_equal(np.bincount(full["depth"]), B * 2 ** np.arange(D + 1))
    paths(full, B)
    check_steps(w, full, range(0, full_n, 97), w_stop=zero, b_stop=1.0)
    check_steps(w, full, range(full_n - 40, full_n), w_stop=zero, b_stop=1.0)
    half = generate(w, w_stop=zero, b_stop=1.0, max_nodes=full_n // 2)
    assert half["n_nodes"] == B + 2 * ((full_n // 2 - B) // 2) and half["truncated"] >= 1
    paths(half, B)
    check_steps(w, half, range(0, half["n_nodes"], 211), w_stop=zero, b_stop=1.0)


def test_closed_forms_limits_and_ragged_sizes():
    print("case topdown closed forms", flush=True)
    # (H = 64, 100, 320: the expansion step on the weight-stationary cell, the last two with a padded K axis)
    for i, (B, H, D) in enumerate([(5, 33, 4), (1, 6, 5), (3, 150, 3), (70, 64, 2), (9, 100, 4), (4, 320, 3)]):
        w = synth.make_topdown(40 + i, "case", B, H, D, B * (2 ** (D + 1) - 1) + 3, 6.0, 0.0)
        zero = np.zeros_like(w.w_stop)
        full = generate(w, w_stop=zero, b_stop=1.0)
        assert full["n_nodes"] == B * (2 ** (D + 1) - 1) and full["truncated"] == 0 and full["frontiers"] == D + 1
        assert np.array_equal(np.bincount(full["depth"]), B * 2 ** np.arange(D + 1))
        paths(full, B)
        check_steps(w, full, range(0, full["n_nodes"], 5), w_stop=zero, b_stop=1.0)
        none = generate(w, w_stop=zero, b_stop=-1.0)
        assert none["n_nodes"] == B and (none["left"] < 0).all() and none["frontiers"] == 1
        edge = generate(w, w_stop=zero, b_stop=0.0)              # a score of exactly zero does not expand
        assert edge["n_nodes"] == B
        flat = generate(w, w_stop=zero, b_stop=1.0, max_depth=0)
        assert flat["n_nodes"] == B
        tight = generate(w, w_stop=zero, b_stop=1.0, max_nodes=B + 7)
        assert tight["n_nodes"] == B + 6 and tight["truncated"] >= 1
        paths(tight, B)
        exact = generate(w, w_stop=zero, b_stop=1.0, max_nodes=B)
        assert exact["n_nodes"] == B and exact["truncated"] == B


def test_argument_checks():
    w = synth.topdown_workload("td_small")
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    L = binding.lib()
    ctx = binding.tl_td_create(w.hidden, dev(w.u_td), dev(w.b_td), dev(w.w_stop), w.b_stop)
    try:
        out = binding.tl_td_generate(ctx, dev(w.h_root), dev(w.c_root), w.max_nodes, w.max_depth)
        assert binding.tl_td_status(ctx) == binding.TL_OK
        p = [out[k].data_ptr() for k in ("h", "c", "parent", "left", "right", "depth", "score", "counts")]
        st = torch.cuda.current_stream().cuda_stream
        assert L.tl_td_generate(ctx, 0, 10, 3, *p, st) == binding.TL_EINVAL
        assert L.tl_td_generate(ctx, 5, 4, 3, *p, st) == binding.TL_EINVAL
        assert L.tl_td_generate(ctx, 5, 100, -1, *p, st) == binding.TL_EINVAL
        assert L.tl_td_generate(ctx, 5, 100, 3, None, *p[1:], st) == binding.TL_EINVAL
        assert L.tl_td_generate(None, 5, 100, 3, *p, st) == binding.TL_EINVAL
    finally:
        binding.tl_td_destroy(ctx)
    import ctypes
    bad = ctypes.c_void_p()
    u, b, ws = dev(w.u_td), dev(w.b_td), dev(w.w_stop)
    assert L.tl_td_create(0, u.data_ptr(), b.data_ptr(), ws.data_ptr(), 0.0, 0, ctypes.byref(bad)) == binding.TL_EINVAL
    assert L.tl_td_create(w.hidden, None, b.data_ptr(), ws.data_ptr(), 0.0, 0, ctypes.byref(bad)) == binding.TL_EINVAL
