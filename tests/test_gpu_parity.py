"""GPU parity: the HIP library, called through its C ABI, against the CPU checker, element by element.

Tolerance (fp32 path): |gpu - ref| <= 1e-4 + 1e-3 |ref| per element; child / root indices bit-exact.
"""
import numpy as np
import pytest

import oracle
from paper_1809_00832_amd import binding, synth
from paper_1809_00832_amd.synth import CELL_TREELSTM

pytestmark = pytest.mark.gpu

SCHEDULERS = ["level_host", "level_device", "ready", "ready_priority", "dataflow"]
ATOL, RTOL = 1e-4, 1e-3


def say(*a):
    print(*a, flush=True)


def assert_close(got, ref, what):
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = ATOL + RTOL * np.abs(ref.astype(np.float64))
    worst = int(np.argmax(err - bound))
    assert (err <= bound).all(), "%s: max abs err %.3e at flat index %d (ref %.6g, got %.6g)" % (
        what, err.max(), worst, ref.flat[worst], got.flat[worst])
    return float(err.max())


def check_against_oracle(params, trees, got, ref=None, what=""):
    if ref is None:
        ref = oracle.forward_params(params, trees, n_threads=8)
    e1 = assert_close(got["h"], ref["h"], what + " h")
    assert_close(got["h_root"], ref["h_root"], what + " h_root")
    if params.cell == CELL_TREELSTM:
        assert_close(got["c"], ref["c"], what + " c")
        assert_close(got["c_root"], ref["c_root"], what + " c_root")
    _, root, _ = oracle.structure(trees.tree_off, trees.left, trees.right)
    assert np.array_equal(got["root"], root), what + " root indices"
    assert np.array_equal(got["h_root"], got["h"][root]), what + " h_root is a copy of the root rows"
    return e1


_ref_cache = {}


def reference(name):
    if name not in _ref_cache:
        w = synth.workload(name)
        _ref_cache[name] = (w, oracle.forward_params(w.params, w.trees, n_threads=8))
    return _ref_cache[name]


@pytest.mark.parametrize("sched", SCHEDULERS)
@pytest.mark.parametrize("name", ["tiny", "sentence", "treernn", "rntn", "throughput"])
def test_workload_matches_oracle(name, sched):
    say("case", name, sched)
    w, ref = reference(name)
    net = binding.TreeNet(w.params, scheduler=sched)
    try:
        got = net.run(w.trees)
        err = check_against_oracle(w.params, w.trees, got, ref, "%s/%s" % (name, sched))
        say("   max abs err h %.3e" % err, binding.tl_last_stats(net.ctx))
    finally:
        net.close()


@pytest.mark.parametrize("sched", SCHEDULERS)
def test_stress_shapes_every_node(sched):
    """Full 64-tree batch of 1024-leaf chains and balanced trees: every node of every tree, h and c, against the
    checker (which evaluates the whole batch once per session, one thread per core)."""
    say("case stress", sched)
    if "stress" not in _ref_cache:
        w = synth.workload("stress")
        _ref_cache["stress"] = (w, oracle.forward_params(w.params, w.trees, n_threads=16))
    w, ref = _ref_cache["stress"]
    net = binding.TreeNet(w.params, scheduler=sched)
    try:
        got = net.run(w.trees)
        err = check_against_oracle(w.params, w.trees, got, ref, "stress/%s" % sched)
        stats = binding.tl_last_stats(net.ctx)
        say("   max abs err h %.3e" % err, stats)
        if sched.startswith("level"):
            assert stats["n_levels"] == 1024
    finally:
        net.close()


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_critical_path_first_on_a_mixed_batch(precision):
    """A few deep chains at the end of a batch of shallow trees: the priority variant of the ready scheduler moves
    the chains' first nodes to the front of the queue and hands each chain back to one gang step by step.  Same
    numbers as every other scheduler, bit for bit; chains and a sample of the shallow trees against the checker."""
    say("case mixed batch", precision)
    w = synth.workload("mixed_small")
    prec = binding.TL_F32 if precision == "f32" else binding.TL_BF16_IN
    outs = {}
    for sched in ("ready_priority", "level_device", "ready"):
        net = binding.TreeNet(w.params, scheduler=sched, precision=prec)
        try:
            outs[sched] = net.run(w.trees)
            if sched == "ready_priority":
                for _ in range(5):                       # tile composition differs from run to run, the bits do not
                    net.batch["h"].fill_(float("nan"))
                    net.forward()
                    assert binding.tl_status(net.ctx) == 0
                    assert np.array_equal(net.batch["h"].cpu().numpy(), outs[sched]["h"])
        finally:
            net.close()
    for sched in ("level_device", "ready"):
        assert np.array_equal(outs[sched]["h"], outs["ready_priority"]["h"]), sched
        assert np.array_equal(outs[sched]["c"], outs["ready_priority"]["c"]), sched
    B = w.trees.n_trees
    pick = [B - 1, B - 3, 0, 17, 200, 511]
    sub, orig = synth.subset(w.trees, pick)
    p = w.params
    if precision == "bf16":          # the checker takes weights that are already bf16-representable
        p = synth.Params(p.cell, p.vocab, p.embed_dim, p.hidden, oracle.to_bf16(p.emb), oracle.to_bf16(p.w_leaf), p.b_leaf,
                         oracle.to_bf16(p.u), p.b, None)
    ref = oracle.forward_params(p, sub, round_bf16=precision == "bf16", n_threads=4)
    got = outs["ready_priority"]
    close = assert_close if precision == "f32" else assert_close_bf16
    close(got["h"][orig], ref["h"], "mixed h")
    close(got["c"][orig], ref["c"], "mixed c")
    close(got["h_root"][pick], ref["h_root"], "mixed h_root")


@pytest.mark.parametrize("sched", SCHEDULERS)
@pytest.mark.parametrize("mode", ["post", "random"])
def test_node_numbering_is_immaterial(mode, sched):
    say("case numbering", mode, sched)
    w, ref = reference("sentence")
    tb, new_of_old = synth.renumber(w.trees, mode, seed=5)
    net = binding.TreeNet(w.params, scheduler=sched)
    try:
        got = net.run(tb)
        assert_close(got["h"][new_of_old], ref["h"], "h")
        assert_close(got["c"][new_of_old], ref["c"], "c")
        _, root, _ = oracle.structure(tb.tree_off, tb.left, tb.right)
        assert np.array_equal(got["root"], root)
    finally:
        net.close()


@pytest.mark.parametrize("sched", SCHEDULERS)
def test_ragged_and_degenerate_batches(sched):
    """Single-node trees, a batch of one tree, two-leaf trees, tiles with a ragged tail, H not a multiple
    of 16 or 4, E not a multiple of 4."""
    say("case ragged", sched)
    cases = [
        (dict(vocab=50, E=7, H=5), [1]),
        (dict(vocab=50, E=7, H=5), [1, 1, 1]),
        (dict(vocab=50, E=12, H=20), [2]),
        (dict(vocab=50, E=10, H=6), [3, 1, 20]),          # rows 8-byte but not 16-byte aligned
        (dict(vocab=50, E=9, H=33), [1, 2, 3, 1, 70, 5]),
        (dict(vocab=50, E=64, H=64), [17] * 9 + [1] + [130]),
    ]
    for i, (dims, leaves) in enumerate(cases):
        params = synth.make_treelstm_params(40 + i, dims["vocab"], dims["E"], dims["H"], "xavier")
        trees = synth.make_trees(40 + i, leaves, ["random"] * len(leaves), dims["vocab"])
        net = binding.TreeNet(params, scheduler=sched)
        try:
            got = net.run(trees)
            check_against_oracle(params, trees, got, None, "ragged%d/%s" % (i, sched))
            # second, smaller batch through the same context (workspace and queue are reused)
            small = synth.make_trees(90 + i, leaves[:1], ["random"], dims["vocab"])
            got = net.run(small)
            check_against_oracle(params, small, got, None, "ragged%d-again/%s" % (i, sched))
        finally:
            net.close()


def test_repeated_forward_is_stable():
    """The same batch evaluated repeatedly by the ready-queue scheduler stays within tolerance of the
    checker every time (tile composition differs from run to run, values must not)."""
    say("case repeat")
    w, ref = reference("sentence")
    net = binding.TreeNet(w.params, scheduler="ready")
    try:
        net.load(w.trees)
        for it in range(20):
            net.batch["h"].fill_(float("nan"))
            net.batch["c"].fill_(float("nan"))
            net.forward()
            assert binding.tl_status(net.ctx) == 0
            assert_close(net.batch["h"].cpu().numpy(), ref["h"], "h iter %d" % it)
            assert_close(net.batch["c"].cpu().numpy(), ref["c"], "c iter %d" % it)
    finally:
        net.close()


_large_cache = {}


@pytest.mark.parametrize("sched", SCHEDULERS)
def test_large_batch_and_wide_hidden(sched):
    """Sizes at the other end: a batch of 6 000 trees (about 320 000 nodes, H=32: queue, counters, frontier lists
    and workspace far beyond one tile per workgroup, frontiers of tens of thousands of rows) and a hidden size
    above what the weight-stationary cell holds (H=576: the persistent kernels fall back to the streaming cell).
    Every node is compared."""
    say("case large", sched)
    if "big" not in _large_cache:
        sizes = synth.Stream(77, "sizes").integers(5, 50, 6000)
        params = synth.make_treelstm_params(77, 500, 16, 32, "xavier")
        trees = synth.make_trees(77, [int(v) for v in sizes], ["random"] * len(sizes), 500)
        wide_p = synth.make_treelstm_params(78, 200, 40, 576, "xavier")
        wide_t = synth.make_trees(78, [9, 1, 30, 2, 70], ["random"] * 5, 200)
        _large_cache["big"] = (params, trees, oracle.forward_params(params, trees, n_threads=8))
        _large_cache["wide"] = (wide_p, wide_t, oracle.forward_params(wide_p, wide_t, n_threads=8))
    for key in ("big", "wide"):
        params, trees, ref = _large_cache[key]
        for prec in (binding.TL_F32, binding.TL_BF16_IN):
            net = binding.TreeNet(params, scheduler=sched, precision=prec)
            try:
                got = net.run(trees)
                if prec == binding.TL_F32:
                    check_against_oracle(params, trees, got, ref, "%s/%s" % (key, sched))
                else:
                    q = round_params_bf16(params)
                    refb = oracle.forward_params(q, trees, n_threads=8, round_bf16=True)
                    assert_close_bf16(got["h"], refb["h"], "%s bf16 h" % key)
                    assert_close_bf16(got["c"], refb["c"], "%s bf16 c" % key)
                say("   %s %s nodes %d" % (key, "f32" if prec == binding.TL_F32 else "bf16", len(trees.left)),
                    binding.tl_last_stats(net.ctx))
            finally:
                net.close()


@pytest.mark.parametrize("sched", ["level_device", "ready"])
def test_hidden_sizes_between_the_register_layouts(sched):
    """Hidden sizes that fall between the sizes the weight-stationary cell is built for (its K axis is padded up to the
    next of 1, 2, 4, 5, 8, 16 k-steps per wave): H = 96, 200, 448 with E = 36, 50, 64, both precisions, a batch whose
    frontiers span several blocks and a ragged tail."""
    say("case hidden sizes", sched)
    for i, (H, E) in enumerate(((96, 36), (200, 50), (448, 64))):
        params = synth.make_treelstm_params(60 + i, 300, E, H, "xavier")
        leaves = [int(v) for v in synth.Stream(60 + i, "sizes").integers(2, 40, 24)] + [1, 90]
        trees = synth.make_trees(60 + i, leaves, ["random"] * len(leaves), 300)
        ref = oracle.forward_params(params, trees, n_threads=8)
        refb = oracle.forward_params(round_params_bf16(params), trees, n_threads=8, round_bf16=True)
        for prec in (binding.TL_F32, binding.TL_BF16_IN):
            net = binding.TreeNet(params, scheduler=sched, precision=prec)
            try:
                got = net.run(trees)
                if prec == binding.TL_F32:
                    check_against_oracle(params, trees, got, ref, "H=%d/%s" % (H, sched))
                else:
                    assert_close_bf16(got["h"], refb["h"], "H=%d bf16 h" % H)
                    assert_close_bf16(got["c"], refb["c"], "H=%d bf16 c" % H)
            finally:
                net.close()


def test_wide_frontiers_at_a_hidden_size_with_uneven_slots():
    """H = 440: 28 column groups, so the 256 workgroups of the level scheduler form 9 slots and 4 stay idle; 100 trees give
    frontiers of several steps of those slots, whose remainders the scheduler leaves to the next frontier.  Every
    node against the checker, all schedulers bit for bit (the data-flow scheduler: to rounding)."""
    say("case wide frontiers, H=440")
    params = synth.make_treelstm_params(71, 400, 52, 440, "xavier")
    leaves = [int(v) for v in synth.Stream(71, "sizes").integers(5, 50, 100)]
    trees = synth.make_trees(71, leaves, ["random"] * len(leaves), 400)
    ref = oracle.forward_params(params, trees, n_threads=8)
    first = None
    for sched in SCHEDULERS:
        net = binding.TreeNet(params, scheduler=sched)
        try:
            got = net.run(trees)
            check_against_oracle(params, trees, got, ref, "H=440/%s" % sched)
            if first is None:
                first = got
            if sched == "dataflow":      # narrow last blocks of its pieces sum in another order (fp32): equal to rounding
                np.testing.assert_allclose(got["h"], first["h"], rtol=2e-5, atol=2e-6, err_msg=sched)
                np.testing.assert_allclose(got["c"], first["c"], rtol=2e-5, atol=2e-6, err_msg=sched)
            else:
                assert np.array_equal(got["h"], first["h"]) and np.array_equal(got["c"], first["c"]), sched
            say("   ", sched, binding.tl_last_stats(net.ctx))
        finally:
            net.close()


def test_rntn_schedulers_agree_bit_for_bit():
    """RNTN: the level schedulers cut a frontier of few tiles into four workgroups per tile and column group (each
    adds up a quarter of the slices, the last one to finish adds the quarters), and so do the gangs of the ready
    schedulers for every tile; large frontiers do not.  The order of summation is the same either way, so all
    schedulers give the same bits, run after run."""
    say("case rntn bits")
    w, ref = reference("rntn")
    first = None
    for sched in SCHEDULERS:
        net = binding.TreeNet(w.params, scheduler=sched)
        try:
            net.load(w.trees)
            for it in range(3):
                net.batch["h"].fill_(float("nan"))
                net.forward()
                assert binding.tl_status(net.ctx) == 0
                h = net.batch["h"].cpu().numpy()
                if first is None:
                    first = h
                    assert_close(h, ref["h"], "rntn h")
                assert np.array_equal(h, first), "rntn %s run %d differs in bits" % (sched, it)
        finally:
            net.close()


# ----------------------------------------------------------------------------- bf16-operand path
def bf16_reference(name):
    """Checker run on bf16-representable weights / embeddings with bf16 rounding of the gathered operand."""
    key = name + "/bf16"
    if key not in _ref_cache:
        w = synth.workload(name)
        p = w.params
        q = synth.Params(p.cell, p.vocab, p.embed_dim, p.hidden, oracle.to_bf16(p.emb),
                         None if p.w_leaf is None else oracle.to_bf16(p.w_leaf), p.b_leaf, oracle.to_bf16(p.u), p.b,
                         None if p.v is None else oracle.to_bf16(p.v))
        _ref_cache[key] = (w, oracle.forward_params(q, w.trees, n_threads=8, round_bf16=True))
    return _ref_cache[key]


def assert_close_bf16(got, ref, what):
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = 2e-2 * np.maximum(1.0, np.abs(ref.astype(np.float64)))
    assert (err <= bound).all(), "%s: max abs err %.3e" % (what, err.max())
    return float(err.max())


@pytest.mark.parametrize("sched", SCHEDULERS)
@pytest.mark.parametrize("name", ["tiny", "sentence", "treernn", "throughput"])
def test_bf16_operands_match_oracle(name, sched):
    """bf16 weights, embeddings and gathered h as matrix operands; fp32 accumulate, gates, c and stored h."""
    say("case bf16", name, sched)
    w, ref = bf16_reference(name)
    net = binding.TreeNet(w.params, scheduler=sched, precision=binding.TL_BF16_IN)
    try:
        got = net.run(w.trees)
        e = assert_close_bf16(got["h"], ref["h"], "h")
        assert_close_bf16(got["h_root"], ref["h_root"], "h_root")
        if w.params.cell == CELL_TREELSTM:
            assert_close_bf16(got["c"], ref["c"], "c")
        _, root, _ = oracle.structure(w.trees.tree_off, w.trees.left, w.trees.right)
        assert np.array_equal(got["root"], root)
        # and the rounding really happens: the result differs from the fp32 path's reference
        _, ref32 = reference(name)
        say("   max abs err vs bf16 checker %.3e; distance to fp32 checker %.3e" % (e, np.abs(got["h"] - ref32["h"]).max()))
    finally:
        net.close()


def round_params_bf16(p):
    return synth.Params(p.cell, p.vocab, p.embed_dim, p.hidden, oracle.to_bf16(p.emb),
                        None if p.w_leaf is None else oracle.to_bf16(p.w_leaf), p.b_leaf, oracle.to_bf16(p.u), p.b,
                        None if p.v is None else oracle.to_bf16(p.v))


@pytest.mark.parametrize("sched", SCHEDULERS)
def test_bf16_ragged_and_degenerate_batches(sched):
    """bf16 operands with sizes that are not multiples of anything: H and E below and across the 8-element
    padding of the bf16 row copies, single-node trees, ragged tiles, a second smaller batch on the same context."""
    say("case bf16 ragged", sched)
    cases = [
        (dict(vocab=50, E=7, H=5), [1]),
        (dict(vocab=50, E=7, H=5), [1, 1, 2]),
        (dict(vocab=50, E=9, H=33), [1, 2, 3, 1, 70, 5]),
        (dict(vocab=50, E=64, H=64), [17] * 9 + [1] + [130]),
        (dict(vocab=60, E=20, H=136), [300, 2, 45]),
    ]
    for i, (dims, leaves) in enumerate(cases):
        params = synth.make_treelstm_params(70 + i, dims["vocab"], dims["E"], dims["H"], "xavier")
        trees = synth.make_trees(70 + i, leaves, ["random"] * len(leaves), dims["vocab"])
        net = binding.TreeNet(params, scheduler=sched, precision=binding.TL_BF16_IN)
        try:
            for batch in (trees, synth.make_trees(95 + i, leaves[:1], ["random"], dims["vocab"])):
                got = net.run(batch)
                ref = oracle.forward_params(round_params_bf16(params), batch, n_threads=4, round_bf16=True)
                assert_close_bf16(got["h"], ref["h"], "bf16 ragged%d h" % i)
                assert_close_bf16(got["c"], ref["c"], "bf16 ragged%d c" % i)
                assert_close_bf16(got["h_root"], ref["h_root"], "bf16 ragged%d h_root" % i)
                _, root, _ = oracle.structure(batch.tree_off, batch.left, batch.right)
                assert np.array_equal(got["root"], root)
        finally:
            net.close()


@pytest.mark.parametrize("sched", SCHEDULERS)
def test_rntn_other_sizes(sched):
    """RNTN at d = 20 and d = 96 (padded K of 64 and 256).  Magnitudes are raised so that tanh is not linear,
    but kept small enough that a level does not amplify rounding differences of its inputs (with large V the
    recursion is chaotic and no two evaluation orders agree)."""
    say("case rntn sizes", sched)
    for d, leaves in ((20, [3, 9, 1, 40]), (96, [5, 2, 70])):
        p = synth.make_rnn_params(50 + d, synth.CELL_RNTN, 300, d, scale=0.05)
        p = synth.Params(p.cell, p.vocab, d, d, p.emb * 8, None, None, p.u * 2, p.b + 0.05, p.v * (40.0 / d))
        trees = synth.make_trees(50 + d, leaves, ["random"] * len(leaves), 300)
        net = binding.TreeNet(p, scheduler=sched)
        try:
            got = net.run(trees)
            check_against_oracle(p, trees, got, None, "rntn d=%d/%s" % (d, sched))
        finally:
            net.close()


@pytest.mark.parametrize("sched", ["level_device", "level_host", "ready"])
def test_rntn_wide_frontiers(sched):
    """RNTN, d = 64, 34 balanced trees of 1 024 leaves and three others: heights of 17 700, 8 900, 4 400 ... rows, so that every way a
    frontier is cut is taken - whole tiles with one workgroup per column group (more tiles than the scratch area has units),
    rounds of whole tiles plus a round of smaller ones shared by four workgroups per column group, one round of small tiles."""
    say("case rntn wide", sched)
    d = 64
    p = synth.make_rnn_params(77, synth.CELL_RNTN, 300, d, scale=0.05)
    p = synth.Params(p.cell, p.vocab, d, d, p.emb * 8, None, None, p.u * 2, p.b + 0.05, p.v * (40.0 / d))
    trees = synth.make_trees(77, [1024] * 34 + [700, 3, 1], ["balanced"] * 34 + ["random"] * 3, 300)
    if "rntn wide" not in _ref_cache:
        _ref_cache["rntn wide"] = oracle.forward_params(p, trees, n_threads=8)
    net = binding.TreeNet(p, scheduler=sched)
    try:
        got = net.run(trees)
        check_against_oracle(p, trees, got, _ref_cache["rntn wide"], "rntn wide/%s" % sched)
        again = net.run(trees)
        assert np.array_equal(got["h"], again["h"])
    finally:
        net.close()


@pytest.mark.parametrize("sched", ["dataflow", "level_device", "ready"])
def test_two_contexts_on_two_streams_ordered_by_events(sched):
    """The documented way to use several contexts on one device: their forwards (persistent kernels that need the
    device to themselves) go to different streams but are ordered with events, here four forwards alternating
    between a TreeLSTM and a TreeRNN context.  Both results against the checker."""
    import torch
    say("case two contexts", sched)
    wa, ra = reference("sentence")
    wb, rb = reference("treernn")
    a = binding.TreeNet(wa.params, scheduler=sched)
    b = binding.TreeNet(wb.params, scheduler=sched)
    try:
        a.load(wa.trees)
        b.load(wb.trees)
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        last = None
        for it in range(4):
            for net, stream in ((a, sa), (b, sb)):
                if last is not None:
                    stream.wait_event(last)
                with torch.cuda.stream(stream):
                    if it == 3:
                        net.batch["h"].fill_(float("nan"))
                    net.forward(stream.cuda_stream)
                    last = torch.cuda.Event()
                    last.record(stream)
        torch.cuda.synchronize()
        assert binding.tl_status(a.ctx) == 0 and binding.tl_status(b.ctx) == 0
        assert_close(a.batch["h"].cpu().numpy(), ra["h"], "context A h")
        assert_close(a.batch["c"].cpu().numpy(), ra["c"], "context A c")
        assert_close(b.batch["h"].cpu().numpy(), rb["h"], "context B h")
    finally:
        a.close()
        b.close()


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_dataflow_on_many_batch_shapes(precision):
    """The data-flow scheduler cuts its private lists into pieces whose composition depends on the shapes of the trees,
    their number and the hidden size (slots per device, rows per slot, narrow last blocks).  Thirty seeded batches that
    vary all of these - single-node trees, chains, balanced and random trees, one tree or hundreds, nodes renumbered
    inside their trees - against the level scheduler on the same batch: identical bits with bf16 operands and in every
    run of its own, equal to rounding in fp32 (narrow blocks sum in another order); a sample against the checker."""
    import torch
    prec = binding.TL_F32 if precision == "f32" else binding.TL_BF16_IN
    pick = synth.Stream(977, "batch shapes")
    hiddens = [16, 40, 64, 150, 256, 512] if precision == "f32" else [64, 256, 512]
    for case in range(30):
        H = hiddens[case % len(hiddens)]
        E = [20, 52, 300][case % 3]
        B = int(pick.integers(1, [3, 40, 300][case % 3], 1)[0])
        kind = ["random", "chain", "balanced", "mixed"][case % 4]
        hi = [2, 12, 70][(case // 2) % 3] if kind != "chain" else 40
        leaves = [int(v) for v in pick.integers(1, hi, B)]
        shapes = [kind if kind != "mixed" else ["random", "chain", "balanced"][int(v)] for v in pick.integers(0, 2, B)]
        trees = synth.make_trees(2000 + case, leaves, shapes, 300)
        if case % 5 == 4:
            trees, _ = synth.renumber(trees, "random", seed=case)
        elif case % 5 == 2:
            trees, _ = synth.renumber(trees, "post")
        params = synth.make_treelstm_params(3000 + case, 300, E, H, "xavier")
        say("case shapes", precision, case, "H", H, "E", E, "trees", B, kind, "nodes", trees.n_nodes)
        outs = {}
        for sched in ("level_device", "dataflow"):
            net = binding.TreeNet(params, scheduler=sched, precision=prec)
            try:
                outs[sched] = net.run(trees)
                if sched == "dataflow":
                    for _ in range(2):
                        net.batch["h"].fill_(float("nan"))
                        net.batch["c"].fill_(float("nan"))
                        net.forward()
                        assert binding.tl_status(net.ctx) == 0
                        assert np.array_equal(net.batch["h"].cpu().numpy(), outs[sched]["h"]), "run-to-run bits, case %d" % case
            finally:
                net.close()
        a, b = outs["dataflow"], outs["level_device"]
        assert np.array_equal(a["root"], b["root"])
        for key in ("h", "c", "h_root", "c_root"):
            if precision == "bf16":
                assert np.array_equal(a[key], b[key]), "case %d %s" % (case, key)
            else:
                np.testing.assert_allclose(a[key], b[key], rtol=2e-5, atol=2e-6, err_msg="case %d %s" % (case, key))
        if case % 6 == 0:
            what = "shapes case %d / dataflow / %s" % (case, precision)
            if precision == "f32":
                check_against_oracle(params, trees, a, None, what)
            else:
                ref = oracle.forward_params(round_params_bf16(params), trees, n_threads=8, round_bf16=True)
                assert_close_bf16(a["h"], ref["h"], what + " h")
                assert_close_bf16(a["c"], ref["c"], what + " c")


@pytest.mark.parametrize("shape", ["balanced", "random", "chain"])
def test_few_large_trees_under_the_dataflow_scheduler(shape):
    """One or two trees of thousands of nodes: fewer trees than the device has sets of workgroups.  The data-flow
    scheduler deals whole trees to the sets, which suits deep narrow trees and would leave the device idle under a
    bushy one, so for such a batch both internal-node kernels are launched and the device picks by the width of the
    first frontier: bushy trees go level by level (the same bits as the level scheduler), chains stay data-flow
    (equal to rounding).  Every node against the checker either way."""
    say("case few large trees", shape)
    params = synth.make_treelstm_params(61, 500, 40, 256, "xavier")
    for B, L in ((1, 3000), (2, 1500)):
        trees = synth.make_trees(62 + B, [L] * B, [shape] * B, 500)
        ref = oracle.forward_params(params, trees, n_threads=8)
        outs = {}
        for sched in ("dataflow", "level_device"):
            net = binding.TreeNet(params, scheduler=sched)
            try:
                outs[sched] = net.run(trees)
                check_against_oracle(params, trees, outs[sched], ref, "%d x %d leaves %s / %s" % (B, L, shape, sched))
            finally:
                net.close()
        if shape == "chain":
            np.testing.assert_allclose(outs["dataflow"]["h"], outs["level_device"]["h"], rtol=2e-5, atol=2e-6)
            assert not np.array_equal(outs["dataflow"]["h"], outs["level_device"]["h"]), "the data-flow kernel was expected to run"
        else:
            assert np.array_equal(outs["dataflow"]["h"], outs["level_device"]["h"])
            assert np.array_equal(outs["dataflow"]["c"], outs["level_device"]["c"])
