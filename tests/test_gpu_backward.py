"""GPU parity of the TreeLSTM backward pass (tl_backward) against the CPU checker, through the C ABI.

Tolerance: |gpu - ref| <= atol + 1e-3 |ref| with atol = 1e-4 * (largest |ref| of the same gradient array): weight
gradients are sums over thousands of nodes of fp32 products, so the absolute part scales with the array.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1809_00832_amd import binding, synth

pytestmark = pytest.mark.gpu


def assert_grad_close(got, ref, what):
    ref = ref.astype(np.float64)
    err = np.abs(got.astype(np.float64) - ref)
    bound = 1e-4 * max(np.abs(ref).max(), 1e-6) + 1e-3 * np.abs(ref)
    worst = int(np.argmax(err - bound))
    assert (err <= bound).all(), "%s: max abs err %.3e (scale %.3e) at %d: ref %.6g got %.6g" % (
        what, err.max(), np.abs(ref).max(), worst, ref.flat[worst], got.flat[worst])
    return float(err.max() / max(np.abs(ref).max(), 1e-30))


def oracle_backward_whole_batch(params, trees, h, c, g_h, n_parts=16):
    """The checker's (single-threaded) backward on n_parts disjoint sets of trees, side by side from Python threads (a
    ctypes call releases the interpreter lock); the sets' weight gradients are added in float64 here, since a gradient
    with respect to a shared parameter is the sum over the trees, and every node's d_x row belongs to one tree."""
    from concurrent.futures import ThreadPoolExecutor
    B = trees.n_trees
    sizes = np.diff(trees.tree_off)
    parts = [[] for _ in range(min(n_parts, B))]
    load = np.zeros(len(parts))
    for t in np.argsort(-sizes, kind="stable"):            # largest first onto the lightest set
        k = int(np.argmin(load))
        parts[k].append(int(t))
        load[k] += sizes[t]

    def one(pick):
        sub, orig = synth.subset(trees, sorted(pick))
        return orig, oracle.backward(params, sub, h[orig], None if c is None else c[orig], g_h[orig])

    with ThreadPoolExecutor(len(parts)) as pool:
        results = list(pool.map(one, parts))
    total = {}
    for orig, r in results:
        for k, v in r.items():
            if k == "d_x":
                total.setdefault(k, np.zeros((trees.n_nodes, v.shape[1]), np.float64))[orig] = v
            else:
                total[k] = total.get(k, 0.0) + v.astype(np.float64)
    return total


def run_case(params, trees, seed, what, keep=False, scheduler="level_device", whole_batch=False):
    rng = np.random.default_rng(seed)
    net = binding.TreeNet(params, scheduler=scheduler)
    try:
        b = net.load(trees)
        binding.tl_set_keep_gates(net.ctx, keep)
        net.forward()
        assert binding.tl_status(net.ctx) == 0
        g_h = rng.standard_normal((trees.n_nodes, params.hidden)).astype(np.float32)
        g_h[rng.random(trees.n_nodes) < 0.3] = 0.0
        got = binding.tl_backward(net.ctx, b, torch.from_numpy(g_h).cuda(), params.embed_dim)
        torch.cuda.synchronize()
        assert binding.tl_status(net.ctx) == 0
        got = {k: v.cpu().numpy() for k, v in got.items()}
        h, c = b["h"].cpu().numpy(), b["c"].cpu().numpy()
    finally:
        net.close()
    # same forward states as the GPU used
    ref = oracle_backward_whole_batch(params, trees, h, c, g_h) if whole_batch else oracle.backward(params, trees, h, c, g_h)
    rel = {k: assert_grad_close(got[k], ref[k], "%s %s" % (what, k)) for k in ref}
    print("   ", what, {k: "%.1e" % v for k, v in rel.items()}, flush=True)
    assert not got["d_x"][trees.left >= 0].any()


@pytest.mark.parametrize("name", ["tiny", "sentence"])
def test_backward_matches_oracle_on_workloads(name):
    print("case backward", name, flush=True)
    w = synth.workload(name)
    run_case(w.params, w.trees, 3, name)


def test_backward_ragged_and_degenerate():
    """Sizes that are multiples of nothing, single-node trees, a batch of one, tiles with a ragged tail."""
    print("case backward ragged", flush=True)
    cases = [
        (dict(vocab=50, E=7, H=5), [1]),
        (dict(vocab=50, E=7, H=5), [1, 1, 2]),
        (dict(vocab=50, E=12, H=20), [2, 9]),
        (dict(vocab=50, E=10, H=6), [3, 1, 20]),
        (dict(vocab=50, E=9, H=33), [1, 2, 3, 1, 70, 5]),
        (dict(vocab=50, E=64, H=64), [17] * 9 + [1] + [130]),
    ]
    for i, (dims, leaves) in enumerate(cases):
        params = synth.make_treelstm_params(60 + i, dims["vocab"], dims["E"], dims["H"], "xavier")
        trees = synth.make_trees(60 + i, leaves, ["random"] * len(leaves), dims["vocab"])
        run_case(params, trees, 60 + i, "ragged%d" % i)


@pytest.mark.parametrize("keep", [False, True])
def test_backward_full_size_whole_batch(keep):
    """The `throughput` workload as it is (256 trees, 13 572 nodes, H = 512, E = 300), gates recomputed and kept:
    every gradient array of the whole batch against the checker, so that every slice of the node axis of the
    weight-gradient contraction is covered."""
    print("case backward throughput, whole batch, kept gates:", keep, flush=True)
    w = synth.workload("throughput")
    run_case(w.params, w.trees, 5, "throughput", keep=keep, whole_batch=True)


def test_whole_batch_reference_equals_the_checker_in_one_piece():
    """The split of the checker's backward over sets of trees (used for the full-size batches) against the checker
    run on the same batch in one piece."""
    w = synth.workload("sentence")
    rng = np.random.default_rng(11)
    fw = oracle.forward_params(w.params, w.trees, n_threads=4)
    g_h = rng.standard_normal(fw["h"].shape).astype(np.float32)
    one = oracle.backward(w.params, w.trees, fw["h"], fw["c"], g_h)
    many = oracle_backward_whole_batch(w.params, w.trees, fw["h"], fw["c"], g_h, n_parts=7)
    for k in one:
        assert np.abs(many[k] - one[k]).max() <= 1e-6 * max(np.abs(one[k]).max(), 1e-30), k


@pytest.mark.parametrize("scheduler", ["level_device", "ready", "level_host", "dataflow"])
def test_backward_from_kept_gate_activations(scheduler):
    """Training mode: the forward keeps every node's gate activations and the backward takes them instead of
    recomputing the contraction.  Same bar against the checker, for every forward data path (weight-stationary cell
    under the two device schedulers, streaming cell under host-driven levels and for sizes the former does not
    take), plus: the forward's own results do not change, and a forward of another batch in between (which
    invalidates what was kept) sends the backward down the recomputing path again."""
    print("case backward kept gates", scheduler, flush=True)
    for name in ("tiny", "sentence"):
        w = synth.workload(name)
        run_case(w.params, w.trees, 7, name + " kept", keep=True, scheduler=scheduler)
    for i, (dims, leaves) in enumerate([(dict(vocab=50, E=7, H=5), [1, 1, 2]), (dict(vocab=50, E=10, H=6), [3, 1, 20]),
                                        (dict(vocab=50, E=9, H=33), [1, 2, 3, 1, 70, 5]),
                                        (dict(vocab=50, E=64, H=64), [17] * 9 + [1] + [130])]):
        params = synth.make_treelstm_params(80 + i, dims["vocab"], dims["E"], dims["H"], "xavier")
        trees = synth.make_trees(80 + i, leaves, ["random"] * len(leaves), dims["vocab"])
        run_case(params, trees, 80 + i, "ragged%d kept" % i, keep=True, scheduler=scheduler)
    w = synth.workload("sentence")
    net = binding.TreeNet(w.params, scheduler=scheduler)
    try:
        b = net.load(w.trees)
        net.forward()
        h_plain = b["h"].clone()
        g_h = torch.randn((w.trees.n_nodes, w.params.hidden), device="cuda")
        recomputed = binding.tl_backward(net.ctx, b, g_h, w.params.embed_dim)
        binding.tl_set_keep_gates(net.ctx, True)
        net.forward()
        assert torch.equal(b["h"], h_plain), "keeping the gates changed the forward"
        kept = binding.tl_backward(net.ctx, b, g_h, w.params.embed_dim)
        for k in kept:
            scale = float(recomputed[k].abs().max())
            assert float((kept[k] - recomputed[k]).abs().max()) <= 1e-4 * max(scale, 1e-6), k
        # another batch through the same context: what was kept no longer belongs to b
        other = binding.TreeNet(w.params, scheduler=scheduler)
        try:
            ob = other.load(synth.make_trees(5, [4, 9], ["random"] * 2, w.params.vocab))
            L = binding.lib()
            st = torch.cuda.current_stream().cuda_stream
            args = [ob[k].data_ptr() for k in ("tree_off", "left", "right", "word", "h", "c", "h_root", "c_root", "root")]
            assert L.tl_forward(net.ctx, ob["B"], ob["N"], *args, st) == binding.TL_OK
            again = binding.tl_backward(net.ctx, b, g_h, w.params.embed_dim)
            torch.cuda.synchronize()
            for k in again:
                scale = float(recomputed[k].abs().max())
                assert float((again[k] - recomputed[k]).abs().max()) <= 1e-4 * max(scale, 1e-6), k
        finally:
            other.close()
    finally:
        net.close()


def _workload_ws(H):
    """37 trees of mixed shapes (a single leaf, chains, balanced and random trees) at H = 128, the smallest hidden size whose
    operand gradient runs on weight-stationary workgroups, or 384, the one whose pieces of a row are not a power of two."""
    counts = [1, 2, 3, 17, 64, 100, 33] + list(synth.Stream(7, "leaves").integers(2, 60, 30))
    shapes = ["random", "chain", "balanced", "chain", "balanced", "random", "chain"] + ["random"] * 30
    return synth.Workload("h%d" % H, synth.make_trees(7, counts, shapes, 1000), synth.make_treelstm_params(7, 1000, 64, H, "xavier"))


@pytest.mark.parametrize("name", ["sentence", "throughput", "stress", "treernn", "h128", "h384"])
def test_backward_that_does_not_wait_gives_the_same_bits(name):
    """tl_set_async_backward: all heights in one persistent kernel (TreeLSTM from kept gate activations, TreeRNN), no read-back
    of the heights.  Same contractions in the same order as the per-height launches, so the gradients that reach the leaves
    must agree bit for bit; a malformed batch is then reported by tl_status, not by the call."""
    print("case backward without waiting", name, flush=True)
    w = _workload_ws(int(name[1:])) if name in ("h128", "h384") else synth.workload(name)
    net = binding.TreeNet(w.params, scheduler="dataflow")
    try:
        b = net.load(w.trees)
        binding.tl_set_keep_gates(net.ctx, True)
        net.forward()
        g_h = torch.randn((w.trees.n_nodes, w.params.hidden), device="cuda", generator=torch.Generator("cuda").manual_seed(3))
        binding.tl_set_async_backward(net.ctx, -1)           # launches per height whatever the number of heights
        waited = {k: v.clone() for k, v in binding.tl_backward(net.ctx, b, g_h, w.params.embed_dim).items()}
        for mode in (1, 0):                                  # 0: the default picks the kernel by the number of heights
            binding.tl_set_async_backward(net.ctx, mode)
            got = binding.tl_backward(net.ctx, b, g_h, w.params.embed_dim)
            assert binding.tl_status(net.ctx) == 0
            assert set(got) == set(waited)
            # d_x is the end of the chain of gate and operand gradients and is summed in a fixed order; the parameter
            # gradients are added up over the nodes with atomics, in an order that differs from run to run
            assert torch.equal(got["d_x"], waited["d_x"])
            for k in got:
                scale = float(waited[k].abs().max())
                assert float((got[k] - waited[k]).abs().max()) <= 2e-5 * max(scale, 1e-6), k
        # another upstream gradient through the same context and workspace: nothing of the first call's intermediate rows may
        # be seen again (the persistent kernel reads them through the caches)
        g_h2 = torch.randn((w.trees.n_nodes, w.params.hidden), device="cuda", generator=torch.Generator("cuda").manual_seed(4))
        binding.tl_set_async_backward(net.ctx, -1)
        waited2 = {k: v.clone() for k, v in binding.tl_backward(net.ctx, b, g_h2, w.params.embed_dim).items()}
        for mode in (1, 0):
            binding.tl_set_async_backward(net.ctx, mode)
            got2 = binding.tl_backward(net.ctx, b, g_h2, w.params.embed_dim)
            assert torch.equal(got2["d_x"], waited2["d_x"])
            assert not torch.equal(got2["d_x"], waited["d_x"])
            got = binding.tl_backward(net.ctx, b, g_h, w.params.embed_dim)       # and back
            assert torch.equal(got["d_x"], waited["d_x"])
        if name in ("throughput", "h128", "h384", "treernn"):  # twenty more calls of the persistent kernel: the same bits every time
            binding.tl_set_async_backward(net.ctx, 1)
            for _ in range(20):
                assert torch.equal(binding.tl_backward(net.ctx, b, g_h, w.params.embed_dim)["d_x"], waited["d_x"])
            assert binding.tl_status(net.ctx) == 0
        if name in ("h128", "h384"):                         # these sizes against the checker as well, through the call that does not wait
            g = g_h.cpu().numpy()
            ref = oracle.backward(w.params, w.trees, b["h"].cpu().numpy(), b["c"].cpu().numpy(), g)
            for k in ref:
                assert_grad_close(got[k].cpu().numpy(), ref[k], "%s without waiting %s" % (name, k))
        if name == "h128":
            # default mode at a size of the weight-stationary form: everything is enqueued before the call waits for the
            # structure pass's status, which it still returns
            bad = dict(b)
            bad["left"] = b["left"].clone()
            bad["left"][w.trees.n_nodes - 1] = 0             # the last leaf gets one child, and that in another tree
            binding.tl_set_async_backward(net.ctx, 0)
            with pytest.raises(RuntimeError):
                binding.tl_backward(net.ctx, bad, g_h, w.params.embed_dim)
            assert binding.tl_status(net.ctx) == binding.TL_ESTRUCT
            again = binding.tl_backward(net.ctx, b, g_h, w.params.embed_dim)        # and the context goes on
            assert torch.equal(again["d_x"], waited["d_x"])
        if name == "sentence":
            bad = dict(b)
            bad["left"] = b["left"].clone()
            bad["left"][w.trees.n_nodes - 1] = 0             # node 0 gets a second parent
            binding.tl_set_async_backward(net.ctx, 1)
            binding.tl_backward(net.ctx, bad, g_h, w.params.embed_dim)
            assert binding.tl_status(net.ctx) == binding.TL_ESTRUCT
            binding.tl_set_async_backward(net.ctx, False)
            with pytest.raises(RuntimeError):
                binding.tl_backward(net.ctx, bad, g_h, w.params.embed_dim)
    finally:
        net.close()


def test_backward_argument_checks():
    print("case backward arguments", flush=True)
    w = synth.workload("tiny")
    net = binding.TreeNet(w.params, scheduler="level_device", precision=binding.TL_BF16_IN)
    try:
        b = net.load(w.trees)
        net.forward()
        with pytest.raises(binding.TLError):
            binding.tl_backward(net.ctx, b, torch.zeros((w.trees.n_nodes, w.params.hidden), device="cuda"), w.params.embed_dim)
    finally:
        net.close()
    w4 = synth.workload("treernn")
    net = binding.TreeNet(w4.params, scheduler="level_device")
    try:
        b = net.load(w4.trees)
        L = binding.lib()
        p = b["h"].data_ptr()
        assert L.tl_backward(net.ctx, b["B"], b["N"], *([p] * 6), None, *([p] * 6), None) == binding.TL_EINVAL      # g_h missing
    finally:
        net.close()


def test_sgd_update_changes_the_context_as_the_formula_says():
    """tl_sgd_update against the definition written out in numpy float32 (theta - lr * g, product rounded, then
    difference): dense parameters bit for bit, the embedding rows (atomics over leaves that share a word) to 1e-6;
    and a forward through the updated context equals the forward of a fresh context created from those
    parameters: everything derived from them was rebuilt."""
    print("case sgd update", flush=True)
    w = synth.workload("sentence")
    p, t = w.params, w.trees
    lr = np.float32(0.05)
    net = binding.TreeNet(p, scheduler="level_device")
    try:
        b = net.load(t)
        binding.tl_set_keep_gates(net.ctx, True)
        net.forward()
        g_h = torch.randn((t.n_nodes, p.hidden), device="cuda")
        grads = binding.tl_backward(net.ctx, b, g_h, p.embed_dim)
        binding.tl_sgd_update(net.ctx, float(lr), b, grads)
        new = {k: v.cpu().numpy() for k, v in binding.tl_get_params(net.ctx, p.vocab, p.embed_dim, p.hidden).items()}
        g = {k: v.cpu().numpy() for k, v in grads.items()}
        for key, old, grad in (("u", p.u, g["d_u"]), ("b", p.b, g["d_b"]), ("w_leaf", p.w_leaf, g["d_w_leaf"]),
                               ("b_leaf", p.b_leaf, g["d_b_leaf"])):
            want = (old.astype(np.float32) - (lr * grad.astype(np.float32)).astype(np.float32)).astype(np.float32)
            assert np.array_equal(new[key], want.reshape(new[key].shape)), key
        emb = p.emb.astype(np.float64).copy()
        leaves = np.flatnonzero(t.left < 0)
        np.add.at(emb, t.word[leaves], -float(lr) * g["d_x"][leaves].astype(np.float64))
        assert np.abs(new["emb"] - emb).max() <= 1e-6
        assert np.abs(new["emb"] - p.emb).max() > 0
        net.forward()
        torch.cuda.synchronize()
        assert binding.tl_status(net.ctx) == 0
        h_after = b["h"].cpu().numpy().copy()
    finally:
        net.close()
    q = synth.Params(p.cell, p.vocab, p.embed_dim, p.hidden, new["emb"], new["w_leaf"], new["b_leaf"], new["u"], new["b"], None)
    fresh = binding.TreeNet(q, scheduler="level_device")
    try:
        got = fresh.run(t)
        assert np.array_equal(got["h"], h_after), "max diff %.3e" % np.abs(got["h"] - h_after).max()
        gb = binding.tl_backward(fresh.ctx, fresh.batch, g_h, p.embed_dim)       # the backward's packed weights too
    finally:
        fresh.close()
    ref = oracle.forward_params(q, t, n_threads=4)
    assert np.allclose(h_after, ref["h"], atol=1e-4, rtol=1e-3)


def test_a_few_training_steps_reduce_the_loss():
    """Forward, head backward, tree backward, update, five times over one batch with fixed labels: the summed
    cross-entropy goes down step after step (head parameters updated with the same rule by torch)."""
    print("case training loop", flush=True)
    w = synth.workload("tiny")
    p, t = w.params, w.trees
    rng = np.random.default_rng(4)
    C = 3
    ws = torch.from_numpy((rng.standard_normal((p.hidden, C)) * 0.3).astype(np.float32)).cuda()
    bs = torch.zeros(C, device="cuda")
    label = torch.from_numpy(rng.integers(0, C, t.n_nodes).astype(np.int32)).cuda()
    net = binding.TreeNet(p, scheduler="ready")
    losses = []
    try:
        b = net.load(t)
        binding.tl_set_keep_gates(net.ctx, True)
        for step in range(6):
            net.forward()
            hb = binding.tl_classify_backward(net.ctx, b["h"], ws, bs, label)
            grads = binding.tl_backward(net.ctx, b, hb["g_h"], p.embed_dim)
            losses.append(float(hb["loss"][0]))
            binding.tl_sgd_update(net.ctx, 0.02, b, grads)
            ws -= 0.02 * hb["d_w_s"]
            bs -= 0.02 * hb["d_b_s"]
        assert binding.tl_status(net.ctx) == 0
    finally:
        net.close()
    print("    losses", ["%.4f" % x for x in losses], flush=True)
    assert all(b_ < a_ for a_, b_ in zip(losses, losses[1:])), losses


def run_rnn_case(params, trees, seed, what, whole_batch=False):
    rng = np.random.default_rng(seed)
    net = binding.TreeNet(params, scheduler="level_device")
    try:
        b = net.load(trees)
        net.forward()
        assert binding.tl_status(net.ctx) == 0
        g_h = rng.standard_normal((trees.n_nodes, params.hidden)).astype(np.float32)
        g_h[rng.random(trees.n_nodes) < 0.3] = 0.0
        got = binding.tl_backward(net.ctx, b, torch.from_numpy(g_h).cuda(), params.embed_dim)
        torch.cuda.synchronize()
        assert binding.tl_status(net.ctx) == 0 and set(got) == {"d_u", "d_b", "d_x"}
        got = {k: v.cpu().numpy() for k, v in got.items()}
        h = b["h"].cpu().numpy()
    finally:
        net.close()
    ref = oracle_backward_whole_batch(params, trees, h, None, g_h) if whole_batch else oracle.backward(params, trees, h, None, g_h)
    rel = {k: assert_grad_close(got[k], ref[k], "%s %s" % (what, k)) for k in ref}
    print("   ", what, {k: "%.1e" % v for k, v in rel.items()}, flush=True)
    assert not got["d_x"][trees.left >= 0].any()


def test_treernn_backward_matches_oracle():
    """TreeRNN: gradients of W, b and of every leaf's embedding row against the checker, on ragged sizes, on the
    whole `treernn` workload (d = 256, 256 trees), and after an SGD step through the context."""
    print("case treernn backward", flush=True)
    for i, (d, leaves) in enumerate([(5, [1]), (6, [1, 1, 2]), (20, [2, 9]), (33, [1, 2, 3, 1, 70, 5]), (64, [17] * 9 + [1] + [130])]):
        params = synth.make_rnn_params(90 + i, synth.CELL_TREERNN, 50, d, scale=0.4)
        trees = synth.make_trees(90 + i, leaves, ["random"] * len(leaves), 50)
        run_rnn_case(params, trees, 90 + i, "rnn ragged%d" % i)
    w = synth.workload("treernn")
    run_rnn_case(w.params, w.trees, 6, "treernn, whole batch", whole_batch=True)
    sub, _ = synth.subset(w.trees, list(range(40)))
    # update: parameters as the formula says, and the next forward equals that of a fresh context
    p = w.params
    lr = np.float32(0.1)
    net = binding.TreeNet(p, scheduler="level_device")
    try:
        b = net.load(sub)
        net.forward()
        grads = binding.tl_backward(net.ctx, b, torch.randn((sub.n_nodes, p.hidden), device="cuda"), p.embed_dim)
        binding.tl_sgd_update(net.ctx, float(lr), b, grads)
        new = {k: v.cpu().numpy() for k, v in binding.tl_get_params(net.ctx, p.vocab, p.embed_dim, p.hidden, cell=p.cell).items()}
        g = {k: v.cpu().numpy() for k, v in grads.items()}
        assert np.array_equal(new["u"], p.u - (lr * g["d_u"]).astype(np.float32))
        assert np.array_equal(new["b"], p.b - (lr * g["d_b"]).astype(np.float32))
        assert np.abs(new["emb"] - p.emb).max() > 0
        net.forward()
        h_after = b["h"].cpu().numpy().copy()
    finally:
        net.close()
    q = synth.Params(p.cell, p.vocab, p.embed_dim, p.hidden, new["emb"], None, None, new["u"], new["b"], None)
    fresh = binding.TreeNet(q, scheduler="level_device")
    try:
        assert np.array_equal(fresh.run(sub)["h"], h_after)
    finally:
        fresh.close()


def test_deep_trees_take_the_persistent_kernel_by_default():
    """More than 64 heights: tl_backward in its default mode walks them in one persistent kernel.  Chains of 100 to 300 leaves
    beside shallow trees, against the checker: TreeLSTM from kept activations at a hidden size of the streaming form (72) and
    of the weight-stationary form (128), and TreeRNN (d = 40, 64, 128)."""
    print("case backward, deep trees, default mode", flush=True)
    leaves = [300, 1, 7, 100, 33, 150, 2]
    shapes = ["chain", "random", "balanced", "chain", "random", "chain", "random"]
    for i, H in enumerate([72, 128]):
        params = synth.make_treelstm_params(120 + i, 60, 24, H, "xavier")
        trees = synth.make_trees(120 + i, leaves, shapes, 60)
        run_case(params, trees, 120 + i, "deep lstm H=%d" % H, keep=True, scheduler="dataflow")
    for i, d in enumerate([40, 64, 128]):                   # (128: weight-stationary form of the persistent kernel)
        params = synth.make_rnn_params(130 + i, synth.CELL_TREERNN, 60, d, scale=0.4)
        trees = synth.make_trees(130 + i, leaves, shapes, 60)
        run_rnn_case(params, trees, 130 + i, "deep rnn d=%d" % d)


def run_rntn_case(params, trees, seed, what, whole_batch=False):
    rng = np.random.default_rng(seed)
    net = binding.TreeNet(params, scheduler="level_device")
    try:
        b = net.load(trees)
        net.forward()
        assert binding.tl_status(net.ctx) == 0
        g_h = rng.standard_normal((trees.n_nodes, params.hidden)).astype(np.float32)
        g_h[rng.random(trees.n_nodes) < 0.3] = 0.0
        got = binding.tl_backward(net.ctx, b, torch.from_numpy(g_h).cuda(), params.embed_dim, rntn=True)
        torch.cuda.synchronize()
        assert binding.tl_status(net.ctx) == 0
        got = {k: v.cpu().numpy() for k, v in got.items()}
        h = b["h"].cpu().numpy()
    finally:
        net.close()
    ref = oracle_backward_whole_batch(params, trees, h, None, g_h) if whole_batch else oracle.backward(params, trees, h, None, g_h)
    rel = {k: assert_grad_close(got["d_w_leaf" if k == "d_v" else k], ref[k], "%s %s" % (what, k)) for k in ref}
    print("   ", what, {k: "%.1e" % v for k, v in rel.items()}, flush=True)
    assert not got["d_x"][trees.left >= 0].any()


def test_rntn_backward_matches_oracle():
    """RNTN: gradients of V, W, b and of every leaf's embedding row against the checker, on ragged sizes and on the
    whole `rntn` workload (d = 64, 256 trees); then an SGD step: parameters as the formula says, and the next
    forward equals that of a fresh context."""
    print("case rntn backward", flush=True)
    for i, (d, leaves) in enumerate([(3, [1]), (5, [1, 1, 2]), (8, [2, 9]), (12, [1, 2, 3, 1, 40, 5]), (32, [17] * 5 + [1] + [70])]):
        params = synth.make_rnn_params(95 + i, synth.CELL_RNTN, 50, d, scale=0.4)
        trees = synth.make_trees(95 + i, leaves, ["random"] * len(leaves), 50)
        run_rntn_case(params, trees, 95 + i, "rntn ragged%d" % i)
    w = synth.workload("rntn")
    run_rntn_case(w.params, w.trees, 8, "rntn, whole batch", whole_batch=True)
    sub, _ = synth.subset(w.trees, list(range(12)))
    p = w.params
    lr = np.float32(0.1)
    net = binding.TreeNet(p, scheduler="level_device")
    try:
        b = net.load(sub)
        net.forward()
        grads = binding.tl_backward(net.ctx, b, torch.randn((sub.n_nodes, p.hidden), device="cuda"), p.embed_dim, rntn=True)
        binding.tl_sgd_update(net.ctx, float(lr), b, grads)
        new = {k: v.cpu().numpy() for k, v in binding.tl_get_params(net.ctx, p.vocab, p.embed_dim, p.hidden, cell=p.cell).items()}
        g = {k: v.cpu().numpy() for k, v in grads.items()}
        assert np.array_equal(new["u"], p.u - (lr * g["d_u"]).astype(np.float32))
        assert np.array_equal(new["b"], p.b - (lr * g["d_b"]).astype(np.float32))
        assert np.array_equal(new["w_leaf"], p.v - (lr * g["d_w_leaf"]).astype(np.float32))
        net.forward()
        h_after = b["h"].cpu().numpy().copy()
    finally:
        net.close()
    q = synth.Params(p.cell, p.vocab, p.embed_dim, p.hidden, new["emb"], None, None, new["u"], new["b"], new["w_leaf"])
    fresh = binding.TreeNet(q, scheduler="level_device")
    try:
        assert np.array_equal(fresh.run(sub)["h"], h_after)
    finally:
        fresh.close()
