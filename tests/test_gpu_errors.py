"""Error paths of the C ABI on the GPU.  Every case is rejected by the host or by the structure pass before any
cell reads through a bad index, or ends in the scheduler's bounded wait: all kernels exit normally."""
import numpy as np
import pytest
import torch

from paper_1809_00832_amd import binding, synth
from paper_1809_00832_amd.synth import TreeBatch

pytestmark = pytest.mark.gpu
SCHEDULERS = ["level_host", "level_device", "ready", "ready_priority", "dataflow"]


def run_expect(params, trees, sched, expect, **kw):
    net = binding.TreeNet(params, scheduler=sched, **kw)
    try:
        net.load(trees)
        net.batch["h"].zero_()
        try:
            net.forward()
            code = binding.tl_status(net.ctx)
        except binding.TLError as e:         # rejected by the host before anything was enqueued
            code = e.code
        assert code == expect, "%s: got %s, expected %s" % (sched, binding.tl_strerror(code), binding.tl_strerror(expect))
        # the context stays usable: a good batch afterwards evaluates without error
        good = synth.make_trees(3, [4, 2], ["random"] * 2, params.vocab)
        net.load(good)
        net.forward()
        assert binding.tl_status(net.ctx) == binding.TL_OK
        assert torch.isfinite(net.batch["h"]).all()
    finally:
        net.close()


def small_params():
    return synth.make_treelstm_params(1, 50, 8, 32, "xavier")


def good_trees():
    return synth.make_trees(2, [5, 3, 6], ["random"] * 3, 50)


@pytest.mark.parametrize("sched", SCHEDULERS)
def test_structure_errors_are_latched(sched):
    print("case structure errors", sched, flush=True)
    p = small_params()
    t = good_trees()
    off = [int(x) for x in t.tree_off]

    def variant(**chg):
        d = dict(tree_off=t.tree_off.copy(), left=t.left.copy(), right=t.right.copy(), word=t.word.copy())
        for k, f in chg.items():
            f(d[k])
        return TreeBatch(**d)

    internal = int(np.flatnonzero(t.left >= 0)[0])
    leaf = int(np.flatnonzero(t.left < 0)[0])
    cases = {
        "child in another tree": variant(left=lambda a: a.__setitem__(off[0], off[1])),
        "child index beyond the batch": variant(right=lambda a: a.__setitem__(internal, t.n_nodes + 5)),
        "one child missing": variant(right=lambda a: a.__setitem__(internal, -1)),
        "node with two parents": variant(left=lambda a: a.__setitem__(internal, int(t.right[internal]))),
        "word id beyond the vocabulary": variant(word=lambda a: a.__setitem__(leaf, 50)),
        "negative word id": variant(word=lambda a: a.__setitem__(leaf, -1)),
        "offsets not ascending": variant(tree_off=lambda a: a.__setitem__(1, off[2])),
        "last offset is not the node count": variant(tree_off=lambda a: a.__setitem__(3, off[3] - 1)),
    }
    for what, bad in cases.items():
        print("   ", what, flush=True)
        run_expect(p, bad, sched, binding.TL_ESTRUCT)


def cyclic_batch():
    """One tree range holding a proper 3-node tree plus a detached 2-cycle with two leaves:
    0 = (1, 2), 3 = (4, 5), 4 = (3, 6); leaves 1, 2, 5, 6.  One root, every node one parent, counts consistent."""
    left = np.array([1, -1, -1, 4, 3, -1, -1], np.int32)
    right = np.array([2, -1, -1, 5, 6, -1, -1], np.int32)
    word = np.array([-1, 3, 4, -1, -1, 5, 6], np.int32)
    return TreeBatch(np.array([0, 7], np.int32), left, right, word)


@pytest.mark.parametrize("sched", SCHEDULERS)
def test_unreachable_nodes(sched):
    """Level schedulers (and validate=1) see that the bottom-up sweep does not reach every node; the ready
    scheduler without validation runs out of its (here: tiny) spin budget and reports a stall."""
    print("case cycle", sched, flush=True)
    p = small_params()
    if sched.startswith("ready"):
        run_expect(p, cyclic_batch(), sched, binding.TL_ESTALL, spin_limit=2000)
        run_expect(p, cyclic_batch(), sched, binding.TL_ESTRUCT, validate=1)
    else:
        run_expect(p, cyclic_batch(), sched, binding.TL_ESTRUCT)


def test_host_side_argument_checks():
    p = small_params()
    t = good_trees()
    net = binding.TreeNet(p, scheduler="ready")
    try:
        b = net.load(t)
        L = binding.lib()
        args = [b["tree_off"], b["left"], b["right"], b["word"], b["h"], b["c"], b["h_root"], b["c_root"], b["root"]]
        ptr = [x.data_ptr() for x in args]
        st = torch.cuda.current_stream().cuda_stream
        assert L.tl_forward(net.ctx, 0, b["N"], *ptr, st) == binding.TL_EINVAL
        assert L.tl_forward(net.ctx, 0, 0, *([None] * 9), st) == binding.TL_OK                      # an empty batch is a no-op
        assert binding.tl_status(net.ctx) == binding.TL_OK
        assert binding.tl_last_stats(net.ctx)["n_workgroups"] == 0
        assert L.tl_forward(net.ctx, b["B"], b["B"] - 1, *ptr, st) == binding.TL_EINVAL
        assert L.tl_forward(net.ctx, b["B"], b["N"], None, *ptr[1:], st) == binding.TL_EINVAL
        assert L.tl_forward(net.ctx, b["B"], b["N"], *ptr[:5], None, *ptr[6:], st) == binding.TL_EINVAL   # c missing
        assert L.tl_forward(net.ctx, b["B"], b["N"] - 1, *ptr, st) == binding.TL_ESTRUCT             # N + B odd
        assert L.tl_forward(None, b["B"], b["N"], *ptr, st) == binding.TL_EINVAL
        assert L.tl_forward(net.ctx, b["B"], b["N"], *ptr, st) == binding.TL_OK
        assert binding.tl_status(net.ctx) == binding.TL_OK
    finally:
        net.close()
    with pytest.raises(binding.TLError):
        binding.tl_create(7, 0, 0, 10, 4, 4, torch.zeros(10, 4, device="cuda"))
    with pytest.raises(binding.TLError):          # TreeRNN needs embed_dim == hidden
        z = torch.zeros(8, 8, device="cuda")
        binding.tl_create(binding.TL_TREERNN, 0, 0, 8, 8, 4, z, u=z, b=z)


@pytest.mark.parametrize("precision", ["f32", "bf16"])
@pytest.mark.parametrize("name", ["sentence", "throughput", "treernn"])
def test_results_do_not_depend_on_the_schedule(name, precision):
    """Every data path sums a node's contraction in the same order (four quarters of the K axis,
    each in k order, added in quarter order), whatever rows share its tile.  So the schedulers agree bit
    for bit with each other and from run to run, although the ready scheduler forms different tiles every time.
    (Same recursion, different execution order, identical numbers: the claim of Section 5's numerical check.)
    One exception: in fp32 the data-flow scheduler evaluates a piece's last block of up to 12 rows with the 4x4x1
    matrix instruction, which sums every quarter as four interleaved chains; which nodes those are is fixed by the
    batch, so it still repeats its own bits from run to run, and agrees with the others to rounding."""
    print("case determinism", name, precision, flush=True)
    w = synth.workload(name)
    outs = []
    for sched in ("ready", "level_device", "level_host", "ready_priority", "dataflow"):
        net = binding.TreeNet(w.params, scheduler=sched, precision=binding.TL_F32 if precision == "f32" else binding.TL_BF16_IN)
        try:
            got = net.run(w.trees)
            outs.append((sched, got["h"].copy(), None if got["c"] is None else got["c"].copy()))
            for again in range(3):
                net.batch["h"].fill_(float("nan"))
                net.forward()
                assert binding.tl_status(net.ctx) == 0
                h2 = net.batch["h"].cpu().numpy()
                diff = int((h2 != got["h"]).sum())
                assert diff == 0, "%s run %d: %d elements differ from the first run, max %.3e" % (
                    sched, again, diff, np.abs(h2 - got["h"]).max())
        finally:
            net.close()
    for sched, h, c in outs[1:]:
        if sched == "dataflow" and precision == "f32":
            np.testing.assert_allclose(h, outs[0][1], rtol=2e-5, atol=2e-6, err_msg="dataflow vs ready: h")
            if c is not None:
                np.testing.assert_allclose(c, outs[0][2], rtol=2e-5, atol=2e-6, err_msg="dataflow vs ready: c")
            continue
        diff = int((h != outs[0][1]).sum())
        assert diff == 0, "%s vs ready: %d h elements differ, max %.3e" % (sched, diff, np.abs(h - outs[0][1]).max())
        assert c is None or np.array_equal(c, outs[0][2]), "%s vs ready: c differs" % sched


@pytest.mark.parametrize("sched", ["ready", "level_device", "ready_priority", "dataflow"])
def test_forward_replayed_from_a_hip_graph(sched):
    """tl_forward of the two device-scheduled variants makes no host round trip and clears its state with fill
    kernels, so it can be captured in a HIP graph.  Every replay, with eager work and synchronisation between
    replays and with new child states poisoned each time, must reproduce the eager result bit for bit."""
    print("case graph", sched, flush=True)
    w = synth.workload("sentence")
    net = binding.TreeNet(w.params, scheduler=sched)
    try:
        net.load(w.trees)
        net.forward()                                   # eager: also sizes the workspace, nothing is allocated later
        torch.cuda.synchronize()
        assert binding.tl_status(net.ctx) == 0
        eager_h = net.batch["h"].clone()
        eager_c = net.batch["c"].clone()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            net.forward()
        for it in range(4):
            net.batch["h"].fill_(float("nan"))
            net.batch["c"].fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(net.batch["h"], eager_h) and torch.equal(net.batch["c"], eager_c), "replay %d differs" % it
            scratch = torch.randn(1 << 16, device="cuda").sum().item()      # unrelated eager work between replays
            assert scratch == scratch
        assert binding.tl_status(net.ctx) == 0
    finally:
        net.close()


@pytest.mark.parametrize("precision", ["f32", "bf16"])
@pytest.mark.parametrize("sched", ["ready", "level_device", "ready_priority", "dataflow"])
@pytest.mark.parametrize("name,iters", [("throughput", 300), ("sentence", 300), ("stress", 20), ("mixed_small", 200)])
def test_many_forwards_give_the_same_bits(name, iters, sched, precision):
    """Many forwards of one batch through one context: every one ends without error and with exactly the bits of
    the first (tile composition, arrival order at the barriers and queue order differ from run to run).  The state
    arrays are poisoned before every checked forward, so a row that is read before it is written shows."""
    print("case soak", name, sched, precision, flush=True)
    w = synth.workload(name)
    net = binding.TreeNet(w.params, scheduler=sched, precision=binding.TL_F32 if precision == "f32" else binding.TL_BF16_IN)
    try:
        net.load(w.trees)
        net.forward()
        torch.cuda.synchronize()
        assert binding.tl_status(net.ctx) == 0
        h0, c0 = net.batch["h"].clone(), net.batch["c"].clone()
        bad = 0
        checked = 0
        for it in range(iters):
            check = it % 10 == 9 or iters <= 20
            if check:
                net.batch["h"].fill_(float("nan"))
                net.batch["c"].fill_(float("nan"))
            net.forward()
            if check:
                checked += 1
                bad += int(not (torch.equal(net.batch["h"], h0) and torch.equal(net.batch["c"], c0)))
        torch.cuda.synchronize()
        assert binding.tl_status(net.ctx) == 0
        assert bad == 0, "%d of %d checked forwards differ from the first" % (bad, checked)
    finally:
        net.close()
