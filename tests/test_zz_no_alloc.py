"""tl_forward_noalloc (the entry point that allocates nothing: its scheduler state lives in a fixed per-GPU array)
against tl_forward, through the C ABI: same kernels, so the outputs must agree bit for bit; two calls in a row on
one context, the second with a smaller batch; both precisions, the device schedulers, all three cells; limits."""
import numpy as np
import pytest
import torch

from paper_1809_00832_amd import binding, synth

pytestmark = pytest.mark.gpu
KEYS = ("h", "c", "h_root", "c_root", "root")


def raw_call(fn, net, b):
    st = torch.cuda.current_stream().cuda_stream
    ptr = lambda t: None if t is None else t.data_ptr()
    return fn(net.ctx, b["B"], b["N"], *[ptr(b[k]) for k in ("tree_off", "left", "right", "word", "h", "c", "h_root", "c_root", "root")], st)


def outputs(net, fn, trees):
    b = net.load(trees)
    for k in ("h", "c", "h_root", "c_root"):
        if b[k] is not None:
            b[k].fill_(float("nan"))
    b["root"].fill_(-7)
    assert raw_call(fn, net, b) == binding.TL_OK
    assert binding.tl_status(net.ctx) == binding.TL_OK
    return {k: None if b[k] is None else b[k].cpu().numpy() for k in KEYS}


def same(a, b, what):
    for k in KEYS:
        if a[k] is None:
            assert b[k] is None
            continue
        assert np.isfinite(a[k]).all(), (what, k)
        assert np.array_equal(a[k], b[k]), "%s: %s differs (max %.3e)" % (what, k, np.abs(a[k].astype(np.float64) - b[k]).max())


CASES = [
    ("sentence workload", lambda: synth.workload("sentence").params, lambda: synth.workload("sentence").trees, 25),
    ("H=33, E=9 (padded bf16 rows)", lambda: synth.make_treelstm_params(40, 50, 9, 33, "xavier"),
     lambda: synth.make_trees(40, [1, 2, 3, 1, 70, 5], ["random"] * 6, 50), 50),
    ("treernn d=64", lambda: synth.make_rnn_params(41, synth.CELL_TREERNN, 50, 64, scale=0.4),
     lambda: synth.make_trees(41, [17] * 9 + [1] + [130], ["random"] * 11, 50), 50),
]


@pytest.mark.parametrize("sched", ["level_device", "ready", "ready_priority"])
@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_noalloc_equals_forward_two_calls_in_a_row(precision, sched):
    print("case noalloc", precision, sched, flush=True)
    L = binding.lib()
    prec = binding.TL_F32 if precision == "f32" else binding.TL_BF16_IN
    for what, make_params, make_trees, vocab in CASES:
        params, big = make_params(), make_trees()
        small = synth.make_trees(77, [3, 1, 6], ["random"] * 3, vocab)
        net = binding.TreeNet(params, scheduler=sched, precision=prec)
        other = binding.TreeNet(params, scheduler=sched, precision=prec)      # a context that only ever uses tl_forward
        try:
            for trees in (big, small, big):                      # the second call has the smaller input
                got = outputs(net, L.tl_forward_noalloc, trees)
                want = outputs(other, L.tl_forward, trees)
                same(got, want, "%s / %d nodes" % (what, trees.n_nodes))
        finally:
            net.close()
            other.close()


def test_noalloc_rntn_and_shared_array_between_contexts():
    """RNTN through the same entry point, and two contexts of different hidden sizes taking turns on the one array
    (a context must not depend on what the array held before its call)."""
    print("case noalloc rntn / shared array", flush=True)
    L = binding.lib()
    p = synth.make_rnn_params(52, synth.CELL_RNTN, 300, 20, scale=0.05)
    t = synth.make_trees(52, [3, 9, 1, 40], ["random"] * 4, 300)
    a = binding.TreeNet(p, scheduler="level_device")
    b = binding.TreeNet(p, scheduler="level_device")
    try:
        same(outputs(a, L.tl_forward_noalloc, t), outputs(b, L.tl_forward, t), "rntn d=20")
    finally:
        a.close()
        b.close()
    p1 = synth.make_treelstm_params(60, 300, 36, 96, "xavier")
    p2 = synth.make_treelstm_params(61, 300, 20, 37, "xavier")
    t1 = synth.make_trees(60, [30, 2, 11, 45], ["random"] * 4, 300)
    t2 = synth.make_trees(61, [9, 60, 1], ["random"] * 3, 300)
    nets = [binding.TreeNet(p1, scheduler="level_device", precision=binding.TL_BF16_IN),
            binding.TreeNet(p2, scheduler="ready", precision=binding.TL_BF16_IN)]
    refs = [binding.TreeNet(p1, scheduler="level_device", precision=binding.TL_BF16_IN),
            binding.TreeNet(p2, scheduler="ready", precision=binding.TL_BF16_IN)]
    try:
        for turn in range(3):
            for net, ref, trees in zip(nets, refs, (t1, t2)):
                same(outputs(net, L.tl_forward_noalloc, trees), outputs(ref, L.tl_forward, trees), "turn %d" % turn)
    finally:
        for n in nets + refs:
            n.close()


def test_noalloc_limits_and_device_memory():
    print("case noalloc limits", flush=True)
    L = binding.lib()
    p = synth.make_treelstm_params(62, 100, 8, 16, "xavier")
    # the largest batch it takes (16 383 nodes) and the first it does not
    n_leaves_ok = binding.TL_NOALLOC_MAX_NODES // 2
    big = synth.make_trees(62, [n_leaves_ok], ["random"], 100)
    assert big.n_nodes == binding.TL_NOALLOC_MAX_NODES - 1
    too_big = synth.make_trees(63, [n_leaves_ok, 2], ["random"] * 2, 100)
    assert too_big.n_nodes > binding.TL_NOALLOC_MAX_NODES
    net = binding.TreeNet(p, scheduler="level_device")
    ref = binding.TreeNet(p, scheduler="level_device")
    try:
        torch.cuda.synchronize()
        b = net.load(big)
        free0 = torch.cuda.mem_get_info()[0]
        assert raw_call(L.tl_forward_noalloc, net, b) == binding.TL_OK       # first call on a context that owns no workspace
        assert binding.tl_status(net.ctx) == binding.TL_OK
        assert torch.cuda.mem_get_info()[0] == free0, "device memory was allocated during the call"
        got = {k: b[k].cpu().numpy() for k in KEYS}
        same(got, outputs(ref, L.tl_forward, big), "largest batch")
        b2 = net.load(too_big)
        b2["h"].zero_()
        assert raw_call(L.tl_forward_noalloc, net, b2) == binding.TL_ELIMIT
        assert not b2["h"].any()                                             # nothing was enqueued
        assert "fixed workspace" in binding.tl_strerror(binding.TL_ELIMIT)
    finally:
        net.close()
        ref.close()
    host = binding.TreeNet(p, scheduler="level_host")
    try:
        b = host.load(synth.make_trees(64, [4, 2], ["random"] * 2, 100))
        assert raw_call(L.tl_forward_noalloc, host, b) == binding.TL_EINVAL
    finally:
        host.close()
