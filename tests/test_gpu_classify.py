"""GPU parity of the per-node classifier head (tl_classify) against the CPU checker, through the C ABI.

Tolerance: |gpu - ref| <= 1e-5 + 1e-4 |ref| per probability (fp32 dot products of up to 512 terms, fp32 exp).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1809_00832_amd import binding, synth

pytestmark = pytest.mark.gpu


def make_net(H):
    p = synth.make_treelstm_params(11, 30, 8, H, "xavier")
    return binding.TreeNet(p, scheduler="level_device")


def check(net, h, w, b, what):
    dev = torch.device("cuda")
    probs = binding.tl_classify(net.ctx, torch.from_numpy(h).to(dev), torch.from_numpy(w).to(dev), torch.from_numpy(b).to(dev))
    torch.cuda.synchronize()
    got = probs.cpu().numpy()
    ref = oracle.classify(h, w, b)
    err = np.abs(got.astype(np.float64) - ref)
    assert (err <= 1e-5 + 1e-4 * np.abs(ref)).all(), "%s: max abs err %.3e" % (what, err.max())
    assert np.allclose(got.sum(axis=1), 1.0, atol=1e-5)
    return float(err.max())


@pytest.mark.parametrize("H,C,N", [(512, 5, 13572), (512, 2, 1), (150, 32, 777), (5, 3, 37), (33, 1, 16), (64, 8, 4097)])
def test_classifier_matches_oracle(H, C, N):
    print("case classify", H, C, N, flush=True)
    rng = np.random.default_rng(H * 1000 + C)
    h = np.tanh(rng.standard_normal((N, H))).astype(np.float32)          # states of a tree network lie in (-1, 1)
    w = (rng.standard_normal((H, C)) * (2.0 / np.sqrt(H))).astype(np.float32)
    b = rng.standard_normal(C).astype(np.float32)
    net = make_net(H)
    try:
        e = check(net, h, w, b, "classify H=%d C=%d N=%d" % (H, C, N))
        print("   max abs err %.3e" % e, flush=True)
    finally:
        net.close()


def test_classifier_labels_a_forward_pass():
    """The head applied to the h rows that tl_forward has just written, on the same stream."""
    print("case classify after forward", flush=True)
    w_ = synth.workload("sentence")
    net = binding.TreeNet(w_.params, scheduler="level_device")
    try:
        net.load(w_.trees)
        net.forward()
        rng = np.random.default_rng(8)
        H = w_.params.hidden
        ws = (rng.standard_normal((H, 5)) * 0.5).astype(np.float32)
        bs = rng.standard_normal(5).astype(np.float32)
        probs = binding.tl_classify(net.ctx, net.batch["h"], torch.from_numpy(ws).cuda(), torch.from_numpy(bs).cuda())
        torch.cuda.synchronize()
        assert binding.tl_status(net.ctx) == 0
        ref_h = oracle.forward_params(w_.params, w_.trees, n_threads=4)["h"]
        ref = oracle.classify(ref_h, ws, bs)
        assert np.abs(probs.cpu().numpy() - ref).max() < 1e-4
    finally:
        net.close()


def test_classifier_argument_checks():
    print("case classify arguments", flush=True)
    net = make_net(512)
    try:
        L = binding.lib()
        z = torch.zeros(512 * 40, device="cuda")
        p = z.data_ptr()
        assert L.tl_classify(net.ctx, 4, p, p, p, 33, p, None) == binding.TL_EINVAL
        assert L.tl_classify(net.ctx, 4, p, p, p, 0, p, None) == binding.TL_EINVAL
        assert L.tl_classify(net.ctx, -1, p, p, p, 2, p, None) == binding.TL_EINVAL
        assert L.tl_classify(net.ctx, 4, None, p, p, 2, p, None) == binding.TL_EINVAL
        assert L.tl_classify(None, 4, p, p, p, 2, p, None) == binding.TL_EINVAL
        assert L.tl_classify(net.ctx, 0, p, p, p, 2, p, None) == binding.TL_OK
    finally:
        net.close()
    big = make_net(1024)
    try:
        z = torch.zeros(1024 * 40, device="cuda")
        p = z.data_ptr()
        assert binding.lib().tl_classify(big.ctx, 4, p, p, p, 32, p, None) == binding.TL_EINVAL     # 32 x 1024 floats of LDS
        assert binding.lib().tl_classify(big.ctx, 4, p, p, p, 16, p, None) == binding.TL_OK
        torch.cuda.synchronize()
    finally:
        big.close()


@pytest.mark.parametrize("H,C,N", [(512, 5, 13572), (512, 2, 1), (150, 32, 777), (5, 3, 37), (33, 1, 16), (64, 8, 4097)])
def test_classifier_backward_matches_oracle(H, C, N):
    """tl_classify_backward against the CPU checker: logits gradient and g_h element by element, the three sums
    (fp32 atomics over up to 13572 rows) relative to the scale of the sum."""
    print("case classify backward", H, C, N, flush=True)
    rng = np.random.default_rng(H * 1000 + C + 1)
    h = np.tanh(rng.standard_normal((N, H))).astype(np.float32)
    w = (rng.standard_normal((H, C)) * (2.0 / np.sqrt(H))).astype(np.float32)
    b = rng.standard_normal(C).astype(np.float32)
    label = rng.integers(0, C, N).astype(np.int32)
    label[rng.random(N) < 0.2] = -1
    ref = oracle.classify_backward(h, w, b, label)
    ref_probs = oracle.classify(h, w, b)
    net = make_net(H)
    try:
        dev = torch.device("cuda")
        got = binding.tl_classify_backward(net.ctx, *(torch.from_numpy(a).to(dev) for a in (h, w, b, label)))
        torch.cuda.synchronize()
        got = {k: v.cpu().numpy().astype(np.float64) for k, v in got.items()}
    finally:
        net.close()
    onehot = np.zeros((N, C))
    onehot[label >= 0, label[label >= 0]] = 1.0
    ref_dl = np.where((label >= 0)[:, None], ref_probs - onehot, 0.0)
    assert (np.abs(got["d_logits"] - ref_dl) <= 1e-5 + 1e-4 * np.abs(ref_dl)).all()
    assert (np.abs(got["g_h"] - ref["g_h"]) <= 1e-5 + 1e-4 * np.abs(ref["g_h"])).all()
    assert not got["g_h"][label < 0].any()
    for key in ("d_w_s", "d_b_s"):
        scale = max(1.0, float(np.abs(ref[key]).max()))
        err = float(np.abs(got[key] - ref[key]).max())
        assert err <= 1e-4 * scale, "%s: max abs err %.3e at scale %.3e" % (key, err, scale)
    assert abs(got["loss"][0] - ref["loss"]) <= 1e-4 * max(1.0, abs(ref["loss"]))
    print("   loss %.4f (ref %.4f)" % (got["loss"][0], ref["loss"]), flush=True)


def test_head_gradient_feeds_the_tree_backward():
    """A whole training step without the parameter update: forward, head, head backward, tree backward, each on
    the device, against the same chain in the CPU checker."""
    print("case training step", flush=True)
    w_ = synth.workload("tiny")
    p, t = w_.params, w_.trees
    rng = np.random.default_rng(21)
    H, C = p.hidden, 5
    ws = (rng.standard_normal((H, C)) * 0.5).astype(np.float32)
    bs = rng.standard_normal(C).astype(np.float32)
    label = rng.integers(0, C, t.n_nodes).astype(np.int32)
    fwd = oracle.forward_params(p, t)
    head = oracle.classify_backward(fwd["h"], ws, bs, label)
    ref = oracle.backward(p, t, fwd["h"], fwd["c"], head["g_h"])
    net = binding.TreeNet(p, scheduler="level_device")
    try:
        net.load(t)
        net.forward()
        hb = binding.tl_classify_backward(net.ctx, net.batch["h"], torch.from_numpy(ws).cuda(), torch.from_numpy(bs).cuda(),
                                          torch.from_numpy(label).cuda())
        got = binding.tl_backward(net.ctx, net.batch, hb["g_h"], p.embed_dim)
        torch.cuda.synchronize()
        assert abs(float(hb["loss"][0]) - head["loss"]) <= 1e-4 * abs(head["loss"])
        for key in ("d_u", "d_b", "d_w_leaf", "d_b_leaf"):
            g = got[key].cpu().numpy().astype(np.float64)
            scale = max(1.0, float(np.abs(ref[key]).max()))
            err = float(np.abs(g - ref[key]).max())
            assert err <= 2e-4 * scale, "%s: max abs err %.3e at scale %.3e" % (key, err, scale)
    finally:
        net.close()
