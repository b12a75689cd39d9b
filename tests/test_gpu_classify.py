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
