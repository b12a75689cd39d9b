"""ctypes binding of libtreelstm.so: same entry points as include/treelstm.h.

Argument marshalling only - every step of the forward pass runs in the HIP library.
PyTorch is used for device memory and for the stream handle.  There is no CPU
fallback: if the library has not been built, loading fails with an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtreelstm.so")

TL_TREELSTM, TL_TREERNN, TL_RNTN = 0, 1, 2
TL_F32, TL_BF16_IN = 0, 1
TL_SCHED_READY, TL_SCHED_LEVEL_DEVICE, TL_SCHED_LEVEL_HOST, TL_SCHED_READY_PRIORITY, TL_SCHED_DATAFLOW = 0, 1, 2, 3, 4
TL_OK, TL_EINVAL, TL_ENOMEM, TL_EHIP, TL_ESTRUCT, TL_ESTALL, TL_ELIMIT = 0, -1, -2, -3, -4, -5, -6
TL_NOALLOC_MAX_NODES = 16384
TL_N_STAGES, TL_PROFILE_RING = 5, 128
SCHEDULERS = {"ready": TL_SCHED_READY, "level_device": TL_SCHED_LEVEL_DEVICE, "level_host": TL_SCHED_LEVEL_HOST,
              "ready_priority": TL_SCHED_READY_PRIORITY, "dataflow": TL_SCHED_DATAFLOW}

EXPORTS = ("tl_create", "tl_forward", "tl_forward_noalloc", "tl_status", "tl_set_profiling", "tl_stage_ms", "tl_last_stats", "tl_backward",
           "tl_set_keep_gates", "tl_set_async_backward", "tl_sgd_update", "tl_get_params", "tl_classify", "tl_classify_backward", "tl_td_create", "tl_td_generate", "tl_td_status", "tl_td_destroy", "tl_strerror", "tl_destroy")


class tl_config(ctypes.Structure):
    _fields_ = [("cell", ctypes.c_int), ("precision", ctypes.c_int), ("scheduler", ctypes.c_int),
                ("validate", ctypes.c_int), ("vocab", ctypes.c_int), ("embed_dim", ctypes.c_int),
                ("hidden", ctypes.c_int), ("spin_limit", ctypes.c_int),
                ("emb", ctypes.c_void_p), ("w_leaf", ctypes.c_void_p), ("b_leaf", ctypes.c_void_p),
                ("u", ctypes.c_void_p), ("b", ctypes.c_void_p), ("v", ctypes.c_void_p)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_1809_00832_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libtreelstm.so is missing: build it with `python -m paper_1809_00832_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.tl_create.restype = ci
        L.tl_create.argtypes = [ctypes.POINTER(tl_config), ctypes.POINTER(vp)]
        L.tl_forward.restype = ci
        L.tl_forward.argtypes = [vp, ci, ci] + [vp] * 10
        L.tl_forward_noalloc.restype = ci
        L.tl_forward_noalloc.argtypes = [vp, ci, ci] + [vp] * 10
        L.tl_status.restype = ci
        L.tl_status.argtypes = [vp]
        L.tl_set_profiling.restype = ci
        L.tl_set_profiling.argtypes = [vp, ci]
        L.tl_stage_ms.restype = ci
        L.tl_stage_ms.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_float)]
        L.tl_last_stats.restype = ci
        L.tl_last_stats.argtypes = [vp] + [ctypes.POINTER(ci)] * 3
        L.tl_strerror.restype = ctypes.c_char_p
        L.tl_backward.restype = ci
        L.tl_backward.argtypes = [vp, ci, ci] + [vp] * 13
        L.tl_sgd_update.restype = ci
        L.tl_sgd_update.argtypes = [vp, ctypes.c_float, ci] + [vp] * 8
        L.tl_get_params.restype = ci
        L.tl_get_params.argtypes = [vp] * 7
        L.tl_set_keep_gates.restype = ci
        L.tl_set_keep_gates.argtypes = [vp, ci]
        L.tl_set_async_backward.restype = ci
        L.tl_set_async_backward.argtypes = [vp, ci]
        L.tl_td_create.restype = ci
        L.tl_td_create.argtypes = [ci, vp, vp, vp, ctypes.c_float, ci, ctypes.POINTER(vp)]
        L.tl_td_generate.restype = ci
        L.tl_td_generate.argtypes = [vp, ci, ci, ci] + [vp] * 9
        L.tl_td_status.restype = ci
        L.tl_td_status.argtypes = [vp]
        L.tl_td_destroy.restype = ci
        L.tl_td_destroy.argtypes = [vp]
        L.tl_classify.restype = ci
        L.tl_classify.argtypes = [vp, ci, vp, vp, vp, ci, vp, vp]
        L.tl_classify_backward.restype = ci
        L.tl_classify_backward.argtypes = [vp, ci, vp, vp, vp, ci] + [vp] * 7
        L.tl_strerror.argtypes = [ci]
        L.tl_destroy.restype = ci
        L.tl_destroy.argtypes = [vp]
        _lib = L
    return _lib


class TLError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, lib().tl_strerror(code).decode(), code))


def _check(code: int, where: str):
    if code != TL_OK:
        raise TLError(code, where)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def tl_create(cell, precision, scheduler, vocab, embed_dim, hidden, emb, w_leaf=None, b_leaf=None, u=None, b=None,
              v=None, validate=0, spin_limit=0) -> int:
    """Device tensors (fp32, contiguous) in, context handle out."""
    for t in (emb, w_leaf, b_leaf, u, b, v):
        if t is not None:
            assert t.is_cuda and t.is_contiguous() and t.dtype.is_floating_point and t.element_size() == 4
    cfg = tl_config(cell, precision, scheduler, validate, vocab, embed_dim, hidden, spin_limit,
                    _ptr(emb), _ptr(w_leaf), _ptr(b_leaf), _ptr(u), _ptr(b), _ptr(v))
    out = ctypes.c_void_p()
    _check(lib().tl_create(ctypes.byref(cfg), ctypes.byref(out)), "tl_create")
    return out.value


def tl_forward(ctx, n_trees, n_nodes, tree_off, left, right, word, h, c=None, h_root=None, c_root=None, root=None,
               stream=None) -> None:
    """int32 / fp32 device tensors in and out; `stream` is a raw hipStream_t (int) or None for torch's current one."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().tl_forward(ctx, n_trees, n_nodes, _ptr(tree_off), _ptr(left), _ptr(right), _ptr(word), _ptr(h),
                            _ptr(c), _ptr(h_root), _ptr(c_root), _ptr(root), stream), "tl_forward")


def tl_forward_noalloc(ctx, n_trees, n_nodes, tree_off, left, right, word, h, c=None, h_root=None, c_root=None, root=None,
                       stream=None) -> None:
    """Same arguments as tl_forward; the library allocates nothing during the call (fixed per-GPU workspace)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().tl_forward_noalloc(ctx, n_trees, n_nodes, _ptr(tree_off), _ptr(left), _ptr(right), _ptr(word), _ptr(h),
                                    _ptr(c), _ptr(h_root), _ptr(c_root), _ptr(root), stream), "tl_forward_noalloc")


def tl_status(ctx) -> int:
    return lib().tl_status(ctx)


def tl_set_profiling(ctx, on: bool) -> None:
    _check(lib().tl_set_profiling(ctx, int(on)), "tl_set_profiling")


def tl_stage_ms(ctx, back: int = 0):
    ms = (ctypes.c_float * TL_N_STAGES)()
    _check(lib().tl_stage_ms(ctx, back, ms), "tl_stage_ms")
    return dict(zip(("structure", "leaves", "internal", "roots", "total"), [float(x) for x in ms]))


def tl_last_stats(ctx):
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().tl_last_stats(ctx, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "tl_last_stats")
    return {"n_levels": a.value, "n_tiles": b.value, "n_workgroups": c.value}


def tl_backward(ctx, batch, g_h, embed_dim, rntn=False, stream=None):
    """Gradients for a batch that tl_forward has evaluated (`batch` is the dict TreeNet.load returns, holding h and
    c); g_h [N x H] float32 CUDA tensor.  Returns dict(d_u, d_b, d_w_leaf, d_b_leaf, d_x) of CUDA tensors for a
    TreeLSTM, dict(d_u [2H x H], d_b [H], d_x) for a TreeRNN (batch["c"] is None there), and with rntn=True also
    d_w_leaf [d x 2d x 2d], the gradient of the tensor V."""
    import torch
    N, H, E = batch["N"], int(batch["h"].shape[1]), int(embed_dim)
    assert g_h.is_cuda and g_h.dtype == torch.float32 and g_h.is_contiguous() and tuple(g_h.shape) == (N, H)
    dev = g_h.device
    lstm = batch.get("c") is not None
    ng = 5 if lstm else 1
    out = {"d_u": torch.empty((2 * H, ng * H), device=dev), "d_b": torch.empty(ng * H, device=dev),
           "d_x": torch.empty((N, E), device=dev)}
    if lstm:
        out["d_w_leaf"] = torch.empty((E, 3 * H), device=dev)
        out["d_b_leaf"] = torch.empty(3 * H, device=dev)
    elif rntn:
        out["d_w_leaf"] = torch.empty((H, 2 * H, 2 * H), device=dev)        # gradient of the tensor V
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib().tl_backward(ctx, batch["B"], N, batch["tree_off"].data_ptr(), batch["left"].data_ptr(),
                             batch["right"].data_ptr(), batch["word"].data_ptr(), batch["h"].data_ptr(),
                             _ptr(batch.get("c")), g_h.data_ptr(), out["d_u"].data_ptr(), out["d_b"].data_ptr(),
                             _ptr(out.get("d_w_leaf")), _ptr(out.get("d_b_leaf")), out["d_x"].data_ptr(), st), "tl_backward")
    return out


def tl_sgd_update(ctx, lr, batch, grads, with_embedding=True, stream=None) -> None:
    """theta -= lr * gradient for the parameters the context holds; `grads` is what tl_backward returned, `batch`
    the dict TreeNet.load returned."""
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib().tl_sgd_update(ctx, float(lr), batch["N"], batch["left"].data_ptr(), batch["word"].data_ptr(),
                               grads["d_u"].data_ptr(), grads["d_b"].data_ptr(), _ptr(grads.get("d_w_leaf")),
                               _ptr(grads.get("d_b_leaf")), grads["d_x"].data_ptr() if with_embedding else None, st),
           "tl_sgd_update")


def tl_get_params(ctx, vocab, embed_dim, hidden, cell=TL_TREELSTM, stream=None):
    """The context's current parameters as new CUDA tensors: dict(u, b, w_leaf, b_leaf, emb); dict(u, b, emb) for a
    TreeRNN; dict(u, b, w_leaf = V [d x 2d x 2d], emb) for an RNTN."""
    import torch
    H, E = int(hidden), int(embed_dim)
    ng = 5 if cell == TL_TREELSTM else 1
    new = lambda *shape: torch.empty(shape, dtype=torch.float32, device="cuda")
    out = {"u": new(2 * H, ng * H), "b": new(ng * H), "emb": new(int(vocab), E)}
    if cell == TL_TREELSTM:
        out["w_leaf"], out["b_leaf"] = new(E, 3 * H), new(3 * H)
    elif cell == TL_RNTN:
        out["w_leaf"] = new(H, 2 * H, 2 * H)
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib().tl_get_params(ctx, out["u"].data_ptr(), out["b"].data_ptr(), _ptr(out.get("w_leaf")), _ptr(out.get("b_leaf")),
                               out["emb"].data_ptr(), st), "tl_get_params")
    return out


def tl_set_keep_gates(ctx, on: bool) -> None:
    _check(lib().tl_set_keep_gates(ctx, 1 if on else 0), "tl_set_keep_gates")


def tl_set_async_backward(ctx, on) -> None:
    """True / 1: never waits; False / 0: the default (picks by the number of heights); -1: always launches per height."""
    _check(lib().tl_set_async_backward(ctx, int(on)), "tl_set_async_backward")


def tl_classify(ctx, h, w_s, b_s, probs=None, stream=None):
    """probs = softmax(h @ w_s + b_s) row by row; all arguments are float32 CUDA tensors.  Returns probs."""
    import torch
    n_rows, n_classes = int(h.shape[0]), int(w_s.shape[1])
    for t in (h, w_s, b_s):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    if probs is None:
        probs = torch.empty((n_rows, n_classes), dtype=torch.float32, device=h.device)
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib().tl_classify(ctx, n_rows, h.data_ptr(), w_s.data_ptr(), b_s.data_ptr(), n_classes, probs.data_ptr(), st),
           "tl_classify")
    return probs


def tl_classify_backward(ctx, h, w_s, b_s, label, stream=None):
    """Cross-entropy over the rows with a label in [0, C) on top of tl_classify.  h, w_s, b_s float32 and label
    int32 CUDA tensors.  Returns dict(loss [1], d_logits, g_h, d_w_s, d_b_s) of new float32 CUDA tensors."""
    import torch
    n_rows, n_classes = int(h.shape[0]), int(w_s.shape[1])
    for t in (h, w_s, b_s):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert label.is_cuda and label.dtype == torch.int32 and label.is_contiguous() and label.numel() == n_rows
    new = lambda *shape: torch.empty(shape, dtype=torch.float32, device=h.device)
    out = {"loss": new(1), "d_logits": new(n_rows, n_classes), "g_h": new(n_rows, int(h.shape[1])),
           "d_w_s": new(int(h.shape[1]), n_classes), "d_b_s": new(n_classes)}
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib().tl_classify_backward(ctx, n_rows, h.data_ptr(), w_s.data_ptr(), b_s.data_ptr(), n_classes,
                                      label.data_ptr(), out["d_logits"].data_ptr(), out["g_h"].data_ptr(),
                                      out["d_w_s"].data_ptr(), out["d_b_s"].data_ptr(), out["loss"].data_ptr(), st),
           "tl_classify_backward")
    return out


def tl_td_create(hidden, u_td, b_td, w_stop, b_stop, spin_limit=0):
    """Context of the top-down generator; u_td [H x 8H], b_td [8H], w_stop [H] float32 CUDA tensors."""
    import torch
    for t in (u_td, b_td, w_stop):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert tuple(u_td.shape) == (hidden, 8 * hidden) and b_td.numel() == 8 * hidden and w_stop.numel() == hidden
    ctx = ctypes.c_void_p()
    _check(lib().tl_td_create(int(hidden), u_td.data_ptr(), b_td.data_ptr(), w_stop.data_ptr(), float(b_stop), int(spin_limit),
                              ctypes.byref(ctx)), "tl_td_create")
    return ctx


def tl_td_generate(ctx, h_root, c_root, max_nodes, max_depth, stream=None):
    """Grows one tree per row of h_root / c_root (float32 CUDA tensors [B x H]).  Returns a dict of new CUDA tensors
    with max_nodes rows each (h, c, parent, left, right, depth, score) and counts [4]; asynchronous."""
    import torch
    B, H = int(h_root.shape[0]), int(h_root.shape[1])
    assert h_root.is_cuda and c_root.is_cuda and h_root.dtype == torch.float32 and tuple(c_root.shape) == (B, H)
    dev = h_root.device
    out = {"h": torch.empty((max_nodes, H), device=dev), "c": torch.empty((max_nodes, H), device=dev),
           "score": torch.empty(max_nodes, device=dev), "counts": torch.zeros(4, dtype=torch.int32, device=dev)}
    for k in ("parent", "left", "right", "depth"):
        out[k] = torch.empty(max_nodes, dtype=torch.int32, device=dev)
    out["h"][:B].copy_(h_root)
    out["c"][:B].copy_(c_root)
    tl_td_generate_into(ctx, B, max_depth, out, stream)
    return out


def tl_td_generate_into(ctx, n_trees, max_depth, out, stream=None):
    """The call itself on buffers that tl_td_generate allocated (root rows in place)."""
    import torch
    st = (stream or torch.cuda.current_stream()).cuda_stream
    _check(lib().tl_td_generate(ctx, int(n_trees), int(out["h"].shape[0]), int(max_depth), out["h"].data_ptr(), out["c"].data_ptr(),
                                out["parent"].data_ptr(), out["left"].data_ptr(), out["right"].data_ptr(),
                                out["depth"].data_ptr(), out["score"].data_ptr(), out["counts"].data_ptr(), st), "tl_td_generate")


def tl_td_status(ctx) -> int:
    return lib().tl_td_status(ctx)


def tl_td_destroy(ctx) -> None:
    _check(lib().tl_td_destroy(ctx), "tl_td_destroy")


def tl_strerror(code: int) -> str:
    return lib().tl_strerror(code).decode()


def tl_destroy(ctx) -> None:
    _check(lib().tl_destroy(ctx), "tl_destroy")


class TreeNet:
    """Holds a context plus device copies of a batch; thin convenience over the calls above."""

    def __init__(self, params, scheduler="ready", precision=TL_F32, validate=0, spin_limit=0, device="cuda:0"):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        dev = lambda a: None if a is None else torch.from_numpy(a).to(self.device).contiguous()
        self.cell, self.H = params.cell, params.hidden
        self.ctx = tl_create(params.cell, precision, SCHEDULERS[scheduler], params.vocab, params.embed_dim,
                             params.hidden, dev(params.emb), dev(params.w_leaf), dev(params.b_leaf), dev(params.u),
                             dev(params.b), dev(params.v), validate=validate, spin_limit=spin_limit)
        self.batch = None

    def load(self, trees):
        """Copies a batch (numpy int32 arrays) to the device and allocates the outputs."""
        torch = self.torch
        dev = lambda a: torch.from_numpy(a).to(self.device).contiguous()
        B, N, H = trees.n_trees, trees.n_nodes, self.H
        out = lambda *s: torch.empty(*s, dtype=torch.float32, device=self.device)
        self.batch = dict(B=B, N=N, tree_off=dev(trees.tree_off), left=dev(trees.left), right=dev(trees.right),
                          word=dev(trees.word), h=out(N, H), c=out(N, H) if self.cell == TL_TREELSTM else None,
                          h_root=out(B, H), c_root=out(B, H) if self.cell == TL_TREELSTM else None,
                          root=torch.empty(B, dtype=torch.int32, device=self.device))
        return self.batch

    def forward(self, stream=None):
        b = self.batch
        tl_forward(self.ctx, b["B"], b["N"], b["tree_off"], b["left"], b["right"], b["word"], b["h"], b["c"],
                   b["h_root"], b["c_root"], b["root"], stream)

    def run(self, trees):
        """load + forward + status check; returns host numpy copies of the outputs."""
        self.load(trees)
        self.forward()
        code = tl_status(self.ctx)
        if code != TL_OK:
            raise TLError(code, "tl_forward (device)")
        b = self.batch
        host = lambda t: None if t is None else t.cpu().numpy()
        return {k: host(b[k]) for k in ("h", "c", "h_root", "c_root", "root")}

    def close(self):
        if self.ctx:
            tl_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
