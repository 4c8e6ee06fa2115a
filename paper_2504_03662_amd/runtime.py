"""Device-buffer plumbing around the binding: torch supplies device memory and the stream, the
library does all the compute.  Used by the GPU tests, the smoke check and the benchmark."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as gx
from .inputs import PARAM_NAMES, LayerShape, bf16_bits, bf16_from_bits

_FLAG_OF_PHASE = {"both": gx.GX_PHASE_ATTN | gx.GX_PHASE_MLP, "attn": gx.GX_PHASE_ATTN, "mlp": gx.GX_PHASE_MLP}


WEIGHT_NAMES = ("w_qkv", "w_o", "w_fc1", "w_fc2")


def cfg_of(shape: LayerShape, phase="both", row_bias_attn=True, row_bias_mlp=True, accumulate=False,
           recompute=False, wgrad_bf16=False, saved_only=False):
    flags = _FLAG_OF_PHASE[phase]
    flags |= gx.GX_ROW_BIAS_ATTN if row_bias_attn else 0
    flags |= gx.GX_ROW_BIAS_MLP if row_bias_mlp else 0
    flags |= gx.GX_ACCUM_WGRAD if accumulate else 0
    flags |= gx.GX_RECOMPUTE if recompute else 0
    flags |= gx.GX_GELU_TANH if shape.gelu_tanh else 0
    flags |= gx.GX_WGRAD_BF16 if wgrad_bf16 else 0
    flags |= gx.GX_DROPOUT if (shape.drop_attn or shape.drop_hidden) else 0
    flags |= gx.GX_FWD_SAVED_ONLY if saved_only else 0
    return gx.make_cfg(shape.hidden, shape.heads, shape.ffn, shape.tp_attn, shape.tp_ffn, shape.tp_rank, shape.seq,
                       shape.micro_batch, gx.GX_BF16 if shape.dtype == "bf16" else gx.GX_F32, flags, shape.ln_eps,
                       shape.drop_attn, shape.drop_hidden, shape.drop_seed)


def to_device(a, dtype, device="cuda:0"):
    """fp32 NumPy array (already holding storage-representable values) -> device tensor."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        t = torch.from_numpy(bf16_bits(a).view(np.int16)).to(device)
        return t.view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host(t):
    """Device tensor (fp32 or bf16) -> fp32 NumPy array, exactly."""
    if t.dtype == torch.bfloat16:
        return bf16_from_bits(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)).reshape(t.shape)
    return t.detach().cpu().numpy()


class DeviceLayer:
    """One rank's share of one block on the GPU: owns parameter, gradient, saved-activation and
    workspace buffers and forwards calls to gx_layer_fwd / gx_layer_bwd."""

    def __init__(self, shape: LayerShape, params, device="cuda:0", wgrad_bf16=False):
        gx.lib()                                   # fail loudly if the library is not built
        self.shape = shape
        self.wgrad_bf16 = wgrad_bf16               # weight-matrix gradients kept in bf16 (GX_WGRAD_BF16)
        self.device = device
        self.tdtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.params = {n: to_device(params[n], shape.dtype, device) for n in PARAM_NAMES}
        self.grads = {n: torch.zeros(self.params[n].shape, device=device,
                                     dtype=torch.bfloat16 if wgrad_bf16 and n in WEIGHT_NAMES else torch.float32)
                      for n in PARAM_NAMES}
        self._bufs = {}

    def _buf(self, key, nbytes):
        b = self._bufs.get(key)
        if b is None or b.numel() < nbytes:
            b = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
            self._bufs[key] = b
        return b

    def empty_act(self):
        return torch.empty((self.shape.tokens, self.shape.hidden), dtype=self.tdtype, device=self.device)

    def forward(self, x, phase="both", row_bias_attn=True, row_bias_mlp=True, want_partials=False, saved_key="saved",
                out=None, saved_only=False, workspace_key="work_fwd"):
        """saved_only: fill only the saved activations the backward pass needs (GX_FWD_SAVED_ONLY)."""
        cfg = cfg_of(self.shape, phase, row_bias_attn, row_bias_mlp, saved_only=saved_only)
        saved = self._buf(saved_key, gx.layer_saved_bytes(cfg))
        y = p_attn = p_mlp = None
        if saved_only:
            pass
        elif phase == "both":
            y = out if out is not None else self.empty_act()
            if want_partials:
                p_attn, p_mlp = self.empty_act(), self.empty_act()
        elif phase == "attn":
            p_attn = out if out is not None else self.empty_act()
        else:
            p_mlp = out if out is not None else self.empty_act()
        nws = gx.layer_workspace_bytes(cfg, False)
        ws = self._buf(workspace_key, nws) if nws else None
        gx.layer_fwd(cfg, self.params, x, y, p_attn, p_mlp, saved, ws, torch.cuda.current_stream().cuda_stream)
        return dict(y=y, p_attn=p_attn, p_mlp=p_mlp)

    def backward(self, x, dy, phase="both", row_bias_attn=True, row_bias_mlp=True, accumulate=False, recompute=False,
                 saved_key="saved", out=None):
        cfg = cfg_of(self.shape, phase, row_bias_attn, row_bias_mlp, accumulate, recompute, self.wgrad_bf16)
        ws = self._buf("work", gx.layer_workspace_bytes(cfg, True))
        saved = None if recompute else self._bufs[saved_key]
        dx = out if out is not None else self.empty_act()
        gx.layer_bwd(cfg, self.params, x, dy, dx, self.grads, saved, ws, torch.cuda.current_stream().cuda_stream)
        return dx


class DeviceStack:
    """Consecutive blocks of one pipeline stage on the GPU.  Each block keeps its own saved
    activations per in-flight micro-batch, or, with recomputation, only its input."""

    def __init__(self, shape: LayerShape, params_list, device="cuda:0", wgrad_bf16=False):
        self.shape = shape
        self.layers = [DeviceLayer(shape, p, device, wgrad_bf16) for p in params_list]
        self.inputs = {}          # micro-batch id -> per-block input tensors

    def forward(self, x, mb=0, keep_saved=True):
        ins = self.inputs.get(mb)
        if ins is None:
            ins = [None] + [self.layers[0].empty_act() for _ in self.layers[1:]] + [self.layers[0].empty_act()]
            self.inputs[mb] = ins
        ins[0] = x
        for k, layer in enumerate(self.layers):
            layer.forward(ins[k], saved_key=("saved", mb) if keep_saved else "saved_scratch", out=ins[k + 1])
        return ins[-1]

    def backward(self, dy, mb=0, recompute=False, accumulate=False, ahead=None):
        """ahead: a stream on which the recomputation of block k-1 runs while block k's backward
        pass runs on the current stream (two scratch blocks of saved activations per stack, shared
        by all layers).  Without it, recomputation happens inside gx_layer_bwd (GX_RECOMPUTE)."""
        ins = self.inputs[mb]
        cur = dy
        if recompute and ahead is not None:
            return self._backward_recompute_ahead(ins, dy, accumulate, ahead)
        for k in reversed(range(len(self.layers))):
            layer = self.layers[k]
            dx = layer._bufs.get(("dx", k % 2))
            if dx is None:
                dx = layer._bufs[("dx", k % 2)] = layer.empty_act()
            cur = layer.backward(ins[k], cur, recompute=recompute, accumulate=accumulate, saved_key=("saved", mb),
                                 out=dx)
        return cur

    def _backward_recompute_ahead(self, ins, dy, accumulate, ahead):
        main = torch.cuda.current_stream()
        if not hasattr(self, "_rc"):
            # scratch saved-activation blocks and forward workspaces are shared by all layers of the
            # stack (same shape): slot k % 2, recycled when block k's backward pass has finished
            self._rc = dict(filled=[torch.cuda.Event() for _ in self.layers],
                            freed=[torch.cuda.Event() for _ in range(2)], bufs={})
        rc = self._rc
        ahead.wait_stream(main)                      # inputs of this micro-batch and earlier uses of the slots
        n = len(self.layers)
        cur = dy
        for k in reversed(range(n)):
            layer, slot = self.layers[k], k % 2
            keys = (("rc", slot), ("rcw", slot))
            with torch.cuda.stream(ahead):
                if k + 2 < n:
                    ahead.wait_event(rc["freed"][slot])
                for key in keys:
                    if key in rc["bufs"]:
                        layer._bufs[key] = rc["bufs"][key]
                layer.forward(ins[k], saved_key=keys[0], saved_only=True, workspace_key=keys[1])
                for key in keys:
                    if key in layer._bufs:
                        rc["bufs"][key] = layer._bufs[key]
                rc["filled"][k].record()
            main.wait_event(rc["filled"][k])
            dx = layer._bufs.get(("dx", k % 2))
            if dx is None:
                dx = layer._bufs[("dx", k % 2)] = layer.empty_act()
            cur = layer.backward(ins[k], cur, recompute=False, accumulate=accumulate, saved_key=("rc", slot), out=dx)
            rc["freed"][slot].record()
        return cur


def one_f_one_b(n_micro, depth_ahead):
    """Order of forward (F, m) and backward (B, m) passes of one pipeline stage that runs
    `depth_ahead` forward passes before its first backward pass, then alternates."""
    order, f, b = [], 0, 0
    while f < min(depth_ahead, n_micro):
        order.append(("F", f))
        f += 1
    while b < n_micro:
        if f < n_micro:
            order.append(("F", f))
            f += 1
        order.append(("B", b))
        b += 1
    return order


class StageSchedule:
    """Issues one pipeline stage's passes in a given order (e.g. one_f_one_b) on two streams:
    forward passes on one, backward passes on the other, each backward pass ordered after the
    forward pass of its own micro-batch.  A forward pass of a later micro-batch is independent of
    the backward pass issued next to it (different activations, read-only weights), so the two
    fill each other's idle compute units; weight gradients are still accumulated in the order of
    the backward passes.  With recomputation, a third stream recomputes block k-1's activations
    while block k's backward pass runs.  With `overlap=False` everything is issued on the current
    stream and recomputation happens inside gx_layer_bwd."""

    def __init__(self, stack: DeviceStack, n_micro, overlap=True):
        self.stack = stack
        self.overlap = overlap
        if overlap:
            self.fwd_stream, self.bwd_stream, self.ahead_stream = (torch.cuda.Stream() for _ in range(3))
            self.done = [torch.cuda.Event() for _ in range(n_micro)]

    def run(self, order, xs, dys, recompute, after_forward=None, after_backward=None):
        """xs / dys: device tensors per micro-batch.  The optional hooks run right after a pass
        has been issued, with that pass's stream current (so a host copy made there waits for it)."""
        cur = torch.cuda.current_stream()
        if self.overlap:
            self.fwd_stream.wait_stream(cur)
            self.bwd_stream.wait_stream(cur)
        seen = False
        for kind, m in order:
            if kind == "F":
                with torch.cuda.stream(self.fwd_stream if self.overlap else cur):
                    y = self.stack.forward(xs[m], mb=m, keep_saved=not recompute)
                    if self.overlap:
                        self.done[m].record()
                    if after_forward:
                        after_forward(m, y)
            else:
                with torch.cuda.stream(self.bwd_stream if self.overlap else cur):
                    if self.overlap:
                        torch.cuda.current_stream().wait_event(self.done[m])
                    dx = self.stack.backward(dys[m], mb=m, recompute=recompute, accumulate=seen,
                                             ahead=self.ahead_stream if self.overlap else None)
                    seen = True
                    if after_backward:
                        after_backward(m, dx)
        if self.overlap:
            cur.wait_stream(self.fwd_stream)
            cur.wait_stream(self.bwd_stream)
