"""The kernels stay inside the buffer sizes the library reports: `saved`, `workspace`, the outputs
and every gradient are allocated at exactly their sizes between pattern-filled guard regions, a
forward and a backward pass run with each combination of variants, and the guards are read back.
Nothing here is meant to fault: a stray write would land in a guard and be seen."""
import numpy as np
import pytest
import torch

from paper_2504_03662_amd import binding as gx
from paper_2504_03662_amd import inputs as I
from paper_2504_03662_amd.runtime import DeviceLayer, to_device, WEIGHT_NAMES

pytestmark = pytest.mark.gpu
GUARD = 1 << 20
PATTERN = 0xA5


class GuardedLayer(DeviceLayer):
    """DeviceLayer whose opaque blocks, outputs and gradients sit between guard regions."""

    def __init__(self, shape, params, wgrad_bf16=False):
        super().__init__(shape, params, wgrad_bf16=wgrad_bf16)
        self.whole = {}
        for n in I.PARAM_NAMES:
            g = self.grads[n]
            view = self._guarded(("grad", n), g.numel() * g.element_size())
            self.grads[n] = view.view(g.dtype).view(g.shape)
            self.grads[n].zero_()

    def _guarded(self, key, nbytes):
        whole = torch.full((2 * GUARD + nbytes,), PATTERN, dtype=torch.uint8, device=self.device)
        self.whole[key] = (whole, nbytes)
        return whole[GUARD:GUARD + nbytes]

    def _buf(self, key, nbytes):
        b = self._bufs.get(key)
        if b is None or b.numel() != nbytes:
            b = self._bufs[key] = self._guarded(key, nbytes)
        return b

    def empty_act(self):
        n = self.shape.tokens * self.shape.hidden
        esz = 2 if self.shape.dtype == "bf16" else 4
        v = self._guarded(("act", len(self.whole)), n * esz)
        return v.view(self.tdtype).view(self.shape.tokens, self.shape.hidden)

    def assert_guards_intact(self):
        torch.cuda.synchronize()
        for key, (whole, nbytes) in self.whole.items():
            lo, hi = whole[:GUARD], whole[GUARD + nbytes:]
            assert bool((lo == PATTERN).all()) and bool((hi == PATTERN).all()), f"guard of {key} ({nbytes} B) was written"


def _run(shape, phase="both", recompute=False, accumulate=False, wgrad_bf16=False, want_partials=False):
    params = I.rank_params(shape, case=71, random_affine=True)
    x, dy = I.activations(shape, case=71)
    layer = GuardedLayer(shape, params, wgrad_bf16=wgrad_bf16)
    xd, dyd = to_device(x, shape.dtype), to_device(dy, shape.dtype)
    out = layer.forward(xd, phase, want_partials=want_partials)
    dx = layer.backward(xd, dyd, phase, accumulate=accumulate, recompute=recompute)
    if accumulate:                                   # a second accumulating pass over the same buffers
        layer.backward(xd, dyd, phase, accumulate=True, recompute=recompute, out=dx)
    layer.assert_guards_intact()
    # the run did write its results (the sizes were not simply too large to matter)
    assert torch.isfinite(dx.float()).all()
    for n in ("w_qkv", "ln1_g") if phase != "mlp" else ("w_fc1", "ln2_g"):
        assert bool(layer.grads[n].float().abs().sum() > 0)
    # saved / workspace were allocated at exactly the queried sizes
    sizes = {k: nb for k, (_, nb) in layer.whole.items() if k in ("saved", "work", "work_fwd")}
    return sizes


ALL = dict(recompute=True, accumulate=True, wgrad_bf16=True)


def test_c3_shape_every_variant():
    shape, _, _ = I.WORKLOADS["C3"]
    _run(shape)
    _run(shape.with_(drop_attn=26, drop_hidden=26, drop_seed=99), want_partials=True, **ALL)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_shapes_every_variant(dtype):
    # nothing is a multiple of a tile: 3 local heads of 64, ragged FFN shard, ragged sequence
    shape = I.LayerShape(384, 6, 1096, 2, 1, 1, 333, 3, dtype, gelu_tanh=True)
    drop = shape.with_(drop_attn=40, drop_hidden=25, drop_seed=7)
    for phase in ("both", "attn", "mlp"):
        _run(shape, phase)
        _run(drop, phase, recompute=True, accumulate=True, wgrad_bf16=(dtype == "bf16"))
    shape128 = I.LayerShape(512, 4, 520, 1, 1, 0, 130, 1, dtype)           # head dim 128, one row past a tile
    _run(shape128)
    _run(shape128.with_(drop_attn=13, drop_seed=3), **dict(ALL, wgrad_bf16=(dtype == "bf16")))
