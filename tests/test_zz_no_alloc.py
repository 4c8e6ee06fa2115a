"""gx_layer_bwd_static (the backward pass with its workspace in a static device array, for callers
that cannot allocate) against gx_layer_bwd: two calls in a row, the second on a smaller input,
every output bit for bit; then a configuration beyond the array's size is refused."""
import numpy as np
import pytest
import torch

from paper_2504_03662_amd import binding as gx
from paper_2504_03662_amd import inputs as I
from paper_2504_03662_amd.runtime import DeviceLayer, cfg_of, to_device

pytestmark = pytest.mark.gpu
STATIC_BYTES = 64 << 20


def _both_ways(shape, case, recompute=False):
    params = I.rank_params(shape, case=case, random_affine=True)
    x, dy = I.activations(shape, case=case)
    ref = DeviceLayer(shape, params)
    xd, dyd = to_device(x, shape.dtype), to_device(dy, shape.dtype)
    ref.forward(xd)
    dx_ref = ref.backward(xd, dyd, recompute=recompute)
    new = DeviceLayer(shape, params)
    new.forward(xd)
    cfg = cfg_of(shape, recompute=recompute)
    assert gx.layer_workspace_bytes(cfg, True) <= STATIC_BYTES
    dx = new.empty_act()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st = gx.layer_bwd_static(cfg, new.params, xd, dyd, dx, new.grads, None if recompute else new._bufs["saved"],
                             torch.cuda.current_stream().cuda_stream, check=False)
    assert st == gx.GX_OK, gx.status_str(st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(dx.view(torch.int16) if dx.dtype == torch.bfloat16 else dx,
                       dx_ref.view(torch.int16) if dx.dtype == torch.bfloat16 else dx_ref)
    for n in I.PARAM_NAMES:
        assert torch.equal(new.grads[n], ref.grads[n]), n
        assert bool(torch.isfinite(new.grads[n]).all()) and bool(new.grads[n].abs().sum() > 0), n


def test_two_calls_in_a_row_the_second_smaller():
    _both_ways(I.LayerShape(2048, 16, 4096, 2, 2, 1, 1000, 2, "bf16"), case=91)            # close to the 64 MiB limit
    _both_ways(I.LayerShape(512, 8, 1096, 2, 1, 0, 200, 1, "bf16", gelu_tanh=True), case=92, recompute=True)
    _both_ways(I.LayerShape(256, 4, 512, 1, 1, 0, 96, 2, "f32"), case=93)


def test_too_large_a_configuration_is_refused():
    shape, _, _ = I.WORKLOADS["C3"]
    cfg = cfg_of(shape)
    assert gx.layer_workspace_bytes(cfg, True) > STATIC_BYTES
    none = {n: None for n in I.PARAM_NAMES}
    assert gx.layer_bwd_static(cfg, none, None, None, None, none, None, 0, check=False) == 2      # GX_ERR_SHAPE
