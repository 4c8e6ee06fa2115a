"""Shared helpers of the GPU parity tests: run one rank's block through the HIP library and
through the CPU oracle on the same seeded inputs and compare tensor by tensor."""
import numpy as np
import torch

from oracle import layer as O
from paper_2504_03662_amd import inputs as I
from paper_2504_03662_amd.runtime import DeviceLayer, to_device, to_host

TOL = {"f32": 1e-4, "bf16": 2e-2}     # max relative error bound per storage type


def rel_errors(got, ref):
    """(max|got - ref| / max|ref|, ||got - ref||_2 / ||ref||_2, max_i |got_i - ref_i| / (|ref_i| + 2 rms(ref)));
    a zero reference demands zeros."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite GPU output"
    scale = np.abs(ref).max()
    if scale == 0.0:
        return (0.0, 0.0, 0.0) if not got.any() else (np.inf, np.inf, np.inf)
    d = np.abs(got - ref)
    rms = np.sqrt(np.mean(ref * ref))
    return (float(d.max() / scale), float(np.linalg.norm(d) / np.linalg.norm(ref)),
            float((d / (np.abs(ref) + 2.0 * rms)).max()))


def check(name, got, ref, tol, report=None):
    """Three bounds per tensor, all at `tol`: the largest error against the largest reference value,
    the relative L2 error, and an element-wise mixed bound |error_i| <= tol * (|ref_i| + 2 rms(ref)),
    which holds a typical element (|ref_i| about one rms) to 3 tol of its own size instead of the
    ~5 tol the global maximum allows."""
    emax, el2, emix = rel_errors(got, ref)
    if report is not None:
        report[name] = (emax, el2, emix)
    assert emax <= tol and el2 <= tol and emix <= tol, \
        f"{name}: max-rel {emax:.3e}, l2-rel {el2:.3e}, element-wise mixed {emix:.3e} > {tol:g}"


def run_both(shape, params, x, dy, phase="both", rb_attn=True, rb_mlp=True, recompute=False, want_partials=False):
    """Returns (gpu dict, oracle dict) with y / p_attn / p_mlp, dx and grads as fp64/fp32 arrays."""
    layer = DeviceLayer(shape, params)
    xd, dyd = to_device(x, shape.dtype), to_device(dy, shape.dtype)
    out = layer.forward(xd, phase, rb_attn, rb_mlp, want_partials=want_partials)
    dxd = layer.backward(xd, dyd, phase, rb_attn, rb_mlp, recompute=recompute)
    torch.cuda.synchronize()
    gpu = {k: to_host(v) for k, v in out.items() if v is not None}
    gpu["dx"] = to_host(dxd)
    gpu["grads"] = {n: to_host(layer.grads[n]) for n in I.PARAM_NAMES}
    ref_out = O.layer_fwd(shape, params, x, phase, rb_attn, rb_mlp)
    dx, g = O.layer_bwd(shape, params, dy, ref_out["cache"], phase, rb_attn, rb_mlp)
    ref = {k: ref_out[k] for k in ("y", "p_attn", "p_mlp") if k in ref_out}
    ref["dx"] = dx
    ref["grads"] = g
    return gpu, ref, layer


def compare(gpu, ref, tol, phase="both", want_partials=False, report=None):
    keys = {"both": ["y"] + (["p_attn", "p_mlp"] if want_partials else []), "attn": ["p_attn"], "mlp": ["p_mlp"]}[phase]
    for k in keys:
        check(k, gpu[k], ref[k], tol, report)
    check("dx", gpu["dx"], ref["dx"], tol, report)
    for n, g in ref["grads"].items():
        check("d" + n, gpu["grads"][n], g, tol, report)
