"""Shared helpers of the GPU parity tests: run one rank's block through the HIP library and
through the CPU oracle on the same seeded inputs and compare tensor by tensor."""
import json
import os

import numpy as np
import torch

from oracle import layer as O
from paper_2504_03662_amd import inputs as I
from paper_2504_03662_amd.runtime import DeviceLayer, to_device, to_host

TOL = {"f32": 1e-4, "bf16": 2e-2}     # max relative error bound per storage type


def rel_errors(got, ref, rows=False):
    """(max|got - ref| / max|ref|, ||got - ref||_2 / ||ref||_2, worst relative L2 error of a row);
    a zero reference demands zeros.  The third figure (rows=True, for [tokens, hidden] activations)
    is the largest ||row of (got - ref)|| / max(||row of ref||, floor) with floor = half the
    root-mean-square row norm, so that a token whose reference vector is almost zero is held to half
    a typical token's absolute error instead of an undefined relative one; otherwise it repeats the
    second figure."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite GPU output"
    scale = np.abs(ref).max()
    if scale == 0.0:
        return (0.0, 0.0, 0.0) if not got.any() else (np.inf, np.inf, np.inf)
    d = got - ref
    el2 = float(np.linalg.norm(d) / np.linalg.norm(ref))
    erow = el2
    if rows and ref.ndim == 2:
        rn = np.sqrt((ref * ref).sum(axis=1))
        dn = np.sqrt((d * d).sum(axis=1))
        erow = float((dn / np.maximum(rn, 0.5 * np.sqrt(np.mean(rn * rn)))).max())
    return float(np.abs(d).max() / scale), el2, erow


_LOG = os.environ.get("GX_PARITY_LOG")


def check(name, got, ref, tol, report=None, rows=None):
    """Bounds per tensor, all at `tol`: the largest error against the largest reference value and
    the relative L2 error of the whole tensor; for activations ([tokens, hidden]: outputs, partial
    sums, input gradients: every tensor not named as a parameter gradient) also the relative L2 error
    of every single token's vector (see rel_errors), so that each token is accurate on its own scale
    and not only the tensor on average; with rows=False that figure is reported but not asserted.  Parameter gradients are sums
    over tokens with heavy cancellation in single rows and columns, whose error scales with the
    terms, not with the sum: they are held to the two whole-tensor bounds."""
    activation = not any(("d" + n) in name for n in I.PARAM_NAMES)
    emax, el2, erow = rel_errors(got, ref, activation)
    if rows is False:                      # reported, not asserted
        report_row, erow = erow, 0.0
    else:
        report_row = erow
    if report is not None:
        report[name] = (emax, el2, report_row)
    if _LOG:
        with open(_LOG, "a") as f:
            f.write(json.dumps(dict(test=os.environ.get("PYTEST_CURRENT_TEST", ""), name=name, shape=list(np.shape(ref)),
                                    emax=emax, el2=el2, erow=report_row, tol=tol)) + "\n")
    assert emax <= tol and el2 <= tol and erow <= tol, \
        f"{name}: max-rel {emax:.3e}, l2-rel {el2:.3e}, worst token l2-rel {erow:.3e} > {tol:g}"


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
