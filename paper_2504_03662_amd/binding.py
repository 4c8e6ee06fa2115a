"""ctypes binding of libgx's C ABI (include/gx.h): argument marshalling only.

Pointers are passed as integers (device addresses) or as any object with ``data_ptr()``; the
stream is a ``hipStream_t`` handle as an integer (0 = default stream).  Every function here has
the name and meaning of the C entry point it wraps; all compute happens in the library.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgx.so")

GX_OK = 0
GX_F32, GX_BF16 = 0, 1
GX_PHASE_ATTN, GX_PHASE_MLP = 1, 2
GX_ROW_BIAS_ATTN, GX_ROW_BIAS_MLP = 4, 8
GX_ACCUM_WGRAD, GX_RECOMPUTE, GX_GELU_TANH, GX_WGRAD_BF16, GX_DROPOUT, GX_FWD_SAVED_ONLY = 16, 32, 64, 128, 256, 512

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
EXPORTS = ("gx_layer_validate", "gx_layer_saved_bytes", "gx_layer_workspace_bytes", "gx_layer_fwd",
           "gx_layer_bwd", "gx_status_str", "gx_version", "gx_prof_enable", "gx_prof_collect", "gx_set_overlap",
           "gx_adamw_step", "gx_params_slice", "gx_params_merge", "gx_plan_search", "gx_strategy_cost", "gx_layer_bwd_static", "gx_peak_mfma", "gx_peak_copy",
           "gx_stage_partition", "gx_stage_moves")
GX_KC_LN_FWD, GX_KC_LN_BWD, GX_KC_ATTN_FWD, GX_KC_ATTN_BWD, GX_KC_COLSUM, GX_KC_GEMM = 1, 2, 3, 4, 5, 100


class LayerCfg(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("hidden", "heads", "ffn", "tp_attn", "tp_ffn", "tp_rank", "seq",
                                               "micro_batch", "dtype", "flags")] + [
        ("ln_eps", ctypes.c_float), ("drop_attn", ctypes.c_int32), ("drop_hidden", ctypes.c_int32),
        ("drop_seed_lo", ctypes.c_uint32), ("drop_seed_hi", ctypes.c_uint32)]


class Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in PARAM_NAMES]


class Grads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in PARAM_NAMES]


class ParamsOut(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in PARAM_NAMES]


class AdamWCfg(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("lr", "beta1", "beta2", "eps", "weight_decay", "grad_scale")] + \
               [("step", ctypes.c_int32)]


class PlanProblem(ctypes.Structure):
    _fields_ = [("layers", ctypes.c_int32), ("strategies", ctypes.c_int32),
                ("time_ms", ctypes.POINTER(ctypes.c_double)), ("mem_bytes", ctypes.POINTER(ctypes.c_double)),
                ("switch_ms", ctypes.POINTER(ctypes.c_double)), ("mem_budget_bytes", ctypes.c_double),
                ("mem_quantum_bytes", ctypes.c_double)]


class PlanResult(ctypes.Structure):
    _fields_ = [("total_ms", ctypes.c_double), ("total_mem_bytes", ctypes.c_double),
                ("pruned", ctypes.c_int64), ("frontier_peak", ctypes.c_int64)]


class StrategyQuery(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("hidden", "heads", "ffn", "seq", "dtype", "gpus", "global_batch",
                                               "tp_attn", "tp_ffn")] + [("link_gbps", ctypes.c_double)]


class StrategyCosts(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("micro_batch_attn", "micro_batch_ffn", "attn_elems", "ffn_elems")] + \
               [(n, ctypes.c_double) for n in ("state_bytes", "tp_comm_ms", "dp_comm_ms", "switch_ms", "flops_attn",
                                               "flops_ffn")]


class GxError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: gx status {self.status} ({status_str(self.status)})")


_lib = None


def lib():
    """Load libgx.so (built by ``python -m paper_2504_03662_amd.build``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not found: build it with `python -m paper_2504_03662_amd.build`")
        # One HIP runtime per process: PyTorch ships its own copy, and the dynamic linker only shares it
        # with libgx when PyTorch's copy is loaded first (its soname then satisfies libgx's dependency);
        # the other order leaves two runtimes on one GPU and libgx's calls fail.  PyTorch supplies the
        # device memory wherever this binding is used, so load it first when it is installed.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        P = ctypes.c_void_p
        L.gx_layer_validate.argtypes = [ctypes.POINTER(LayerCfg)]
        L.gx_layer_validate.restype = ctypes.c_int
        L.gx_layer_saved_bytes.argtypes = [ctypes.POINTER(LayerCfg)]
        L.gx_layer_saved_bytes.restype = ctypes.c_size_t
        L.gx_layer_workspace_bytes.argtypes = [ctypes.POINTER(LayerCfg), ctypes.c_int]
        L.gx_layer_workspace_bytes.restype = ctypes.c_size_t
        L.gx_layer_fwd.argtypes = [ctypes.POINTER(LayerCfg), ctypes.POINTER(Params), P, P, P, P, P, P, P]
        L.gx_layer_fwd.restype = ctypes.c_int
        L.gx_layer_bwd.argtypes = [ctypes.POINTER(LayerCfg), ctypes.POINTER(Params), P, P, P, ctypes.POINTER(Grads),
                                   P, P, P]
        L.gx_layer_bwd.restype = ctypes.c_int
        L.gx_layer_bwd_static.argtypes = [ctypes.POINTER(LayerCfg), ctypes.POINTER(Params), P, P, P,
                                          ctypes.POINTER(Grads), P, P]
        L.gx_layer_bwd_static.restype = ctypes.c_int
        L.gx_status_str.argtypes = [ctypes.c_int]
        L.gx_status_str.restype = ctypes.c_char_p
        L.gx_version.argtypes = []
        L.gx_version.restype = ctypes.c_char_p
        L.gx_set_overlap.argtypes = [ctypes.c_int]
        L.gx_set_overlap.restype = ctypes.c_int
        L.gx_prof_enable.argtypes = [ctypes.c_int]
        L.gx_prof_enable.restype = ctypes.c_int
        L.gx_prof_collect.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float), ctypes.c_int]
        L.gx_prof_collect.restype = ctypes.c_int
        L.gx_adamw_step.argtypes = [ctypes.POINTER(AdamWCfg), ctypes.c_size_t, P, P, P, P, P, ctypes.c_int, P]
        L.gx_adamw_step.restype = ctypes.c_int
        L.gx_params_slice.argtypes = [ctypes.POINTER(LayerCfg), ctypes.POINTER(Params), ctypes.POINTER(ParamsOut), P]
        L.gx_params_slice.restype = ctypes.c_int
        L.gx_params_merge.argtypes = [ctypes.POINTER(LayerCfg), ctypes.POINTER(Params), ctypes.POINTER(ParamsOut), P]
        L.gx_params_merge.restype = ctypes.c_int
        L.gx_plan_search.argtypes = [ctypes.POINTER(PlanProblem), ctypes.POINTER(ctypes.c_int32),
                                     ctypes.POINTER(PlanResult)]
        L.gx_plan_search.restype = ctypes.c_int
        L.gx_peak_mfma.argtypes = [P, ctypes.c_int, ctypes.POINTER(ctypes.c_double), P]
        L.gx_peak_mfma.restype = ctypes.c_int
        L.gx_peak_copy.argtypes = [P, P, ctypes.c_size_t, ctypes.c_int, ctypes.POINTER(ctypes.c_double), P]
        L.gx_peak_copy.restype = ctypes.c_int
        L.gx_strategy_cost.argtypes = [ctypes.POINTER(StrategyQuery), ctypes.POINTER(StrategyCosts)]
        L.gx_strategy_cost.restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def make_cfg(hidden, heads, ffn, tp_attn=1, tp_ffn=1, tp_rank=0, seq=1, micro_batch=1, dtype=GX_F32, flags=3,
             ln_eps=1e-5, drop_attn=0, drop_hidden=0, drop_seed=0):
    """drop_attn / drop_hidden are probabilities in 1/256ths and only read with GX_DROPOUT in flags."""
    return LayerCfg(hidden, heads, ffn, tp_attn, tp_ffn, tp_rank, seq, micro_batch, dtype, flags, ln_eps,
                    drop_attn, drop_hidden, drop_seed & 0xFFFFFFFF, (drop_seed >> 32) & 0xFFFFFFFF)


def _struct(cls, tensors):
    s = cls()
    for n in PARAM_NAMES:
        t = tensors.get(n) if tensors else None
        setattr(s, n, None if t is None else _ptr(t).value)
    return s


def status_str(status):
    return lib().gx_status_str(int(status)).decode()


def version():
    return lib().gx_version().decode()


def layer_validate(cfg):
    return int(lib().gx_layer_validate(ctypes.byref(cfg)))


def layer_saved_bytes(cfg):
    return int(lib().gx_layer_saved_bytes(ctypes.byref(cfg)))


def layer_workspace_bytes(cfg, is_backward):
    return int(lib().gx_layer_workspace_bytes(ctypes.byref(cfg), int(bool(is_backward))))


def layer_fwd(cfg, params, x, y, p_attn, p_mlp, saved, workspace, stream=0, check=True):
    p = _struct(Params, params)
    st = lib().gx_layer_fwd(ctypes.byref(cfg), ctypes.byref(p), _ptr(x), _ptr(y), _ptr(p_attn), _ptr(p_mlp),
                            _ptr(saved), _ptr(workspace), ctypes.c_void_p(stream))
    if check and st != GX_OK:
        raise GxError(st, "gx_layer_fwd")
    return int(st)


def layer_bwd(cfg, params, x, dy, dx, grads, saved, workspace, stream=0, check=True):
    p = _struct(Params, params)
    g = _struct(Grads, grads)
    st = lib().gx_layer_bwd(ctypes.byref(cfg), ctypes.byref(p), _ptr(x), _ptr(dy), _ptr(dx), ctypes.byref(g),
                            _ptr(saved), _ptr(workspace), ctypes.c_void_p(stream))
    if check and st != GX_OK:
        raise GxError(st, "gx_layer_bwd")
    return int(st)


def layer_bwd_static(cfg, params, x, dy, dx, grads, saved, stream=0, check=True):
    p = _struct(Params, params)
    g = _struct(Grads, grads)
    st = lib().gx_layer_bwd_static(ctypes.byref(cfg), ctypes.byref(p), _ptr(x), _ptr(dy), _ptr(dx), ctypes.byref(g),
                                   _ptr(saved), ctypes.c_void_p(stream))
    if check and st != GX_OK:
        raise GxError(st, "gx_layer_bwd_static")
    return int(st)


def prof_enable(on):
    st = lib().gx_prof_enable(int(bool(on)))
    if st != GX_OK:
        raise GxError(st, "gx_prof_enable")


def prof_collect(capacity=8192):
    """Returns [(kernel_class, milliseconds), ...] in launch order and clears the record."""
    cls = (ctypes.c_int * capacity)()
    ms = (ctypes.c_float * capacity)()
    n = lib().gx_prof_collect(cls, ms, capacity)
    if n < 0:
        raise RuntimeError("gx_prof_collect: HIP error")
    return [(int(cls[i]), float(ms[i])) for i in range(n)]


def set_overlap(on):
    st = lib().gx_set_overlap(int(bool(on)))
    if st != GX_OK:
        raise GxError(st, "gx_set_overlap")


def adamw_step(n, master, m, v, grad, param_out=None, param_dtype=GX_BF16, *, step, lr, beta1=0.9, beta2=0.999,
               eps=1e-8, weight_decay=0.0, grad_scale=1.0, stream=0, check=True):
    c = AdamWCfg(lr, beta1, beta2, eps, weight_decay, grad_scale, step)
    st = lib().gx_adamw_step(ctypes.byref(c), int(n), _ptr(master), _ptr(m), _ptr(v), _ptr(grad), _ptr(param_out),
                             int(param_dtype), ctypes.c_void_p(stream))
    if check and st != GX_OK:
        raise GxError(st, "gx_adamw_step")
    return int(st)


def params_slice(cfg, whole, shard, stream=0, check=True):
    w = _struct(Params, whole)
    s = _struct(ParamsOut, shard)
    st = lib().gx_params_slice(ctypes.byref(cfg), ctypes.byref(w), ctypes.byref(s), ctypes.c_void_p(stream))
    if check and st != GX_OK:
        raise GxError(st, "gx_params_slice")
    return int(st)


def params_merge(cfg, shard, whole, stream=0, check=True):
    s = _struct(Params, shard)
    w = _struct(ParamsOut, whole)
    st = lib().gx_params_merge(ctypes.byref(cfg), ctypes.byref(s), ctypes.byref(w), ctypes.c_void_p(stream))
    if check and st != GX_OK:
        raise GxError(st, "gx_params_merge")
    return int(st)


def plan_search(time_ms, mem_bytes, switch_ms=None, *, budget, quantum=0.0, check=True):
    """time_ms, mem_bytes: [layers][strategies] nested sequences; switch_ms: [strategies][strategies] or None.
    Returns (status, choice list, PlanResult)."""
    L, S = len(time_ms), len(time_ms[0])
    flat = lambda a: (ctypes.c_double * (len(a) * len(a[0])))(*[float(x) for row in a for x in row])
    t, m = flat(time_ms), flat(mem_bytes)
    sw = flat(switch_ms) if switch_ms is not None else None
    prob = PlanProblem(L, S, t, m, sw, float(budget), float(quantum))
    choice = (ctypes.c_int32 * L)()
    res = PlanResult()
    st = lib().gx_plan_search(ctypes.byref(prob), choice, ctypes.byref(res))
    if check and st != GX_OK:
        raise GxError(st, "gx_plan_search")
    return int(st), list(choice), res


def strategy_cost(hidden, heads, ffn, seq, dtype, gpus, global_batch, tp_attn, tp_ffn, link_gbps, check=True):
    """Returns (status, StrategyCosts)."""
    q = StrategyQuery(hidden, heads, ffn, seq, dtype, gpus, global_batch, tp_attn, tp_ffn, float(link_gbps))
    out = StrategyCosts()
    st = lib().gx_strategy_cost(ctypes.byref(q), ctypes.byref(out))
    if check and st != GX_OK:
        raise GxError(st, "gx_strategy_cost")
    return int(st), out


def stage_partition(layers, stages, layer_ms=None, check=True):
    """Returns (status, first list of stages + 1 entries, bottleneck_ms)."""
    ms = (ctypes.c_double * layers)(*[float(t) for t in layer_ms]) if layer_ms is not None else None
    first = (ctypes.c_int32 * (max(stages, 0) + 1))()
    bott = ctypes.c_double()
    st = lib().gx_stage_partition(ctypes.c_int32(layers), ctypes.c_int32(stages), ms, first, ctypes.byref(bott))
    if check and st != GX_OK:
        raise GxError(st, "gx_stage_partition")
    return int(st), list(first), bott.value


def stage_moves(layers, old_first, new_first, check=True):
    """Returns (status, new stage of every layer, number of layers whose stage changes)."""
    of = (ctypes.c_int32 * len(old_first))(*old_first)
    nf = (ctypes.c_int32 * len(new_first))(*new_first)
    out = (ctypes.c_int32 * max(layers, 1))()
    moved = ctypes.c_int32()
    st = lib().gx_stage_moves(ctypes.c_int32(layers), ctypes.c_int32(len(old_first) - 1), of,
                              ctypes.c_int32(len(new_first) - 1), nf, out, ctypes.byref(moved))
    if check and st != GX_OK:
        raise GxError(st, "gx_stage_moves")
    return int(st), list(out)[:layers], moved.value


def peak_mfma(scratch, launches=20, stream=0):
    """TFLOP/s of the register-only MFMA loop."""
    out = ctypes.c_double()
    st = lib().gx_peak_mfma(_ptr(scratch), int(launches), ctypes.byref(out), ctypes.c_void_p(stream))
    if st != GX_OK:
        raise GxError(st, "gx_peak_mfma")
    return out.value


def peak_copy(src, dst, nbytes, launches=20, stream=0):
    """GB/s (read + write) of the plain copy."""
    out = ctypes.c_double()
    st = lib().gx_peak_copy(_ptr(src), _ptr(dst), int(nbytes), int(launches), ctypes.byref(out), ctypes.c_void_p(stream))
    if st != GX_OK:
        raise GxError(st, "gx_peak_copy")
    return out.value

