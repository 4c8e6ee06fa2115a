"""Plain fp64 NumPy definition of one rank's share of a pre-LN GPT block, forward and backward.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may call this module; it shares no code with the HIP path and never imports it.

What is computed.  The paper (section 2, "Layer-Specific Parallelism Optimization"; section 3,
"NVIDIA Megatron-LM"; section 5.1) says only *which* matrix products of a transformer layer are
split across GPUs: the attention projections and the feed-forward projections, column-wise for
the first product of each half and row-wise for the second, so that one rank's row-parallel
output is a partial sum.  It prints no layer equations, so the layer itself is the textbook
pre-LayerNorm GPT block written out directly:

    LN(u; g, b)  = g * (u - mean(u)) / sqrt(var(u) + eps) + b       biased variance, per token
    attention    : y1 = LN(x; g1, b1);  [Q|K|V] = y1 @ Wqkv + bqkv
                   per sample and local head: S = Q K^T / sqrt(dh), S_ij = -inf for j > i,
                   P = softmax_j(S), O = P V;  ctx = heads side by side
                   p_attn = ctx @ Wo (+ bo when this rank owns the row-parallel bias)
    feed-forward : y2 = LN(h1; g2, b2);  z = y2 @ W1 + b1;  act = gelu(z)
                   p_mlp = act @ W2 (+ b2 when this rank owns the row-parallel bias)
    gelu(z)      = z * Phi(z),  Phi the standard normal CDF (erf form); a configuration may select
                   the tanh form 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))) instead
    both halves  : h1 = x + p_attn;  y = h1 + p_mlp          (the rank's partial sum stands in
                                                               for the reduced sum; exact at TP=1)
    one half     : returns p_attn (from x) or p_mlp (from h1) alone, no residual, so that a
                   harness can add simulated ranks' partials itself

    dropout      : a variant a configuration may select (drop_attn, drop_hidden in 1/256ths,
                   drop_seed; all 0 = none).  P is replaced by P * keep * 256/(256 - drop_attn)
                   before O = P V; with both halves, h1 = x + drop(p_attn) and y = h1 +
                   drop(p_mlp) with their own masks.  A lone half returns its partial sum
                   undropped (the harness that adds the ranks' partials owns that dropout).
                   Masks come from oracle/dropout.py and are part of the function: the backward
                   pass differentiates with the masks held fixed.

Everything is evaluated with full S x S score matrices and no tiling, blocking or online
softmax, in float64.  The backward pass is the exact gradient of the function above.

Layouts (row-major): activations [T, H] with token t = b*S + s; Wqkv [H, 3*Hl] with columns
[Q heads | K heads | V heads], each head's dh columns contiguous; Wo [Hl, H]; W1 [H, Fl];
W2 [Fl, H]  ("in x out": y = x @ W).  Hl = H / tp_attn, Fl = F / tp_ffn.

Pins (tests/test_oracle_*.py): brute-force loops on tiny layers, finite differences, the
partial-sum / column-concatenation identities of sharding, torch's fp64 CPU layer_norm / gelu /
scaled_dot_product_attention / autograd as library special cases, closed forms (normal-CDF table
values, a hand-computable softmax) and invariants (causality, sample independence, linearity of
the backward pass).  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

from . import dropout as _dropout

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
ATTN_PARAMS = PARAM_NAMES[:6]
MLP_PARAMS = PARAM_NAMES[6:]


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------- pieces

def layer_norm_fwd(u, g, b, eps):
    """Per-token LayerNorm over the last axis: biased variance, eps inside the square root."""
    u = _f64(u)
    mu = u.mean(axis=-1, keepdims=True)
    var = ((u - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (u - mu) * rstd
    return _f64(g) * xhat + _f64(b), xhat, rstd


def layer_norm_bwd(dy, xhat, rstd, g):
    """Gradient of LayerNorm: returns (du, dg, db)."""
    dy = _f64(dy)
    dg = (dy * xhat).sum(axis=0)
    db = dy.sum(axis=0)
    dxhat = dy * _f64(g)
    du = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return du, dg, db


def gelu(z):
    """Exact (erf) GELU: z * Phi(z)."""
    z = _f64(z)
    return 0.5 * z * (1.0 + _erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    """d gelu / dz = Phi(z) + z * phi(z)."""
    z = _f64(z)
    cdf = 0.5 * (1.0 + _erf(z / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)
    return cdf + z * pdf


def gelu_tanh(z):
    """The tanh form of GELU (a variant selected per configuration, `gelu_tanh`):
    0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3)))."""
    z = _f64(z)
    return 0.5 * z * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)))


def gelu_tanh_grad(z):
    """Derivative of gelu_tanh: with u = sqrt(2/pi) (z + 0.044715 z^3) and t = tanh(u),
    0.5 (1 + t) + 0.5 z (1 - t^2) sqrt(2/pi) (1 + 3 * 0.044715 z^2)."""
    z = _f64(z)
    c = np.sqrt(2.0 / np.pi)
    t = np.tanh(c * (z + 0.044715 * z ** 3))
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * c * (1.0 + 3.0 * 0.044715 * z * z)


def _activation(cfg):
    """(function, derivative) of the feed-forward activation the configuration selects."""
    return (gelu_tanh, gelu_tanh_grad) if getattr(cfg, "gelu_tanh", False) else (gelu, gelu_grad)


def causal_attention_fwd(q, k, v, keep=None, keep_scale=1.0):
    """q, k, v: [S, dh] of one sample and head.  Returns (O [S, dh], P [S, S]).  With a keep mask
    [S, S] the probabilities that multiply V are P * keep * keep_scale; the returned P is the
    softmax itself."""
    S, dh = q.shape
    s = (q @ k.T) / np.sqrt(dh)
    masked = np.triu(np.ones((S, S), dtype=bool), k=1)        # j > i
    s = np.where(masked, -np.inf, s)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)                                             # exp(-inf) = 0 exactly
    p = e / e.sum(axis=-1, keepdims=True)
    pd = p if keep is None else p * keep * keep_scale
    return pd @ v, p


def causal_attention_bwd(do, q, k, v, p, keep=None, keep_scale=1.0):
    """Gradient of causal_attention_fwd (same keep mask): returns (dq, dk, dv)."""
    dh = q.shape[1]
    pd = p if keep is None else p * keep * keep_scale
    dv = pd.T @ do
    dp = do @ v.T                                             # gradient w.r.t. the dropped probabilities
    if keep is not None:
        dp = dp * keep * keep_scale
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))      # softmax Jacobian; 0 where p = 0
    dq = (ds @ k) / np.sqrt(dh)
    dk = (ds.T @ q) / np.sqrt(dh)
    return dq, dk, dv


# ----------------------------------------------------------------------------- shapes

class Shape:
    """Derived sizes of one rank's share.  `cfg` is any object with the integer attributes
    hidden, heads, ffn, tp_attn, tp_ffn, seq, micro_batch (and optionally ln_eps)."""

    def __init__(self, cfg):
        self.H = int(cfg.hidden)
        self.nh = int(cfg.heads)
        self.F = int(cfg.ffn)
        self.a = int(cfg.tp_attn)
        self.f = int(cfg.tp_ffn)
        self.S = int(cfg.seq)
        self.B = int(cfg.micro_batch)
        self.eps = float(getattr(cfg, "ln_eps", 1e-5))
        if self.H % self.nh or self.nh % self.a or self.F % self.f:
            raise ValueError("indivisible shape")
        self.rank = int(getattr(cfg, "tp_rank", 0))
        self.drop_attn = int(getattr(cfg, "drop_attn", 0))
        self.drop_hidden = int(getattr(cfg, "drop_hidden", 0))
        self.drop_seed = int(getattr(cfg, "drop_seed", 0))
        self.dh = self.H // self.nh
        self.nl = self.nh // self.a
        self.Hl = self.nl * self.dh
        self.Fl = self.F // self.f
        self.T = self.B * self.S


# ----------------------------------------------------------------------------- halves

def attn_half_fwd(cfg, p, x, row_bias=True):
    """Attention half of one rank: p_attn [T, H] from x [T, H].  Returns (p_attn, cache)."""
    sh = Shape(cfg)
    x = _f64(x)
    y1, xhat1, rstd1 = layer_norm_fwd(x, p["ln1_g"], p["ln1_b"], sh.eps)
    qkv = y1 @ _f64(p["w_qkv"]) + _f64(p["b_qkv"])
    ctx = np.empty((sh.T, sh.Hl))
    probs, keeps = {}, {}
    keep_scale = _dropout.scale_of(sh.drop_attn)
    for b in range(sh.B):
        rows = slice(b * sh.S, (b + 1) * sh.S)
        for h in range(sh.nl):
            cq = slice(h * sh.dh, (h + 1) * sh.dh)
            ck = slice(sh.Hl + h * sh.dh, sh.Hl + (h + 1) * sh.dh)
            cv = slice(2 * sh.Hl + h * sh.dh, 2 * sh.Hl + (h + 1) * sh.dh)
            keep = None
            if sh.drop_attn:
                # the mask belongs to the head of the whole model, whichever rank holds it
                keep = _dropout.keep_attention(sh.drop_seed, sh.drop_attn, sh.S, b,
                                               (sh.rank % sh.a) * sh.nl + h, sh.nh)
            o, pr = causal_attention_fwd(qkv[rows, cq], qkv[rows, ck], qkv[rows, cv], keep, keep_scale)
            ctx[rows, cq] = o
            probs[(b, h)] = pr
            keeps[(b, h)] = keep
    p_attn = ctx @ _f64(p["w_o"])
    if row_bias:
        p_attn = p_attn + _f64(p["b_o"])
    cache = dict(xhat1=xhat1, rstd1=rstd1, y1=y1, qkv=qkv, ctx=ctx, probs=probs, keeps=keeps, keep_scale=keep_scale)
    return p_attn, cache


def attn_half_bwd(cfg, p, dp_attn, cache, row_bias=True):
    """Gradient of attn_half_fwd w.r.t. x (LayerNorm path only) and its parameters."""
    sh = Shape(cfg)
    dp_attn = _f64(dp_attn)
    g = {}
    g["w_o"] = cache["ctx"].T @ dp_attn
    g["b_o"] = dp_attn.sum(axis=0) if row_bias else np.zeros(sh.H)
    dctx = dp_attn @ _f64(p["w_o"]).T
    qkv = cache["qkv"]
    dqkv = np.empty_like(qkv)
    for b in range(sh.B):
        rows = slice(b * sh.S, (b + 1) * sh.S)
        for h in range(sh.nl):
            cq = slice(h * sh.dh, (h + 1) * sh.dh)
            ck = slice(sh.Hl + h * sh.dh, sh.Hl + (h + 1) * sh.dh)
            cv = slice(2 * sh.Hl + h * sh.dh, 2 * sh.Hl + (h + 1) * sh.dh)
            dq, dk, dv = causal_attention_bwd(dctx[rows, cq], qkv[rows, cq], qkv[rows, ck],
                                              qkv[rows, cv], cache["probs"][(b, h)],
                                              cache["keeps"][(b, h)], cache["keep_scale"])
            dqkv[rows, cq] = dq
            dqkv[rows, ck] = dk
            dqkv[rows, cv] = dv
    g["w_qkv"] = cache["y1"].T @ dqkv
    g["b_qkv"] = dqkv.sum(axis=0)
    dy1 = dqkv @ _f64(p["w_qkv"]).T
    dx, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(dy1, cache["xhat1"], cache["rstd1"], p["ln1_g"])
    return dx, g


def mlp_half_fwd(cfg, p, h1, row_bias=True):
    """Feed-forward half of one rank: p_mlp [T, H] from h1 [T, H].  Returns (p_mlp, cache)."""
    sh = Shape(cfg)
    h1 = _f64(h1)
    y2, xhat2, rstd2 = layer_norm_fwd(h1, p["ln2_g"], p["ln2_b"], sh.eps)
    z = y2 @ _f64(p["w_fc1"]) + _f64(p["b_fc1"])
    act = _activation(cfg)[0](z)
    p_mlp = act @ _f64(p["w_fc2"])
    if row_bias:
        p_mlp = p_mlp + _f64(p["b_fc2"])
    cache = dict(xhat2=xhat2, rstd2=rstd2, y2=y2, z=z, act=act)
    return p_mlp, cache


def mlp_half_bwd(cfg, p, dp_mlp, cache, row_bias=True):
    """Gradient of mlp_half_fwd w.r.t. h1 (LayerNorm path only) and its parameters."""
    sh = Shape(cfg)
    dp_mlp = _f64(dp_mlp)
    g = {}
    g["w_fc2"] = cache["act"].T @ dp_mlp
    g["b_fc2"] = dp_mlp.sum(axis=0) if row_bias else np.zeros(sh.H)
    dact = dp_mlp @ _f64(p["w_fc2"]).T
    dz = dact * _activation(cfg)[1](cache["z"])
    g["w_fc1"] = cache["y2"].T @ dz
    g["b_fc1"] = dz.sum(axis=0)
    dy2 = dz @ _f64(p["w_fc1"]).T
    dh1, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(dy2, cache["xhat2"], cache["rstd2"], p["ln2_g"])
    return dh1, g


# ----------------------------------------------------------------------------- whole block

def layer_fwd(cfg, p, x, phase="both", row_bias_attn=True, row_bias_mlp=True):
    """One rank's block forward.

    phase "both": x -> h1 = x + p_attn -> y = h1 + p_mlp; returns dict(y, h1, p_attn, p_mlp, cache).
    phase "attn": returns dict(p_attn, cache) for input x (no residual).
    phase "mlp" : returns dict(p_mlp, cache) for input h1 given as `x` (no residual).
    """
    x = _f64(x)
    if phase == "attn":
        p_attn, ca = attn_half_fwd(cfg, p, x, row_bias_attn)
        return dict(p_attn=p_attn, cache=dict(attn=ca))
    if phase == "mlp":
        p_mlp, cm = mlp_half_fwd(cfg, p, x, row_bias_mlp)
        return dict(p_mlp=p_mlp, cache=dict(mlp=cm))
    if phase != "both":
        raise ValueError(phase)
    sh = Shape(cfg)
    p_attn, ca = attn_half_fwd(cfg, p, x, row_bias_attn)
    m_attn = m_mlp = 1.0
    if sh.drop_hidden:
        hs = _dropout.scale_of(sh.drop_hidden)
        m_attn = hs * _dropout.keep_hidden(sh.drop_seed, sh.drop_hidden, sh.T, sh.H, _dropout.STREAM_ATTN_OUT)
        m_mlp = hs * _dropout.keep_hidden(sh.drop_seed, sh.drop_hidden, sh.T, sh.H, _dropout.STREAM_MLP_OUT)
    h1 = x + p_attn * m_attn
    p_mlp, cm = mlp_half_fwd(cfg, p, h1, row_bias_mlp)
    y = h1 + p_mlp * m_mlp
    return dict(y=y, h1=h1, p_attn=p_attn, p_mlp=p_mlp, cache=dict(attn=ca, mlp=cm, m_attn=m_attn, m_mlp=m_mlp))


def layer_bwd(cfg, p, dy, cache, phase="both", row_bias_attn=True, row_bias_mlp=True):
    """Gradient of layer_fwd for the same phase.  Returns (d_input, grads dict of fp64 arrays).

    Parameters the phase does not touch get no entry in the dict.
    """
    dy = _f64(dy)
    if phase == "attn":
        return attn_half_bwd(cfg, p, dy, cache["attn"], row_bias_attn)
    if phase == "mlp":
        return mlp_half_bwd(cfg, p, dy, cache["mlp"], row_bias_mlp)
    if phase != "both":
        raise ValueError(phase)
    dh1_ln, gm = mlp_half_bwd(cfg, p, dy * cache["m_mlp"], cache["mlp"], row_bias_mlp)
    dh1 = dy + dh1_ln
    dx_ln, ga = attn_half_bwd(cfg, p, dh1 * cache["m_attn"], cache["attn"], row_bias_attn)
    dx = dh1 + dx_ln
    g = dict(ga)
    g.update(gm)
    return dx, g


# ----------------------------------------------------------------------------- stacks

def stack_fwd(cfg, plist, x, **kw):
    """Consecutive blocks, each fed the previous block's output.  Returns (y, [per-block out])."""
    outs = []
    cur = _f64(x)
    for p in plist:
        o = layer_fwd(cfg, p, cur, "both", **kw)
        outs.append(o)
        cur = o["y"]
    return cur, outs


def stack_bwd(cfg, plist, dy, outs, **kw):
    """Backward through the blocks of stack_fwd in reverse.  Returns (dx, [per-block grads])."""
    grads = [None] * len(plist)
    cur = _f64(dy)
    for i in reversed(range(len(plist))):
        cur, grads[i] = layer_bwd(cfg, plist[i], cur, outs[i]["cache"], "both", **kw)
    return cur, grads


def pipeline_stage(cfg, plist, xs, dys, **kw):
    """One pipeline stage's share over several micro-batches (section 2, "Training Phase
    Adaptation": a batch is cut into micro-batches that flow through the stage; section 3's
    manager recombines them).  Outputs per micro-batch are independent; weight gradients are the
    sum over micro-batches taken in index order.  The order in which forward and backward passes
    interleave (1F1B) and activation recomputation do not change any value, so neither appears
    here.  Returns (ys, dxs, [per-block summed grads])."""
    ys, dxs, total = [], [], None
    for x, dy in zip(xs, dys):
        y, outs = stack_fwd(cfg, plist, x, **kw)
        dx, grads = stack_bwd(cfg, plist, dy, outs, **kw)
        ys.append(y)
        dxs.append(dx)
        if total is None:
            total = grads
        else:
            for gt, gn in zip(total, grads):
                for k in gt:
                    gt[k] = gt[k] + gn[k]
    return ys, dxs, total


def model_flops(cfg, blocks=1, micro_batches=1):
    """Model FLOPs of forward + backward (backward = 2 x forward), causal attention counted on
    the S(S+1)/2 unmasked pairs only; used by the benchmark's CPU-baseline leg."""
    sh = Shape(cfg)
    fwd = (2.0 * sh.T * sh.H * 3 * sh.Hl + 2.0 * sh.T * sh.Hl * sh.H
           + 2.0 * sh.T * sh.H * sh.Fl + 2.0 * sh.T * sh.Fl * sh.H
           + 4.0 * sh.B * sh.nl * sh.dh * sh.S * (sh.S + 1) / 2.0)
    return 3.0 * fwd * blocks * micro_batches
