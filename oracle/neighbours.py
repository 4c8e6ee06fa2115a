"""Plain fp64 NumPy definitions of two neighbours of the layer step: the optimizer update on fp32
master weights, and the re-partitioning of a block's parameters between tensor-parallel degrees.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may call this module; it shares no code with the HIP path and never imports it.

Optimizer step.  The paper (section 3, "Microsoft DeepSpeed"; section 5.2) relies on partitioned
optimizer states next to the layer compute but prints no update rule, so the rule is the textbook
AdamW (decoupled weight decay, bias-corrected moments), per element and for step number t >= 1:

    g'  = grad_scale * g
    m'  = beta1 * m + (1 - beta1) * g'
    v'  = beta2 * v + (1 - beta2) * g'^2
    w'  = w - lr * ( (m' / (1 - beta1^t)) / (sqrt(v' / (1 - beta2^t)) + eps) + weight_decay * w )

It acts on any flat range of elements, which is what a rank owning a 1/d partition of the states
updates.  The low-precision copy of the parameters handed back to the layer is w' rounded to
bf16 (round to nearest even); that rounding is not done here (fp64 has no business deciding it);
tests round the result with the shared bf16 helper.

Shard transitions.  Section 4 ("Handling Transitions") describes moving between strategies as
cutting a rank's shard out of whole weights, or putting shards back side by side into whole
weights.  With the layouts of this repository (whole Wqkv [H, 3H] with columns [Q | K | V], each
head's dh columns contiguous; Wo [H, H]; W1 [H, F]; W2 [F, H]; "in x out"):

    rank r of a attention ranks owns columns [r*Hl, (r+1)*Hl) of each of the Q, K and V column
    blocks (its heads), and the same index range of the rows of Wo;    Hl = H / a
    rank r of f feed-forward ranks owns columns [r*Fl, (r+1)*Fl) of W1 and b1 and the same rows
    of W2;                                                              Fl = F / f
    LayerNorm parameters and the row-parallel biases bo, b2 are whole on every rank.

slice_params writes one rank's shards element by element from that statement; merge_params is
its inverse (every shard's elements back in place).  Both are pure index movement: exact.

Pins (tests/test_oracle_neighbours.py): torch.optim.AdamW in float64 over several steps as a
library special case, the closed form of the first step from zero moments, pure decay at zero
gradient, scale invariance at eps = 0; for the transitions, the round trip over all ranks, a
per-element index formula on tiny shapes, and the property that the layer oracle fed with the
slices reproduces the unsharded layer (partial sums add up), which no wrong slicing satisfies.
"""
from __future__ import annotations

import numpy as np

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def adamw_step(w, m, v, g, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0):
    """One AdamW update (formula in the module header).  Returns new (w, m, v) as float64 arrays."""
    if step < 1:
        raise ValueError("step numbers start at 1")
    w = np.asarray(w, np.float64)
    m = np.asarray(m, np.float64)
    v = np.asarray(v, np.float64)
    gs = grad_scale * np.asarray(g, np.float64)
    m_new = beta1 * m + (1.0 - beta1) * gs
    v_new = beta2 * v + (1.0 - beta2) * gs * gs
    m_hat = m_new / (1.0 - beta1 ** step)
    v_hat = v_new / (1.0 - beta2 ** step)
    w_new = w - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * w)
    return w_new, m_new, v_new


def _dims(hidden, heads, ffn, tp_attn, tp_ffn):
    if hidden % heads or heads % tp_attn or ffn % tp_ffn:
        raise ValueError("indivisible sharding")
    return hidden // tp_attn, ffn // tp_ffn


def slice_params(full, hidden, heads, ffn, tp_attn, tp_ffn, rank_attn, rank_ffn):
    """One rank's shards of whole parameters (dict of arrays), element by element."""
    H, F = hidden, ffn
    Hl, Fl = _dims(hidden, heads, ffn, tp_attn, tp_ffn)
    out = {n: np.array(full[n], copy=True) for n in ("ln1_g", "ln1_b", "b_o", "ln2_g", "ln2_b", "b_fc2")}
    wq = np.empty((H, 3 * Hl), full["w_qkv"].dtype)
    bq = np.empty((3 * Hl,), full["b_qkv"].dtype)
    for part in range(3):                       # Q, K, V column blocks of the whole matrix
        for c in range(Hl):
            src = part * H + rank_attn * Hl + c
            wq[:, part * Hl + c] = full["w_qkv"][:, src]
            bq[part * Hl + c] = full["b_qkv"][src]
    out["w_qkv"], out["b_qkv"] = wq, bq
    wo = np.empty((Hl, H), full["w_o"].dtype)
    for r in range(Hl):
        wo[r, :] = full["w_o"][rank_attn * Hl + r, :]
    out["w_o"] = wo
    w1 = np.empty((H, Fl), full["w_fc1"].dtype)
    b1 = np.empty((Fl,), full["b_fc1"].dtype)
    for c in range(Fl):
        w1[:, c] = full["w_fc1"][:, rank_ffn * Fl + c]
        b1[c] = full["b_fc1"][rank_ffn * Fl + c]
    out["w_fc1"], out["b_fc1"] = w1, b1
    w2 = np.empty((Fl, H), full["w_fc2"].dtype)
    for r in range(Fl):
        w2[r, :] = full["w_fc2"][rank_ffn * Fl + r, :]
    out["w_fc2"] = w2
    return out


def merge_params(full, shard, hidden, heads, ffn, tp_attn, tp_ffn, rank_attn, rank_ffn, replicated=True):
    """Write one rank's shards back into their place in whole parameters (in place, returns `full`).
    Replicated tensors (LayerNorm parameters, row-parallel biases) are copied whole when asked."""
    H, F = hidden, ffn
    Hl, Fl = _dims(hidden, heads, ffn, tp_attn, tp_ffn)
    if replicated:
        for n in ("ln1_g", "ln1_b", "b_o", "ln2_g", "ln2_b", "b_fc2"):
            full[n][...] = shard[n]
    for part in range(3):
        for c in range(Hl):
            dst = part * H + rank_attn * Hl + c
            full["w_qkv"][:, dst] = shard["w_qkv"][:, part * Hl + c]
            full["b_qkv"][dst] = shard["b_qkv"][part * Hl + c]
    for r in range(Hl):
        full["w_o"][rank_attn * Hl + r, :] = shard["w_o"][r, :]
    for c in range(Fl):
        full["w_fc1"][:, rank_ffn * Fl + c] = shard["w_fc1"][:, c]
        full["b_fc1"][rank_ffn * Fl + c] = shard["b_fc1"][c]
    for r in range(Fl):
        full["w_fc2"][rank_ffn * Fl + r, :] = shard["w_fc2"][r, :]
    return full
