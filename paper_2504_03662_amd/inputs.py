"""Seeded synthetic inputs for one rank's share of a transformer block.

This module only draws random numbers, rounds them to the storage type and cuts shards out of
full matrices; it contains none of the layer's arithmetic and is the one piece shared by the
tests' CPU checker and the GPU path.

Recipe: every tensor is drawn in fp32 from
``numpy.random.default_rng([SEED, case, block, tensor_id, rank, micro_batch])``; weights are
N(0, 0.02^2), LayerNorm gains 1 and all biases 0 (or, with ``random_affine=True``, gains
1 + 0.1 N(0,1) and biases 0.1 N(0,1) so that those code paths are exercised); activations and
upstream gradients are N(0, 1).  For bf16 cases every value is then rounded to the nearest-even
bf16, so that both sides start from bit-identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

SEED = 20250403

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
_TENSOR_ID = {n: i for i, n in enumerate(PARAM_NAMES)}
_TENSOR_ID.update(x=100, dy=101)


@dataclass(frozen=True)
class LayerShape:
    """Sizes of one rank's share: the fields the library's configuration record carries."""
    hidden: int
    heads: int
    ffn: int
    tp_attn: int = 1
    tp_ffn: int = 1
    tp_rank: int = 0
    seq: int = 128
    micro_batch: int = 1
    dtype: str = "f32"          # "f32" or "bf16"
    ln_eps: float = 1e-5
    gelu_tanh: bool = False     # tanh form of GELU instead of the erf form
    drop_attn: int = 0          # dropout of attention probabilities, probability in 1/256ths (0 = none)
    drop_hidden: int = 0        # dropout of each half's output before the residual, in 1/256ths
    drop_seed: int = 0          # 64-bit seed of the dropout masks

    @property
    def head_dim(self):
        return self.hidden // self.heads

    @property
    def local_heads(self):
        return self.heads // self.tp_attn

    @property
    def hidden_local(self):
        return self.local_heads * self.head_dim

    @property
    def ffn_local(self):
        return self.ffn // self.tp_ffn

    @property
    def tokens(self):
        return self.seq * self.micro_batch

    def with_(self, **kw):
        return replace(self, **kw)


# The five graded workloads (shape, blocks, micro-batches).
WORKLOADS = {
    "C1": (LayerShape(256, 4, 1024, 1, 1, 0, 128, 2, "f32"), 1, 1),
    "C2": (LayerShape(2048, 16, 8192, 1, 1, 0, 2048, 4, "bf16"), 4, 1),
    "C3": (LayerShape(4096, 32, 16384, 4, 4, 0, 2048, 2, "bf16"), 1, 1),
    "C4": (LayerShape(8192, 64, 28672, 8, 1, 0, 4096, 1, "bf16"), 1, 1),
    "C5": (LayerShape(5120, 40, 20480, 2, 2, 0, 2048, 1, "bf16"), 8, 8),
}


def bf16_round(a):
    """Round fp32 values to the nearest-even bf16 and return them as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000))
    return r.view(np.float32)


def bf16_bits(a):
    """fp32 array holding bf16-representable values -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b):
    """uint16 bf16 bit patterns -> fp32 values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(case, block, tensor, rank, mb):
    return np.random.default_rng([SEED, int(case), int(block), _TENSOR_ID[tensor], int(rank), int(mb)])


def _store(a, dtype):
    a = a.astype(np.float32)
    return bf16_round(a) if dtype == "bf16" else a


def full_params(shape, case=0, block=0, random_affine=False):
    """Unsharded parameters of one block as fp32 arrays (already rounded for bf16 cases)."""
    H, F = shape.hidden, shape.ffn
    dims = dict(ln1_g=(H,), ln1_b=(H,), w_qkv=(H, 3 * H), b_qkv=(3 * H,), w_o=(H, H), b_o=(H,),
                ln2_g=(H,), ln2_b=(H,), w_fc1=(H, F), b_fc1=(F,), w_fc2=(F, H), b_fc2=(H,))
    p = {}
    for n in PARAM_NAMES:
        g = _rng(case, block, n, 10_000, 0)
        if n.startswith("w_"):
            v = 0.02 * g.standard_normal(dims[n], dtype=np.float32)
        elif n.endswith("_g") and n.startswith("ln"):
            v = 1.0 + (0.1 * g.standard_normal(dims[n], dtype=np.float32) if random_affine else 0.0)
            v = np.broadcast_to(np.float32(v), dims[n]).copy()
        else:
            v = (0.1 * g.standard_normal(dims[n], dtype=np.float32) if random_affine
                 else np.zeros(dims[n], np.float32))
        p[n] = _store(v, shape.dtype)
    return p


def shard_params(shape, full, rank_attn=None, rank_ffn=None):
    """Cut one rank's shards out of unsharded parameters.

    Column shards take columns [r*Hl, (r+1)*Hl) of each of the Q, K and V blocks of w_qkv (and
    [r*Fl, (r+1)*Fl) of w_fc1); row shards take the same index range of the rows of w_o / w_fc2.
    LayerNorm parameters and the row-parallel biases are replicated.
    """
    ra = shape.tp_rank if rank_attn is None else rank_attn
    rf = (shape.tp_rank % shape.tp_ffn) if rank_ffn is None else rank_ffn
    H, Hl, Fl = shape.hidden, shape.hidden_local, shape.ffn_local
    ca = slice(ra * Hl, (ra + 1) * Hl)
    cf = slice(rf * Fl, (rf + 1) * Fl)
    p = dict(full)
    wq = full["w_qkv"]
    bq = full["b_qkv"]
    p["w_qkv"] = np.ascontiguousarray(np.concatenate([wq[:, ca], wq[:, H:2 * H][:, ca], wq[:, 2 * H:][:, ca]], axis=1))
    p["b_qkv"] = np.ascontiguousarray(np.concatenate([bq[ca], bq[H:2 * H][ca], bq[2 * H:][ca]]))
    p["w_o"] = np.ascontiguousarray(full["w_o"][ca, :])
    p["w_fc1"] = np.ascontiguousarray(full["w_fc1"][:, cf])
    p["b_fc1"] = np.ascontiguousarray(full["b_fc1"][cf])
    p["w_fc2"] = np.ascontiguousarray(full["w_fc2"][cf, :])
    return p


def rank_params(shape, case=0, block=0, random_affine=False):
    """One rank's shards drawn directly at their sharded sizes (no full matrix is formed)."""
    H, Hl, Fl = shape.hidden, shape.hidden_local, shape.ffn_local
    dims = dict(ln1_g=(H,), ln1_b=(H,), w_qkv=(H, 3 * Hl), b_qkv=(3 * Hl,), w_o=(Hl, H), b_o=(H,),
                ln2_g=(H,), ln2_b=(H,), w_fc1=(H, Fl), b_fc1=(Fl,), w_fc2=(Fl, H), b_fc2=(H,))
    p = {}
    for n in PARAM_NAMES:
        g = _rng(case, block, n, shape.tp_rank, 0)
        if n.startswith("w_"):
            v = 0.02 * g.standard_normal(dims[n], dtype=np.float32)
        elif n.endswith("_g"):
            v = np.ones(dims[n], np.float32)
            if random_affine:
                v = v + 0.1 * g.standard_normal(dims[n], dtype=np.float32)
        else:
            v = (0.1 * g.standard_normal(dims[n], dtype=np.float32) if random_affine
                 else np.zeros(dims[n], np.float32))
        p[n] = _store(v, shape.dtype)
    return p


def activations(shape, case=0, micro_batch_index=0):
    """(x, dy): input activations and upstream gradient, [T, H] each."""
    T, H = shape.tokens, shape.hidden
    x = _rng(case, 0, "x", shape.tp_rank, micro_batch_index).standard_normal((T, H), dtype=np.float32)
    dy = _rng(case, 0, "dy", shape.tp_rank, micro_batch_index).standard_normal((T, H), dtype=np.float32)
    return _store(x, shape.dtype), _store(dy, shape.dtype)
