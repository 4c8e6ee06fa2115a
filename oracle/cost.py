"""Plain definition of the per-layer cost model that fills the strategy cost table beside the
measured compute times.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests may call this module; it shares no code with the
library's cost model and never imports it.

The paper's model profiler (section 3, "Model Profiler") records parameter counts and per-layer
memory, and its strategy selector (section 3, "Dynamic Strategy Selector") weighs communication
overhead against compute; no formula is printed.  The reading taken here, also stated in the
library's header, is the textbook one, each quantity written as the sum of its parts:

  strategy      (tp_attn, tp_ffn) on a group of `gpus` devices, the rest of the group data parallel:
                a half of degree d is replicated gpus / d times and each replica's tensor-parallel
                group runs micro-batches of global_batch / (gpus / d) samples.
  shard sizes   one rank's parameters, tensor by tensor (shapes as the layer oracle takes them).
  state bytes   per parameter element: the stored parameter (e bytes), an fp32 gradient, an fp32
                master copy and two fp32 optimizer moments (4 x 4 bytes).
  ring          all-reduce of n bytes over p ranks as p - 1 reduce-scatter steps followed by
                p - 1 all-gather steps, each moving one chunk of n / p bytes over every link at
                the same time; the time is the steps' sum at link_gbps * 1e9 bytes per second.
  tp comm       per half: one all-reduce of its [micro_batch * seq, hidden] activations in the
                forward pass (after the row-parallel product) and one in the backward pass (after
                the column-parallel input gradient), over its tensor-parallel group.
  dp comm       per half: one all-reduce of its fp32 gradients over its data-parallel group.
  switch        every GPU moves its 1 / gpus share of the step's [global_batch * seq, hidden]
                activations once in the forward and once in the backward pass.
  flops         forward multiply-adds counted product by product (2 per multiply-add), causal
                attention on the visible (query, key) pairs only; backward = twice the forward.

Pins (tests/test_oracle_cost.py): a hand-counted tiny layer, the sizes of arrays actually built by
the input generator, a step-by-step simulation of a ring all-reduce on arrays (result and bytes
sent per rank), hand-worked ring times, multiply-adds counted by loops on tiny sizes, and the
layer oracle's own FLOP count.
"""
from __future__ import annotations


def micro_batch(global_batch, gpus, degree):
    replicas = gpus // degree
    if gpus % degree or global_batch % replicas:
        raise ValueError("the group or the batch does not divide")
    return global_batch // replicas


def shard_shapes(hidden, heads, ffn, tp_attn, tp_ffn):
    """{tensor: shape} of one rank's parameters, per half."""
    H = hidden
    Hl = (heads // tp_attn) * (H // heads)
    Fl = ffn // tp_ffn
    attn = dict(ln1_g=(H,), ln1_b=(H,), w_qkv=(H, 3 * Hl), b_qkv=(3 * Hl,), w_o=(Hl, H), b_o=(H,))
    mlp = dict(ln2_g=(H,), ln2_b=(H,), w_fc1=(H, Fl), b_fc1=(Fl,), w_fc2=(Fl, H), b_fc2=(H,))
    return attn, mlp


def _count(shapes):
    total = 0
    for shape in shapes.values():
        n = 1
        for d in shape:
            n *= d
        total += n
    return total


def shard_elems(hidden, heads, ffn, tp_attn, tp_ffn):
    attn, mlp = shard_shapes(hidden, heads, ffn, tp_attn, tp_ffn)
    return _count(attn), _count(mlp)


def state_bytes(elems, elem_bytes):
    parameter, gradient, master, moment1, moment2 = elem_bytes, 4, 4, 4, 4
    return elems * (parameter + gradient + master + moment1 + moment2)


def ring_all_reduce_ms(nbytes, ranks, link_gbps):
    if ranks <= 1:
        return 0.0
    chunk = nbytes / ranks
    seconds = 0.0
    for _ in range(ranks - 1):          # reduce-scatter
        seconds += chunk / (link_gbps * 1e9)
    for _ in range(ranks - 1):          # all-gather
        seconds += chunk / (link_gbps * 1e9)
    return seconds * 1e3


def half_forward_flops(hidden, heads, ffn, seq, degree, mb, phase):
    """Forward FLOPs of one half on one rank, product by product."""
    T, H, S = mb * seq, hidden, seq
    if phase == "attn":
        nl, dh = heads // degree, H // heads
        Hl = nl * dh
        qkv = 2 * T * H * (3 * Hl)
        visible_pairs = S * (S + 1) // 2
        scores = 2 * mb * nl * visible_pairs * dh          # Q K^T on visible pairs
        mix = 2 * mb * nl * visible_pairs * dh             # P V on visible pairs
        out = 2 * T * Hl * H
        return qkv + scores + mix + out
    Fl = ffn // degree
    return 2 * T * H * Fl + 2 * T * Fl * H


def strategy_costs(hidden, heads, ffn, seq, elem_bytes, gpus, global_batch, tp_attn, tp_ffn, link_gbps):
    mba = micro_batch(global_batch, gpus, tp_attn)
    mbf = micro_batch(global_batch, gpus, tp_ffn)
    ea, ef = shard_elems(hidden, heads, ffn, tp_attn, tp_ffn)
    act_a = mba * seq * hidden * elem_bytes
    act_f = mbf * seq * hidden * elem_bytes
    tp = (ring_all_reduce_ms(act_a, tp_attn, link_gbps) * 2 + ring_all_reduce_ms(act_f, tp_ffn, link_gbps) * 2)
    dp = (ring_all_reduce_ms(ea * 4, gpus // tp_attn, link_gbps) + ring_all_reduce_ms(ef * 4, gpus // tp_ffn, link_gbps))
    share = global_batch * seq * hidden * elem_bytes / gpus
    switch = (share + share) / (link_gbps * 1e9) * 1e3
    return dict(micro_batch_attn=mba, micro_batch_ffn=mbf, attn_elems=ea, ffn_elems=ef,
                state_bytes=state_bytes(ea + ef, elem_bytes), tp_comm_ms=tp, dp_comm_ms=dp, switch_ms=switch,
                flops_attn=3 * half_forward_flops(hidden, heads, ffn, seq, tp_attn, mba, "attn"),
                flops_ffn=3 * half_forward_flops(hidden, heads, ffn, seq, tp_ffn, mbf, "mlp"))
