"""Pins for the cost-model oracle: hand counts, arrays actually built, a simulated ring, loops."""
import numpy as np
import pytest

from oracle import cost as C
from oracle import layer as O
from paper_2504_03662_amd import inputs as I


def test_hand_counted_tiny_layer():
    # H 4, 2 heads, F 8, both degrees 2: Hl = 2, Fl = 4
    # attention: gain 4 + bias 4 + Wqkv 4x6 + bqkv 6 + Wo 2x4 + bo 4 = 50
    # feed-forward: 4 + 4 + W1 4x4 + b1 4 + W2 4x4 + b2 4 = 48
    assert C.shard_elems(4, 2, 8, 2, 2) == (50, 48)
    assert C.state_bytes(98, 2) == 98 * 18 and C.state_bytes(98, 4) == 98 * 20
    assert C.micro_batch(16, 8, 2) == 4 and C.micro_batch(16, 8, 8) == 16 and C.micro_batch(8, 8, 1) == 1
    with pytest.raises(ValueError):
        C.micro_batch(1, 8, 2)


@pytest.mark.parametrize("a,f", [(1, 1), (2, 4), (4, 2)])
def test_shard_sizes_equal_the_arrays_the_generator_builds(a, f):
    shape = I.LayerShape(64, 8, 256, a, f, 0, 4, 1, "bf16")
    p = I.rank_params(shape)
    ea, ef = C.shard_elems(64, 8, 256, a, f)
    assert ea == sum(p[n].size for n in I.PARAM_NAMES[:6])
    assert ef == sum(p[n].size for n in I.PARAM_NAMES[6:])


@pytest.mark.parametrize("p", [2, 3, 4, 8])
def test_ring_steps_do_reduce_and_move_what_the_model_charges(p):
    """A ring all-reduce carried out on arrays with exactly the steps the model counts: every rank
    ends with the sum, and each rank has sent (p - 1) + (p - 1) chunks of n / p."""
    rng = np.random.default_rng(p)
    chunk = 5
    data = [rng.integers(-9, 9, (p, chunk)).astype(np.int64) for _ in range(p)]      # rank -> p chunks
    want = sum(data)
    sent = [0] * p
    for step in range(p - 1):                       # reduce-scatter: rank r passes chunk (r - step) on
        moved = [(r, (r - step) % p, data[r][(r - step) % p].copy()) for r in range(p)]
        for r, c, payload in moved:
            data[(r + 1) % p][c] += payload
            sent[r] += payload.size
    for step in range(p - 1):                       # all-gather: rank r passes its finished chunk on
        moved = [(r, (r + 1 - step) % p, data[r][(r + 1 - step) % p].copy()) for r in range(p)]
        for r, c, payload in moved:
            data[(r + 1) % p][c] = payload
            sent[r] += payload.size
    for r in range(p):
        assert np.array_equal(data[r], want)
        assert sent[r] == 2 * (p - 1) * chunk
    n_bytes = p * chunk * 8
    per_rank_bytes = sent[0] * 8
    # the model's time is exactly those bytes over the link rate
    assert C.ring_all_reduce_ms(n_bytes, p, 1.0) == pytest.approx(per_rank_bytes / 1e9 * 1e3, rel=1e-12)


def test_ring_hand_worked_times():
    assert C.ring_all_reduce_ms(1e9, 1, 1.0) == 0.0
    assert C.ring_all_reduce_ms(1e9, 2, 1.0) == pytest.approx(1000.0)        # 2 * (1/2) * 1 s
    assert C.ring_all_reduce_ms(1e9, 4, 1.0) == pytest.approx(1500.0)        # 2 * (3/4) * 1 s
    assert C.ring_all_reduce_ms(33554432, 4, 150.0) == pytest.approx(2 * 0.75 * 33554432 / 150e9 * 1e3)


def test_flops_counted_by_loops_on_a_tiny_layer():
    H, heads, F, S, mb = 8, 2, 12, 5, 2
    dh, T = H // heads, mb * S
    count = 0
    for _ in range(T):                              # QKV: every token, every output column, every input
        count += 2 * (3 * H) * H
    for _b in range(mb):
        for _h in range(heads):
            for i in range(S):
                for _j in range(i + 1):             # visible keys only
                    count += 2 * dh                 # score
                    count += 2 * dh                 # mix
    for _ in range(T):
        count += 2 * H * H                          # output projection
    assert C.half_forward_flops(H, heads, F, S, 1, mb, "attn") == count
    assert C.half_forward_flops(H, heads, F, S, 1, mb, "mlp") == T * (2 * H * F + 2 * F * H)
    # sharded by 2: half the heads, half the columns
    assert C.half_forward_flops(H, heads, F, S, 2, mb, "attn") * 2 == count
    assert C.half_forward_flops(H, heads, F, S, 2, mb, "mlp") * 2 == T * 4 * H * F


def test_flops_agree_with_the_layer_oracles_count():
    shape, _, _ = I.WORKLOADS["C3"]
    c = C.strategy_costs(shape.hidden, shape.heads, shape.ffn, shape.seq, 2, 4, 2, 4, 4, 150.0)
    assert c["micro_batch_attn"] == 2 and c["micro_batch_ffn"] == 2
    assert c["flops_attn"] + c["flops_ffn"] == pytest.approx(O.model_flops(shape), rel=1e-12)


def test_strategy_costs_hand_worked():
    # H 4, 2 heads, F 8, seq 3, bf16, 4 GPUs, global batch 4, strategy (2, 1), link 1 GB/s
    c = C.strategy_costs(4, 2, 8, 3, 2, 4, 4, 2, 1, 1.0)
    # attention degree 2: 2 replicas, micro-batch 2; feed-forward degree 1: 4 replicas, micro-batch 1
    assert (c["micro_batch_attn"], c["micro_batch_ffn"]) == (2, 1)
    # attention shard 50 elements (as above); unsharded feed-forward: 4 + 4 + 32 + 8 + 32 + 4 = 84
    assert (c["attn_elems"], c["ffn_elems"]) == (50, 84)
    assert c["state_bytes"] == 134 * 18
    # tp: attention activations 2 * 3 * 4 * 2 B = 48 B, ring over 2 ranks: 48 B per all-reduce, twice;
    # feed-forward degree 1: none -> 96 B at 1e9 B/s = 9.6e-5 ms
    assert c["tp_comm_ms"] == pytest.approx(96 / 1e9 * 1e3)
    # dp: attention gradients 200 B over 2 ranks -> 200 B; feed-forward 336 B over 4 ranks -> 2 * 3/4 * 336 = 504 B
    assert c["dp_comm_ms"] == pytest.approx((200 + 504) / 1e9 * 1e3)
    # switch: share = 4 * 3 * 4 * 2 / 4 = 24 B, both ways 48 B
    assert c["switch_ms"] == pytest.approx(48 / 1e9 * 1e3)
