"""CPU-only checks of the host-side pieces around the library: seeded inputs, shard slicing, the
pipeline-stage schedule, and the benchmark's FLOP model and argument handling."""
import os
import subprocess
import sys

import numpy as np
import torch

from oracle import layer as O
from paper_2504_03662_amd import inputs as I
from paper_2504_03662_amd.runtime import one_f_one_b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bf16_rounding_is_round_to_nearest_even():
    a = (np.random.default_rng(0).standard_normal(200000) * 7).astype(np.float32)
    a[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]          # exact ties between bf16 neighbours
    r = I.bf16_round(a)
    assert np.array_equal(r, torch.from_numpy(a).to(torch.bfloat16).float().numpy())
    assert np.array_equal(I.bf16_from_bits(I.bf16_bits(r)), r)


def test_inputs_are_seeded_and_rank_specific():
    sh = I.LayerShape(64, 4, 128, 2, 2, 1, 8, 2, "bf16")
    a, b = I.rank_params(sh, case=9), I.rank_params(sh, case=9)
    assert all(np.array_equal(a[n], b[n]) for n in I.PARAM_NAMES)
    c = I.rank_params(sh.with_(tp_rank=0), case=9)
    assert not np.array_equal(a["w_fc1"], c["w_fc1"])
    assert a["w_qkv"].shape == (64, 3 * 32) and a["w_o"].shape == (32, 64)
    assert a["w_fc1"].shape == (64, 64) and a["w_fc2"].shape == (64, 64)
    assert np.all(a["ln1_g"] == 1) and not a["b_fc1"].any()          # graded recipe: gain 1, biases 0
    assert abs(float(a["w_fc1"].std()) - 0.02) < 0.002
    x, dy = I.activations(sh, case=9, micro_batch_index=3)
    assert x.shape == (16, 64) and abs(float(x.std()) - 1.0) < 0.1 and not np.array_equal(x, dy)
    assert np.array_equal(I.bf16_round(x), x)                         # already bf16-representable


def test_shards_tile_the_full_matrices():
    sh = I.LayerShape(32, 4, 64, 2, 4, 0, 4, 1, "f32")
    full = I.full_params(sh.with_(tp_attn=1, tp_ffn=1), case=3, random_affine=True)
    q = [I.shard_params(sh, full, rank_attn=r, rank_ffn=0) for r in range(2)]
    for i in range(3):   # Q, K, V blocks
        cat = np.concatenate([s["w_qkv"][:, i * 16:(i + 1) * 16] for s in q], axis=1)
        assert np.array_equal(cat, full["w_qkv"][:, i * 32:(i + 1) * 32])
    assert np.array_equal(np.concatenate([s["w_o"] for s in q], axis=0), full["w_o"])
    f = [I.shard_params(sh, full, rank_attn=0, rank_ffn=r) for r in range(4)]
    assert np.array_equal(np.concatenate([s["w_fc1"] for s in f], axis=1), full["w_fc1"])
    assert np.array_equal(np.concatenate([s["w_fc2"] for s in f], axis=0), full["w_fc2"])
    assert np.array_equal(np.concatenate([s["b_fc1"] for s in f]), full["b_fc1"])


def test_one_f_one_b_order():
    order = one_f_one_b(8, 3)
    text = " ".join(f"{k}{m}" for k, m in order)
    assert text == "F0 F1 F2 F3 B0 F4 B1 F5 B2 F6 B3 F7 B4 B5 B6 B7"
    for n, d in ((1, 3), (2, 3), (5, 1), (4, 8)):
        o = one_f_one_b(n, d)
        assert sorted(o) == sorted([("F", m) for m in range(n)] + [("B", m) for m in range(n)])
        assert all(o.index(("F", m)) < o.index(("B", m)) for m in range(n))          # forward before its backward
        assert [m for k, m in o if k == "B"] == list(range(n))                        # gradients summed in order


def test_bench_flop_model_and_gpu_count_guard():
    sys.path.insert(0, ROOT)
    import bench
    for name, (shape, blocks, mbs) in I.WORKLOADS.items():
        assert abs(bench.model_flops(shape, blocks, mbs) / O.model_flops(shape, blocks, mbs) - 1) < 1e-12, name
        per_class = bench.gemm_flops_by_class(shape, False)
        gemms = sum(sum(v) for v in per_class.values())
        attn = 3 * 4.0 * shape.micro_batch * shape.local_heads * shape.head_dim * shape.seq * (shape.seq + 1) / 2
        assert abs((gemms + attn) / O.model_flops(shape) - 1) < 1e-12, name
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
