"""Host-side checks of the cost table and plan pipeline (FLOP-model times: no GPU needed)."""
import os

import pytest

from paper_2504_03662_amd import binding as gx
from paper_2504_03662_amd import inputs as I
from paper_2504_03662_amd import profiler as PF


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(gx.LIB_PATH):
        from paper_2504_03662_amd.build import build
        build(verbose=False)
    return gx.lib()


def test_candidate_rules():
    m = PF.Model(4096, 32, 16384, 2048, 4)
    c = PF.candidates(m, 8, 16)
    assert (1, 1) in c and (8, 8) in c and len(c) == 16
    # one sample per step: only degrees that keep a whole sample per replica survive (d = 8)
    assert PF.candidates(m, 8, 1) == [(8, 8)]
    # 6 heads: degree 4 and 8 do not divide them
    assert {a for a, _ in PF.candidates(PF.Model(768, 6, 3072, 128, 2), 8, 8)} == {1, 2}


def test_rows_match_the_graded_shard_shape():
    shape, _, _ = I.WORKLOADS["C3"]                         # TP 4 on both halves, micro-batch 2
    m = PF.Model(shape.hidden, shape.heads, shape.ffn, shape.seq, 1)
    rows = PF.cost_table(m, gpus=4, global_batch=2, measure=False, assumed_tflops=1000.0)
    r = next(r for r in rows if (r["tp_attn"], r["tp_ffn"]) == (4, 4))
    assert r["micro_batch_attn"] == 2 and r["micro_batch_ffn"] == 2
    H, Hl, Fl = shape.hidden, shape.hidden_local, shape.ffn_local
    n = H * 3 * Hl + Hl * H + 2 * H * Fl + 3 * Hl + Fl + 6 * H
    assert r["state_bytes"] == n * 18                       # bf16 weight + fp32 grad, master, two moments
    import bench
    assert abs(r["compute_ms"] * 1e9 * 1000.0 - bench.model_flops(shape, 1, 1)) < 1e-3 * bench.model_flops(shape, 1, 1)
    # saved activations: the two halves' blocks together are the whole layer's minus h1 (kept only with both)
    from paper_2504_03662_amd.runtime import cfg_of
    assert r["saved_bytes"] == gx.layer_saved_bytes(cfg_of(shape)) - shape.tokens * H * 2


def test_plan_pipeline_prefers_a_mix_when_the_budget_sits_between_uniform_plans():
    m = PF.Model(4096, 32, 16384, 2048, 24)
    rows = PF.cost_table(m, gpus=8, global_batch=16, measure=False)
    fastest = min(rows, key=lambda r: r["time_ms"])
    lightest = min(rows, key=lambda r: r["mem_bytes"])
    assert fastest["mem_bytes"] > lightest["mem_bytes"]
    budget = 0.5 * (fastest["mem_bytes"] + lightest["mem_bytes"]) * m.layers
    st, chosen, res = PF.plan(m, rows, 8, 16, budget, quantum_bytes=2 ** 20)
    assert st == gx.GX_OK and len(chosen) == m.layers
    assert res.total_mem_bytes <= budget
    uniform_ok = [r["time_ms"] * m.layers for r in rows if r["mem_bytes"] * m.layers <= budget]
    assert res.total_ms <= min(uniform_ok) + 1e-9
    st2, _, _ = PF.plan(m, rows, 8, 16, 0.5 * lightest["mem_bytes"] * m.layers)
    assert st2 == 9                                          # nothing fits
