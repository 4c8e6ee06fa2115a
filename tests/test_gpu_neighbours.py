"""GPU parity of the layer step's neighbours against the CPU oracle, through the C ABI:
the AdamW update (fp32 arithmetic against the fp64 definition, tolerance 1e-4 of each tensor's
largest value like every fp32 path here; the bf16 copy must be the exact round-to-nearest-even of
the fp32 result) and the shard transitions (pure data movement: bit-exact)."""
import numpy as np
import pytest
import torch

from oracle import neighbours as N
from paper_2504_03662_amd import binding as gx
from paper_2504_03662_amd import inputs as I
from paper_2504_03662_amd.runtime import to_device, to_host
from parity import TOL, check

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def _adam_inputs(n, seed):
    rng = np.random.default_rng([I.SEED, 700, seed])
    w = (0.02 * rng.standard_normal(n)).astype(np.float32)
    m = (1e-3 * rng.standard_normal(n)).astype(np.float32)
    v = ((1e-3 * rng.standard_normal(n)) ** 2 + 1e-8).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32) * np.float32(1e-2)
    return w, m, v, g


@pytest.mark.parametrize("n", [1, 3, 4, 1023, 1_000_003])
@pytest.mark.parametrize("out", [None, gx.GX_BF16, gx.GX_F32])
def test_adamw_matches_oracle_over_steps(n, out):
    hp = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, grad_scale=0.125)
    w, m, v, _ = _adam_inputs(n, 1)
    wd, md, vd = _dev32(w), _dev32(m), _dev32(v)
    po = None if out is None else torch.empty(n, dtype=torch.bfloat16 if out == gx.GX_BF16 else torch.float32, device=DEV)
    rw, rm, rv = w.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    for step in (1, 2, 3):
        g = _adam_inputs(n, 10 + step)[3]
        gd = _dev32(g)
        gx.adamw_step(n, wd, md, vd, gd, po, out if out is not None else gx.GX_BF16, step=step,
                      stream=torch.cuda.current_stream().cuda_stream, **hp)
        torch.cuda.synchronize()
        rw, rm, rv = N.adamw_step(rw, rm, rv, g, step, **hp)
        check("w", wd.cpu().numpy(), rw, TOL["f32"])
        check("m", md.cpu().numpy(), rm, TOL["f32"])
        check("v", vd.cpu().numpy(), rv, TOL["f32"])
        # elementwise bound as well (the tensors have no large outliers to hide behind)
        assert np.all(np.abs(wd.cpu().numpy() - rw) <= 1e-5 * np.abs(rw) + 1e-7)
        if out == gx.GX_BF16:
            got = po.view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(got, I.bf16_bits(I.bf16_round(wd.cpu().numpy())))      # exact RNE of the fp32 result
            check("param", I.bf16_from_bits(got), rw, TOL["bf16"])
        elif out == gx.GX_F32:
            assert np.array_equal(po.cpu().numpy(), wd.cpu().numpy())


def test_adamw_full_size_shard_sampled():
    """One rank's parameters of the TP-shard workload (50.3 M elements), one step; sampled elements
    against the oracle (the update is elementwise, so a sample is computed one by one)."""
    shape, _, _ = I.WORKLOADS["C3"]
    H, Hl, Fl = shape.hidden, shape.hidden_local, shape.ffn_local
    n = H * 3 * Hl + Hl * H + 2 * H * Fl + 3 * Hl + Fl + 6 * H
    gen = torch.Generator(device=DEV).manual_seed(I.SEED)
    wd = 0.02 * torch.randn(n, device=DEV, generator=gen)
    md = 1e-3 * torch.randn(n, device=DEV, generator=gen)
    vd = (1e-2 * torch.randn(n, device=DEV, generator=gen)) ** 2
    gd = 1e-2 * torch.randn(n, device=DEV, generator=gen)
    idx = torch.from_numpy(np.random.default_rng(4).integers(0, n, 20000)).to(DEV)
    idx[:4] = torch.tensor([0, 1, n - 2, n - 1], device=DEV)
    before = [t[idx].cpu().numpy().astype(np.float64) for t in (wd, md, vd, gd)]
    po = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    gx.adamw_step(n, wd, md, vd, gd, po, gx.GX_BF16, step=7, stream=torch.cuda.current_stream().cuda_stream, **hp)
    torch.cuda.synchronize()
    rw, rm, rv = N.adamw_step(*before, 7, **hp)
    check("w", wd[idx].cpu().numpy(), rw, TOL["f32"])
    check("m", md[idx].cpu().numpy(), rm, TOL["f32"])
    check("v", vd[idx].cpu().numpy(), rv, TOL["f32"])
    assert torch.equal(po, wd.to(torch.bfloat16))            # same rounding rule everywhere, every element
    assert torch.isfinite(wd).all()


def _whole(shape, dtype, case):
    full = I.full_params(shape.with_(tp_attn=1, tp_ffn=1, dtype=dtype), case=case, random_affine=True)
    return {k: np.ascontiguousarray(v) for k, v in full.items()}


def _empty_like(arrs, dtype):
    return {k: torch.empty(v.shape, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=DEV)
            for k, v in arrs.items()}


def _bits(t):
    return to_host(t).astype(np.float32).view(np.uint32)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("a,f,rank", [(1, 1, 0), (2, 2, 1), (4, 2, 3), (2, 4, 3)])
@pytest.mark.parametrize("phase", ["both", "attn", "mlp"])
def test_slice_and_merge_bit_exact(dtype, a, f, rank, phase):
    # H / a and F / f stay multiples of 8 elements (16 bytes of bf16); the pieces are ragged against the 32 KB blocks
    shape = I.LayerShape(256, 8, 704, a, f, rank, 8, 1, dtype)
    whole = _whole(shape, dtype, 40 + a)
    flags = {"both": 3, "attn": gx.GX_PHASE_ATTN, "mlp": gx.GX_PHASE_MLP}[phase]
    cfg = gx.make_cfg(256, 8, 704, a, f, rank, 8, 1, gx.GX_BF16 if dtype == "bf16" else gx.GX_F32, flags)
    ref = N.slice_params(whole, 256, 8, 704, a, f, rank % a, rank % f)
    wd = {k: to_device(v, dtype) for k, v in whole.items()}
    sd = _empty_like(ref, dtype)
    for t in sd.values():
        t.fill_(float("nan"))
    st = torch.cuda.current_stream().cuda_stream
    gx.params_slice(cfg, wd, sd, stream=st)
    torch.cuda.synchronize()
    mine = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o") if phase == "attn" else \
           ("ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2") if phase == "mlp" else I.PARAM_NAMES
    for k in I.PARAM_NAMES:
        got = to_host(sd[k])
        if k in mine:
            assert np.array_equal(got.astype(np.float32).view(np.uint32),
                                  np.asarray(ref[k], np.float32).view(np.uint32)), k
        else:
            assert np.isnan(got).all(), k                       # the other half is not touched
    # merge into a NaN-filled whole: exactly this rank's elements appear, everything else stays NaN
    blank = {k: np.full(v.shape, np.nan, np.float32) for k, v in whole.items()}
    expect = N.merge_params({k: v.copy() for k, v in blank.items()}, {k: np.asarray(v, np.float32) for k, v in ref.items()},
                            256, 8, 704, a, f, rank % a, rank % f)
    bd = {k: to_device(v, dtype) for k, v in blank.items()}
    gx.params_merge(cfg, sd, bd, stream=st)
    torch.cuda.synchronize()
    for k in mine:
        got = to_host(bd[k]).astype(np.float32)
        e = expect[k]
        assert np.array_equal(np.isnan(got), np.isnan(e)), k
        assert np.array_equal(got[~np.isnan(e)], e[~np.isnan(e)]), k


def test_full_size_transition_round_trip():
    """The TP-shard workload's block (402 MB of bf16 weights): slice every rank out of the whole
    block, merge them into an empty one, and get the whole block back bit for bit; one rank's
    shard is also compared with the oracle's."""
    shape, _, _ = I.WORKLOADS["C3"]
    H, F, a, f = shape.hidden, shape.ffn, shape.tp_attn, shape.tp_ffn
    gen = torch.Generator(device=DEV).manual_seed(I.SEED + 1)
    dims = dict(ln1_g=(H,), ln1_b=(H,), w_qkv=(H, 3 * H), b_qkv=(3 * H,), w_o=(H, H), b_o=(H,),
                ln2_g=(H,), ln2_b=(H,), w_fc1=(H, F), b_fc1=(F,), w_fc2=(F, H), b_fc2=(H,))
    whole = {k: torch.randn(d, device=DEV, generator=gen).to(torch.bfloat16) for k, d in dims.items()}
    back = {k: torch.full(d, float("nan"), device=DEV, dtype=torch.bfloat16) for k, d in dims.items()}
    Hl, Fl = H // a, F // f
    sdims = dict(dims, w_qkv=(H, 3 * Hl), b_qkv=(3 * Hl,), w_o=(Hl, H), w_fc1=(H, Fl), b_fc1=(Fl,), w_fc2=(Fl, H))
    st = torch.cuda.current_stream().cuda_stream
    for r in range(a):
        cfg = gx.make_cfg(H, shape.heads, F, a, f, r, 1, 1, gx.GX_BF16, 3)
        shard = {k: torch.empty(d, device=DEV, dtype=torch.bfloat16) for k, d in sdims.items()}
        gx.params_slice(cfg, whole, shard, stream=st)
        gx.params_merge(cfg, shard, back, stream=st)
        if r == 2:
            torch.cuda.synchronize()
            wh = {k: v.float().cpu().numpy() for k, v in whole.items()}
            ref = N.slice_params(wh, H, shape.heads, F, a, f, r, r)
            for k in I.PARAM_NAMES:
                assert np.array_equal(shard[k].float().cpu().numpy(), ref[k]), k
    torch.cuda.synchronize()
    for k in dims:
        assert torch.equal(back[k].view(torch.int16), whole[k].view(torch.int16)), k


def test_cost_table_row_is_measured_on_the_gpu():
    """The model profiler's compute column comes from timing single-phase calls of the library;
    a row at a graded shard shape must land in a sane band around the bench's rate."""
    from paper_2504_03662_amd import profiler as PF
    shape, _, _ = I.WORKLOADS["C3"]
    m = PF.Model(shape.hidden, shape.heads, shape.ffn, shape.seq, 1)
    rows = PF.cost_table(m, gpus=4, global_batch=2, measure=True)
    r = next(r for r in rows if (r["tp_attn"], r["tp_ffn"]) == (4, 4))
    assert 300.0 < r["tflops_per_gpu"] < 2500.0, r
    assert r["compute_ms"] > 0 and r["mem_bytes"] > r["state_bytes"]
