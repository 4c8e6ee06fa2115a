"""Pins for the oracle of the layer step's neighbours (optimizer update, shard transitions).
None of these call the HIP path."""
import numpy as np
import pytest
import torch

from oracle import layer as O
from oracle import neighbours as N
from paper_2504_03662_amd import inputs as I


# ------------------------------------------------------------------ AdamW

def test_adamw_matches_torch_float64_over_steps():
    rng = np.random.default_rng(11)
    w0 = rng.standard_normal(257)
    hp = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    tw = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tw], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                            weight_decay=hp["weight_decay"])
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for step in range(1, 8):
        g = rng.standard_normal(257) * (0.1 if step % 2 else 10.0)
        tw.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = N.adamw_step(w, m, v, g, step, **hp)
        assert np.allclose(w, tw.detach().numpy(), rtol=1e-12, atol=1e-14)
        st = opt.state[tw]
        assert np.allclose(m, st["exp_avg"].numpy(), rtol=1e-13, atol=0)
        assert np.allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-13, atol=0)


def test_adamw_first_step_closed_form():
    # zero moments, step 1: m_hat = g, v_hat = g^2  ->  w' = w - lr * (g / (|g| + eps) + wd * w)
    g = np.array([2.0, -0.5, 1e-3, -7.0])
    w = np.array([1.0, -2.0, 0.5, 4.0])
    lr, eps, wd = 0.01, 1e-8, 0.2
    w1, m1, v1 = N.adamw_step(w, np.zeros(4), np.zeros(4), g, 1, lr, 0.9, 0.999, eps, wd)
    assert np.allclose(w1, w - lr * (g / (np.abs(g) + eps) + wd * w), rtol=1e-14)
    assert np.allclose(m1, 0.1 * g, rtol=1e-14) and np.allclose(v1, 0.001 * g * g, rtol=1e-12)
    # with eps -> 0 the first update is lr * sign(g)
    w2, _, _ = N.adamw_step(w, np.zeros(4), np.zeros(4), g, 1, lr, 0.9, 0.999, 0.0, 0.0)
    assert np.allclose(w - w2, lr * np.sign(g), rtol=1e-14)


def test_adamw_zero_gradient_is_pure_decay_and_moments_decay():
    w = np.array([3.0, -1.0])
    m = np.array([0.5, -0.25])
    v = np.array([0.0, 0.0])
    w1, m1, v1 = N.adamw_step(w, np.zeros(2), np.zeros(2), np.zeros(2), 5, 0.1, 0.9, 0.999, 1e-8, 0.5)
    assert np.allclose(w1, w * (1 - 0.1 * 0.5), rtol=1e-15)
    _, m2, v2 = N.adamw_step(w, m, v, np.zeros(2), 3, 0.1, 0.9, 0.999, 1e-8, 0.0)
    assert np.allclose(m2, 0.9 * m) and np.all(v2 == 0)


def test_adamw_scale_invariance_and_grad_scale():
    rng = np.random.default_rng(5)
    w, m, v, g = (rng.standard_normal(64) for _ in range(4))
    v = v * v
    # eps = 0: scaling gradient history by c leaves the update direction unchanged
    a = N.adamw_step(w, m, v, g, 4, 1e-2, 0.9, 0.99, 0.0, 0.0)[0]
    b = N.adamw_step(w, 7.0 * m, 49.0 * v, 7.0 * g, 4, 1e-2, 0.9, 0.99, 0.0, 0.0)[0]
    assert np.allclose(a, b, rtol=1e-12)
    # grad_scale s on g equals passing s * g
    c = N.adamw_step(w, m, v, g, 4, 1e-2, 0.9, 0.99, 1e-8, 0.01, grad_scale=0.125)
    d = N.adamw_step(w, m, v, 0.125 * g, 4, 1e-2, 0.9, 0.99, 1e-8, 0.01)
    for x, y in zip(c, d):
        assert np.array_equal(x, y)
    with pytest.raises(ValueError):
        N.adamw_step(w, m, v, g, 0, 1e-2)


# ------------------------------------------------------------------ shard transitions

def _full(H=32, heads=4, F=64, seed=3):
    shape = I.LayerShape(H, heads, F, 1, 1, 0, 8, 2, "f32")
    full = {k: v.astype(np.float64) for k, v in I.full_params(shape, case=91, random_affine=True).items()}
    return shape, {k: (v * 10 if k.startswith("w_") else v) for k, v in full.items()}


@pytest.mark.parametrize("a,f", [(1, 1), (2, 2), (4, 2), (2, 4), (4, 1)])
def test_slice_index_formula_and_round_trip(a, f):
    shape, full = _full()
    H, F = shape.hidden, shape.ffn
    Hl, Fl = H // a, F // f
    blank = {k: np.full_like(v, np.nan) for k, v in full.items()}
    for r in range(max(a, f)):
        ra, rf = r % a, r % f
        s = N.slice_params(full, H, shape.heads, F, a, f, ra, rf)
        assert s["w_qkv"].shape == (H, 3 * Hl) and s["w_o"].shape == (Hl, H)
        assert s["w_fc1"].shape == (H, Fl) and s["w_fc2"].shape == (Fl, H)
        # independent statement of the map: shard column c of block p is whole column p*H + r*Hl + c
        rng = np.random.default_rng(r)
        for _ in range(50):
            i, p, c = rng.integers(H), rng.integers(3), rng.integers(Hl)
            assert s["w_qkv"][i, p * Hl + c] == full["w_qkv"][i, p * H + ra * Hl + c]
            assert s["b_qkv"][p * Hl + c] == full["b_qkv"][p * H + ra * Hl + c]
            assert s["w_o"][c, i] == full["w_o"][ra * Hl + c, i]
            k = rng.integers(Fl)
            assert s["w_fc1"][i, k] == full["w_fc1"][i, rf * Fl + k]
            assert s["b_fc1"][k] == full["b_fc1"][rf * Fl + k]
            assert s["w_fc2"][k, i] == full["w_fc2"][rf * Fl + k, i]
        # a rank's heads stay whole: its Q block is heads [r*nl, (r+1)*nl) of the whole Q block
        dh = H // shape.heads
        nl = shape.heads // a
        assert np.array_equal(s["w_qkv"][:, :dh], full["w_qkv"][:, ra * nl * dh:ra * nl * dh + dh])
        for n in ("ln1_g", "ln1_b", "b_o", "ln2_g", "ln2_b", "b_fc2"):
            assert np.array_equal(s[n], full[n])
        N.merge_params(blank, s, H, shape.heads, F, a, f, ra, rf)
    for k in full:
        assert np.array_equal(blank[k], full[k]), k       # every element was written back in place


@pytest.mark.parametrize("a,f", [(2, 2), (4, 2), (1, 4)])
def test_slices_reproduce_the_unsharded_layer(a, f):
    """The property that defines a correct shard: partial sums over ranks give the whole layer."""
    shape, full = _full()
    rng = np.random.default_rng(8)
    x = rng.standard_normal((16, shape.hidden))
    ref = O.layer_fwd(shape, full, x)
    sa = shape.with_(tp_attn=a, tp_ffn=f)
    h1 = x.copy()
    for r in range(a):
        pr = N.slice_params(full, shape.hidden, shape.heads, shape.ffn, a, f, r, 0)
        h1 = h1 + O.layer_fwd(sa, pr, x, "attn", row_bias_attn=(r == 0))["p_attn"]
    assert np.allclose(h1, ref["h1"], atol=1e-12)
    y = h1.copy()
    for r in range(f):
        pr = N.slice_params(full, shape.hidden, shape.heads, shape.ffn, a, f, 0, r)
        y = y + O.layer_fwd(sa, pr, h1, "mlp", row_bias_mlp=(r == 0))["p_mlp"]
    assert np.allclose(y, ref["y"], atol=1e-12)


def test_wrong_slicing_is_caught_by_the_layer_property():
    """Planted mistake (on the CPU): interleaving Q/K/V per rank instead of per block breaks the sum."""
    shape, full = _full()
    a = 2
    sa = shape.with_(tp_attn=a)
    x = np.random.default_rng(2).standard_normal((16, shape.hidden))
    ref = O.layer_fwd(shape, full, x)
    h1 = x.copy()
    Hl = shape.hidden // a
    for r in range(a):
        pr = N.slice_params(full, shape.hidden, shape.heads, shape.ffn, a, 1, r, 0)
        pr["w_qkv"] = np.ascontiguousarray(full["w_qkv"][:, r * 3 * Hl:(r + 1) * 3 * Hl])   # the mistake
        h1 = h1 + O.layer_fwd(sa, pr, x, "attn", row_bias_attn=(r == 0))["p_attn"]
    assert not np.allclose(h1, ref["h1"], atol=1e-6)


def test_indivisible_sharding_raises():
    shape, full = _full()
    with pytest.raises(ValueError):
        N.slice_params(full, shape.hidden, shape.heads, shape.ffn, 3, 1, 0, 0)
