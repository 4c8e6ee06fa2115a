"""Pins for the dropout variant of the oracle: the counter-based generator against its published
known-answer vectors, the byte order and keep rule, and the layer with dropout against finite
differences and the sharding identities.  None of these call the HIP path."""
import numpy as np
import pytest

from oracle import dropout as D
from oracle import layer as O
from paper_2504_03662_amd import inputs as I


def _kat():
    """(counter, key, output) triples from tests/golden/philox4x32_10_kat.txt."""
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                w = [int(t, 16) for t in line.split()]
                rows.append((tuple(w[:4]), tuple(w[4:6]), tuple(w[6:])))
    return rows


KAT = _kat()


@pytest.mark.parametrize("ctr,key,out", KAT)
def test_philox_known_answers(ctr, key, out):
    assert len(KAT) == 3
    got = D.philox4x32_10(*ctr, *key)
    assert tuple(int(w) for w in got) == out


def test_philox_is_vectorised_consistently():
    # arrays of counters give what single counters give
    c0 = np.array([0, 0xffffffff, 0x243f6a88], dtype=np.uint64)
    single = [D.philox4x32_10(int(c), 5, 6, 7, 11, 13) for c in c0]
    many = D.philox4x32_10(c0, 5, 6, 7, 11, 13)
    for n in range(3):
        assert [int(w[n]) for w in many] == [int(w) for w in single[n]]


def test_byte_order_and_seed_split():
    # seed = k1 * 2^32 + k0; bytes are the words in order, least-significant byte first
    seed = (0x299f31d0 << 32) | 0xa4093822
    b = D.random_bytes(0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344, seed)
    assert b.shape == (16,)
    assert list(b[:4]) == [0x09, 0xfe, 0x6c, 0xd1] and list(b[12:]) == [0xa1, 0x6e, 0x12, 0x24]


def test_keep_rule_counters_and_frequency():
    seed, t, S = 77, 64, 96
    keep = D.keep_attention(seed, t, S, sample=1, head=2, heads=4)
    assert keep.shape == (S, S)
    # element (i, j) reads byte j % 16 of counter (i, j // 16, sample * heads + head, 1)
    for i, j in [(0, 0), (5, 15), (5, 16), (95, 95), (33, 70)]:
        byte = D.random_bytes(i, j // 16, 1 * 4 + 2, D.STREAM_ATTN_PROBS, seed)[j % 16]
        assert keep[i, j] == (byte >= t)
    # kept fraction 1 - t/256 = 0.75 within 5 binomial standard deviations
    n = S * S
    assert abs(keep.mean() - 0.75) < 5 * np.sqrt(0.75 * 0.25 / n)
    # the two hidden streams and other heads are different masks
    a = D.keep_hidden(seed, t, 40, 72, D.STREAM_ATTN_OUT)
    m = D.keep_hidden(seed, t, 40, 72, D.STREAM_MLP_OUT)
    assert a.shape == (40, 72) and (a != m).mean() > 0.2
    assert (D.keep_attention(seed, t, S, 1, 3, 4) != keep).mean() > 0.2
    assert (D.keep_attention(seed + 1, t, S, 1, 2, 4) != keep).mean() > 0.2
    # t = 0 keeps everything, scale 1
    assert D.keep_attention(seed, 0, S, 0, 0, 1).all() and D.scale_of(0) == 1.0
    assert D.scale_of(64) == pytest.approx(4.0 / 3.0)
    with pytest.raises(ValueError):
        D.scale_of(256)


def test_keep_hidden_counters_element_by_element():
    """Element (token, column) of a half's output reads byte column % 16 of counter
    (token, column // 16, 0, stream): the expectation is rebuilt from the generator for single
    elements, with sizes that differ in every index (a swapped token / column group, a wrong third
    word or stream would fail), including the last, partly used column group."""
    seed, t, T, H = (0x1234 << 32) | 99, 100, 37, 72           # 72 = 4 groups of 16 + 8 columns
    for stream in (D.STREAM_ATTN_OUT, D.STREAM_MLP_OUT):
        keep = D.keep_hidden(seed, t, T, H, stream)
        assert keep.shape == (T, H)
        for tok, col in [(0, 0), (0, 15), (0, 16), (1, 0), (5, 33), (33, 5), (36, 71), (36, 64), (17, 48), (2, 70)]:
            byte = D.random_bytes(tok, col // 16, 0, stream, seed)[col % 16]
            assert keep[tok, col] == (byte >= t), (stream, tok, col)
        # every element of two whole rows, one counter at a time
        for tok in (3, 36):
            row = np.concatenate([D.random_bytes(tok, g, 0, stream, seed) for g in range(5)])[:H]
            assert np.array_equal(keep[tok], row >= t)
    # the mask is not symmetric in (token, column group): the transposed reading differs
    sq = D.keep_hidden(seed, t, 64, 64 * 16, D.STREAM_ATTN_OUT)
    swapped = np.array([[D.random_bytes(c // 16, tok, 0, D.STREAM_ATTN_OUT, seed)[c % 16] >= t for c in range(0, 64 * 16, 97)]
                        for tok in range(0, 64, 7)])
    assert (sq[0:64:7, 0:64 * 16:97] != swapped).mean() > 0.2
    n = T * H
    assert abs(D.keep_hidden(seed, 64, T, H, 2).mean() - 0.75) < 5 * np.sqrt(0.75 * 0.25 / n)


def _tiny(drop_attn=0, drop_hidden=0, seed=5, **kw):
    base = dict(hidden=32, heads=4, ffn=48, seq=12, micro_batch=2, dtype="f32", drop_attn=drop_attn,
                drop_hidden=drop_hidden, drop_seed=seed)
    base.update(kw)
    shape = I.LayerShape(**base)
    full = {k: v.astype(np.float64) for k, v in
            I.full_params(shape.with_(tp_attn=1, tp_ffn=1), case=81, random_affine=True).items()}
    full = {k: (v * 8 if k.startswith("w_") else v) for k, v in full.items()}
    x, dy = (a.astype(np.float64) for a in I.activations(shape, case=81))
    return shape, full, x, dy


def test_zero_probability_is_the_plain_layer():
    shape, p, x, dy = _tiny()
    shape0 = shape.with_(drop_seed=1234)
    a, b = O.layer_fwd(shape, p, x), O.layer_fwd(shape0, p, x)
    assert np.array_equal(a["y"], b["y"])


def test_attention_dropout_by_brute_force():
    # one head, written out with loops: O_i = sum_j P_ij keep_ij scale V_j
    shape, p, x, _ = _tiny(drop_attn=96, heads=1, hidden=16, seq=9, micro_batch=1, ffn=16)
    out = O.layer_fwd(shape, p, x, "attn")
    ca = out["cache"]["attn"]
    q, k, v = ca["qkv"][:, :16], ca["qkv"][:, 16:32], ca["qkv"][:, 32:]
    keep = D.keep_attention(shape.drop_seed, 96, 9, 0, 0, 1)
    assert not keep[np.tril_indices(9)].all() and keep.any()          # the case does drop something
    ctx = np.zeros((9, 16))
    for i in range(9):
        s = np.array([q[i] @ k[j] / 4.0 for j in range(i + 1)])
        pr = np.exp(s - s.max())
        pr /= pr.sum()
        for j in range(i + 1):
            if keep[i, j]:
                ctx[i] += pr[j] * (256.0 / 160.0) * v[j]
    assert np.allclose(ca["ctx"], ctx, rtol=1e-12, atol=1e-14)


def test_hidden_dropout_definition():
    shape, p, x, _ = _tiny(drop_hidden=128)
    out = O.layer_fwd(shape, p, x)
    ka = D.keep_hidden(shape.drop_seed, 128, shape.tokens, shape.hidden, D.STREAM_ATTN_OUT)
    km = D.keep_hidden(shape.drop_seed, 128, shape.tokens, shape.hidden, D.STREAM_MLP_OUT)
    h1 = x + np.where(ka, 2.0 * out["p_attn"], 0.0)
    assert np.allclose(out["h1"], h1, rtol=1e-14)
    assert np.allclose(out["y"], h1 + np.where(km, 2.0 * out["p_mlp"], 0.0), rtol=1e-14)
    # a lone half returns its partial undropped
    lone = O.layer_fwd(shape, p, x, "attn")["p_attn"]
    assert np.array_equal(lone, O.layer_fwd(shape.with_(drop_hidden=0), p, x, "attn")["p_attn"])


@pytest.mark.parametrize("phase", ["both", "attn", "mlp"])
def test_gradients_with_dropout_match_finite_differences(phase):
    shape, p, x, dy = _tiny(drop_attn=64, drop_hidden=80)
    out_key = {"both": "y", "attn": "p_attn", "mlp": "p_mlp"}[phase]
    f = lambda pp, xx: float((O.layer_fwd(shape, pp, xx, phase)[out_key] * dy).sum())
    out = O.layer_fwd(shape, p, x, phase)
    dx, g = O.layer_bwd(shape, p, dy, out["cache"], phase)
    rng = np.random.default_rng(3)
    eps = 1e-6
    for _ in range(12):
        i = tuple(rng.integers(n) for n in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[i] += eps
        xm[i] -= eps
        assert (f(p, xp) - f(p, xm)) / (2 * eps) == pytest.approx(dx[i], rel=2e-5, abs=1e-7)
    for name, grad in g.items():
        for _ in range(4):
            i = tuple(rng.integers(n) for n in p[name].shape)
            pp, pm = dict(p), dict(p)
            pp[name] = p[name].copy()
            pm[name] = p[name].copy()
            pp[name][i] += eps
            pm[name][i] -= eps
            assert (f(pp, x) - f(pm, x)) / (2 * eps) == pytest.approx(grad[i], rel=2e-5, abs=1e-7), name


def test_rank_partials_with_attention_dropout_add_up():
    """The mask is indexed by the global head, so the sharded attention halves still sum to the
    unsharded one."""
    from oracle import neighbours as N
    shape, full, x, _ = _tiny(drop_attn=100)
    ref = O.layer_fwd(shape, full, x, "attn")["p_attn"]
    total = np.zeros_like(ref)
    for r in range(2):
        sr = shape.with_(tp_attn=2, tp_rank=r)
        pr = N.slice_params(full, shape.hidden, shape.heads, shape.ffn, 2, 1, r, 0)
        total += O.layer_fwd(sr, pr, x, "attn", row_bias_attn=(r == 0))["p_attn"]
    assert np.allclose(total, ref, atol=1e-12)
    # and it differs from the layer without dropout
    assert not np.allclose(ref, O.layer_fwd(shape.with_(drop_attn=0), full, x, "attn")["p_attn"], atol=1e-3)


def test_dropout_is_unbiased_over_seeds():
    shape, p, x, _ = _tiny(drop_attn=64, drop_hidden=64)
    plain = O.layer_fwd(shape.with_(drop_attn=0, drop_hidden=0), p, x, "attn")["p_attn"]
    acc = np.zeros_like(plain)
    n = 300
    for s in range(n):
        acc += O.layer_fwd(shape.with_(drop_seed=1000 + s), p, x, "attn")["p_attn"]
    # mean over masks -> the undropped half (attention dropout is linear in the mask)
    assert np.abs(acc / n - plain).max() < 0.15 * np.abs(plain).max()
