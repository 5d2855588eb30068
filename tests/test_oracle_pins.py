"""Pins for oracle/decoder.py: each test fixes the oracle to something that is
not the oracle itself -- scalar brute force, closed forms, textbook special
cases, or an independent library routine (torch CPU) used as a third opinion."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import hat_inputs as hi
from oracle import decoder as od

CFG = dict(n_layers=2, d_model=32, n_heads=4, head_dim=8, d_ffn=48, rms_eps=1e-6, rope_theta=1e4)


def small_weights(cfg, layer, seed=3, jitter=0.2):
    return hi.layer_weights(cfg, layer, seed, gain_jitter=jitter, round_bf16=False, std=0.3)


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_constant_row_closed_form():
    eps = 1e-6
    for c in (2.0, -0.5, 1e-3):
        x = np.full((1, 16), c)
        y = od.rmsnorm(x, np.ones(16), eps)
        assert np.allclose(y, np.sign(c) / math.sqrt(1 + eps / c ** 2), rtol=1e-12)


def test_rmsnorm_matches_torch_and_uses_gain():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 24))
    g = rng.standard_normal(24)
    y = od.rmsnorm(x, g, 1e-5)
    yt = F.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(g), 1e-5).numpy()
    assert np.allclose(y, yt, rtol=1e-12, atol=1e-14)
    # eps sits inside the root, on the mean of squares: a zero row stays zero
    assert np.all(od.rmsnorm(np.zeros((1, 8)), np.ones(8), 1e-6) == 0)
    # and for a tiny row the eps term dominates: x / sqrt(eps)
    tiny = np.full((1, 8), 1e-9)
    assert np.allclose(od.rmsnorm(tiny, np.ones(8), 1e-6), 1e-9 / math.sqrt(1e-18 + 1e-6), rtol=1e-12)


# ------------------------------------------------------------------ RoPE
def test_rope_explicit_values_fix_pairing_and_sign():
    # hd = 4: pairs (0,2) and (1,3); angles pos*1 and pos*1e4**(-1/2) = pos*0.01
    x = np.zeros((1, 1, 4)); x[0, 0, 0] = 1.0; x[0, 0, 1] = 2.0
    y = od.rope_rotate_half(x, [3], 1e4)[0, 0]
    assert np.allclose(y, [math.cos(3.0), 2 * math.cos(0.03), math.sin(3.0), 2 * math.sin(0.03)], rtol=1e-12)
    x = np.zeros((1, 1, 4)); x[0, 0, 2] = 1.0
    y = od.rope_rotate_half(x, [3], 1e4)[0, 0]
    assert np.allclose(y, [-math.sin(3.0), 0, math.cos(3.0), 0], atol=1e-15)


def test_rope_pos0_identity_norm_and_relative_property():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((1, 2, 8)); k = rng.standard_normal((1, 2, 8))
    assert np.array_equal(od.rope_rotate_half(q, [0], 1e4), q)
    for m, n, c in ((5, 2, 100), (17, 17, 4000), (8000, 7990, 333)):
        a = np.sum(od.rope_rotate_half(q, [m], 1e4) * od.rope_rotate_half(k, [n], 1e4), -1)
        b = np.sum(od.rope_rotate_half(q, [m + c], 1e4) * od.rope_rotate_half(k, [n + c], 1e4), -1)
        assert np.allclose(a, b, rtol=1e-9, atol=1e-9)
        assert np.allclose(np.linalg.norm(od.rope_rotate_half(q, [m], 1e4)), np.linalg.norm(q))


def test_rope_matches_complex_rotation():
    rng = np.random.default_rng(2)
    n, H, hd = 6, 3, 16
    x = rng.standard_normal((n, H, hd)); pos = np.array([0, 1, 7, 100, 4095, 8511])
    z = x[..., : hd // 2] + 1j * x[..., hd // 2:]
    ang = pos[:, None] * (1e4 ** (-np.arange(0, hd, 2) / hd))[None, :]
    zr = z * np.exp(1j * ang)[:, None, :]
    y = od.rope_rotate_half(x, pos, 1e4)
    assert np.allclose(y[..., : hd // 2], zr.real, rtol=1e-12, atol=1e-12)
    assert np.allclose(y[..., hd // 2:], zr.imag, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ attention
def brute_attention(q, K, V, start):
    """Explicit [n, len] score matrix, -inf mask, naive softmax; scalar loops."""
    n, H, hd = q.shape
    L = K.shape[0]
    out = np.zeros_like(q)
    for h in range(H):
        for t in range(n):
            sc = []
            for j in range(L):
                if j > start + t:
                    sc.append(-math.inf)
                else:
                    sc.append(sum(q[t, h, i] * K[j, h, i] for i in range(hd)) / math.sqrt(hd))
            m = max(sc)
            e = [math.exp(s - m) for s in sc]
            z = sum(e)
            for i in range(hd):
                out[t, h, i] = sum(e[j] / z * V[j, h, i] for j in range(L))
    return out


@pytest.mark.parametrize("n,start", [(1, 0), (3, 0), (4, 5), (1, 9)])
def test_attention_matches_brute_force(n, start):
    rng = np.random.default_rng(10 + n + start)
    H, hd = 2, 4
    q = rng.standard_normal((n, H, hd)); K = rng.standard_normal((start + n, H, hd)) * 2
    V = rng.standard_normal((start + n, H, hd))
    assert np.allclose(od.prefix_causal_attention(q, K, V, start), brute_attention(q, K, V, start),
                       rtol=1e-12, atol=1e-13)


def test_attention_matches_torch_sdpa_with_prefix_mask():
    rng = np.random.default_rng(5)
    n, start, H, hd = 7, 13, 3, 16
    q = rng.standard_normal((n, H, hd)); K = rng.standard_normal((start + n, H, hd))
    V = rng.standard_normal((start + n, H, hd))
    mask = torch.arange(start + n)[None, :] <= (start + torch.arange(n))[:, None]
    o = F.scaled_dot_product_attention(torch.from_numpy(q).permute(1, 0, 2)[None],
                                       torch.from_numpy(K).permute(1, 0, 2)[None],
                                       torch.from_numpy(V).permute(1, 0, 2)[None], attn_mask=mask)
    assert np.allclose(od.prefix_causal_attention(q, K, V, start), o[0].permute(1, 0, 2).numpy(),
                       rtol=1e-10, atol=1e-12)


def test_attention_special_cases():
    rng = np.random.default_rng(6)
    H, hd = 2, 8
    # one key: output is that key's value row whatever q is
    q = rng.standard_normal((1, H, hd)); K = rng.standard_normal((1, H, hd)); V = rng.standard_normal((1, H, hd))
    assert np.allclose(od.prefix_causal_attention(q, K, V, 0), V)
    # all keys equal: uniform weights, output is the mean of the visible values
    L = 6
    K = np.repeat(rng.standard_normal((1, H, hd)), L, 0); V = rng.standard_normal((L, H, hd))
    q = rng.standard_normal((2, H, hd))
    o = od.prefix_causal_attention(q, K, V, 4)
    assert np.allclose(o[0], V[:5].mean(0)) and np.allclose(o[1], V[:6].mean(0))
    # two keys, scores a and b: weights are the logistic of (a-b); pins the 1/sqrt(hd) scale
    q = np.zeros((1, 1, 4)); q[0, 0, 0] = 2.0
    K = np.zeros((2, 1, 4)); K[0, 0, 0] = 3.0; K[1, 0, 0] = 1.0
    V = np.zeros((2, 1, 4)); V[0, 0, 0] = 1.0
    w0 = 1 / (1 + math.exp(-(2 * 3 - 2 * 1) / 2.0))
    assert np.allclose(od.prefix_causal_attention(q, K, V, 1)[0, 0, 0], w0, rtol=1e-12)
    # huge scores do not overflow
    q = np.full((1, 1, 4), 300.0); K = np.full((3, 1, 4), 300.0); V = np.arange(12.).reshape(3, 1, 4)
    assert np.all(np.isfinite(od.prefix_causal_attention(q, K, V, 2)))


def test_silu_values():
    assert od.silu(np.array(0.0)) == 0
    assert math.isclose(float(od.silu(np.array(1.0))), 0.7310585786300049, rel_tol=1e-12)
    z = np.linspace(-20, 20, 41)
    assert np.allclose(od.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------------ whole layer
def torch_layer(x, start, w, Kp, Vp, cfg):
    """Third opinion: the same layer with torch CPU ops and a complex-number RoPE."""
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    H, hd, n = cfg["n_heads"], cfg["head_dim"], x.shape[0]
    x = t(x)
    xn = F.rms_norm(x, (x.shape[1],), t(w["attn_norm"]), cfg["rms_eps"])
    q, k, v = (F.linear(xn, t(w[nm])).view(n, H, hd) for nm in ("wq", "wk", "wv"))
    pos = torch.arange(start, start + n, dtype=torch.float64)
    ang = pos[:, None] * cfg["rope_theta"] ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]

    def rope(a):
        z = torch.complex(a[..., : hd // 2], a[..., hd // 2:]) * rot
        return torch.cat([z.real, z.imag], -1)
    q, k = rope(q), rope(k)
    K = torch.cat([t(Kp), k]); V = torch.cat([t(Vp), v])
    mask = torch.arange(start + n)[None, :] <= (start + torch.arange(n))[:, None]
    o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], K.permute(1, 0, 2)[None],
                                       V.permute(1, 0, 2)[None], attn_mask=mask)[0].permute(1, 0, 2).reshape(n, -1)
    h = x + F.linear(o, t(w["wo"]))
    hn = F.rms_norm(h, (h.shape[1],), t(w["ffn_norm"]), cfg["rms_eps"])
    y = h + F.linear(F.silu(F.linear(hn, t(w["w_gate"]))) * F.linear(hn, t(w["w_up"])), t(w["w_down"]))
    return y.numpy(), K.numpy(), V.numpy()


def test_layer_matches_torch_third_opinion():
    cfg = CFG
    w = {k: v.astype(np.float64) for k, v in small_weights(cfg, 0).items()}
    rng = np.random.default_rng(7)
    H, hd = cfg["n_heads"], cfg["head_dim"]
    Kp = rng.standard_normal((5, H, hd)); Vp = rng.standard_normal((5, H, hd))
    x = rng.standard_normal((6, cfg["d_model"]))
    kv = [Kp.copy(), Vp.copy()]
    y = od.decoder_layer(x, 5, w, kv, cfg)
    yt, Kt, Vt = torch_layer(x, 5, w, Kp, Vp, cfg)
    assert np.allclose(y, yt, rtol=1e-10, atol=1e-11)
    assert np.allclose(kv[0], Kt, rtol=1e-11, atol=1e-12) and np.allclose(kv[1], Vt, rtol=1e-11, atol=1e-12)


def test_layer_is_identity_when_output_projections_vanish():
    cfg = CFG
    w = {k: v.astype(np.float64) for k, v in small_weights(cfg, 0).items()}
    w["wo"] = np.zeros_like(w["wo"]); w["w_down"] = np.zeros_like(w["w_down"])
    x = np.random.default_rng(8).standard_normal((4, cfg["d_model"]))
    H, hd = cfg["n_heads"], cfg["head_dim"]
    y = od.decoder_layer(x, 0, w, [np.zeros((0, H, hd)), np.zeros((0, H, hd))], cfg)
    assert np.array_equal(y, x)


def scalar_layer(x, w, cfg):
    """A whole layer at start 0 with nothing but Python floats and loops."""
    n, d = len(x), cfg["d_model"]
    H, hd, Fd = cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"]

    def norm(row, g):
        ms = sum(v * v for v in row) / len(row)
        return [v / math.sqrt(ms + cfg["rms_eps"]) * g[i] for i, v in enumerate(row)]

    def lin(row, W):
        return [sum(W[o][i] * row[i] for i in range(len(row))) for o in range(len(W))]

    def rope(vec, pos):
        out = list(vec)
        for h in range(H):
            for i in range(hd // 2):
                a = pos * cfg["rope_theta"] ** (-2.0 * i / hd)
                lo, hi_ = vec[h * hd + i], vec[h * hd + i + hd // 2]
                out[h * hd + i] = lo * math.cos(a) - hi_ * math.sin(a)
                out[h * hd + i + hd // 2] = hi_ * math.cos(a) + lo * math.sin(a)
        return out
    xn = [norm(r, w["attn_norm"]) for r in x]
    q = [rope(lin(r, w["wq"]), t) for t, r in enumerate(xn)]
    k = [rope(lin(r, w["wk"]), t) for t, r in enumerate(xn)]
    v = [lin(r, w["wv"]) for r in xn]
    y = []
    for t in range(n):
        o = [0.0] * d
        for h in range(H):
            sc = [sum(q[t][h * hd + i] * k[j][h * hd + i] for i in range(hd)) / math.sqrt(hd) for j in range(t + 1)]
            m = max(sc); e = [math.exp(s - m) for s in sc]; z = sum(e)
            for i in range(hd):
                o[h * hd + i] = sum(e[j] / z * v[j][h * hd + i] for j in range(t + 1))
        hrow = [x[t][i] + val for i, val in enumerate(lin(o, w["wo"]))]
        hn = norm(hrow, w["ffn_norm"])
        g = lin(hn, w["w_gate"]); u = lin(hn, w["w_up"])
        a = [gg / (1 + math.exp(-gg)) * uu for gg, uu in zip(g, u)]
        y.append([hrow[i] + val for i, val in enumerate(lin(a, w["w_down"]))])
    return np.array(y)


def test_layer_matches_scalar_python():
    cfg = dict(n_layers=1, d_model=8, n_heads=2, head_dim=4, d_ffn=12, rms_eps=1e-6, rope_theta=1e4)
    w = {k: v.astype(np.float64) for k, v in small_weights(cfg, 0, seed=4).items()}
    x = np.random.default_rng(9).standard_normal((5, 8))
    H, hd = 2, 4
    y = od.decoder_layer(x, 0, w, [np.zeros((0, H, hd)), np.zeros((0, H, hd))], cfg)
    ys = scalar_layer(x.tolist(), {k: v.tolist() for k, v in w.items()}, cfg)
    assert np.allclose(y, ys, rtol=1e-11, atol=1e-12)
