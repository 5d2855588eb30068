"""Invariants the method fixes (paper Sec. 2.1: chunked prefill only
re-schedules the prompt; Sec. 3.4: a draft sequence is verified in a single
step; Sec. 2.1: batching is a throughput device) checked on the oracle."""
import numpy as np
import pytest

import hat_inputs as hi
from oracle import OracleMiddle

CFG = dict(n_layers=2, d_model=32, n_heads=4, head_dim=8, d_ffn=48, rms_eps=1e-6, rope_theta=1e4)


def make(cfg=CFG, seed=5):
    layers = [hi.layer_weights(cfg, l, seed, gain_jitter=0.2, round_bf16=False, std=0.3) for l in range(cfg["n_layers"])]
    return OracleMiddle(cfg, layers)


def kv_equal(a, b, dev_a=0, dev_b=0):
    for la, lb in zip(a.kv[dev_a], b.kv[dev_b]):
        for x, y in zip(la, lb):
            assert x.shape == y.shape and np.allclose(x, y, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("split", [[21], [1] * 21, [16, 5], [3, 7, 11], [8, 8, 5]])
def test_chunk_split_invariance(split):
    x = np.random.default_rng(0).standard_normal((21, CFG["d_model"]))
    ref = make(); y_ref = ref.forward([(0, 0, x)])[0]
    m = make(); outs = []; s = 0
    for n in split:
        outs.append(m.forward([(0, s, x[s:s + n])])[0]); s += n
    assert np.allclose(np.concatenate(outs), y_ref, rtol=1e-9, atol=1e-11)
    kv_equal(m, ref)


def test_verify_at_once_equals_sequential_steps():
    rng = np.random.default_rng(1)
    prompt = rng.standard_normal((10, CFG["d_model"])); draft = rng.standard_normal((5, CFG["d_model"]))
    a = make(); a.forward([(0, 0, prompt)]); ya = a.forward([(0, 10, draft)])[0]
    b = make(); b.forward([(0, 0, prompt)])
    yb = np.concatenate([b.forward([(0, 10 + i, draft[i:i + 1])])[0] for i in range(5)])
    assert np.allclose(ya, yb, rtol=1e-9, atol=1e-11)
    kv_equal(a, b)


def test_batch_independence_and_permutation():
    rng = np.random.default_rng(2)
    xs = {d: rng.standard_normal((n, CFG["d_model"])) for d, n in ((0, 7), (1, 3), (2, 12))}
    solo = {d: make().forward([(d, 0, x)])[0] for d, x in xs.items()}
    m = make(); outs = m.forward([(d, 0, xs[d]) for d in (2, 0, 1)])
    for d, y in zip((2, 0, 1), outs):
        assert np.allclose(y, solo[d], rtol=1e-12, atol=1e-13)
    # second step: mixed chunk + verify rows, again independent of company
    x2 = {d: rng.standard_normal((n, CFG["d_model"])) for d, n in ((0, 4), (2, 9))}
    outs2 = m.forward([(0, 7, x2[0]), (2, 12, x2[2])])
    s0 = make(); s0.forward([(0, 0, xs[0])]); y0 = s0.forward([(0, 7, x2[0])])[0]
    assert np.allclose(outs2[0], y0, rtol=1e-12, atol=1e-13)


def test_rollback_equals_never_appended():
    rng = np.random.default_rng(3)
    prompt = rng.standard_normal((9, CFG["d_model"])); d1 = rng.standard_normal((4, CFG["d_model"]))
    d2 = rng.standard_normal((4, CFG["d_model"]))
    a = make(); a.forward([(0, 0, prompt)]); a.forward([(0, 9, d1)])
    ya = a.forward([(0, 11, d2)])[0]                 # 2 of 4 draft rows accepted
    b = make(); b.forward([(0, 0, prompt)]); b.forward([(0, 9, d1[:2])])
    yb = b.forward([(0, 11, d2)])[0]
    assert np.allclose(ya, yb, rtol=1e-12, atol=1e-13)
    assert a.kv_len(0) == 15
    kv_equal(a, b)


def test_causality_future_rows_do_not_matter():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((8, CFG["d_model"])); x2 = x.copy(); x2[5:] += 1.0
    y = make().forward([(0, 0, x)])[0]; y2 = make().forward([(0, 0, x2)])[0]
    assert np.array_equal(y[:5], y2[:5]) and not np.allclose(y[5:], y2[5:])


def test_errors_and_release():
    m = make(); x = np.zeros((2, CFG["d_model"]))
    with pytest.raises(ValueError):
        m.forward([(0, 1, x)])
    with pytest.raises(ValueError):
        m.forward([(0, 0, x), (0, 2, x)])
    m.forward([(0, 0, x)]); assert m.kv_len(0) == 2
    m.release(0); assert m.kv_len(0) == 0


def test_import_kv_equals_computed_prefix():
    rng = np.random.default_rng(6)
    p = rng.standard_normal((6, CFG["d_model"])); x = rng.standard_normal((3, CFG["d_model"]))
    a = make(); a.forward([(0, 0, p)]); ya = a.forward([(0, 6, x)])[0]
    b = make()
    for l in range(CFG["n_layers"]):
        b.import_kv(0, l, 0, a.kv[0][l][0][:6], a.kv[0][l][1][:6])
    yb = b.forward([(0, 6, x)])[0]
    assert np.allclose(ya, yb, rtol=1e-12, atol=1e-13)


def test_float32_variant_close_to_float64():
    layers = [hi.layer_weights(CFG, l, 5, round_bf16=False, std=0.3) for l in range(2)]
    x = np.random.default_rng(7).standard_normal((6, CFG["d_model"]))
    y64 = OracleMiddle(CFG, layers).forward([(0, 0, x)])[0]
    y32 = OracleMiddle(CFG, layers, dtype=np.float32).forward([(0, 0, x)])[0]
    assert y32.dtype == np.float32
    assert np.max(np.abs(y32 - y64)) / np.max(np.abs(y64)) < 1e-5


def test_lazy_layers_callable():
    layers = [hi.layer_weights(CFG, l, 5, round_bf16=False, std=0.3) for l in range(2)]
    x = np.random.default_rng(8).standard_normal((4, CFG["d_model"]))
    y1 = OracleMiddle(CFG, layers).forward([(0, 0, x)])[0]
    y2 = OracleMiddle(CFG, lambda l: layers[l]).forward([(0, 0, x)])[0]
    assert np.array_equal(y1, y2)
