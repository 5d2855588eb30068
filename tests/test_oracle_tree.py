"""Tree verification on the oracle (paper Sec. 2.2: the candidates of one step
form a tree whose every branch is a possible accepted path, verified in a single
step).  What that fixes without reference to the oracle's own code: a node's
result is the result of its path submitted alone as an ordinary draft chain,
and after the accepted path has been kept the cache is the chain's cache."""
import math

import numpy as np
import pytest

import hat_inputs as hi
from oracle import OracleMiddle
from oracle.decoder import check_tree, tree_attention, tree_depths, prefix_causal_attention

CFG = dict(n_layers=2, d_model=32, n_heads=4, head_dim=8, d_ffn=48, rms_eps=1e-6, rope_theta=1e4)


def make(cfg=CFG, seed=5):
    layers = [hi.layer_weights(cfg, l, seed, gain_jitter=0.2, round_bf16=False, std=0.3) for l in range(cfg["n_layers"])]
    return OracleMiddle(cfg, layers)


TREES = [hi.MEDUSA_LIKE_TREE, [-1], [-1, -1, -1], [-1, 0, 1, 2, 3, 4, 5, 6], [-1, 0, 0, 0, 0, 0, 0, 0]] + \
        [hi.random_tree(3, n, k) for n in (2, 5, 8) for k in range(3)]


@pytest.mark.parametrize("parents", TREES)
def test_every_path_equals_that_path_submitted_alone(parents):
    n = len(parents); masks = hi.tree_masks(parents)
    rng = np.random.default_rng(11)
    prompt = rng.standard_normal((13, CFG["d_model"])); cand = rng.standard_normal((n, CFG["d_model"]))
    t = make(); t.forward([(0, 0, prompt)]); y = t.forward([(0, 13, cand, masks)])[0]
    assert t.kv_len(0) == 13 + n
    for node in range(n):
        path = hi.tree_path(parents, node)
        c = make(); c.forward([(0, 0, prompt)]); yc = c.forward([(0, 13, cand[path])])[0]
        assert np.allclose(y[path], yc, rtol=1e-9, atol=1e-11), (node, path)


def test_chain_shaped_tree_is_the_chain():
    rng = np.random.default_rng(12)
    prompt = rng.standard_normal((9, CFG["d_model"])); cand = rng.standard_normal((6, CFG["d_model"]))
    a = make(); a.forward([(0, 0, prompt)]); ya = a.forward([(0, 9, cand, hi.tree_masks([-1, 0, 1, 2, 3, 4]))])[0]
    b = make(); b.forward([(0, 0, prompt)]); yb = b.forward([(0, 9, cand)])[0]
    assert np.allclose(ya, yb, rtol=1e-12, atol=1e-13)
    for la, lb in zip(a.kv[0], b.kv[0]):
        assert np.allclose(la[0], lb[0], rtol=1e-12, atol=1e-13) and np.allclose(la[1], lb[1], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("node", [0, 4, 6, 7])
def test_compaction_leaves_the_chains_cache(node):
    parents = hi.MEDUSA_LIKE_TREE; masks = hi.tree_masks(parents); path = hi.tree_path(parents, node)
    rng = np.random.default_rng(13)
    prompt = rng.standard_normal((20, CFG["d_model"])); cand = rng.standard_normal((8, CFG["d_model"]))
    nxt = rng.standard_normal((3, CFG["d_model"]))
    t = make(); t.forward([(0, 0, prompt)]); t.forward([(0, 20, cand, masks)]); t.compact(0, 20, path)
    c = make(); c.forward([(0, 0, prompt)]); c.forward([(0, 20, cand[path])])
    assert t.kv_len(0) == c.kv_len(0) == 20 + len(path)
    for lt, lc in zip(t.kv[0], c.kv[0]):
        assert np.allclose(lt[0], lc[0], rtol=1e-10, atol=1e-12) and np.allclose(lt[1], lc[1], rtol=1e-10, atol=1e-12)
    yt = t.forward([(0, 20 + len(path), nxt)])[0]; yc = c.forward([(0, 20 + len(path), nxt)])[0]
    assert np.allclose(yt, yc, rtol=1e-9, atol=1e-11)


def test_tree_attention_against_scalar_loops_from_parent_pointers():
    # visibility derived here from the parent pointers, not from the masks; softmax in scalar loops
    parents = hi.MEDUSA_LIKE_TREE; n = len(parents); start, H, hd = 5, 2, 4
    rng = np.random.default_rng(14)
    q = rng.standard_normal((n, H, hd)); K = rng.standard_normal((start + n, H, hd)); V = rng.standard_normal((start + n, H, hd))
    got = tree_attention(q, K, V, start, hi.tree_masks(parents))
    for t in range(n):
        vis = list(range(start)); a = t
        while a != -1:
            vis.append(start + a); a = parents[a]
        for h in range(H):
            sc = [sum(q[t, h, e] * K[r, h, e] for e in range(hd)) / math.sqrt(hd) for r in vis]
            mx = max(sc); ws = [math.exp(v - mx) for v in sc]; z = sum(ws)
            for e in range(hd):
                ref = sum(w / z * V[r, h, e] for w, r in zip(ws, vis))
                assert abs(got[t, h, e] - ref) < 1e-12


def test_tree_attention_of_a_chain_is_prefix_causal_attention():
    rng = np.random.default_rng(15); n, start, H, hd = 7, 6, 3, 8
    q = rng.standard_normal((n, H, hd)); K = rng.standard_normal((start + n, H, hd)); V = rng.standard_normal((start + n, H, hd))
    masks = [(2 << i) - 1 for i in range(n)]
    assert np.allclose(tree_attention(q, K, V, start, masks), prefix_causal_attention(q, K, V, start), rtol=1e-13, atol=1e-14)


def test_siblings_do_not_see_each_other_and_depth_sets_the_position():
    # two roots with the SAME hidden state must give the same output (same position, same view),
    # which fails if the second were placed one position later or saw the first
    rng = np.random.default_rng(16)
    prompt = rng.standard_normal((7, CFG["d_model"])); row = rng.standard_normal((1, CFG["d_model"]))
    m = make(); m.forward([(0, 0, prompt)])
    y = m.forward([(0, 7, np.concatenate([row, row, row]), hi.tree_masks([-1, -1, 0]))])[0]
    assert np.allclose(y[0], y[1], rtol=1e-12, atol=1e-13)
    assert not np.allclose(y[0], y[2], rtol=1e-3, atol=1e-3)
    assert list(tree_depths(hi.tree_masks(hi.MEDUSA_LIKE_TREE))) == [0, 1, 1, 2, 2, 2, 3, 0]


def test_mask_validation():
    assert check_tree(hi.tree_masks(hi.MEDUSA_LIKE_TREE))
    assert check_tree([1, 2, 4]) and check_tree([1, 3, 7]) and check_tree([])
    assert not check_tree([0])            # does not see itself
    assert not check_tree([3])            # sees a later node
    assert not check_tree([1, 2, 7])      # nodes 0 and 1 are both roots: not one path
    assert not check_tree([1, 3, 6])      # sees 1 but not 1's parent 0
    assert not check_tree([1, 2, 0x104])  # a bit beyond itself
    m = make(); x = np.zeros((2, CFG["d_model"]))
    with pytest.raises(ValueError):
        m.forward([(0, 0, x, [1, 1])])
    with pytest.raises(ValueError):
        m.forward([(0, 0, x, [1])])
    m.forward([(0, 0, x, [1, 3])])
    with pytest.raises(ValueError):
        m.compact(0, 0, [1, 0])
    with pytest.raises(ValueError):
        m.compact(0, 1, [0, 1])
    m.compact(0, 0, [1]); assert m.kv_len(0) == 1
