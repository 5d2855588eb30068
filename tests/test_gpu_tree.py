"""GPU parity for tree verification (paper Sec. 2.2: candidates of one step arranged in a tree and
verified in a single step; trees of 8 in Sec. 4.1) and for keeping the accepted path.

Bar as for every other step: max|gpu - ref| / max|ref| <= 2e-2 per segment against the float64
oracle; page tables and cache lengths bit-exact against the page model; moved cache rows byte-exact."""
import numpy as np
import pytest

import hat_inputs as hi
from gpu_util import Pair, rel_err, rel_l2, to_dev_bf16, to_np

pytestmark = pytest.mark.gpu
TOL = 6e-3     # every model here has at most 3 layers: the depth-appropriate bar (gpu_util.tol_for_depth)

SMALL64 = dict(name="small64", n_layers=3, d_model=256, n_heads=4, head_dim=64, d_ffn=688, rms_eps=1e-6, rope_theta=1e4)
SMALL128 = dict(name="small128", n_layers=2, d_model=512, n_heads=4, head_dim=128, d_ffn=1408, rms_eps=1e-5, rope_theta=1e4)


def check(outs, refs, tol=TOL):
    for o, r in zip(outs, refs):
        assert o.shape == r.shape and np.all(np.isfinite(o))
        e = rel_err(o, r)
        assert e <= tol, "rel err %.3e (l2 %.3e)" % (e, rel_l2(o, r))


def tree(parents):
    return hi.tree_masks(parents)


@pytest.mark.parametrize("cfg", [SMALL64, SMALL128], ids=["hd64", "hd128"])
@pytest.mark.parametrize("kv", ["bf16", "f16"])
def test_tree_steps_compaction_and_what_follows(cfg, kv):
    import torch
    p = Pair(cfg, 41, n_pages=120, max_devices=8, max_step_tokens=512, max_pos=1024, kv_dtype=kv)
    # prefixes chosen so that the 8 tree rows end a page (8..15), straddle pages (28..35, 253..260),
    # start a page (64..) and start the cache (device 4: no prefix at all)
    check(*p.step([(0, hi.CHUNK, 0, 28), (1, hi.CHUNK, 0, 8), (2, hi.CHUNK, 0, 253), (3, hi.CHUNK, 0, 64)]))
    med = hi.MEDUSA_LIKE_TREE
    segs = [(0, hi.VERIFY, 28, 8, tree(med)),
            (1, hi.VERIFY, 8, 8, tree([-1, 0, 0, 0, 0, 0, 0, 0])),        # one root, seven leaves
            (2, hi.VERIFY, 253, 8, tree([-1, -1, -1, -1, -1, -1, -1, -1])),  # eight roots
            (3, hi.VERIFY, 64, 5, tree(hi.random_tree(7, 5))),
            (4, hi.VERIFY, 0, 8, tree(hi.random_tree(7, 8))),
            (5, hi.CHUNK, 0, 70),                                         # other kinds in the same step
            (6, hi.VERIFY, 0, 1, tree([-1]))]
    check(*p.step(segs))
    p.check_pages(range(8))
    # keep one path per device; moved rows must be byte-identical to where they came from
    keeps = {0: hi.tree_path(med, 6), 1: hi.tree_path([-1, 0, 0, 0, 0, 0, 0, 0], 7), 2: [5],
             3: hi.tree_path(hi.random_tree(7, 5), 4), 4: hi.tree_path(hi.random_tree(7, 8), 7), 6: []}
    base = {0: 28, 1: 8, 2: 253, 3: 64, 4: 0, 6: 0}
    for d, keep in keeps.items():
        before = [p.gpu.kv_export(d, l, base[d], p.gpu.kv_query(d)[0] - base[d]) for l in range(cfg["n_layers"])] if keep else []
        p.compact(d, base[d], keep)
        assert p.gpu.kv_query(d) == p.pages.query(d) and p.gpu.kv_query(d)[0] == base[d] + len(keep)
        for l in range(cfg["n_layers"] if keep else 0):
            k1, v1 = p.gpu.kv_export(d, l, base[d], len(keep))
            assert torch.equal(k1.view(torch.int16), before[l][0][keep].view(torch.int16))
            assert torch.equal(v1.view(torch.int16), before[l][1][keep].view(torch.int16))
            kr = p.ref.kv[d][l][0][base[d]:]; vr = p.ref.kv[d][l][1][base[d]:]
            assert rel_err(to_np(k1), kr) <= TOL and rel_err(to_np(v1), vr) <= TOL
    p.check_pages(range(8))
    # what follows: chains, a chunk and a new tree continue from the kept paths
    nxt = [(0, hi.VERIFY, 28 + len(keeps[0]), 5), (1, hi.CHUNK, 8 + len(keeps[1]), 40),
           (2, hi.VERIFY, 254, 8, tree(med)), (3, hi.VERIFY, 64 + len(keeps[3]), 3),
           (4, hi.VERIFY, len(keeps[4]), 6, tree(hi.random_tree(8, 6))), (6, hi.CHUNK, 0, 9)]
    check(*p.step(nxt))
    p.check_pages(range(8))
    p.close()


@pytest.mark.parametrize("target", [64, 4096])
def test_tree_over_a_long_cache_split_and_whole(target):
    p = Pair(SMALL128, 42, n_pages=160, max_devices=4, max_step_tokens=2048, max_pos=4096)
    p.gpu.set_attn_targets(target, target)
    check(*p.step([(0, hi.CHUNK, 0, 1500), (1, hi.CHUNK, 0, 333)]))
    check(*p.step([(0, hi.VERIFY, 1500, 8, tree(hi.MEDUSA_LIKE_TREE)), (1, hi.VERIFY, 333, 8, tree(hi.random_tree(9, 8)))]))
    p.compact(0, 1500, hi.tree_path(hi.MEDUSA_LIKE_TREE, 5)); p.compact(1, 333, [])
    check(*p.step([(0, hi.VERIFY, 1503, 8, tree(hi.random_tree(10, 8))), (1, hi.VERIFY, 333, 5)]))
    p.check_pages([0, 1])
    p.close()


def test_chain_shaped_tree_equals_plain_verify_bit_for_bit():
    import torch
    from paper_2503_18989_amd import Segment
    p = Pair(SMALL64, 43, n_pages=40, max_devices=4, max_step_tokens=256, max_pos=512)
    p.step([(0, hi.CHUNK, 0, 100), (1, hi.CHUNK, 0, 100)], inputs=[hi.hidden_rows(100, 256, 43, 0)] * 2)
    x = to_dev_bf16(hi.hidden_rows(6, 256, 43, 1))
    a, b = p.gpu.forward([Segment(0, hi.VERIFY, 100, x), Segment(1, hi.VERIFY, 100, x.clone(), tree_mask=tree([-1, 0, 1, 2, 3, 4]))])
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    p.close()


@pytest.mark.parametrize("cfg,seed", [(SMALL128, 7), (SMALL64, 8)], ids=["hd128", "hd64"])
def test_randomized_tree_decoding(cfg, seed):
    # 6 devices in the decode phase: every step each submits a random tree (1..8 nodes) or a chain,
    # then a random node's path (or nothing) is kept; sometimes a device leaves and rejoins with a prompt
    rng = np.random.default_rng(seed)
    ndev, max_pos = 6, 1024
    p = Pair(cfg, 95 + seed, n_pages=ndev * max_pos // 16 + 8, max_devices=ndev, max_step_tokens=1024, max_pos=max_pos)
    ln = [0] * ndev
    for step in range(30):
        segs, trees = [], {}
        for d in map(int, rng.permutation(ndev)):
            r = rng.random()
            if ln[d] == 0 or (r < 0.1 and ln[d] + 300 < max_pos):
                n = int(rng.choice([1, 15, 16, 17, 90, 250])); segs.append((d, hi.CHUNK, ln[d], n)); ln[d] += n
            elif r < 0.2:
                p.gpu.release(d); p.ref.release(d); p.pages.release(d); ln[d] = 0
            elif ln[d] + 8 <= max_pos:
                n = int(rng.integers(1, 9))
                if r < 0.35:
                    segs.append((d, hi.VERIFY, ln[d], n)); trees[d] = list(range(-1, n - 1))
                else:
                    trees[d] = hi.random_tree(seed, n, step, d); segs.append((d, hi.VERIFY, ln[d], n, tree(trees[d])))
        if not segs:
            continue
        check(*p.step(segs))
        for d, parents in trees.items():
            node = int(rng.integers(-1, len(parents)))
            keep = hi.tree_path(parents, node) if node >= 0 else []
            p.compact(d, ln[d], keep); ln[d] += len(keep)
        p.check_pages(range(ndev))
        assert [p.gpu.kv_query(d)[0] for d in range(ndev)] == ln
    p.close()


def test_tree_and_compact_errors_are_atomic():
    from paper_2503_18989_amd import HatError, Segment
    p = Pair(hi.TINY, 44, n_pages=6, max_devices=4, max_step_tokens=64, max_pos=100)
    p.step([(0, hi.CHUNK, 0, 20)]); p.step([(0, hi.VERIFY, 20, 4, tree([-1, 0, 0, -1]))])
    snap = [p.gpu.kv_query(d) for d in range(4)]
    x = lambda n: to_dev_bf16(np.zeros((n, 256), np.float32))
    bad = [[0], [3], [1, 2, 7], [1, 3, 6], [1, 1], [1, 2, 0x14]]
    for m in bad:
        with pytest.raises(HatError) as e:
            p.gpu.forward([Segment(1, hi.VERIFY, 0, x(len(m)), tree_mask=m)])
        assert e.value.code == -1, m
        assert [p.gpu.kv_query(d) for d in range(4)] == snap
    with pytest.raises(HatError) as e:                        # a tree on a chunk segment
        p.gpu.forward([Segment(1, hi.CHUNK, 0, x(2), tree_mask=[1, 3])])
    assert e.value.code == -1
    for args in ((9, 20, [0]), (0, 20, [1, 1]), (0, 20, [2, 1]), (0, 20, [-1]), (0, 20, [8]), (0, -1, [0]),
                 (0, 20, [4]), (0, 25, []), (0, 22, [0, 2]), (0, 20, list(range(9)))):
        with pytest.raises(HatError) as e:
            p.gpu.kv_compact(*args)
        with pytest.raises(Exception) as e2:
            p.pages.compact(*args)
        assert e.value.code == e2.value.code, args
        assert [p.gpu.kv_query(d) for d in range(4)] == snap
    p.compact(0, 20, [0, 2]); p.check_pages(range(4))
    check(*p.step([(0, hi.VERIFY, 22, 3)]))
    p.close()


@pytest.mark.parametrize("start", [0, 1, 8, 15, 16, 31])
@pytest.mark.parametrize("kv", ["bf16", "f16"])
def test_verify_over_tiny_caches(start, kv):
    # with almost no prefix the segment's own rows carry all the attention weight, so a row that
    # failed to see them (or saw one too many) is far outside the bar -- a long prefix would hide it
    p = Pair(SMALL64, 45, n_pages=8, max_devices=4, max_step_tokens=64, max_pos=64, kv_dtype=kv)
    if start:
        check(*p.step([(0, hi.CHUNK, 0, start), (1, hi.CHUNK, 0, start)]))
    check(*p.step([(0, hi.VERIFY, start, 8), (1, hi.VERIFY, start, 8, tree(hi.MEDUSA_LIKE_TREE))]), tol=6e-3)
    p.check_pages([0, 1])
    p.close()


def test_tree_steps_fed_from_host_memory():
    # the host-fed entry point carries the tree masks through: same bits as the device-fed call
    import torch
    from paper_2503_18989_amd import Segment
    pa = Pair(SMALL64, 46, n_pages=40, max_devices=4, max_step_tokens=256, max_pos=512)
    pb = Pair(SMALL64, 46, n_pages=40, max_devices=4, max_step_tokens=256, max_pos=512)
    x0 = hi.hidden_rows(50, 256, 46, 0); x1 = hi.hidden_rows(8, 256, 46, 1)
    masks = tree(hi.MEDUSA_LIKE_TREE)
    for p_, host in ((pa, False), (pb, True)):
        f = p_.gpu.forward_host if host else p_.gpu.forward
        mk = (lambda x: to_dev_bf16(x).cpu().pin_memory()) if host else to_dev_bf16
        f([Segment(0, hi.CHUNK, 0, mk(x0))])
        p_.out = f([Segment(0, hi.VERIFY, 50, mk(x1), tree_mask=masks)])[0]
        torch.cuda.synchronize()
    assert torch.equal(pa.out.cpu(), pb.out.cpu())
    pa.close(); pb.close()


def test_long_mixed_run_all_features():
    # 150 steps over 10 devices mixing everything the boundary offers: prompt chunks, chains with
    # rollback, trees with path compaction, departures, and some steps fed from host memory; outputs
    # against the oracle and page state against the page model at every step
    import torch
    from paper_2503_18989_amd import Segment
    rng = np.random.default_rng(99)
    cfg, ndev, max_pos, max_step = SMALL64, 10, 1536, 1024
    p = Pair(cfg, 199, n_pages=ndev * max_pos // 16 // 2, max_devices=ndev, max_step_tokens=max_step, max_pos=max_pos)
    ln = [0] * ndev
    worst = 0.0
    for step in range(150):
        segs, trees, rows = [], {}, 0
        for d in map(int, rng.permutation(ndev)):
            r = rng.random()
            if r < 0.3:
                continue
            if (r < 0.36 and ln[d] > 0) or ln[d] + 300 > max_pos:
                p.gpu.release(d); p.ref.release(d); p.pages.release(d); ln[d] = 0
                continue
            if ln[d] == 0 or r < 0.5:
                n = int(min(rng.choice([3, 16, 31, 64, 130, 256, 290]), max_step - rows))
                if n <= 0:
                    continue
                segs.append((d, hi.CHUNK, ln[d], n)); ln[d] += n
            elif r < 0.75:
                back = int(min(rng.integers(0, 4), ln[d]))
                n = int(min(rng.integers(1, 9), max_step - rows))
                if n <= 0:
                    continue
                segs.append((d, hi.VERIFY, ln[d] - back, n)); ln[d] += n - back
            else:
                n = int(min(rng.integers(1, 9), max_step - rows))
                if n <= 0:
                    continue
                trees[d] = hi.random_tree(199, n, step, d)
                segs.append((d, hi.VERIFY, ln[d], n, hi.tree_masks(trees[d])))
            rows += segs[-1][3]
        if not segs:
            continue
        if step % 5 == 4:     # this step arrives from pinned host memory
            xs = [hi.hidden_rows(sg[3], cfg["d_model"], 199, step, sg[0]) for sg in segs]
            gs = [Segment(sg[0], sg[1], sg[2], to_dev_bf16(x).cpu().pin_memory(), tree_mask=sg[4] if len(sg) > 4 else None)
                  for sg, x in zip(segs, xs)]
            outs = p.gpu.forward_host(gs)
            torch.cuda.synchronize()
            outs = [to_np(o) for o in outs]
            refs = p.ref.forward([(sg[0], sg[2], x, sg[4] if len(sg) > 4 else None) for sg, x in zip(segs, xs)])
            p.pages.step([tuple(sg[:4]) for sg in segs])
        else:
            outs, refs = p.step(segs)
        for o, r_ in zip(outs, refs):
            e = rel_err(o, r_)
            worst = max(worst, e)
            assert np.all(np.isfinite(o)) and e <= TOL, (step, e)
        for d, parents in trees.items():
            node = int(rng.integers(-1, len(parents)))
            keep = hi.tree_path(parents, node) if node >= 0 else []
            p.compact(d, ln[d], keep); ln[d] += len(keep)
        p.check_pages(range(ndev))
        assert [p.gpu.kv_query(d)[0] for d in range(ndev)] == ln
    print("long run: worst rel err %.3e" % worst)
    p.close()
