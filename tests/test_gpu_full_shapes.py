"""GPU parity at the full widths of the benchmark configurations.

The oracle cannot run whole 30/38-layer workloads in test time, so each case
either (a) runs the oracle on a sample it can afford -- reduced depth at full
width, or a subset of the devices of a step (segments never interact, so the
oracle may follow any subset while the GPU processes the whole batch) -- or
(b) checks a property that holds at any size (chunk-split invariance at full
depth, integer page state against the page model at every step).
Tolerance: max|gpu - ref| / max|ref| per segment <= 2e-2 at full depth (30 layers) and <= 6e-3 for
the 1- and 2-layer models (gpu_util.tol_for_depth: a shallow stack sits near the bf16 output rounding,
so the full-depth bar would let a kernel-sized error pass there).  The same workloads at their full
depth are in test_gpu_depth.py."""
import numpy as np
import pytest

import hat_inputs as hi
from gpu_util import added_err, progress, rel_err, rel_l2, to_dev_bf16, to_np, dev_weights, tol_for_depth

pytestmark = pytest.mark.gpu
TOL = 2e-2                      # full depth
TOL_SHALLOW = tol_for_depth(2)  # 1- and 2-layer models


def build(cfg, seed, n_pages, weights=None, **kw):
    from concurrent.futures import ThreadPoolExecutor
    from paper_2503_18989_amd import HatMid
    if weights is None:
        with ThreadPoolExecutor(max_workers=16) as ex:
            weights = list(ex.map(lambda l: hi.layer_weights(cfg, l, seed), range(cfg["n_layers"])))
    gpu = HatMid(cfg, [dev_weights(w) for w in weights], n_pages=n_pages, **kw)
    return gpu, weights


def device_random_kv(n, H, hd, seed):
    import torch
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    k = (torch.randn((n, H, hd), generator=g, device="cuda") * 1.28).to(torch.bfloat16)
    v = (torch.randn((n, H, hd), generator=g, device="cuda") * 1.28).to(torch.bfloat16)
    return k, v


def check(o, r, what="", tol=TOL_SHALLOW):
    assert np.all(np.isfinite(o)), what
    e = rel_err(o, r)
    assert e <= tol, "%s rel err %.3e (l2 %.3e)" % (what, e, rel_l2(o, r))
    return e


def test_cfg2_7b_two_layers_all_chunks():
    """Full width, 2 layers: all 8 chunks of the 2048-row prompt against the oracle."""
    import torch
    from oracle import OracleMiddle, PageModel
    from paper_2503_18989_amd import Segment
    cfg = hi.with_layers(hi.MID7B, 2)
    seed = 2000
    gpu, weights = build(cfg, seed, n_pages=2048 // 16 + 8, max_devices=2, max_step_tokens=256, max_pos=2048)
    ref = OracleMiddle(cfg, weights)
    pm = PageModel(2048 // 16 + 8, max_devices=2, max_step_tokens=256, max_pos=2048)
    worst = 0.0
    for i, step in enumerate(hi.single_prompt_schedule()):
        dev, kind, start, n = step[0]
        x = hi.hidden_rows(n, cfg["d_model"], seed, i)
        y = to_np(gpu.forward([Segment(dev, kind, start, to_dev_bf16(x))])[0])
        torch.cuda.synchronize()
        worst = max(worst, check(y, ref.forward([(dev, start, x)])[0], "chunk %d" % i))
        pm.step(step)
        assert gpu.kv_query(0) == pm.query(0)
    progress("cfg2 2 layers: worst rel err %.3e" % worst)
    gpu.close()


def test_cfg3_7b_mixed_step_sampled_devices():
    """30 devices, prefixes U[256,4096] installed by import, one mixed step (10 chunks from
    {128,256,512} + 20 verify segments of 5 rows); the oracle follows 3 chunk devices and
    4 verify devices, the page model all 30."""
    import torch
    from oracle import OracleMiddle, PageModel
    from paper_2503_18989_amd import Segment
    cfg = hi.with_layers(hi.MID7B, 2)
    seed = 3000
    H, hd, d = cfg["n_heads"], cfg["head_dim"], cfg["d_model"]
    pref = hi.mixed_prefixes(seed)
    segs = hi.mixed_step(seed, 0, pref)
    T = sum(s[3] for s in segs)
    n_pages = sum((p + s[3] + 15) // 16 for p, s in zip(pref, segs)) + 32
    gpu, weights = build(cfg, seed, n_pages=n_pages, max_devices=30, max_step_tokens=T, max_pos=8192)
    ref = OracleMiddle(cfg, weights)
    pm = PageModel(n_pages, max_devices=30, max_step_tokens=8192, max_pos=8192)
    chunk_devs = [s[0] for s in segs if s[1] == hi.CHUNK]
    verify_devs = [s[0] for s in segs if s[1] == hi.VERIFY]
    sampled = set(sorted(chunk_devs, key=lambda dv: segs[dv][3])[:2] + chunk_devs[-1:] + verify_devs[:4])
    for dev in range(30):
        pm.step([(dev, 0, 0, pref[dev])])
        for l in range(cfg["n_layers"]):
            if dev in sampled:
                k, v = hi.kv_prefix(pref[dev], H, hd, seed, dev, l)
                gpu.kv_import(dev, l, 0, to_dev_bf16(k).view(-1, H, hd), to_dev_bf16(v).view(-1, H, hd))
                ref.import_kv(dev, l, 0, k, v)
            else:
                k, v = device_random_kv(pref[dev], H, hd, seed * 100 + dev * 4 + l)
                gpu.kv_import(dev, l, 0, k, v)
        assert gpu.kv_query(dev) == pm.query(dev)
    xs = [hi.hidden_rows(s[3], d, seed, s[0]) for s in segs]
    outs = gpu.forward([Segment(s[0], s[1], s[2], to_dev_bf16(x)) for s, x in zip(segs, xs)])
    torch.cuda.synchronize()
    pm.step(segs)
    for dev in range(30):
        assert gpu.kv_query(dev) == pm.query(dev)
    refs = ref.forward([(s[0], s[2], x) for s, x in zip(segs, xs) if s[0] in sampled])
    got = [to_np(o) for s, o in zip(segs, outs) if s[0] in sampled]
    worst = max(check(o, r, "device") for o, r in zip(got, refs))
    for o in outs:
        assert torch.isfinite(o.float()).all()
    progress("cfg3 2 layers: T=%d, sampled %d segments, worst rel err %.3e" % (T, len(refs), worst))
    gpu.close()


def test_cfg4_7b_verify_heavy_64_steps_with_rollback():
    """30 devices x 5 draft rows per step, cache lengths U[1024,8192], 64 steps with the
    seeded accept/rollback pattern.  Page ids, slots and lengths of all 30 devices are
    compared with the page model after every step; the oracle follows 3 devices through
    all 64 steps (outputs compared at every step, so drift after 63 rollbacks shows)."""
    import torch
    from oracle import OracleMiddle, PageModel
    from paper_2503_18989_amd import Segment
    cfg = hi.with_layers(hi.MID7B, 2)
    seed = 4000
    H, hd, d = cfg["n_heads"], cfg["head_dim"], cfg["d_model"]
    lengths = hi.verify_lengths(seed)
    sched = hi.verify_schedule(seed, lengths, steps=64)
    n_pages = sum((ln + 64 * 5 + 15) // 16 for ln in lengths) + 32
    gpu, weights = build(cfg, seed, n_pages=n_pages, max_devices=30, max_step_tokens=256, max_pos=8192 + 64 * 5 + 16)
    ref = OracleMiddle(cfg, weights)
    pm = PageModel(n_pages, max_devices=30, max_step_tokens=16384, max_pos=8192 + 64 * 5 + 16)
    order = np.argsort(lengths)
    sampled = {int(order[0]), int(order[15]), int(order[-1])}      # shortest, median, longest cache
    for dev in range(30):
        pm.step([(dev, 0, 0, lengths[dev])])
        for l in range(cfg["n_layers"]):
            if dev in sampled:
                k, v = hi.kv_prefix(lengths[dev], H, hd, seed, dev, l)
                gpu.kv_import(dev, l, 0, to_dev_bf16(k).view(-1, H, hd), to_dev_bf16(v).view(-1, H, hd))
                ref.import_kv(dev, l, 0, k, v)
            else:
                k, v = device_random_kv(lengths[dev], H, hd, seed * 100 + dev * 4 + l)
                gpu.kv_import(dev, l, 0, k, v)
    worst = 0.0
    for it, step in enumerate(sched):
        xs = [hi.hidden_rows(5, d, seed, it, s[0]) for s in step]
        outs = gpu.forward([Segment(s[0], s[1], s[2], to_dev_bf16(x)) for s, x in zip(step, xs)])
        torch.cuda.synchronize()
        pm.step(step)
        for dev in range(30):
            assert gpu.kv_query(dev) == pm.query(dev), "step %d device %d" % (it, dev)
        refs = ref.forward([(s[0], s[2], x) for s, x in zip(step, xs) if s[0] in sampled])
        got = [to_np(o) for s, o in zip(step, outs) if s[0] in sampled]
        for o, r in zip(got, refs):
            worst = max(worst, check(o, r, "step %d" % it))
    progress("cfg4 2 layers: 64 steps, worst rel err %.3e" % worst)
    gpu.close()


def test_tree_decoding_7b_30_devices_16_steps():
    """The verify-heavy shape with trees (Sec. 2.2 / 4.1: 8 candidates per step): 30 devices,
    cache lengths U[1024,8192]; every step each device submits a seeded random tree of 8 and then
    keeps a seeded random path of it (or nothing).  Page state of all 30 devices against the page
    model after every step and every compaction; the oracle follows 3 devices through all steps."""
    import torch
    from oracle import OracleMiddle, PageModel
    from paper_2503_18989_amd import Segment
    cfg = hi.with_layers(hi.MID7B, 2)
    seed = 4100
    H, hd, d = cfg["n_heads"], cfg["head_dim"], cfg["d_model"]
    lengths = list(hi.verify_lengths(seed))
    steps = 16
    n_pages = sum((ln + steps * 8 + 15) // 16 for ln in lengths) + 32
    max_pos = 8192 + steps * 8 + 16
    gpu, weights = build(cfg, seed, n_pages=n_pages, max_devices=30, max_step_tokens=256, max_pos=max_pos)
    ref = OracleMiddle(cfg, weights)
    pm = PageModel(n_pages, max_devices=30, max_step_tokens=16384, max_pos=max_pos)
    order = np.argsort(lengths)
    sampled = {int(order[0]), int(order[15]), int(order[-1])}
    for dev in range(30):
        pm.step([(dev, 0, 0, lengths[dev])])
        for l in range(cfg["n_layers"]):
            if dev in sampled:
                k, v = hi.kv_prefix(lengths[dev], H, hd, seed, dev, l)
                gpu.kv_import(dev, l, 0, to_dev_bf16(k).view(-1, H, hd), to_dev_bf16(v).view(-1, H, hd))
                ref.import_kv(dev, l, 0, k, v)
            else:
                k, v = device_random_kv(lengths[dev], H, hd, seed * 100 + dev * 4 + l)
                gpu.kv_import(dev, l, 0, k, v)
    rng = np.random.default_rng(seed)
    worst = 0.0
    for it in range(steps):
        trees = [hi.random_tree(seed, 8, it, dev) for dev in range(30)]
        xs = [hi.hidden_rows(8, d, seed, it, dev) for dev in range(30)]
        outs = gpu.forward([Segment(dev, hi.VERIFY, lengths[dev], to_dev_bf16(xs[dev]), tree_mask=hi.tree_masks(trees[dev]))
                            for dev in range(30)])
        torch.cuda.synchronize()
        pm.step([(dev, hi.VERIFY, lengths[dev], 8) for dev in range(30)])
        refs = ref.forward([(dev, lengths[dev], xs[dev], hi.tree_masks(trees[dev])) for dev in sorted(sampled)])
        for dev, r in zip(sorted(sampled), refs):
            worst = max(worst, check(to_np(outs[dev]), r, "step %d device %d" % (it, dev)))
        for dev in range(30):
            node = int(rng.integers(-1, 8))
            keep = hi.tree_path(trees[dev], node) if node >= 0 else []
            gpu.kv_compact(dev, lengths[dev], keep)
            pm.compact(dev, lengths[dev], keep)
            if dev in sampled:
                ref.compact(dev, lengths[dev], keep)
            lengths[dev] += len(keep)
        torch.cuda.synchronize()
        for dev in range(30):
            assert gpu.kv_query(dev) == pm.query(dev), "step %d device %d" % (it, dev)
    progress("tree decoding 2 layers: %d steps, worst rel err %.3e" % (steps, worst))
    gpu.close()


@pytest.mark.parametrize("chunk", [64, 128, 256, 512, 1024])
def test_cfg5_13b_last_chunk_of_each_size(chunk):
    """13B width (d 5120, 40 heads, FFN 13824), 2 layers: 8 devices with 8192-row prompts,
    the LAST chunk of each chunk size batched over the 8 devices (T = 8*chunk rows, prefix
    8192-chunk installed by import); the oracle follows one device."""
    import torch
    from oracle import OracleMiddle
    from paper_2503_18989_amd import Segment
    cfg = hi.with_layers(hi.MID13B, 2)
    seed = 5000
    H, hd, d = cfg["n_heads"], cfg["head_dim"], cfg["d_model"]
    start = 8192 - chunk
    n_pages = 8 * (8192 // 16) + 16
    gpu, weights = build(cfg, seed, n_pages=n_pages, max_devices=8, max_step_tokens=8 * chunk, max_pos=8192)
    ref = OracleMiddle(cfg, weights)
    for dev in range(8):
        for l in range(2):
            if dev == 3:
                k, v = hi.kv_prefix(start, H, hd, seed, dev, l)
                gpu.kv_import(dev, l, 0, to_dev_bf16(k).view(-1, H, hd), to_dev_bf16(v).view(-1, H, hd))
                ref.import_kv(dev, l, 0, k, v)
            else:
                k, v = device_random_kv(start, H, hd, seed * 100 + dev * 4 + l)
                gpu.kv_import(dev, l, 0, k, v)
    xs = [hi.hidden_rows(chunk, d, seed, chunk, dev) for dev in range(8)]
    outs = gpu.forward([Segment(dev, hi.CHUNK, start, to_dev_bf16(xs[dev])) for dev in range(8)])
    torch.cuda.synchronize()
    for dev in range(8):
        assert gpu.kv_query(dev)[0] == 8192 and torch.isfinite(outs[dev].float()).all()
    y = ref.forward([(3, start, xs[3])])[0]
    e = check(to_np(outs[3]), y, "chunk %d" % chunk)
    progress("cfg5 2 layers, chunk %d: rel err %.3e" % (chunk, e))
    gpu.close()


def test_widest_model_the_library_accepts():
    """d_model = 8192 (64 heads x 128), the upper limit of the configuration check: one layer, a 70-row
    chunk, then a chain and a tree over it."""
    import torch
    from oracle import OracleMiddle
    from paper_2503_18989_amd import Segment
    cfg = dict(name="wide", n_layers=1, d_model=8192, n_heads=64, head_dim=128, d_ffn=2048, rms_eps=1e-6, rope_theta=1e4)
    seed = 6000
    gpu, weights = build(cfg, seed, n_pages=32, max_devices=2, max_step_tokens=128, max_pos=256)
    ref = OracleMiddle(cfg, weights)
    x0 = hi.hidden_rows(70, 8192, seed, 0); x1 = hi.hidden_rows(8, 8192, seed, 1); x2 = hi.hidden_rows(5, 8192, seed, 2)
    steps = [[(0, hi.CHUNK, 0, x0, None)], [(0, hi.VERIFY, 70, x1, hi.tree_masks(hi.MEDUSA_LIKE_TREE))], [(0, hi.VERIFY, 70, x2, None)]]
    for st in steps:
        outs = gpu.forward([Segment(d, k, s, to_dev_bf16(x), tree_mask=m) for d, k, s, x, m in st])
        torch.cuda.synchronize()
        refs = ref.forward([(d, s, x, m) for d, k, s, x, m in st])
        for o, r in zip(outs, refs):
            check(to_np(o), r, "d_model 8192")
    gpu.close()
