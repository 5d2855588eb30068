"""The library's own planner on the CPU (no GPU): validation, page bookkeeping, rotary positions,
write targets and attention work lists of hat_mid_forward, through a host-only handle.

Integer work: everything is compared exactly -- pages, lengths and write targets against the
independent page model of oracle/, positions against the definition (start + row, or start + depth
for a tree), and the work lists against what the kernels assume of them."""
import numpy as np
import pytest

import hat_inputs as hi
from oracle.page_model import PageModel, PageModelError
from paper_2503_18989_amd import HatError, HatPlanner

SHAPE = dict(hi.MID7B)        # only the head count and head size matter to the planner


def both(n_pages, **kw):
    return HatPlanner(SHAPE, n_pages, **kw), PageModel(n_pages, 16, kw.get("max_devices", 64), kw.get("max_step_tokens", 8192),
                                                       kw.get("max_pos", 16384))


def check_items(plan, segs, part_rows_seen):
    """Properties the attention kernels rely on."""
    tok0 = np.cumsum([0] + [sg[3] for sg in segs])
    by_seg_c, by_seg_v = {}, {}
    for it in plan["chunk_items"]:
        by_seg_c.setdefault((it["seg"], it["q0"]), []).append(it)
    for it in plan["verify_items"]:
        by_seg_v.setdefault(it["seg"], []).append(it)
    merges = {m["row0"]: m for m in plan["merge_items"]}
    for i, sg in enumerate(segs):
        dev, kind, start, n = sg[:4]
        if kind == hi.CHUNK:
            assert i not in by_seg_v
            for q0 in range(0, n, 256):
                nq = min(256, n - q0)
                items = sorted(by_seg_c[(i, q0)], key=lambda it: it["kv_begin"])
                need = start + q0 + nq
                assert items[0]["kv_begin"] == 0 and items[-1]["kv_end"] == need
                for a, b in zip(items, items[1:]):
                    assert a["kv_end"] == b["kv_begin"]
                for k, it in enumerate(items):
                    assert it["kv_begin"] % 64 == 0 and it["kv_begin"] < it["kv_end"]
                    assert (it["nq"], it["start"], it["tok0"], it["kv_len"]) == (nq, start, tok0[i], start + n)
                    if len(items) == 1:
                        assert it["part_row"] == -1
                    else:
                        assert it["part_row"] == items[0]["part_row"] + k * nq
                        part_rows_seen.append((it["part_row"], nq))
                if len(items) > 1:
                    covered = 0
                    for g0 in range(0, nq, 16):           # merged in groups of at most 16 rows
                        m = merges[tok0[i] + q0 + g0]
                        assert (m["nsplit"], m["stride"], m["part_row"]) == (len(items), nq, items[0]["part_row"] + g0)
                        covered += m["nrows"]
                    assert covered == nq
        else:
            assert not any(s_ == i for s_, _ in by_seg_c)
            items = sorted(by_seg_v[i], key=lambda it: it["kv_begin"])
            ln = start + n
            assert items[0]["kv_begin"] == 0 and items[-1]["kv_end"] == ln
            for a, b in zip(items, items[1:]):
                assert a["kv_end"] == b["kv_begin"]
            masks = sg[4] if len(sg) > 4 and sg[4] is not None else [(2 << r) - 1 for r in range(n)]
            for k, it in enumerate(items):
                assert it["kv_begin"] % 64 == 0 and it["kv_begin"] < it["kv_end"] and it["q0"] == 0
                assert (it["nq"], it["start"], it["tok0"], it["kv_len"]) == (n, start, tok0[i], ln)
                vis = it["vis_lo"] | (it["vis_hi"] << 32)
                assert [(vis >> (8 * r)) & 0xFF for r in range(n)] == list(masks) and vis >> (8 * n) == 0
                if len(items) == 1:
                    assert it["part_row"] == -1
                else:
                    assert it["part_row"] == items[0]["part_row"] + k * n
                    part_rows_seen.append((it["part_row"], n))
            if len(items) > 1:
                m = merges[tok0[i]]
                assert (m["nrows"], m["nsplit"], m["stride"], m["part_row"]) == (n, len(items), n, items[0]["part_row"])


def disjoint(part_rows):
    spans = sorted(part_rows)
    for (a, na), (b, _) in zip(spans, spans[1:]):
        assert a + na <= b, "partial rows overlap"


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_traffic_pages_targets_positions_and_work_lists(seed):
    rng = np.random.default_rng(seed)
    ndev, max_pos, max_step = 12, 6000, 4096
    lib, pm = both(ndev * max_pos // 16 // 2, max_devices=ndev, max_step_tokens=max_step, max_pos=max_pos)
    ln = [0] * ndev
    for step in range(120):
        segs, trees, rows = [], {}, 0
        for d in map(int, rng.permutation(ndev)):
            r = rng.random()
            if r < 0.3:
                continue
            if (r < 0.36 and ln[d] > 0) or ln[d] + 1100 > max_pos:
                lib.release(d); pm.release(d); ln[d] = 0
                continue
            if ln[d] == 0 or r < 0.55:
                n = int(min(rng.choice([1, 15, 16, 17, 100, 255, 256, 257, 512, 700, 1024]), max_step - rows))
                if n <= 0:
                    continue
                segs.append((d, hi.CHUNK, ln[d], n)); ln[d] += n
            elif r < 0.8:
                back = int(min(rng.integers(0, 6), ln[d]))
                n = int(min(rng.integers(1, 9), max_step - rows))
                if n <= 0:
                    continue
                segs.append((d, hi.VERIFY, ln[d] - back, n)); ln[d] += n - back
            else:
                n = int(min(rng.integers(1, 9), max_step - rows))
                if n <= 0:
                    continue
                trees[d] = hi.random_tree(seed, n, step, d)
                segs.append((d, hi.VERIFY, ln[d], n, hi.tree_masks(trees[d])))
            rows += segs[-1][3]
        if not segs:
            continue
        plan = lib.plan(segs)
        targets = pm.step([tuple(sg[:4]) for sg in segs])
        want_dst = [pg * 16 + slot for tg in targets for pg, slot in tg]
        assert plan["kv_dst"] == want_dst
        want_pos = []
        for sg in segs:
            if len(sg) > 4:
                want_pos += [sg[2] + bin(m).count("1") - 1 for m in sg[4]]
            else:
                want_pos += list(range(sg[2], sg[2] + sg[3]))
        assert plan["pos"] == want_pos
        part_rows = []
        check_items(plan, segs, part_rows)
        disjoint(part_rows)
        for d, parents in trees.items():
            node = int(rng.integers(-1, len(parents)))
            keep = hi.tree_path(parents, node) if node >= 0 else []
            lib.kv_compact(d, ln[d], keep); pm.compact(d, ln[d], keep); ln[d] += len(keep)
        for d in range(ndev):
            assert lib.kv_query(d) == pm.query(d), (step, d)
    lib.close()


def test_errors_match_the_page_model_and_change_nothing():
    lib, pm = both(4, max_devices=4, max_step_tokens=64, max_pos=100)
    lib.plan([(0, 0, 0, 20)]); pm.step([(0, 0, 0, 20)])
    snap = [lib.kv_query(d) for d in range(4)]
    cases = [[(0, 0, 21, 4)], [(1, 0, 1, 4)], [(0, 0, 20, 4), (0, 0, 24, 4)], [(4, 0, 0, 4)], [(-1, 0, 0, 4)],
             [(1, 1, 0, 9)], [(1, 0, 0, 65)], [(0, 0, 20, 81)], [(0, 0, 10, 4), (1, 0, 0, 49)], [(1, 2, 0, 4)], [(1, 0, 0, 0)]]
    for segs in cases:
        with pytest.raises(HatError) as e:
            lib.plan(segs)
        with pytest.raises(PageModelError) as e2:
            pm.step(segs)
        assert e.value.code == e2.value.code, segs
        assert [lib.kv_query(d) for d in range(4)] == snap
    for masks in ([0], [3], [1, 2, 7], [1, 3, 6], [1, 1]):
        with pytest.raises(HatError) as e:
            lib.plan([(1, 1, 0, len(masks), masks)])
        assert e.value.code == -1 and [lib.kv_query(d) for d in range(4)] == snap
    with pytest.raises(HatError) as e:
        lib.plan([(1, 0, 0, 2, [1, 3])])          # a tree on a chunk segment
    assert e.value.code == -1
    plan = lib.plan([(0, 0, 10, 4), (1, 0, 0, 48)]); pm.step([(0, 0, 10, 4), (1, 0, 0, 48)])   # exactly fills the pool
    assert [lib.kv_query(d) for d in range(4)] == [pm.query(d) for d in range(4)]
    assert lib.plan([]) == dict(pos=[], kv_dst=[], chunk_items=[], verify_items=[], merge_items=[])
    lib.close()


@pytest.mark.parametrize("which", ["mixed", "verify", "sweep"])
def test_benchmark_shaped_steps_fit_every_capacity(which):
    # the largest steps the benchmark configurations produce: the plan must fit its buffers (a plan
    # that did not would be rejected with an internal error) and obey the work-list properties
    if which == "mixed":
        pref = hi.mixed_prefixes(3003)
        segs = [(d, k, p, n) for (d, k, p, n) in hi.mixed_step(3003, 0, pref)]
        pre = [(d, hi.CHUNK, 0, p) for d, p in enumerate(pref)]
        lib, pm = both(sum((p + 600) // 16 + 1 for p in pref) + 64, max_devices=32, max_step_tokens=8192, max_pos=8192)
    elif which == "verify":
        lengths = hi.verify_lengths(4004)
        pre = [(d, hi.CHUNK, 0, ln) for d, ln in enumerate(lengths)]
        segs = [(d, hi.VERIFY, ln, 8, hi.tree_masks(hi.MEDUSA_LIKE_TREE)) for d, ln in enumerate(lengths)]
        lib, pm = both(sum((ln + 8) // 16 + 1 for ln in lengths) + 64, max_devices=32, max_step_tokens=8192, max_pos=8192 + 64)
    else:
        pre = [(d, hi.CHUNK, 0, 7168) for d in range(8)]
        segs = [(d, hi.CHUNK, 7168, 1024) for d in range(8)]
        lib, pm = both(8 * 8192 // 16 + 8, max_devices=8, max_step_tokens=8192, max_pos=8192)
    for sg in pre:                                   # prefixes, one device per step (each fits max_step_tokens)
        lib.plan([sg]); pm.step([sg])
    plan = lib.plan(segs); pm.step([tuple(sg[:4]) for sg in segs])
    part_rows = []
    check_items(plan, segs, part_rows)
    disjoint(part_rows)
    assert [lib.kv_query(sg[0]) for sg in segs] == [pm.query(sg[0]) for sg in segs]
    lib.close()


def test_plan_capacity_failure_undoes_the_page_movements():
    # the "plan exceeds capacity" failure is only found after the step's rollbacks and allocations have
    # been made: every length, page list and the free set must come back exactly, and the handle must
    # carry on as if the failed call had never happened (compared with a planner that never saw it)
    a, pm = both(64, max_devices=4, max_step_tokens=256, max_pos=512)
    b = HatPlanner(SHAPE, 64, max_devices=4, max_step_tokens=256, max_pos=512)
    first = [(0, hi.CHUNK, 0, 100), (1, hi.CHUNK, 0, 40), (2, hi.CHUNK, 0, 33)]
    for h in (a, b):
        h.plan(first)
    pm.step(first)
    snap = [a.kv_query(d) for d in range(4)]
    # rolls device 0 back over three pages, extends device 1, restarts device 2, admits device 3
    step = [(0, hi.VERIFY, 60, 5), (1, hi.CHUNK, 40, 100), (2, hi.CHUNK, 0, 20), (3, hi.CHUNK, 0, 50)]
    a.limit_plan(8)
    with pytest.raises(HatError) as e:
        a.plan(step)
    assert e.value.code == -1 and "capacity" in str(e.value)
    assert [a.kv_query(d) for d in range(4)] == snap
    a.limit_plan(0)
    pa, pb = a.plan(step), b.plan(step)
    pm.step(step)
    assert pa == pb
    for d in range(4):
        assert a.kv_query(d) == b.kv_query(d) == pm.query(d)
    # the free set is intact as well: the next allocations take the same lowest ids on both
    nxt = [(3, hi.CHUNK, 50, 200), (0, hi.VERIFY, 65, 8)]
    assert a.plan(nxt) == b.plan(nxt)
    pm.step(nxt)
    for d in range(4):
        assert a.kv_query(d) == b.kv_query(d) == pm.query(d)
    a.close(); b.close()
