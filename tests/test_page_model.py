"""Pins for oracle/page_model.py: hand-computed tables and policy properties."""
import random

import pytest

import hat_inputs as hi
from oracle.page_model import PageModel, PageModelError, EINVAL, ENOMEM, EPOS, EDUP, EDEVICE


def test_tiny_schedule_hand_table():
    pm = PageModel(n_pages=8)
    want_len = [16, 32, 48, 64, 68, 70, 74]
    want_pages = [[0], [0, 1], [0, 1, 2], [0, 1, 2, 3], [0, 1, 2, 3, 4], [0, 1, 2, 3, 4], [0, 1, 2, 3, 4]]
    for step, L, P in zip(hi.tiny_schedule(), want_len, want_pages):
        tg = pm.step(step)
        assert pm.query(0) == (L, P)
        dev, kind, start, n = step[0]
        assert tg[0] == [(P[q // 16], q % 16) for q in range(start, start + n)]


def test_two_devices_interleave_and_lowest_free_id():
    pm = PageModel(n_pages=8)
    pm.step([(3, 0, 0, 20), (1, 0, 0, 5)])           # dev3 takes 0,1 ; dev1 takes 2
    assert pm.query(3) == (20, [0, 1]) and pm.query(1) == (5, [2])
    pm.step([(1, 0, 5, 30)])                          # dev1 grows to 35 -> pages 2,3,4
    assert pm.query(1) == (35, [2, 3, 4])
    pm.release(3)                                     # frees 0,1
    pm.step([(5, 1, 0, 8), (1, 1, 17, 8)])            # dev1 rolls back to 17 (frees 4) before dev5 allocates
    assert pm.query(5) == (8, [0]) and pm.query(1) == (25, [2, 3])
    pm.step([(1, 0, 25, 40)])                         # 65 tokens -> 5 pages: 2,3 + lowest free 1,4,5
    assert pm.query(1) == (65, [2, 3, 1, 4, 5])


def test_rollback_frees_precede_allocations_of_the_same_step():
    pm = PageModel(n_pages=4)
    pm.step([(0, 0, 0, 48)]); pm.step([(1, 0, 0, 16)])        # pool full: dev0 0,1,2 ; dev1 3
    # dev1 (listed first) needs a page that only dev0's rollback (listed second) frees
    pm.step([(1, 0, 16, 16), (0, 1, 30, 2)])
    assert pm.query(1) == (32, [3, 2]) and pm.query(0) == (32, [0, 1])


def test_errors_leave_state_untouched():
    pm = PageModel(n_pages=4, max_devices=4, max_step_tokens=64, max_pos=100)
    pm.step([(0, 0, 0, 20)])
    snap = (pm.query(0), set(pm.free))
    for segs, code in [
        ([(0, 0, 21, 4)], EPOS), ([(1, 0, 1, 4)], EPOS),
        ([(0, 0, 20, 4), (0, 0, 24, 4)], EDUP),
        ([(4, 0, 0, 4)], EDEVICE), ([(-1, 0, 0, 4)], EDEVICE),
        ([(1, 1, 0, 9)], EINVAL), ([(1, 0, 0, 0)], EINVAL), ([(1, 0, 0, 65)], EINVAL),
        ([(0, 0, 20, 81)], EINVAL),                       # beyond max_pos
        ([(0, 0, 10, 4), (1, 0, 0, 49)], ENOMEM),         # 10+4 -> 1 page, 49 -> 4 pages > 3 free after rollback
    ]:
        with pytest.raises(PageModelError) as e:
            pm.step(segs)
        assert e.value.code == code
        assert (pm.query(0), set(pm.free)) == snap
    pm.step([(0, 0, 10, 4), (1, 0, 0, 48)])               # exactly fits
    assert pm.query(0) == (14, [0]) and pm.query(1) == (48, [1, 2, 3])


def test_policy_properties_under_random_traffic():
    rnd = random.Random(1234)
    pm = PageModel(n_pages=40, max_devices=6, max_step_tokens=200)
    for it in range(600):
        if rnd.random() < 0.08:
            pm.release(rnd.randrange(6)); continue
        devs = rnd.sample(range(6), rnd.randint(1, 4))
        segs = []
        for d in devs:
            L = pm.query(d)[0]
            start = rnd.randint(max(0, L - 6), L + (1 if rnd.random() < 0.05 else 0))
            kind = rnd.randint(0, 1)
            n = rnd.randint(1, 8 if kind else 60)
            segs.append((d, kind, start, n))
        before_free = set(pm.free); before = {d: pm.query(d) for d in range(6)}
        try:
            tg = pm.step(segs)
        except PageModelError:
            assert set(pm.free) == before_free and all(pm.query(d) == before[d] for d in range(6))
            continue
        owned = [p for d in range(6) for p in pm.query(d)[1]]
        assert len(owned) == len(set(owned)) and set(owned).isdisjoint(pm.free)
        assert set(owned) | pm.free == set(range(40))
        # replay the policy by hand: frees first, then lowest-id allocation in array order
        free = set(before_free)
        for d, kind, start, n in segs:
            keep = -(-start // 16)
            free |= set(before[d][1][keep:])
        for (d, kind, start, n), t in zip(segs, tg):
            L, P = pm.query(d)
            assert L == start + n and len(P) == -(-L // 16)
            keep = -(-start // 16)
            assert P[:keep] == before[d][1][:keep]
            for newp in P[keep:]:
                assert newp == min(free); free.remove(newp)
            assert t == [(P[q // 16], q % 16) for q in range(start, start + n)]
        assert free == pm.free


def test_compact_hand_table():
    pm = PageModel(n_pages=8)
    pm.step([(0, 0, 0, 28)])                          # pages 0,1
    pm.step([(0, 1, 28, 8)])                          # tree of 8 at 28..35 -> pages 0,1,2
    assert pm.query(0) == (36, [0, 1, 2])
    moves = pm.compact(0, 28, [1, 4, 6])              # rows 29, 32, 34 -> 28, 29, 30
    assert moves == [((1, 13), (1, 12)), ((2, 0), (1, 13)), ((2, 2), (1, 14))]
    assert pm.query(0) == (31, [0, 1]) and 2 in pm.free
    pm.step([(1, 0, 0, 1)])                           # the freed page is the lowest free one again
    assert pm.query(1) == (1, [2])
    assert pm.compact(0, 31, []) == [] and pm.query(0) == (31, [0, 1])
    assert pm.compact(0, 16, []) == [] and pm.query(0) == (16, [0])   # an empty keep list is a rollback


def test_compact_errors_leave_state_untouched():
    pm = PageModel(n_pages=8, max_devices=4)
    pm.step([(0, 0, 0, 20)]); pm.step([(0, 1, 20, 4)])
    snap = (pm.query(0), set(pm.free))
    for args, code in (((9, 20, [0]), EDEVICE), ((0, 20, [1, 1]), EINVAL), ((0, 20, [2, 1]), EINVAL),
                       ((0, 20, [-1]), EINVAL), ((0, 20, [8]), EINVAL), ((0, -1, [0]), EINVAL),
                       ((0, 20, [4]), EPOS), ((0, 25, []), EPOS), ((0, 22, [0, 2]), EPOS)):
        with pytest.raises(PageModelError) as e:
            pm.compact(*args)
        assert e.value.code == code, args
        assert (pm.query(0), set(pm.free)) == snap
    assert pm.compact(1, 0, []) == [] and pm.query(1) == (0, [])      # unknown device, nothing kept: no-op
