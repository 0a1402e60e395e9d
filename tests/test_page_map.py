"""The page table's checkpoint field (GPU page -> host page): host bookkeeping, checked against
a dictionary model under seeded random traffic, plus the cases the contract spells out."""
import random

import pytest

from paper_2410_01228_amd import binding as cs


class Model:
    """The same life cycle with dictionaries; host pages are only checked for validity (any
    ascending free run is a correct answer), not predicted."""

    def __init__(self, G, H):
        self.G, self.H = G, H
        self.host_of = {}          # gpu -> host
        self.state = {}            # host -> gpu page, or "evicted"

    def free(self):
        return self.H - len(self.state)


def check_same(m, model):
    assert m.free_host_pages() == model.free()
    for g in range(model.G):
        assert m.host_of(g) == model.host_of.get(g, -1)
    for h in range(model.H):
        want = model.state.get(h, None)
        assert m.gpu_of(h) == (-2 if want is None else -1 if want == "evicted" else want)


def longest_free_run(model):
    best = run = 0
    for h in range(model.H):
        run = run + 1 if h not in model.state else 0
        best = max(best, run)
    return best


@pytest.mark.parametrize("seed", range(6))
def test_random_traffic_against_the_model(seed):
    rnd = random.Random(seed)
    G, H = rnd.choice([(40, 25), (64, 64), (30, 90)])
    m, model = cs.PageMap(G, H), Model(G, H)
    evicted = []                    # host pages waiting for a resume
    for step in range(400):
        op = rnd.choice(["ckpt", "ckpt", "evict", "bind", "drop"])
        if op == "ckpt":
            pages = [rnd.randrange(G) for _ in range(rnd.randint(0, 8))]
            need = []
            for g in pages:
                if g not in model.host_of and g not in need:
                    need.append(g)
            if len(need) > longest_free_run(model):
                with pytest.raises(cs.CsError) as e:
                    m.checkpoint(pages)
                assert e.value.status == cs.CS_ERR_NO_HOST_PAGES
            else:
                dirty, first = m.checkpoint(pages)
                assert dirty == need
                if need:
                    run = list(range(first, first + len(need)))
                    assert all(0 <= h < H and h not in model.state for h in run)   # a free ascending run
                    for g, h in zip(need, run):
                        model.host_of[g] = h
                        model.state[h] = g
                else:
                    assert first == -1
        elif op == "evict":
            pages = rnd.sample(range(G), rnd.randint(0, 6))
            got = m.evict(pages)
            for g, h in zip(pages, got):
                assert h == model.host_of.get(g, -1)
                if h >= 0:
                    del model.host_of[g]
                    model.state[h] = "evicted"
                    evicted.append(h)
        elif op == "bind" and evicted:
            k = rnd.randint(1, min(4, len(evicted)))
            hs = [evicted.pop(rnd.randrange(len(evicted))) for _ in range(k)]
            free_gpu = [g for g in range(G) if g not in model.host_of]
            if len(free_gpu) < k:
                evicted += hs
                continue
            gs = rnd.sample(free_gpu, k)
            m.bind(hs, gs)
            for h, g in zip(hs, gs):
                model.host_of[g] = h
                model.state[h] = g
        elif op == "drop" and model.state:
            hs = rnd.sample(sorted(model.state), rnd.randint(1, min(5, len(model.state))))
            m.drop(hs)
            for h in hs:
                g = model.state.pop(h)
                if g == "evicted":
                    evicted.remove(h)
                else:
                    del model.host_of[g]
        if step % 20 == 0:
            check_same(m, model)
    check_same(m, model)
    m.close()


def test_a_round_takes_one_ascending_run_and_saves_each_page_once():
    m = cs.PageMap(16, 8)
    dirty, first = m.checkpoint([5, 2, 5, 9])
    assert (dirty, first) == ([5, 2, 9], 0)
    assert [m.host_of(g) for g in (5, 2, 9)] == [0, 1, 2]
    # the next round only takes what is new (incremental checkpointing)
    dirty, first = m.checkpoint([5, 2, 9, 11])
    assert (dirty, first) == ([11], 3)
    assert m.checkpoint([5, 11]) == ([], -1)
    assert m.free_host_pages() == 4


def test_no_run_long_enough_changes_nothing():
    m = cs.PageMap(16, 6)
    m.checkpoint([0, 1, 2, 3, 4, 5])
    m.drop([1, 3, 5])                                   # three free pages, no two adjacent
    with pytest.raises(cs.CsError) as e:
        m.checkpoint([10, 11])
    assert e.value.status == cs.CS_ERR_NO_HOST_PAGES
    assert m.host_of(10) == -1 and m.host_of(11) == -1 and m.free_host_pages() == 3
    assert m.checkpoint([10])[0] == [10]                # a single page still fits


def test_the_search_wraps_around_to_freed_pages():
    m = cs.PageMap(16, 6)
    m.checkpoint([0, 1, 2, 3])
    m.drop([0, 1, 2])
    dirty, first = m.checkpoint([7, 8, 9])              # pages 4, 5 are free, but a run of 3 is only at 0
    assert first == 0 and dirty == [7, 8, 9]


def test_evict_then_resume_into_fresh_pages():
    m = cs.PageMap(16, 8)
    m.checkpoint([4, 6, 7])
    assert m.evict([4, 6, 7, 12]) == [0, 1, 2, -1]      # page 12 was never saved: recompute
    assert m.host_of(4) == -1 and m.gpu_of(0) == -1 and m.free_host_pages() == 5
    m.bind([0, 1, 2], [10, 3, 4])
    assert [m.host_of(g) for g in (10, 3, 4)] == [0, 1, 2] and m.gpu_of(2) == 4
    assert m.checkpoint([10, 3, 4]) == ([], -1)         # restored pages need no second save


def test_bind_and_drop_are_all_or_nothing():
    m = cs.PageMap(8, 8)
    m.checkpoint([0, 1, 2])
    m.evict([0, 1])
    with pytest.raises(cs.CsError):
        m.bind([0, 1], [5, 2])                          # GPU page 2 still has a host copy
    assert m.host_of(5) == -1 and m.gpu_of(0) == -1 and m.gpu_of(1) == -1
    with pytest.raises(cs.CsError):
        m.bind([0, 0], [5, 6])                          # the same host page twice
    assert m.host_of(5) == -1 and m.host_of(6) == -1 and m.gpu_of(0) == -1
    with pytest.raises(cs.CsError):
        m.bind([2], [5])                                # host page 2 is tied to GPU page 2, not evicted
    with pytest.raises(cs.CsError):
        m.drop([0, 7])                                  # 7 is free
    assert m.gpu_of(0) == -1 and m.free_host_pages() == 5
    with pytest.raises(cs.CsError):
        m.drop([1, 1])
    assert m.gpu_of(1) == -1 and m.free_host_pages() == 5
    m.drop([0, 2])
    assert m.host_of(2) == -1 and m.free_host_pages() == 7


def test_bad_arguments():
    with pytest.raises(cs.CsError):
        cs.PageMap(0, 4)
    m = cs.PageMap(4, 4)
    with pytest.raises(cs.CsError):
        m.checkpoint([4])
    with pytest.raises(cs.CsError):
        m.evict([-1])
    assert m.host_of(99) == -1 and m.gpu_of(99) == -2
    assert cs.ascending_runs([3, 4, 5, 9, 1, 2]) == [(0, 3), (3, 1), (4, 2)]
    assert cs.ascending_runs([]) == []
