"""Host logic of the planned causal launches (no GPU): the lists the library gives the workgroups.

What is fixed independently of the planner: every work item appears exactly once; an item stays on its XCD class
(index % 8); the reported loads are the sums of the stated item costs (twice the key tiles an item's last row sees,
plus 4); on small cases the largest load is the optimum found by brute force; a plan is used only where it beats
dispatch in index order by 3 %."""
import itertools

import pytest

import paper_2503_01873_amd as P


def _query_tile(i, nqt, G, ngroups):
    """Query tile of work item i as the attention kernel decodes it (items are numbered longest first per XCD)."""
    if ngroups % 8 == 0:
        return nqt - 1 - (i >> 3) // ((ngroups >> 3) * G)
    if 8 % ngroups == 0 and (nqt * G) % (8 // ngroups) == 0:
        span = 8 // ngroups
        return nqt - 1 - ((i >> 3) * span + ((i & 7) % span)) // G
    return nqt - 1 - i // (ngroups * G)


def _costs(B, Hq, Hkv, Nq, row0, N):
    nqt = (Nq + 255) // 256
    ntile = (N + 127) // 128
    out = []
    for i in range(nqt * Hq * B):
        last = min(_query_tile(i, nqt, Hq // Hkv, B * Hkv) * 256 + 255, Nq - 1)
        out.append(2 * min((row0 + last) // 128 + 1, ntile) + 4)
    return out


SHAPES = [(1, 28, 4, 8192, 0, 8192), (1, 20, 4, 8192, 0, 8192), (1, 12, 2, 16384, 0, 16384), (2, 14, 2, 5000, 0, 5000),
          (3, 36, 4, 1280, 0, 1280), (1, 40, 8, 8192, 0, 8192), (1, 28, 4, 3000, 3144, 6144), (5, 9, 3, 2100, 0, 2100)]


@pytest.mark.parametrize("shape", SHAPES)
def test_every_item_once_on_its_own_xcd_with_the_stated_loads(shape):
    B, Hq, Hkv, Nq, row0, N = shape
    plan = P.pasa_work_plan(B, Hq, Hkv, Nq, row0, N, 256)
    assert plan is not None
    lists, worst, ordinary, used = plan
    cost = _costs(B, Hq, Hkv, Nq, row0, N)
    assert sorted(i for l in lists for i in l) == list(range(len(cost)))
    assert all(i % 8 == w % 8 for w, l in enumerate(lists) for i in l)
    loads = [sum(cost[i] for i in l) for l in lists]
    assert max(loads) == worst
    assert all([cost[i] for i in l] == sorted((cost[i] for i in l), reverse=True) for l in lists)   # longest first
    # dispatch in index order, recomputed: each item of a class to the place of the class that is free first
    hi = 0
    for x in range(8):
        busy = [0] * len(range(x, 256, 8))
        for i in range(x, len(cost), 8):
            busy[busy.index(min(busy))] += cost[i]
        hi = max(hi, max(busy))
    assert hi == ordinary
    assert worst <= ordinary
    assert used == (worst * 103 <= ordinary * 100)
    # no class can do better than its mean
    for x in range(8):
        total = sum(cost[i] for i in range(x, len(cost), 8))
        assert max(loads[w] for w in range(x, 256, 8)) >= total / 32


def test_the_benchmark_shape_reaches_the_lower_bound_and_stays_ordinary():
    lists, worst, ordinary, used = P.pasa_work_plan(1, 28, 4, 8192, 0, 8192, 256)
    # 896 items of 2 .. 64 tiles: costs are multiples of 4 and a class of 112 items on 32 places averages 246 or 244
    assert (worst, ordinary) == (248, 252)
    assert not used            # 1.6 % on paper is less than the list-walking kernel costs


def test_shapes_that_follow_their_plan():
    for shape in [(1, 20, 4, 8192, 0, 8192), (1, 28, 4, 6144, 0, 6144), (1, 12, 2, 16384, 0, 16384)]:
        assert P.pasa_work_plan(*shape, 256)[3], shape
    for shape in [(1, 32, 4, 4096, 0, 4096), (1, 64, 8, 4096, 0, 4096)]:      # powers of two divide evenly anyway
        assert not P.pasa_work_plan(*shape, 256)[3], shape


def test_sizes_that_are_never_planned():
    assert P.pasa_work_plan(1, 8, 8, 4096, 0, 4096, 256) is None        # not more items than places
    assert P.pasa_work_plan(2, 28, 4, 32768, 0, 32768, 256) is None     # more items than a kernel argument holds
    assert P.pasa_work_plan(1, 28, 4, 8192, 0, 8192, 4) is None         # fewer places than XCDs
    with pytest.raises(P.PasaError):
        P.pasa_work_plan(1, 28, 5, 8192, 0, 8192, 256)


@pytest.mark.parametrize("Hq,nqt", [(2, 12), (3, 8), (1, 20)])
def test_small_cases_against_brute_force(Hq, nqt):
    """16 places, two per XCD class: the best split of a class's handful of items is found by enumeration."""
    N = 256 * nqt
    lists, worst, ordinary, used = P.pasa_work_plan(1, Hq, 1, N, 0, N, 16)
    cost = _costs(1, Hq, 1, N, 0, N)
    best = 0
    for x in range(8):
        items = [cost[i] for i in range(x, len(cost), 8)]
        total = sum(items)
        opt = min(max(s, total - s) for r in range(len(items) + 1) for c in itertools.combinations(items, r) for s in [sum(c)])
        best = max(best, opt)
    assert worst == best


def test_switch_returns_the_previous_setting():
    was = P.pasa_work_plan_enable(False)
    assert P.pasa_work_plan_enable(True) is False
    assert P.pasa_work_plan_enable(was) is True
