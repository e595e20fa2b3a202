"""Host logic of the grouped streaming launch: the per-workgroup tile lists (no GPU call is made)."""
import numpy as np
import pytest

import paper_2601_21238_amd as P

TILE_M, TILE_O, BK = 128, 256, 128


def tiles_of(shape):
    M, K, N = shape
    return ((M + TILE_M - 1) // TILE_M) * ((N + TILE_O - 1) // TILE_O)


def tile_cost(shape):
    """K stages plus 3.4 for epilogue and switch (the model the library balances with), in fifths of a stage."""
    return 5 * ((shape[1] + BK - 1) // BK) + 17


def tile_table(shapes, order):
    """(problem, cost) of every tile id, tiles numbered along the problems in processing order."""
    table = []
    for i in order:
        table += [(int(i), tile_cost(shapes[i]))] * tiles_of(shapes[i])
    return table


def decode_step_shapes(layers):
    shapes = []
    for _ in range(layers):
        shapes += [(128, 1280, 3840), (128, 1280, 5120), (128, 5120, 1280)]      # configuration 4: qkv, fc1, fc2
    return shapes


def check_lists(shapes, order, lists, workgroups):
    table = tile_table(shapes, order)
    assert sorted(order.tolist()) == list(range(len(shapes)))
    ks = [shapes[i][1] for i in order]
    assert ks == sorted(ks, reverse=True)                     # longest K first
    got = sorted(t for l in lists for t in l)
    assert got == list(range(len(table)))                     # every tile exactly once
    for l in lists:
        assert l == sorted(l)                                 # the kernel walks its list with a forward-only cursor
    assert len(lists) == min(workgroups, len(table))
    loads = [sum(table[t][1] for t in l) for l in lists]
    return table, loads


def test_decode_step_plan_is_balanced_and_xcd_local():
    shapes = decode_step_shapes(24)
    order, lists = P.stwq_linear_grouped_plan(shapes, 256)
    table, loads = check_lists(shapes, order, lists, 256)
    avg = sum(loads) / len(loads)
    biggest = max(c for _, c in table)
    # list scheduling with the longest tiles first: nobody exceeds the average by a whole tile
    assert max(loads) <= avg + biggest
    # dealing the same tiles out in turn is a third worse than the average; the plan stays within 10 %
    in_turn = [sum(c for _, c in table[g::256]) for g in range(256)]
    assert max(in_turn) > 1.25 * avg and max(loads) < 1.10 * avg
    # each problem's tiles run on the workgroups of one XCD (workgroup ids go to the 8 XCDs in turn)
    xcd_of = {}
    for g, l in enumerate(lists):
        for t in l:
            xcd_of.setdefault(table[t][0], set()).add(g % 8)
    assert all(len(x) == 1 for x in xcd_of.values())


def test_plan_prefers_balance_when_problems_do_not_split_over_xcds():
    # three problems cannot be dealt to eight XCDs without leaving five idle: tiles go to any workgroup
    shapes = [(128, 1024, 65536), (128, 2048, 40000), (128, 512, 30000)]
    order, lists = P.stwq_linear_grouped_plan(shapes, 256)
    table, loads = check_lists(shapes, order, lists, 256)
    assert all(len(l) > 0 for l in lists)
    assert max(loads) <= sum(loads) / len(loads) + max(c for _, c in table)


def test_plan_is_cached_and_redone_when_shapes_change():
    a = decode_step_shapes(8)
    o1, l1 = P.stwq_linear_grouped_plan(a, 64)
    o2, l2 = P.stwq_linear_grouped_plan(a, 64)
    assert l1 == l2 and np.array_equal(o1, o2)
    b = list(a)
    b[4] = (128, 2560, 1280)
    o3, l3 = P.stwq_linear_grouped_plan(b, 64)
    check_lists(b, o3, l3, 64)
    o4, l4 = P.stwq_linear_grouped_plan(a, 128)               # another grid: other lists
    check_lists(a, o4, l4, 128)


def test_no_lists_when_they_are_not_needed_or_do_not_fit():
    assert P.stwq_linear_grouped_plan([(128, 1280, 3840)], 256)[1] is None           # 15 tiles, 256 workgroups
    many = [(128, 1280, 5120)] * 100                                                   # 2000 tiles: too many for the arguments
    assert P.stwq_linear_grouped_plan(many, 256)[1] is None
    with pytest.raises(P.StwqError):
        P.stwq_linear_grouped_plan([(0, 64, 64)], 256)
    with pytest.raises(P.StwqError):
        P.stwq_linear_grouped_plan([(128, 1280, 3840)], 0)
