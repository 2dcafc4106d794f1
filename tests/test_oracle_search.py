"""Pins for the oracle's searches (weak shortest path of Sec. 7.2, strict brute force of Sec. 6.2)."""
import random
import time

from oracle import redist_oracle as O


def _weak(mesh, t1, t2):
    return O.weak_search(O.globaltype(t1), list(mesh.values()), O.localtype(t1), O.localtype(t2))


def test_a8_example_costs_8_with_merged_alltoall():
    mesh, t1, t2 = O.decompose({"a": 8}, O.parse_type("[1{a}8, 8]"), O.parse_type("[8, 1{a}8]"))
    cost, path = _weak(mesh, t1, t2)
    assert cost == 8 and [(e[0], e[1], e[2], e[3]) for e in path] == [("alltoall", 0, 1, 8)]
    scost, spath = O.strict_search(mesh, t1, t2)
    assert scost == 8 and [k for k, _ in spath] == ["alltoall"]


def test_factor_decomposition_example_weak_cost_12_all_local_sizes_6():
    mesh, t1, t2 = O.decompose({"x": 4, "y": 6}, O.parse_type("[3{x}12, 2{y}12]"), O.parse_type("[2{y}12, 3{x}12]"))
    cost, path = _weak(mesh, t1, t2)
    assert cost == 12 and all(e[0] == "alltoall" for e in path)
    import numpy as np
    assert all(int(np.prod(e[4])) == 6 for e in path)
    scost, spath = O.strict_search(mesh, t1, t2)
    # the printed strict chain (alltoall, permute, alltoall, permute) costs 24; the optimum is in between
    # (strict sequences need bookkeeping permutes; the weak optimum drops them)
    assert 12 <= scost <= 24


def test_oversharding_example_upper_bound():
    mesh = {"x": 4, "y": 2, "z": 4}
    t1, t2 = O.parse_type("[1{y,x}8, 8, 8, 4]"), O.parse_type("[8, 4{y}8, 2{x}8, 4]")
    cost, path = _weak(mesh, t1, t2)
    assert cost <= 384                                   # the figure's over-partitioned sequence
    assert cost < 512                                    # over-partitioning beats the plain sequence
    assert any(e[0] == "dynslice" for e in path)         # and it is found through zero-cost slices
    sizes = [O.localsize(t1)] + [O.prod(e[4]) for e in path]
    assert O.height(sizes) <= max(O.localsize(t1), O.localsize(t2))
    assert O.sequence_cost([e[0] for e in path], sizes) == cost


def test_dynslice_only_problem():
    mesh = {"x": 4, "y": 4}
    cost, path = _weak(mesh, O.parse_type("[16]"), O.parse_type("[4{x}16]"))
    assert cost == 0 and all(e[0] == "dynslice" for e in path)
    scost, spath = O.strict_search(*O.decompose(mesh, O.parse_type("[16]"), O.parse_type("[4{x}16]")))
    assert scost == 0


def _random_problem(rng, mesh, gshape):
    names = list(mesh)

    def one():
        while True:
            assign = [rng.randrange(-1, len(gshape)) for _ in names]
            dims, ok = [], True
            for t, n in enumerate(gshape):
                ax = [x for x, a in zip(names, assign) if a == t]
                rng.shuffle(ax)
                k = O.prod(mesh[x] for x in ax)
                if n % k:
                    ok = False
                    break
                dims.append(O.Dim(n // k, tuple(ax), n))
            if ok:
                return tuple(dims)
    return one(), one()


def test_weak_optimum_never_exceeds_strict_optimum():
    rng = random.Random(11)
    t0 = time.time()
    checked = 0
    for _ in range(40):
        mesh = rng.choice([{"a": 2, "b": 2}, {"a": 2, "b": 3}, {"a": 2, "b": 2, "c": 2}, {"a": 4, "b": 2}])
        gshape = rng.choice([(12, 12), (8, 12), (4, 6, 8), (24,)])
        t1, t2 = _random_problem(rng, mesh, gshape)
        pm, p1, p2 = O.decompose(mesh, t1, t2)
        wcost, wpath = _weak(pm, p1, p2)
        scost, spath = O.strict_search(pm, p1, p2)
        assert wcost is not None and scost is not None
        # Lifting Lemma: dropping the permutes of any strict sequence gives a weak one, so the weak
        # optimum never exceeds the strict optimum.  (A lowered weak optimum plus one final permute
        # of size L(t2) is then within L(t2) of ANY sequence's cost: Near Optimality theorem.)
        assert wcost <= scost, (mesh, O.format_type(t1), O.format_type(t2))
        sizes = [O.localsize(p1)] + [O.prod(e[4]) for e in wpath]
        assert O.height(sizes) <= max(O.localsize(t1), O.localsize(t2))
        checked += 1
        if time.time() - t0 > 60:
            break
    assert checked >= 10


def test_weak_search_cost_is_reachable_in_normal_form():
    # Lemma "cost-weak-nf": a normal-form weak sequence of no greater cost exists, so restricting
    # the search to label strings dynslice* alltoall* allgather* must not change the optimum.
    rng = random.Random(5)
    for _ in range(60):
        mesh = rng.choice([{"a": 2, "b": 2, "c": 3}, {"a": 4, "b": 2, "c": 2}, {"a": 2, "b": 6}])
        t1, t2 = _random_problem(rng, mesh, rng.choice([(12, 12, 6), (24, 8), (4, 6, 12)]))
        g, sizes = O.globaltype(t1), list(mesh.values())
        cost, path = O.weak_search(g, sizes, O.localtype(t1), O.localtype(t2))
        ncost, npath = O.weak_search(g, sizes, O.localtype(t1), O.localtype(t2), normal_form=True)
        assert cost == ncost
        kinds = [e[0] for e in npath]
        assert O.is_normal_form(kinds)
        assert O.sequence_cost(kinds, [O.localsize(t1)] + [O.prod(e[4]) for e in npath]) == ncost
