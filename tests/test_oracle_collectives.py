"""Pins for the oracle's collectives: printed chains, closed forms, rule violations."""
import random

import numpy as np
import pytest

from oracle import redist_oracle as O


def _global(gshape, seed=0, dtype=np.int32):
    n = int(np.prod(gshape))
    if n <= 1 << 16:
        return np.arange(n, dtype=dtype).reshape(gshape)          # iota: any misplacement shows
    rng = np.random.default_rng(seed)
    return rng.integers(0, 2 ** 16, size=gshape, dtype=np.uint16)


def _apply(shards, mesh, typ, op, args, printed):
    if op == "allgather":
        i = int(args[0]); k = int(args[1]) if len(args) > 1 else 1
        return O.allgather(shards, mesh, typ, i, k)
    if op == "dynslice":
        return O.dynslice(shards, mesh, typ, int(args[0]), tuple(args[1].split(",")))
    if op == "alltoall":
        i, j = int(args[0]), int(args[1]); k = int(args[2]) if len(args) > 2 else 1
        return O.alltoall(shards, mesh, typ, i, j, k)
    if op == "allpermute":
        return O.allpermute(shards, mesh, typ, printed)
    raise AssertionError(op)


def test_every_printed_chain_typechecks_and_matches_direct_slicing(paper_chains):
    assert len(paper_chains) >= 18
    for blk in paper_chains:
        mesh = blk["mesh"]
        typ = O.parse_type(blk["start"])
        assert O.wf_type(mesh, typ), blk["cite"]
        G = _global(O.globaltype(typ))
        shards = O.distribute(G, mesh, typ)
        for op, args, printed_text in blk["steps"]:
            printed = O.parse_type(printed_text)
            shards, typ = _apply(shards, mesh, typ, op, args, printed)
            assert typ == printed, (blk["cite"], op, O.format_type(typ), printed_text)
            assert O.wf_type(mesh, typ)
            # Def. 4.3: the type fixes the data -- compare with slicing G directly by T[[printed]]
            want = O.distribute(G, mesh, printed)
            for a, b in zip(shards, want):
                assert a.shape == b.shape and a.tobytes() == b.tobytes(), (blk["cite"], op)


def test_printed_costs(paper_chains, paper_values):
    by_cite = {b["cite"]: b for b in paper_chains}

    def costs(blk):
        typ = O.parse_type(blk["start"])
        out = []
        for op, _a, printed in blk["steps"]:
            nt = O.parse_type(printed)
            out.append(O.step_cost(op, O.localsize(typ), O.localsize(nt)))
            typ = nt
        return out

    left = costs(by_cite['Fig. "oversharding", left (no over-partitioning), mesh {x:4,y:2,z:4}'])
    right = costs(by_cite['Fig. "oversharding", right (with over-partitioning), mesh {x:4,y:2,z:4}'])
    l_txt, l_sum = paper_values["cost_overshard_left"].split("=")
    r_txt, r_sum = paper_values["cost_overshard_right"].split("=")
    assert left == [int(v) for v in l_txt.split()] and sum(left) == int(l_sum)
    assert right == [int(v) for v in r_txt.split()] and sum(right) == int(r_sum)

    three = costs(by_cite['Example "single extra permutation" (Sec. 6.2), first chain (one permutation at the end)'])
    assert sum(three[:3]) == int(paper_values["cost_a8_three_alltoalls"]) and three[3] == 8
    merged = costs(by_cite["Example in Sec. 7.1, merged multi-axis alltoall over {a0,a1,a2}"])
    assert merged == [int(paper_values["cost_a8_merged_alltoall"])]


def test_allgather_on_1d_mesh_is_concatenate():
    mesh = {"x": 4}
    typ = O.parse_type("[3{x}12, 5]")
    G = _global((12, 5))
    shards = O.distribute(G, mesh, typ)
    out, t = O.allgather(shards, mesh, typ, 0)
    assert t == O.parse_type("[12, 5]")
    cat = np.concatenate(shards, axis=0)
    assert all(np.array_equal(o, cat) and np.array_equal(o, G) for o in out)


def test_listing_alltoall_is_split_and_concatenate():
    # [32, 64{devs}2048] -> [1{devs}32, 2048]: device q ends with row q of the global matrix
    mesh = {"devs": 32}
    t1 = O.parse_type("[32, 64{devs}2048]")
    G = _global((32, 2048), dtype=np.int64)
    shards = [np.ascontiguousarray(p) for p in np.split(G, 32, axis=1)]
    for a, b in zip(shards, O.distribute(G, mesh, t1)):
        assert np.array_equal(a, b)
    out, t2 = O.alltoall(shards, mesh, t1, 1, 0)
    assert t2 == O.parse_type("[1{devs}32, 2048]")
    for q in range(32):
        expect = np.concatenate([np.split(s, 32, axis=0)[q] for s in shards], axis=1)
        assert np.array_equal(out[q], expect) and np.array_equal(out[q], G[q:q + 1])


def test_swap_across_dims_on_square_mesh_transposes_the_grid_of_shards():
    mesh = {"x": 4, "y": 4}
    t1, t2 = O.parse_type("[3{x}12, 2{y}8]"), O.parse_type("[3{y}12, 2{x}8]")
    G = _global((12, 8))
    shards = O.distribute(G, mesh, t1)
    out, _ = O.allpermute(shards, mesh, t1, t2)
    grid = [[shards[ix * 4 + iy] for iy in range(4)] for ix in range(4)]
    for ix in range(4):
        for iy in range(4):
            assert np.array_equal(out[ix * 4 + iy], grid[iy][ix])


def test_dynslice_is_local_and_keeps_chunk_i_x():
    mesh = {"x": 2, "y": 3}
    t1 = O.parse_type("[4{x}8, 6]")
    G = _global((8, 6))
    shards = O.distribute(G, mesh, t1)
    out, t2 = O.dynslice(shards, mesh, t1, 1, ("y",))
    assert t2 == O.parse_type("[4{x}8, 2{y}6]")
    for k, c in enumerate(O.mesh_coords(mesh)):
        assert np.array_equal(out[k], shards[k][:, 2 * c["y"]:2 * c["y"] + 2])


def test_multi_axis_equals_single_axis_steps():
    mesh = {"a": 2, "b": 3, "c": 2}
    t1 = O.parse_type("[2{a,b}12, 12]")
    G = _global((12, 12))
    sh = O.distribute(G, mesh, t1)
    one, t_one = O.alltoall(sh, mesh, t1, 0, 1, 2)
    s, t = O.alltoall(sh, mesh, t1, 0, 1, 1)
    # after moving a, dim 0 is 4{b}; moving b next puts b in FRONT of a on dim 1, so the
    # two-step result differs from the merged one by an axis order -- both are direct slicings
    s, t = O.alltoall(s, mesh, t, 0, 1, 1)
    assert t_one == O.parse_type("[12, 2{a,b}12]") and t == O.parse_type("[12, 2{b,a}12]")
    for got, typ in ((one, t_one), (s, t)):
        for a, b in zip(got, O.distribute(G, mesh, typ)):
            assert a.tobytes() == b.tobytes()
    g2, tg2 = O.allgather(sh, mesh, t1, 0, 2)
    s, t = O.allgather(sh, mesh, t1, 0, 1)
    s, t = O.allgather(s, mesh, t, 0, 1)
    assert t == tg2 and all(a.tobytes() == b.tobytes() for a, b in zip(s, g2))


def test_rule_violations():
    mesh = {"x": 2, "y": 2, "z": 3}
    t = O.parse_type("[4{x}8, 6]")
    with pytest.raises(ValueError):
        O.rule_dynslice(mesh, t, 1, ("x",))            # axis already in use
    with pytest.raises(ValueError):
        O.rule_dynslice(mesh, O.parse_type("[4{x}8, 5]"), 1, ("y",))      # 5 not divisible by 2
    with pytest.raises(ValueError):
        O.rule_alltoall(mesh, O.parse_type("[4{x}8, 5]"), 0, 1)           # c_j mod n != 0
    with pytest.raises(ValueError):
        O.rule_allgather(mesh, t, 1)                   # nothing to gather
    with pytest.raises(ValueError):
        O.allpermute(O.distribute(_global((8, 6)), mesh, t), mesh, t, O.parse_type("[8, 3{y}6]"))
    assert not O.rule_allpermute_ok(O.parse_type("[4{x}8]"), O.parse_type("[4{x}8, 1]"))


def test_naive_redistribution_reaches_target_with_height_globalsize():
    mesh = {"x": 4, "y": 2}
    t1, t2 = O.parse_type("[2{x}8, 8{y}16]"), O.parse_type("[4{y}8, 4{x}16]")
    G = _global((8, 16))
    out, types = O.naive_redistribute(O.distribute(G, mesh, t1), mesh, t1, t2)
    for a, b in zip(out, O.distribute(G, mesh, t2)):
        assert a.tobytes() == b.tobytes()
    sizes = [O.localsize(t) for t in types]
    assert O.height(sizes) == O.globalsize(t1) > max(O.localsize(t1), O.localsize(t2))   # Eq. (3) violated


def test_redistribute_by_definition_roundtrip_random():
    rng = random.Random(7)
    mesh = {"a": 2, "b": 2, "c": 3}
    for _ in range(25):
        names = list(mesh)
        def rand_type(gshape_c):
            assign = [rng.randrange(-1, 2) for _ in names]
            dims = []
            for t in range(2):
                ax = [x for x, a in zip(names, assign) if a == t]
                rng.shuffle(ax)
                dims.append(O.Dim(gshape_c[t] // int(np.prod([mesh[x] for x in ax])), tuple(ax), gshape_c[t]))
            return tuple(dims)
        g = (12, 24)
        t1, t2 = rand_type(g), rand_type(g)
        G = _global(g)
        dst = O.redistribute_by_definition(O.distribute(G, mesh, t1), mesh, t1, t2)
        assert np.array_equal(O.undistribute(dst, mesh, t2), G)          # undistribute(redistribute(x)) == x
        for a, b in zip(dst, O.distribute(G, mesh, t2)):
            assert a.tobytes() == b.tobytes()


def test_normal_form_and_height():
    assert O.is_normal_form(["dynslice", "dynslice", "alltoall", "allpermute", "alltoall", "allgather"])
    assert O.is_normal_form([])
    assert not O.is_normal_form(["allgather", "dynslice"])
    assert not O.is_normal_form(["alltoall", "dynslice"])
    assert not O.is_normal_form(["allgather", "allpermute"])
    assert O.height([64, 16, 16, 128]) == 128


# ---- low-level forms -------------------------------------------------------
def _state(G, mesh, typ):
    return O.DeviceState(G.shape, O.localtype(typ), O.offset_table(typ, mesh), O.distribute(G, mesh, typ))


def test_low_level_allgather_on_a_non_front_axis_needs_no_data_movement_first():
    # [2{y,x}..]: gathering x (major) groups NON-adjacent tiles under the strict rule; the low-level
    # rule relabels devices so that groups are the adjacent tiles.  Result must be a weak [4{?}..] type.
    mesh = {"x": 2, "y": 2}
    typ = O.parse_type("[2{y,x}8, 3]")
    G = _global((8, 3))
    st = _state(G, mesh, typ)
    by_off = {o[0]: d for d, o in enumerate(st.offs)}
    groups = [[by_off[0], by_off[2]], [by_off[4], by_off[6]]]
    out = O.ll_allgather(st, 0, groups)
    out.check_weak_type()
    out.check_data(G)
    assert out.shape == (4, 3)
    with pytest.raises(AssertionError):
        O.ll_allgather(st, 0, [[by_off[0], by_off[4]], [by_off[2], by_off[6]]])   # strict x-groups: not adjacent


def test_low_level_alltoall_equals_strict_when_axis_is_in_front():
    mesh = {"x": 2, "y": 2}
    typ = O.parse_type("[2{x,y}8, 4]")
    G = _global((8, 4))
    st = _state(G, mesh, typ)
    coords = O.mesh_coords(mesh)
    groups = []
    for iy in range(2):
        groups.append([k for ix in range(2) for k, c in enumerate(coords) if c["x"] == ix and c["y"] == iy])
    out = O.ll_alltoall(st, 0, 1, groups)
    out.check_weak_type(); out.check_data(G)
    strict, t2 = O.alltoall(O.distribute(G, mesh, typ), mesh, typ, 0, 1)
    assert out.offs == O.offset_table(t2, mesh)
    assert all(a.tobytes() == b.tobytes() for a, b in zip(out.tiles, strict))


def test_low_level_dynslice_must_stay_balanced_and_permute_must_be_bijective():
    mesh = {"x": 2, "y": 2}
    typ = O.parse_type("[4{x}8]")
    G = _global((8,))
    st = _state(G, mesh, typ)
    coords = O.mesh_coords(mesh)
    ok = O.ll_dynslice(st, 0, 2, [c["y"] for c in coords])
    ok.check_data(G)
    assert ok.offs == O.offset_table(O.parse_type("[2{y,x}8]"), mesh)
    with pytest.raises(AssertionError):
        O.ll_dynslice(st, 0, 2, [0, 0, 0, 0])             # both replicas keep chunk 0: no longer a cover
    with pytest.raises(AssertionError):
        O.ll_allpermute(st, [0, 0, 1, 2])
    p = O.ll_allpermute(st, [2, 3, 0, 1])
    p.check_data(G)
    assert p.offs == O.offset_table(O.parse_type("[4{x}8]"), {"x": 2, "y": 2})[2:] + O.offset_table(typ, mesh)[:2]
