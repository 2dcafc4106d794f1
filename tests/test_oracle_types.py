"""Pins for the oracle's types, base-offset maps, well-formedness and distribute/undistribute."""
import itertools
import random

import numpy as np
import pytest

from conftest import parse_mesh
from oracle import redist_oracle as O


def test_offset_example_sec_2_1(paper_values):
    # Sec. 2.1: [8{x,y}32] on {x:2,y:2}: split in 2 over y, then each half in 2 over x.
    typ = O.parse_type(paper_values["offset_example_type"])
    mesh = parse_mesh(paper_values["offset_example_mesh"])
    halves_over_y = {0: (0, 16), 1: (16, 32)}
    for c in O.mesh_coords(mesh):
        lo, hi = halves_over_y[c["y"]]
        quarter = lo + c["x"] * (hi - lo) // 2
        assert O.T(typ, mesh, c) == (quarter,)
        assert O.T(typ, mesh, c) == (8 * c["x"] + 16 * c["y"],)
    # reversing the axis order keeps the tile shape but changes the assignment
    rev = O.parse_type("[8{y,x}32]")
    assert O.localtype(rev) == O.localtype(typ)
    assert O.T(rev, mesh, {"x": 1, "y": 0}) == (16,)


def test_base_case_requires_c_equals_n():
    with pytest.raises(ValueError):
        O.D(O.Dim(4, (), 8), {}, {})
    assert O.D(O.Dim(8, (), 8), {}, {}) == 0


def test_shard_order_is_row_major_last_axis_fastest():
    mesh = {"a": 2, "b": 3}
    coords = O.mesh_coords(mesh)
    assert [(c["a"], c["b"]) for c in coords] == [(0, 0), (0, 1), (0, 2), (1, 0), (1, 1), (1, 2)]


def _random_wf_type(rng, mesh, rank, max_c=5):
    names = list(mesh)
    assign = [rng.randrange(-1, rank) for _ in names]
    dims = []
    for t in range(rank):
        ax = [x for x, a in zip(names, assign) if a == t]
        rng.shuffle(ax)
        c = rng.randint(1, max_c)
        n = c
        for x in ax:
            n *= mesh[x]
        dims.append(O.Dim(c, tuple(ax), n))
    return tuple(dims)


def test_lemma_4_1_image_is_all_multiples_of_c_below_n():
    rng = random.Random(1)
    for _ in range(200):
        mesh = {"p": rng.choice([2, 3, 4]), "q": rng.choice([2, 3, 5]), "r": rng.choice([1, 2])}
        typ = _random_wf_type(rng, mesh, 1)
        d = typ[0]
        image = sorted({O.D(d, mesh, c) for c in O.mesh_coords(mesh)})
        assert image == list(range(0, d.n, d.c))


def test_lemma_4_2_tiles_cover_global_array_and_roundtrip():
    rng = random.Random(2)
    for _ in range(60):
        mesh = {"p": rng.choice([2, 3]), "q": rng.choice([2, 4]), "r": 2}
        rank = rng.randint(1, 3)
        typ = _random_wf_type(rng, mesh, rank, max_c=3)
        assert O.wf_type(mesh, typ)
        gshape = O.globaltype(typ)
        offs = set(O.offset_table(typ, mesh))
        expect = set(itertools.product(*[range(0, n, c) for n, c in zip(gshape, O.localtype(typ))]))
        assert offs == expect
        G = np.arange(np.prod(gshape), dtype=np.int64).reshape(gshape)
        shards = O.distribute(G, mesh, typ)
        assert len(shards) == O.mesh_size(mesh)
        assert all(s.shape == O.localtype(typ) for s in shards)
        assert np.array_equal(O.undistribute(shards, mesh, typ), G)


def test_shard_of_is_the_tile_the_base_offset_map_names():
    """shard_of (one shard at a time, for arrays too large to shard at once) against what Sec. 4.1 and
    Fig. "Base offset maps" fix: shard k is the tile of localtype extents whose first element is global element
    T[[type]](coordinate k).  Checked three ways that do not go through shard_of itself: byte for byte against
    distribute (pinned above by Lemma 4.2) on random well-formed types, replicated ones included; element by
    element from the linear index of an iota array; and on the printed example of Sec. 2.1."""
    rng = random.Random(5)
    replicated = 0
    for _ in range(80):
        mesh = {"p": rng.choice([2, 3]), "q": rng.choice([2, 4]), "r": rng.choice([1, 2])}
        rank = rng.randint(1, 4)
        typ = _random_wf_type(rng, mesh, rank, max_c=3)
        gshape = O.globaltype(typ)
        G = np.arange(int(np.prod(gshape)), dtype=np.int64).reshape(gshape)
        shards = O.distribute(G, mesh, typ)
        replicated += len(set(O.offset_table(typ, mesh))) < len(shards)
        strides = [int(np.prod(gshape[t + 1:])) for t in range(rank)]
        lshape = O.localtype(typ)
        for k, coord in enumerate(O.mesh_coords(mesh)):
            got = O.shard_of(G, mesh, typ, k)
            assert got.flags["C_CONTIGUOUS"] and got.shape == lshape
            assert got.tobytes() == shards[k].tobytes()
            # iota data: local element l of shard k is global element T(k) + l
            base = O.T(typ, mesh, coord)
            for l in itertools.islice(itertools.product(*[range(c) for c in lshape]), 0, None, 7):
                assert got[l] == sum((b + i) * s for b, i, s in zip(base, l, strides))
        assert np.array_equal(O.undistribute([O.shard_of(G, mesh, typ, k) for k in range(len(shards))], mesh, typ), G)
    assert replicated >= 10
    # Sec. 2.1: [8{x,y}32] on {x:2,y:2}; shard index = 2*i_x + i_y (last axis fastest); first element 8*i_x + 16*i_y
    mesh, typ = {"x": 2, "y": 2}, O.parse_type("[8{x,y}32]")
    G = np.arange(32)
    for ix in range(2):
        for iy in range(2):
            assert O.shard_of(G, mesh, typ, 2 * ix + iy).tolist() == list(range(8 * ix + 16 * iy, 8 * ix + 16 * iy + 8))


def test_undistribute_detects_bad_replica():
    mesh = {"x": 2, "y": 2}
    typ = O.parse_type("[2{x}4]")
    G = np.arange(4)
    sh = O.distribute(G, mesh, typ)
    sh[1] = sh[1] + 1           # coordinate (x=0,y=1) is a replica of (x=0,y=0)
    with pytest.raises(ValueError):
        O.undistribute(sh, mesh, typ)


def test_replicated_type_means_full_copies():
    mesh = {"x": 2, "y": 2}
    typ = O.parse_type("[4, 6]")
    G = np.arange(24).reshape(4, 6)
    for s in O.distribute(G, mesh, typ):
        assert np.array_equal(s, G)


def test_wellformedness_rules():
    mesh = {"x": 4, "y": 8}
    assert O.wf_type(mesh, O.parse_type("[64{x}256, 128{y}1024]"))
    assert not O.wf_type(mesh, O.parse_type("[64{x}256, 128{x}512]"))      # axis used twice across dims
    assert not O.wf_type(mesh, O.parse_type("[16{x,x}256]"))               # axis repeated in a dim
    assert not O.wf_type(mesh, O.parse_type("[64{z}256]"))                 # unknown axis
    assert not O.wf_type(mesh, O.parse_type("[64{x}255]"))                 # c*k != n
    assert not O.wf_type(mesh, O.parse_type("[64{}256]"))                  # c != n with no axes


def test_listing_types_are_well_formed(paper_values):
    t, m = [p.strip() for p in paper_values["listing1_type"].split(";")]
    assert O.wf_type(parse_mesh(m), O.parse_type(t))
    *ts, m = [p.strip() for p in paper_values["listing2_types"].split(";")]
    for t in ts:
        assert O.wf_type(parse_mesh(m), O.parse_type(t))
    # partial replication: [64{xdev}256,1024] on a 4x8 mesh has 4 distinct tiles, each held 8 times
    tab = O.offset_table(O.parse_type(ts[0]), parse_mesh(m))
    assert len(set(tab)) == 4 and all(tab.count(o) == 8 for o in set(tab))


def test_invalid_redistributions_sec_2_5(paper_values):
    for key in ("invalid_1", "invalid_2"):
        a, b, m = [p.strip() for p in paper_values[key].split(";")]
        ta, tb, mesh = O.parse_type(a), O.parse_type(b), parse_mesh(m)
        assert O.wf_type(mesh, ta) and O.wf_type(mesh, tb)
        assert not O.valid_redistribution(ta, tb) and not O.valid_redistribution(tb, ta)
    a, b, m = [p.strip() for p in paper_values["invalid_2"].split(";")]
    assert O.localtype(O.parse_type(a)) == O.localtype(O.parse_type(b))    # same tiles, still invalid


def test_adversarial_table_sizes(paper_values):
    mesh = {"a": 2, "b": 2, "c": 2}
    for key in ("adversarial_P1", "adversarial_P2", "adversarial_P3", "adversarial_P4"):
        a, b, mb = [p.strip() for p in paper_values[key].split(";")]
        ta, tb = O.parse_type(a), O.parse_type(b)
        assert O.wf_type(mesh, ta) and O.wf_type(mesh, tb) and O.valid_redistribution(ta, tb)
        assert int(O.globalsize(ta) * 4 / 2 ** 20 + 0.5) == int(mb)      # MiB, rounded half up


def test_prime_decomposition_preserves_offsets():
    rng = random.Random(3)
    for _ in range(40):
        mesh = {"x": rng.choice([4, 6, 8, 12]), "y": rng.choice([1, 2, 6, 9])}
        typ = _random_wf_type(rng, mesh, 2, max_c=3)
        pm, pt = O.decompose(mesh, typ)
        assert all(len(O.prime_factors(k)) == 1 for k in pm.values())
        assert O.wf_type(pm, pt) and O.localtype(pt) == O.localtype(typ)
        # same shard order, same offsets: the decomposed problem is equivalent
        assert O.offset_table(pt, pm) == O.offset_table(typ, mesh)


def test_factor_decomposition_example_mesh():
    pm, t1 = O.decompose({"x": 4, "y": 6}, O.parse_type("[3{x}12, 2{y}12]"))
    assert sorted(pm.values()) == [2, 2, 2, 3] and O.mesh_size(pm) == 24
    assert [len(d.axes) for d in t1] == [2, 2]
