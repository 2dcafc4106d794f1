"""redist_options: the explicit knobs of plan lowering (no environment variables), the launches they lead to, the
latency term of the search, and the limits of the entry point that allocates nothing.  CPU only: plans are built
through the C-ABI and carried out by the host model of the kernels."""
import random

import numpy as np
import pytest

import paper_2112_01075_amd as R
import synthetic_inputs as S
from kernel_model import run_plan
from oracle import redist_oracle as O
from test_planner import _random_type, _shrunk, replay


def _model_matches_oracle(plan, mesh, a, b, elem, seed=0):
    t1, t2 = O.parse_type(a), O.parse_type(b)
    G = S.random_bytes_array(O.globaltype(t1), elem, seed)
    gv = G.view(np.dtype((np.void, elem)))[..., 0]
    src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in O.distribute(gv, mesh, t1)]
    want = [s.tobytes() for s in O.distribute(gv, mesh, t2)]
    assert [x.tobytes() for x in run_plan(plan, src)] == want, (a, b)


def test_defaults_and_rejected_struct_size():
    o = R.Options()
    assert (o.merge_runs, o.fold_permute, o.lds_staging, o.span_form, o.dest_major) == (1, 1, 1, 1, 1)
    assert (o.unroll, o.dest_major_min_bytes, o.max_grid, o.step_latency_elems) == (0, 32 << 20, 16777215, 0)
    assert (o.launch_latency_ns, o.sustained_gbs, o.dest_major_fanout) == (3000, 5500, 0)
    o.struct_size = 8
    with pytest.raises(R.RedistError) as e:
        R.redist_plan({"x": 2}, "[2{x}4]", "[4]", 4, options=o)
    assert e.value.status == 9


def test_which_steps_share_a_launch():
    """Stepwise plans: runs of dynslices / allgathers are one launch, dynslices ride on the launch after them, the
    allpermute rides on the alltoall before it, else on the allgathers after it; alltoalls and a run of allgathers
    after another collective stay launches of their own.  Whatever is merged, the step list, cost and height stay,
    and the result is the oracle's."""
    literal, no_fold = R.Options(merge_runs=0), R.Options(fold_permute=0)
    rng = random.Random(31)
    meshes = [{"a": 2, "b": 2}, {"a": 2, "b": 3}, {"a": 4, "b": 2}, {"a": 2, "b": 2, "c": 2}, {"a": 6, "b": 4}]
    shapes = [(12, 12), (24, 8), (4, 6, 8), (48,), (6, 4, 2, 12), (36, 24)]
    seen = {"a2a+perm": 0, "perm+gather": 0, "slice+": 0, "perm alone": 0}
    for n in range(120):
        mesh, g = rng.choice(meshes), rng.choice(shapes)
        a, b = _random_type(rng, mesh, g), _random_type(rng, mesh, g)
        elem = rng.choice([1, 2, 4, 8])
        plans = [R.redist_plan(mesh, a, b, elem, options=o) for o in (None, no_fold, literal)]
        kinds = [s["kind"] for s in plans[0].steps()]
        for p in plans:
            assert [s["kind"] for s in p.steps()] == kinds
            assert (p.cost_elems, p.height_elems, p.bound_elems) == (plans[0].cost_elems, plans[0].height_elems, plans[0].bound_elems)
            _model_matches_oracle(p, mesh, a, b, elem, seed=n)
        assert plans[2].num_ops == max(1, len(kinds))
        # expected grouping of the default lowering, written out from the rules above
        groups, k = [], 0
        while k < len(kinds):
            first = k
            if kinds[k] == "dynslice":
                while k + 1 < len(kinds) and kinds[k + 1] == "dynslice":
                    k += 1
                if k + 1 < len(kinds):
                    k += 1
                    seen["slice+"] += 1
            if kinds[k] == "allgather":
                while k + 1 < len(kinds) and kinds[k + 1] == "allgather":
                    k += 1
            elif kinds[k] == "alltoall" and k + 1 < len(kinds) and kinds[k + 1] == "allpermute":
                k += 1
                seen["a2a+perm"] += 1
            elif kinds[k] == "allpermute":
                if k + 1 < len(kinds):
                    k += 1
                    while k + 1 < len(kinds) and kinds[k + 1] == "allgather":
                        k += 1
                    seen["perm+gather"] += 1
                else:
                    seen["perm alone"] += 1
            groups.append((first, k))
            k += 1
        assert [plans[0].op_last_step(i) for i in range(plans[0].num_ops)] == [g_[1] for g_ in groups] or not kinds
        assert plans[1].num_ops >= plans[0].num_ops
        # a launch holds its first input and last output: never more than source tile + target tile ... per launch
        sizes = [int(np.prod(O.localtype(O.parse_type(a))))] + [int(np.prod(s["shape_after"])) for s in plans[0].steps()]
        ends = [0] + [plans[0].op_last_step(i) + 1 for i in range(plans[0].num_ops)] if kinds else [0, 0]
        assert plans[0].peak_live_bytes_per_shard == max(sizes[x] + sizes[y] for x, y in zip(ends, ends[1:])) * elem
        assert plans[0].footprint_bytes_per_shard == (sizes[0] + sizes[-1]) * elem + plans[0].workspace_bytes // plans[0].num_devices
    assert all(v >= 3 for v in seen.values()), seen


def test_weight_reshard_is_one_launch_when_the_permute_is_folded():
    mesh, pairs = _shrunk("c3_fp32_weight_4x2", 128)
    a, b = pairs[0]
    p = R.redist_plan(mesh, a, b, 4)
    assert [s["kind"] for s in p.steps()] == ["alltoall", "allpermute"]
    assert p.num_ops == 1 and p.workspace_bytes == 0 and p.step_kernel(0).startswith("redist_alltoall")
    q = R.redist_plan(mesh, a, b, 4, options=R.Options(fold_permute=0))
    assert q.num_ops == 2 and q.workspace_bytes > 0
    assert p.footprint_bytes_per_shard < q.footprint_bytes_per_shard


def test_options_are_part_of_the_cache_key():
    R.redist_plan_cache_clear()
    mesh, a, b = {"x": 4, "y": 2}, "[2{x}8, 8{y}16]", "[4{y}8, 4{x}16]"
    p1 = R.redist_plan(mesh, a, b, 4, cached=True)
    p2 = R.redist_plan(mesh, a, b, 4, cached=True, options=R.Options())          # the defaults, spelled out
    p3 = R.redist_plan(mesh, a, b, 4, cached=True, options=R.Options(fold_permute=0))
    p4 = R.redist_plan(mesh, a, b, 4, cached=True, options=R.Options(step_latency_elems=5))
    assert p1._h.value == p2._h.value and len({p1._h.value, p3._h.value, p4._h.value}) == 3
    assert R.redist_plan_cache_size() == 3
    assert p1.num_ops == 1 and p3.num_ops == 2
    R.redist_plan_cache_clear()


def test_latency_term_changes_which_sequence_the_planner_prefers():
    """step_latency_elems: the planner's normal-form search with that term against the oracle's, and the plans it
    leads to replayed through the oracle's collectives.  The getters keep reporting the paper's cost."""
    cases = [({"a": 2, "b": 3, "c": 2}, "[6{a,c}24, 8, 4]", "[24, 4{a}8, 2{c}4]"),
             ({"a": 4, "b": 2, "c": 3}, "[6{b}12, 4, 4{a}16]", "[3{a}12, 2{b}4, 16]"),
             ({"a": 4, "b": 2, "c": 3}, "[6{a}24, 24, 16]", "[24, 4{b,c}24, 16]")]
    fewer = 0
    for mesh, a, b in cases:
        t1, t2 = O.parse_type(a), O.parse_type(b)
        base = R.redist_plan(mesh, a, b, 4)
        for lam in (0, 7, 10 ** 6):
            p = R.redist_plan(mesh, a, b, 4, options=R.Options(step_latency_elems=lam))
            kinds, sizes = replay(p, mesh, a, b)
            comm = sum(1 for k in kinds if k in ("alltoall", "allgather"))
            pm, _, _ = O.decompose(mesh, t1, t2)
            want, _ = O.weak_search(O.globaltype(t1), list(pm.values()), O.localtype(t1), O.localtype(t2),
                                    normal_form=True, step_latency=lam)
            assert p.weak_cost_elems + lam * comm == want, (a, b, lam)
            assert p.weak_cost_elems == O.sequence_cost([k for k in kinds if k != "allpermute"],
                                                        [s for s, k in zip(sizes, ["x"] + kinds) if k != "allpermute"]) \
                or "allpermute" in kinds
            assert p.height_elems <= p.bound_elems
            base_comm = sum(1 for s in base.steps() if s["kind"] in ("alltoall", "allgather"))
            assert comm <= base_comm and p.weak_cost_elems >= base.weak_cost_elems
            fewer += comm < base_comm
    assert fewer >= 2


def test_ops_beyond_the_grid_limit_take_several_launches():
    """The runtime refuses 2^32 threads and more per grid dimension, i.e. more than 16777215 workgroups of 256: a
    2 GiB array gathered to 32 full replicas has 2^24 tiles of 4 KiB and goes out as two launches.  A small
    max_grid reaches the same path on a small problem (the model runs every launch index once either way)."""
    mesh = {"x": 2, "y": 4, "z": 4}
    p = R.redist_plan(mesh, "[4{x,y,z}128, 2048, 4096]", "[128, 2048, 4096]", 2, R.MODE_FUSED)
    info = p.op(0)[0]
    assert info.n_tiles == 1 << 24 and info.max_grid == 16777215 and -(-info.n_tiles // info.max_grid) == 2
    q = R.redist_plan({"a": 2, "b": 2}, "[6{a}12, 30]", "[12, 15{b}30]", 4, R.MODE_FUSED, options=R.Options(max_grid=3))
    assert q.op(0)[0].max_grid == 3 and q.row_op(0)[0].max_grid == 3
    _model_matches_oracle(q, {"a": 2, "b": 2}, "[6{a}12, 30]", "[12, 15{b}30]", 4)
    assert R.redist_plan({"a": 2}, "[2{a}4]", "[4]", 4, options=R.Options(max_grid=1 << 30)).op(0)[0].max_grid == 16777215


def test_which_plans_fit_the_static_scratch_area():
    w = S.WORKLOADS["c2_bf16_act_1x8"]
    assert R.redist_plan(w["mesh"], *w["pairs"][0], 2, R.MODE_FUSED).static_fits          # one launch: descriptors only
    w = S.WORKLOADS["c4_bf16_act_2x4x4"]
    big = R.redist_plan(w["mesh"], *w["pairs"][1], 2, R.MODE_STEPWISE)
    assert big.num_ops == 2 and big.workspace_bytes > R.STATIC_SCRATCH_BYTES and not big.static_fits
    small = R.redist_plan({"x": 4, "y": 2}, "[2{x}8, 8{y}16]", "[4{y}8, 4{x}16]", 4, options=R.Options(fold_permute=0))
    assert small.num_ops == 2 and 0 < small.workspace_bytes < R.STATIC_SCRATCH_BYTES and small.static_fits
    assert not R.redist_plan({"x": 64, "y": 4}, "[8{x}512, 6{y}24]", "[2{y,x}512, 24]", 4).static_fits   # 256 devices
    assert R.lib().redist_plan_static_fits(None) == -1


def test_auto_mode_keeps_the_plan_with_the_smaller_predicted_time():
    """REDIST_MODE_AUTO: predicted time = sum over launches of (launch latency + bytes moved / sustained rate); the
    collective sequence is kept on a tie (one launch of the same bytes), else whichever is predicted faster; the
    paper's cost stays what the getters report."""
    mesh = {"x": 8}
    a, b = "[128{x}1024, 2048]", "[1024, 256{x}2048]"                     # one alltoall: a tie, the sequence stays
    auto, step, fused = (R.redist_plan(mesh, a, b, 2, m) for m in (R.MODE_AUTO, R.MODE_STEPWISE, R.MODE_FUSED))
    assert step.num_ops == 1 and step.predicted_ns == fused.predicted_ns == auto.predicted_ns
    assert auto.mode == R.MODE_STEPWISE and [s["kind"] for s in auto.steps()] == ["alltoall"]
    assert auto.predicted_ns == 3000 + 2 * 1024 * 2048 * 2 // 5500
    # two alltoalls in a row stay two launches: the one-pass gather is predicted (and is) faster
    mesh = {"x": 4, "y": 4}
    a, b = "[32{x}128, 512, 32{y}128]", "[128, 32{y,x}512, 128]"
    auto, step, fused = (R.redist_plan(mesh, a, b, 2, m) for m in (R.MODE_AUTO, R.MODE_STEPWISE, R.MODE_FUSED))
    assert step.num_ops == 2 and step.predicted_ns > fused.predicted_ns == auto.predicted_ns
    assert auto.mode == R.MODE_FUSED and auto.num_ops == 1 and auto.workspace_bytes == 0
    assert 0 <= 2 * 3000 + step.algorithmic_bytes(R.BYTES_MOVED_BY_PLAN) // 5500 - step.predicted_ns <= 2   # floors per launch
    # the constants are options
    slow = R.redist_plan(mesh, a, b, 2, R.MODE_STEPWISE, options=R.Options(launch_latency_ns=10000, sustained_gbs=1000))
    assert 0 <= 2 * 10000 + slow.algorithmic_bytes(R.BYTES_MOVED_BY_PLAN) // 1000 - slow.predicted_ns <= 2
    # AUTO results are what the oracle says, like any plan's
    _model_matches_oracle(R.redist_plan(mesh, a, b, 2, R.MODE_AUTO), mesh, a, b, 2)
    with pytest.raises(R.RedistError) as e:
        R.redist_plan(mesh, a, b, 2, 4)
    assert e.value.status == 9


def test_search_limits_are_reported():
    """redist_plan_search_limits_hit: a bit mask of the synthesis limits that were reached, 0 for ordinary problems
    (none of 300 paper-shaped ones reaches a limit); -1 for a null plan."""
    assert R.redist_plan({"x": 4, "y": 2}, "[2{x}8, 8{y}16]", "[4{y}8, 4{x}16]", 4).search_limits_hit == 0
    assert R.lib().redist_plan_search_limits_hit(None) == -1
    mesh = {"a": 2, "b": 2, "c": 2, "d": 2, "e": 2, "f": 2}      # six slices that commute: one canonical order is kept
    p = R.redist_plan(mesh, "[4, 4, 4, 4, 4, 4]", "[2{a}4, 2{b}4, 2{c}4, 2{d}4, 2{e}4, 2{f}4]", 1)
    assert p.cost_elems == 0 and all(s["kind"] == "dynslice" for s in p.steps()) and p.search_limits_hit == 0
    for g, a, b in S.sample_paper_problems(300):
        assert R.redist_plan(S.PAPER_MESH, a, b, 4).search_limits_hit == 0


def test_destination_major_fanout():
    """Workgroups of the generic destination-major kernel store to 2 destinations when a tile has up to 8 of them,
    else to 1; the option fixes the number.  Every setting, under the host model, also on a list that does not
    divide into groups."""
    mesh = {"a": 2, "b": 3, "c": 2}
    a, b = "[20{a}40, 6, 10]", "[40, 2{b}6, 10]"        # every tile to 4 shards (a and c are free in the target)
    for fan, want in ((0, 2), (1, 1), (2, 2), (4, 2)):
        o = R.Options(dest_major_min_bytes=0, dest_major_fanout=fan)
        p = R.redist_plan(mesh, a, b, 4, R.MODE_FUSED, options=o)
        info = p.op(0)[0]
        assert info.dest_major == 1 and info.dm_count == 4 and info.dm_fanout == want
        assert info.dm_groups == -(-4 // want) and info.n_tiles == info.src_tiles * info.dm_groups
        _model_matches_oracle(p, mesh, a, b, 4, seed=fan)
    mesh = {"a": 3}                                      # 3 destinations in groups of 2: the last group is short
    a, b = "[8{a}24, 10]", "[24, 10]"
    p = R.redist_plan(mesh, a, b, 2, R.MODE_FUSED, options=R.Options(dest_major_min_bytes=0))
    info = p.op(0)[0]
    assert (info.dm_count, info.dm_fanout, info.dm_groups) == (3, 2, 2)
    _model_matches_oracle(p, mesh, a, b, 2)
    mesh = {"a": 2}                                      # 2 destinations: one group, the launch has as many workgroups as tiles
    p = R.redist_plan(mesh, "[12{a}24, 10]", "[24, 10]", 2, R.MODE_FUSED, options=R.Options(dest_major_min_bytes=0))
    info = p.op(0)[0]
    assert (info.dm_count, info.dm_fanout, info.dm_groups, info.n_tiles) == (2, 2, 1, info.src_tiles)
    _model_matches_oracle(p, mesh, "[12{a}24, 10]", "[24, 10]", 2)
    w = S.WORKLOADS["c4_bf16_act_2x4x4"]                 # 32 destinations: one per workgroup
    info = R.redist_plan(w["mesh"], *w["pairs"][1], 2, R.MODE_FUSED).op(0)[0]
    assert (info.dest_major, info.dm_count, info.dm_fanout, info.dm_groups) == (1, 32, 1, 32)
