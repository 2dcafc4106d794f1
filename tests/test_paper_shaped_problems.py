"""The paper's own evaluation shape (Sec. 8): problems on a 2x2x2 mesh, arrays of up to six dimensions,
64-800 MB, each mesh axis replicated or partitioning one dimension.  Planner latency and plan invariants on
1000 seeded problems (the paper reports under a second per problem for its Python search), the four printed
adversarial problems, and agreement of the plan cost with the oracle's own weak search on a subset."""
import time

import paper_2112_01075_amd as R
import synthetic_inputs as S
from oracle import redist_oracle as O


def _invariants(plan, t1, t2):
    kinds = [s["kind"] for s in plan.steps()]
    L1, L2 = O.localsize(t1), O.localsize(t2)
    assert plan.bound_elems == max(L1, L2) and plan.height_elems <= plan.bound_elems        # Eq. (3)
    assert O.is_normal_form(kinds) and kinds.count("allpermute") <= 1                        # Def. 4.5
    if "allpermute" in kinds:
        assert all(k == "allgather" for k in kinds[kinds.index("allpermute") + 1:])          # hoisted, Sec. 7.3
    assert plan.cost_elems <= plan.weak_cost_elems + L2                                      # one permute at most
    assert plan.step_offsets(-1) == O.offset_table(t1, S.PAPER_MESH)
    last = plan.num_steps - 1
    if last >= 0:
        assert plan.step_offsets(last) == O.offset_table(t2, S.PAPER_MESH)
    return kinds


def test_planner_latency_and_invariants_on_1000_sampled_problems():
    problems = S.sample_paper_problems(1000)
    assert len(problems) == 1000 and problems == S.sample_paper_problems(1000)
    worst, total = 0.0, 0.0
    for n, (g, a, b) in enumerate(problems):
        t0 = time.perf_counter()
        plan = R.redist_plan(S.PAPER_MESH, a, b, S.PAPER_ELEM_SIZE)
        dt = time.perf_counter() - t0
        worst, total = max(worst, dt), total + dt
        t1, t2 = O.parse_type(a), O.parse_type(b)
        assert O.globaltype(t1) == g and 64 <= O.globalsize(t1) * 4 / 2 ** 20 <= 800
        _invariants(plan, t1, t2)
        if n % 10 == 0:          # cost against the oracle's independent search (Sec. 7.2)
            wcost, _ = O.weak_search(g, [2, 2, 2], O.localtype(t1), O.localtype(t2))
            assert plan.weak_cost_elems == wcost
    print("planner: mean %.3f ms, worst %.3f ms per problem" % (total / len(problems) * 1e3, worst * 1e3))
    assert worst < 1.0          # the paper's budget: under a second per problem


def test_printed_adversarial_problems(paper_values):
    for key in ("adversarial_P1", "adversarial_P2", "adversarial_P3", "adversarial_P4"):
        a, b, _mb = [p.strip() for p in paper_values[key].split(";")]
        a, b = O.format_type(O.parse_type(a)), O.format_type(O.parse_type(b))
        plan = R.redist_plan(S.PAPER_MESH, a, b, 4)
        kinds = _invariants(plan, O.parse_type(a), O.parse_type(b))
        # the paper notes that its search answers these with dynslice / alltoall / allpermute steps
        # (no memory-hungry allgather-then-slice); P4 needs gathers because its target is less partitioned
        if key != "adversarial_P4":
            assert set(kinds) <= {"dynslice", "alltoall", "allpermute", "allgather"} and plan.height_elems <= plan.bound_elems
