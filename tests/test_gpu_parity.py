"""GPU parity: the HIP path (through the C-ABI) against the oracle, bit for bit."""
import os
import random

import numpy as np
import pytest

import paper_2112_01075_amd as R
import synthetic_inputs as S
from oracle import redist_oracle as O

pytestmark = pytest.mark.gpu

ALL = [R.MODE_STEPWISE, R.MODE_FUSED, R.MODE_NAIVE]


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (there is no CPU fallback)")
    import gpu_util
    return gpu_util


def _void(G, elem):
    """uint8 array with trailing axis `elem` -> array of opaque elem-byte items."""
    return np.ascontiguousarray(G).view(np.dtype((np.void, elem)))[..., 0]


def test_c1_int32_both_directions_seeded_and_iota(gpu):
    w = S.WORKLOADS["c1_int32_2x2"]
    for pattern in ("seeded", "iota"):
        G = S.global_array("c1_int32_2x2", pattern)
        for a, b in w["pairs"]:
            gpu.parity(w["mesh"], a, b, 4, G, ALL, "c1/" + pattern)


def test_paper_examples_on_gpu(gpu, paper_chains):
    # first and last type of every printed chain, all modes
    for blk in paper_chains:
        a, b = blk["start"], blk["steps"][-1][2]
        t1 = O.parse_type(a)
        if O.globalsize(t1) > 1 << 22:
            G = np.random.default_rng(1).integers(0, 2 ** 16, O.globaltype(t1), dtype=np.uint16)
            elem = 2
        else:
            G = np.arange(O.globalsize(t1), dtype=np.int32).reshape(O.globaltype(t1))
            elem = 4
        gpu.parity(blk["mesh"], a, b, elem, G, ALL, blk["cite"][:30])


def test_element_sizes_and_ragged_shapes(gpu):
    from test_planner import _random_type
    rng = random.Random(4242)
    meshes = [{"a": 2, "b": 3}, {"a": 4, "b": 2}, {"a": 2, "b": 2, "c": 2}, {"a": 6}, {"a": 3, "b": 5}, {"a": 8, "b": 4}]
    shapes = [(120, 60), (60, 6, 40), (30, 1, 120), (1200,), (6, 10, 2, 60), (240, 7), (8, 15, 16)]
    n = 0
    while n < 40:
        mesh, g = rng.choice(meshes), rng.choice(shapes)
        nd = int(np.prod(list(mesh.values())))
        if any(s % nd for s in g[:1]) and rng.random() < 0.5:
            continue
        try:
            a, b = _random_type(rng, mesh, g), _random_type(rng, mesh, g)
        except Exception:
            continue
        elem = rng.choice([1, 2, 4, 8, 16])
        G = _void(S.random_bytes_array(g, elem, 1000 + n), elem)
        gpu.parity(mesh, a, b, elem, G, ALL, "ragged%d" % n)
        n += 1


def test_rows_that_start_off_the_vector_grid(gpu):
    """The span form of the LDS-staged kernels (aligned 16-byte blocks over misaligned rows), every granule size,
    plus larger odd shapes that give several tiles per chunk and ragged last tiles."""
    from test_copy_descriptors import SPAN_CASES
    for n, (mesh, g, a, b, elem, gran) in enumerate(SPAN_CASES):
        G = _void(S.random_bytes_array(g, elem, 1200 + n), elem)
        plans = gpu.parity(mesh, a, b, elem, G, ALL, "span%d" % n)
        ri = plans[R.MODE_FUSED].row_op(0)[0]
        assert ri.enabled and (ri.span == 1) == (gran < 16 and not (ri.dir == 1 and (ri.narrow_count > 1 or (ri.vw, ri.vn) == (16, 8)))), (a, b)
    m3, m1 = {"a": 2, "b": 2, "c": 2}, {"c": 2}
    big = [(m3, (7, 1000, 90), "[7, 1000, 45{a}90]", "[7, 500{a}1000, 90]", 4),
           (m1, (3, 2050, 74), "[3, 1025{c}2050, 74]", "[3, 2050, 37{c}74]", 4),
           (m1, (2, 4096, 30), "[2, 4096, 30]", "[2, 4096, 15{c}30]", 2),
           (m3, (5, 600, 149 * 2), "[5, 600, 149{a}298]", "[5, 300{a}600, 298]", 4),
           (m3, (2, 3000, 7 * 8), "[2, 3000, 7{a,b,c}56]", "[2, 375{a,b,c}3000, 56]", 1)]
    for n, (mesh, g, a, b, elem) in enumerate(big):
        G = _void(S.random_bytes_array(g, elem, 1300 + n), elem)
        plans = gpu.parity(mesh, a, b, elem, G, ALL, "spanbig%d" % n)
        assert plans[R.MODE_FUSED].row_op(0)[0].span == 1, (a, b)


def test_random_odd_shapes(gpu):
    """Forty seeded random problems that split or merge odd last dimensions (every form of the staged kernels)."""
    from test_copy_descriptors import odd_shape_problems
    spans = 0
    for n, (mesh, g, a, b, elem) in enumerate(odd_shape_problems(40)):
        G = _void(S.random_bytes_array(g, elem, 1700 + n), elem)
        plans = gpu.parity(mesh, a, b, elem, G, ALL, "odd%d" % n)
        ri = plans[R.MODE_FUSED].row_op(0)[0]
        spans += int(bool(ri.enabled and ri.span))
    assert spans >= 10


def test_identity_and_degenerate_cases(gpu):
    G = np.arange(8 * 6, dtype=np.int32).reshape(8, 6)
    gpu.parity({"x": 2, "y": 2}, "[4{x}8, 6]", "[4{x}8, 6]", 4, G, ALL, "identity")
    gpu.parity({"x": 1}, "[8, 6]", "[8{x}8, 6]", 4, G, ALL, "one-device")
    g1 = np.arange(4, dtype=np.uint8).reshape(4)
    gpu.parity({"x": 4}, "[1{x}4]", "[4]", 1, g1, ALL, "one-byte tiles")
    gpu.parity({"x": 2, "y": 2}, "[4]", "[1{x,y}4]", 1, g1, ALL, "slice to one byte")


def test_c2_activation_full_size(gpu):
    w = S.WORKLOADS["c2_bf16_act_1x8"]
    G = S.global_array("c2_bf16_act_1x8")
    for a, b in w["pairs"]:
        gpu.parity(w["mesh"], a, b, 2, G, ALL, "c2")
    G = S.global_array("c2_bf16_act_1x8", "iota")
    gpu.parity(w["mesh"], *w["pairs"][0], 2, G, [R.MODE_STEPWISE, R.MODE_FUSED], "c2/iota")


def test_c3_weight_full_size(gpu):
    w = S.WORKLOADS["c3_fp32_weight_4x2"]
    G = S.global_array("c3_fp32_weight_4x2")
    gpu.parity(w["mesh"], *w["pairs"][0], 4, G, ALL, "c3")


def test_c4_activation_full_size_both_stages(gpu):
    w = S.WORKLOADS["c4_bf16_act_2x4x4"]
    G = S.global_array("c4_bf16_act_2x4x4")
    gpu.parity(w["mesh"], *w["pairs"][0], 2, G, ALL, "c4a")
    gpu.parity(w["mesh"], *w["pairs"][1], 2, G, [R.MODE_STEPWISE, R.MODE_FUSED], "c4b")


def test_c5_attention_sampled_pairs_full_size(gpu):
    w = S.WORKLOADS["c5_bf16_attn_8x8"]
    G = S.global_array("c5_bf16_attn_8x8")
    for n, (a, b) in enumerate(S.pairs_of("c5_bf16_attn_8x8")):
        gpu.parity(w["mesh"], a, b, 2, G, [R.MODE_STEPWISE, R.MODE_FUSED], "c5/%d" % n)


def test_paper_shaped_problems_full_size(gpu, paper_values):
    """Sampled problems of the paper's evaluation shape (2x2x2 mesh, 4-byte elements, 64-800 MB, up to 6-D) and
    the four printed adversarial problems, iota data so that any misplaced element shows.  40 problems by default;
    REDIST_TEST_PAPER_PROBLEMS=1000 runs the whole seeded set at full size (about three minutes)."""
    count = int(os.environ.get("REDIST_TEST_PAPER_PROBLEMS", "40"))
    if count > 40:
        problems = list(S.sample_paper_problems(1000)[:count])
    else:
        problems = [(g, a, b) for g, a, b in S.sample_paper_problems(count, seed=S.BASE_SEED + 77, max_mb=400)]
    for key in ("adversarial_P1", "adversarial_P2", "adversarial_P3", "adversarial_P4"):
        a, b, _mb = [p.strip() for p in paper_values[key].split(";")]
        t = O.parse_type(a)
        problems.append((O.globaltype(t), O.format_type(t), O.format_type(O.parse_type(b))))
    for n, (g, a, b) in enumerate(problems):
        G = np.arange(int(np.prod(g)), dtype=np.int32).reshape(g)
        gpu.parity(S.PAPER_MESH, a, b, 4, G, [R.MODE_STEPWISE, R.MODE_FUSED], "paper-shaped/%d" % n)


def test_shards_larger_than_4_gib(gpu):
    """Byte offsets beyond 2^32 inside one shard (5 GiB shards, 1.25 GiB runs)."""
    n = 671088640
    G = np.arange(4 * n, dtype=np.uint32).view(np.int32).reshape(4, n)          # 10 GiB, every element distinct
    gpu.parity({"x": 2}, "[2{x}4, %d]" % n, "[4, %d{x}%d]" % (n // 2, n), 4, G, [R.MODE_STEPWISE, R.MODE_FUSED], "5 GiB shards")


def test_meshes_beyond_the_kernel_argument_limit(gpu):
    """More than 128 devices: shard pointers go through a device-side table instead of kernel arguments."""
    G = np.arange(512 * 24, dtype=np.int32).reshape(512, 24)
    mesh = {"x": 64, "y": 4}
    gpu.parity(mesh, "[8{x}512, 6{y}24]", "[2{y,x}512, 24]", 4, G, ALL, "256 devices")
    gpu.parity(mesh, "[2{x,y}512, 24]", "[512, 24]", 4, G, ALL, "256 devices, gather")
    gpu.parity({"x": 512}, "[1{x}512, 24]", "[512, 24]", 4, G, [R.MODE_STEPWISE, R.MODE_FUSED], "512 devices")
    # steps on the last dimension: the three forms of the LDS-staged kernels with the device-side pointer table
    plans = gpu.parity(mesh, "[512, 6{y}24]", "[8{x}512, 24]", 4, G, ALL, "256 devices, span form")
    assert plans[R.MODE_FUSED].row_op(0)[0].span == 1
    G2 = np.arange(512 * 32, dtype=np.int32).reshape(512, 32)
    plans = gpu.parity(mesh, "[512, 8{y}32]", "[8{x}512, 32]", 4, G2, ALL, "256 devices, power-of-two form")
    assert plans[R.MODE_FUSED].row_op(0)[0].enabled == 1 and plans[R.MODE_FUSED].row_op(0)[0].general == 0
    G3 = np.arange(512 * 48, dtype=np.int32).reshape(512, 48)
    plans = gpu.parity(mesh, "[8{x}512, 48]", "[512, 12{y}48]", 4, G3, ALL, "256 devices, general form")
    assert plans[R.MODE_FUSED].row_op(0)[0].general == 1 and plans[R.MODE_FUSED].row_op(0)[0].span == 0


def test_destination_major_order_forced(gpu):
    """Destination-major order on small problems (the option lowers its size threshold to zero): partial chunks,
    ragged tiles, narrow vectors, and the device-side pointer table of meshes beyond 128 devices."""
    forced = R.Options(dest_major_min_bytes=0)
    G = np.arange(512 * 24, dtype=np.int32).reshape(512, 24)
    plans = gpu.parity({"x": 64, "y": 4}, "[2{x,y}512, 24]", "[512, 24]", 4, G, ALL, "dm 256 devices", options=forced)
    assert plans[R.MODE_FUSED].op(0)[0].dest_major == 1
    gpu.parity({"x": 512}, "[1{x}512, 24]", "[512, 24]", 4, G, [R.MODE_STEPWISE, R.MODE_FUSED], "dm 512 devices",
               options=forced)
    rng = random.Random(321)
    from test_planner import _random_type
    meshes = [{"a": 2, "b": 3}, {"a": 4, "b": 2}, {"a": 2, "b": 2, "c": 2}, {"a": 8, "b": 4}]
    shapes = [(120, 60), (60, 6, 40), (1200,), (240, 7), (96, 40, 90)]
    seen = 0
    for n in range(30):
        mesh, g = rng.choice(meshes), rng.choice(shapes)
        nd = int(np.prod(list(mesh.values())))
        if g[0] % nd:
            continue
        a, b = _random_type(rng, mesh, g), _random_type(rng, mesh, g)
        elem = rng.choice([1, 2, 4, 8, 16])
        G2 = _void(S.random_bytes_array(g, elem, 2100 + n), elem)
        plans = gpu.parity(mesh, a, b, elem, G2, ALL, "dm%d" % n, options=forced)
        seen += plans[R.MODE_FUSED].op(0)[0].dest_major
        if n % 3 == 0:          # one destination per workgroup
            gpu.parity(mesh, a, b, elem, G2, [R.MODE_FUSED], "dm%d fanout 1" % n,
                       options=R.Options(dest_major_min_bytes=0, dest_major_fanout=1))
    assert seen >= 5


@pytest.mark.parametrize("mesh, a, b, gshape", [
    ({"x": 4, "y": 2}, "[4{x}16, 48{y}96]", "[8{y}16, 24{x}96]", (16, 96)),
    # beyond 128 devices the shard pointers reach the kernels through a device-side table that earlier
    # launches of the same call write: those launches are part of the recorded graph
    ({"x": 64, "y": 4}, "[8{x}512, 6{y}24]", "[128{y}512, 24]", (512, 24)),
])
def test_execute_can_be_captured_into_a_graph(gpu, mesh, a, b, gshape):
    """After redist_plan_prepare, redist_execute only enqueues kernels, so a multi-launch stepwise plan can be
    captured once and replayed; every replay, with new contents in the same buffers and eager work in between,
    must match the oracle."""
    import torch
    elem = 4
    t1, t2 = O.parse_type(a), O.parse_type(b)
    plan = R.redist_plan(mesh, a, b, elem, R.MODE_STEPWISE, options=R.Options(fold_permute=0))   # several launches
    assert plan.num_ops >= 2 and plan.workspace_bytes > 0
    plan.prepare()
    nd = plan.num_devices
    src = [torch.zeros(O.localsize(t1) * elem, dtype=torch.uint8, device=gpu.DEV) for _ in range(nd)]
    dst = [torch.zeros(O.localsize(t2) * elem, dtype=torch.uint8, device=gpu.DEV) for _ in range(nd)]
    ws = torch.zeros(plan.workspace_bytes, dtype=torch.uint8, device=gpu.DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        R.redist_execute(plan, src, dst, ws)          # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        R.redist_execute(plan, src, dst, ws)
    for rep in range(4):
        G = np.random.default_rng(3000 + rep).integers(-2**31, 2**31 - 1, size=gshape, dtype=np.int64).astype(np.int32)
        for k in range(nd):
            src[k].copy_(gpu.to_dev(O.shard_of(G, mesh, t1, k)))
        for d in dst:
            d.fill_(0xEE)                               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        gpu.check_against_oracle(dst, G, mesh, t2, "graph replay %d" % rep)


def test_destination_major_order_of_the_general_and_span_forms(gpu):
    from test_copy_descriptors import ROW_DM_GENERAL_FULL, ROW_DM_GENERAL_SMALL
    forced = R.Options(dest_major_min_bytes=0)
    for n, (mesh, g, a, b, elem) in enumerate(ROW_DM_GENERAL_SMALL):
        G = _void(S.random_bytes_array(g, elem, 2400 + n), elem)
        plans = gpu.parity(mesh, a, b, elem, G, ALL, "general/span dm small %d" % n, options=forced)
        assert plans[R.MODE_FUSED].row_op(0)[0].dest_major == 1
    for n, (mesh, g, a, b, elem, (general, span)) in enumerate(ROW_DM_GENERAL_FULL):   # whole chunks, XCD-blocked order
        G = np.arange(int(np.prod(g)), dtype=np.int32).reshape(g)
        plans = gpu.parity(mesh, a, b, elem, G, [R.MODE_STEPWISE, R.MODE_FUSED], "general/span dm full %d" % n)
        ri = plans[R.MODE_FUSED].row_op(0)[0]
        assert (ri.general, ri.span, ri.dest_major) == (general, span, 1) and ri.src_tiles > ri.chunk_tiles


def test_destination_major_order_of_the_staged_kernels(gpu):
    from test_copy_descriptors import ROW_DM_CASES
    for mesh, g, a, b, elem, direction in ROW_DM_CASES:
        G = _void(S.random_bytes_array(g, elem, 2300 + direction), elem)
        for fan in (0, 1):      # two receiving shards per workgroup (the default for so few), and one
            plans = gpu.parity(mesh, a, b, elem, G, ALL, "staged dm dir %d fanout %d" % (direction, fan),
                               options=R.Options(dest_major_fanout=fan))
            ri = plans[R.MODE_FUSED].row_op(0)[0]
            assert ri.dest_major == 1 and ri.dm_fanout == (1 if fan else 2)


def test_largest_rank_and_largest_mesh(gpu):
    """Rank 8, and 4096 devices (the most the boundary accepts): a gather to every device, a permutation of all
    tiles, and a two-axis alltoall, all through the device-side pointer tables."""
    mesh = {"a": 2, "b": 2, "c": 2}
    g = (3, 4, 2, 5, 2, 3, 2, 6)
    G = np.arange(int(np.prod(g)), dtype=np.int32).reshape(g)
    gpu.parity(mesh, "[3, 2{a}4, 2, 5, 1{c}2, 3, 2, 6]", "[3, 4, 1{b}2, 5, 2, 3, 1{a}2, 3{c}6]", 4, G, ALL, "rank 8")
    big = {"x": 64, "y": 64}
    G = np.arange(4096 * 8, dtype=np.int32).reshape(4096, 8)
    gpu.parity(big, "[1{x,y}4096, 8]", "[4096, 8]", 4, G, [R.MODE_STEPWISE, R.MODE_FUSED], "4096 devices, gather")
    G = np.arange(4096 * 64, dtype=np.int32).reshape(4096, 64)
    gpu.parity(big, "[64{x}4096, 1{y}64]", "[64{y}4096, 1{x}64]", 4, G, [R.MODE_STEPWISE, R.MODE_FUSED], "4096 devices, permute")
    gpu.parity(big, "[64{x}4096, 1{y}64]", "[1{x,y}4096, 64]", 4, G, [R.MODE_STEPWISE, R.MODE_FUSED], "4096 devices, alltoall")


def test_plans_on_two_streams_at_once(gpu):
    """Two plans (one of them with several launches and a workspace) enqueued alternately on two streams of the
    default priority: neither touches state of the other; results against the oracle."""
    import torch
    mesh, elem = {"x": 4, "y": 2}, 4
    jobs = [("[4{x}16, 48{y}96]", "[8{y}16, 24{x}96]", (16, 96), R.MODE_STEPWISE),
            ("[512, 6{y}12]", "[128{x}512, 12]", (512, 12), R.MODE_FUSED)]
    state = []
    for n, (a, b, g, mode) in enumerate(jobs):
        t1, t2 = O.parse_type(a), O.parse_type(b)
        G = np.random.default_rng(4100 + n).integers(-2**31, 2**31 - 1, size=g, dtype=np.int64).astype(np.int32)
        plan = R.redist_plan(mesh, a, b, elem, mode, options=R.Options(fold_permute=0))
        assert plan.num_ops >= 2 or mode == R.MODE_FUSED
        plan.prepare()
        src = gpu.upload_shards(G, mesh, t1)
        dst = [torch.zeros(O.localsize(t2) * elem, dtype=torch.uint8, device=gpu.DEV) for _ in range(plan.num_devices)]
        ws = torch.zeros(max(256, plan.workspace_bytes), dtype=torch.uint8, device=gpu.DEV)
        state.append((plan, src, dst, ws, G, t2, torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(20):
        for plan, src, dst, ws, G, t2, stream in state:
            R.redist_execute(plan, src, dst, ws, stream=stream.cuda_stream)
    torch.cuda.synchronize()
    for n, (plan, src, dst, ws, G, t2, stream) in enumerate(state):
        gpu.check_against_oracle(dst, G, mesh, t2, "two streams, job %d" % n)


def test_execute_error_paths(gpu):
    import torch
    plan = R.redist_plan({"x": 4, "y": 2}, "[2{x}8, 8{y}16]", "[4{y}8, 4{x}16]", 4,
                         options=R.Options(fold_permute=0))   # alltoall, then the permute on its own: needs workspace
    assert plan.workspace_bytes > 0
    src = [torch.zeros(64, dtype=torch.uint8, device="cuda:0") for _ in range(8)]
    dst = [torch.zeros(64, dtype=torch.uint8, device="cuda:0") for _ in range(8)]
    with pytest.raises(R.RedistError) as e:
        R.redist_execute(plan, src, dst, None)
    assert e.value.status == 6
    with pytest.raises(R.RedistError) as e:
        R.redist_execute(plan, [0] * 8, dst, torch.zeros(plan.workspace_bytes, dtype=torch.uint8, device="cuda:0"))
    assert e.value.status == 1
    ws = torch.zeros(plan.workspace_bytes + 256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(R.RedistError) as e:
        R.redist_execute(plan, [s.data_ptr() + 4 for s in src], dst, ws, torch.cuda.current_stream().cuda_stream)
    assert e.value.status == 9
    with pytest.raises(ValueError):                               # wrong number of shards is caught by the binding
        R.redist_execute(plan, src[:3], dst, ws)


def test_copy_baseline_kernel(gpu):
    import torch
    a = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda:0")
    b = torch.zeros_like(a)
    R.redist_copy_baseline(b, a, a.numel())
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def _states_case(gpu, mesh, a, b, elem, G, label):
    """Stepwise plan, launch by launch, against the oracle's device states (Def. 4.3; Fig. "Semantics of low-level
    collective operations"): once as the library groups steps into launches, once with one launch per plan step."""
    from test_planner import replay
    for options, tag in ((None, "grouped"), (R.Options(merge_runs=0), "literal")):
        plan = R.redist_plan(mesh, a, b, elem, options=options)
        states = []
        replay(plan, mesh, a, b, G, states_out=states)
        done = gpu.stepwise_states_against_oracle(mesh, a, b, elem, G, states, "%s/%s" % (label, tag), options=options)
        if tag == "literal":
            assert done.num_ops == max(1, done.num_steps)


def test_every_intermediate_state_against_the_oracle(gpu):
    from test_planner import _shrunk
    w = S.WORKLOADS["c1_int32_2x2"]
    for a, b in w["pairs"]:
        _states_case(gpu, w["mesh"], a, b, 4, S.global_array("c1_int32_2x2"), "c1")
    mesh, pairs = _shrunk("c3_fp32_weight_4x2", 8)                      # 16 MiB, alltoall + allpermute
    t = O.parse_type(pairs[0][0])
    G = np.arange(O.globalsize(t), dtype=np.int32).reshape(O.globaltype(t))
    _states_case(gpu, mesh, *pairs[0], 4, G, "c3/8")
    mesh, pairs = _shrunk("c4_bf16_act_2x4x4", 4)                       # both stages, incl. alltoall + allgather
    for a, b in pairs:
        G = np.random.default_rng(5).integers(0, 2 ** 16, O.globaltype(O.parse_type(a)), dtype=np.uint16)
        _states_case(gpu, mesh, a, b, 2, G, "c4/4")
    # attention pairs and paper-shaped problems with the longest step lists
    mesh, pairs = _shrunk("c5_bf16_attn_8x8", 4)
    ranked = sorted(pairs, key=lambda ab: -R.redist_plan(mesh, ab[0], ab[1], 2).num_steps)
    kinds_seen = set()
    for a, b in ranked[:6]:
        kinds_seen |= {s["kind"] for s in R.redist_plan(mesh, a, b, 2).steps()}
        G = np.random.default_rng(6).integers(0, 2 ** 16, O.globaltype(O.parse_type(a)), dtype=np.uint16)   # shrunk per pair
        _states_case(gpu, mesh, a, b, 2, G, "c5/4")
    assert {"dynslice", "alltoall", "allgather"} <= kinds_seen
    problems = [p for p in S.sample_paper_problems(200) if int(np.prod(p[0])) * 4 <= 100 << 20]
    ranked = sorted(problems, key=lambda p: -R.redist_plan(S.PAPER_MESH, p[1], p[2], 4).num_steps)
    for g, a, b in ranked[:3]:
        G = np.arange(int(np.prod(g)), dtype=np.int32).reshape(g)
        _states_case(gpu, S.PAPER_MESH, a, b, 4, G, "paper-shaped")


def test_cached_plans_execute(gpu):
    """Plans handed out by the plan cache (one shared object per distinct problem) carry out the redistribution
    like any other; the second holder finds the plan already prepared."""
    R.redist_plan_cache_clear()
    mesh = {"x": 4, "y": 2}
    a, b = "[4{x}16, 48{y}96]", "[8{y}16, 24{x}96]"
    t1, t2 = O.parse_type(a), O.parse_type(b)
    G = np.random.default_rng(8).integers(-2 ** 31, 2 ** 31 - 1, size=(16, 96), dtype=np.int64).astype(np.int32)
    src = gpu.upload_shards(G, mesh, t1)
    for mode in ALL:
        for rep in range(2):
            plan = R.redist_plan(mesh, a, b, 4, mode, cached=True)
            dst = gpu.run_plan(plan, src, O.localsize(t2) * 4, label="cached")
            gpu.check_against_oracle(dst, G, mesh, t2, "cached plan, mode %d, holder %d" % (mode, rep))
    assert R.redist_plan_cache_size() == 3
    R.redist_plan_cache_clear()


def test_ops_split_over_several_launches(gpu):
    """max_grid = 5 workgroups per launch: every body (generic, destination-major, the three staged forms) goes out
    as many launches, each told the index of its first workgroup."""
    from test_copy_descriptors import ROW_DM_CASES, SPAN_CASES
    few = R.Options(max_grid=5)
    G = np.arange(96 * 40 * 90, dtype=np.int32).reshape(96, 40, 90)
    mesh = {"a": 2, "b": 2, "c": 2}
    gpu.parity(mesh, "[48{a}96, 20{b}40, 90]", "[96, 10{c,b}40, 45{a}90]", 4, G, ALL, "split generic/staged", options=few)
    gpu.parity(mesh, "[48{a}96, 20{b}40, 90]", "[96, 40, 90]", 4, G, ALL, "split dest-major",
               options=R.Options(max_grid=5, dest_major_min_bytes=0))
    m, g, a, b, elem, gran = SPAN_CASES[0]
    gpu.parity(m, a, b, elem, _void(S.random_bytes_array(g, elem, 77), elem), ALL, "split span", options=few)
    G2 = np.arange(512 * 32, dtype=np.int32).reshape(512, 32)
    plans = gpu.parity({"x": 64, "y": 4}, "[512, 8{y}32]", "[8{x}512, 32]", 4, G2, ALL, "split, 256 devices", options=few)
    assert plans[R.MODE_FUSED].row_op(0)[0].max_grid == 5
    m, g, a, b, elem, direction = ROW_DM_CASES[0]
    gpu.parity(m, a, b, elem, _void(S.random_bytes_array(g, elem, 78), elem), [R.MODE_FUSED], "split staged dm",
               options=R.Options(max_grid=1000))


def test_cell_staged_kernel(gpu):
    """The cell-staged kernel on the seeded problems of the host-model test (forced on wherever a launch qualifies:
    1 to 3 cell dims, granules of 4, 8 and 16 bytes, replicated destinations, several tiles per box with a ragged
    last one), and by the default choice on a reduced copy of the slowest paper-shaped problem."""
    from test_copy_descriptors import cell_problems
    forced = R.Options(cell_form=2)
    seen = set()
    for n, (mesh, g, a, b, elem) in enumerate(cell_problems(40)):
        G = _void(S.random_bytes_array(g, elem, 2600 + n), elem)
        plans = gpu.parity(mesh, a, b, elem, G, [R.MODE_STEPWISE, R.MODE_FUSED], "cell %d" % n, options=forced)
        for plan in plans.values():
            for k in range(plan.num_ops):
                ci = plan.cell_op(k)[0]
                if ci.enabled:
                    seen.add((ci.n_cell, ci.gran))
    assert {c[0] for c in seen} == {1, 2, 3} and {c[1] for c in seen} == {4, 8, 16}, seen
    mesh = {"a": 2, "b": 2, "c": 2}
    a, b, g = "[6, 74, 16{b}32, 9{a,c}36, 8]", "[6, 74, 32, 18{a}36, 4{b}8]", (6, 74, 32, 36, 8)
    G = np.arange(int(np.prod(g)), dtype=np.int32).reshape(g)
    plans = gpu.parity(mesh, a, b, 4, G, ALL, "cell default")
    assert plans[R.MODE_FUSED].step_kernel(0) == "redist_fused_gather_cell_kernel"


def test_sibling_boxes(gpu):
    """Destination-major launches whose sibling boxes (adjacent pieces of the destination's rows, from different
    shards) take turns tile by tile, with one and two receivers per workgroup; among them the 32-shard gather
    reduced to a few rows."""
    from test_copy_descriptors import SIBLING_CASES
    for n, (mesh, g, a, b, elem, pieces, m) in enumerate(SIBLING_CASES):
        G = _void(S.random_bytes_array(g, elem, 2800 + n), elem)
        for fan in (0, 1, 2):
            plans = gpu.parity(mesh, a, b, elem, G, [R.MODE_FUSED] if fan else [R.MODE_STEPWISE, R.MODE_FUSED],
                               "siblings %d fanout %d" % (n, fan),
                               options=R.Options(dest_major_min_bytes=0, dest_major_fanout=fan))
            assert plans[R.MODE_FUSED].op(0)[0].sib_count == pieces


@pytest.mark.gpu
def test_sibling_boxes_of_ordinary_ops(gpu):
    """The ordinary order with alternating sibling boxes: pieces of the destination's rows and pieces of the source's
    rows (boxes in source order), groups of 2, 3 and 8, a chain of 16 boxes in two groups."""
    from test_copy_descriptors import ORDINARY_SIBLING_CASES
    for n, (mesh, g, a, b, elem, p, side) in enumerate(ORDINARY_SIBLING_CASES):
        G = _void(S.random_bytes_array(g, elem, 2900 + n), elem)
        plans = gpu.parity(mesh, a, b, elem, G, [R.MODE_STEPWISE, R.MODE_FUSED], "ordinary siblings %d" % n,
                           options=R.Options(cell_form=0, lds_staging=0))
        info = plans[R.MODE_FUSED].op(0)[0]
        assert info.sib_count == p and info.dest_major == 0
        assert plans[R.MODE_FUSED].step_kernel(0) == "redist_fused_gather_kernel"


@pytest.mark.gpu
def test_sibling_boxes_with_runs_of_several_tiles(gpu):
    """Sibling boxes whose runs are two and four tiles wide (the tiles of a run stay together), ordinary and
    destination-major order."""
    cases = [({"x": 4}, (12, 8192), "[12, 2048{x}8192]", "[3{x}12, 8192]", 4, 4, 1, 1 << 40),
             ({"x": 4}, (12, 8192), "[3{x}12, 8192]", "[12, 2048{x}8192]", 4, 1, 0, 1 << 40),   # (source side: usual order)
             ({"x": 2, "y": 2}, (6, 8192), "[6, 4096{x}8192]", "[3{y}6, 8192]", 4, 2, 2, 0)]
    for n, (mesh, g, a, b, elem, p, lg, dm_min) in enumerate(cases):
        G = _void(S.random_bytes_array(g, elem, 3000 + n), elem)
        plans = gpu.parity(mesh, a, b, elem, G, [R.MODE_STEPWISE, R.MODE_FUSED], "sibling runs %d" % n,
                           options=R.Options(sibling_sources=65536, cell_form=0, lds_staging=0, dest_major_min_bytes=dm_min))
        info = plans[R.MODE_FUSED].op(0)[0]
        assert (info.sib_count, info.sib_inner_log2) == (p, lg)


@pytest.mark.gpu
def test_staged_boxes_in_destination_order(gpu):
    """Staged scatter whose boxes are cut into destination-contiguous parts and sorted by destination address (seq
    blocks of two shards per destination row), and the same op with the boxes kept."""
    mesh, a, b = {"q": 2, "p": 2}, "[2{q}4, 4, 256{p}512, 128]", "[4, 2{p}4, 512, 64{q}128]"
    G = _void(S.random_bytes_array((4, 4, 512, 128), 1, 3100), 1)
    for k, boxes in ((1, 32), (2, 8)):
        plans = gpu.parity(mesh, a, b, 1, G, [R.MODE_STEPWISE, R.MODE_FUSED], "staged boxes, lds_staging=%d" % k,
                           options=R.Options(cell_form=0, lds_staging=k))
        assert plans[R.MODE_FUSED].step_kernel(0) == "redist_fused_gather_lds_kernel"
        assert plans[R.MODE_FUSED].row_op(0)[0].n_boxes == boxes


@pytest.mark.gpu
def test_sibling_boxes_with_the_device_side_pointer_table(gpu):
    """Sibling boxes on a mesh of 256 devices (shard pointers in a device-side table): rows dealt out in 512-byte
    pieces to all devices and collected again -- chains of 256 boxes, alternating in groups of 8."""
    mesh = {"x": 64, "y": 4}
    G = _void(S.random_bytes_array((256, 32768), 4, 3200), 4)
    for a, b in (("[1{x,y}256, 32768]", "[256, 128{x,y}32768]"), ("[256, 128{x,y}32768]", "[1{x,y}256, 32768]")):
        plans = gpu.parity(mesh, a, b, 4, G, [R.MODE_STEPWISE, R.MODE_FUSED], "siblings, 256 devices")
        info = plans[R.MODE_FUSED].op(0)[0]
        assert info.sib_count == 8 and info.dest_major == 0 and plans[R.MODE_FUSED].step_kernel(0) == "redist_fused_gather_kernel"

