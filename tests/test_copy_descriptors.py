"""Copy descriptors of every mode, interpreted by the host model of the kernel (bounds, exactly-once
writes, alignment) and compared bit for bit with the oracle's direct slicing."""
import random

import numpy as np
import pytest

import paper_2112_01075_amd as R
import synthetic_inputs as S
from kernel_model import run_plan
from oracle import redist_oracle as O
from test_planner import _random_type, _shrunk

MODES = [R.MODE_STEPWISE, R.MODE_FUSED, R.MODE_NAIVE]


def _check(mesh, a, b, elem, modes=MODES, seed=0):
    t1, t2 = O.parse_type(a), O.parse_type(b)
    G = S.random_bytes_array(O.globaltype(t1), elem, seed)
    gview = G.reshape(G.shape[:-1] + (elem,))
    src = [s.reshape(-1).copy() for s in O.distribute(gview.view(np.dtype((np.void, elem)))[..., 0], mesh, t1)]
    src = [np.frombuffer(s.tobytes(), dtype=np.uint8) for s in src]
    want = [np.frombuffer(s.tobytes(), dtype=np.uint8)
            for s in O.distribute(gview.view(np.dtype((np.void, elem)))[..., 0], mesh, t2)]
    for mode in modes:
        plan = R.redist_plan(mesh, a, b, elem, mode)
        got = run_plan(plan, src)
        for d, (x, y) in enumerate(zip(got, want)):
            assert x.tobytes() == y.tobytes(), (a, b, elem, mode, d)
        moved = plan.algorithmic_bytes(R.BYTES_MOVED_BY_PLAN)
        assert moved > 0
    return plan


def test_small_workload_c1_all_modes():
    w = S.WORKLOADS["c1_int32_2x2"]
    for a, b in w["pairs"]:
        _check(w["mesh"], a, b, 4)


def test_shrunk_workloads_all_modes():
    for name, factor in (("c2_bf16_act_1x8", 32), ("c3_fp32_weight_4x2", 128), ("c4_bf16_act_2x4x4", 16)):
        mesh, pairs = _shrunk(name, factor)
        for a, b in pairs:
            _check(mesh, a, b, S.WORKLOADS[name]["elem_size"])


def test_shrunk_attention_pairs_stepwise_and_fused():
    mesh, pairs = _shrunk("c5_bf16_attn_8x8", 8)
    for n, (a, b) in enumerate(pairs):
        _check(mesh, a, b, 2, modes=[R.MODE_STEPWISE, R.MODE_FUSED] if n % 5 else MODES, seed=n)


def test_every_element_size_and_odd_shapes():
    rng = random.Random(99)
    meshes = [{"a": 2, "b": 3}, {"a": 4, "b": 2}, {"a": 2, "b": 2, "c": 2}, {"a": 6}, {"a": 3, "b": 5}]
    shapes = [(12, 30), (60, 6, 4), (30, 1, 12), (120,), (6, 10, 2, 6)]
    for n in range(60):
        mesh, g = rng.choice(meshes), rng.choice(shapes)
        try:
            a, b = _random_type(rng, mesh, g), _random_type(rng, mesh, g)
        except Exception:
            continue
        _check(mesh, a, b, rng.choice([1, 2, 4, 8, 16]), seed=n)


def test_non_nested_tilings_give_non_uniform_boxes():
    # 3-element source tiles against 2-element target tiles: destination tiles straddle source tiles
    plan = _check({"x": 4, "y": 6}, "[3{x}12, 2{y}12]", "[2{y}12, 3{x}12]", 4, modes=[R.MODE_FUSED])
    info, boxes, _ = plan.op(0)
    assert len({b.n_tiles for b in boxes}) >= 1 and len({(b.rows, b.run_vecs) for b in boxes}) > 1


def test_replicated_destinations_share_one_read():
    # allgather to a full replica: every box is read once and stored to all shards
    plan = R.redist_plan({"x": 4}, "[4{x}16, 8]", "[16, 8]", 4, R.MODE_FUSED)
    info, boxes, dst_list = plan.op(0)
    assert all(b.dst_count == 4 for b in boxes) and sorted(dst_list) == [0, 1, 2, 3]
    assert plan.algorithmic_bytes(R.BYTES_MOVED_BY_PLAN) == 16 * 8 * 4 * (1 + 4)


def test_magic_division_is_exact():
    rng = random.Random(5)
    plan = R.redist_plan({"a": 2, "b": 3, "c": 2}, "[10{a}20, 14{b}42, 6{c}12, 10]", "[20, 7{a,b}42, 12, 5{c}10]", 2,
                         R.MODE_FUSED)
    info, boxes, _ = plan.op(0)
    seen = 0
    for bx in boxes:
        for k in range(1, info.n_outer):
            d = bx.len[k]
            if d == 1:
                continue
            for n in [0, 1, d - 1, d, d + 1, 2 * d - 1, 2 ** 31 - 1, 2 ** 31 - d] + [rng.randrange(2 ** 31) for _ in range(50)]:
                assert ((n * bx.magic[k]) >> 32) >> bx.shift[k] == n // d
                seen += 1
    assert seen > 0
