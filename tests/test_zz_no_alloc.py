"""The entry point that allocates nothing (redist_execute_static) against redist_execute, through the C-ABI."""
import numpy as np
import pytest

import paper_2112_01075_amd as R
import synthetic_inputs as S
from oracle import redist_oracle as O

pytestmark = pytest.mark.gpu


def _both_ways(gpu, torch, mesh, a, b, elem, G, mode, options=None, label=""):
    t1, t2 = O.parse_type(a), O.parse_type(b)
    plan = R.redist_plan(mesh, a, b, elem, mode, options=options)
    assert plan.static_fits, label
    src = gpu.upload_shards(G, mesh, t1)
    nbytes = O.localsize(t2) * elem
    want = gpu.run_plan(plan, src, nbytes, label=label + " (redist_execute)")       # the existing entry point
    dst = [gpu.Guarded(nbytes, 0x3C) for _ in range(plan.num_devices)]
    fresh = R.redist_plan(mesh, a, b, elem, mode, options=options)                  # never prepared: nothing allocated for it
    print("    static %s mode=%d %s -> %s launches=%d workspace=%d" % (label, mode, a, b, fresh.num_ops, fresh.workspace_bytes),
          flush=True)
    R.redist_execute_static(fresh, src, [g.buf for g in dst])
    torch.cuda.synchronize()
    for k, g in enumerate(dst):
        g.check("%s: static, destination shard %d" % (label, k))
        assert torch.equal(g.buf, want[k]), "%s: shard %d differs from redist_execute" % (label, k)
    gpu.check_against_oracle([g.buf for g in dst], G, mesh, t2, label + " static vs oracle")


def test_static_entry_point_matches_execute_two_calls_in_a_row():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (there is no CPU fallback)")
    import gpu_util as gpu
    mesh = {"x": 4, "y": 2}
    literal = R.Options(merge_runs=0)
    # first call: three launches (alltoall, allpermute kept apart, then the gathers) with intermediates in the scratch area
    G = np.random.default_rng(11).integers(-2 ** 31, 2 ** 31 - 1, size=(256, 384), dtype=np.int64).astype(np.int32)
    a, b = "[64{x}256, 192{y}384]", "[128{y}256, 384]"
    big = R.redist_plan(mesh, a, b, 4, R.MODE_STEPWISE, options=literal)
    assert big.num_ops >= 2 and big.workspace_bytes > 0
    _both_ways(gpu, torch, mesh, a, b, 4, G, R.MODE_STEPWISE, literal, "first call")
    # second call, right after, on a smaller input: what the first call left in the area must not show
    G2 = np.random.default_rng(12).integers(-2 ** 31, 2 ** 31 - 1, size=(16, 96), dtype=np.int64).astype(np.int32)
    _both_ways(gpu, torch, mesh, "[4{x}16, 48{y}96]", "[8{y}16, 24{x}96]", 4, G2, R.MODE_STEPWISE, literal, "second call, smaller")
    # every mode, and a staged (LDS) op
    for mode in (R.MODE_STEPWISE, R.MODE_FUSED, R.MODE_NAIVE):
        _both_ways(gpu, torch, mesh, "[4{x}16, 48{y}96]", "[8{y}16, 24{x}96]", 4, G2, mode, None, "mode %d" % mode)
    G3 = np.arange(512 * 32, dtype=np.int32).reshape(512, 32)
    _both_ways(gpu, torch, mesh, "[512, 16{y}32]", "[128{x}512, 32]", 4, G3, R.MODE_FUSED, None, "staged")
    # a full-size workload whose plan is one launch: descriptors only
    w = S.WORKLOADS["c2_bf16_act_1x8"]
    _both_ways(gpu, torch, w["mesh"], *w["pairs"][0], 2, S.global_array("c2_bf16_act_1x8"), R.MODE_STEPWISE, None, "c2")


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    w = S.WORKLOADS["c4_bf16_act_2x4x4"]
    plan = R.redist_plan(w["mesh"], *w["pairs"][1], 2, R.MODE_STEPWISE)
    assert not plan.static_fits
    dummy = [torch.zeros(16, dtype=torch.uint8, device="cuda:0") for _ in range(32)]
    with pytest.raises(R.RedistError) as e:
        R.redist_execute_static(plan, dummy, dummy)          # refused before anything is enqueued
    assert e.value.status == 10
    torch.cuda.synchronize()
