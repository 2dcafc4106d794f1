"""Helpers of the GPU parity tests: move shards to the device, run a plan through the C-ABI binding,
compare destination shards bit for bit with the oracle's direct slicing."""
import numpy as np
import torch

import paper_2112_01075_amd as R
from oracle import redist_oracle as O

DEV = "cuda:0"


def to_dev(arr):
    """NumPy array of any dtype -> uint8 device tensor of its bytes."""
    flat = np.ascontiguousarray(arr).reshape(-1).view(np.uint8)
    return torch.from_numpy(flat).to(DEV)


def upload_shards(G, mesh, typ):
    """Source shards on the device; replicas of a tile are device-side clones of one upload."""
    table = O.offset_table(typ, mesh)
    first = {}
    out = []
    for k, off in enumerate(table):
        if off in first:
            out.append(out[first[off]].clone())
        else:
            first[off] = k
            out.append(to_dev(O.shard_of(G, mesh, typ, k)))
    return out


def run_plan(plan, src, shard_bytes, fill=0xA5):
    nd = plan.num_devices
    dst = [torch.full((shard_bytes,), fill, dtype=torch.uint8, device=DEV) for _ in range(nd)]
    ws = None
    if plan.workspace_bytes:
        ws = torch.full((plan.workspace_bytes,), 0x5A, dtype=torch.uint8, device=DEV)
    R.redist_execute(plan, src, dst, ws)
    torch.cuda.synchronize()
    return dst


def check_against_oracle(dst, G, mesh, typ, label=""):
    """Every destination shard must equal the oracle's slice of G, byte for byte."""
    table = O.offset_table(typ, mesh)
    cache = {}
    for k, off in enumerate(table):
        if off not in cache:
            cache.clear()                     # keep one expected tile on the device at a time
            cache[off] = to_dev(O.shard_of(G, mesh, typ, k))
        want = cache[off]
        got = dst[k]
        assert got.numel() == want.numel(), (label, k)
        if not torch.equal(got, want):
            bad = (got != want).nonzero()
            raise AssertionError("%s: shard %d differs at %d bytes, first at byte %d"
                                 % (label, k, bad.numel(), int(bad[0])))


def parity(mesh, a, b, elem, G, modes, label=""):
    """G: NumPy array whose itemsize is `elem` (or a void view).  Runs every mode, checks every shard."""
    t1, t2 = O.parse_type(a), O.parse_type(b)
    src = upload_shards(G, mesh, t1)
    shard_bytes = O.localsize(t2) * elem
    plans = {}
    for mode in modes:
        print("    parity %s mode=%d %s -> %s" % (label, mode, a, b), flush=True)
        plan = R.redist_plan(mesh, a, b, elem, mode)
        dst = run_plan(plan, src, shard_bytes)
        check_against_oracle(dst, G, mesh, t2, "%s mode %d %s -> %s" % (label, mode, a, b))
        # the sources must be untouched
        del dst
        plans[mode] = plan
    ref = upload_shards(G, mesh, t1) if len(src) <= 8 and src[0].numel() <= (1 << 24) else None
    if ref is not None:
        for x, y in zip(src, ref):
            assert torch.equal(x, y), "source shard modified"
    return plans
