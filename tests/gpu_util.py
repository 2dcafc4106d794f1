"""Helpers of the GPU parity tests: move shards to the device, run a plan through the C-ABI binding,
compare destination shards bit for bit with the oracle's direct slicing.

Every buffer the library writes (destination shards, workspace) is carved out of a larger allocation with a
guard band of sentinel bytes on both sides; after every run the bands must be untouched, so that a store that
leaves its buffer shows on the GPU too, not only under the host model of the kernels."""
import numpy as np
import torch

import paper_2112_01075_amd as R
from oracle import redist_oracle as O

DEV = "cuda:0"
GUARD = 4096          # bytes of sentinel in front of and behind every buffer the library writes
SENTINEL = 0xC3


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


class Guarded:
    """A device buffer of `nbytes` bytes (filled with `fill`) between two guard bands of SENTINEL bytes.
    The payload starts 4096 bytes into a fresh allocation, so it keeps the allocator's 256-byte alignment."""

    def __init__(self, nbytes, fill):
        self.whole = torch.full((nbytes + 2 * GUARD,), SENTINEL, dtype=torch.uint8, device=DEV)
        self.buf = self.whole[GUARD:GUARD + nbytes]
        self.buf.fill_(fill)

    def check(self, label):
        lo, hi = self.whole[:GUARD], self.whole[GUARD + self.buf.numel():]
        if not (bool((lo == SENTINEL).all()) and bool((hi == SENTINEL).all())):
            where = "below" if not bool((lo == SENTINEL).all()) else "above"
            raise AssertionError("%s: bytes written %s the buffer (guard band damaged)" % (label, where))


def guarded_buffers(plan, shard_bytes, fill=0xA5):
    nd = plan.num_devices
    dst = [Guarded(shard_bytes, fill) for _ in range(nd)]
    ws = Guarded(plan.workspace_bytes, 0x5A) if plan.workspace_bytes else None
    return dst, ws


def check_guards(dst, ws, label):
    for k, g in enumerate(dst):
        g.check("%s: destination shard %d" % (label, k))
    if ws is not None:
        ws.check("%s: workspace" % label)


def run_plan(plan, src, shard_bytes, fill=0xA5, label=""):
    dst, ws = guarded_buffers(plan, shard_bytes, fill)
    R.redist_execute(plan, src, [g.buf for g in dst], ws.buf if ws else None)
    torch.cuda.synchronize()
    check_guards(dst, ws, label)
    return [g.buf for g in dst]


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


def parity(mesh, a, b, elem, G, modes, label="", options=None):
    """G: NumPy array whose itemsize is `elem` (or a void view).  Runs every mode, checks every shard."""
    t1, t2 = O.parse_type(a), O.parse_type(b)
    src = upload_shards(G, mesh, t1)
    shard_bytes = O.localsize(t2) * elem
    plans = {}
    for mode in modes:
        print("    parity %s mode=%d %s -> %s" % (label, mode, a, b), flush=True)
        plan = R.redist_plan(mesh, a, b, elem, mode, options=options)
        what = "%s mode %d %s -> %s" % (label, mode, a, b)
        dst = run_plan(plan, src, shard_bytes, label=what)
        check_against_oracle(dst, G, mesh, t2, what)
        # the sources must be untouched
        del dst
        plans[mode] = plan
    ref = upload_shards(G, mesh, t1) if len(src) <= 8 and src[0].numel() <= (1 << 24) else None
    if ref is not None:
        for x, y in zip(src, ref):
            assert torch.equal(x, y), "source shard modified"
    return plans


def stepwise_states_against_oracle(mesh, a, b, elem, G, states, label="", options=None):
    """Runs the stepwise plan launch by launch (redist_execute_range) and, after every launch, reads back what it
    wrote -- the workspace intermediate, or the destination shards for the last launch -- and compares it, shard by
    shard and bit for bit, with the oracle's state after the last plan step that launch carries out.
    `states[k]` = list of the oracle's tiles (NumPy) after plan step k, one per device."""
    t1, t2 = O.parse_type(a), O.parse_type(b)
    plan = R.redist_plan(mesh, a, b, elem, R.MODE_STEPWISE, options=options)
    assert plan.num_steps == len(states), (plan.num_steps, len(states))
    src = upload_shards(G, mesh, t1)
    dst, ws = guarded_buffers(plan, O.localsize(t2) * elem)
    nd, n_ops = plan.num_devices, plan.num_ops
    for k in range(n_ops):
        last = plan.op_last_step(k)
        print("    states %s launch %d/%d (plan steps up to %d) %s -> %s" % (label, k, n_ops, last, a, b), flush=True)
        R.redist_execute_range(plan, src if k == 0 else None, [g.buf for g in dst] if k == n_ops - 1 else None,
                               ws.buf if ws else None, k, k + 1)
        torch.cuda.synchronize()
        check_guards(dst, ws, "%s launch %d" % (label, k))
        want = states[last]
        for d in range(nd):
            tile = np.ascontiguousarray(want[d])
            nbytes = tile.size * tile.itemsize
            if k == n_ops - 1:
                got = dst[d].buf
            else:
                off, stride = plan.op_output(k)
                got = ws.buf[off + d * stride: off + d * stride + nbytes]
            assert got.numel() == nbytes, (label, k, d)
            assert got.cpu().numpy().tobytes() == tile.tobytes(), \
                "%s: after launch %d (plan step %d) device %d does not hold the oracle's tile" % (label, k, last, d)
    return plan
