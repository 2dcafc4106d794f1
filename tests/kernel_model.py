"""Host model of the gather kernel's index arithmetic, for checking copy descriptors without a GPU.

It walks the descriptor tables exactly as a workgroup does (tile -> box -> row/column of every lane
-> byte offsets through the multiply-high division) on NumPy byte buffers, and adds what the GPU
cannot report: every access is bounds-checked against the shard extents and every destination byte
must be written exactly once.  Test infrastructure; the library never runs this.
"""
import numpy as np



def run_op(info, boxes, dst_list, src_bufs, n_dst):
    """Apply one launch.  src_bufs: list of uint8 arrays (one per shard).  Returns the destination buffers."""
    V, tcl, n_outer = info.vec_bytes, info.tc_log2, info.n_outer
    TILE_VECS = 256 * info.unroll            # 256 threads x `unroll` vectors
    tc, tr = 1 << tcl, TILE_VECS >> tcl
    dst_bufs = [np.zeros(info.dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    hits = [np.zeros(info.dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    firsts = [b.tile_first for b in boxes]
    e = np.arange(TILE_VECS, dtype=np.uint64)
    lane_bytes = np.arange(V, dtype=np.int64)
    assert sum(b.n_tiles for b in boxes) == info.n_tiles
    for tile in range(info.n_tiles):
        if info.tiles_per_box:
            b = tile if info.tiles_per_box == 1 else ((tile * info.tpb_magic) >> 32) >> info.tpb_shift
            assert b == tile // info.tiles_per_box
        else:
            lo, hi = 0, len(boxes) - 1
            while lo < hi:
                mid = (lo + hi + 1) >> 1
                if firsts[mid] <= tile:
                    lo = mid
                else:
                    hi = mid - 1
            b = lo
        bx = boxes[b]
        t_in = tile - bx.tile_first
        assert 0 <= t_in < bx.n_tiles
        rb = t_in // bx.col_blocks
        cb = t_in - rb * bx.col_blocks
        row = rb * tr + (e >> np.uint64(tcl))
        col = cb * tc + (e & np.uint64(tc - 1))
        live = (row < bx.rows) & (col < bx.run_vecs)
        so = (col * np.uint64(V)).astype(np.int64)
        do = so.copy()
        n = row.copy()
        for k in range(n_outer - 1, 0, -1):
            ln = int(bx.len[k])
            if ln == 1:
                q = n
            else:
                q = ((n * np.uint64(bx.magic[k])) >> np.uint64(32)) >> np.uint64(bx.shift[k])
            idx = (n - q * np.uint64(ln)).astype(np.int64)
            assert (idx[live] < ln).all() and (idx[live] >= 0).all()
            so += idx * info.sstride[k]
            do += idx * info.dstride[k]
            n = q
        if n_outer > 0:
            assert (n[live] < bx.len[0]).all()
            so += n.astype(np.int64) * info.sstride[0]
            do += n.astype(np.int64) * info.dstride[0]
        so, do = so[live] + bx.src_off, do[live] + bx.dst_off
        if so.size == 0:
            continue
        assert so.min() >= 0 and so.max() + V <= info.src_shard_bytes, "source access out of bounds"
        assert do.min() >= 0 and do.max() + V <= info.dst_shard_bytes, "destination access out of bounds"
        assert (so % V == 0).all() and (do % V == 0).all(), "misaligned vector access"
        data = src_bufs[bx.src_dev][so[:, None] + lane_bytes[None, :]]
        addr = do[:, None] + lane_bytes[None, :]
        assert bx.dst_count >= 1 and bx.dst_dev0 == dst_list[bx.dst_first]
        for d in [bx.dst_dev0] + dst_list[bx.dst_first + 1:bx.dst_first + bx.dst_count]:
            dst_bufs[d][addr] = data
            np.add.at(hits[d], addr.reshape(-1), 1)
    for d in range(n_dst):
        assert (hits[d] == 1).all(), "destination shard %d not written exactly once" % d
    return dst_bufs


def run_plan(plan, src_bufs):
    """All launches of a plan, chained through per-step intermediates (the workspace)."""
    cur = src_bufs
    nd = plan.num_devices
    for k in range(plan.num_ops):
        info, boxes, dst_list = plan.op(k)
        assert all(len(b) == info.src_shard_bytes for b in cur)
        cur = run_op(info, boxes, dst_list, cur, nd)
    return cur
