"""Host model of the gather kernel's index arithmetic, for checking copy descriptors without a GPU.

It walks the descriptor tables exactly as a workgroup does (tile -> box -> row/column of every lane
-> byte offsets through the multiply-high division) on NumPy byte buffers, and adds what the GPU
cannot report: every access is bounds-checked against the shard extents and every destination byte
must be written exactly once.  Test infrastructure; the library never runs this.
"""
import numpy as np



def run_op(info, boxes, dst_list, src_bufs, n_dst):
    """Apply one launch.  src_bufs: list of uint8 arrays (one per shard).  Returns the destination buffers."""
    V, n_outer = info.vec_bytes, info.n_outer
    TILE_VECS = 256 * info.unroll            # 256 threads x `unroll` vectors
    tc, tr = info.tc, info.tr
    assert 1 <= tc and 1 <= tr and tc * tr <= TILE_VECS
    dst_bufs = [np.zeros(info.dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    hits = [np.zeros(info.dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    firsts = [b.tile_first for b in boxes]
    e = np.arange(TILE_VECS, dtype=np.uint64)
    lane_bytes = np.arange(V, dtype=np.int64)
    assert sum(b.n_tiles for b in boxes) == info.src_tiles
    m = info.dm_count if info.dest_major else 1
    fan, groups = info.dm_fanout, info.dm_groups
    assert (m > 1) == bool(info.dest_major) and fan in (1, 2, 4) and groups == -(-m // fan)
    assert info.n_tiles == info.src_tiles * groups
    for launch in range(info.n_tiles):
        tile, k_dst = launch, None
        if info.dest_major:
            # destination-major order: launch index = (chunk, group of destinations, tile of the chunk), chunks running
            # over the op's tiles whatever box they belong to; dm_fanout destinations per workgroup
            ct = info.chunk_tiles
            assert ct >= 8 and ct & (ct - 1) == 0
            t_hi = launch // ct
            c = t_hi if groups == 1 else ((t_hi * info.dm_magic) >> 32) >> info.dm_shift   # the kernel's division by dm_groups
            assert c == t_hi // groups
            r = launch - c * ct * groups
            here = min(ct, info.src_tiles - c * ct)
            assert here > 0
            g = r // here
            if here == ct:
                assert g == t_hi - c * groups and r - g * here == launch % ct
            assert g < groups
            k_dst = range(g * fan, min(m, g * fan + fan))
            assert len(k_dst) >= 1
            tile = c * ct + (r - g * here)
            assert tile < info.src_tiles
        sib_t = None
        if info.sib_count > 1:
            # sibling boxes: groups of sib_count boxes of one shape whose tiles alternate
            P, T = info.sib_count, info.tiles_per_box
            assert T > 0 and len(boxes) % P == 0 and info.unroll == 1 and V == 16
            g = tile // (P * T)
            tig = tile - g * P * T
            lg = info.sib_inner_log2                   # runs of 2^lg tiles (column blocks) stay together
            q = tig >> lg
            o = ((q * info.sib_magic) >> 32) >> info.sib_shift
            assert o == q // P and (lg == 0 or (tr == 1 and boxes[0].col_blocks == 1 << lg))
            sib_t = (o << lg) | (tig & ((1 << lg) - 1))
            b = g * P + (q - o * P)
            assert boxes[b].tile_first == b * T and boxes[b].n_tiles == T
        elif info.tiles_per_box:
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
        assert sib_t is not None or 0 <= t_in < bx.n_tiles
        src_dev, src_off, dst_off = bx.src_dev, bx.src_off, bx.dst_off
        if sib_t is not None:
            t_in = sib_t
        dsts = [bx.dst_dev0] + dst_list[bx.dst_first + 1:bx.dst_first + bx.dst_count]
        assert bx.dst_count >= 1 and bx.dst_dev0 == dst_list[bx.dst_first] and len(dsts) == bx.dst_count
        if info.dest_major:
            assert bx.dst_count == m
            dsts = [dsts[k] for k in k_dst]
        rb = t_in if bx.col_blocks == 1 else ((t_in * bx.cb_magic) >> 32) >> bx.cb_shift
        assert rb == t_in // bx.col_blocks
        cb = t_in - rb * bx.col_blocks
        er = e if tc == 1 else ((e * np.uint64(info.tc_magic)) >> np.uint64(32)) >> np.uint64(info.tc_shift)
        assert (er == e // np.uint64(tc)).all()
        row = rb * tr + er
        col = cb * tc + (e - er * np.uint64(tc))
        live = (er < tr) & (row < bx.rows) & (col < bx.run_vecs)
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
        so, do = so[live] + src_off, do[live] + dst_off
        if so.size == 0:
            continue
        assert so.min() >= 0 and so.max() + V <= info.src_shard_bytes, "source access out of bounds"
        assert do.min() >= 0 and do.max() + V <= info.dst_shard_bytes, "destination access out of bounds"
        assert (so % V == 0).all() and (do % V == 0).all(), "misaligned vector access"
        data = src_bufs[src_dev][so[:, None] + lane_bytes[None, :]]
        addr = do[:, None] + lane_bytes[None, :]
        for d in dsts:
            dst_bufs[d][addr] = data
            np.add.at(hits[d], addr.reshape(-1), 1)
    for d in range(n_dst):
        assert (hits[d] == 1).all(), "destination shard %d not written exactly once" % d
    return dst_bufs


ROW_TILE_BYTES = 16384


def _stage_addr(r, col, w_log2):
    mask = (1 << (w_log2 - 4)) - 1
    return (r << w_log2) + ((((col >> 4) ^ (r & mask)) << 4) | (col & 15))


def _div(n, d, magic, shift):
    """n // d the way the kernel does it (d == 1 is special-cased there)."""
    if d == 1:
        return n
    q = ((n * magic) >> 32) >> shift
    assert (q == n // d).all()
    return q


def _row_dm_index(info, launch, m):
    """Destination-major order of the staged kernels: launch index -> (tile of the op, which receiving shard)."""
    ct = info.chunk_tiles
    fan, groups = info.dm_fanout, info.dm_groups
    assert ct >= 8 and ct & (ct - 1) == 0 and fan in (1, 2) and groups == -(-m // fan)
    t_hi = launch // ct
    c = t_hi if groups == 1 else ((t_hi * info.dm_magic) >> 32) >> info.dm_shift
    assert c == t_hi // groups
    r = launch - c * ct * groups
    here = min(ct, info.src_tiles - c * ct)
    g = r // here
    assert here > 0 and g < groups
    which = range(g * fan, min(m, g * fan + fan))
    l = r - g * here
    if here == ct and info.dir == 0:
        # gathers: XCD x (workgroups go to the 8 XCDs in turn) takes the x-th eighth of a whole chunk's tiles
        l = (l & 7) * (ct >> 3) + (l >> 3)
    tile = c * ct + l
    assert tile < info.src_tiles
    return tile, which


def run_row_op(info, boxes, pieces, dev_list, src_bufs, n_dst):
    """One launch of the LDS-staged (row-complete) kernel, walked tile by tile like a workgroup does.
    Covers both forms: power-of-two sizes (shifts, XOR-swizzled staging) and the general one (reciprocal
    divisions, padded staging rows, one vector width on both sides)."""
    general = bool(info.general)
    R, VN = (info.rpt if general else 1 << info.r_log2), info.vn   # general form: any number of rows per tile
    if general:
        W, N, VW, pitch = info.w_bytes, info.n_bytes, info.vw, info.pitch
        assert VW in (16, VN) and W % VW == 0 and N % VN == 0 and info.cpn * VN == N and info.wpr * VW == W
        assert pitch >= W and pitch % 16 == 0 and R * pitch <= ROW_TILE_BYTES
    else:
        W, N, VW, pitch = 1 << info.w_log2, 1 << info.n_log2, 16, 1 << info.w_log2
        assert VN == min(16, N) and R * W <= ROW_TILE_BYTES
    assert info.n_pieces * N == W and R <= (1024 if not general and W <= 32 else 256)
    assert info.n_pieces * info.narrow_count <= 512
    gather = info.dir == 0
    dst_bufs = [np.zeros(info.dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    hits = [np.zeros(info.dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    wide_bytes = info.dst_shard_bytes if gather else info.src_shard_bytes
    narrow_bytes = info.src_shard_bytes if gather else info.dst_shard_bytes
    firsts = [b.tile_first for b in boxes]
    # narrow-side elements: vector c of piece k in staged row r; wide-side elements: vector w of staged row r
    n_total = R * W // VN
    e = np.arange(n_total, dtype=np.int64)
    if general:
        t = _div(e, info.cpn, info.cpn_magic, info.cpn_shift)
        kk = _div(t, R, info.rpt_magic, info.rpt_shift)
        c, rr = e - t * info.cpn, t - kk * R
        narrow_stage = rr * pitch + kk * N + c * VN
        ew = np.arange(R * info.wpr, dtype=np.int64)
        rw = _div(ew, info.wpr, info.wpr_magic, info.wpr_shift)
        ww = ew - rw * info.wpr
        wide_stage = rw * pitch + ww * VW
        wide_col = ww * VW
    else:
        lv = VN.bit_length() - 1
        cpl = info.n_log2 - lv
        c = e & ((1 << cpl) - 1)
        rr = (e >> cpl) & (R - 1)
        kk = e >> (cpl + info.r_log2)
        narrow_stage = _stage_addr(rr, (kk << info.n_log2) + (c << lv), info.w_log2)
        ew = np.arange((R * W) >> 4, dtype=np.int64)
        ww = ew & ((1 << (info.w_log2 - 4)) - 1)
        rw = ew >> (info.w_log2 - 4)
        wide_stage = _stage_addr(rw, ww << 4, info.w_log2)
        wide_col = ww << 4
    assert (kk < info.n_pieces).all() and (rr < R).all() and (rw < R).all()
    narrow_col = c * VN
    vb = np.arange(VN, dtype=np.int64)
    wb = np.arange(VW, dtype=np.int64)
    m = info.dm_count if info.dest_major else 1
    assert sum(b.n_tiles for b in boxes) == info.src_tiles and info.n_tiles == info.src_tiles * info.dm_groups
    assert (m > 1) == bool(info.dest_major) and (not info.dest_major or general or R <= 256)
    for launch in range(info.n_tiles):
        tile, which = launch, None
        if info.dest_major:      # (chunk, which of the m receiving shards, tile of the chunk), as in run_op
            tile, which = _row_dm_index(info, launch, m)
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
        row0 = (tile - bx.tile_first) * R
        assert 0 <= tile - bx.tile_first < bx.n_tiles and row0 < bx.rows
        rows_here = min(R, bx.rows - row0)
        # phase 0: row offsets
        n = np.arange(row0, row0 + rows_here, dtype=np.uint64)
        wo = np.zeros(rows_here, dtype=np.int64)
        no = np.zeros(rows_here, dtype=np.int64)
        for k in range(info.n_outer - 1, 0, -1):
            ln = int(bx.len[k])
            q = n if ln == 1 else ((n * np.uint64(bx.magic[k])) >> np.uint64(32)) >> np.uint64(bx.shift[k])
            idx = (n - q * np.uint64(ln)).astype(np.int64)
            assert (idx < ln).all()
            wo += idx * info.wstride[k]
            no += idx * info.nstride[k]
            n = q
        if info.n_outer > 0:
            assert (n < bx.len[0]).all()
            wo += n.astype(np.int64) * info.wstride[0]
            no += n.astype(np.int64) * info.nstride[0]
        pcs = pieces[bx.piece_first:bx.piece_first + info.n_pieces]
        assert len(pcs) == info.n_pieces
        stage = np.zeros(ROW_TILE_BYTES, dtype=np.uint8)
        stage_hits = np.zeros(ROW_TILE_BYTES, dtype=np.uint8)
        live_n = rr < rows_here
        live_w = rw < rows_here
        wide_devs = dev_list[bx.wide_first:bx.wide_first + bx.wide_count]
        assert len(wide_devs) == bx.wide_count >= 1
        woff_w = bx.wide_off + wo[np.minimum(rw, rows_here - 1)] + wide_col
        assert (woff_w[live_w] >= 0).all() and (woff_w[live_w] + VW <= wide_bytes).all() and (woff_w % VW == 0).all()
        assert (wide_stage % VW == 0).all() and (narrow_stage % VN == 0).all()
        if gather:
            for k, pc in enumerate(pcs):
                sel = live_n & (kk == k)
                if not sel.any():
                    continue
                addr = pc.narrow_off + no[rr[sel]] + narrow_col[sel]
                assert (addr >= 0).all() and (addr + VN <= narrow_bytes).all() and (addr % VN == 0).all()
                sdev = dev_list[pc.dev_first]
                data = src_bufs[sdev][addr[:, None] + vb[None, :]]
                sa = narrow_stage[sel][:, None] + vb[None, :]
                assert sa.max() < ROW_TILE_BYTES
                stage[sa] = data
                np.add.at(stage_hits, sa.reshape(-1), 1)
            sa = wide_stage[live_w][:, None] + wb[None, :]
            assert sa.max() < ROW_TILE_BYTES
            assert (stage_hits[sa] == 1).all(), "wide phase reads staging bytes not written exactly once"
            data = stage[sa]
            da = woff_w[live_w][:, None] + wb[None, :]
            if info.dest_major:
                assert bx.wide_count == m
            for d in (wide_devs if which is None else [wide_devs[k] for k in which]):
                dst_bufs[d][da] = data
                np.add.at(hits[d], da.reshape(-1), 1)
        else:
            sa = wide_stage[live_w][:, None] + wb[None, :]
            assert sa.max() < ROW_TILE_BYTES
            stage[sa] = src_bufs[wide_devs[0]][woff_w[live_w][:, None] + wb[None, :]]
            np.add.at(stage_hits, sa.reshape(-1), 1)
            for k, pc in enumerate(pcs):
                sel = live_n & (kk == k)
                if not sel.any():
                    continue
                addr = pc.narrow_off + no[rr[sel]] + narrow_col[sel]
                assert (addr >= 0).all() and (addr + VN <= narrow_bytes).all() and (addr % VN == 0).all()
                sa = narrow_stage[sel][:, None] + vb[None, :]
                assert (stage_hits[sa] == 1).all()
                data = stage[sa]
                da = addr[:, None] + vb[None, :]
                ndevs = dev_list[pc.dev_first:pc.dev_first + info.narrow_count]
                assert len(ndevs) == info.narrow_count and (not info.dest_major or info.narrow_count == m)
                for d in (ndevs if which is None else [ndevs[k] for k in which]):
                    dst_bufs[d][da] = data
                    np.add.at(hits[d], da.reshape(-1), 1)
    for d in range(n_dst):
        assert (hits[d] == 1).all(), "destination shard %d not written exactly once (row op)" % d
    return dst_bufs


def run_span_op(info, boxes, pieces, dev_list, src_bufs, n_dst):
    """One launch of the span form of the LDS-staged kernel.  A tile is up to mct virtual chunks (whole chunks of
    contiguous rows, or stretches of rpt rows of a long one), each one contiguous span per side, covered by
    16-byte aligned blocks: whole blocks move as vectors, the granules of edge blocks one by one; loads read a
    block whole when it lies inside the shard.  The staging area holds virtual chunk c at c*slot, in the wide
    span's byte order, shifted by the span's misalignment.  Checked here: the index arithmetic (reciprocals),
    bounds and alignment of every access, exactly-once coverage of spans, staging area and destinations."""
    W, N, G, R, P = info.w_bytes, info.n_bytes, info.gran, info.rpt, info.n_pieces
    assert info.general and info.span and G in (1, 2, 4, 8) and G == info.vn
    assert W % G == 0 and N % G == 0 and P * N == W and info.cpn * G == N and R >= 1
    n_outer, cd, M = info.n_outer, info.chunk_dims, info.mct
    assert cd in (n_outer, n_outer - 1) and 1 <= M <= 64 and M * P * info.narrow_count <= 512
    if cd == n_outer - 1:
        assert info.wstride[n_outer - 1] == W and info.nstride[n_outer - 1] == N
    STAGE = ROW_TILE_BYTES + 32
    assert info.slot == 16 * info.cbw and M * info.slot <= STAGE
    gather = info.dir == 0
    GP = 16 // G
    dst_bufs = [np.zeros(info.dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    hits = [np.zeros(info.dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    wide_bytes = info.dst_shard_bytes if gather else info.src_shard_bytes
    narrow_bytes = info.src_shard_bytes if gather else info.dst_shard_bytes
    firsts = [b.tile_first for b in boxes]
    gb = np.arange(G, dtype=np.int64)
    gofs = np.arange(GP, dtype=np.int64) * G
    assert sum(b.n_tiles for b in boxes) == info.src_tiles

    def geometry(bx, v):
        o = v if bx.tpc == 1 else ((v * bx.tpc_magic) >> 32) >> bx.tpc_shift
        assert o == v // bx.tpc
        r0 = (v - o * bx.tpc) * bx.vrows
        assert r0 < bx.chunk_rows and bx.tpc == -(-bx.chunk_rows // bx.vrows) and bx.vrows <= R
        rows = min(bx.vrows, bx.chunk_rows - r0)
        wo, no, n = r0 * W, r0 * N, o
        for k in range(cd - 1, 0, -1):
            ln = int(bx.len[k])
            q = n if ln == 1 else ((n * int(bx.magic[k])) >> 32) >> int(bx.shift[k])
            assert q == n // ln
            wo += (n - q * ln) * info.wstride[k]
            no += (n - q * ln) * info.nstride[k]
            n = q
        if cd > 0:
            assert n < bx.len[0]
            wo += n * info.wstride[0]
            no += n * info.nstride[0]
        else:
            assert n == 0
        return wo, no, rows

    m = info.dm_count if info.dest_major else 1
    assert info.n_tiles == info.src_tiles * info.dm_groups and (m > 1) == bool(info.dest_major)
    for launch in range(info.n_tiles):
        tile, which = launch, None
        if info.dest_major:      # (chunk, which group of the m receiving shards, tile of the chunk), as in run_row_op
            tile, which = _row_dm_index(info, launch, m)
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
        cr = bx.len[n_outer - 1] if cd == n_outer - 1 else 1
        assert 0 <= t_in < bx.n_tiles and bx.chunk_rows == cr and bx.rows % cr == 0
        assert 1 <= bx.vrows <= R and bx.tpc == -(-cr // bx.vrows) and bx.n_vchunks == bx.rows // cr * bx.tpc
        assert bx.n_tiles == -(-bx.n_vchunks // M)
        v0 = t_in * M
        m_here = min(M, bx.n_vchunks - v0)
        assert m_here >= 1
        pcs = pieces[bx.piece_first:bx.piece_first + P]
        assert len(pcs) == P
        wide_devs = dev_list[bx.wide_first:bx.wide_first + bx.wide_count]
        assert len(wide_devs) == bx.wide_count >= 1
        stage = np.zeros(STAGE, dtype=np.uint8)
        stage_hits = np.zeros(STAGE, dtype=np.uint8)
        geo = [geometry(bx, v0 + c) for c in range(m_here)]
        # ---- wide side: (virtual chunk, block) pairs ----
        ew = np.arange(m_here * info.cbw, dtype=np.int64)
        cw_ = np.zeros_like(ew) if M == 1 else _div(ew, info.cbw, info.cbw_magic, info.cbw_shift)
        jw = ew - cw_ * info.cbw
        woff = np.array([bx.wide_off + g[0] for g in geo], dtype=np.int64)
        lenw = np.array([g[2] * W for g in geo], dtype=np.int64)
        assert (woff % G == 0).all() and (woff >= 0).all() and (woff + lenw <= wide_bytes).all()
        pw = woff & 15
        wblk = woff - pw
        s0w = (jw << 4) - pw[cw_]
        sw = s0w[:, None] + gofs[None, :]
        okw = (sw >= 0) & (sw < lenw[cw_][:, None]) & (s0w < lenw[cw_])[:, None]
        w_glob = (wblk[cw_] + (jw << 4))[:, None] + gofs[None, :]
        w_stage = (cw_ * info.slot + (jw << 4))[:, None] + gofs[None, :]
        assert (w_stage[okw] + G <= STAGE).all()
        for c in range(m_here):          # the blocks of a span cover it exactly once
            cover = np.zeros(lenw[c], dtype=np.uint8)
            np.add.at(cover, (sw[(cw_ == c)[:, None] & okw][:, None] + gb[None, :]).reshape(-1), 1)
            assert (cover == 1).all(), "wide span not covered exactly once"
        w_in_shard = (w_glob[:, 0] >= 0) & (w_glob[:, 0] + 16 <= wide_bytes)
        assert (w_in_shard | ~okw.all(axis=1)).all() and (w_glob[okw.any(axis=1), 0] % 16 == 0).all()
        assert (okw.any(axis=1) & ~w_in_shard).sum() <= 1, "only a shard's last block may reach past its end"
        # ---- narrow side: (virtual chunk, piece, block) triples ----
        e = np.arange(m_here * P * info.nbm, dtype=np.int64)
        vk = _div(e, info.nbm, info.nbm_magic, info.nbm_shift)
        jj = e - vk * info.nbm
        cc, kk = vk // P, vk % P
        noff = np.array([[pc.narrow_off + g[1] for pc in pcs] for g in geo], dtype=np.int64).reshape(-1)   # by vk
        lenn = np.array([[g[2] * N for _ in pcs] for g in geo], dtype=np.int64).reshape(-1)
        assert (noff % G == 0).all() and (noff >= 0).all() and (noff + lenn <= narrow_bytes).all()
        pn = noff & 15
        nblk = noff - pn
        sbase = (np.repeat(np.arange(m_here), P) * info.slot + np.repeat(pw, P) + np.tile(np.arange(P), m_here) * N)
        assert (sbase < 65536).all() and (lenn < (1 << 28)).all()
        s0 = (jj << 4) - pn[vk]
        sn = s0[:, None] + gofs[None, :]
        okn = (sn >= 0) & (sn < lenn[vk][:, None]) & (s0 < lenn[vk])[:, None]
        sg = np.where(okn, sn, 0) // G
        row = _div(sg, info.cpn, info.cpn_magic, info.cpn_shift)
        n_stage = sbase[vk][:, None] + row * W + (sg - row * info.cpn) * G
        n_glob = (nblk[vk] + (jj << 4))[:, None] + gofs[None, :]
        assert (n_stage[okn] % G == 0).all() and (n_stage[okn] + G <= STAGE).all()
        assert (row[okn] < np.broadcast_to((lenn[vk] // N)[:, None], row.shape)[okn]).all()
        n_in_shard = (n_glob[:, 0] >= 0) & (n_glob[:, 0] + 16 <= narrow_bytes)
        assert (n_glob[okn.any(axis=1), 0] % 16 == 0).all() and (n_in_shard | ~okn.all(axis=1)).all()
        assert (okn.any(axis=1) & ~n_in_shard).sum() <= P
        for q in range(m_here * P):
            cover = np.zeros(lenn[q], dtype=np.uint8)
            np.add.at(cover, (sn[(vk == q)[:, None] & okn][:, None] + gb[None, :]).reshape(-1), 1)
            assert (cover == 1).all(), "narrow span not covered exactly once"
        if gather:
            for k, pc in enumerate(pcs):
                sel = okn & (kk == k)[:, None]
                sdev = dev_list[pc.dev_first]
                sa = n_stage[sel][:, None] + gb[None, :]
                stage[sa] = src_bufs[sdev][n_glob[sel][:, None] + gb[None, :]]
                np.add.at(stage_hits, sa.reshape(-1), 1)
            sa = w_stage[okw][:, None] + gb[None, :]
            assert (stage_hits[sa] == 1).all(), "wide phase reads staging bytes not written exactly once"
            da = w_glob[okw][:, None] + gb[None, :]
            assert not info.dest_major or bx.wide_count == m
            for d in (wide_devs if which is None else [wide_devs[k] for k in which]):
                dst_bufs[d][da] = stage[sa]
                np.add.at(hits[d], da.reshape(-1), 1)
        else:
            sa = w_stage[okw][:, None] + gb[None, :]
            stage[sa] = src_bufs[wide_devs[0]][w_glob[okw][:, None] + gb[None, :]]
            np.add.at(stage_hits, sa.reshape(-1), 1)
            for k, pc in enumerate(pcs):
                sel = okn & (kk == k)[:, None]
                sa = n_stage[sel][:, None] + gb[None, :]
                assert (stage_hits[sa] == 1).all()
                da = n_glob[sel][:, None] + gb[None, :]
                ndevs = dev_list[pc.dev_first:pc.dev_first + info.narrow_count]
                assert len(ndevs) == info.narrow_count and (not info.dest_major or info.narrow_count == m)
                for d in (ndevs if which is None else [ndevs[k] for k in which]):
                    dst_bufs[d][da] = stage[sa]
                    np.add.at(hits[d], da.reshape(-1), 1)
    for d in range(n_dst):
        assert (hits[d] == 1).all(), "destination shard %d not written exactly once (span op)" % d
    return dst_bufs


def run_plan(plan, src_bufs, stats=None):
    """All launches of a plan, chained through per-step intermediates (the workspace)."""
    cur = src_bufs
    nd = plan.num_devices
    for k in range(plan.num_ops):
        info, boxes, dst_list = plan.op(k)
        assert all(len(b) == info.src_shard_bytes for b in cur)
        rinfo, rboxes, pieces, dev_list = plan.row_op(k)
        generic = run_op(info, boxes, dst_list, cur, nd)      # the generic descriptors are always valid
        if rinfo.enabled:
            assert rinfo.src_shard_bytes == info.src_shard_bytes and rinfo.dst_shard_bytes == info.dst_shard_bytes
            staged = (run_span_op if rinfo.span else run_row_op)(rinfo, rboxes, pieces, dev_list, cur, nd)
            for x, y in zip(generic, staged):
                assert x.tobytes() == y.tobytes(), "generic and row-complete descriptors disagree"
            if stats is not None:
                stats["row_ops"] = stats.get("row_ops", 0) + 1
                stats["general_row_ops"] = stats.get("general_row_ops", 0) + int(rinfo.general)
                stats["span_row_ops"] = stats.get("span_row_ops", 0) + int(rinfo.span)
        cinfo, cboxes, clist = plan.cell_op(k)
        if cinfo.enabled:
            cells = run_cell_op(cinfo, cboxes, clist, cur, nd, info.dst_shard_bytes)
            for x, y in zip(generic, cells):
                assert x.tobytes() == y.tobytes(), "generic and cell-complete descriptors disagree"
            if stats is not None:
                stats["cell_ops"] = stats.get("cell_ops", 0) + 1
        cur = generic
    return cur


def run_cell_op(info, boxes, dev_list, src_bufs, n_dst, dst_shard_bytes):
    """The cell-staged kernel, workgroup by workgroup: every source part's stretch of the tile's rows is staged part
    after part; every destination part's stretch is put together granule by granule from the staging area through the
    digits of the granule's position in the cell, with the kernel's reciprocal divisions."""
    VS, VD, G = info.vs, info.vd, info.gran
    assert G in (4, 8, 16) and VS in (G, 16) and VD in (G, 16)
    ps, pd, rep, nc, no = info.ps, info.pd, info.rep, info.n_cell, info.n_outer
    assert 1 <= ps <= 64 and 1 <= pd * rep <= 64 and 1 <= nc <= 3 and 1 <= no <= 7
    STAGE = 16384
    assert info.part_pitch % 16 == 0 and ps * info.part_pitch <= STAGE
    assert info.rows_per_tile * info.src_row_bytes <= info.part_pitch
    assert info.src_row_bytes % VS == 0 and info.dst_row_bytes % VD == 0 and info.dst_row_bytes % G == 0
    assert info.drow_gran * G == info.dst_row_bytes
    assert info.sstride[no - 1] == info.src_row_bytes and info.dstride[no - 1] == info.dst_row_bytes
    assert info.spv * VS == info.rows_per_tile * info.src_row_bytes
    assert info.dpv * VD == info.rows_per_tile * info.dst_row_bytes
    assert info.n_list == len(dev_list) and info.base_first + pd <= len(dev_list)
    dst_bufs = [np.zeros(dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    hits = [np.zeros(dst_shard_bytes, dtype=np.uint8) for _ in range(n_dst)]
    firsts = [b.tile_first for b in boxes]
    assert sum(b.n_tiles for b in boxes) == info.n_tiles
    srow_vecs, drow_vecs = info.src_row_bytes // VS, info.dst_row_bytes // VD
    GPV = VD // G

    def last_term(x):
        addr = np.zeros_like(x)
        if info.piece[0]:
            p = _div(x, info.piece[0], info.piece_magic[0], info.piece_shift[0])
            x = x - p * info.piece[0]
            addr = p * info.part_step[0]
        return addr + x * info.lds_step[0]

    def row_terms(base, gi):
        row = _div(gi, info.drow_gran, info.drg_magic, info.drg_shift)
        jj = gi - row * info.drow_gran
        addr = base + row * info.src_row_bytes
        if nc == 1:
            x0 = jj
        else:
            q = _div(jj, info.dext[0], info.dext_magic[0], info.dext_shift[0])
            x0 = jj - q * info.dext[0]
            jj = q
        for i in range(1, nc):
            x = jj
            if i + 1 < nc:
                q = _div(jj, info.dext[i], info.dext_magic[i], info.dext_shift[i])
                x = jj - q * info.dext[i]
                jj = q
            else:
                assert (x < info.dext[i]).all()
            if info.piece[i]:
                p = _div(x, info.piece[i], info.piece_magic[i], info.piece_shift[i])
                x = x - p * info.piece[i]
                addr = addr + p * info.part_step[i]
            addr = addr + x * info.lds_step[i]
        return addr, x0

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
        tb = tile - bx.tile_first
        assert 0 <= tb < bx.n_tiles
        rest = tb if bx.row_tiles == 1 else ((tb * bx.rt_magic) >> 32) >> bx.rt_shift
        assert rest == tb // bx.row_tiles
        row0 = (tb - rest * bx.row_tiles) * info.rows_per_tile
        assert row0 < bx.len[no - 1]
        rows = min(info.rows_per_tile, bx.len[no - 1] - row0)
        so, do = bx.src_off + row0 * info.src_row_bytes, bx.dst_off + row0 * info.dst_row_bytes
        for k in range(no - 2, 0, -1):
            ln = bx.len[k]
            q = rest if ln == 1 else ((rest * bx.magic[k]) >> 32) >> bx.shift[k]
            assert q == rest // ln
            idx = rest - q * ln
            so += idx * info.sstride[k]
            do += idx * info.dstride[k]
            rest = q
        if no > 1:
            assert rest < bx.len[0]
            so += rest * info.sstride[0]
            do += rest * info.dstride[0]
        else:
            assert rest == 0
        full = rows == info.rows_per_tile
        stage = np.zeros(STAGE, dtype=np.uint8)
        staged = np.zeros(STAGE, dtype=np.uint8)
        # ---- source parts -> staging area ----
        spv = info.spv if full else rows * srow_vecs
        e = np.arange(ps * spv, dtype=np.int64)
        s = np.zeros_like(e) if ps == 1 else (_div(e, spv, info.spv_magic, info.spv_shift) if full else e // spv)
        i = e - s * spv
        for part in range(ps):
            sel = i[s == part]
            dev = dev_list[bx.src_first + part]
            buf = src_bufs[dev]
            lo_b, hi_b = so + int(sel.min()) * VS, so + int(sel.max()) * VS + VS
            assert 0 <= lo_b and hi_b <= len(buf), ("cell source read out of bounds", tile, part, lo_b, hi_b, len(buf))
            at = part * info.part_pitch
            n = len(sel) * VS
            assert at + n <= STAGE
            stage[at:at + n] = buf[so:so + n]
            staged[at:at + n] += 1
        # ---- staging area -> destination parts ----
        dpv = info.dpv if full else rows * drow_vecs
        e = np.arange(pd * dpv, dtype=np.int64)
        q = np.zeros_like(e) if pd == 1 else (_div(e, dpv, info.dpv_magic, info.dpv_shift) if full else e // dpv)
        i = e - q * dpv
        base = np.array([dev_list[info.base_first + int(x)] for x in range(pd)], dtype=np.int64)[q]
        out = np.zeros((len(e), VD), dtype=np.uint8)
        hi_t, x0 = row_terms(base, i * GPV)
        for k in range(GPV):
            same = x0 + k < info.dext[0]
            hi_k, x_k = row_terms(base, i * GPV + k)
            at_slow = hi_k + last_term(x_k)
            at_fast = hi_t + last_term(np.where(same, x0 + k, 0))
            assert (at_fast[same] == at_slow[same]).all(), "fast and slow staging addresses disagree"
            at = np.where(same, at_fast, at_slow)
            assert (at >= 0).all() and (at + G <= STAGE).all() and (at % G == 0).all()
            idx = at[:, None] + np.arange(G)[None, :]
            assert (staged[idx] == 1).all(), "granule read from a part of the staging area that was not staged"
            out[:, k * G:(k + 1) * G] = stage[idx]
        for part in range(pd):
            sel = np.nonzero(q == part)[0]
            ii = i[sel]
            assert (ii == np.arange(len(sel))).all()
            n = len(sel) * VD
            for j in range(rep):
                dev = dev_list[bx.dst_first + part * rep + j]
                assert 0 <= do and do + n <= dst_shard_bytes, ("cell destination write out of bounds", tile, part, do, n)
                dst_bufs[dev][do:do + n] = out[sel].reshape(-1)
                hits[dev][do:do + n] += 1
    for d in range(n_dst):
        assert (hits[d] == 1).all(), "destination shard %d: bytes written %s" % (d, "never" if (hits[d] == 0).any() else "twice")
    return dst_bufs
